// Chooses the kernel family for a call.  Host code only.
#include "gspn_common.hpp"
#include <stdlib.h>
#include <atomic>

namespace gspn {

enum FwdPlan { FWD_GENERIC = 0, FWD_TILE = 1, FWD_STREAM = 2, FWD_PLANE = 3, FWD_PAIR = 4, FWD_CHUNK = 5 };
enum BwdPlan { BWD_GENERIC = 0, BWD_TILE = 1, BWD_PLANE = 2, BWD_TWOPASS = 3 };

// Testing aids that keep every kernel family reachable on every shape it accepts.  The environment is read once, on
// the first call of a process (and again only when reload_env_knobs() is called, which the tests do after they change
// it): a launch costs one atomic load, and no call races with a setenv elsewhere in the process.
// GSPN_FORCE_GENERIC=1: the generic kernels; GSPN_FWD_NO_PLANE=1 / GSPN_BWD_NO_PLANE=1: skip the plane kernels;
// GSPN_BWD_NO_TWOPASS=1: skip the two-pass backward; GSPN_FWD_NO_PAIR=1: skip the two-channel kernels (forward and the
// reverse sweep of the two-pass backward); GSPN_STREAM_NO_STAGED=1: the stream kernel whose horizontal phases request one
// row per lane instead of the one with whole-line requests; GSPN_FWD_NO_CHUNK=1: skip the per-stretch kernels of GSPN-local
// (forward and the reverse sweep of the two-pass backward); GSPN_STREAM_ONE_CHANNEL=1: the whole-line stream kernel with one
// channel per workgroup on the maps where two channels of a group normally share a workgroup; GSPN_STREAM_TWO_CHANNELS=1:
// two channels per workgroup there also in calls with too few planes to fill the chip that way.
enum : unsigned { K_FORCE_GENERIC = 1, K_FWD_NO_PLANE = 2, K_BWD_NO_PLANE = 4, K_BWD_NO_TWOPASS = 8, K_FWD_NO_PAIR = 16, K_STREAM_NO_STAGED = 32, K_FWD_NO_CHUNK = 64, K_STREAM_ONE_CHANNEL = 128, K_STREAM_TWO_CHANNELS = 256, K_VALID = 1u << 31 };
static std::atomic<unsigned> g_knobs{0};
static bool env_flag(const char* name) { const char* v = getenv(name); return v && v[0] == '1'; }
void reload_env_knobs() {
    unsigned k = K_VALID;
    if (env_flag("GSPN_FORCE_GENERIC")) k |= K_FORCE_GENERIC;
    if (env_flag("GSPN_FWD_NO_PLANE")) k |= K_FWD_NO_PLANE;
    if (env_flag("GSPN_BWD_NO_PLANE")) k |= K_BWD_NO_PLANE;
    if (env_flag("GSPN_BWD_NO_TWOPASS")) k |= K_BWD_NO_TWOPASS;
    if (env_flag("GSPN_FWD_NO_PAIR")) k |= K_FWD_NO_PAIR;
    if (env_flag("GSPN_STREAM_NO_STAGED")) k |= K_STREAM_NO_STAGED;
    if (env_flag("GSPN_FWD_NO_CHUNK")) k |= K_FWD_NO_CHUNK;
    if (env_flag("GSPN_STREAM_ONE_CHANNEL")) k |= K_STREAM_ONE_CHANNEL;
    if (env_flag("GSPN_STREAM_TWO_CHANNELS")) k |= K_STREAM_TWO_CHANNELS;
    g_knobs.store(k, std::memory_order_release);
}
struct Knobs { bool force_generic, fwd_no_plane, bwd_no_plane, bwd_no_twopass, fwd_no_pair, stream_no_staged, fwd_no_chunk, stream_one_channel, stream_two_channels; };
static Knobs knobs() {
    unsigned k = g_knobs.load(std::memory_order_acquire);
    if (!(k & K_VALID)) { reload_env_knobs(); k = g_knobs.load(std::memory_order_acquire); }
    return Knobs{(k & K_FORCE_GENERIC) != 0, (k & K_FWD_NO_PLANE) != 0, (k & K_BWD_NO_PLANE) != 0, (k & K_BWD_NO_TWOPASS) != 0, (k & K_FWD_NO_PAIR) != 0, (k & K_STREAM_NO_STAGED) != 0, (k & K_FWD_NO_CHUNK) != 0, (k & K_STREAM_ONE_CHANNEL) != 0, (k & K_STREAM_TWO_CHANNELS) != 0};
}
bool pair_kernels_enabled() { return !knobs().fwd_no_pair; }
bool staged_stream_enabled() { return !knobs().stream_no_staged; }
bool chunk_kernels_enabled() { return !knobs().fwd_no_chunk; }
bool stream_two_channels_enabled() { return !knobs().stream_one_channel; }
bool stream_two_channels_forced() { return knobs().stream_two_channels; }

static FwdPlan choose_fwd(const FwdParams& p, int dtype) {
    const Knobs k = knobs();
    if (k.force_generic) return FWD_GENERIC;
    // GSPN-local with few planes: the stretches as work items (Sec. 4.1), before any one-workgroup-per-plane kernel
    if (!k.fwd_no_chunk && fwd_chunk_applicable(p, dtype)) return FWD_CHUNK;
    if (!k.fwd_no_plane && fwd_plane_applicable(p, dtype)) {
        // the largest planes the plane kernel takes in 16-bit storage (more than 6.5 KB: 64x56, 64x64), forward without
        // h_save: the tile kernel was measured faster (B = 8, C = 768: 64x64 0.250 -> 0.207 ms, 64x56 0.233 -> 0.193 ms;
        // one image with 1152 channels 85 -> 56 us); with h_save, and from 56x56 down, the plane kernel is
        if (dtype != 0 && !p.hs && (size_t)p.H * p.W * 2 > 6656 && fwd_tile_applicable(p, dtype)) return FWD_TILE;
        return FWD_PLANE;
    }
    if (!k.fwd_no_pair && fwd_pair_applicable(p, dtype)) return FWD_PAIR;
    if (fwd_tile_applicable(p, dtype)) return FWD_TILE;
    return fwd_stream_applicable(p, dtype) ? FWD_STREAM : FWD_GENERIC;
}
static BwdPlan choose_bwd(const BwdParams& p, int dtype) {
    const Knobs k = knobs();
    if (k.force_generic) return BWD_GENERIC;
    const bool twopass = !k.bwd_no_twopass && bwd_twopass_applicable(p, dtype);
    if (!k.bwd_no_plane && bwd_plane_applicable(p, dtype)) {
        // the single-launch plane kernel, except where the two passes were measured faster: bf16 storage, shared
        // weights, lines of more than 16 positions (28x28x192, B = 64, G = 8: 382 -> 270 us; B = 32, G = 4, where a bf16
        // group cannot be split over workgroups: 1401 -> 177 us; 32x32x256 G = 16: 250 -> 73 us; the shorter lines of
        // the later classifier stages and the fp32 maps run as fast or faster on the plane kernel)
        const int m = p.H > p.W ? p.H : p.W;
        if (twopass && dtype != 0 && p.cpg > 1 && m > 16) return BWD_TWOPASS;
        return BWD_PLANE;
    }
    // the two-pass backward before the single-launch tile kernel: measured faster on every map both take (56x56x96
    // 506 -> 365 us bf16, 64x64x256 457 -> 186 us, 64x128x256 438 -> 193 us)
    if (twopass) return BWD_TWOPASS;
    // (the single-launch tile kernel exists in fp32 and bf16 storage)
    return (dtype != 2 && bwd_tile_applicable(p, dtype)) ? BWD_TILE : BWD_GENERIC;
}

hipError_t launch_fwd(const FwdParams& p, int dtype, hipStream_t s) {
    switch (choose_fwd(p, dtype)) {
        case FWD_TILE: return launch_fwd_tile(p, dtype, s);
        case FWD_STREAM: return launch_fwd_stream(p, dtype, s);
        case FWD_PLANE: return launch_fwd_plane(p, dtype, s);
        case FWD_PAIR: return launch_fwd_pair(p, dtype, s);
        case FWD_CHUNK: return launch_fwd_chunk(p, dtype, s);
        default: return launch_fwd_generic(p, dtype, s);
    }
}

hipError_t launch_bwd(const BwdParams& p, int dtype, hipStream_t s) {
    switch (choose_bwd(p, dtype)) {
        case BWD_TILE: return launch_bwd_tile(p, dtype, s);
        case BWD_PLANE: return launch_bwd_plane(p, dtype, s);
        case BWD_TWOPASS: return launch_bwd_twopass(p, dtype, s);
        default: return launch_bwd_generic(p, dtype, s);
    }
}

const char* fwd_plan_name(const FwdParams& p, int dtype) {
    switch (choose_fwd(p, dtype)) {
        case FWD_TILE: return "tile";
        case FWD_STREAM: return "stream";
        case FWD_PLANE: return "plane";
        case FWD_PAIR: return "pair";
        case FWD_CHUNK: return "chunk";
        default: return "generic";
    }
}

const char* bwd_plan_name(const BwdParams& p, int dtype) {
    switch (choose_bwd(p, dtype)) {
        case BWD_TILE: return "tile";
        case BWD_PLANE: return "plane";
        case BWD_TWOPASS: return "twopass";
        default: return "generic";
    }
}

}  // namespace gspn
