import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def _reload_library_env():
    """The library reads its GSPN_* testing aids once per process; tell it that they changed."""
    from paper_2512_07884_amd import binding
    if os.path.exists(binding.lib_path()):
        binding.gspn_reload_env()


@pytest.fixture
def monkeypatch(monkeypatch):
    """pytest's monkeypatch, with one addition: a change to a GSPN_* environment variable reaches the library."""
    setenv, delenv = monkeypatch.setenv, monkeypatch.delenv

    def setenv_and_reload(name, value, prepend=None):
        setenv(name, value, prepend)
        if name.startswith("GSPN_"):
            _reload_library_env()

    def delenv_and_reload(name, raising=True):
        delenv(name, raising)
        if name.startswith("GSPN_"):
            _reload_library_env()

    monkeypatch.setenv = setenv_and_reload
    monkeypatch.delenv = delenv_and_reload
    yield monkeypatch
    monkeypatch.undo()
    _reload_library_env()
