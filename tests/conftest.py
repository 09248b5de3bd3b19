import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest


@pytest.fixture
def knobs(monkeypatch):
    """Sets diagnostic settings of the library through the environment.  The library reads its settings once and
    again after lstm_shutdown(), so every change is followed by one: knobs(LSTM_NO_PAD="1"), knobs(LSTM_NO_PAD=None)."""
    from paper_1604_01946_amd import binding

    def set_(**kv):
        for k, v in kv.items():
            if v is None:
                monkeypatch.delenv(k, raising=False)
            else:
                monkeypatch.setenv(k, str(v))
        binding.lstm_shutdown()

    yield set_
    monkeypatch.undo()
    binding.lstm_shutdown()
