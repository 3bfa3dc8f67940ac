"""Progress lines that reach the terminal while pytest captures output: a full-size GPU case runs for minutes, and
a run that prints nothing for minutes looks hung to whatever watches it."""
from __future__ import annotations

_capman = None


def bind(config) -> None:
    global _capman
    _capman = config.pluginmanager.getplugin("capturemanager")


def say(*parts) -> None:
    msg = " ".join(str(p) for p in parts)
    if _capman is not None:
        with _capman.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)
