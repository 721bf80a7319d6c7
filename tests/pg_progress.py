"""Progress lines that reach the terminal while pytest captures output: the full-size GPU tests run the CPU
checker for minutes, and a run that prints nothing for that long looks hung from outside."""
_config = None


def set_config(config):
    global _config
    _config = config


def say(msg):
    capman = _config.pluginmanager.getplugin("capturemanager") if _config is not None else None
    if capman is None:
        print(msg, flush=True)
        return
    with capman.global_and_fixture_disabled():
        print(msg, flush=True)
