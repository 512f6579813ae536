import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (HIP library is called)")


def pytest_runtest_setup(item):
    """Name every GPU case on the terminal before it touches the device, so that a run the
    device ends abruptly still says which case it was in."""
    if item.get_closest_marker("gpu") is None:
        return
    reporter = item.config.pluginmanager.getplugin("terminalreporter")
    capture = item.config.pluginmanager.getplugin("capturemanager")
    if reporter is not None and capture is not None:
        with capture.global_and_fixture_disabled():
            reporter.ensure_newline()
            reporter.write(f"[gpu case] {item.nodeid}\n", flush=True)
