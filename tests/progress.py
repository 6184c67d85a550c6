"""Progress lines of the long GPU tests, written past pytest's output capture.

A pass of the float64 oracle over an 80-layer decoder takes minutes; a runner that watches the test
process's output for signs of life must see the work advance, and under capture a test's prints only
appear after it has ended.  conftest.py hands over pytest's capture manager; without one (the scripts
that are run by name) the lines are plain prints.
"""
_capture_manager = None


def set_capture_manager(manager):
    global _capture_manager
    _capture_manager = manager


def say(*parts):
    if _capture_manager is not None:
        with _capture_manager.global_and_fixture_disabled():
            print(*parts, flush=True)
    else:
        print(*parts, flush=True)
