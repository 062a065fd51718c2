"""Progress lines of the GPU tests, printed past pytest's capture."""
CAPTURE_MANAGER = None      # set by conftest.pytest_configure


def say(msg):
    """Names the case (and marks progress of the long ones) on the real terminal: if a GPU step takes
    the machine down, the last line printed says which case it was."""
    if CAPTURE_MANAGER is None:
        print(msg, flush=True)
        return
    with CAPTURE_MANAGER.global_and_fixture_disabled():
        print(msg, flush=True)
