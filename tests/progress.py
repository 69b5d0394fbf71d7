"""Step lines of the GPU tests ("[case] ..."), printed past pytest's output capture so that a long
test shows where it is while it runs (and names its case should the process die under it)."""
import sys

capture_manager = None   # set by conftest.pytest_configure


def say(*a):
    line = "[case] " + " ".join(str(x) for x in a)
    if capture_manager is not None:
        with capture_manager.global_and_fixture_disabled():
            print(line, flush=True)
    else:
        print(line, flush=True)
    sys.stdout.flush()
