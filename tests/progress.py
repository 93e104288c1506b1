"""Progress lines of the long GPU tests.  pytest captures stdout and stderr at the file-descriptor
level, so a quiet run of several minutes looks hung from outside; `say` suspends the capture for the
one line it prints (conftest.py hands over pytest's capture manager)."""
import sys

capman = None


def say(msg):
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print(msg, file=sys.stderr, flush=True)
    else:
        print(msg, flush=True)
