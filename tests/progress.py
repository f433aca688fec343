"""Progress lines for the long parity runs.  Under pytest's output capture a test that runs the
oracle for minutes prints nothing, and a harness that watches the output takes it for hung:
`say` writes through the capture."""
import time

capman = None          # set by conftest.pytest_configure
_last = [0.0]


def say(msg):
    _last[0] = time.monotonic()
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print("\n" + msg, end="", flush=True)
    else:
        print(msg, flush=True)


def tick(msg, every=20.0):
    """`say`, but at most once per `every` seconds."""
    if time.monotonic() - _last[0] >= every:
        say(msg)
