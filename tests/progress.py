"""Progress lines of the long GPU tests: written past pytest's output capture, so that a run that is watched for
signs of life (the full-size cases spend a minute or two in the CPU oracle) shows what it is doing."""
import sys

capture_manager = None   # set by conftest.pytest_configure


def say(msg):
    cm = capture_manager
    if cm is not None:
        cm.suspend_global_capture(in_=False)
    try:
        sys.stdout.write(f"\n[{msg}]")
        sys.stdout.flush()
    finally:
        if cm is not None:
            cm.resume_global_capture()
