"""The shared harness helpers (harness.py at the repository root) under the name the tests use."""
from harness import *  # noqa: F401,F403
from harness import NAMES  # noqa: F401
