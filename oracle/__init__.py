"""CPU oracle (test infrastructure only; the product path never imports this)."""
from .oracle import *  # noqa: F401,F403
