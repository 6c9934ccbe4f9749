"""CPU oracle (test infrastructure only).  See block_transformer.py."""
from .block_transformer import *  # noqa: F401,F403
from . import block_transformer  # noqa: F401
