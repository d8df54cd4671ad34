"""CPU oracle (test infrastructure only; see flashcache_ref.py)."""
from . import flashcache_ref  # noqa: F401
