"""MI355X-native Multipole Attention decode path (C-ABI library + thin binding)."""
from . import inputs  # noqa: F401
