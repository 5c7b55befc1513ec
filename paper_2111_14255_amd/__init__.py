"""MI355X-native staged multi-tenant CNN inference (arXiv 2111.14255): Python side of libmtsched.so."""
from . import binding  # noqa: F401
