"""Fused primitive operators of Relay-compiled vision models on MI355X (gfx950).

``binding`` exposes the C entry points of librelayfused.so one to one; ``stack`` chains
them into ResNet-/MobileNet-shaped networks.  Importing the package loads nothing; the
first call loads the library and raises if it has not been built.
"""
from . import binding  # noqa: F401
