"""paper_2310_17723_amd: Python binding of libhero, the MI355X-native W8A8 transformer
layer forward of ZeroQuant-HERO (arXiv 2310.17723).

The binding only marshals arguments: every step of the path runs in the HIP kernels of
``libhero.so`` (C ABI in ``include/hero.h``).  PyTorch is used for device memory and
streams.  There is no CPU fallback: ``load()`` raises if the library is missing.
"""
from __future__ import annotations

import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhero.so")

_hero = None


def load():
    """Load libhero.so (built beforehand with ``python -m paper_2310_17723_amd.build``)."""
    global _hero
    if _hero is None:
        from .binding import Hero
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2310_17723_amd.build` "
                               "(there is no fallback path)")
        _hero = Hero(LIB_PATH)
    return _hero
