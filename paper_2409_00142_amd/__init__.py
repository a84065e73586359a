"""MI355X (gfx950) Dynamic Depth Decoding draft-round library: thin Python binding over libddd.so.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/ddd.h;
this package only marshals arguments (torch tensors -> device pointers, streams).
"""
from .binding import *  # noqa: F401,F403
