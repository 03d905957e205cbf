"""MI355X-native batched 2D rigid-body step (hand-written HIP behind the C ABI of include/k2d.h)."""
from .binding import Batch, get_layout, lib, pack_scenes, state_bytes, unpack_state  # noqa: F401
