"""MI355X-native BitStack linear layer: thin ctypes binding over libbitstack.so.

Every step of the forward pass runs inside the HIP library; this package only
marshals arguments.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    BitStackError,
    PackedStack,
    BlockManager,
    TokenPlan,
    order_check,
    budget_position,
    KERNEL_AUTO, KERNEL_REFERENCE, KERNEL_DECODE, KERNEL_PANEL, KERNEL_MATERIALISE,
    OPT_DECODE_BGROUPS, OPT_DECODE_TILES, OPT_DECODE_KS_CHUNKS, OPT_DECODE_EARLY, OPT_DENSE_TILE,
    block_bytes,
    block_staging_bytes,
    dense_bytes,
    decompose,
    choose_kernel,
    restore_max_blocks,
    stage_block_host,
    lib,
    linear_many,
    make_jobs,
    lib_path,
    pack_image_host,
    pack_signs_from_f32,
    packed_bytes,
    probe_read,
    set_option,
    strerror,
    unpack_image_host,
)
