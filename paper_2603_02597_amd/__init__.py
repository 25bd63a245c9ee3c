"""MI355X-native byte-level BPE merge loop (HIP library + thin ctypes binding)."""
from .binding import (  # noqa: F401
    BpeError,
    EncodeOptions,
    Pool,
    Table,
    bpe_encode,
    bpe_encode_status,
    bpe_encode_timed,
    KERNEL_NAMES,
    bpe_table_build,
    bpe_table_capacity,
    bpe_table_image_build,
    bpe_table_lookup,
    bpe_workspace_bytes,
    encode,
    library_path,
    load_library,
)
