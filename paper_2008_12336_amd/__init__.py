"""MI355X-native GOSH training path: HIP kernels behind a C ABI (libgosh.so) and a
ctypes binding with the same entry-point names."""
from .binding import (  # noqa: F401
    GOSH_FLAG_ATOMIC_ADDS,
    GOSH_FLAG_PLAIN_STORES,
    GOSH_FLAG_SEQUENTIAL,
    GOSH_MAX_DIM,
    GOSH_MAX_NEG,
    GoshError,
    Hierarchy,
    csr_view,
    gosh_coarsen,
    gosh_csr,
    gosh_csr_validate,
    gosh_embed,
    gosh_epoch_split,
    gosh_init_embedding,
    gosh_last_error,
    gosh_lr,
    gosh_project,
    gosh_sample_epoch,
    gosh_train_epoch,
    lib,
)
