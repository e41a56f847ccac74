"""MI355X-native prover hot path of TensorCommitments (tensor commitments + Terkle trees).

The package is a thin ctypes binding over `libtc.so` (hand-written HIP for gfx950,
C ABI in include/tc.h).  There is no CPU path: importing works anywhere, but creating a
context needs the built library and a GPU."""
from .binding import (  # noqa: F401
    TC_F16,
    TC_FR,
    TC_I8,
    TC_I16,
    TC_INTERP_BARYCENTRIC,
    TC_INTERP_GREGORY,
    TC_INTERP_NEWTON,
    TC_LEAF_ENTRIES,
    TC_LEAF_TENSORS,
    TC_OK,
    TC_SRS_FIXED_BASE,
    TC_SRS_MONOMIAL,
    TC_SRS_OPEN_TABLE,
    TC_SRS_SUFFIX,
    Context,
    PairingVerifier,
    Srs,
    TcError,
    Tree,
    library_path,
    load_library,
)
