"""MI355X-native tile level-3 BLAS on host-resident matrices (single-GPU hot path of BLASX).

``blasx`` is the binding of the C ABI declared in ``include/blasx.h``; the HIP library is
built by ``__graft_entry__.build()`` into ``paper_1510_05041_amd/libblasx.so``.
"""
from . import blasx  # noqa: F401
from .blasx import (BlasxError, HostBuffer, ColMajor, ConjTrans, Left, Library, Lower, NonUnit, NoTrans, Right,  # noqa: F401
                    RowMajor, Trans, Unit, Upper, default, pinned_matrix)
