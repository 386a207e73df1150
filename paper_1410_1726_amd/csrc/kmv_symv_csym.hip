// SYMV for complex symmetric matrices: the kernels of the Hermitian product
// without the conjugation and with the diagonal taken as stored.
#include "kmv_symv_impl.hpp"

namespace kmv {
template hipError_t launch_symv_kind<cf32, false>(const SymvArgs<cf32>&, bool, hipStream_t, int64_t);
template hipError_t launch_symv_kind<cf64, false>(const SymvArgs<cf64>&, bool, hipStream_t, int64_t);
}  // namespace kmv
