// HEMV: complex Hermitian matrices.  The planner's instances for the complex
// types live here as well (its occupancy query names the Hermitian kernels).
#include "kmv_symv_impl.hpp"

namespace kmv {
template SymvPlan<cf32> plan_symv<cf32>(bool, int64_t, const void*, int64_t);
template SymvPlan<cf64> plan_symv<cf64>(bool, int64_t, const void*, int64_t);
template const SymvBalanced* symv_shares<cf32>(bool, int64_t, int, int, int, int64_t, int, int);
template const SymvBalanced* symv_shares<cf64>(bool, int64_t, int, int, int, int64_t, int, int);
template hipError_t launch_symv_kind<cf32, true>(const SymvArgs<cf32>&, bool, hipStream_t, int64_t);
template hipError_t launch_symv_kind<cf64, true>(const SymvArgs<cf64>&, bool, hipStream_t, int64_t);
}  // namespace kmv
