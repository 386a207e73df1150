// SYMV for the real precisions.
#include "kmv_symv_impl.hpp"

namespace kmv {
template SymvPlan<float> plan_symv<float>(bool, int64_t, const void*, int64_t);
template SymvPlan<double> plan_symv<double>(bool, int64_t, const void*, int64_t);
template const SymvBalanced* symv_shares<float>(bool, int64_t, int, int, int, int64_t, int, int);
template const SymvBalanced* symv_shares<double>(bool, int64_t, int, int, int, int64_t, int, int);
template hipError_t launch_symv_kind<float, false>(const SymvArgs<float>&, bool, hipStream_t, int64_t);
template hipError_t launch_symv_kind<double, false>(const SymvArgs<double>&, bool, hipStream_t, int64_t);
}  // namespace kmv
