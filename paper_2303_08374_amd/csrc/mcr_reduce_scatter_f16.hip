// reduce_scatter kernels for one element type.
#include "mcr_reduce_scatter_impl.hpp"

namespace mcr {
template int launch_reduce_scatter_dt<MCR_F16>(const PtrTab&, const CPtrTab&, size_t, int, int, int, int, hipStream_t);
}  // namespace mcr
