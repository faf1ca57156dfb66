// all_reduce kernels for one element type.
#include "mcr_allreduce_impl.hpp"

namespace mcr {
template int launch_allreduce_dt<MCR_I32>(const PtrTab&, size_t, unsigned, int, int, int, int, int, hipStream_t);
}  // namespace mcr
