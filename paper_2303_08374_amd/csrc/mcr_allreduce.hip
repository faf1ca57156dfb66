// all_reduce over P rank buffers in one GPU's memory (API listing of the paper): the dispatch
// over the element type.  The kernels are in mcr_allreduce_impl.hpp, instantiated per element
// type in mcr_allreduce_<type>.hip.
#include "mcr_dispatch.hpp"

namespace mcr {

template <int DT>
int launch_allreduce_dt(const PtrTab& bufs, size_t count, int op, int P, int root, int variant, hipStream_t stream);
extern template int launch_allreduce_dt<MCR_F32>(const PtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_BF16>(const PtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_F16>(const PtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_I32>(const PtrTab&, size_t, int, int, int, int, hipStream_t);

int launch_allreduce(mcr_ctx*, const PtrTab& bufs, size_t count, int dtype, int op, int P, int root,
                     int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  return dispatch_dtype(dtype, [&](auto dt) {
    return launch_allreduce_dt<decltype(dt)::value>(bufs, count, op, P, root, variant, stream);
  });
}

}  // namespace mcr
