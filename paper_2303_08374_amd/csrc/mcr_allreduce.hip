// all_reduce over P rank buffers in one GPU's memory (API listing of the paper): the dispatch
// over the element type.  The kernels are in mcr_allreduce_impl.hpp, instantiated per element
// type in mcr_allreduce_<type>.hip.
#include "mcr_dispatch.hpp"

namespace mcr {

template <int DT>
int launch_allreduce_dt(const PtrTab& bufs, size_t count, unsigned head, int op, int P, int root, int variant, int n_cu,
                        hipStream_t stream);
extern template int launch_allreduce_dt<MCR_F32>(const PtrTab&, size_t, unsigned, int, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_BF16>(const PtrTab&, size_t, unsigned, int, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_F16>(const PtrTab&, size_t, unsigned, int, int, int, int, int, hipStream_t);
extern template int launch_allreduce_dt<MCR_I32>(const PtrTab&, size_t, unsigned, int, int, int, int, int, hipStream_t);

// `head`: elements of the message that lie in front of bufs (see the kernel); 0 for the element path.
int launch_allreduce(mcr_ctx* ctx, const PtrTab& bufs, size_t count, unsigned head, int dtype, int op, int P, int root,
                     int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  return dispatch_dtype(dtype, [&](auto dt) {
    return launch_allreduce_dt<decltype(dt)::value>(bufs, count, head, op, P, root, variant, ctx->n_cu, stream);
  });
}

}  // namespace mcr
