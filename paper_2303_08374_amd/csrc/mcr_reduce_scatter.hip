// reduce_scatter over P rank buffers in one GPU's memory (API listing of the paper; it has no
// root): the dispatch over the element type.  The kernels are in mcr_reduce_scatter_impl.hpp,
// instantiated per element type in mcr_reduce_scatter_<type>.hip.
#include "mcr_dispatch.hpp"

namespace mcr {

template <int DT>
int launch_reduce_scatter_dt(const PtrTab& out, const CPtrTab& in, size_t count, int op, int P, int variant, int n_cu,
                             hipStream_t stream);
extern template int launch_reduce_scatter_dt<MCR_F32>(const PtrTab&, const CPtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_reduce_scatter_dt<MCR_BF16>(const PtrTab&, const CPtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_reduce_scatter_dt<MCR_F16>(const PtrTab&, const CPtrTab&, size_t, int, int, int, int, hipStream_t);
extern template int launch_reduce_scatter_dt<MCR_I32>(const PtrTab&, const CPtrTab&, size_t, int, int, int, int, hipStream_t);

int launch_reduce_scatter(mcr_ctx* ctx, const PtrTab& out, const CPtrTab& in, size_t count, int dtype,
                          int op, int P, int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  return dispatch_dtype(dtype, [&](auto dt) {
    return launch_reduce_scatter_dt<decltype(dt)::value>(out, in, count, op, P, variant, ctx->n_cu, stream);
  });
}

}  // namespace mcr
