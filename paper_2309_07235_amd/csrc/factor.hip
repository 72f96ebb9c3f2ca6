// placeholder: factorisation drivers come next
#include "host_common.hpp"
namespace dla {
int resolve_factor_params(dla_dtype dt, int64_t n, const dla_factor_params* in, int op, int* nb, int* lookahead,
                          GemmSchedule* upd) {
  (void)n;
  *nb = (in && in->nb) ? in->nb : 128;
  *lookahead = 0;
  return resolve_schedule(dt, in ? &in->update : nullptr, op, upd);
}
size_t factor_workspace_bytes_impl(int64_t, dla_dtype, const dla_factor_params*) { return 256; }
template <typename T>
int lu_factor_impl(T*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*) { return DLA_ERR_UNSUPPORTED_PARAMS; }
template <typename T>
int cholesky_factor_impl(T*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*) { return DLA_ERR_UNSUPPORTED_PARAMS; }
template int lu_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*);
template int lu_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*);
template int cholesky_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*);
template int cholesky_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t, int*);
}
