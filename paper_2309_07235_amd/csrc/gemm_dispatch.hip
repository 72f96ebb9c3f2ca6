// Central switch from a runtime schedule to the per-tile translation units.
#include "gemm_dispatch.hpp"
#include "dla_codes.hpp"

namespace dla {

#define DLA_DECL(TM, TN, WM, WN)                                                                           \
  template <>                                                                                              \
  int launch_gemm_tile<double, TM, TN, WM, WN>(const GemmSchedule&, int, const GemmGroup<double>&,        \
                                               hipStream_t);                                               \
  template <>                                                                                              \
  int launch_gemm_tile<float, TM, TN, WM, WN>(const GemmSchedule&, int, const GemmGroup<float>&, hipStream_t);
DLA_TILE_MENU(DLA_DECL)
#undef DLA_DECL

template <typename T>
int launch_gemm(const GemmSchedule& s, int op, const GemmGroup<T>& g, hipStream_t st) {
  if (g.total_tiles <= 0) return DLA_SUCCESS;
#define DLA_CASE(TM, TN, WM, WN) \
  if (s.tm == TM && s.tn == TN && s.wm == WM && s.wn == WN) return launch_gemm_tile<T, TM, TN, WM, WN>(s, op, g, st);
  DLA_TILE_MENU(DLA_CASE)
#undef DLA_CASE
  return DLA_ERR_UNSUPPORTED_PARAMS;
}

template int launch_gemm<double>(const GemmSchedule&, int, const GemmGroup<double>&, hipStream_t);
template int launch_gemm<float>(const GemmSchedule&, int, const GemmGroup<float>&, hipStream_t);

}  // namespace dla
