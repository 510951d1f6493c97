// Explicit instantiations of the main bf16 attention kernel's launchers for one head size and one
// set of group sizes, chosen by the build (see build.py):
//   -DPV_INST_D=<64|128>  -DPV_INST_SET=<0..3>
// set 0: G = 1, 2, 3;  set 1: G = 4 and the query-tile launcher;  set 2: G = 5, 6, 7;  set 3: G = 8.
#include "pv_attn_bf16_main.h"

#if !defined(PV_INST_D) || !defined(PV_INST_SET)
#error "compile with -DPV_INST_D=<64|128> -DPV_INST_SET=<0..3>"
#endif

namespace pv {

#define PV_INST(GG)                                                                               \
  template hipError_t launch_main<PV_INST_D, GG>(                                                 \
      const int32_t*, const PlanHeader&, const uint16_t*, const uint16_t*, const uint16_t*,       \
      const float2*, void*, float*, int, int, float, bool, bool, int, float*, hipStream_t);

#if PV_INST_SET == 0
PV_INST(1) PV_INST(2) PV_INST(3)
#elif PV_INST_SET == 1
PV_INST(4)
template hipError_t launch_query_tiles<PV_INST_D>(const int32_t*, const PlanHeader&, const uint16_t*,
                                                  const uint16_t*, const uint16_t*, const float2*,
                                                  void*, float*, int, int, float, bool, bool,
                                                  hipStream_t);
#elif PV_INST_SET == 2
PV_INST(5) PV_INST(6) PV_INST(7)
#elif PV_INST_SET == 3
PV_INST(8)
#else
#error "PV_INST_SET must be 0..3"
#endif

}  // namespace pv
