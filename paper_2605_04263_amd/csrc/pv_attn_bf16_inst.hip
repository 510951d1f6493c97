// Explicit instantiations of the main bf16 attention kernel's launchers for one head size and one
// group size, chosen by the build (see build.py):
//   -DPV_INST_D=<64|128>  -DPV_INST_SET=<1..9>
// set G (1..8): the launcher of group size G;  set 9: the query-tile launcher.
#include "pv_attn_bf16_main.h"

#if !defined(PV_INST_D) || !defined(PV_INST_SET)
#error "compile with -DPV_INST_D=<64|128> -DPV_INST_SET=<1..9>"
#endif

namespace pv {

#define PV_INST(GG)                                                                               \
  template hipError_t launch_main<PV_INST_D, GG>(                                                 \
      const int32_t*, const PlanHeader&, const uint16_t*, const uint16_t*, const uint16_t*,       \
      const float2*, void*, float*, int, int, float, bool, bool, int, float*, const KvSource&, float,  \
      int, hipStream_t);

#if PV_INST_SET >= 1 && PV_INST_SET <= 8
PV_INST(PV_INST_SET)
#elif PV_INST_SET == 9
template hipError_t launch_query_tiles<PV_INST_D>(const int32_t*, const PlanHeader&, const uint16_t*,
                                                  const uint16_t*, const uint16_t*, const float2*,
                                                  void*, float*, int, int, float, bool, bool,
                                                  const KvSource&, float, int, hipStream_t);
#else
#error "PV_INST_SET must be 1..9"
#endif

}  // namespace pv
