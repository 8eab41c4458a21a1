// placeholder until the MFMA streaming kernel lands
#include "plan.h"
namespace dsattn {
bool mfma_plan(dsattn_plan_t &) { return false; }
hipError_t launch_mfma(const dsattn_plan_t &, const void *, const void *, const void *, void *, hipStream_t) { return hipErrorNotSupported; }
}
