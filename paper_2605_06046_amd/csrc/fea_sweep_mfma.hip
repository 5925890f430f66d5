#include <hip/hip_runtime.h>
#include "fea_plan.h"
namespace fea {
void launch_sweep_mfma(const SweepArgs&, int, void*) {}
}
