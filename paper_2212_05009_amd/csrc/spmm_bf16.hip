// bf16-feature instances of the sparse-times-dense kernel (fp32 accumulation).
#include "spmm_kernel.h"

namespace gcn {
int spmm_dispatch_bf16(SpmmK& k, const Schedule* sc, const SpmmProf& pf, int V, bool narrow, hipStream_t s) {
  switch (V) {
    case 8: return launch_v<bf16_t, 8>(k, sc, pf, narrow, s);
    case 4: return launch_v<bf16_t, 4>(k, sc, pf, narrow, s);
    case 2: return launch_v<bf16_t, 2>(k, sc, pf, narrow, s);
    default: return launch_v<bf16_t, 1>(k, sc, pf, narrow, s);
  }
}
}  // namespace gcn
