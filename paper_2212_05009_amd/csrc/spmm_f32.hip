// fp32-feature instances of the sparse-times-dense kernel.
#include "spmm_kernel.h"

namespace gcn {
int spmm_dispatch_f32(SpmmK& k, const Schedule* sc, const SpmmProf& pf, int V, bool narrow, hipStream_t s) {
  switch (V) {
    case 4: return launch_v<float, 4>(k, sc, pf, narrow, s);
    case 2: return launch_v<float, 2>(k, sc, pf, narrow, s);
    default: return launch_v<float, 1>(k, sc, pf, narrow, s);
  }
}
}  // namespace gcn
