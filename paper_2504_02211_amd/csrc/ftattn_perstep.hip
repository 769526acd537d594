// Instantiations of the fused attention kernel with verification after every step (the paper's
// EFTA before the unified verification of Section 3.4), kept apart from the main translation unit
// so that the two compile side by side.
#include "ftattn_main.h"

namespace ftattn {

template <int D, bool INJ>
static void (*pick_perstep(bool causal))(const KArgs) {
  return causal ? ftattn_main<D, true, true, INJ, true> : ftattn_main<D, true, false, INJ, true>;
}

void (*select_perstep(int D, bool causal, bool inject))(const KArgs) {
  if (D == 128) return inject ? pick_perstep<128, true>(causal) : pick_perstep<128, false>(causal);
  if (D == 64) return inject ? pick_perstep<64, true>(causal) : pick_perstep<64, false>(causal);
  return nullptr;
}

}  // namespace ftattn
