// Instantiations of the fused attention kernel in its ablation modes: verification after every
// step (the paper's EFTA before the unified verification of Section 3.4; optionally with its
// duplicated softmax), kept apart from the main translation unit so that the two compile side by
// side.  The traditional-checksum mode is in a third translation unit.
#include "ftattn_main.h"

namespace ftattn {

template <int D, bool INJ, int MODE>
static void (*pick_perstep(bool causal))(const KArgs) {
  return causal ? ftattn_main<D, true, true, INJ, MODE> : ftattn_main<D, true, false, INJ, MODE>;
}

template <int MODE>
static void (*by_shape(int D, bool causal, bool inject))(const KArgs) {
  if (D == 128) return inject ? pick_perstep<128, true, MODE>(causal) : pick_perstep<128, false, MODE>(causal);
  if (D == 64) return inject ? pick_perstep<64, true, MODE>(causal) : pick_perstep<64, false, MODE>(causal);
  return nullptr;
}

// mode 1: verification after every step; mode 2: the same with the softmax protected by duplication
void (*select_perstep(int D, bool causal, bool inject, int mode))(const KArgs) {
  return mode == 2 ? by_shape<2>(D, causal, inject) : by_shape<1>(D, causal, inject);
}

}  // namespace ftattn
