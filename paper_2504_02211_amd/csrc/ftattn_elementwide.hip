// Instantiations of the fused attention kernel with the traditional checksum (one class per tile
// row, stride 1 of eq. (13)) in place of the strided one: the comparison of Sections 3.3 and 4.2.
#include "ftattn_main.h"

namespace ftattn {

template <int D, bool INJ>
static void (*pick_elementwide(bool causal))(const KArgs) {
  return causal ? ftattn_main<D, true, true, INJ, 3> : ftattn_main<D, true, false, INJ, 3>;
}

void (*select_elementwide(int D, bool causal, bool inject))(const KArgs) {
  if (D == 128) return inject ? pick_elementwide<128, true>(causal) : pick_elementwide<128, false>(causal);
  if (D == 64) return inject ? pick_elementwide<64, true>(causal) : pick_elementwide<64, false>(causal);
  return nullptr;
}

}  // namespace ftattn
