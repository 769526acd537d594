// Instantiations of the fused attention kernel with the lazily renewed reference maximum
// (rescale_margin > 0 of the configuration; an extension), protected and unprotected, kept apart
// from the main translation unit so that they compile side by side.
#include "ftattn_main.h"

namespace ftattn {

template <int D, bool FT, bool INJ>
static void (*pick_lazy(bool causal))(const KArgs) {
  return causal ? ftattn_main<D, FT, true, INJ, 4> : ftattn_main<D, FT, false, INJ, 4>;
}

template <int D>
static void (*by_flags(bool ft, bool causal, bool inject))(const KArgs) {
  if (ft) return inject ? pick_lazy<D, true, true>(causal) : pick_lazy<D, true, false>(causal);
  return inject ? pick_lazy<D, false, true>(causal) : pick_lazy<D, false, false>(causal);
}

void (*select_lazy(int D, bool ft, bool causal, bool inject))(const KArgs) {
  if (D == 128) return by_flags<128>(ft, causal, inject);
  if (D == 64) return by_flags<64>(ft, causal, inject);
  return nullptr;
}

}  // namespace ftattn
