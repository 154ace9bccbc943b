// Device code of libsprnn: the persistent kernel's instantiations that consume the copy of h in two parts
// (options.overlap): forward pass of the vanilla cells at batch 1, 2 and 4; with the phase timeline at batch 4; and
// the instantiations with binary16 activations (options.activations): vanilla forward pass, batch 4 and 8.
#include "sprnn_persistent.h"

namespace sprnn {

const void* persistent_overlap_kernel_for(int batch, int template_words, bool timeline) {
  if (timeline) return batch == 4 ? pick_nw<4, 10, true>(template_words) : nullptr;
  switch (batch) {
    case 1: return pick_nw<1, 10, false>(template_words);
    case 2: return pick_nw<2, 10, false>(template_words);
    case 4: return pick_nw<4, 10, false>(template_words);
    default: return nullptr;
  }
}

const void* persistent_half_kernel_for(int batch, int template_words) {
  return batch == 4 ? pick_nw<4, 11, false>(template_words) : (batch == 8 ? pick_nw<8, 11, false>(template_words) : nullptr);
}

}  // namespace sprnn
