// Device code of libsprnn: the persistent kernel's instantiations with the phase timeline (options.timeline), forward
// pass of the vanilla cells and the LSTM.
#include "sprnn_persistent.h"

namespace sprnn {

// (also home of the narrow-gather instantiations of the ablation: batch 4, vanilla forward)
const void* persistent_narrow_kernel_for(int batch, int template_words) {
  return batch == 4 ? pick_nw<4, 9, false>(template_words) : nullptr;
}

const void* persistent_timeline_kernel_for(int batch, int template_words, bool lstm) {
  return lstm ? pick_b<1, true>(batch, template_words) : pick_b<0, true>(batch, template_words);
}

}  // namespace sprnn
