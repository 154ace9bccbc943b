// Device code of libsprnn: the persistent kernel's instantiations for the backward pass through time of the vanilla
// cells, plain and with the weight gradient fused in.
#include "sprnn_persistent.h"

namespace sprnn {

const void* persistent_backward_kernel_for(int batch, int template_words, int cell) {
  if (cell == kCellBackward) return pick_b<3, false>(batch, template_words);
  if (cell == kCellBackwardGrad) return pick_b<4, false>(batch, template_words);
  return nullptr;
}

}  // namespace sprnn
