// Device code of libsprnn: instantiations of the lane-pool kernel (sprnn_pool.h), forward pass.
#include "sprnn_pool.h"

namespace sprnn {

const void* pool_backward_kernel_for(int batch, int template_words);
const void* pool_backward_grad_kernel_for(int batch, int template_words);

const void* pool_kernel_for(int batch, int template_words, int cell, bool timeline) {
  if (timeline) return (batch == 4 && cell >= SPRNN_ACT_RELU && cell <= SPRNN_ACT_IDENTITY) ? pick_pool_nw<4, 0, true>(template_words) : nullptr;
  if (cell == kCellBackward) return pool_backward_kernel_for(batch, template_words);
  if (cell == kCellBackwardGrad) return pool_backward_grad_kernel_for(batch, template_words);
  if (cell >= SPRNN_ACT_RELU && cell <= SPRNN_ACT_IDENTITY) return pick_pool_b<0>(batch, template_words);
  return nullptr;
}

}  // namespace sprnn
