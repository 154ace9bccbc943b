// Device code of libsprnn: instantiations of the lane-pool kernel (sprnn_pool.h), backward pass with the weight gradient fused in.
#include "sprnn_pool.h"

namespace sprnn {

const void* pool_backward_grad_kernel_for(int batch, int template_words) { return pick_pool_b<4>(batch, template_words); }

}  // namespace sprnn
