// Device code of libsprnn: instantiations of the lane-pool kernel (sprnn_pool.h), backward pass through time.
#include "sprnn_pool.h"

namespace sprnn {

const void* pool_backward_kernel_for(int batch, int template_words) { return pick_pool_b<3>(batch, template_words); }

}  // namespace sprnn
