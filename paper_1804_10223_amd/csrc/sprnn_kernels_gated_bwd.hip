// Device code of libsprnn: the persistent kernel's instantiations for the backward pass through time of the gated
// cells (LSTM and GRU, each plain and with the weight gradient fused in).
#include "sprnn_persistent.h"

namespace sprnn {

const void* persistent_gated_backward_kernel_for(int batch, int template_words, int cell) {
  if (cell == SPRNN_CELL_LSTM_BACKWARD) return pick_b<5, false>(batch, template_words);
  if (cell == kCellLstmBackwardGrad) return pick_b<6, false>(batch, template_words);
  if (cell == SPRNN_CELL_GRU_BACKWARD) return pick_b<7, false>(batch, template_words);
  if (cell == kCellGruBackwardGrad) return pick_b<8, false>(batch, template_words);
  return nullptr;
}

}  // namespace sprnn
