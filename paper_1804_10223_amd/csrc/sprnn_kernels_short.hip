// Device code of libsprnn: the persistent kernel's forward instantiations for layers whose h takes at most three
// rounds of the copy (vanilla cells, LSTM, GRU; all batch sizes): the copy issues exactly as many loads as h needs.
#include "sprnn_persistent.h"

namespace sprnn {

const void* persistent_short_kernel_for(int batch, int template_words, int cell) {
  if (cell == SPRNN_CELL_LSTM) return pick_b<13, false>(batch, template_words);
  if (cell == SPRNN_CELL_GRU) return pick_b<14, false>(batch, template_words);
  if (cell >= SPRNN_ACT_RELU && cell <= SPRNN_ACT_IDENTITY) return pick_b<12, false>(batch, template_words);
  return nullptr;
}

}  // namespace sprnn
