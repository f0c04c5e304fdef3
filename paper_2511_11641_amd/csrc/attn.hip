// Attention block (placeholder until the kernels land): reports an unsupported configuration.
#include "block.h"

int attn_forward(ecospa_ctx*, const ecospa_block_desc&, const BlockWs&, const void*, void*, const ecospa_saved*) {
  return ECOSPA_ERR_DTYPE;
}
int attn_backward(ecospa_ctx*, const ecospa_block_desc&, const BlockWs&, const void*, const void*, const ecospa_saved&,
                  void*, const ecospa_grads&) {
  return ECOSPA_ERR_DTYPE;
}
