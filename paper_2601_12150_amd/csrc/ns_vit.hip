// Pre-LayerNorm transformer block around the sparse attention (not implemented yet).
#include "ns_common.h"

using namespace ns;

extern "C" {

size_t vit_block_workspace_bytes(const ns_vit_block_desc *desc) {
  (void)desc;
  return 0;
}

ns_status vit_block_forward(const ns_vit_block_desc *desc, const ns_vit_block_weights *weights,
                            const void *x_in, void *x_out, float *scores_out, void *workspace,
                            size_t workspace_bytes, void *stream) {
  (void)desc; (void)weights; (void)x_in; (void)x_out; (void)scores_out;
  (void)workspace; (void)workspace_bytes; (void)stream;
  return fail(NS_ERR_UNSUPPORTED, "vit_block_forward is not implemented in this build");
}

}  // extern "C"
