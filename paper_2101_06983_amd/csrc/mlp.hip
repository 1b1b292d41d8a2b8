// Stand-in encoder kernels (Step 1 forward, Step 3 surrogate backward).  Placeholder until written.
#include "gc_common.h"
extern "C" {
size_t gc_mlp_workspace_bytes(int rows, const gc_mlp_params* w) { (void)rows; (void)w; return 0; }
int gc_mlp_forward_nograd_bf16(const void*, int, const gc_mlp_params*, void*, void*, size_t, void*) { return GC_ERR_UNSUPPORTED; }
int gc_chunk_surrogate_backward_bf16(const void*, int, const gc_mlp_params*, const float*, const gc_mlp_grads*, void*, size_t, void*) { return GC_ERR_UNSUPPORTED; }
size_t gc_step_mlp_workspace_bytes(int, int, int, int, const gc_mlp_params*) { return 0; }
int gc_step_mlp_bf16(const void*, int, const void*, int, const int32_t*, int, int, const gc_mlp_params*, float, float, float*, const gc_mlp_grads*, void*, void*, float*, float*, void*, size_t, void*) { return GC_ERR_UNSUPPORTED; }
}
