// bf16 MFMA causal attention for gfx950 -- placeholder until the tiled kernels land: reports "unsupported".
#include "pp_kernels.h"
namespace pp {
int k_attn_fwd_mfma(hipStream_t, const void*, void*, float*, int, int, int, int) { return 1; }
int k_attn_bwd_mfma(hipStream_t, const void*, const void*, const float*, const void*, void*, float*, int, int, int, int) { return 1; }
}
