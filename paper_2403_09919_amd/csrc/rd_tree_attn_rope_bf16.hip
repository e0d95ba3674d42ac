// rd_tree_attn_rope, bf16: the MFMA kernel of rd_tree_attn_mfma.h instantiated with the rotary
// embedding applied in the kernel (query rows on their way into LDS, packed keys as their tiles are
// walked), for LLaMA-family LLMs such as the paper's Vicuna models (Sec. 4).
#include "rd_tree_attn_mfma.h"

RD_TRACE_DEFINE(rd_debug_set_trace_rope_bf16)

namespace rd {
int tree_attn_rope_bf16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream)
{
    return tree_attn_mfma<__bf16, false, true>(a, D, waves, rg_tiles, stream);
}
}  // namespace rd
