// rd_tree_attn, fp16 path: the MFMA kernel of rd_tree_attn_mfma.h instantiated for IEEE half
// K/V/Q (v_mfma_f32_16x16x32_f16; probabilities are rounded to fp16 before P.V, accumulation and
// softmax statistics stay fp32 exactly as in the bf16 path).
#include "rd_tree_attn_mfma.h"

RD_TRACE_DEFINE(rd_debug_set_trace_f16)

namespace rd {
int tree_attn_f16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream)
{
    return tree_attn_mfma<_Float16, false>(a, D, waves, rg_tiles, stream);
}
}  // namespace rd
