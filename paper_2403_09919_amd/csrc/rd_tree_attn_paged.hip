// rd_tree_attn_paged: the MFMA kernel of rd_tree_attn_mfma.h instantiated for a paged KV cache
// (context keys and values in fixed-size pages found through a block table), bf16 and fp16.
#include "rd_tree_attn_mfma.h"

RD_TRACE_DEFINE(rd_debug_set_trace_paged)

namespace rd {
int tree_attn_paged(const AttnArgs &a, int D, int waves, int rg_tiles, bool f16, hipStream_t stream)
{
    return f16 ? tree_attn_mfma<_Float16, true>(a, D, waves, rg_tiles, stream)
               : tree_attn_mfma<__bf16, true>(a, D, waves, rg_tiles, stream);
}
}  // namespace rd
