// rd_tree_attn, bf16 path: tree-masked attention of the packed candidates against the KV
// cache (Sec. 3.3, 3.4) as a split-key flash kernel on the gfx950 matrix cores.
//
// Decoding attention is bound by streaming K and V from HBM (512 bytes per key and head at
// D = 128) while the packed rows (a few dozen to a few hundred) are reused for every key, so the kernel is
// organised around the stream:
//   * a workgroup (4 waves) owns a contiguous key range of one (sequence, head) and walks
//     it in blocks of 128 keys; wave w loads rows 32w..32w+31 of the block for K and for V
//     with fully coalesced 16-byte-per-lane loads (a wave instruction covers 1 KB of
//     consecutive rows), one block ahead of the arithmetic, and parks them in LDS;
//   * scores are produced transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: the wave
//     reads its own K tile back from LDS in the A-operand layout (XOR-swizzled, conflict
//     free) and Q (resident in LDS for the whole kernel) as the B operand;
//   * tree mask (bit test against tree_mask_bits) and range limits are applied to the
//     accumulators in registers, only in tiles that need them; the four waves exchange their
//     per-row tile maxima through LDS so the block has one running maximum per packed row
//     (online softmax, log2 units);
//   * the probabilities, rounded to bf16, are written to LDS already in B-operand layout;
//     the accumulator layout of S^T makes each lane's eight values exactly one B operand
//     once the 32 keys of a tile are taken in the order (4g+i, 16+4g+i);
//   * O^T = V^T P^T: wave w owns d-tiles 2w and 2w+1 (D = 128) for all 128 keys of the
//     block; the A operand V^T needs eight keys of one column per lane, which
//     ds_read_b64_tr_b16 (LDS transpose read) delivers from the row-major V tiles, taken in
//     the same key order.  The output accumulators therefore need no cross-wave reduction.
//   * the partial state goes to the workspace and the last workgroup of the head merges; a head
//     whose keys are all walked by one workgroup writes its output directly;
//   * beams too wide for one workgroup's registers are cut into row groups, each walking the
//     same keys (a workgroup = one key range x one row group).
#include "rd_tree_attn_mfma.h"

RD_TRACE_DEFINE(rd_debug_set_trace)

namespace rd {
int tree_attn_bf16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream)
{
    return tree_attn_mfma<__bf16, false>(a, D, waves, rg_tiles, stream);
}
}  // namespace rd
