// Tree-drafting regime of the draft head (hundreds to a thousand hidden-state rows): the
// projection of Section 2.3 of the paper, z[r,j] = sum_i h[r,i] W_sub[j,i], is now a dense
// contraction with ~500-1000 FLOP per byte and runs on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// MFMA roles: the A operand is a W_sub tile (matrix rows = draft tokens), the B operand an h
// tile (matrix columns = hidden-state rows).  In the 32x32 accumulator layout a lane then owns
// ONE hidden-state row (column l%32) and 16 draft tokens per sub-tile, so the fused epilogue
// (softmax statistics and the k best candidates over the tile's vocabulary slice) runs
// lane-private on the accumulators with no shuffles and no LDS, in ascending token order.
// Each lane's partial goes to the workspace; the merge kernel finishes the row.  Logits are
// never written (except in the test hook).
//
// Data movement: both operands are K-contiguous, so a tile row is 64 bf16 = 128 B = eight
// 16-byte pieces.  Global loads are 128-bit, 8 adjacent lanes per row segment; LDS rows are
// 128 B with the piece index XOR-swizzled by (row/2)%8 so that the 16-byte fragment reads of
// 32 different rows spread over all banks.  Two LDS stages; the next stage's global loads
// are issued before the current stage's MFMAs.
#include "vt_internal.h"

namespace vt {

hipError_t launch_gemm(const Plan& p, const HeadArgs& a, hipStream_t s)
{
    GemmArgs ga;
    ga.h = a.h;
    ga.W = a.W;
    ga.rows = p.rows;
    ga.nchunk = p.H / 8;
    ga.Vd = p.Vd;
    ga.P = p.P;
    ga.n_vtiles = p.n_vtiles;
    ga.n_rtiles = p.n_rtiles;
    ga.part_val = a.part_val;
    ga.part_idx = a.part_idx;
    ga.part_stat = a.part_stat;
    ga.logits_out = a.logits_out;
    switch (p.KP) {
    case 1: return launch_gemm_kp1(p, ga, s);
    case 2: return launch_gemm_kp2(p, ga, s);
    case 4: return launch_gemm_kp4(p, ga, s);
    case 8: return launch_gemm_kp8(p, ga, s);
    case 16: return launch_gemm_kp16(p, ga, s);
    case 32: return launch_gemm_kp32(p, ga, s);
    case 64: return launch_gemm_kp64(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
