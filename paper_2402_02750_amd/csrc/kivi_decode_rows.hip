// Attention over the fp16 residual window alone (KIVI Equation 4, the X_R terms; Algorithm 1
// Decoding), as a launch of its own: one workgroup per (batch, kv-head) unit, one wavefront per
// 32-token tile, a single barrier at the end, few registers -- so that a compute unit holds many
// wavefronts and the chain  rows -> logits -> softmax -> rows -> outputs  of one tile is hidden
// behind the chains of the others.  The workgroup merges its tiles in LDS and leaves one part
// (m, l, o[128]) per query head in the workspace; the launch of the all-quantised chunks that
// follows merges it into its results.
//
// Used when a workgroup of the persistent kernel would own several units (large batches): there
// the fp16-row chunks of those units run one after the other, each such chain exposed.
// Precondition (checked by the caller): n_kq == n_vq, so every tile from tiles_a on holds fp16 rows
// of both K and V and nothing quantised.
#include "kivi_rows_block.h"

namespace kivi {
namespace {

template <int REP>
__global__ __launch_bounds__(1024) void residual_rows_kernel(DecodeParams p) {
    extern __shared__ float sm_dyn[];
    rows::residual_rows_block<REP>(p, sm_dyn, blockIdx.x, blockDim.x >> 6, threadIdx.x);
}

}  // namespace

bool residual_rows_possible(int tiles_b, int rep_variant) {
    return tiles_b >= 1 && tiles_b <= 16 && tiles_b * rep_variant <= 64;
}

hipError_t launch_residual_rows(const DecodeParams& p, hipStream_t stream) {
    const int tiles_b = p.plan.tiles_total - p.plan.tiles_a;
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    const int rep = p.rep_variant <= 2 ? p.rep_variant : (p.rep_variant <= 4 ? 4 : 8);
    if (!residual_rows_possible(tiles_b, rep) || p.plan.n_splits_b != 1 || p.n_kq != p.n_vq || units > 0x7fffffff)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)units), block(64 * tiles_b);
    const size_t lds = rows::rows_lds_bytes(tiles_b, rep);
    if (rep == 1) residual_rows_kernel<1><<<grid, block, lds, stream>>>(p);
    else if (rep == 2) residual_rows_kernel<2><<<grid, block, lds, stream>>>(p);
    else if (rep == 4) residual_rows_kernel<4><<<grid, block, lds, stream>>>(p);
    else residual_rows_kernel<8><<<grid, block, lds, stream>>>(p);
    return hipGetLastError();
}

}  // namespace kivi
