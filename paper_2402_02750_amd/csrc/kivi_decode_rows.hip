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
#include "kivi_internal.h"

#include <hip/hip_fp16.h>

namespace kivi {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

// sum over the 16 lanes of a row (every lane of the row gets it)
__device__ __forceinline__ float row_sum(float v) {
    v += dpp<kDppXor1>(v); v += dpp<kDppXor2>(v);
    v += dpp<kDppHalfMirror>(v); v += dpp<kDppMirror>(v);
    return v;
}
__device__ __forceinline__ float wave_max32(float v) {      // over lanes 0..63, all lanes get it
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, __shfl_xor(v, m));
    return v;
}
__device__ __forceinline__ float wave_sum32(float v) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
    return v;
}

__device__ __forceinline__ float dot8(half8 a, half8 b) {
    float r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), 0.f, false);
    r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), r, false);
    r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), r, false);
    return __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), r, false);
}

__device__ __forceinline__ int ring_slot(int start, int i, int cap) {
    int s = start + i;
    s -= (s >= cap) ? cap : 0;
    return s;
}

// REP: query heads per kv-head this instantiation holds (p.rep_here <= REP of them are live).
constexpr int kPartFloats = kHeadDim + 2;      // o[128], m, l
template <int REP>
__global__ __launch_bounds__(1024) void residual_rows_kernel(DecodeParams p) {
    // dynamic LDS: per wavefront REP x 32 probabilities, then per wavefront REP parts
    extern __shared__ float sm_dyn[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seg = lane & 15, row = lane >> 4;           // channels seg*8.., rows row, row+4, ...
    const int tiles_b = blockDim.x >> 6;                   // one wavefront per tile of fp16 rows
    float (*sm_p)[kTileTokens] = reinterpret_cast<float (*)[kTileTokens]>(sm_dyn) + wave * REP;   // [REP][32] of this wavefront
    float* sm_part = sm_dyn + tiles_b * REP * kTileTokens;                                          // [tiles_b][REP][130]
    const int64_t unit = blockIdx.x;
    const int tt = (p.plan.tiles_a + wave) * kTileTokens;  // first token of the tile
    const int b = (int)(unit / p.n_kv_heads), h = (int)(unit % p.n_kv_heads);
    const int rep = p.rep_here, rep_total = p.n_q_heads / p.n_kv_heads;
    const int64_t q_row0 = (int64_t)b * p.n_q_heads + (int64_t)h * rep_total + p.q_head0;
    const bool fused_append = p.k_new != nullptr;
    const int last = p.length - 1;

    // the key rows of the tile are requested up front: 8 rows per lane
    half8 kr[8], vr[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int t = min(tt + j * 4 + row, last);         // rows past the end re-read the last row (unused)
        const __half* ks = p.k_resid + (unit * p.cap_r + ring_slot(p.k_r_start, t - p.n_kq, p.cap_r)) * kHeadDim;
        if (fused_append && t == last) ks = p.k_new + unit * kHeadDim;     // the newest token is not in the rings yet
        kr[j] = *reinterpret_cast<const half8*>(ks + seg * 8);
    }
    // Fused append: the wavefront of the newest token's tile also stores that token's rows in the
    // rings (lanes 0-15 the key row, 16-31 the value row).  Nobody reads those slots in this launch.
    const bool owns_new = fused_append && last >= tt && last < tt + kTileTokens && lane < 32;
    uint4 new_row = {0u, 0u, 0u, 0u};
    __half* new_dst = nullptr;
    if (owns_new) {
        const bool is_v = lane >= 16;
        const int slot = is_v ? ring_slot(p.v_r_start, last - p.n_vq, p.cap_r) : ring_slot(p.k_r_start, last - p.n_kq, p.cap_r);
        new_row = *reinterpret_cast<const uint4*>((is_v ? p.v_new : p.k_new) + unit * kHeadDim + (lane & 15) * 8);
        new_dst = const_cast<__half*>(is_v ? p.v_resid : p.k_resid) + (unit * p.cap_r + slot) * kHeadDim + (lane & 15) * 8;
    }

    // logits: lane (seg, row) holds a partial dot product of rows row + 4j; the 16 lanes of a row add up
    float m[REP], l[REP];
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        const half8 qh = hh < rep ? *reinterpret_cast<const half8*>(p.q + (q_row0 + hh) * kHeadDim + seg * 8) : half8{};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float a = row_sum(dot8(kr[j], qh));
            const int tl = j * 4 + row;
            if (seg == 0) sm_p[hh][tl] = tt + tl <= last ? a * p.softmax_scale : -INFINITY;
        }
    }
    __builtin_amdgcn_wave_barrier();
    // The value rows are requested only now: with the key rows consumed, a wavefront needs fewer
    // registers at its peak, more wavefronts fit a compute unit, and their chains hide this latency
    // (measured: 3 % on the whole step of the streaming configuration against requesting both up front).
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int t = min(tt + j * 4 + row, last);
        const __half* vs = p.v_resid + (unit * p.cap_r + ring_slot(p.v_r_start, t - p.n_vq, p.cap_r)) * kHeadDim;
        if (fused_append && t == last) vs = p.v_new + unit * kHeadDim;
        vr[j] = *reinterpret_cast<const half8*>(vs + seg * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
    // softmax of the tile: lane t < 32 takes token t
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        const float a = lane < kTileTokens ? sm_p[hh][lane] : -INFINITY;
        m[hh] = wave_max32(a);                             // finite: the tile holds at least one token
        const float pt = lane < kTileTokens ? __expf(a - m[hh]) : 0.f;
        l[hh] = wave_sum32(pt);
        if (lane < kTileTokens) sm_p[hh][lane] = pt;
    }
    __builtin_amdgcn_wave_barrier();
    // outputs: lane (seg, row) accumulates channels seg*8.. over rows row + 4j, then the 4 row groups add up
    const int row_stride = p.plan.n_splits();
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float pt = sm_p[hh][j * 4 + row];            // 0 for tokens past the end
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(pt, (float)vr[j][e], o[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            o[e] += __shfl_xor(o[e], 16);
            o[e] += __shfl_xor(o[e], 32);
        }
        if (lane < 16) {
            float* dst = sm_part + (wave * REP + hh) * kPartFloats;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[seg * 8 + e] = o[e];
            if (lane == 0) {
                dst[kHeadDim] = m[hh];
                dst[kHeadDim + 1] = l[hh];
            }
        }
    }
    if (owns_new) *reinterpret_cast<uint4*>(new_dst) = new_row;
    __syncthreads();
    // merge the tiles of the unit: part 0 of every live query head
    for (int idx = threadIdx.x; idx < rep * kHeadDim; idx += blockDim.x) {
        const int hh = idx / kHeadDim, c = idx % kHeadDim;
        float mm = -INFINITY;
        for (int w = 0; w < tiles_b; ++w) mm = fmaxf(mm, sm_part[(w * REP + hh) * kPartFloats + kHeadDim]);
        float ll = 0.f, oo = 0.f;
        for (int w = 0; w < tiles_b; ++w) {
            const float* src = sm_part + (w * REP + hh) * kPartFloats;
            const float f = __expf(src[kHeadDim] - mm);
            ll = fmaf(src[kHeadDim + 1], f, ll);
            oo = fmaf(src[c], f, oo);
        }
        const int64_t prow = (q_row0 + hh) * row_stride;
        p.part_o[prow * kHeadDim + c] = oo;
        if (c == 0) {
            p.part_ml[prow * 2 + 0] = mm;
            p.part_ml[prow * 2 + 1] = ll;
        }
    }
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
    const size_t lds = (size_t)tiles_b * rep * (kTileTokens + kPartFloats) * sizeof(float);
    if (rep == 1) residual_rows_kernel<1><<<grid, block, lds, stream>>>(p);
    else if (rep == 2) residual_rows_kernel<2><<<grid, block, lds, stream>>>(p);
    else if (rep == 4) residual_rows_kernel<4><<<grid, block, lds, stream>>>(p);
    else residual_rows_kernel<8><<<grid, block, lds, stream>>>(p);
    return hipGetLastError();
}

}  // namespace kivi
