// Attention over the fp16 residual window alone as a device function (see kivi_decode_rows.hip for
// what it computes and why it is a launch of its own); shared by the plain rows kernel and by the
// launch that also quantises the residual tokens a decode step flushes.
#pragma once

#include "kivi_internal.h"

#include <hip/hip_fp16.h>

namespace kivi {
namespace rows {


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
// bytes of LDS the rows of `tiles_b` tiles need on the instantiation for `rep` heads
__host__ __device__ inline size_t rows_lds_bytes(int tiles_b, int rep) {
    return (size_t)tiles_b * rep * (kTileTokens + kPartFloats) * sizeof(float);
}
// One workgroup serves (batch, kv-head) unit `unit_index` with its first 64 * tiles_b threads (one
// wavefront per tile of fp16 rows); any further threads of the workgroup only keep the barrier.
// sm_dyn: rows_lds_bytes() of LDS.  A device function so that it can also run as a role of a wider launch.
template <int REP>
__device__ __forceinline__ void residual_rows_block(const DecodeParams& p, float* sm_dyn, int64_t unit_index,
                                                    int tiles_b, int tid) {
    const int n_threads = 64 * tiles_b;
    if (tid >= n_threads) {         // surplus wavefronts of a wider workgroup
        __syncthreads();
        return;
    }
    // LDS: per wavefront REP x 32 probabilities, then per wavefront REP parts
    const int lane = tid & 63, wave = tid >> 6;
    const int seg = lane & 15, row = lane >> 4;           // channels seg*8.., rows row, row+4, ...
    float (*sm_p)[kTileTokens] = reinterpret_cast<float (*)[kTileTokens]>(sm_dyn) + wave * REP;   // [REP][32] of this wavefront
    float* sm_part = sm_dyn + tiles_b * REP * kTileTokens;                                          // [tiles_b][REP][130]
    const int64_t unit = unit_index;
    const int b = (int)(unit / p.n_kv_heads), h = (int)(unit % p.n_kv_heads);
    // the sequence's counters: the launch's, or (batches of different lengths) its entry of seq_state
    int n_q = p.n_kq, length = p.length, k_start = p.k_r_start, v_start = p.v_r_start;
    if (p.seq_state) {
        const int4 st = reinterpret_cast<const int4*>(p.seq_state)[b];      // n_q, n_r, k_r_start, v_r_start
        n_q = st.x; length = st.x + st.y; k_start = st.z; v_start = st.w;
    }
    const int tt = (n_q / kTileTokens + wave) * kTileTokens;  // first token of the tile (past the end for a shorter sequence's surplus wavefronts)
    const int rep = p.rep_here, rep_total = p.n_q_heads / p.n_kv_heads;
    const int64_t q_row0 = (int64_t)b * p.n_q_heads + (int64_t)h * rep_total + p.q_head0;
    const bool fused_append = p.k_new != nullptr;
    const int last = length - 1;

    // the key rows of the tile are requested up front: 8 rows per lane
    half8 kr[8], vr[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int t = min(tt + j * 4 + row, last);         // rows past the end re-read the last row (unused)
        const __half* ks = p.k_resid + (unit * p.cap_r + ring_slot(k_start, t - n_q, p.cap_r)) * kHeadDim;
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
        const int slot = is_v ? ring_slot(v_start, last - n_q, p.cap_r) : ring_slot(k_start, last - n_q, p.cap_r);
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
        const __half* vs = p.v_resid + (unit * p.cap_r + ring_slot(v_start, t - n_q, p.cap_r)) * kHeadDim;
        if (fused_append && t == last) vs = p.v_new + unit * kHeadDim;
        vr[j] = *reinterpret_cast<const half8*>(vs + seg * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
    // softmax of the tile: lane t < 32 takes token t
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        const float a = lane < kTileTokens ? sm_p[hh][lane] : -INFINITY;
        m[hh] = wave_max32(a);                             // -inf only for a tile past the end of a shorter sequence
        const float pt = lane < kTileTokens ? __expf(a - (m[hh] == -INFINITY ? 0.f : m[hh])) : 0.f;
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
    for (int idx = tid; idx < rep * kHeadDim; idx += n_threads) {
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


}  // namespace rows
}  // namespace kivi
