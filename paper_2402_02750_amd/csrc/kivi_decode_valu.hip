// Decode attention, vector-ALU family (KIVI Equation 4 + Algorithm 1 Decoding), and the
// split-merge kernel shared by both decode families.
//
// One workgroup (4 wavefronts) owns one context split of one (batch, kv-head) and all the query
// heads that read that kv-head.  It runs three phases over its token range, so no online-softmax
// rescaling is needed inside a split:
//   1. logits   a_t = scale * sum_c q_c * K'[t,c]   -> LDS   (quantised tiles or fp16 rows)
//   2. softmax statistics of the split: m = max a_t, p_t = exp(a_t - m), l = sum p_t
//   3. output   o_c = sum_t p_t * V'[t,c]            (quantised tiles or fp16 rows)
// and writes (m, l, o[128]) per query head to the workspace; merge_kernel combines the splits.
//
// Scale and zero-point are folded into the small operand (Section 3.1's x' = code*s + z):
//   sum_c q_c (code*s_c + z_c) = sum_c (q_c s_c) code + sum_c q_c z_c        (keys)
//   sum_t p_t (code*s_t + z_t) = sum_t (p_t s_t) code + sum_t p_t z_t        (values)
// so each code costs an extract, a convert and one FMA.
#include "kivi_internal.h"

#include <hip/hip_fp16.h>

namespace kivi {
namespace {

constexpr int kMaxSplitTokens = kMaxSplitTiles * kTileTokens;   // 1024

struct alignas(16) Half8 { __half2 v[4]; };

__device__ __forceinline__ void unpack8(const Half8& h, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 t = __half22float2(h.v[i]);
        f[2 * i] = t.x;
        f[2 * i + 1] = t.y;
    }
}

__device__ __forceinline__ int ring_slot(int start, int i, int cap) {
    int s = start + i;
    s -= (s >= cap) ? cap : 0;
    return s;
}

template <int BITS>
__device__ __forceinline__ float code_at(const uint32_t* w, int u, int e) {
    // w: the lane's words of the tile (4 at B=2, 8 at B=4) in plane-major order
    if (BITS == 2) {
        const int bit = (e & 1) * 16 + 2 * ((u & 1) * 4 + (e >> 1));
        return (float)((w[u >> 1] >> bit) & 3u);
    } else {
        const int i = (u >> 1) * 2 + (e >> 2);
        const int bit = (e & 1) * 16 + 4 * ((u & 1) * 2 + ((e >> 1) & 1));
        return (float)((w[i] >> bit) & 15u);
    }
}

template <int BITS>
__device__ __forceinline__ void load_tile_words(const uint32_t* tile, int lane, uint32_t* w) {
    constexpr int kPlanes = BITS / 2;
#pragma unroll
    for (int pl = 0; pl < kPlanes; ++pl) {
        const uint4 v = *reinterpret_cast<const uint4*>(tile + pl * 256 + lane * 4);
        w[pl * 4 + 0] = v.x; w[pl * 4 + 1] = v.y; w[pl * 4 + 2] = v.z; w[pl * 4 + 3] = v.w;
    }
}

template <int BITS, int REP>
__global__ __launch_bounds__(256) void decode_valu_kernel(DecodeParams p) {
    // logits / probabilities of the split; reused as the cross-wave output staging area
    __shared__ __align__(16) float sm_buf[REP * kMaxSplitTokens];
    __shared__ __align__(16) float sm_q[REP][kHeadDim];
    __shared__ float sm_red[4];
    __shared__ float sm_m[REP], sm_l[REP];

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    constexpr int kLaneWords = BITS * 2;

    // token range of this split
    int tile0, tile1;
    if (split < p.plan.n_splits_a) {
        tile0 = split * p.plan.tiles_per_split_a;
        tile1 = min(tile0 + p.plan.tiles_per_split_a, p.plan.tiles_a);
    } else {
        tile0 = p.plan.tiles_a + (split - p.plan.n_splits_a) * p.plan.tiles_per_split_b;
        tile1 = min(tile0 + p.plan.tiles_per_split_b, p.plan.tiles_total);
    }
    const int t0 = tile0 * kTileTokens;
    const int n_tok = min(tile1 * kTileTokens, p.length) - t0;      // valid tokens in the split
    const int n_tiles = tile1 - tile0;

    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    // REP is the instantiation's head count; the layout may have fewer query heads per kv-head
    // (3, 5, 6, 7): the surplus heads run on a zero query and are never stored
    const int rep = p.rep_here;
    const int hq0 = h * (p.n_q_heads / p.n_kv_heads) + p.q_head0;

    for (int i = tid; i < REP * kHeadDim; i += 256) {
        const int hh = i / kHeadDim, c = i % kHeadDim;
        sm_q[hh][c] = hh < rep ? __half2float(p.q[((int64_t)b * p.n_q_heads + hq0 + hh) * kHeadDim + c]) : 0.f;
    }
    __syncthreads();

    // ---------------- phase 1: logits ----------------
    for (int ti = wave; ti < n_tiles; ti += 4) {
        const int tile = tile0 + ti;
        const int tt = tile * kTileTokens;
        if (tt < p.n_kq) {
            // quantised key tile: lane (r, kq) holds tokens {r, r+16} x channels ks*32 + kq*8 + e
            const int r = lane & 15, kq = lane >> 4;
            uint32_t w[kLaneWords];
            load_tile_words<BITS>(p.k_codes + (unit * p.cap_tiles + tile) * kWords, lane, w);
            const __half* sc = p.k_scale + ((unit * p.cap_tiles + tile) >> p.kg_shift) * kHeadDim;
            const __half* zr = p.k_zero + ((unit * p.cap_tiles + tile) >> p.kg_shift) * kHeadDim;
            float acc0[REP], acc1[REP];
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) acc0[hh] = acc1[hh] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int c0 = ks * 32 + kq * 8;
                float s[8], z[8];
                unpack8(*reinterpret_cast<const Half8*>(sc + c0), s);
                unpack8(*reinterpret_cast<const Half8*>(zr + c0), z);
                float k0[8], k1[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    k0[e] = code_at<BITS>(w, ks * 2 + 0, e);
                    k1[e] = code_at<BITS>(w, ks * 2 + 1, e);
                }
#pragma unroll
                for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float qv = sm_q[hh][c0 + e];
                        const float qs = qv * s[e];
                        const float qz = qv * z[e];
                        acc0[hh] = fmaf(qs, k0[e], acc0[hh] + qz);
                        acc1[hh] = fmaf(qs, k1[e], acc1[hh] + qz);
                    }
                }
            }
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                float a0 = acc0[hh], a1 = acc1[hh];
                a0 += __shfl_xor(a0, 16); a1 += __shfl_xor(a1, 16);
                a0 += __shfl_xor(a0, 32); a1 += __shfl_xor(a1, 32);
                if (kq == 0) {
                    sm_buf[hh * kMaxSplitTokens + ti * kTileTokens + r] = a0 * p.softmax_scale;
                    sm_buf[hh * kMaxSplitTokens + ti * kTileTokens + 16 + r] = a1 * p.softmax_scale;
                }
            }
        } else {
            // fp16 residual keys: lane (seg, row): 4 rows per step, 8 channels per lane
            const int seg = lane & 15, row = lane >> 4;
            float qv[REP][8];
#pragma unroll
            for (int hh = 0; hh < REP; ++hh)
#pragma unroll
                for (int e = 0; e < 8; ++e) qv[hh][e] = sm_q[hh][seg * 8 + e];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int t = tt + it * 4 + row;
                const bool valid = t < p.length;
                float k[8];
                if (valid) {
                    const int slot = ring_slot(p.k_r_start, t - p.n_kq, p.cap_r);
                    unpack8(*reinterpret_cast<const Half8*>(
                                p.k_resid + (unit * p.cap_r + slot) * kHeadDim + seg * 8), k);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) k[e] = 0.f;
                }
#pragma unroll
                for (int hh = 0; hh < REP; ++hh) {
                    float a = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) a = fmaf(qv[hh][e], k[e], a);
                    a += __shfl_xor(a, 1); a += __shfl_xor(a, 2);
                    a += __shfl_xor(a, 4); a += __shfl_xor(a, 8);
                    if (seg == 0)
                        sm_buf[hh * kMaxSplitTokens + ti * kTileTokens + it * 4 + row] =
                            valid ? a * p.softmax_scale : -INFINITY;
                }
            }
        }
    }
    __syncthreads();

    // ---------------- phase 2: softmax statistics of the split ----------------
    const int n_slots = n_tiles * kTileTokens;     // includes the invalid tail (-inf logits)
    for (int hh = 0; hh < REP; ++hh) {
        float* a = sm_buf + hh * kMaxSplitTokens;
        float mx = -INFINITY;
        for (int i = tid; i < n_slots; i += 256) mx = fmaxf(mx, a[i]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        if (lane == 0) sm_red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(sm_red[0], sm_red[1]), fmaxf(sm_red[2], sm_red[3]));
        __syncthreads();
        float sum = 0.f;
        for (int i = tid; i < n_slots; i += 256) {
            const float e = __expf(a[i] - mx);
            a[i] = e;
            sum += e;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane == 0) sm_red[wave] = sum;
        __syncthreads();
        if (tid == 0) {
            sm_m[hh] = mx;
            sm_l[hh] = sm_red[0] + sm_red[1] + sm_red[2] + sm_red[3];
        }
        __syncthreads();
    }
    (void)n_tok;

    // ---------------- phase 3: output ----------------
    float acc[REP][8], zacc[REP][4], racc[REP][8];
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[hh][u] = racc[hh][u] = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) zacc[hh][i] = 0.f;
    }
    for (int ti = wave; ti < n_tiles; ti += 4) {
        const int tile = tile0 + ti;
        const int tt = tile * kTileTokens;
        const int n_vq_here = min(max(p.n_vq - tt, 0), kTileTokens);   // quantised tokens of this tile
        if (n_vq_here > 0) {
            // quantised value tile: lane (r, kq) holds channels u*16 + r x tokens kq*8 + e
            const int kq = lane >> 4;
            uint32_t w[kLaneWords];
            load_tile_words<BITS>(p.v_codes + (unit * p.cap_tiles + tile) * kWords, lane, w);
            const int64_t tok = (unit * p.cap_tiles + tile) * kTileTokens + kq * 8;
            float s[8][4], z[8][4];
            if (p.kg_shift == 0) {
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {      // 2 tokens (8 halves) per 16-byte load
                    float fs[8], fz[8];
                    unpack8(*reinterpret_cast<const Half8*>(p.v_scale + (tok + e2 * 2) * 4), fs);
                    unpack8(*reinterpret_cast<const Half8*>(p.v_zero + (tok + e2 * 2) * 4), fz);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        s[e2 * 2][i] = fs[i]; s[e2 * 2 + 1][i] = fs[4 + i];
                        z[e2 * 2][i] = fz[i]; z[e2 * 2 + 1][i] = fz[4 + i];
                    }
                }
            } else {
                // G = 64 / 128: 2 or 1 entries per token, shared by 2 or 4 of the 32-channel blocks
                const int per_token = 4 >> p.kg_shift;
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int64_t o = (tok + e) * per_token + (i >> p.kg_shift);
                        s[e][i] = __half2float(p.v_scale[o]);
                        z[e][i] = __half2float(p.v_zero[o]);
                    }
            }
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool valid = kq * 8 + e < n_vq_here;
                    const float pt = valid ? sm_buf[hh * kMaxSplitTokens + ti * kTileTokens + kq * 8 + e] : 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float ps = valid ? pt * s[e][i] : 0.f;
                        zacc[hh][i] = fmaf(pt, valid ? z[e][i] : 0.f, zacc[hh][i]);
                        acc[hh][2 * i] = fmaf(ps, code_at<BITS>(w, 2 * i, e), acc[hh][2 * i]);
                        acc[hh][2 * i + 1] = fmaf(ps, code_at<BITS>(w, 2 * i + 1, e), acc[hh][2 * i + 1]);
                    }
                }
            }
        }
        if (n_vq_here < kTileTokens) {
            // fp16 residual values: lane (seg, row)
            const int seg = lane & 15, row = lane >> 4;
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int tl = it * 4 + row;
                const int t = tt + tl;
                if (tl >= n_vq_here && t < p.length) {
                    const int slot = ring_slot(p.v_r_start, t - p.n_vq, p.cap_r);
                    float v[8];
                    unpack8(*reinterpret_cast<const Half8*>(
                                p.v_resid + (unit * p.cap_r + slot) * kHeadDim + seg * 8), v);
#pragma unroll
                    for (int hh = 0; hh < REP; ++hh) {
                        const float pt = sm_buf[hh * kMaxSplitTokens + ti * kTileTokens + tl];
#pragma unroll
                        for (int e = 0; e < 8; ++e) racc[hh][e] = fmaf(pt, v[e], racc[hh][e]);
                    }
                }
            }
        }
    }
    __syncthreads();   // everyone is done reading probabilities: sm_buf becomes the staging area

    // reduce over the 4 lane groups, stage per wave: stage[wave][hh][2][128]
    float* stage = sm_buf;
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float zz = zacc[hh][i];
            zz += __shfl_xor(zz, 16); zz += __shfl_xor(zz, 32);
            zacc[hh][i] = zz;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float a = acc[hh][u], rr = racc[hh][u];
            a += __shfl_xor(a, 16); a += __shfl_xor(a, 32);
            rr += __shfl_xor(rr, 16); rr += __shfl_xor(rr, 32);
            if (lane < 16) {
                float* st = stage + ((wave * REP + hh) * 2) * kHeadDim;
                st[u * 16 + lane] = a + zacc[hh][u >> 1];
                st[kHeadDim + lane * 8 + u] = rr;
            }
        }
    }
    __syncthreads();
    const int n_splits = p.plan.n_splits();
    for (int i = tid; i < REP * kHeadDim; i += 256) {
        const int hh = i / kHeadDim, c = i % kHeadDim;
        float o = 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float* st = stage + ((wv * REP + hh) * 2) * kHeadDim;
            o += st[c] + st[kHeadDim + c];
        }
        if (hh >= rep) continue;
        const int64_t row = ((int64_t)b * p.n_q_heads + hq0 + hh) * n_splits + split;
        p.part_o[row * kHeadDim + c] = o;
        if (c == 0) {
            p.part_ml[row * 2 + 0] = sm_m[hh];
            p.part_ml[row * 2 + 1] = sm_l[hh];
        }
    }
}

// Combine the splits of one (batch, query head):  m = max m_i,  l = sum l_i e^{m_i - m},
// o = sum o_i e^{m_i - m} / l.
__global__ __launch_bounds__(128) void merge_kernel(DecodeParams p) {
    const int row = blockIdx.x;          // b * H_q + hq
    const int c = threadIdx.x;
    const int n = p.plan.n_splits();
    const float* ml = p.part_ml + (int64_t)row * n * 2;
    const float* po = p.part_o + (int64_t)row * n * kHeadDim;
    float m = -INFINITY;
    for (int i = 0; i < n; ++i) m = fmaxf(m, ml[2 * i]);
    float l = 0.f, o = 0.f;
    for (int i = 0; i < n; ++i) {
        const float w = __expf(ml[2 * i] - m);
        l = fmaf(ml[2 * i + 1], w, l);
        o = fmaf(po[(int64_t)i * kHeadDim + c], w, o);
    }
    p.out[(int64_t)row * kHeadDim + c] = o / l;
}

template <int BITS>
hipError_t launch_bits(const DecodeParams& p, hipStream_t stream) {
    const int rep = p.rep_variant;
    dim3 grid(p.plan.n_splits(), p.n_kv_heads, p.batch), block(256);
    // the smallest instantiation that holds the layout's query heads per kv-head
    if (rep == 1) decode_valu_kernel<BITS, 1><<<grid, block, 0, stream>>>(p);
    else if (rep == 2) decode_valu_kernel<BITS, 2><<<grid, block, 0, stream>>>(p);
    else if (rep <= 4) decode_valu_kernel<BITS, 4><<<grid, block, 0, stream>>>(p);
    else if (rep <= 8) decode_valu_kernel<BITS, 8><<<grid, block, 0, stream>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_valu(const DecodeParams& p, hipStream_t stream) {
    return p.bits == 2 ? launch_bits<2>(p, stream) : launch_bits<4>(p, stream);
}

hipError_t launch_merge(const DecodeParams& p, hipStream_t stream) {
    merge_kernel<<<p.batch * p.n_q_heads, 128, 0, stream>>>(p);
    return hipGetLastError();
}

}  // namespace kivi
