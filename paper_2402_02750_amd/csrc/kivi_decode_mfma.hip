// Decode attention, matrix-core family for gfx950 (KIVI Equation 4 + Algorithm 1 Decoding).
//
// Why matrix cores for a bandwidth-bound scan: at 2 bits a cached element is 3/8 of a byte, so at
// HBM speed a compute unit sees ~28 elements per clock while its vector ALUs retire 64 lane-ops
// per clock.  Extract + convert + FMA + cross-lane reduction does not fit in ~2.3 lane-ops per
// element.  Here the vector ALUs only *extract*: a code left in place inside an fp16 lane by one
// AND is the exact subnormal/normal fp16 number code * 4^j * 2^-24, and the v_mfma 16x16x32 f16
// instruction multiplies, accumulates in fp32 and reduces over the contraction index.  The
// position factor 4^j and the group's scale go into the small operand:
//   keys  : a_t = sum_c [code_tc 4^j] [q_c s_c 4^-j]     + sum_c q_c z_c        (per tile of 32 tokens)
//   values: o_c = sum_t [code_tc 4^j] [p_t s_t,g 4^-j]   + sum_t p_t z_t,g
// and the small operand is split into fp16 hi + lo parts in two matrix columns, which restores
// fp32-class accuracy.  The z-term of the keys is itself a 16x16x32 product (zero-points are
// exact fp16).  The fp16 residual rows are 5x the bytes per element, so they stay on the vector
// ALUs.
//
// A workgroup (4 wavefronts) owns one context split of one (batch, kv-head) and all query heads
// reading it; each wavefront takes every 4th tile of the split as an independent sub-split with
// its own softmax maximum (no barrier between logits and outputs); the four are merged in LDS and
// one (m, l, o[128]) per query head goes to the workspace for merge_kernel.
#include "kivi_internal.h"

#include <hip/hip_fp16.h>

namespace kivi {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kWaveTiles = kMaxSplitTiles / 4;          // 8 tiles per wavefront at most
constexpr int kWaveTokens = kWaveTiles * kTileTokens;   // 256
constexpr int kKRow = 136;   // halves per column of the key-side B staging (272 B: bank skew)
constexpr int kVRow = 40;    // halves per column of the value-side B staging (80 B: bank skew)
constexpr int kBStage = 4 * 16 * kVRow;                 // 2560 halves >= 16 * kKRow = 2176
constexpr float kUnscale = 16777216.0f;                 // 2^24: codes enter as code * 2^-24

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

// LDS traffic between the lanes of one wavefront needs no hardware barrier (a wavefront's LDS
// operations execute in order); this only stops the compiler from reordering across it.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// value of lane+1 inside each pair of lanes (quad_perm [1,1,3,3])
__device__ __forceinline__ float dpp_pair_next(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xF5, 0xF, 0xF, false));
}

__device__ __forceinline__ float pow2_neg(int e) {   // 2^-e, 0 <= e < 64
    return __int_as_float((127 - e) << 23);
}

// 1 / (position factor) of contraction slot pair j = e >> 1 (e in [0,8)) -- see the tile layout
template <int BITS>
__device__ __forceinline__ float inv_pos_factor(int j) {
    return BITS == 2 ? pow2_neg(2 * (j & 3)) : pow2_neg(4 * (j & 1));
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

// A-operand fragment (8 fp16 = 4 registers) of tile coordinate u = pair * 2 + odd.
template <int BITS>
__device__ __forceinline__ half8 code_fragment(const uint32_t* w, int pair, int odd) {
    union { uint32_t r[4]; half8 h; } f;
    if (BITS == 2) {
        const uint32_t x = w[pair] >> (8 * odd);
        f.r[0] = x & 0x00030003u; f.r[1] = x & 0x000C000Cu;
        f.r[2] = x & 0x00300030u; f.r[3] = x & 0x00C000C0u;
    } else {
        const uint32_t x0 = w[pair * 2] >> (8 * odd), x1 = w[pair * 2 + 1] >> (8 * odd);
        f.r[0] = x0 & 0x000F000Fu; f.r[1] = x0 & 0x00F000F0u;
        f.r[2] = x1 & 0x000F000Fu; f.r[3] = x1 & 0x00F000F0u;
    }
    return f.h;
}

__device__ __forceinline__ void split_hi_lo(float x, __half& hi, __half& lo) {
    hi = __float2half_rn(x);
    lo = __float2half_rn(x - __half2float(hi));
}

template <int BITS, int REP>
__global__ __launch_bounds__(256) void decode_mfma_kernel(DecodeParams p) {
    constexpr int NC = 2 * REP;                       // live matrix columns: (head, hi/lo)
    __shared__ __align__(16) float sm_q[REP][kHeadDim];               // scale * q
    __shared__ __align__(16) __half sm_qf[16][kKRow];                 // its hi/lo columns (z-term operand)
    __shared__ __align__(16) float sm_p[4][REP][kWaveTokens];         // logits -> probabilities -> staging
    __shared__ __align__(16) __half sm_b[4][kBStage];                 // per-wave small-operand staging
    __shared__ float sm_zt[4][REP][kWaveTiles];
    __shared__ float sm_ml[4][REP][2];

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, rq = lane >> 4;          // matrix column / row-quad (= k-quad for operands)
    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    constexpr int kLaneWords = BITS * 2;

    int tile0, tile1;
    if (split < p.plan.n_splits_a) {
        tile0 = split * p.plan.tiles_per_split_a;
        tile1 = min(tile0 + p.plan.tiles_per_split_a, p.plan.tiles_a);
    } else {
        tile0 = p.plan.tiles_a + (split - p.plan.n_splits_a) * p.plan.tiles_per_split_b;
        tile1 = min(tile0 + p.plan.tiles_per_split_b, p.plan.tiles_total);
    }
    const int n_tiles = tile1 - tile0;
    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    const int hq0 = h * REP;

    // ---------------- phase 0: query operands ----------------
    for (int i = tid; i < 16 * kHeadDim; i += 256) {
        const int col = i / kHeadDim, c = i % kHeadDim;
        __half v = __float2half_rn(0.f);
        if (col < NC) {
            const int hh = col >> 1;
            const float x = p.softmax_scale *
                            __half2float(p.q[((int64_t)b * p.n_q_heads + hq0 + hh) * kHeadDim + c]);
            __half hi, lo;
            split_hi_lo(x, hi, lo);
            v = (col & 1) ? lo : hi;
            if (!(col & 1)) sm_q[hh][c] = x;
        }
        sm_qf[col][c] = v;
    }
    __syncthreads();

    // tiles of this wavefront: ti = wave + 4*i
    const int cnt = n_tiles > wave ? (n_tiles - wave + 3) / 4 : 0;
    // how many of them are quantised key tiles (they come first in token order)
    int cnt_kq = 0;
    for (int i = 0; i < cnt; ++i) cnt_kq += ((tile0 + wave + 4 * i) * kTileTokens < p.n_kq) ? 1 : 0;

    __half* bw = sm_b[wave];
    const int ncol = n & (NC - 1);

    // ---------------- key z-terms of all quantised tiles of the wave: one 16x16x128 product ----
    if (cnt_kq > 0) {
        const int ti = wave + 4 * min(n, cnt_kq - 1);           // row n of A = n-th tile of the wave
        const __half* zrow = p.k_zero + (unit * p.cap_tiles + tile0 + ti) * kHeadDim;
        float4v d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const half8 a = *reinterpret_cast<const half8*>(zrow + ks * 32 + rq * 8);
            const half8 bq = *reinterpret_cast<const half8*>(&sm_qf[n][ks * 32 + rq * 8]);
            d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq, d, 0, 0, 0);
        }
        // d[i]: tile index rq*4 + i of the wave, column n; hi + lo columns
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float v = d[i] + dpp_pair_next(d[i]);
            const int idx = rq * 4 + i;
            if (!(n & 1) && n < NC && idx < kWaveTiles) sm_zt[wave][n >> 1][idx] = v;
        }
        wave_lds_sync();
    }

    // per-lane key-side query factors: channels 2*lane, 2*lane+1 times 1/position factor
    float qpf[REP][2];
    {
        const float pf = inv_pos_factor<BITS>(lane & 3);
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            qpf[hh][0] = sm_q[hh][2 * lane] * pf;
            qpf[hh][1] = sm_q[hh][2 * lane + 1] * pf;
        }
    }

    // ---------------- phase 1: logits of the wave's tiles ----------------
    for (int i = 0; i < cnt; ++i) {
        const int tile = tile0 + wave + 4 * i;
        const int tt = tile * kTileTokens;
        if (tt < p.n_kq) {
            uint32_t w[kLaneWords];
            load_tile_words<BITS>(p.k_codes + (unit * p.cap_tiles + tile) * kWords, lane, w);
            const __half2 s2 = *reinterpret_cast<const __half2*>(
                p.k_scale + (unit * p.cap_tiles + tile) * kHeadDim + 2 * lane);
            const float s0 = __low2float(s2), s1 = __high2float(s2);
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                __half h0, l0, h1, l1;
                split_hi_lo(qpf[hh][0] * s0, h0, l0);
                split_hi_lo(qpf[hh][1] * s1, h1, l1);
                *reinterpret_cast<__half2*>(bw + (2 * hh) * kKRow + 2 * lane) = __halves2half2(h0, h1);
                *reinterpret_cast<__half2*>(bw + (2 * hh + 1) * kKRow + 2 * lane) = __halves2half2(l0, l1);
            }
            wave_lds_sync();
            half8 bf[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                bf[ks] = *reinterpret_cast<const half8*>(bw + ncol * kKRow + ks * 32 + rq * 8);
            wave_lds_sync();
            float4v d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                d0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, ks, 0), bf[ks], d0, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, ks, 1), bf[ks], d1, 0, 0, 0);
            }
            // d0[j]: token rq*4 + j, d1[j]: token 16 + rq*4 + j; column n
            float v0[4], v1[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v0[j] = d0[j] + dpp_pair_next(d0[j]);
                v1[j] = d1[j] + dpp_pair_next(d1[j]);
            }
            if (!(n & 1) && n < NC) {
                const int hh = n >> 1;
                const float zt = sm_zt[wave][hh][i];
                float* dst = &sm_p[wave][hh][i * kTileTokens + rq * 4];
                *reinterpret_cast<float4*>(dst) = make_float4(
                    fmaf(v0[0], kUnscale, zt), fmaf(v0[1], kUnscale, zt),
                    fmaf(v0[2], kUnscale, zt), fmaf(v0[3], kUnscale, zt));
                *reinterpret_cast<float4*>(dst + 16) = make_float4(
                    fmaf(v1[0], kUnscale, zt), fmaf(v1[1], kUnscale, zt),
                    fmaf(v1[2], kUnscale, zt), fmaf(v1[3], kUnscale, zt));
            }
        } else {
            // fp16 residual keys on the vector ALUs: lane (seg, row): 4 rows per step, 8 channels per lane
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
                    if (seg == 0) sm_p[wave][hh][i * kTileTokens + it * 4 + row] = valid ? a : -INFINITY;
                }
            }
        }
    }
    wave_lds_sync();

    // ---------------- phase 2: softmax statistics of the wave's sub-split ----------------
    float m_w[REP], l_w[REP];
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        m_w[hh] = -INFINITY;
        l_w[hh] = 0.f;
        if (cnt > 0) {
            float4 a = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            const bool live = lane * 4 < cnt * kTileTokens;
            if (live) a = *reinterpret_cast<const float4*>(&sm_p[wave][hh][lane * 4]);
            float mx = fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w));
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            a.x = __expf(a.x - mx); a.y = __expf(a.y - mx); a.z = __expf(a.z - mx); a.w = __expf(a.w - mx);
            if (live) *reinterpret_cast<float4*>(&sm_p[wave][hh][lane * 4]) = a;
            float sum = live ? (a.x + a.y) + (a.z + a.w) : 0.f;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            m_w[hh] = mx;
            l_w[hh] = sum;
        }
    }
    wave_lds_sync();

    // ---------------- phase 3: outputs of the wave's tiles ----------------
    float4v acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};
    float zacc[REP][2], racc[REP][8];
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        zacc[hh][0] = zacc[hh][1] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) racc[hh][e] = 0.f;
    }
    for (int i = 0; i < cnt; ++i) {
        const int tile = tile0 + wave + 4 * i;
        const int tt = tile * kTileTokens;
        const int n_vq_here = min(max(p.n_vq - tt, 0), kTileTokens);
        if (n_vq_here > 0) {
            uint32_t w[kLaneWords];
            load_tile_words<BITS>(p.v_codes + (unit * p.cap_tiles + tile) * kWords, lane, w);
            // lane -> token t = lane/2, channel groups (lane%2)*2 + {0,1}
            const int t = lane >> 1, cg0 = (lane & 1) * 2;
            const bool valid = t < n_vq_here;
            const int64_t so = ((unit * p.cap_tiles + tile) * kTileTokens) * 4 + 2 * lane;
            const __half2 s2 = *reinterpret_cast<const __half2*>(p.v_scale + so);
            const __half2 z2 = *reinterpret_cast<const __half2*>(p.v_zero + so);
            const float pf = inv_pos_factor<BITS>((t >> 1) & 3);
            const float s0 = valid ? __low2float(s2) * pf : 0.f, s1 = valid ? __high2float(s2) * pf : 0.f;
            const float z0 = valid ? __low2float(z2) : 0.f, z1 = valid ? __high2float(z2) : 0.f;
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                const float pt = valid ? sm_p[wave][hh][i * kTileTokens + t] : 0.f;
                __half h0, l0, h1, l1;
                split_hi_lo(pt * s0, h0, l0);
                split_hi_lo(pt * s1, h1, l1);
                bw[((cg0 + 0) * 16 + 2 * hh) * kVRow + t] = h0;
                bw[((cg0 + 0) * 16 + 2 * hh + 1) * kVRow + t] = l0;
                bw[((cg0 + 1) * 16 + 2 * hh) * kVRow + t] = h1;
                bw[((cg0 + 1) * 16 + 2 * hh + 1) * kVRow + t] = l1;
                zacc[hh][0] = fmaf(pt, z0, zacc[hh][0]);
                zacc[hh][1] = fmaf(pt, z1, zacc[hh][1]);
            }
            wave_lds_sync();
            half8 bf[4];
#pragma unroll
            for (int cg = 0; cg < 4; ++cg)
                bf[cg] = *reinterpret_cast<const half8*>(bw + (cg * 16 + ncol) * kVRow + rq * 8);
            wave_lds_sync();
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, u >> 1, u & 1),
                                                                bf[u >> 1], acc[u], 0, 0, 0);
        }
        if (n_vq_here < kTileTokens) {
            // fp16 residual values on the vector ALUs: lane (seg, row)
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
                        const float pt = sm_p[wave][hh][i * kTileTokens + tl];
#pragma unroll
                        for (int e = 0; e < 8; ++e) racc[hh][e] = fmaf(pt, v[e], racc[hh][e]);
                    }
                }
            }
        }
    }
    wave_lds_sync();

    // ---------------- wave results -> LDS (the probability area becomes the staging area) -------
    // stage[hh][0][c]: matrix-core part (+ z-terms), stage[hh][1][c]: vector-ALU residual part
    {
        // z-term sums: lanes of equal parity hold the same channel-group pair
#pragma unroll
        for (int hh = 0; hh < REP; ++hh)
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float zz = zacc[hh][k];
                zz += __shfl_xor(zz, 2); zz += __shfl_xor(zz, 4); zz += __shfl_xor(zz, 8);
                zz += __shfl_xor(zz, 16); zz += __shfl_xor(zz, 32);
                zacc[hh][k] = zz;
            }
        // every lane needs all four channel-group sums of "its" head (n >> 1)
        float zs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            const float o0 = __shfl_xor(zacc[hh][0], 1), o1 = __shfl_xor(zacc[hh][1], 1);
            const bool odd = lane & 1;
            const float g0 = odd ? o0 : zacc[hh][0], g1 = odd ? o1 : zacc[hh][1];
            const float g2 = odd ? zacc[hh][0] : o0, g3 = odd ? zacc[hh][1] : o1;
            if ((n >> 1) == hh) { zs[0] = g0; zs[1] = g1; zs[2] = g2; zs[3] = g3; }
        }
        float* stage = &sm_p[wave][0][0];       // REP * 256 floats = REP * (2 * 128)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[u][j] + dpp_pair_next(acc[u][j]);
            if (!(n & 1) && n < NC) {
                const float z = zs[u >> 1];
                *reinterpret_cast<float4*>(stage + (n >> 1) * 256 + u * 16 + rq * 4) = make_float4(
                    fmaf(v[0], kUnscale, z), fmaf(v[1], kUnscale, z), fmaf(v[2], kUnscale, z), fmaf(v[3], kUnscale, z));
            }
        }
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float rr = racc[hh][e];
                rr += __shfl_xor(rr, 16); rr += __shfl_xor(rr, 32);
                racc[hh][e] = rr;
            }
            if (lane < 16) {
                float* dst = stage + hh * 256 + 128 + lane * 8;
                *reinterpret_cast<float4*>(dst) = make_float4(racc[hh][0], racc[hh][1], racc[hh][2], racc[hh][3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(racc[hh][4], racc[hh][5], racc[hh][6], racc[hh][7]);
            }
            if (lane == 0) { sm_ml[wave][hh][0] = m_w[hh]; sm_ml[wave][hh][1] = l_w[hh]; }
        }
    }
    __syncthreads();

    // ---------------- merge the four sub-splits, write the split's partial result ----------------
    const int n_splits = p.plan.n_splits();
    for (int idx = tid; idx < REP * kHeadDim; idx += 256) {
        const int hh = idx / kHeadDim, c = idx % kHeadDim;
        float m = -INFINITY;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) m = fmaxf(m, sm_ml[wv][hh][0]);
        float l = 0.f, o = 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float mw = sm_ml[wv][hh][0];
            if (mw > -INFINITY) {
                const float wgt = __expf(mw - m);
                const float* st = &sm_p[wv][0][0] + hh * 256;
                l = fmaf(sm_ml[wv][hh][1], wgt, l);
                o = fmaf(st[c] + st[128 + c], wgt, o);
            }
        }
        const int64_t row = ((int64_t)b * p.n_q_heads + hq0 + hh) * n_splits + split;
        p.part_o[row * kHeadDim + c] = o;
        if (c == 0) {
            p.part_ml[row * 2 + 0] = m;
            p.part_ml[row * 2 + 1] = l;
        }
    }
}

template <int BITS>
hipError_t launch_bits(const DecodeParams& p, hipStream_t stream) {
    const int rep = p.n_q_heads / p.n_kv_heads;
    dim3 grid(p.plan.n_splits(), p.n_kv_heads, p.batch), block(256);
    switch (rep) {
        case 1: decode_mfma_kernel<BITS, 1><<<grid, block, 0, stream>>>(p); break;
        case 2: decode_mfma_kernel<BITS, 2><<<grid, block, 0, stream>>>(p); break;
        case 4: decode_mfma_kernel<BITS, 4><<<grid, block, 0, stream>>>(p); break;
        case 8: decode_mfma_kernel<BITS, 8><<<grid, block, 0, stream>>>(p); break;
        default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeParams& p, hipStream_t stream) {
    return p.bits == 2 ? launch_bits<2>(p, stream) : launch_bits<4>(p, stream);
}

}  // namespace kivi
