// Group-wise quantisation kernels for gfx950 (KIVI Section 3.1 formula; Section 3.3 grouping).
//
// One workgroup stages one 32-token x 128-channel fp16 tile in LDS (coalesced 16-byte loads),
// derives the per-group zero-point/scale, then every thread assembles whole 32-bit words of the
// packed tile, so all global stores are full, coalesced dwords.  The value of a code is
// bit-contract: fp32 subtract, IEEE fp32 division, round-half-even, clamp (encode()).  The fast
// path reaches the same code with one explicit fused multiply-add per element (encode_fast()) and
// falls back to encode() for a word whenever a quotient lies close enough to a rounding tie for
// the two to differ.  This file is compiled with -ffp-contract=off, so the only fused operations
// are the ones written as fmaf().
#include "kivi_internal.h"
#include "kivi_rows_block.h"

#include <hip/hip_fp16.h>

#include <algorithm>
#include <type_traits>

namespace kivi {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
// packed fp16 minimum / maximum (v_pk_min_f16 / v_pk_max_f16): exact, no arithmetic.  Written as
// instructions: the builtins make the compiler quiet signalling NaNs first (one more instruction per
// operand), which finite inputs -- the precondition of the quantiser -- do not need.
__device__ __forceinline__ half2v pk_min(half2v a, half2v b) {
    half2v r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ half2v pk_max(half2v a, half2v b) {
    half2v r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// consecutive value tiles one workgroup walks, the next tile's rows prefetched (measured at the
// 3968-token prefill of 512 units: 209 us with 1, 190 us with 4; the key kernel got slower with it)
constexpr int kValueTilesPerGroup = 4;
constexpr int kRowPad = 136;  // halves per LDS row: 272 B keeps 16-byte alignment, skews banks

__device__ __forceinline__ int64_t row_offset(const RowSource& s, int b, int h, int t) {
    int slot = t;
    if (s.ring_cap > 0) {
        slot = s.ring_start + t;
        slot -= (slot >= s.ring_cap) ? s.ring_cap : 0;
        slot -= (slot >= s.ring_cap) ? s.ring_cap : 0;
    }
    return (int64_t)b * s.stride_b + (int64_t)h * s.stride_h + (int64_t)slot * s.stride_t;
}

__device__ __forceinline__ uint32_t encode(float x, float z, float s, float levels) {
    float r = (x - z) / s;                 // IEEE fp32 division (correctly rounded)
    r = __builtin_rintf(r);                // round half to even
    r = fminf(fmaxf(r, 0.0f), levels);     // NaN (0/0) -> 0
    return s == 0.0f ? 0u : (uint32_t)r;
}

// Group constants: zero-point and scale (for the exact path), and for the fast path y ~ 1/s,
// c0 = fl(-z * y) and the tolerance below (y = c0 = 0 when the scale is 0, which makes every code
// of the group 0).  The key kernel keeps them in LDS as one array per constant, so that the
// constants of the consecutive channels a word covers are read as vectors (3 % on that kernel; the
// same for the consecutive tokens of a value word gained 3 % at 4 bits and lost 4 % at 2 bits).
struct GroupConst { float z, s, y, c0, tol; };

__device__ __forceinline__ GroupConst group_const(float lo, float s) {
    // y: the hardware reciprocal (1 ulp: relative error <= 2^-23), one instruction instead of a division
    const float y = s == 0.0f ? 0.0f : __builtin_amdgcn_rcpf(s);
    const float c0 = -lo * y;
    // q' = fl(x * y + c0) against the contract's q = fl(fl(x - z) / s), with Q the exact quotient:
    // |q - Q| <= Q * 2^-23 and |q' - Q| <= Q * 2^-22 + |z / s| * 2^-22 * 1.001 (error of y in both
    // products, roundings of c0 and of the sum), so for Q <= 16.1:  |q' - q| < 5.8e-6 + |c0| * 2.4e-7.
    // Twice that as tolerance.
    // (scale below the smallest normal fp16 number: its rounding error is not relative, the quotient
    // can pass `levels`: tolerance 1 = always the exact path)
    return GroupConst{lo, s, y, c0, (s != 0.0f && s < 6.103515625e-05f) ? 1.0f : 1.2e-5f + fabsf(c0) * 4.8e-7f};
}

// The same code as encode() without a division per element: one fused multiply-add straight from
// the fp16 input.  rint(q') == rint(q) unless q' lies within |q' - q| of a half-integer; `dev`
// collects the largest distance |q' - rint(q')| over the codes of a word, and the caller redoes the
// word with encode() when it exceeds 0.5 - tolerance.  No clamp: x >= z keeps the quotient at or
// above -tolerance, and with a normal fp16 scale s >= (max - min) / levels * (1 - 2^-11) it stays
// below levels + 0.008; a group whose scale is an fp16 subnormal gets a tolerance that sends its
// tile down the exact path (group_const).  Returns the code as a float.
__device__ __forceinline__ float encode_fast(__half x, float y, float c0, float& dev) {
    const float q = fmaf(__half2float(x), y, c0);
    const float r = __builtin_rintf(q);
    dev = fmaxf(dev, fabsf(q - r));
    return r;
}

// maximum over the 64 lanes of a wavefront (every lane gets it): DPP moves inside the rows of 16
// lanes, then the four rows through scalar registers
__device__ __forceinline__ float wave_max(float v) {
    auto dpp = [](float x, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    v = fmaxf(v, dpp(v, std::integral_constant<int, 0xB1>{}));     // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp(v, std::integral_constant<int, 0x4E>{}));     // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp(v, std::integral_constant<int, 0x141>{}));    // lane i <-> 7 - i within 8
    v = fmaxf(v, dpp(v, std::integral_constant<int, 0x140>{}));    // lane i <-> 15 - i within 16
    auto lane = [&](int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); };
    return fmaxf(fmaxf(lane(0), lane(16)), fmaxf(lane(32), lane(48)));
}

// A 32-bit word assembled from float codes: the low and the high 16 bits each stay exact in fp32.
struct WordAcc {
    float lo = 0.f, hi = 0.f;
    __device__ __forceinline__ void add(float code, int bit) {
        if (bit < 16) lo = fmaf(code, (float)(1u << bit), lo);
        else hi = fmaf(code, (float)(1u << (bit - 16)), hi);
    }
    __device__ __forceinline__ uint32_t word() const { return (uint32_t)lo | ((uint32_t)hi << 16); }
};

// (u, e) of the code at bit `bit` of word `wd`; lane is implied by wd.
template <int BITS>
__device__ __forceinline__ void word_coords(int wd, int bit, int& lane, int& u, int& e) {
    const int hf = bit >> 4;
    if (BITS == 2) {
        lane = wd >> 2;
        const int r = (bit & 15) >> 1;     // (u&1)*4 + (e>>1)
        u = (wd & 3) * 2 + (r >> 2);
        e = (r & 3) * 2 + hf;
    } else {
        lane = (wd & 255) >> 2;
        const int i = (wd >> 8) * 4 + (wd & 3);   // (u>>1)*2 + (e>>2)
        const int r = (bit & 15) >> 2;            // (u&1)*2 + ((e>>1)&1)
        u = (i >> 1) * 2 + (r >> 1);
        e = (i & 1) * 4 + (r & 1) * 2 + hf;
    }
}

// One workgroup quantises one key group: TG tiles of 32 tokens (G = 32 * TG tokens per group).
// Scale and zero-point rows are stored once per group (row (tile / TG) of the arrays).
// (A device function so that it can also run as a role of a wider launch: group g of kv-head h of
// batch entry b; 256 threads work, any further threads of the workgroup only keep the barriers.)
template <int BITS, int TG>
__device__ __forceinline__ void quantize_key_block(const QuantKeyParams& p, int g, int h, int b, int tid) {
    constexpr int kRows = TG * kTileTokens;
    __shared__ __align__(16) __half tile[kRows][kRowPad];
    __shared__ __align__(16) float sh_y[kHeadDim], sh_c0[kHeadDim], sh_z[kHeadDim], sh_s[kHeadDim];
    __shared__ float sh_tol[4];         // per wavefront: largest fast-path tolerance of its groups
    __shared__ half2v sh_lo[4][kHeadDim / 2], sh_hi[4][kHeadDim / 2];
    const bool active = tid < 256;
    constexpr float levels = (float)((1 << BITS) - 1);
    const int64_t unit = (int64_t)b * p.n_kv_heads + h;

    if (!active) {
        // nothing to load
    } else if (p.src.ring_cap > 0) {
#pragma unroll
        for (int pass = 0; pass < 2 * TG; ++pass) {
            const int row = pass * 16 + (tid >> 4), seg = tid & 15;
            *reinterpret_cast<uint4*>(&tile[row][seg * 8]) = *reinterpret_cast<const uint4*>(
                p.src.base + row_offset(p.src, b, h, g * kRows + row) + seg * 8);
        }
    } else {
        // a plain source (prefill): one row address per thread, the other passes lie 16 rows further each
        const __half* src = p.src.base + row_offset(p.src, b, h, g * kRows + (tid >> 4)) + (tid & 15) * 8;
        const int64_t step = 16 * p.src.stride_t;
#pragma unroll
        for (int pass = 0; pass < 2 * TG; ++pass)
            *reinterpret_cast<uint4*>(&tile[pass * 16 + (tid >> 4)][(tid & 15) * 8]) =
                *reinterpret_cast<const uint4*>(src + pass * step);
    }
    __syncthreads();

    const int dst_tile = p.first_tile + g * TG;
    // Group minimum / maximum with all 256 threads: wavefront w scans a quarter of the group's
    // tokens for a channel pair with packed fp16 min / max (exact: no arithmetic), then 128 threads
    // combine the four partial results of their channel.
    if (active) {
        const int cp = tid & 63, tq = tid >> 6;
        half2v lo2 = *reinterpret_cast<const half2v*>(&tile[tq * (kRows / 4)][2 * cp]), hi2 = lo2;
#pragma unroll
        for (int i = 1; i < kRows / 4; ++i) {
            const half2v x = *reinterpret_cast<const half2v*>(&tile[tq * (kRows / 4) + i][2 * cp]);
            lo2 = pk_min(lo2, x);
            hi2 = pk_max(hi2, x);
        }
        sh_lo[tq][cp] = lo2;
        sh_hi[tq][cp] = hi2;
    }
    __syncthreads();
    if (tid < kHeadDim) {
        const __half* plo = reinterpret_cast<const __half*>(&sh_lo[0][0]);
        const __half* phi = reinterpret_cast<const __half*>(&sh_hi[0][0]);
        float lo = __half2float(plo[tid]), hi = __half2float(phi[tid]);
#pragma unroll
        for (int tq = 1; tq < 4; ++tq) {
            lo = fminf(lo, __half2float(plo[tq * kHeadDim + tid]));
            hi = fmaxf(hi, __half2float(phi[tq * kHeadDim + tid]));
        }
        const __half s16 = __float2half_rn((hi - lo) / levels);
        {
            // one row of scales / zero-points per group (dst_tile is a multiple of TG, and so is cap_tiles)
            const int64_t o = (unit * p.cap_tiles + dst_tile) / TG * kHeadDim + tid;
            p.scale[o] = s16;
            p.zero[o] = __float2half_rn(lo);
        }
        const GroupConst gc = group_const(lo, __half2float(s16));
        sh_y[tid] = gc.y; sh_c0[tid] = gc.c0; sh_z[tid] = gc.z; sh_s[tid] = gc.s;
        const float wt = wave_max(gc.tol);                    // tid < 128: wavefronts 0 and 1, all lanes active
        if ((tid & 63) == 0) sh_tol[tid >> 6] = wt;
    }
    __syncthreads();
    const float tile_tol = fmaxf(sh_tol[0], sh_tol[1]);

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;     // the TG tiles are consecutive
    // A word of a key tile holds, for two tokens (t0, t0 + 16), a run of 8 (B = 2) or 4 (B = 4)
    // consecutive channels: read each run from LDS as one vector (2-byte reads of a column of
    // 16-byte-aligned rows hit only every fourth bank) and the group constants of the run once.
    constexpr int RUN = 16 / BITS;
    for (int wi = active ? tid : TG * kWords; wi < TG * kWords; wi += 256) {
        const int ti = wi / kWords, wd = wi % kWords;
        int lane, c0;
        if (BITS == 2) {
            lane = wd >> 2;
            c0 = (wd & 3) * 32 + (lane >> 4) * 8;
        } else {
            lane = (wd & 255) >> 2;
            const int i = (wd >> 8) * 4 + (wd & 3);
            c0 = (i >> 1) * 32 + (lane >> 4) * 8 + (i & 1) * 4;
        }
        const int t0 = ti * kTileTokens + (lane & 15);
        union Run { uint4 v4; uint2 v2; __half h[8]; } x[2];
#pragma unroll
        for (int uo = 0; uo < 2; ++uo) {
            if (BITS == 2) x[uo].v4 = *reinterpret_cast<const uint4*>(&tile[t0 + uo * 16][c0]);
            else x[uo].v2 = *reinterpret_cast<const uint2*>(&tile[t0 + uo * 16][c0]);
        }
        WordAcc acc;
        float dev = 0.0f;
        float ys[RUN], cs[RUN];
#pragma unroll
        for (int el = 0; el < RUN; el += 4) {
            *reinterpret_cast<float4*>(&ys[el]) = *reinterpret_cast<const float4*>(&sh_y[c0 + el]);
            *reinterpret_cast<float4*>(&cs[el]) = *reinterpret_cast<const float4*>(&sh_c0[c0 + el]);
        }
#pragma unroll
        for (int el = 0; el < RUN; ++el) {
#pragma unroll
            for (int uo = 0; uo < 2; ++uo) {
                const int bit = (el & 1) * 16 + (BITS == 2 ? 2 * (uo * 4 + (el >> 1)) : 4 * (uo * 2 + ((el >> 1) & 1)));
                acc.add(encode_fast(x[uo].h[el], ys[el], cs[el], dev), bit);
            }
        }
        uint32_t w = acc.word();
        if (dev > 0.5f - tile_tol) {     // rare: a quotient next to a rounding tie; redo the word with true divisions
            w = 0;
#pragma unroll
            for (int el = 0; el < RUN; ++el) {
#pragma unroll
                for (int uo = 0; uo < 2; ++uo) {
                    const int bit = (el & 1) * 16 + (BITS == 2 ? 2 * (uo * 4 + (el >> 1)) : 4 * (uo * 2 + ((el >> 1) & 1)));
                    w |= encode(__half2float(x[uo].h[el]), sh_z[c0 + el], sh_s[c0 + el], levels) << bit;
                }
            }
        }
        dst[wi] = w;
    }
}

// One workgroup quantises kValueTilesPerGroup consecutive value tiles (block index bx along the
// tiles).  A device function for the same reason as quantize_key_block.
template <int BITS>
__device__ __forceinline__ void quantize_value_block(const QuantValueParams& p, int bx, int h, int b, int tid) {
    __shared__ __align__(16) __half tile[kTileTokens][kRowPad];
    __shared__ GroupConst sh_g[kTileTokens][4];
    __shared__ float2 sh_mm[kTileTokens][4];    // per (token, 32-channel block): group minimum, maximum
    __shared__ float sh_tol[4];         // per wavefront: largest fast-path tolerance of its groups
    const bool active = tid < 256;
    constexpr float levels = (float)((1 << BITS) - 1);
    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    // kValueTilesPerGroup consecutive destination tiles per workgroup, next tile's rows prefetched
    const int first_tile = p.first_token / kTileTokens;
    const int n_tiles = (p.first_token + p.n_tokens - 1) / kTileTokens - first_tile + 1;
    const int i_lo = bx * kValueTilesPerGroup, i_hi = min(i_lo + kValueTilesPerGroup, n_tiles);
    uint4 rows[2];
    auto request = [&](int i) {
        const int dt = first_tile + i;
        const int lo = max(p.first_token - dt * kTileTokens, 0);
        const int hi = min(p.first_token + p.n_tokens - dt * kTileTokens, kTileTokens);
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int row = pass * 16 + (tid >> 4), seg = tid & 15;
            rows[pass] = uint4{0u, 0u, 0u, 0u};
            if (active && row >= lo && row < hi)
                rows[pass] = *reinterpret_cast<const uint4*>(
                    p.src.base + row_offset(p.src, b, h, dt * kTileTokens + row - p.first_token) + seg * 8);
        }
    };
    request(i_lo);
    for (int i = i_lo; i < i_hi; ++i) {
    const int dst_tile = first_tile + i;
    // destination tokens of this tile that this call writes: [lo, hi) within the tile
    const int lo_tok = max(p.first_token - dst_tile * kTileTokens, 0);
    const int hi_tok = min(p.first_token + p.n_tokens - dst_tile * kTileTokens, kTileTokens);
    if (active) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass)
            *reinterpret_cast<uint4*>(&tile[pass * 16 + (tid >> 4)][(tid & 15) * 8]) = rows[pass];
    }
    __syncthreads();
    if (i + 1 < i_hi) request(i + 1);
    const bool full = (lo_tok == 0 && hi_tok == kTileTokens);

    // Group minimum / maximum with all 256 threads: two threads per (token, channel group), each
    // reduces 16 channels with packed fp16 min / max (exact), partner lanes combine.
    if (active) {
        const int t = tid >> 3, cg = (tid >> 1) & 3, part = tid & 1;
        union { uint4 v; half2v h[4]; } a, c;
        a.v = *reinterpret_cast<const uint4*>(&tile[t][cg * 32 + part * 16]);
        c.v = *reinterpret_cast<const uint4*>(&tile[t][cg * 32 + part * 16 + 8]);
        const half2v lo2 = pk_min(pk_min(pk_min(a.h[0], a.h[1]), pk_min(a.h[2], a.h[3])),
                              pk_min(pk_min(c.h[0], c.h[1]), pk_min(c.h[2], c.h[3])));
        const half2v hi2 = pk_max(pk_max(pk_max(a.h[0], a.h[1]), pk_max(a.h[2], a.h[3])),
                              pk_max(pk_max(c.h[0], c.h[1]), pk_max(c.h[2], c.h[3])));
        float lo = fminf((float)lo2.x, (float)lo2.y), hi = fmaxf((float)hi2.x, (float)hi2.y);
        // partner lanes by DPP moves: xor 1 and xor 2 as quad permutations; for xor 4 the mirror
        // inside 8 lanes does, because by then the four lanes of a quad hold the same value
        auto dpp = [](float x, auto ctrl) {
            return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true));
        };
        const std::integral_constant<int, 0xB1> xor1{};
        const std::integral_constant<int, 0x4E> xor2{};
        const std::integral_constant<int, 0x141> mirror8{};
        lo = fminf(lo, dpp(lo, xor1));
        hi = fmaxf(hi, dpp(hi, xor1));
        // G = 64 or 128 channels per group: combine 2 or 4 neighbouring 32-channel blocks (every block
        // then holds the group's minimum and maximum; the first one stores its scale and zero-point)
        if (p.group_blocks >= 2) { lo = fminf(lo, dpp(lo, xor2)); hi = fmaxf(hi, dpp(hi, xor2)); }
        if (p.group_blocks >= 4) { lo = fminf(lo, dpp(lo, mirror8)); hi = fmaxf(hi, dpp(hi, mirror8)); }
        if (part == 0) sh_mm[t][cg] = make_float2(lo, hi);
    }
    __syncthreads();
    // the group constants on two wavefronts with every lane busy (one (token, channel block) each)
    // instead of on every other lane of all four
    if (tid < 4 * kTileTokens) {
        const int t = tid >> 2, cg = tid & 3;
        float my_tol = 0.0f;
        if (t >= lo_tok && t < hi_tok) {
            const float2 mm = sh_mm[t][cg];
            const __half s16 = __float2half_rn((mm.y - mm.x) / levels);
            // one entry per group: 4 / group_blocks of them per token, written by the group's first block
            if (cg % p.group_blocks == 0) {
                const int64_t o = ((unit * p.cap_tiles + dst_tile) * kTileTokens + t) * (4 / p.group_blocks) + cg / p.group_blocks;
                p.scale[o] = s16;
                p.zero[o] = __float2half_rn(mm.x);
            }
            const GroupConst gc = group_const(mm.x, __half2float(s16));
            sh_g[t][cg] = gc;
            my_tol = gc.tol;
        }
        const float wt = wave_max(my_tol);
        if ((tid & 63) == 0) sh_tol[tid >> 6] = wt;
    }
    __syncthreads();
    const float tile_tol = fmaxf(sh_tol[0], sh_tol[1]);

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;
    // One word of the packed tile.  FULL: every token of the tile is written by this call (the case
    // of a prefill) -- no test per code; otherwise only the tokens [lo_tok, hi_tok) are encoded and
    // the other codes of the word, written by earlier calls, are kept.
    auto encode_word = [&](int wd, auto full_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value;
        WordAcc acc;
        uint32_t mask = 0;
        float dev = 0.0f;
#pragma unroll
        for (int bit = 0; bit < 32; bit += BITS) {
            int lane, u, e;
            word_coords<BITS>(wd, bit, lane, u, e);
            const int c = u * 16 + (lane & 15);
            const int t = (lane >> 4) * 8 + e;
            if (FULL || (t >= lo_tok && t < hi_tok)) {
                acc.add(encode_fast(tile[t][c], sh_g[t][c >> 5].y, sh_g[t][c >> 5].c0, dev), bit);
                mask |= (uint32_t)((1 << BITS) - 1) << bit;
            }
        }
        uint32_t w = acc.word();
        if (dev > 0.5f - tile_tol) {     // rare: a quotient next to a rounding tie; redo the word with true divisions
            w = 0;
#pragma unroll
            for (int bit = 0; bit < 32; bit += BITS) {
                int lane, u, e;
                word_coords<BITS>(wd, bit, lane, u, e);
                const int c = u * 16 + (lane & 15);
                const int t = (lane >> 4) * 8 + e;
                if (FULL || (t >= lo_tok && t < hi_tok))
                    w |= encode(__half2float(tile[t][c]), sh_g[t][c >> 5].z, sh_g[t][c >> 5].s, levels) << bit;
            }
        }
        if (FULL) {
            dst[wd] = w;
        } else if (mask) {
            // a partly filled tile: keep the codes of the tokens written by earlier calls
            dst[wd] = (dst[wd] & ~mask) | w;
        }
    };
    if (full) {
        for (int wd = active ? tid : kWords; wd < kWords; wd += 256) encode_word(wd, std::true_type{});
    } else {
        for (int wd = active ? tid : kWords; wd < kWords; wd += 256) encode_word(wd, std::false_type{});
    }
    __syncthreads();          // the tile and the group constants are overwritten by the next tile
    }
}

// ---- prefill forms: one wavefront per tile, everything in registers ----
// The kernels above stage a tile in LDS and pass three barriers; at prefill sizes they are bound by
// instruction issue (868 / 1022 vector instructions per tile for keys / values at 2 bits).  For
// the bulk case -- a plain (non-ring) source, G = 32, whole tiles -- these forms give every wavefront
// a tile of its own: the lanes load the elements whose codes they will pack, group minimum and
// maximum come from packed fp16 min / max in registers plus at most two cross-lane steps, the
// partial words of the lanes that share a word are combined with DPP moves, and nothing goes
// through LDS.  Same arithmetic contract as above (encode_fast with the exact redo).
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xF, 0xF, true));
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E;      // quad_perm [1,0,3,2], [2,3,0,1]
__device__ __forceinline__ uint32_t as_bits(half2v x) {
    union { half2v h; uint32_t u; } a;
    a.h = x;
    return a.u;
}
__device__ __forceinline__ half2v as_half2(uint32_t x) {
    union { half2v h; uint32_t u; } a;
    a.u = x;
    return a.h;
}
__device__ __forceinline__ float half_bits_to_float(uint32_t low16) { return (float)as_half2(low16).x; }
// {a.x, b.x} and {a.y, b.y} (one byte-permute instruction each)
__device__ __forceinline__ half2v low_halves(half2v a, half2v b) {
    return as_half2(__builtin_amdgcn_perm(as_bits(b), as_bits(a), 0x05040100u));
}
__device__ __forceinline__ half2v high_halves(half2v a, half2v b) {
    return as_half2(__builtin_amdgcn_perm(as_bits(b), as_bits(a), 0x07060302u));
}
template <int CTRL>
__device__ __forceinline__ half2v dpp_h2(half2v x) {
    union { half2v h; int i; } a, r;
    a.h = x;
    r.i = __builtin_amdgcn_mov_dpp(a.i, CTRL, 0xF, 0xF, true);
    return r.h;
}
// A wavefront-uniform pointer pinned to scalar registers: keeps the compiler from folding a lane offset
// into it early and then carrying every row address in vector registers (64-bit vector multiply-adds).
typedef const half2v __attribute__((address_space(1)))* GlobalHalf2Ptr;       // keeps the loads global (not flat)
__device__ __forceinline__ GlobalHalf2Ptr uniform_pointer(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<GlobalHalf2Ptr>(((uint64_t)hi << 32) | lo);
}
// mask ? a : b per bit (one bitfield-insert instruction)
__device__ __forceinline__ uint32_t select_bits(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

__device__ __forceinline__ float encode_fast16(_Float16 x, float y, float c0, float& dev) {
    const float q = fmaf((float)x, y, c0);
    const float r = __builtin_rintf(q);
    dev = fmaxf(dev, fabsf(q - r));
    return r;
}

// Keys: lane l holds channels 2l, 2l + 1 of all 32 tokens (each row load of the wavefront is one
// contiguous 256-byte row).  A channel's group is the lane's own column: no cross-lane step for
// minimum and maximum.  A word of the packed tile (tokens t0 and t0 + 16, 8 or 4 consecutive
// channels) is shared by 4 (B = 2) or 2 (B = 4) neighbouring lanes.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_keys_stream_kernel(QuantKeyParams p) {
    const int lane = threadIdx.x & 63;
    const int g = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // group = tile
    if (g >= p.n_tiles) return;                     // whole wavefronts leave; the kernel has no barrier
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    constexpr float levels = (float)((1 << BITS) - 1);
    // (the row address stays wavefront-uniform and the lane adds a 32-bit offset: scalar address arithmetic)
    const __half* src = p.src.base + (int64_t)b * p.src.stride_b + (int64_t)h * p.src.stride_h
                        + (int64_t)g * kTileTokens * p.src.stride_t;
    half2v x[kTileTokens];
#pragma unroll
    for (int t = 0; t < kTileTokens; ++t)
        x[t] = __builtin_nontemporal_load(uniform_pointer(src + t * p.src.stride_t) + (uint32_t)lane);

    half2v mn[16], mx[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { mn[i] = pk_min(x[i], x[i + 16]); mx[i] = pk_max(x[i], x[i + 16]); }
#pragma unroll
    for (int w = 8; w >= 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w; ++i) { mn[i] = pk_min(mn[i], mn[i + w]); mx[i] = pk_max(mx[i], mx[i + w]); }

    float y[2], c0[2], zf[2], sf[2], tol = 0.f;
    half2v s2, z2;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float lo = (float)mn[0][i], hi = (float)mx[0][i];
        const _Float16 s16 = (_Float16)((hi - lo) / levels);          // fp32 division, rounded to nearest even
        const GroupConst gc = group_const(lo, (float)s16);
        y[i] = gc.y; c0[i] = gc.c0; zf[i] = gc.z; sf[i] = gc.s;
        tol = fmaxf(tol, gc.tol);
        s2[i] = s16;
        z2[i] = mn[0][i];
    }
    const int dst_tile = p.first_tile + g;
    const int64_t o = (unit * p.cap_tiles + dst_tile) * kHeadDim + 2 * lane;
    *reinterpret_cast<half2v*>(p.scale + o) = s2;
    *reinterpret_cast<half2v*>(p.zero + o) = z2;

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;
    const int ks = lane >> 4, q = (lane >> 2) & 3, k = lane & 3;     // channel 2l = ks*32 + q*8 + 2k
    const int shift = BITS == 2 ? 2 * k : 4 * (k & 1);
    const uint32_t m0 = 0u - (uint32_t)(k & 1), m1 = 0u - (uint32_t)(k >> 1);
    const float thr = 0.5f - tol;
    // four tokens t0 (and their partners t0 + 16) at a time: byte i*2 + uo of the lane's partial word
    // holds the code of (channel 2l + i, token t0 + 16 uo) -- bits (e&1)*16 + 8*uo of the layout --
    // and the shift moves it to the lane's channel pair
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
        uint32_t pw[4];
        float dev = 0.f;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const int t0 = blk * 4 + tt;
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int uo = 0; uo < 2; ++uo)
                    w = __builtin_amdgcn_cvt_pk_u8_f32(encode_fast16(x[t0 + 16 * uo][i], y[i], c0[i], dev), i * 2 + uo, w);
            pw[tt] = w;
        }
        if (dev > thr) {      // rare: a quotient next to a rounding tie; redo the lane's 16 codes with true divisions
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int t0 = blk * 4 + tt;
                uint32_t w = 0;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int uo = 0; uo < 2; ++uo)
                        w |= encode((float)x[t0 + 16 * uo][i], zf[i], sf[i], levels) << (8 * (i * 2 + uo));
                pw[tt] = w;
            }
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) pw[tt] <<= shift;
        // The lanes that share a word combine their partial words so that each ends up with a different
        // token's complete word (a transpose over the lane group, 3 instructions per exchange): with the
        // odd neighbour, the odd lane keeps the odd tokens and hands over the even ones, and vice versa;
        // at 2 bits the same once more two lanes apart.
        const uint32_t a = select_bits(m0, pw[1], pw[0]) | dpp_u32<kQuadXor1>(select_bits(m0, pw[0], pw[1]));   // token (k & 1)
        const uint32_t c = select_bits(m0, pw[3], pw[2]) | dpp_u32<kQuadXor1>(select_bits(m0, pw[2], pw[3]));   // token 2 + (k & 1)
        if (BITS == 2) {
            const uint32_t w = select_bits(m1, c, a) | dpp_u32<kQuadXor2>(select_bits(m1, a, c));               // token k
            dst[(q * 16 + blk * 4 + k) * 4 + ks] = w;
        } else {
            const int i = ks * 2 + (k >> 1);
            dst[(i >> 2) * 256 + (q * 16 + blk * 4 + (k & 1)) * 4 + (i & 3)] = a;
            dst[(i >> 2) * 256 + (q * 16 + blk * 4 + 2 + (k & 1)) * 4 + (i & 3)] = c;
        }
    }
}

// Values: lane (tl = l / 16, seg = l % 16) holds channels seg*8 .. seg*8 + 7 of tokens 8 tl .. 8 tl + 7
// (a 16-byte load per token).  A group is 32 channels of a token = the 4 lanes of a quad; lane jj of
// the quad derives the constants of tokens jj and jj + 4 and the others get them by quad broadcasts.
// A word (8 tokens, channels c and c + 16) is shared by the lanes seg and seg ^ 2.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_values_stream_kernel(QuantValueParams p) {
    const int lane = threadIdx.x & 63;
    const int ti = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (ti >= p.n_tokens / kTileTokens) return;     // whole wavefronts leave; the kernel has no barrier
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    constexpr float levels = (float)((1 << BITS) - 1);
    const int dst_tile = p.first_token / kTileTokens + ti;
    const int tl = lane >> 4, seg = lane & 15, g = seg >> 2, jj = seg & 3, odd = (seg >> 1) & 1;
    const __half* src = p.src.base + (int64_t)b * p.src.stride_b + (int64_t)h * p.src.stride_h
                        + ((int64_t)ti * kTileTokens + tl * 8) * p.src.stride_t + seg * 8;
    typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
    union Row { uint4v v4; half2v h2[4]; _Float16 h[8]; } x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i].v4 = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(src + i * p.src.stride_t));

    // Group minimum / maximum of every token.  In the lane: packed fp16 min / max over its 8 channels
    // (exact, no arithmetic); the halves of two tokens are then combined into one register
    // (token i in the low half, token i + 1 in the high half), so that the two exchanges inside the quad
    // serve two tokens at once.  Lane jj adopts the tokens jj and jj + 4.
    half2v pmn[4], pmx[4];
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        half2v lo2[2], hi2[2];
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            lo2[d] = pk_min(pk_min(x[i + d].h2[0], x[i + d].h2[1]), pk_min(x[i + d].h2[2], x[i + d].h2[3]));
            hi2[d] = pk_max(pk_max(x[i + d].h2[0], x[i + d].h2[1]), pk_max(x[i + d].h2[2], x[i + d].h2[3]));
        }
        half2v mn = pk_min(low_halves(lo2[0], lo2[1]), high_halves(lo2[0], lo2[1]));
        half2v mx = pk_max(low_halves(hi2[0], hi2[1]), high_halves(hi2[0], hi2[1]));
        mn = pk_min(mn, dpp_h2<kQuadXor1>(mn)); mx = pk_max(mx, dpp_h2<kQuadXor1>(mx));
        mn = pk_min(mn, dpp_h2<kQuadXor2>(mn)); mx = pk_max(mx, dpp_h2<kQuadXor2>(mx));
        pmn[i >> 1] = mn;
        pmx[i >> 1] = mx;
    }
    float my_lo[2], my_hi[2];
    {
        const uint32_t upper = 0u - (uint32_t)(jj >> 1);     // tokens 2, 3 (6, 7) are in the second register of a slot
        const int sh = 16 * (jj & 1);
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            my_lo[sl] = half_bits_to_float(select_bits(upper, as_bits(pmn[2 * sl + 1]), as_bits(pmn[2 * sl])) >> sh);
            my_hi[sl] = half_bits_to_float(select_bits(upper, as_bits(pmx[2 * sl + 1]), as_bits(pmx[2 * sl])) >> sh);
        }
    }
    float gy[2], gc0[2], gz[2], gs[2], tol = 0.f;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
        const _Float16 s16 = (_Float16)((my_hi[sl] - my_lo[sl]) / levels);
        const GroupConst gc = group_const(my_lo[sl], (float)s16);
        gy[sl] = gc.y; gc0[sl] = gc.c0; gz[sl] = gc.z; gs[sl] = gc.s;
        tol = fmaxf(tol, gc.tol);
        const int64_t o = ((unit * p.cap_tiles + dst_tile) * kTileTokens + tl * 8 + jj + 4 * sl) * 4 + g;
        reinterpret_cast<_Float16*>(p.scale)[o] = s16;
        reinterpret_cast<_Float16*>(p.zero)[o] = (_Float16)my_lo[sl];
    }
    tol = fmaxf(tol, dpp_f32<kQuadXor1>(tol));
    tol = fmaxf(tol, dpp_f32<kQuadXor2>(tol));
    const float thr = 0.5f - tol;
    // constants of token i for every lane of the quad: from lane i & 3, slot i >> 2
    auto quad_bcast = [](float v, auto sel) {
        constexpr int S = decltype(sel)::value;
        return dpp_f32<S | (S << 2) | (S << 4) | (S << 6)>(v);
    };
    float yi[8], ci[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        auto pick = [&](const float (&a)[2]) {
            const float v = a[i >> 2];
            switch (i & 3) {
                case 0: return quad_bcast(v, std::integral_constant<int, 0>{});
                case 1: return quad_bcast(v, std::integral_constant<int, 1>{});
                case 2: return quad_bcast(v, std::integral_constant<int, 2>{});
                default: return quad_bcast(v, std::integral_constant<int, 3>{});
            }
        };
        yi[i] = pick(gy);
        ci[i] = pick(gc0);
    }

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    constexpr int WPC = BITS / 2;                    // words per channel: tokens 0-7 (B = 2) or 0-3, 4-7 (B = 4)
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;
    uint32_t wq[8][WPC];
    // two channels at a time; bit of token e inside its word: (e&1)*16 + B*((e>>1) & (8/B - 1)), plus 8 for
    // the lanes whose channels are the upper 16 of their 32-channel group (odd)
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        float dev = 0.f;
#pragma unroll
        for (int j = 2 * jb; j < 2 * jb + 2; ++j) {
            // the codes of a word lie in bits 0-7 and 16-23: their sum is exact in one fp32 number
            float acc[WPC];
#pragma unroll
            for (int a = 0; a < WPC; ++a) acc[a] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int bit = (e & 1) * 16 + BITS * ((e >> 1) & (8 / BITS - 1));
                float& dstf = acc[BITS == 2 ? 0 : (e >> 2)];
                dstf = fmaf(encode_fast16(x[e].h[j], yi[e], ci[e], dev), (float)(1u << bit), dstf);
            }
#pragma unroll
            for (int a = 0; a < WPC; ++a) wq[j][a] = (uint32_t)acc[a];
        }
        // a quotient next to a rounding tie anywhere in the wavefront (rare): all lanes redo these two
        // channels with true divisions (uniform branch: the quad broadcasts inside need every lane)
        if (__builtin_amdgcn_ballot_w64(dev > thr) != 0) {
            float zi[8], si[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                auto pick = [&](const float (&a)[2]) {
                    const float v = a[i >> 2];
                    switch (i & 3) {
                        case 0: return quad_bcast(v, std::integral_constant<int, 0>{});
                        case 1: return quad_bcast(v, std::integral_constant<int, 1>{});
                        case 2: return quad_bcast(v, std::integral_constant<int, 2>{});
                        default: return quad_bcast(v, std::integral_constant<int, 3>{});
                    }
                };
                zi[i] = pick(gz);
                si[i] = pick(gs);
            }
#pragma unroll
            for (int j = 2 * jb; j < 2 * jb + 2; ++j) {
                uint32_t w[WPC];
#pragma unroll
                for (int a = 0; a < WPC; ++a) w[a] = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int bit = (e & 1) * 16 + BITS * ((e >> 1) & (8 / BITS - 1));
                    w[BITS == 2 ? 0 : (e >> 2)] |= encode((float)x[e].h[j], zi[e], si[e], levels) << bit;
                }
#pragma unroll
                for (int a = 0; a < WPC; ++a) wq[j][a] = w[a];
            }
        }
    }
    // combine with the lane that holds the other 16 channels of the group, then each of the two stores
    // four of the eight channels' words
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int a = 0; a < WPC; ++a) {
            uint32_t w = wq[j][a] << (8 * odd);
            w |= dpp_u32<kQuadXor2>(w);
            wq[j][a] = w;
        }
    const uint32_t omask = 0u - (uint32_t)odd;
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int a = 0; a < WPC; ++a) {
            const uint32_t mine = (wq[m + 4][a] & omask) | (wq[m][a] & ~omask);     // a bitfield insert, not an indexed array
            const int r = (seg & 1) * 8 + m + 4 * odd;             // channel % 16
            if (BITS == 2) {
                dst[(tl * 16 + r) * 4 + g] = mine;
            } else {
                const int i = g * 2 + a;
                dst[(i >> 2) * 256 + (tl * 16 + r) * 4 + (i & 3)] = mine;
            }
        }
}

template <int BITS, int TG>
__global__ __launch_bounds__(256) void quantize_keys_kernel(QuantKeyParams p) {
    quantize_key_block<BITS, TG>(p, blockIdx.x, blockIdx.y, blockIdx.z, threadIdx.x);
}

template <int BITS>
__global__ __launch_bounds__(256) void quantize_values_kernel(QuantValueParams p) {
    quantize_value_block<BITS>(p, blockIdx.x, blockIdx.y, blockIdx.z, threadIdx.x);
}

// A residual flush in one launch: the first n_key_blocks workgroups along x quantise key groups, the
// others value tiles (Algorithm 1, Decoding: both residual parts are flushed in the same step).
template <int BITS, int TG>
__global__ __launch_bounds__(256) void flush_quantize_kernel(QuantKeyParams kp, QuantValueParams vp, int n_key_blocks) {
    if ((int)blockIdx.x < n_key_blocks) quantize_key_block<BITS, TG>(kp, blockIdx.x, blockIdx.y, blockIdx.z, threadIdx.x);
    else quantize_value_block<BITS>(vp, (int)blockIdx.x - n_key_blocks, blockIdx.y, blockIdx.z, threadIdx.x);
}

// The first launch of a two-launch decode step that also flushes (Algorithm 1, Decoding): workgroups
// [0, units) serve the fp16 rows of one (batch, kv-head) unit each -- the rows that stay in the window
// -- and the following ones quantise, per unit, the key group and the value tokens that leave it.
// The two kinds touch disjoint memory; the launch of the all-quantised chunks that follows sees both
// results.  The workgroup size is the larger of the two roles' (the surplus threads idle).
template <int REP, int BITS>
__global__ __launch_bounds__(1024) void rows_flush_kernel(DecodeParams p, QuantKeyParams kp, QuantValueParams vp,
                                                          int tiles_b, int n_key_blocks, int n_value_blocks) {
    extern __shared__ float sm_dyn[];
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    int64_t bx = blockIdx.x;
    if (bx < units) {
        rows::residual_rows_block<REP>(p, sm_dyn, bx, tiles_b, threadIdx.x);
        return;
    }
    bx -= units;
    const int per_unit = n_key_blocks + n_value_blocks;
    const int unit = (int)(bx / per_unit), r = (int)(bx % per_unit);
    const int h = unit % kp.n_kv_heads, b = unit / kp.n_kv_heads;
    if (r < n_key_blocks) quantize_key_block<BITS, 1>(kp, r, h, b, threadIdx.x);
    else quantize_value_block<BITS>(vp, r - n_key_blocks, h, b, threadIdx.x);
}

__global__ __launch_bounds__(256) void copy_rows_kernel(CopyRowsParams p) {
    // one thread moves 16 bytes; blockIdx.x covers job 0's rows, then job 1's
    const int blocks0 = (p.job[0].n_tokens * 16 + 255) / 256;
    const int which = (int)blockIdx.x >= blocks0 ? 1 : 0;
    const CopyRowsParams::Job& j = p.job[which];
    const int i = ((int)blockIdx.x - (which ? blocks0 : 0)) * 256 + (int)threadIdx.x;
    const int h = blockIdx.y, b = blockIdx.z;
    if (i >= j.n_tokens * 16) return;
    const int t = i >> 4, seg = i & 15;
    const __half* src = j.src + (int64_t)b * j.stride_b + (int64_t)h * j.stride_h
                        + (int64_t)(j.src_t0 + t) * j.stride_t + seg * 8;
    const int slot = (j.dst_slot0 + t) % p.cap_r;
    __half* dst = j.dst + (((int64_t)b * p.n_kv_heads + h) * p.cap_r + slot) * kHeadDim + seg * 8;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}

// Measurement yardstick: plain read-only stream.  Every workgroup reads one contiguous 64 KB piece
// with four independent 16-byte loads per thread and trip (the fastest plain pattern found on this
// chip: 6.3-6.5 TB/s on 1 GiB against 5.3 TB/s for a 4096-workgroup grid-stride loop); the folded
// value goes to `sink` so that the loads cannot be dropped.
constexpr size_t kStreamPiece16 = 65536 / 16;     // 16-byte words per workgroup
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* src, size_t n16, uint32_t* sink) {
    const size_t lo = (size_t)blockIdx.x * kStreamPiece16, hi = min(lo + kStreamPiece16, n16);
    uint32_t x = 0;
    size_t i = lo + threadIdx.x;
    typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
    const uint4v* srcv = reinterpret_cast<const uint4v*>(src);
    for (; i + 768 < hi; i += 1024) {
        const uint4v a = __builtin_nontemporal_load(srcv + i), b = __builtin_nontemporal_load(srcv + i + 256), c = __builtin_nontemporal_load(srcv + i + 512), d = __builtin_nontemporal_load(srcv + i + 768);
        x ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < hi; i += 256) {
        const uint4 a = src[i];
        x ^= a.x ^ a.y ^ a.z ^ a.w;
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) x ^= __shfl_xor(x, m);
    if (threadIdx.x == 0) sink[blockIdx.x & 4095] = x;
}

}  // namespace

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t grid = (n16 + kStreamPiece16 - 1) / kStreamPiece16;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    stream_read_kernel<<<(unsigned)grid, 256, 0, stream>>>(static_cast<const uint4*>(src), n16, sink);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_keys_bits(const QuantKeyParams& p, hipStream_t stream) {
    const int tg = p.tiles_per_group;
    if (p.n_tiles % tg != 0) return hipErrorInvalidValue;
    dim3 grid(p.n_tiles / tg, p.n_kv_heads, p.batch), block(256);
    if (tg == 1) quantize_keys_kernel<BITS, 1><<<grid, block, 0, stream>>>(p);
    else if (tg == 2) quantize_keys_kernel<BITS, 2><<<grid, block, 0, stream>>>(p);
    else if (tg == 4) quantize_keys_kernel<BITS, 4><<<grid, block, 0, stream>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_quantize_keys(const QuantKeyParams& p, hipStream_t stream) {
    if (p.n_tiles <= 0) return hipSuccess;
    if (p.src.ring_cap == 0 && p.tiles_per_group == 1) {        // the bulk case: one wavefront per group
        dim3 grid((p.n_tiles + 3) / 4, p.n_kv_heads, p.batch), block(256);
        if (p.bits == 2) quantize_keys_stream_kernel<2><<<grid, block, 0, stream>>>(p);
        else quantize_keys_stream_kernel<4><<<grid, block, 0, stream>>>(p);
        return hipGetLastError();
    }
    return p.bits == 2 ? launch_keys_bits<2>(p, stream) : launch_keys_bits<4>(p, stream);
}

hipError_t launch_quantize_values(const QuantValueParams& p_in, hipStream_t stream) {
    if (p_in.n_tokens <= 0) return hipSuccess;
    QuantValueParams p = p_in;
    if (p.src.ring_cap == 0 && p.group_blocks == 1 && p.first_token % kTileTokens == 0 && p.n_tokens >= kTileTokens) {
        // the bulk case: whole tiles, one wavefront each; a last, partly filled tile goes the general way
        const int whole = p.n_tokens / kTileTokens;
        QuantValueParams pw = p;
        pw.n_tokens = whole * kTileTokens;
        dim3 grid((whole + 3) / 4, p.n_kv_heads, p.batch), block(256);
        if (p.bits == 2) quantize_values_stream_kernel<2><<<grid, block, 0, stream>>>(pw);
        else quantize_values_stream_kernel<4><<<grid, block, 0, stream>>>(pw);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
        p.src.base += (int64_t)pw.n_tokens * p.src.stride_t;
        p.first_token += pw.n_tokens;
        p.n_tokens -= pw.n_tokens;
        if (p.n_tokens == 0) return hipSuccess;
    }
    const int first_tile = p.first_token / kTileTokens;
    const int last_tile = (p.first_token + p.n_tokens - 1) / kTileTokens;
    dim3 grid((last_tile - first_tile + kValueTilesPerGroup) / kValueTilesPerGroup, p.n_kv_heads, p.batch), block(256);
    if (p.bits == 2) quantize_values_kernel<2><<<grid, block, 0, stream>>>(p);
    else quantize_values_kernel<4><<<grid, block, 0, stream>>>(p);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_flush_bits(const QuantKeyParams& kp, const QuantValueParams& vp, hipStream_t stream) {
    const int tg = kp.tiles_per_group;
    if (kp.n_tiles % tg != 0) return hipErrorInvalidValue;
    const int n_key_blocks = kp.n_tiles / tg;
    const int first_tile = vp.first_token / kTileTokens, last_tile = (vp.first_token + vp.n_tokens - 1) / kTileTokens;
    const int n_value_blocks = (last_tile - first_tile + kValueTilesPerGroup) / kValueTilesPerGroup;
    dim3 grid(n_key_blocks + n_value_blocks, kp.n_kv_heads, kp.batch), block(256);
    if (tg == 1) flush_quantize_kernel<BITS, 1><<<grid, block, 0, stream>>>(kp, vp, n_key_blocks);
    else if (tg == 2) flush_quantize_kernel<BITS, 2><<<grid, block, 0, stream>>>(kp, vp, n_key_blocks);
    else if (tg == 4) flush_quantize_kernel<BITS, 4><<<grid, block, 0, stream>>>(kp, vp, n_key_blocks);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_flush_quantize(const QuantKeyParams& kp, const QuantValueParams& vp, hipStream_t stream) {
    if (kp.n_tiles <= 0) return launch_quantize_values(vp, stream);
    if (vp.n_tokens <= 0) return launch_quantize_keys(kp, stream);
    return kp.bits == 2 ? launch_flush_bits<2>(kp, vp, stream) : launch_flush_bits<4>(kp, vp, stream);
}

hipError_t launch_rows_and_flush(const DecodeParams& p, const QuantKeyParams& kp, const QuantValueParams& vp,
                                 hipStream_t stream) {
    const int tiles_b = p.plan.tiles_total - p.plan.tiles_a;
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    const int rep = p.rep_variant <= 2 ? p.rep_variant : (p.rep_variant <= 4 ? 4 : 8);
    if (kp.tiles_per_group != 1 || vp.group_blocks != 1) return hipErrorNotSupported;
    if (!residual_rows_possible(tiles_b, rep) || p.plan.n_splits_b != 1 || p.n_kq != p.n_vq) return hipErrorInvalidValue;
    if (kp.bits != vp.bits || kp.n_tiles < 0 || vp.n_tokens < 0 || kp.n_tiles + vp.n_tokens <= 0) return hipErrorInvalidValue;
    const int n_key_blocks = kp.n_tiles;
    int n_value_blocks = 0;
    if (vp.n_tokens > 0) {
        const int first_tile = vp.first_token / kTileTokens, last_tile = (vp.first_token + vp.n_tokens - 1) / kTileTokens;
        n_value_blocks = (last_tile - first_tile + kValueTilesPerGroup) / kValueTilesPerGroup;
    }
    const int64_t blocks = units * (1 + n_key_blocks + n_value_blocks);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(std::max(256, 64 * tiles_b));
    const size_t lds = rows::rows_lds_bytes(tiles_b, rep);
    auto go = [&](auto rep_tag) {
        constexpr int R = decltype(rep_tag)::value;
        if (kp.bits == 2) rows_flush_kernel<R, 2><<<grid, block, lds, stream>>>(p, kp, vp, tiles_b, n_key_blocks, n_value_blocks);
        else rows_flush_kernel<R, 4><<<grid, block, lds, stream>>>(p, kp, vp, tiles_b, n_key_blocks, n_value_blocks);
    };
    if (rep == 1) go(std::integral_constant<int, 1>{});
    else if (rep == 2) go(std::integral_constant<int, 2>{});
    else if (rep == 4) go(std::integral_constant<int, 4>{});
    else go(std::integral_constant<int, 8>{});
    return hipGetLastError();
}

hipError_t launch_copy_rows(const CopyRowsParams& p, hipStream_t stream) {
    const int blocks = (p.job[0].n_tokens * 16 + 255) / 256 + (p.job[1].n_tokens * 16 + 255) / 256;
    if (blocks <= 0) return hipSuccess;
    dim3 grid(blocks, p.n_kv_heads, p.batch), block(256);
    copy_rows_kernel<<<grid, block, 0, stream>>>(p);
    return hipGetLastError();
}

}  // namespace kivi
