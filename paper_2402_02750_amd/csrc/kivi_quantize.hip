// Group-wise quantisation kernels for gfx950 (KIVI Section 3.1 formula; Section 3.3 grouping).
//
// One workgroup stages one 32-token x 128-channel fp16 tile in LDS (coalesced 16-byte loads),
// derives the per-group zero-point/scale, then every thread assembles whole 32-bit words of the
// packed tile, so all global stores are full, coalesced dwords.  The arithmetic of a code is
// bit-contract: fp32 subtract, IEEE fp32 division, round-half-even, clamp.  This file is
// compiled with -ffp-contract=off so no FMA can slip into it.
#include "kivi_internal.h"

#include <hip/hip_fp16.h>

namespace kivi {
namespace {

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

template <int BITS>
__global__ __launch_bounds__(256) void quantize_keys_kernel(QuantKeyParams p) {
    __shared__ __align__(16) __half tile[kTileTokens][kRowPad];
    __shared__ float sh_s[kHeadDim], sh_z[kHeadDim];
    const int g = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    constexpr float levels = (float)((1 << BITS) - 1);

#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int row = pass * 16 + (tid >> 4), seg = tid & 15;
        const __half* src = p.src.base + row_offset(p.src, b, h, g * kTileTokens + row) + seg * 8;
        *reinterpret_cast<uint4*>(&tile[row][seg * 8]) = *reinterpret_cast<const uint4*>(src);
    }
    __syncthreads();

    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    const int dst_tile = p.first_tile + g;
    if (tid < kHeadDim) {
        float lo = __half2float(tile[0][tid]), hi = lo;
#pragma unroll 8
        for (int t = 1; t < kTileTokens; ++t) {
            const float x = __half2float(tile[t][tid]);
            lo = fminf(lo, x);
            hi = fmaxf(hi, x);
        }
        const __half s16 = __float2half_rn((hi - lo) / levels);
        const int64_t o = (unit * p.cap_tiles + dst_tile) * kHeadDim + tid;
        p.scale[o] = s16;
        p.zero[o] = __float2half_rn(lo);
        sh_s[tid] = __half2float(s16);
        sh_z[tid] = lo;
    }
    __syncthreads();

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;
    for (int wd = tid; wd < kWords; wd += 256) {
        uint32_t w = 0;
#pragma unroll
        for (int bit = 0; bit < 32; bit += BITS) {
            int lane, u, e;
            word_coords<BITS>(wd, bit, lane, u, e);
            const int t = (u & 1) * 16 + (lane & 15);
            const int c = (u >> 1) * 32 + (lane >> 4) * 8 + e;
            w |= encode(__half2float(tile[t][c]), sh_z[c], sh_s[c], levels) << bit;
        }
        dst[wd] = w;
    }
}

template <int BITS>
__global__ __launch_bounds__(256) void quantize_values_kernel(QuantValueParams p) {
    __shared__ __align__(16) __half tile[kTileTokens][kRowPad];
    __shared__ float sh_s[kTileTokens][4], sh_z[kTileTokens][4];
    const int h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    constexpr float levels = (float)((1 << BITS) - 1);

    const int dst_tile = p.first_token / kTileTokens + blockIdx.x;
    // destination tokens of this tile that this call writes: [lo, hi) within the tile
    const int lo_tok = max(p.first_token - dst_tile * kTileTokens, 0);
    const int hi_tok = min(p.first_token + p.n_tokens - dst_tile * kTileTokens, kTileTokens);

#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int row = pass * 16 + (tid >> 4), seg = tid & 15;
        if (row >= lo_tok && row < hi_tok) {
            const int t_src = dst_tile * kTileTokens + row - p.first_token;
            const __half* src = p.src.base + row_offset(p.src, b, h, t_src) + seg * 8;
            *reinterpret_cast<uint4*>(&tile[row][seg * 8]) = *reinterpret_cast<const uint4*>(src);
        }
    }
    __syncthreads();

    const int64_t unit = (int64_t)b * p.n_kv_heads + h;
    if (tid < kTileTokens * 4) {
        const int t = tid >> 2, cg = tid & 3;
        if (t >= lo_tok && t < hi_tok) {
            float lo = __half2float(tile[t][cg * 32]), hi = lo;
#pragma unroll 8
            for (int k = 1; k < 32; ++k) {
                const float x = __half2float(tile[t][cg * 32 + k]);
                lo = fminf(lo, x);
                hi = fmaxf(hi, x);
            }
            const __half s16 = __float2half_rn((hi - lo) / levels);
            const int64_t o = ((unit * p.cap_tiles + dst_tile) * kTileTokens + t) * 4 + cg;
            p.scale[o] = s16;
            p.zero[o] = __float2half_rn(lo);
            sh_s[t][cg] = __half2float(s16);
            sh_z[t][cg] = lo;
        }
    }
    __syncthreads();

    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    uint32_t* dst = p.codes + (unit * p.cap_tiles + dst_tile) * kWords;
    const bool full = (lo_tok == 0 && hi_tok == kTileTokens);
    for (int wd = tid; wd < kWords; wd += 256) {
        uint32_t w = 0, mask = 0;
#pragma unroll
        for (int bit = 0; bit < 32; bit += BITS) {
            int lane, u, e;
            word_coords<BITS>(wd, bit, lane, u, e);
            const int c = u * 16 + (lane & 15);
            const int t = (lane >> 4) * 8 + e;
            if (t >= lo_tok && t < hi_tok) {
                w |= encode(__half2float(tile[t][c]), sh_z[t][c >> 5], sh_s[t][c >> 5], levels) << bit;
                mask |= (uint32_t)((1 << BITS) - 1) << bit;
            }
        }
        if (full) {
            dst[wd] = w;
        } else if (mask) {
            // a partly filled tile: keep the codes of the tokens written by earlier calls
            dst[wd] = (dst[wd] & ~mask) | w;
        }
    }
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

}  // namespace

hipError_t launch_quantize_keys(const QuantKeyParams& p, hipStream_t stream) {
    if (p.n_tiles <= 0) return hipSuccess;
    dim3 grid(p.n_tiles, p.n_kv_heads, p.batch), block(256);
    if (p.bits == 2) quantize_keys_kernel<2><<<grid, block, 0, stream>>>(p);
    else quantize_keys_kernel<4><<<grid, block, 0, stream>>>(p);
    return hipGetLastError();
}

hipError_t launch_quantize_values(const QuantValueParams& p, hipStream_t stream) {
    if (p.n_tokens <= 0) return hipSuccess;
    const int first_tile = p.first_token / kTileTokens;
    const int last_tile = (p.first_token + p.n_tokens - 1) / kTileTokens;
    dim3 grid(last_tile - first_tile + 1, p.n_kv_heads, p.batch), block(256);
    if (p.bits == 2) quantize_values_kernel<2><<<grid, block, 0, stream>>>(p);
    else quantize_values_kernel<4><<<grid, block, 0, stream>>>(p);
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
