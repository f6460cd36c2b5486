// Decode attention, matrix-core family for gfx950 (KIVI Equation 4 + Algorithm 1 Decoding).
//
// Why matrix cores for a bandwidth-bound scan: at 2 bits a cached element is 3/8 of a byte, so at
// HBM speed a compute unit sees ~28 elements per clock while its vector ALUs retire 64 lane-ops
// per clock.  Extract + convert + FMA + cross-lane reduction does not fit in ~2.3 lane-ops per
// element.  Here the vector ALUs only *extract*: a code left in place inside an fp16 lane by one
// AND is the exact subnormal fp16 number code * 4^j * 2^-24, and the v_mfma 16x16x32 f16
// instruction multiplies, accumulates in fp32 and reduces over the contraction index.  The
// position factor 4^j and the group's scale go into the small operand:
//   keys  : a_t = sum_c [code_tc 4^j] [q_c s_c 4^-j]     + sum_c q_c z_c        (per tile of 32 tokens)
//   values: o_c = sum_t [code_tc 4^j] [p_t s_t,g 4^-j]   + sum_t p_t z_t,g
// and the small operand is split into fp16 hi + (magnified) lo parts in two matrix columns, which
// restores fp32-class accuracy.  The z-term of the keys is itself a 16x16x32 product (zero-points are
// exact fp16).  The fp16 residual rows are 5x the bytes per element, so they stay on the vector
// ALUs.
//
// The token axis of every (batch, kv-head) unit is cut into chunks: all-quantised chunks of 4 * SLOTS
// tiles (SLOTS tile slots per wavefront, every 4th tile of the chunk) and chunks of up to 16 tiles
// that hold fp16 rows.  The kernel is persistent: the grid is sized to what the chip holds at once.
// All chunks lie on one cost axis (unit by unit: its fp16-row chunks, then its all-quantised
// chunks) that is cut into equal intervals, one per workgroup (4 wavefronts).  A workgroup first
// walks its fp16-row chunks (phase 1: every row load of a tile issued up front), then its
// all-quantised chunks (phase 2, software-pipelined: the next chunk's packed data is requested into
// the registers of the current chunk as soon as a slot has been consumed, so HBM requests are in
// flight all the time).  The phases are separate because the registers of an in-flight quantised
// chunk and the row registers / accumulators of phase 1 do not fit side by side.  A wavefront keeps
// a running softmax maximum and un-normalised output across the chunks of a unit (it rescales only
// when the maximum grows).  All-quantised chunks run branch-free (slots past the end of the chunk
// re-read its last tile and are masked).  When a workgroup leaves a unit it merges its four
// wavefronts in LDS; each (workgroup, phase) that touched the unit contributes one part
// (m, l, o[128]) per query head to the workspace, and the last contributor to arrive merges the
// parts (a counter in the workspace tells which).  A workgroup that owns a unit alone carries the
// unit's state from phase 1 into phase 2 and writes the output directly.
#include "kivi_internal.h"

#include <hip/hip_fp16.h>

#include <algorithm>
#include <atomic>

#ifndef KIVI_EARLY_REP
#define KIVI_EARLY_REP 2
#endif

namespace kivi {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kMaxSlots = kMfmaSplitTiles / 4;          // most tile slots per wavefront (4)
constexpr int kWaveTokens = kMaxSlots * kTileTokens;    // 128: token slots of a wavefront's LDS rows
// Floats per row of the logit / probability rows: the lanes that hold the matrix columns of one
// row-quad write 16 bytes each at the same offset of their rows, so the row stride must not be a
// multiple of 32 dwords (8-way conflicts with 4 heads per kv-head: 45.6 -> 44.1 us there).
constexpr int kLrRow = kWaveTokens + 4;
constexpr int kKRow = 136;   // halves per column of the key-side B staging (272 B: bank skew)
constexpr int kVRow = 40;    // halves per column of the value-side B staging (80 B: bank skew)
// Extra halves between the columns of consecutive channel groups: the even and the odd lanes of a
// wavefront write the operands of channel groups two apart in one instruction, and without the skew
// those land on the same banks whenever (matrix columns x kVRow / 2) is a multiple of 32 dwords
// (4 query heads per kv-head: 47.3 -> 45.5 us at the Mistral-shaped configuration).
constexpr int kVSkew = 16;
constexpr float kUnscale = 16777216.0f;                 // 2^24: codes enter as code * 2^-24
constexpr float kDownscale = 1.0f / 16777216.0f;

__device__ __forceinline__ int ring_slot(int start, int i, int cap) {
    int s = start + i;
    s -= (s >= cap) ? cap : 0;
    return s;
}

// LDS traffic between the lanes of one wavefront needs no hardware barrier and no wait: a
// wavefront's LDS instructions execute in issue order, so a read issued after a write sees it.
// This only keeps the compiler from moving memory operations across the point (a real fence
// would also make the wave wait for all its outstanding global loads).
__device__ __forceinline__ void wave_lds_sync() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load of the wavefront, i.e. for the next chunk's data requested ahead.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// data-parallel-primitive lane moves (all source lanes are valid for these patterns)
template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i within 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i within 16
constexpr int kDppRor4 = 0x124;        // rotate right by 4 within 16
constexpr int kDppRor8 = 0x128;        // rotate right by 8 within 16

__device__ __forceinline__ float readlane(float x, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

// all-lanes reductions over the 64 lanes (result uniform)
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp<kDppXor1>(v)); v = fmaxf(v, dpp<kDppXor2>(v));
    v = fmaxf(v, dpp<kDppHalfMirror>(v)); v = fmaxf(v, dpp<kDppMirror>(v));
    return fmaxf(fmaxf(readlane(v, 0), readlane(v, 16)), fmaxf(readlane(v, 32), readlane(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp<kDppXor1>(v); v += dpp<kDppXor2>(v);
    v += dpp<kDppHalfMirror>(v); v += dpp<kDppMirror>(v);
    return (readlane(v, 0) + readlane(v, 16)) + (readlane(v, 32) + readlane(v, 48));
}

// Device-scope (all compute dies) relaxed accesses: they bypass the per-die L2's write-back /
// stale-line behaviour, which is what lets workgroups exchange results without cache flushes.
__device__ __forceinline__ void device_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float device_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// fp16 x fp16 dot product of 8 elements with fp32 accumulation (v_dot2_f32_f16)
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot8(half8 a, half8 b) {
    float r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), 0.f, false);
    r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), r, false);
    r = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), r, false);
    return __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), r, false);
}

__device__ __forceinline__ float pow2_neg(int e) {   // 2^-e, 0 <= e < 64
    return __int_as_float((127 - e) << 23);
}

// 1 / (position factor) of contraction slot pair j = e >> 1 (e in [0,8)) -- see the tile layout
template <int BITS>
__device__ __forceinline__ float inv_pos_factor(int j) {
    return BITS == 2 ? pow2_neg(2 * (j & 3)) : pow2_neg(4 * (j & 1));
}

// streaming (non-temporal) load of two fp16 numbers
__device__ __forceinline__ __half2 nt_half2(const __half* p) {
    union { uint32_t u; __half2 h; } r;
    r.u = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
    return r.h;
}

// Scales (or zero-points) of the two channel groups a lane stages for the value side: lane l takes
// token l / 2 of a tile and the 32-channel blocks 2 (l % 2) and 2 (l % 2) + 1.  The array holds
// 4 >> kg entries per token (one per group of G = 32 << kg channels): with G = 32 the pair is one
// aligned 4-byte word; with G = 64 / 128 both blocks share the entry at half-word
// ((tile * 128 + 2 l) >> kg), so the aligned word that holds it is loaded and, when the data is
// consumed (nothing may touch a requested word earlier: that would wait for the load), the entry is
// copied into both halves by one byte permute with a lane-constant selector.  Only the instantiations
// for G > 32 (CS) carry this; with G = 32 it all folds away.
struct ValueScaleLane {
    int off;            // lane's part of the word offset, in halves (even)
    uint32_t sel;       // byte-permute selector: "low half twice" / "high half twice"
};
template <bool CS>
__device__ __forceinline__ ValueScaleLane value_scale_lane(int lane, int kg) {
    ValueScaleLane v;
    const int h = CS ? (2 * lane) >> kg : 2 * lane;
    v.off = CS ? h & ~1 : h;
    v.sel = (h & 1) ? 0x03020302u : 0x01000100u;
    return v;
}
template <bool CS>
__device__ __forceinline__ __half2 value_scale_word(const __half* base, int64_t tile, int kg, ValueScaleLane v) {
    return nt_half2(base + (CS ? (tile * (kTileTokens * 4)) >> kg : tile * (kTileTokens * 4)) + v.off);
}
template <bool CS>
__device__ __forceinline__ __half2 value_scale_pair(__half2 word, ValueScaleLane v) {
    if constexpr (!CS) return word;
    union { uint32_t u; __half2 h; } a, r;
    a.h = word;
    r.u = __builtin_amdgcn_perm(a.u, a.u, v.sel);
    return r.h;
}

template <int BITS>
__device__ __forceinline__ void load_tile_words(const uint32_t* tile, int lane, uint32_t* w) {
    constexpr int kPlanes = BITS / 2;
#pragma unroll
    for (int pl = 0; pl < kPlanes; ++pl) {
        typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
        const uint4v v = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(tile + pl * 256 + lane * 4));
        w[pl * 4 + 0] = v[0]; w[pl * 4 + 1] = v[1]; w[pl * 4 + 2] = v[2]; w[pl * 4 + 3] = v[3];
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

// x = hi + lo * 2^-11 with hi = fp16(x).  The remainder is stored magnified by 2^11: it stays a
// normal fp16 number wherever hi is one, and when x is so small that hi is subnormal (products
// with tiny softmax probabilities) it still adds 11 bits below fp16's subnormal spacing.
constexpr float kLoMagnify = 2048.0f, kLoShrink = 1.0f / 2048.0f;
__device__ __forceinline__ void split_hi_lo(float x, __half& hi, __half& lo) {
    hi = __float2half_rn(x);
    lo = __float2half_rn((x - __half2float(hi)) * kLoMagnify);
}
__device__ __forceinline__ float join_hi_lo(float hi, float lo) { return fmaf(lo, kLoShrink, hi); }

// LDS of one wavefront.  `lr` holds, per matrix column (head, hi/lo), the raw matrix-core logits
// of the wave's 128 token slots; after the softmax the hi column of a head holds its
// probabilities and the lo column becomes the head's output staging row.
template <int REP, int SS>
struct WaveLds {
    static constexpr int NC = 2 * REP;
    static constexpr int kStageSlots = SS;              // tile slots staged at once
    static constexpr int kKSlot = NC * kKRow;          // halves per staged key-side operand
    static constexpr int kVSlot = 4 * NC * kVRow + 3 * kVSkew;      // halves per staged value-side operand
    static constexpr int kBHalves = kStageSlots * (kKSlot > kVSlot ? kKSlot : kVSlot);
    __align__(16) float lr[NC][kLrRow];
    __align__(16) __half b[kBHalves];
    __align__(16) float zt[NC][kMaxSlots];
};

// Write the key-side small operand of one tile: columns (2hh, 2hh+1) = hi/lo of q_c s_c / posfactor.
template <int REP>
__device__ __forceinline__ void stage_key_operand(__half* bw, __half2 s2, const float (&qpf)[REP][2], int lane) {
    const float s0 = __low2float(s2), s1 = __high2float(s2);
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        __half h0, l0, h1, l1;
        split_hi_lo(qpf[hh][0] * s0, h0, l0);
        split_hi_lo(qpf[hh][1] * s1, h1, l1);
        *reinterpret_cast<__half2*>(bw + (2 * hh) * kKRow + 2 * lane) = __halves2half2(h0, h1);
        *reinterpret_cast<__half2*>(bw + (2 * hh + 1) * kKRow + 2 * lane) = __halves2half2(l0, l1);
    }
}

// Raw logits of one quantised key tile: D = codes x operand; column n of D goes to lr[n][slot*32 + token].
template <int BITS, int REP>
__device__ __forceinline__ void key_tile_mfma(const uint32_t* w, const __half* bw, float (*lr)[kLrRow],
                                              int slot, int lane) {
    constexpr int NC = 2 * REP;
    const int n = lane & 15, rq = lane >> 4, ncol = n & (NC - 1);
    float4v d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const half8 bf = *reinterpret_cast<const half8*>(bw + ncol * kKRow + ks * 32 + rq * 8);
        d0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, ks, 0), bf, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, ks, 1), bf, d1, 0, 0, 0);
    }
    // d0[j]: token rq*4 + j, d1[j]: token 16 + rq*4 + j
    if (n < NC) {
        float* dst = &lr[n][slot * kTileTokens + rq * 4];
        *reinterpret_cast<float4*>(dst) = make_float4(d0[0], d0[1], d0[2], d0[3]);
        *reinterpret_cast<float4*>(dst + 16) = make_float4(d1[0], d1[1], d1[2], d1[3]);
    }
}

// Write the value-side small operand of one tile (lane -> token lane/2, channel groups
// (lane%2)*2 + {0,1}) and accumulate the z-term  sum_t p_t z_t,g.
// MASKED: only the tile's first n_valid tokens are quantised values (a tile that also holds fp16
// rows); otherwise every token counts -- slots past the end of an all-quantised chunk need no mask,
// the softmax has set their probabilities to 0 and their (re-read) scales are finite.
template <int BITS, int REP, bool MASKED>
__device__ __forceinline__ void stage_value_operand(__half* bw, __half2 s2, __half2 z2, int n_valid,
                                                    const float (*lr)[kLrRow], int slot,
                                                    float (&zacc)[REP][2], int lane) {
    constexpr int NC = 2 * REP;
    const int t = lane >> 1, cg0 = (lane & 1) * 2;
    const bool valid = !MASKED || t < n_valid;
    const float pf = inv_pos_factor<BITS>((t >> 1) & 3);
    const float s0 = valid ? __low2float(s2) * pf : 0.f, s1 = valid ? __high2float(s2) * pf : 0.f;
    const float z0 = valid ? __low2float(z2) : 0.f, z1 = valid ? __high2float(z2) : 0.f;
#pragma unroll
    for (int hh = 0; hh < REP; ++hh) {
        const float pt = valid ? lr[2 * hh][slot * kTileTokens + t] : 0.f;
        __half h0, l0, h1, l1;
        split_hi_lo(pt * s0, h0, l0);
        split_hi_lo(pt * s1, h1, l1);
        bw[((cg0 + 0) * NC + 2 * hh) * kVRow + (cg0 + 0) * kVSkew + t] = h0;
        bw[((cg0 + 0) * NC + 2 * hh + 1) * kVRow + (cg0 + 0) * kVSkew + t] = l0;
        bw[((cg0 + 1) * NC + 2 * hh) * kVRow + (cg0 + 1) * kVSkew + t] = h1;
        bw[((cg0 + 1) * NC + 2 * hh + 1) * kVRow + (cg0 + 1) * kVSkew + t] = l1;
        zacc[hh][0] = fmaf(pt, z0, zacc[hh][0]);
        zacc[hh][1] = fmaf(pt, z1, zacc[hh][1]);
    }
}

template <int BITS, int REP>
__device__ __forceinline__ void value_tile_mfma(const uint32_t* w, const __half* bw, float4v (&acc)[8], int lane) {
    constexpr int NC = 2 * REP;
    const int n = lane & 15, rq = lane >> 4, ncol = n & (NC - 1);
    half8 bf[4];
#pragma unroll
    for (int cg = 0; cg < 4; ++cg)
        bf[cg] = *reinterpret_cast<const half8*>(bw + (cg * NC + ncol) * kVRow + cg * kVSkew + rq * 8);
#pragma unroll
    for (int u = 0; u < 8; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_fragment<BITS>(w, u >> 1, u & 1), bf[u >> 1],
                                                        acc[u], 0, 0, 0);
}

// SLOTS: tile slots per wavefront of an all-quantised chunk (chunk = 4 * SLOTS tiles); OCC: workgroups
// per compute unit the register budget is sized for.
// MODE: kBothPhases = the whole attention in one launch.  When a workgroup would own several units
// the fp16 rows are served by a launch of their own (residual_rows_kernel: one wavefront per tile,
// many wavefronts per compute unit, one part per tile in the workspace) and this kernel follows as
// kQuantisedOnly: the all-quantised chunks only; whoever finishes a unit merges the parts of the
// first launch into it.
// kQuantisedRagged: kQuantisedOnly over a batch whose sequences differ in length (every unit's own
// number of all-quantised tiles from p.seq_state); an instantiation of its own so that batches of
// one length pay nothing for it.
constexpr int kBothPhases = 0, kQuantisedOnly = 1, kQuantisedRagged = 2;
constexpr int kRuntimeHeadGroups = 15;      // value of HSHIFT: the number of head runs per kv-head is a launch parameter

template <int BITS, int REP, int SLOTS, int OCC, int MODE, int HSHIFT = 0, bool CS = false>
__global__ __launch_bounds__(256, OCC) void decode_mfma_kernel(DecodeParams p) {
    constexpr bool kQOnly = MODE != kBothPhases, kRagged = MODE == kQuantisedRagged;
    constexpr int kSlots = SLOTS;
    // tile slots staged at once: two where that divides the slots and the registers allow
    constexpr int kStage = REP > 2 ? 1 : (SLOTS % 2 == 0 ? 2 : SLOTS);
    using WL = WaveLds<REP, kStage>;
    constexpr int NC = 2 * REP;                       // live matrix columns: (head, hi/lo)
    constexpr int SS = WL::kStageSlots;
    // fp16-row chunks: rows held in registers at once, and whether the first tile's value rows are
    // requested ahead of the logits (both cut for the wider instantiations: register pressure)
    constexpr int RB = (OCC >= 3 || REP > 4) ? 4 : 8;
    constexpr bool kPreloadV = OCC < 3 && REP <= 4;
    __shared__ __align__(16) float sm_q[REP][kHeadDim];               // scale * q
    __shared__ __align__(16) __half sm_qf[NC][kKRow];                 // its hi/lo columns (z-term operand)
    __shared__ WL sm_w[4];
    __shared__ __align__(16) float sm_r[4][REP][kHeadDim];            // vector-ALU (fp16 residual) outputs
    __shared__ float sm_zs[4][REP][4];                                // value z-term sums per channel group
    __shared__ float sm_ml[4][REP][2];
    __shared__ int sm_last;
    // Parts that never leave the workgroup: when this workgroup is the only contributor to a unit in
    // both phases, the unit's phase-1 result waits here for phase 2 instead of going through the
    // workspace (no device-scope traffic, no counter).
    constexpr int kHold = REP <= 2 ? 8 : (REP == 4 ? 4 : 0);
    __shared__ float sm_hold_o[kHold * REP * kHeadDim + 1];
    __shared__ float sm_hold_ml[kHold * REP * 2 + 1];
    __shared__ int sm_hold_unit[kHold + 1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps tile arithmetic scalar
    const int n = lane & 15, rq = lane >> 4;          // matrix column / row-quad (= k-quad for operands)
    const int ncol = n & (NC - 1);
    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    constexpr int kLaneWords = BITS * 2;
    WL& wl = sm_w[wave];
    // CS: scales and zero-points stored once per group of G = 32 << kg tokens (keys) / channels (values), G > 32
    const int kg = CS ? p.kg_shift : 0;
    const ValueScaleLane vlane = CS ? value_scale_lane<CS>(lane, kg) : ValueScaleLane{0, 0u};

    // REP is the instantiation's head count; the layout may have fewer query heads per kv-head
    // (3, 5, 6, 7): the surplus heads run on a zero query and are never stored
    const int rep = p.rep_here, rep_total = p.n_q_heads / p.n_kv_heads;
    // HSHIFT > 0: a unit of the work axis is (batch, kv-head, one of 2^HSHIFT equal parts of the
    // kv-head's query heads) -- unit u reads the cache of (batch, kv-head) u >> HSHIFT and serves the
    // query heads (u & (2^HSHIFT - 1)) * rep .. + rep of its group; parts, counters and held results go by u.
    // HSHIFT == kRuntimeHeadGroups: groups wider than REP heads (multi-query attention) in ONE launch --
    // a unit is (batch, kv-head, one of p.head_groups runs of REP consecutive query heads; the last run
    // may be shorter): every run reads the same cache, which the chip's caches serve after the first.
    constexpr bool kRunGroups = HSHIFT == kRuntimeHeadGroups;
    constexpr int kPartMask = kRunGroups ? 0 : (1 << HSHIFT) - 1;
    const int n_groups = kRunGroups ? p.head_groups : 1;
    auto kv_unit = [&](int u) -> int { return kRunGroups ? u / n_groups : u >> HSHIFT; };
    auto part_of = [&](int u) -> int { return kRunGroups ? u - (u / n_groups) * n_groups : u & kPartMask; };
    auto first_q_head = [&](int u) -> int {
        return (kv_unit(u) % p.n_kv_heads) * rep_total + p.q_head0 + part_of(u) * (kRunGroups ? REP : rep);
    };
    // live query heads of unit u on this instantiation
    auto rep_of = [&](int u) -> int { return kRunGroups ? min(REP, rep_total - part_of(u) * REP) : rep; };
    auto batch_of = [&](int u) -> int { return kv_unit(u) / p.n_kv_heads; };
    // chunks per unit on this launch's cost axis: all-quantised / with fp16 rows
    const int n_a = p.plan.n_splits_a, n_b = kQOnly ? 0 : p.plan.n_splits_b;
    const int cpu = p.plan.n_splits_a + p.plan.n_splits_b;       // workspace rows per (batch, query head)
    // this workgroup's ranges in the two global chunk index spaces (unit-major)
    // Index arithmetic on the cost axis; 32-bit whenever the products fit (64-bit division costs
    // more than a hundred instructions each and every workgroup does about a dozen).
    const int n_wgs = gridDim.x, cost_unit = p.cost_unit, cost_b = p.cost_b;
    const bool small_axis = (p.total_cost + 1) * n_wgs < 0x7fffffffLL;
    auto wg_start = [&](int g) -> int64_t {                // first cost position of workgroup g
        return small_axis ? (int64_t)((uint32_t)g * (uint32_t)p.total_cost / (uint32_t)n_wgs)
                          : (int64_t)g * p.total_cost / n_wgs;
    };
    auto owner = [&](int64_t pos) -> int {                 // workgroup whose cost interval holds `pos`
        return small_axis ? (int)((((uint32_t)pos + 1u) * (uint32_t)n_wgs - 1u) / (uint32_t)p.total_cost)
                          : (int)(((pos + 1) * n_wgs - 1) / p.total_cost);
    };
    auto chunks_before = [&](int64_t pos, int& nb, int& na) {   // chunks of either kind that start before `pos`
        const int u = small_axis ? (int)((uint32_t)pos / (uint32_t)cost_unit) : (int)(pos / cost_unit);
        const int r = (int)(pos - (int64_t)u * cost_unit);
        nb = u * n_b + min(n_b, (r + cost_b - 1) / cost_b);
        na = u * n_a + min(max(r - n_b * cost_b, 0), n_a);
    };
    int first_a, last_a, first_b, last_b;
    chunks_before(wg_start(blockIdx.x), first_b, first_a);
    chunks_before(wg_start(blockIdx.x + 1), last_b, last_a);

    // registers holding the packed data of one all-quantised chunk (4 slots of this wavefront)
    uint32_t kw[kSlots][kLaneWords], vw[kSlots][kLaneWords];
    __half2 ks2[kSlots], vs2[kSlots], vz2[kSlots];
    half8 zf[4];

    // The all-quantised chunk whose data is being requested ("next"): unit, chunk index inside the
    // unit, and derived tile range.  Advanced without divisions.
    // Inside a unit the workgroup's chunks are visited in rotated order, starting at a chunk that
    // depends on the unit (attention does not care about the order): the workgroups, which run in
    // lockstep, then read different relative offsets of their units at any one time instead of all
    // the same one, which keeps their requests from meeting on the same HBM channels whatever the
    // per-unit stride is.
    int nx_u = 0, nx_j = 0, nx_nt = 1;
    int nx_lo = 0, nx_len = 1, nx_rot = 0;     // this workgroup's chunk range in unit nx_u, rotation
    int nx_tiles_a = p.plan.tiles_a;           // all-quantised tiles of unit nx_u
    bool nx_ok = false;
    int64_t nx_base = 0;
    auto set_next = [&](int ck, bool first_call) {
        nx_ok = ck < last_a;
        bool new_unit = first_call;
        if (first_call) {
            nx_u = n_a ? ck / n_a : 0;
            nx_j = ck - nx_u * n_a;
        } else if (++nx_j == n_a) {
            nx_j = 0;
            ++nx_u;
            new_unit = true;
        }
        if (new_unit) {
            nx_lo = max(first_a - nx_u * n_a, 0);
            nx_len = max(min(last_a - nx_u * n_a, n_a) - nx_lo, 1);
            nx_rot = (nx_u * 3) % nx_len;
            if constexpr (kRagged) {
                // a batch of different lengths: the unit's own number of all-quantised tiles (the plan
                // holds the longest sequence's; a shorter one's surplus chunks come out empty)
                nx_tiles_a = nx_ok ? p.seq_state[4 * batch_of(nx_u)] / kTileTokens : p.plan.tiles_a;
            }
        }
        int j_phys = nx_j + nx_rot;                          // nx_j runs over [nx_lo, nx_lo + nx_len)
        j_phys -= j_phys >= nx_lo + nx_len ? nx_len : 0;
        const int tile0 = j_phys * p.plan.tiles_per_split_a;
        nx_nt = min(p.plan.tiles_per_split_a, nx_tiles_a - tile0);
        nx_base = (int64_t)kv_unit(nx_u) * p.cap_tiles + tile0;
        if constexpr (kRagged) {
            if (nx_nt <= 0) nx_base -= tile0;                // an empty chunk: its (masked) slots re-read the unit's tile 0
        }
    };
    auto chunk_tile = [&](int slot_or_row) -> int64_t {
        const int t = min(wave + 4 * slot_or_row, nx_nt - 1);
        return nx_base + (kRagged ? max(t, 0) : t);
    };
    // row of the key scale / zero-point arrays (one per group of G = 32 << kg tokens) of that tile:
    // the chunk's first tile is a multiple of G / 32, so base and offset can be shifted apart (the
    // offset may differ from lane to lane: a 32-bit shift instead of a 64-bit one)
    auto chunk_key_row = [&](int slot_or_row) -> int64_t {
        const int t = min(wave + 4 * slot_or_row, nx_nt - 1);
        return (nx_base >> kg) + ((kRagged ? max(t, 0) : t) >> kg);
    };
    // Requests for the "next" all-quantised chunk.  They are issued unconditionally so that the
    // compiler can count outstanding loads exactly (a conditional load forces a wait for *all*
    // outstanding loads at the next use); when there is no next chunk they read tile 0 of unit 0,
    // which stays in L2, and the result is never used.
    auto request_zero_rows = [&]() {
        int64_t row;                                                         // A row n = slot n
        if constexpr (CS) row = nx_ok ? chunk_key_row(min(n, kSlots - 1)) : 0;
        else row = nx_ok ? chunk_tile(min(n, kSlots - 1)) : 0;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            zf[ks] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(p.k_zero + row * kHeadDim + ks * 32 + rq * 8));
    };
    auto request_key_slot = [&](int i) {
        const int64_t tile = nx_ok ? chunk_tile(i) : 0;
        load_tile_words<BITS>(p.k_codes + tile * kWords, lane, kw[i]);
        if constexpr (CS) ks2[i] = nt_half2(p.k_scale + (nx_ok ? chunk_key_row(i) : 0) * kHeadDim + 2 * lane);
        else ks2[i] = nt_half2(p.k_scale + tile * kHeadDim + 2 * lane);
    };
    auto request_value_slot = [&](int i) {
        const int64_t tile = nx_ok ? chunk_tile(i) : 0;
        load_tile_words<BITS>(p.v_codes + tile * kWords, lane, vw[i]);
        if constexpr (CS) {
            vs2[i] = value_scale_word<CS>(p.v_scale, tile, kg, vlane);
            vz2[i] = value_scale_word<CS>(p.v_zero, tile, kg, vlane);
        } else {
            vs2[i] = nt_half2(p.v_scale + tile * kTileTokens * 4 + 2 * lane);
            vz2[i] = nt_half2(p.v_zero + tile * kTileTokens * 4 + 2 * lane);
        }
    };

    // per-wave running state of the current unit
    float4v acc[8];
    float zacc[REP][2], m_run[REP], l_lane[REP], qpf[REP][2];
    auto reset_state = [&]() {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            zacc[hh][0] = zacc[hh][1] = 0.f;
            m_run[hh] = -INFINITY;
            l_lane[hh] = 0.f;
        }
        // fp16-residual (vector-ALU) outputs of the unit accumulate in this wavefront's LDS rows
        for (int i = lane; i < REP * kHeadDim; i += 64) (&sm_r[wave][0][0])[i] = 0.f;
    };

    // workgroups whose all-quantised range / fp16-row range touches unit u: first index and count
    auto contributors = [&](int u, int& ga0, int& len_a, int& gb0, int& len_b) {
        const int64_t base = (int64_t)u * cost_unit, a0 = base + n_b * cost_b;
        gb0 = n_b ? owner(base) : 0;
        len_b = n_b ? owner(base + (n_b - 1) * cost_b) - gb0 + 1 : 0;
        ga0 = n_a ? owner(a0) : 0;
        len_a = n_a ? owner(a0 + n_a - 1) - ga0 + 1 : 0;
        if (kQOnly) {       // the parts the fp16-row launch left for the unit: one per tile
            gb0 = 0;
            len_b = p.plan.n_splits_b;
        }
    };

    // kQuantisedOnly: part 0 of the current unit (what the fp16-row launch left), requested when the
    // unit is entered so that it has arrived long before the unit is left (with eight heads, for want
    // of registers, only when the unit is left); thread tid holds the values of its elements
    // idx = tid + 256 k of finish_unit's loop.
    constexpr int kIdx = (REP * kHeadDim + 255) / 256;
    constexpr bool kPrefetchPart = REP <= 4;
    // kQuantisedOnly also requests the next unit's query one unit ahead and separates the units with
    // LDS-only barriers: the next chunk's data, in flight when a unit is left, then keeps travelling
    // while the workgroup merges, writes the output and stages the next query.  (kBothPhases keeps
    // __syncthreads(): its launches have one unit per workgroup where this would matter.)
    auto unit_barrier = [&]() {
        if constexpr (kQOnly) lds_barrier();
        else __syncthreads();
    };
    __half q_pre[kIdx];
    auto request_q = [&](int u) {
        const int hq0 = first_q_head(u);
        const int b = batch_of(u);
#pragma unroll
        for (int k = 0; k < kIdx; ++k) {
            const int idx = min(tid + 256 * k, rep_of(u) * kHeadDim - 1);  // unconditional loads (clamped)
            q_pre[k] = p.q[((int64_t)b * p.n_q_heads + hq0 + idx / kHeadDim) * kHeadDim + idx % kHeadDim];
        }
    };
    float pre_m[kIdx], pre_l[kIdx], pre_o[kIdx];
    auto request_rows_part = [&](int u) {
        const int hq0 = first_q_head(u);
        const int b = batch_of(u);
#pragma unroll
        for (int k = 0; k < kIdx; ++k) {
            const int idx = min(tid + 256 * k, rep_of(u) * kHeadDim - 1);  // unconditional loads (clamped)
            const int64_t row = ((int64_t)b * p.n_q_heads + hq0 + idx / kHeadDim) * cpu;
            pre_m[k] = p.part_ml[row * 2 + 0];
            pre_l[k] = p.part_ml[row * 2 + 1];
            pre_o[k] = p.part_o[row * kHeadDim + idx % kHeadDim];
        }
    };

    // ---- leave a unit: merge the four wavefronts, write the output or this workgroup's part ----
    // sole: single part, output written directly; hold_put >= 0: the part is parked in that LDS slot;
    // hold_get >= 0: the part parked in that slot is merged in and the output written directly.
    auto finish_unit = [&](int u, bool fp16_phase, bool sole, int hold_put, int hold_get) __attribute__((always_inline)) {
        const int hq0 = first_q_head(u);
        const int b = batch_of(u);
        // raw matrix-core outputs: column n of acc[u8] -> lr[n][channel]
        if (n < NC) {
#pragma unroll
            for (int u8 = 0; u8 < 8; ++u8)
                *reinterpret_cast<float4*>(&wl.lr[n][u8 * 16 + rq * 4]) =
                    make_float4(acc[u8][0], acc[u8][1], acc[u8][2], acc[u8][3]);
        }
        // z-term sums over tokens: lanes of equal parity hold the same channel-group pair, so
        // reduce with parity-preserving moves (xor 2, rotate by 4 and 8 inside a row, then rows)
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float zz = zacc[hh][k];
                zz += dpp<kDppXor2>(zz); zz += dpp<kDppRor4>(zz); zz += dpp<kDppRor8>(zz);
                zz += __shfl_xor(zz, 16); zz += __shfl_xor(zz, 32);
                if (lane < 2) sm_zs[wave][hh][lane * 2 + k] = zz;      // lane 0: groups 0,1; lane 1: groups 2,3
            }
            const float l_w = wave_sum(l_lane[hh]);
            if (lane == 0) { sm_ml[wave][hh][0] = m_run[hh]; sm_ml[wave][hh][1] = l_w; }
        }
        unit_barrier();

        // Parts of unit u: one per workgroup whose fp16-row range touches it (these come first), then
        // one per workgroup whose all-quantised range touches it.
        // (`sole`: this workgroup carried the unit's state from phase 1 into phase 2 and nobody
        // else touches the unit -- a single part.)
        const int g = blockIdx.x;
        int ga0, len_a, gb0, len_b;
        contributors(u, ga0, len_a, gb0, len_b);
        // kQuantisedOnly: the only workgroup of a unit's all-quantised range merges the first launch's
        // parts into its own and writes the output; otherwise the counter runs over the workgroups of
        // this launch and the last one merges all parts.
        const bool merge_rows_parts = kQOnly && len_a == 1 && len_b > 0;
        const int n_parts = (sole || hold_put >= 0 || hold_get >= 0 || merge_rows_parts) ? 1 : len_a + len_b;
        const int n_counted = kQOnly ? len_a : n_parts;
        const int part = fp16_phase ? g - gb0 : len_b + g - ga0;
        const int row_stride = cpu;                               // workspace rows per (batch, query head)
        // one output element (query head hh, channel c); p0_*: part 0 of the fp16-row launch (kQuantisedOnly)
        auto finish_element = [&](int idx, float p0_m, float p0_l, float p0_o) __attribute__((always_inline)) {
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
                    const float ow = fmaf(join_hi_lo(sm_w[wv].lr[2 * hh][c], sm_w[wv].lr[2 * hh + 1][c]), kUnscale,
                                          sm_zs[wv][hh][c >> 5]) + sm_r[wv][hh][c];
                    l = fmaf(sm_ml[wv][hh][1], wgt, l);
                    o = fmaf(ow, wgt, o);
                }
            }
            const int64_t row = (int64_t)b * p.n_q_heads + hq0 + hh;
            if (hold_put >= 0) {
                sm_hold_o[(hold_put * REP + hh) * kHeadDim + c] = o;
                if (c == 0) {
                    sm_hold_ml[(hold_put * REP + hh) * 2 + 0] = m;
                    sm_hold_ml[(hold_put * REP + hh) * 2 + 1] = l;
                }
            } else if (hold_get >= 0) {
                const float mh = sm_hold_ml[(hold_get * REP + hh) * 2 + 0], lh = sm_hold_ml[(hold_get * REP + hh) * 2 + 1];
                const float oh = sm_hold_o[(hold_get * REP + hh) * kHeadDim + c];
                const float mn = fmaxf(m, mh);                        // at least one of the two is finite
                const float f_own = __expf(m - mn), f_held = __expf(mh - mn);
                p.out[row * kHeadDim + c] = fmaf(o, f_own, oh * f_held) / fmaf(l, f_own, lh * f_held);
            } else if (merge_rows_parts) {
                // plain loads: the parts were written by the previous launch
                // (part 0 was requested when the unit was entered; any further ones eight at a time,
                // all loads of a batch issued before the first is used)
                float mm = m, ll = l, oo = o;
                if (p0_m > -INFINITY) {
                    const float mn = fmaxf(mm, p0_m);
                    const float f_old = __expf(mm - mn), f_new = __expf(p0_m - mn);
                    ll = fmaf(ll, f_old, p0_l * f_new);
                    oo = fmaf(oo, f_old, p0_o * f_new);
                    mm = mn;
                }
                const float* ml = p.part_ml + (row * row_stride + 1) * 2;
                const float* po = p.part_o + (row * row_stride + 1) * kHeadDim + c;
                for (int i0 = 0; i0 < len_b - 1; i0 += 8) {
                    float mv[8], lv[8], ov[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int i = min(i0 + j, len_b - 2);
                        mv[j] = ml[2 * i];
                        lv[j] = ml[2 * i + 1];
                        ov[j] = po[(int64_t)i * kHeadDim];
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (i0 + j < len_b - 1 && mv[j] > -INFINITY) {
                            const float mn = fmaxf(mm, mv[j]);
                            const float f_old = __expf(mm - mn), f_new = __expf(mv[j] - mn);
                            ll = fmaf(ll, f_old, lv[j] * f_new);
                            oo = fmaf(oo, f_old, ov[j] * f_new);
                            mm = mn;
                        }
                    }
                }
                p.out[row * kHeadDim + c] = oo / ll;
            } else if (n_parts == 1) {
                p.out[row * kHeadDim + c] = o / l;
            } else {
                // device-scope stores: they go through to memory, no cache flush is needed to publish them
                device_store(p.part_o + (row * row_stride + part) * kHeadDim + c, o);
                if (c == 0) {
                    device_store(p.part_ml + (row * row_stride + part) * 2 + 0, m);
                    device_store(p.part_ml + (row * row_stride + part) * 2 + 1, l);
                }
            }
        };
        if constexpr (kQOnly && kPrefetchPart) {
#pragma unroll
            for (int k = 0; k < kIdx; ++k)
                if (tid + 256 * k < rep_of(u) * kHeadDim) finish_element(tid + 256 * k, pre_m[k], pre_l[k], pre_o[k]);
        } else {
            for (int idx = tid; idx < rep_of(u) * kHeadDim; idx += 256) {
                float p0_m = -INFINITY, p0_l = 0.f, p0_o = 0.f;
                if (merge_rows_parts) {
                    const int64_t row = ((int64_t)b * p.n_q_heads + hq0 + idx / kHeadDim) * cpu;
                    p0_m = p.part_ml[row * 2 + 0];
                    p0_l = p.part_ml[row * 2 + 1];
                    p0_o = p.part_o[row * kHeadDim + idx % kHeadDim];
                }
                finish_element(idx, p0_m, p0_l, p0_o);
            }
        }
        if (n_parts > 1) {
            // The last workgroup to finish this unit merges the parts.  How the parts are published:
            // they are written with device-scope atomic stores, which go through to memory instead
            // of staying dirty in the die's L2.  Every thread then waits until its own stores have
            // been acknowledged (vmcnt(0): on this target stores count on the same counter as
            // loads) -- this is the wait a device-scope release fence consists of, without the
            // write-back of the whole L2 that such a fence adds for data written with plain stores,
            // of which there is none here (measured with the full fences: config 4 84.8 -> 234.9 us,
            // config 5 46.5 -> 58.7 us).  After the barrier every part store of the workgroup is
            // therefore visible device-wide, and only then is the unit's counter incremented.
            // Whoever reads the final count does so after all contributors' stores were
            // acknowledged; its part loads are device-scope atomic loads issued after the barrier
            // that follows, and such loads are served from memory, not from a possibly stale L2
            // line, so no invalidation (the other half of an acquire fence) is needed either.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0) {
                const int done = __hip_atomic_fetch_add(p.counters + u, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sm_last = (done == n_counted - 1);
            }
            __syncthreads();
            if (sm_last) {
                for (int idx = tid; idx < rep_of(u) * kHeadDim; idx += 256) {
                    const int hh = idx / kHeadDim, c = idx % kHeadDim;
                    const int64_t row = (int64_t)b * p.n_q_heads + hq0 + hh;
                    const float* ml = p.part_ml + row * row_stride * 2;
                    const float* po = p.part_o + row * row_stride * kHeadDim;
                    // one pass, eight parts at a time: the device-scope loads of a batch are all
                    // issued before the first is used (each is a trip to memory, not to a cache)
                    float m = -INFINITY, l = 0.f, o = 0.f;
                    for (int i0 = 0; i0 < n_parts; i0 += 8) {
                        float mv[8], lv[8], ov[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int i = min(i0 + j, n_parts - 1);
                            mv[j] = device_load(ml + 2 * i);
                            lv[j] = device_load(ml + 2 * i + 1);
                            ov[j] = device_load(po + (int64_t)i * kHeadDim + c);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            if (i0 + j < n_parts && mv[j] > -INFINITY) {
                                const float mn = fmaxf(m, mv[j]);
                                const float f_old = __expf(m - mn), f_new = __expf(mv[j] - mn);   // m = -inf: f_old = 0
                                l = fmaf(l, f_old, lv[j] * f_new);
                                o = fmaf(o, f_old, ov[j] * f_new);
                                m = mn;
                            }
                        }
                    }
                    p.out[row * kHeadDim + c] = o / l;
                }
                if (tid == 0) __hip_atomic_store(p.counters + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        unit_barrier();           // LDS is reused by the next unit
    };

    // ---- enter a unit: query operands ----
    auto enter_unit = [&](int u) {
        const int hq0 = first_q_head(u);
        const int b = batch_of(u);
        auto stage = [&](int i, float x) {
            const int hh = i / kHeadDim, c = i % kHeadDim;
            __half hi, lo;
            split_hi_lo(x, hi, lo);
            sm_q[hh][c] = x;
            sm_qf[2 * hh][c] = hi;
            sm_qf[2 * hh + 1][c] = lo;
        };
        if constexpr (kQOnly) {
#pragma unroll
            for (int k = 0; k < kIdx; ++k) {           // the query was requested one unit ahead
                const int i = tid + 256 * k;
                if (i < REP * kHeadDim) stage(i, i / kHeadDim < rep_of(u) ? p.softmax_scale * __half2float(q_pre[k]) : 0.f);
            }
        } else {
            for (int i = tid; i < REP * kHeadDim; i += 256) {
                const int hh = i / kHeadDim, c = i % kHeadDim;
                stage(i, hh < rep_of(u) ? p.softmax_scale * __half2float(p.q[((int64_t)b * p.n_q_heads + hq0 + hh) * kHeadDim + c]) : 0.f);
            }
        }
        unit_barrier();
        // per-lane key-side query factors: channels 2*lane, 2*lane+1 times 1/position factor
        const float pf = inv_pos_factor<BITS>(lane & 3);
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            qpf[hh][0] = sm_q[hh][2 * lane] * pf;
            qpf[hh][1] = sm_q[hh][2 * lane + 1] * pf;
        }
        reset_state();
    };

    // Probabilities of the wave's 128 token slots against the running maximum (2 slots per lane);
    // rescales the running state when the maximum grows.
    auto softmax_step = [&](int cnt) {
        {
            const int slot = lane >> 4;
            const bool live = slot < cnt;
            float a0[REP], a1[REP], scale_lane = 1.f;
            bool any_rescale = false;
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                const float2 hi = *reinterpret_cast<const float2*>(&wl.lr[2 * hh][2 * lane]);
                const float2 lo = *reinterpret_cast<const float2*>(&wl.lr[2 * hh + 1][2 * lane]);
                const float zt = join_hi_lo(wl.zt[2 * hh][slot], wl.zt[2 * hh + 1][slot]);
                a0[hh] = live ? fmaf(join_hi_lo(hi.x, lo.x), kUnscale, zt) : -INFINITY;
                a1[hh] = live ? fmaf(join_hi_lo(hi.y, lo.y), kUnscale, zt) : -INFINITY;
                const float mx = wave_max(fmaxf(a0[hh], a1[hh]));
                if (mx > m_run[hh]) {                       // wave-uniform: the running maximum grows
                    const float f = __expf(m_run[hh] - mx); // 0 on the first chunk (m_run = -inf)
                    l_lane[hh] *= f;
                    zacc[hh][0] *= f; zacc[hh][1] *= f;
                    sm_r[wave][hh][lane] *= f; sm_r[wave][hh][lane + 64] *= f;
                    if ((n >> 1) == hh) scale_lane = f;
                    any_rescale = true;
                    m_run[hh] = mx;
                }
            }
            if (any_rescale) {
#pragma unroll
                for (int u8 = 0; u8 < 8; ++u8)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[u8][j] *= scale_lane;
            }
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                const float ms = m_run[hh] == -INFINITY ? 0.f : m_run[hh];
                const float p0 = __expf(a0[hh] - ms), p1 = __expf(a1[hh] - ms);
                *reinterpret_cast<float2*>(&wl.lr[2 * hh][2 * lane]) = make_float2(p0, p1);
                l_lane[hh] += p0 + p1;
            }
        }
        wave_lds_sync();

    };

    // ================= phase 1: this workgroup's chunks that hold fp16 rows =================
    // They run before any all-quantised data is requested: the row loads, the vector-ALU
    // accumulators and the registers of an in-flight quantised chunk do not fit side by side.
    // Every unit touched here gets a part of its own (merged with the other parts of the unit by
    // whichever workgroup finishes the unit last).
    // The first all-quantised chunk's key-side data is requested before the fp16-row phase where the
    // registers allow it (one or two query heads per kv-head): it then travels while that phase
    // runs; the value-side data follows when the phase has freed its row registers.
    constexpr bool kEarlyKeys = MODE == kBothPhases && REP <= KIVI_EARLY_REP;
    auto initial_request_keys = [&]() {
        if (first_a < last_a) {
            set_next(first_a, true);
            request_zero_rows();
#pragma unroll
            for (int i = 0; i < kSlots; ++i) request_key_slot(i);
        }
    };
    auto initial_request_values = [&]() {
        if (first_a < last_a) {
#pragma unroll
            for (int i = 0; i < kSlots; ++i) request_value_slot(i);
        }
    };
    if constexpr (kEarlyKeys) initial_request_keys();
    // A unit's phase-1 part is parked in LDS if this workgroup is the unit's only contributor in both
    // phases and a slot is free; phase 2 meets the parked units in the same order.
    int n_held = 0, n_popped = 0;
    auto finish_fp16_unit = [&](int u) __attribute__((always_inline)) {
        int ga0, len_a, gb0, len_b;
        contributors(u, ga0, len_a, gb0, len_b);
        const bool park = n_held < kHold && len_a == 1 && len_b == 1 && ga0 == (int)blockIdx.x && gb0 == (int)blockIdx.x;
        if (park && tid == 0) sm_hold_unit[n_held] = u;
        finish_unit(u, true, false, park ? n_held : -1, -1);
        n_held += park ? 1 : 0;
    };
    const int ub_lo = first_b < last_b ? first_b / max(n_b, 1) : 0;
    const int ub_hi = first_b < last_b ? (last_b - 1) / max(n_b, 1) : -1;
    if constexpr (!kQOnly) {
    for (int u = ub_lo; u <= ub_hi; ++u) {
        const int b_lo = max(first_b, u * n_b), b_hi = min(last_b, (u + 1) * n_b);
        if (u > ub_lo) finish_fp16_unit(u - 1);
        enter_unit(u);

        // ---------- chunks that hold fp16 rows ----------
        for (int ck = b_lo; ck < b_hi; ++ck) {
            const int tile0 = p.plan.tiles_a + (ck - u * n_b) * p.plan.tiles_per_split_b;
            const int n_tiles = min(p.plan.tiles_per_split_b, p.plan.tiles_total - tile0);
            const int64_t unit = kv_unit(u);
            const bool fused_append = p.k_new != nullptr;
            const int cnt = n_tiles > wave ? (n_tiles - wave + 3) / 4 : 0;
            const int64_t ubase = unit * p.cap_tiles + tile0;
            if (lane < NC * kMaxSlots) (&wl.zt[0][0])[lane] = 0.f;
            // how many of the wave's tiles are quantised key tiles (they come first in token order)
            int cnt_kq = 0;
            for (int i = 0; i < cnt; ++i) cnt_kq += ((tile0 + wave + 4 * i) * kTileTokens < p.n_kq) ? 1 : 0;
            if (cnt_kq > 0) {
                const __half* zrow = p.k_zero + ((ubase + wave + 4 * min(n, cnt_kq - 1)) >> kg) * kHeadDim;
                float4v d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const half8 za = *reinterpret_cast<const half8*>(zrow + ks * 32 + rq * 8);
                    const half8 bq = *reinterpret_cast<const half8*>(&sm_qf[ncol][ks * 32 + rq * 8]);
                    d = __builtin_amdgcn_mfma_f32_16x16x32_f16(za, bq, d, 0, 0, 0);
                }
                wave_lds_sync();
                if (n < NC && rq == 0) *reinterpret_cast<float4*>(&wl.zt[n][0]) = make_float4(d[0], d[1], d[2], d[3]);
            }
            // fp16 value rows of the wave's first tile are requested now, ahead of the logits
            // lane (seg, row): row j*4 + (lane >> 4) of the tile, channels (lane & 15)*8 ..; clamped rows are not used
            auto load_value_row = [&](int tt, int j) -> half8 {
                const int t = min(max(tt + j * 4 + (lane >> 4), p.n_vq), p.length - 1);
                const int slot = ring_slot(p.v_r_start, t - p.n_vq, p.cap_r);
                const __half* src = p.v_resid + (unit * p.cap_r + slot) * kHeadDim;
                if (fused_append && t == p.length - 1) src = p.v_new + unit * kHeadDim;   // not in the ring yet
                return *reinterpret_cast<const half8*>(src + (lane & 15) * 8);
            };
            // Fused append: the wavefront that owns the tile of the newest token also stores that
            // token's rows in the residual rings (lanes 0-15 the key row, 16-31 the value row).
            // Nobody reads those slots in this launch -- every reader of token length-1 takes it from
            // k_new / v_new -- and the row is requested here, long before it is stored.
            bool owns_new = false;
            uint4 new_row = {0u, 0u, 0u, 0u};
            __half* new_dst = nullptr;
            if (fused_append) {
                const int last = p.length - 1, last_tile = last / kTileTokens;
                owns_new = last_tile >= tile0 && last_tile < tile0 + n_tiles && ((last_tile - tile0) & 3) == wave && lane < 32 &&
                           part_of(u) == 0;           // the parts of a kv-head's group would all store the same rows
                if (owns_new) {
                    const bool is_v = lane >= 16;
                    const int slot = is_v ? ring_slot(p.v_r_start, last - p.n_vq, p.cap_r)
                                          : ring_slot(p.k_r_start, last - p.n_kq, p.cap_r);
                    new_row = *reinterpret_cast<const uint4*>((is_v ? p.v_new : p.k_new) + unit * kHeadDim + (lane & 15) * 8);
                    new_dst = const_cast<__half*>(is_v ? p.v_resid : p.k_resid) + (unit * p.cap_r + slot) * kHeadDim + (lane & 15) * 8;
                }
            }
            half8 vr0[kPreloadV ? 8 : 1];
            if (kPreloadV) {
#pragma unroll
                for (int j = 0; j < 8; ++j) vr0[j] = half8{};
                if (cnt > 0 && p.n_vr > 0 && p.n_vq < (tile0 + wave + 1) * kTileTokens) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) vr0[j] = load_value_row((tile0 + wave) * kTileTokens, j);
                }
            }
            // ---- phase 1: raw logits ----
            for (int i = 0; i < cnt; ++i) {
                const int tile = tile0 + wave + 4 * i;
                const int tt = tile * kTileTokens;
                if (tt < p.n_kq) {
                    uint32_t w[kLaneWords];
                    load_tile_words<BITS>(p.k_codes + (ubase + wave + 4 * i) * kWords, lane, w);
                    const __half2 s2 = *reinterpret_cast<const __half2*>(
                        p.k_scale + ((ubase + wave + 4 * i) >> kg) * kHeadDim + 2 * lane);
                    stage_key_operand<REP>(wl.b, s2, qpf, lane);
                    wave_lds_sync();
                    key_tile_mfma<BITS, REP>(w, wl.b, wl.lr, i, lane);
                    wave_lds_sync();
                } else {
                    // fp16 residual keys on the vector ALUs: lane (seg, row) takes channels seg*8.. of rows
                    // row, row+4, ...; fp16 x fp16 dot products (v_dot2) with fp32 accumulation.  The
                    // finished logit a is stored as a * 2^-24 in the head's hi column (lo column and
                    // z-term 0), which the softmax turns back into a exactly.
                    const int seg = lane & 15, row = lane >> 4;
                    const int64_t qrow = ((int64_t)batch_of(u) * p.n_q_heads + first_q_head(u)) * kHeadDim;
#pragma unroll
                    for (int j0 = 0; j0 < 8; j0 += RB) {
                        half8 kr[RB];
#pragma unroll
                        for (int j = 0; j < RB; ++j) {   // the batch's row loads first; rows past the end re-read the last row
                            const int t = min(tt + (j0 + j) * 4 + row, p.length - 1);
                            const int slot = ring_slot(p.k_r_start, t - p.n_kq, p.cap_r);
                            const __half* src = p.k_resid + (unit * p.cap_r + slot) * kHeadDim;
                            if (fused_append && t == p.length - 1) src = p.k_new + unit * kHeadDim;   // not in the ring yet
                            kr[j] = *reinterpret_cast<const half8*>(src + seg * 8);
                        }
#pragma unroll
                        for (int hh = 0; hh < REP; ++hh) {
                            const half8 qh = hh < rep_of(u) ? *reinterpret_cast<const half8*>(p.q + qrow + hh * kHeadDim + seg * 8) : half8{};
#pragma unroll
                            for (int j = 0; j < RB; ++j) {
                                const int tl = (j0 + j) * 4 + row;
                                float a = dot8(kr[j], qh);
                                a += dpp<kDppXor1>(a); a += dpp<kDppXor2>(a);
                                a += dpp<kDppHalfMirror>(a); a += dpp<kDppMirror>(a);
                                if (seg == 0) {
                                    wl.lr[2 * hh][i * kTileTokens + tl] =
                                        tt + tl < p.length ? a * (p.softmax_scale * kDownscale) : -INFINITY;
                                    wl.lr[2 * hh + 1][i * kTileTokens + tl] = 0.f;
                                }
                            }
                        }
                    }
                }
            }
            wave_lds_sync();
            softmax_step(cnt);
            wave_lds_sync();
            // ---- phase 3: outputs ----
            // (query heads in groups of at most four: with eight the accumulators of the fp16 rows
            // would not fit in registers; the rows are then loaded once per group)
            constexpr int HG = REP > 4 ? 4 : REP;
#pragma unroll 1
            for (int h0 = 0; h0 < REP; h0 += HG) {
                float racc[HG][8];
#pragma unroll
            for (int hh = 0; hh < HG; ++hh)
#pragma unroll
                for (int e = 0; e < 8; ++e) racc[hh][e] = 0.f;
            for (int i = 0; i < cnt; ++i) {
                const int tile = tile0 + wave + 4 * i;
                const int tt = tile * kTileTokens;
                const int n_vq_here = min(max(p.n_vq - tt, 0), kTileTokens);
                if (n_vq_here > 0 && h0 == 0) {
                    uint32_t w[kLaneWords];
                    load_tile_words<BITS>(p.v_codes + (ubase + wave + 4 * i) * kWords, lane, w);
                    __half2 s2, z2;
                    if constexpr (CS) {
                        s2 = value_scale_pair<CS>(value_scale_word<CS>(p.v_scale, ubase + wave + 4 * i, kg, vlane), vlane);
                        z2 = value_scale_pair<CS>(value_scale_word<CS>(p.v_zero, ubase + wave + 4 * i, kg, vlane), vlane);
                    } else {
                        const int64_t so = (ubase + wave + 4 * i) * kTileTokens * 4 + 2 * lane;
                        s2 = *reinterpret_cast<const __half2*>(p.v_scale + so);
                        z2 = *reinterpret_cast<const __half2*>(p.v_zero + so);
                    }
                    stage_value_operand<BITS, REP, true>(wl.b, s2, z2, n_vq_here, wl.lr, i, zacc, lane);
                    wave_lds_sync();
                    value_tile_mfma<BITS, REP>(w, wl.b, acc, lane);
                    wave_lds_sync();
                }
                if (n_vq_here < kTileTokens && p.n_vr > 0) {
                    // fp16 residual values on the vector ALUs: lane (seg, row)
#pragma unroll
                    for (int j0 = 0; j0 < 8; j0 += RB) {
                        half8 vr[RB];
                        if (kPreloadV && i == 0) {
#pragma unroll
                            for (int j = 0; j < RB; ++j) vr[j] = vr0[j];     // requested before the logits were computed
                        } else {
#pragma unroll
                            for (int j = 0; j < RB; ++j) vr[j] = load_value_row(tt, j0 + j);
                        }
#pragma unroll
                        for (int j = 0; j < RB; ++j) {
                            const int tl = (j0 + j) * 4 + (lane >> 4);
                            const bool use = tl >= n_vq_here && tt + tl < p.length;
#pragma unroll
                            for (int hh = 0; hh < HG; ++hh) {
                                const float pt = use ? wl.lr[2 * (h0 + hh)][i * kTileTokens + tl] : 0.f;
#pragma unroll
                                for (int e = 0; e < 8; ++e) racc[hh][e] = fmaf(pt, (float)vr[j][e], racc[hh][e]);
                            }
                        }
                    }
                }
            }
            // lane (seg, row) holds channels seg*8.. of every 4th row: add the four row groups into LDS
            wave_lds_sync();
#pragma unroll
            for (int hh = 0; hh < HG; ++hh) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float rr = racc[hh][e];
                    rr += __shfl_xor(rr, 16); rr += __shfl_xor(rr, 32);
                    racc[hh][e] = rr;
                }
                if (lane < 16) {
                    float* dst = &sm_r[wave][h0 + hh][lane * 8];
                    float4 a = *reinterpret_cast<float4*>(dst), c = *reinterpret_cast<float4*>(dst + 4);
                    a.x += racc[hh][0]; a.y += racc[hh][1]; a.z += racc[hh][2]; a.w += racc[hh][3];
                    c.x += racc[hh][4]; c.y += racc[hh][5]; c.z += racc[hh][6]; c.w += racc[hh][7];
                    *reinterpret_cast<float4*>(dst) = a;
                    *reinterpret_cast<float4*>(dst + 4) = c;
                }
            }
            }
            wave_lds_sync();
            if (owns_new) *reinterpret_cast<uint4*>(new_dst) = new_row;
        }
    }
    }

    // ================= phase 2: this workgroup's all-quantised chunks =================
    // Software-pipelined across chunk and unit borders: the next chunk's data is requested while
    // the current one is consumed.
    if constexpr (kQOnly) {         // the first query ahead of the first chunk: loads return in order
        if (first_a < last_a) request_q(first_a / n_a);
    }
    if constexpr (!kEarlyKeys) initial_request_keys();
    initial_request_values();                       // overlaps the merge of the last fp16-row unit
    // If the last unit of phase 1 is the first unit of phase 2 and no other workgroup touches it, its
    // running state simply carries over: no part, no merge.
    bool carry = false;
    const int ua_lo = first_a < last_a ? first_a / n_a : 0, ua_hi = first_a < last_a ? (last_a - 1) / n_a : -1;
    if (ub_lo <= ub_hi) {
        if (ua_lo <= ua_hi && ua_lo == ub_hi) {
            int ga0, len_a, gb0, len_b;
            contributors(ub_hi, ga0, len_a, gb0, len_b);
            carry = len_a == 1 && len_b == 1;
        }
        if (!carry) finish_fp16_unit(ub_hi);
    }
    for (int u = ua_lo; u <= ua_hi; ++u) {
        const int a_lo = max(first_a, u * n_a), a_hi = min(last_a, (u + 1) * n_a);
        const bool carried = carry && u == ua_lo;
        if (kQOnly && kPrefetchPart) request_rows_part(u);
        if (!carried) enter_unit(u);
        if (kQOnly && u < ua_hi) request_q(u + 1);
        for (int ck = a_lo; ck < a_hi; ++ck) {
            const int n_tiles = nx_nt;                   // the chunk requested last is the one processed now
            set_next(ck + 1, false);
            const int cnt = n_tiles > wave ? (n_tiles - wave + 3) / 4 : 0;     // valid slots of this wavefront
            if constexpr (kRagged) {
                // A batch of different lengths: a chunk past the end of a shorter sequence is empty.  Its
                // data (a re-read tile that may never have been written) is dropped unseen; only the
                // requests for the chunk after it are made, in the usual order.
                if (n_tiles <= 0) {
                    request_zero_rows();
#pragma unroll
                    for (int i = 0; i < kSlots; ++i) request_key_slot(i);
#pragma unroll
                    for (int i = 0; i < kSlots; ++i) request_value_slot(i);
                    continue;
                }
            }
            // key z-terms of the wave's four slots: one 16x16x128 product
            {
                float4v d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const half8 bq = *reinterpret_cast<const half8*>(&sm_qf[ncol][ks * 32 + rq * 8]);
                    d = __builtin_amdgcn_mfma_f32_16x16x32_f16(zf[ks], bq, d, 0, 0, 0);
                }
                // d[j]: slot rq*4 + j (rows 0..3 are the wave's slots), column n
                if (n < NC && rq == 0) *reinterpret_cast<float4*>(&wl.zt[n][0]) = make_float4(d[0], d[1], d[2], d[3]);
            }
            request_zero_rows();

            // ---- phase 1: raw logits ----
#pragma unroll
            for (int c0 = 0; c0 < kSlots; c0 += SS) {
#pragma unroll
                for (int s = 0; s < SS; ++s) stage_key_operand<REP>(wl.b + s * WL::kKSlot, ks2[c0 + s], qpf, lane);
                wave_lds_sync();
#pragma unroll
                for (int s = 0; s < SS; ++s) {
                    key_tile_mfma<BITS, REP>(kw[c0 + s], wl.b + s * WL::kKSlot, wl.lr, c0 + s, lane);
                    request_key_slot(c0 + s);                  // the slot's registers are free again
                }
                wave_lds_sync();
            }
            wave_lds_sync();
            softmax_step(cnt);
            wave_lds_sync();
            // ---- phase 3: outputs ----
#pragma unroll
            for (int c0 = 0; c0 < kSlots; c0 += SS) {
#pragma unroll
                for (int s = 0; s < SS; ++s)
                    stage_value_operand<BITS, REP, false>(wl.b + s * WL::kVSlot, value_scale_pair<CS>(vs2[c0 + s], vlane), value_scale_pair<CS>(vz2[c0 + s], vlane),
                                                          kTileTokens, wl.lr, c0 + s, zacc, lane);
                wave_lds_sync();
#pragma unroll
                for (int s = 0; s < SS; ++s) {
                    value_tile_mfma<BITS, REP>(vw[c0 + s], wl.b + s * WL::kVSlot, acc, lane);
                    request_value_slot(c0 + s);
                }
                wave_lds_sync();
            }
            wave_lds_sync();
        }

        int get = -1;
        if (n_popped < n_held && sm_hold_unit[n_popped] == u) get = n_popped++;     // its phase-1 part waits in LDS
        finish_unit(u, false, carried, -1, get);
    }
}

// Workgroups the current device holds at once for one instantiation: an occupancy query, whose
// answer is kept per device (the only state the library keeps; a plain integer per device and
// instantiation, written once with the same value by whichever thread asks first).
constexpr int kMaxDevices = 64;
template <int BITS, int REP, int SLOTS, int OCC, int MODE = kBothPhases, int HSHIFT = 0, bool CS = false>
int resident_workgroups() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256 * OCC;
    const bool keep = dev >= 0 && dev < kMaxDevices;
    if (keep) {
        const int c = cached[dev].load(std::memory_order_relaxed);
        if (c > 0) return c;
    }
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_mfma_kernel<BITS, REP, SLOTS, OCC, MODE, HSHIFT, CS>, 256, 0) != hipSuccess ||
        cus <= 0 || per_cu <= 0)
        return 256 * OCC;
    if (keep) cached[dev].store(cus * per_cu, std::memory_order_relaxed);
    return cus * per_cu;
}

// ---- the all-quantised part with one (batch, kv-head) unit per WAVEFRONT ----
// Second launch of the two-launch form for batches with at least as many units as the chip holds
// wavefronts of this kernel.  In decode_mfma_kernel<..., kQuantisedOnly> the four wavefronts of a
// workgroup share every unit (each takes every 4th tile), so leaving a unit means merging four
// states through LDS between workgroup barriers and staging the next query behind another one:
// 2.0-2.3 us per unit at the streaming configuration (device timestamps), four times per
// workgroup, 13 % of the launch.  Here a wavefront walks whole units by itself, four consecutive
// tiles at a time through the same register pipeline (next group's data requested while the current
// one is consumed, across unit borders; next unit's query and the first launch's part requested one
// unit ahead): no barrier, no cross-wavefront merge, no device-scope traffic; leaving a unit is
// a reduction inside the wavefront and the output store.  Same tile arithmetic (the device functions
// above), same running-maximum softmax, same merge with the part of the fp16-row launch.
// SLICES: instead of whole units in a stride, a wavefront walks a SLICE of the unit-major axis of
// four-tile groups (first unit, first group, number of groups: p.wave_desc, made by the host so that
// all slices are equally long whatever the sequences' lengths are).  A unit that several slices touch
// gets one part per slice in the workspace (device-scope stores, then the unit's counter); the
// wavefront that finds the counter complete merges the parts and the fp16-row launch's part and
// writes the output -- all inside wavefronts, still no barrier.  p.unit_parts holds, per unit, the
// first slice that touches it and the number of slices that do.
template <int BITS, int REP, int OCC, bool CS = false, bool SLICES = false>
__global__ __launch_bounds__(256, OCC) void decode_wave_units_kernel(DecodeParams p) {
    constexpr int kSlots = 4;
    constexpr int kStage = REP > 2 ? 1 : 2;
    using WL = WaveLds<REP, kStage>;
    constexpr int NC = 2 * REP, SS = WL::kStageSlots;
    constexpr int kWords = kTileTokens * kHeadDim * BITS / 32;
    constexpr int kLaneWords = BITS * 2;
    constexpr int kIdx = 2 * REP;                       // output elements per lane: (head, channel lane + 64 k)
    __shared__ WL sm_w[4];
    __shared__ __align__(16) float sm_q[4][REP][kHeadDim];
    __shared__ __align__(16) __half sm_qf[4][NC][kKRow];
    __shared__ float sm_zs[4][REP][4];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 15, rq = lane >> 4, ncol = n & (NC - 1);
    WL& wl = sm_w[wave];
    const int kg = CS ? p.kg_shift : 0;
    const ValueScaleLane vlane = CS ? value_scale_lane<CS>(lane, kg) : ValueScaleLane{0, 0u};
    const int rep = p.rep_here, rep_total = p.n_q_heads / p.n_kv_heads;
    const int units = p.batch * p.n_kv_heads;
    const int n_waves = (int)gridDim.x * 4, gw = (int)blockIdx.x * 4 + wave;
    // all-quantised tiles of a unit (>= 1): the plan's, or -- a batch of different lengths -- the
    // sequence's own from seq_state (the host has checked that every sequence has at least one)
    auto tiles_of = [&](int u) -> int {
        return p.seq_state ? __builtin_amdgcn_readfirstlane(p.seq_state[4 * (u / p.n_kv_heads)]) / kTileTokens : p.plan.tiles_a;
    };
    const int row_stride = p.plan.n_splits();           // workspace rows per (batch, query head); row 0: the fp16-row launch's part
    if (gw >= (SLICES ? p.n_slices : units)) return;    // whole wavefronts leave; the kernel has no barrier
    // this wavefront's slice (SLICES): first unit, first group in it, groups to do
    int sl_unit = 0, sl_group = 0, sl_count = 0;
    if constexpr (SLICES) {
        sl_unit = __builtin_amdgcn_readfirstlane(p.wave_desc[4 * gw + 0]);
        sl_group = __builtin_amdgcn_readfirstlane(p.wave_desc[4 * gw + 1]);
        sl_count = __builtin_amdgcn_readfirstlane(p.wave_desc[4 * gw + 2]);
    }

    auto first_q_head = [&](int u) -> int { return (u % p.n_kv_heads) * rep_total + p.q_head0; };
    auto batch_of = [&](int u) -> int { return u / p.n_kv_heads; };

    uint32_t kw[kSlots][kLaneWords], vw[kSlots][kLaneWords];
    __half2 ks2[kSlots], vs2[kSlots], vz2[kSlots];
    half8 zf[4];
    // the group whose data is being requested ("next"); requests are unconditional (past the end they
    // re-read tile 0 of unit 0) so that the compiler counts the outstanding loads exactly
    int nx_u = SLICES ? sl_unit : gw, nx_g = SLICES ? sl_group : 0, nx_tiles = tiles_of(nx_u);
    int nx_left = sl_count;                             // SLICES: groups of the slice not requested yet
    bool nx_ok = true;
    auto next_tile = [&](int slot) -> int64_t {
        return nx_ok ? (int64_t)nx_u * p.cap_tiles + min(nx_g * kSlots + slot, nx_tiles - 1) : 0;
    };
    // row of the key scale / zero-point arrays (one per group of G = 32 << kg tokens) of that tile
    auto next_key_row = [&](int slot) -> int64_t {
        return nx_ok ? (((int64_t)nx_u * p.cap_tiles) >> kg) + (min(nx_g * kSlots + slot, nx_tiles - 1) >> kg) : 0;
    };
    auto advance_next = [&]() {
        if constexpr (SLICES) {
            nx_ok = --nx_left > 0;
            if (++nx_g * kSlots >= nx_tiles) {
                nx_g = 0;
                ++nx_u;
                nx_ok = nx_ok && nx_u < units;
                nx_tiles = nx_ok ? tiles_of(nx_u) : 1;
            }
        } else {
            if (++nx_g * kSlots >= nx_tiles) {
                nx_g = 0;
                nx_u += n_waves;
                nx_ok = nx_u < units;
                nx_tiles = nx_ok ? tiles_of(nx_u) : 1;
            }
        }
    };
    auto request_zero_rows = [&]() {
        int64_t row;                                                       // A row n = slot n
        if constexpr (CS) row = next_key_row(min(n, kSlots - 1));
        else row = next_tile(min(n, kSlots - 1));
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            zf[ks] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(p.k_zero + row * kHeadDim + ks * 32 + rq * 8));
    };
    auto request_key_slot = [&](int i) {
        const int64_t tile = next_tile(i);
        load_tile_words<BITS>(p.k_codes + tile * kWords, lane, kw[i]);
        if constexpr (CS) ks2[i] = nt_half2(p.k_scale + next_key_row(i) * kHeadDim + 2 * lane);
        else ks2[i] = nt_half2(p.k_scale + tile * kHeadDim + 2 * lane);
    };
    auto request_value_slot = [&](int i) {
        const int64_t tile = next_tile(i);
        load_tile_words<BITS>(p.v_codes + tile * kWords, lane, vw[i]);
        if constexpr (CS) {
            vs2[i] = value_scale_word<CS>(p.v_scale, tile, kg, vlane);
            vz2[i] = value_scale_word<CS>(p.v_zero, tile, kg, vlane);
        } else {
            vs2[i] = nt_half2(p.v_scale + tile * kTileTokens * 4 + 2 * lane);
            vz2[i] = nt_half2(p.v_zero + tile * kTileTokens * 4 + 2 * lane);
        }
    };
    // query and fp16-row part of a unit: lane l holds the elements (head k / 2, channel l + 64 (k % 2))
    __half q_pre[kIdx];
    float pre_m[kIdx], pre_l[kIdx], pre_o[kIdx];
    auto request_unit = [&](int u_req) {
        const int u = min(u_req, units - 1);                              // unconditional loads (clamped)
        const int64_t row0 = (int64_t)batch_of(u) * p.n_q_heads + first_q_head(u);
#pragma unroll
        for (int k = 0; k < kIdx; ++k) {
            const int64_t row = row0 + min(k >> 1, rep - 1);
            const int c = lane + 64 * (k & 1);
            q_pre[k] = p.q[row * kHeadDim + c];
            pre_m[k] = p.part_ml[row * row_stride * 2 + 0];
            pre_l[k] = p.part_ml[row * row_stride * 2 + 1];
            pre_o[k] = p.part_o[row * row_stride * kHeadDim + c];
        }
    };

    float4v acc[8];
    float zacc[REP][2], m_run[REP], l_lane[REP], qpf[REP][2];

    // probabilities of the wavefront's 128 token slots against the running maximum (2 slots per lane)
    auto softmax_step = [&](int cnt) {
        const int slot = lane >> 4;
        const bool live = slot < cnt;
        float a0[REP], a1[REP], scale_lane = 1.f;
        bool any_rescale = false;
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            const float2 hi = *reinterpret_cast<const float2*>(&wl.lr[2 * hh][2 * lane]);
            const float2 lo = *reinterpret_cast<const float2*>(&wl.lr[2 * hh + 1][2 * lane]);
            const float zt = join_hi_lo(wl.zt[2 * hh][slot], wl.zt[2 * hh + 1][slot]);
            a0[hh] = live ? fmaf(join_hi_lo(hi.x, lo.x), kUnscale, zt) : -INFINITY;
            a1[hh] = live ? fmaf(join_hi_lo(hi.y, lo.y), kUnscale, zt) : -INFINITY;
            const float mx = wave_max(fmaxf(a0[hh], a1[hh]));
            if (mx > m_run[hh]) {                       // wave-uniform: the running maximum grows
                const float f = __expf(m_run[hh] - mx); // 0 on the first group (m_run = -inf)
                l_lane[hh] *= f;
                zacc[hh][0] *= f; zacc[hh][1] *= f;
                if ((n >> 1) == hh) scale_lane = f;
                any_rescale = true;
                m_run[hh] = mx;
            }
        }
        if (any_rescale) {
#pragma unroll
            for (int u8 = 0; u8 < 8; ++u8)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[u8][j] *= scale_lane;
        }
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            const float p0 = __expf(a0[hh] - m_run[hh]), p1 = __expf(a1[hh] - m_run[hh]);   // a group has at least one live slot
            *reinterpret_cast<float2*>(&wl.lr[2 * hh][2 * lane]) = make_float2(p0, p1);
            l_lane[hh] += p0 + p1;
        }
        wave_lds_sync();
    };

    request_unit(SLICES ? sl_unit : gw);
    request_zero_rows();
#pragma unroll
    for (int i = 0; i < kSlots; ++i) request_key_slot(i);
#pragma unroll
    for (int i = 0; i < kSlots; ++i) request_value_slot(i);

    int g_first = sl_group, left = sl_count;
    for (int u = SLICES ? sl_unit : gw; SLICES ? left > 0 : u < units; u += SLICES ? 1 : n_waves) {
        // ---- enter the unit: query operands of this wavefront ----
        int first_slice = 0, n_parts = 1;               // SLICES: the slices that touch this unit
        if constexpr (SLICES) {
            first_slice = __builtin_amdgcn_readfirstlane(p.unit_parts[2 * u + 0]);
            n_parts = __builtin_amdgcn_readfirstlane(p.unit_parts[2 * u + 1]);
        }
        float um[kIdx], ul[kIdx], uo[kIdx];              // the fp16-row launch's part of this unit
#pragma unroll
        for (int k = 0; k < kIdx; ++k) {
            const int hh = k >> 1, c = lane + 64 * (k & 1);
            const float x = hh < rep ? p.softmax_scale * __half2float(q_pre[k]) : 0.f;
            __half hi, lo;
            split_hi_lo(x, hi, lo);
            sm_q[wave][hh][c] = x;
            sm_qf[wave][2 * hh][c] = hi;
            sm_qf[wave][2 * hh + 1][c] = lo;
            um[k] = pre_m[k]; ul[k] = pre_l[k]; uo[k] = pre_o[k];
        }
        wave_lds_sync();
        request_unit(SLICES ? u + 1 : u + n_waves);     // one unit ahead
        {
            const float pf = inv_pos_factor<BITS>(lane & 3);
#pragma unroll
            for (int hh = 0; hh < REP; ++hh) {
                qpf[hh][0] = sm_q[wave][hh][2 * lane] * pf;
                qpf[hh][1] = sm_q[wave][hh][2 * lane + 1] * pf;
            }
        }
#pragma unroll
        for (int u8 = 0; u8 < 8; ++u8) acc[u8] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
            zacc[hh][0] = zacc[hh][1] = 0.f;
            m_run[hh] = -INFINITY;
            l_lane[hh] = 0.f;
        }

        const int tiles = tiles_of(u);
        const int g_lo = SLICES ? g_first : 0;
        const int g_hi = SLICES ? min((tiles + kSlots - 1) / kSlots, g_first + left) : (tiles + kSlots - 1) / kSlots;
        if constexpr (SLICES) {
            left -= g_hi - g_lo;
            g_first = 0;
        }
        for (int g = g_lo; g < g_hi; ++g) {
            const int cnt = min(kSlots, tiles - g * kSlots);          // tiles of this group
            advance_next();                                             // the requests below are for the group after this one
            // key z-terms of the four slots: one 16x16x128 product
            {
                float4v d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const half8 bq = *reinterpret_cast<const half8*>(&sm_qf[wave][ncol][ks * 32 + rq * 8]);
                    d = __builtin_amdgcn_mfma_f32_16x16x32_f16(zf[ks], bq, d, 0, 0, 0);
                }
                if (n < NC && rq == 0) *reinterpret_cast<float4*>(&wl.zt[n][0]) = make_float4(d[0], d[1], d[2], d[3]);
            }
            request_zero_rows();
            // ---- raw logits ----
#pragma unroll
            for (int c0 = 0; c0 < kSlots; c0 += SS) {
#pragma unroll
                for (int sl = 0; sl < SS; ++sl) stage_key_operand<REP>(wl.b + sl * WL::kKSlot, ks2[c0 + sl], qpf, lane);
                wave_lds_sync();
#pragma unroll
                for (int sl = 0; sl < SS; ++sl) {
                    key_tile_mfma<BITS, REP>(kw[c0 + sl], wl.b + sl * WL::kKSlot, wl.lr, c0 + sl, lane);
                    request_key_slot(c0 + sl);                          // the slot's registers are free again
                }
                wave_lds_sync();
            }
            wave_lds_sync();
            softmax_step(cnt);
            // ---- outputs ----
#pragma unroll
            for (int c0 = 0; c0 < kSlots; c0 += SS) {
#pragma unroll
                for (int sl = 0; sl < SS; ++sl)
                    stage_value_operand<BITS, REP, false>(wl.b + sl * WL::kVSlot, value_scale_pair<CS>(vs2[c0 + sl], vlane), value_scale_pair<CS>(vz2[c0 + sl], vlane),
                                                          kTileTokens, wl.lr, c0 + sl, zacc, lane);
                wave_lds_sync();
#pragma unroll
                for (int sl = 0; sl < SS; ++sl) {
                    value_tile_mfma<BITS, REP>(vw[c0 + sl], wl.b + sl * WL::kVSlot, acc, lane);
                    request_value_slot(c0 + sl);
                }
                wave_lds_sync();
            }
            wave_lds_sync();
        }

        // ---- leave the unit: raw matrix-core outputs and z-term sums through this wavefront's LDS ----
        if (n < NC) {
#pragma unroll
            for (int u8 = 0; u8 < 8; ++u8)
                *reinterpret_cast<float4*>(&wl.lr[n][u8 * 16 + rq * 4]) =
                    make_float4(acc[u8][0], acc[u8][1], acc[u8][2], acc[u8][3]);
        }
        float l_w[REP];
#pragma unroll
        for (int hh = 0; hh < REP; ++hh) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float zz = zacc[hh][k];
                zz += dpp<kDppXor2>(zz); zz += dpp<kDppRor4>(zz); zz += dpp<kDppRor8>(zz);
                zz += __shfl_xor(zz, 16); zz += __shfl_xor(zz, 32);
                if (lane < 2) sm_zs[wave][hh][lane * 2 + k] = zz;      // lane 0: groups 0,1; lane 1: groups 2,3
            }
            l_w[hh] = wave_sum(l_lane[hh]);
        }
        wave_lds_sync();
        const int64_t row0 = (int64_t)batch_of(u) * p.n_q_heads + first_q_head(u);
        if (!SLICES || n_parts == 1) {
#pragma unroll
            for (int k = 0; k < kIdx; ++k) {
                const int hh = k >> 1, c = lane + 64 * (k & 1);
                if (hh < rep) {
                    float mm = m_run[hh], ll = l_w[hh];
                    float oo = fmaf(join_hi_lo(wl.lr[2 * hh][c], wl.lr[2 * hh + 1][c]), kUnscale, sm_zs[wave][hh][c >> 5]);
                    if (um[k] > -INFINITY) {                 // the fp16-row launch's part (the window is never empty in this form)
                        const float mn = fmaxf(mm, um[k]);
                        const float f_old = __expf(mm - mn), f_new = __expf(um[k] - mn);
                        ll = fmaf(ll, f_old, ul[k] * f_new);
                        oo = fmaf(oo, f_old, uo[k] * f_new);
                    }
                    p.out[(row0 + hh) * kHeadDim + c] = oo / ll;
                }
            }
        } else {
            // several slices share the unit: this one's part goes to the workspace (slot 0 is the fp16-row
            // launch's), published as in decode_mfma_kernel: device-scope stores, the wait for their
            // acknowledgement, then the counter; whoever completes the count merges
            const int slot = 1 + gw - first_slice;
#pragma unroll
            for (int k = 0; k < kIdx; ++k) {
                const int hh = k >> 1, c = lane + 64 * (k & 1);
                if (hh < rep) {
                    const float oo = fmaf(join_hi_lo(wl.lr[2 * hh][c], wl.lr[2 * hh + 1][c]), kUnscale, sm_zs[wave][hh][c >> 5]);
                    const int64_t prow = (row0 + hh) * row_stride + slot;
                    device_store(p.part_o + prow * kHeadDim + c, oo);
                    if (c == 0) {
                        device_store(p.part_ml + prow * 2 + 0, m_run[hh]);
                        device_store(p.part_ml + prow * 2 + 1, l_w[hh]);
                    }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            int done = 0;
            if (lane == 0) done = __hip_atomic_fetch_add(p.counters + u, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            done = __builtin_amdgcn_readfirstlane(done);
            if (done == n_parts - 1) {
#pragma unroll
                for (int k = 0; k < kIdx; ++k) {
                    const int hh = k >> 1, c = lane + 64 * (k & 1);
                    if (hh < rep) {
                        const int64_t prow = (row0 + hh) * row_stride;
                        float mm = um[k], ll = ul[k], oo = uo[k];          // slot 0: written by the previous launch
                        if (!(mm > -INFINITY)) { mm = -INFINITY; ll = 0.f; oo = 0.f; }
                        // eight parts at a time: the device-scope loads of a batch are all issued before
                        // the first is used (each is a trip to memory, not to a cache)
                        for (int i0 = 1; i0 <= n_parts; i0 += 8) {
                            float mv[8], lv[8], ov[8];
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const int i = min(i0 + j, n_parts);
                                mv[j] = device_load(p.part_ml + (prow + i) * 2 + 0);
                                lv[j] = device_load(p.part_ml + (prow + i) * 2 + 1);
                                ov[j] = device_load(p.part_o + (prow + i) * kHeadDim + c);
                            }
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                if (i0 + j <= n_parts && mv[j] > -INFINITY) {
                                    const float mn = fmaxf(mm, mv[j]);
                                    const float f_old = __expf(mm - mn), f_new = __expf(mv[j] - mn);   // mm = -inf: f_old = 0
                                    ll = fmaf(ll, f_old, lv[j] * f_new);
                                    oo = fmaf(oo, f_old, ov[j] * f_new);
                                    mm = mn;
                                }
                            }
                        }
                        p.out[(row0 + hh) * kHeadDim + c] = oo / ll;
                    }
                }
                if (lane == 0) __hip_atomic_store(p.counters + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        wave_lds_sync();                                 // this wavefront's LDS is reused by its next unit
    }
}

// Wavefronts the device holds at once for decode_wave_units_kernel (per device, as above).
template <int BITS, int REP, int OCC, bool CS = false, bool SLICES = false>
int resident_wave_unit_workgroups() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256 * OCC;
    const bool keep = dev >= 0 && dev < kMaxDevices;
    if (keep) {
        const int c = cached[dev].load(std::memory_order_relaxed);
        if (c > 0) return c;
    }
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_wave_units_kernel<BITS, REP, OCC, CS, SLICES>, 256, 0) != hipSuccess ||
        cus <= 0 || per_cu <= 0)
        return 256 * OCC;
    if (keep) cached[dev].store(cus * per_cu, std::memory_order_relaxed);
    return cus * per_cu;
}

template <int BITS, int REP, int SLOTS, int OCC, int HSHIFT = 0, bool CS = false>
hipError_t launch_one(DecodeParams p, hipStream_t stream) {
    if (p.plan.tiles_per_split_a != 4 * SLOTS || p.plan.tiles_per_split_b > kMfmaSplitTiles) return hipErrorInvalidValue;
    const int64_t units = HSHIFT == kRuntimeHeadGroups ? (int64_t)p.batch * p.n_kv_heads * p.head_groups
                                                        : ((int64_t)p.batch * p.n_kv_heads) << HSHIFT;
    const int64_t total_a = units * p.plan.n_splits_a, total_b = units * p.plan.n_splits_b;
    // Cost of an fp16-row chunk in units of an all-quantised chunk: by the bytes they stream, times
    // a measured factor per instantiation -- with 5 to 8 query heads per kv-head, and with 3 or 4 at
    // 4 bits, the chain  rows -> logits -> softmax -> rows -> outputs  of an fp16-row chunk takes about
    // as long as two all-quantised chunks (sweep of the weight from 1 to 5 over 8-512 units, contexts
    // 1k-16k, windows 64-192: 2 is best for all three, 2-7 % on average and up to 36 % faster than 1;
    // odd weights leave workgroups with an fp16-row chunk and all-quantised chunks and are slower).
    // One head or two, and 3 or 4 heads at 2 bits: 1.
    constexpr int kRowsFactor = (REP > 4 || (REP > 2 && BITS == 4)) ? 2 : 1;
    const int64_t bytes_a = (int64_t)4 * SLOTS * kTileTokens * 2 * (kHeadDim * BITS / 8 + 16);
    const int64_t bytes_b = (int64_t)p.plan.tiles_per_split_b * kTileTokens * 2 * kHeadDim * 2;
    p.cost_b = kRowsFactor * (int)std::max<int64_t>(1, (bytes_b + bytes_a / 2) / bytes_a);
    p.cost_unit = p.plan.n_splits_b * p.cost_b + p.plan.n_splits_a;
    p.total_cost = units * p.cost_unit;
    if (p.total_cost <= 0 || p.total_cost > 0x3fffffff || total_a + total_b > 0x7fffffff) return hipErrorInvalidValue;
    p.total_chunks_a = (int)total_a;
    p.total_chunks_b = (int)total_b;
    // every resident workgroup gets an equal share of the cost axis (within one unit of cost)
    const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(resident_workgroups<BITS, REP, SLOTS, OCC, kBothPhases, HSHIFT, CS>(),
                                                                  p.total_cost / p.cost_b));
    decode_mfma_kernel<BITS, REP, SLOTS, OCC, kBothPhases, HSHIFT, CS><<<grid, 256, 0, stream>>>(p);
    return hipGetLastError();
}

// The two-launch form: the fp16 rows of all units (residual_rows_kernel), then the all-quantised
// chunks on a cost axis of their own (unit-major, one unit of cost per chunk).
template <int BITS, int REP, int SLOTS, int OCC, bool CS = false>
hipError_t launch_two(DecodeParams p, hipStream_t stream) {
    if (p.plan.tiles_per_split_a != 4 * SLOTS || p.plan.n_splits_a < 1) return hipErrorInvalidValue;
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    const int64_t total_a = units * p.plan.n_splits_a;
    if (total_a > 0x3fffffff) return hipErrorInvalidValue;
    // (with a residual flush to carry out, the first launch also quantises the flushed tokens)
    if (hipError_t e = p.flush_k ? launch_rows_and_flush(p, *p.flush_k, *p.flush_v, stream) : launch_residual_rows(p, stream);
        e != hipSuccess)
        return e;
    p.flush_k = nullptr;
    p.flush_v = nullptr;
    p.k_new = p.v_new = nullptr;                   // the first launch has stored the new token's rows
    p.total_chunks_a = (int)total_a;
    p.total_chunks_b = 0;
    p.cost_b = 1;
    p.cost_unit = p.plan.n_splits_a;
    p.total_cost = total_a;
    // One unit per wavefront where that fills the chip evenly: at least as many units as resident
    // wavefronts, and the last round of units at most 12 % short of a full one.
    if constexpr (REP <= 4 && !CS) {
        if (p.wave_desc != nullptr) {
            // equally long slices of the unit-major group axis, one per wavefront (tables made by the host)
            if (p.n_slices < 1 || p.unit_parts == nullptr) return hipErrorInvalidValue;
            decode_wave_units_kernel<BITS, REP, OCC, false, true><<<(p.n_slices + 3) / 4, 256, 0, stream>>>(p);
            return hipGetLastError();
        }
    }
    if constexpr (REP <= 4) {
        if (!p.seq_state || (!CS && p.ragged_min_tiles >= 1)) {
            const int64_t waves = 4 * (int64_t)resident_wave_unit_workgroups<BITS, REP, OCC, CS>();
            const int64_t rounds = (units + waves - 1) / waves;
            if (units >= waves && rounds * waves * 100 <= units * 112 && p.plan.tiles_a >= 1 && p.plan.n_splits_b == 1) {
                const int grid = (int)std::min<int64_t>(waves / 4, (units + 3) / 4);
                decode_wave_units_kernel<BITS, REP, OCC, CS><<<grid, 256, 0, stream>>>(p);
                return hipGetLastError();
            }
        }
    }
    if (p.seq_state) {
        if constexpr (CS) {
            return hipErrorNotSupported;        // batches of different lengths with G > 32 go run by run (the host does not send them here)
        } else {
            const int grid = (int)std::min<int64_t>(resident_workgroups<BITS, REP, SLOTS, OCC, kQuantisedRagged>(), total_a);
            decode_mfma_kernel<BITS, REP, SLOTS, OCC, kQuantisedRagged><<<grid, 256, 0, stream>>>(p);
        }
    } else {
        const int grid = (int)std::min<int64_t>(resident_workgroups<BITS, REP, SLOTS, OCC, kQuantisedOnly, 0, CS>(), total_a);
        decode_mfma_kernel<BITS, REP, SLOTS, OCC, kQuantisedOnly, 0, CS><<<grid, 256, 0, stream>>>(p);
    }
    return hipGetLastError();
}

// The instantiation that serves (bits, query heads per kv-head): tile slots per wavefront and
// workgroups per compute unit.  `fn` is called with the four template arguments as a tag.
template <int B, int R, int S, int O> struct Variant {
    static constexpr int bits = B, rep = R, slots = S, occ = O;
};
template <class F>
bool with_variant(int bits, int rep_layout, F&& fn) {
    // the smallest instantiation that holds the layout's query heads per kv-head
    const int rep = rep_layout <= 2 ? rep_layout : (rep_layout <= 4 ? 4 : (rep_layout <= 8 ? 8 : 0));
    if (bits == 2 && rep == 1) { fn(Variant<2, 1, 4, 2>{}); return true; }
    if (bits == 2 && rep == 2) { fn(Variant<2, 2, 4, 2>{}); return true; }
    if (bits == 2 && rep == 4) { fn(Variant<2, 4, 4, 2>{}); return true; }
    if (bits == 4 && rep == 1) { fn(Variant<4, 1, 4, 2>{}); return true; }
    if (bits == 4 && rep == 2) { fn(Variant<4, 2, 4, 2>{}); return true; }
    if (bits == 4 && rep == 4) { fn(Variant<4, 4, 2, 2>{}); return true; }
    if (bits == 2 && rep == 8) { fn(Variant<2, 8, 4, 2>{}); return true; }
    if (bits == 4 && rep == 8) { fn(Variant<4, 8, 2, 2>{}); return true; }
    return false;                       // no instantiation for this shape: the vector-ALU family serves it
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeParams& p, hipStream_t stream) {
    hipError_t e = hipErrorNotSupported;
    if ((p.head_groups > 1 || p.head_split > 0) && p.kg_shift > 0) return hipErrorNotSupported;   // G > 32: whole groups, one pass per 8 heads
    if (p.head_groups > 1) {
        // runs of 4 (or 8) query heads of every kv-head as units of one single-form launch
        if (p.two_launches > 0 || p.head_split > 0 || p.q_head0 != 0 || (p.rep_here != 4 && p.rep_here != 8) || p.rep_variant != p.rep_here ||
            p.seq_state != nullptr || p.head_groups != (p.n_q_heads / p.n_kv_heads + p.rep_here - 1) / p.rep_here)
            return hipErrorInvalidValue;
        if (p.bits == 2 && p.rep_here == 8) return launch_one<2, 8, 4, 2, kRuntimeHeadGroups>(p, stream);
        if (p.bits == 4 && p.rep_here == 8) return launch_one<4, 8, 2, 2, kRuntimeHeadGroups>(p, stream);
        if (p.bits == 2 && p.rep_here == 4) return launch_one<2, 4, 4, 2, kRuntimeHeadGroups>(p, stream);
        if (p.bits == 4 && p.rep_here == 4) return launch_one<4, 4, 2, 2, kRuntimeHeadGroups>(p, stream);
        return hipErrorNotSupported;
    }
    if (p.head_split > 0) {
        // 2^head_split equal parts of every kv-head's query heads as units of their own, on the
        // instantiation for one part
        if (p.two_launches > 0 || p.q_head0 != 0 || (p.rep_here << p.head_split) != p.n_q_heads / p.n_kv_heads ||
            p.rep_variant < p.rep_here)
            return hipErrorInvalidValue;
        if (p.head_split == 1 && p.bits == 2 && p.rep_variant == 4) return launch_one<2, 4, 4, 2, 1>(p, stream);
        if (p.head_split == 1 && p.bits == 4 && p.rep_variant == 4) return launch_one<4, 4, 2, 2, 1>(p, stream);
        if (p.head_split == 1 && p.bits == 2 && p.rep_variant == 2) return launch_one<2, 2, 4, 2, 1>(p, stream);
        if (p.head_split == 2 && p.bits == 2 && p.rep_variant == 2) return launch_one<2, 2, 4, 2, 2>(p, stream);
        return hipErrorNotSupported;
    }
    if (p.kg_shift > 0) {
        // G = 64 / 128: the instantiations that read one scale / zero-point pair per group
        with_variant(p.bits, p.rep_variant, [&](auto v) {
            using V = decltype(v);
            e = p.two_launches > 0 ? launch_two<V::bits, V::rep, V::slots, V::occ, true>(p, stream)
                                   : launch_one<V::bits, V::rep, V::slots, V::occ, 0, true>(p, stream);
        });
        return e;
    }
    with_variant(p.bits, p.rep_variant, [&](auto v) {
        using V = decltype(v);
        e = p.two_launches > 0 ? launch_two<V::bits, V::rep, V::slots, V::occ>(p, stream)
                               : launch_one<V::bits, V::rep, V::slots, V::occ>(p, stream);
    });
    return e;
}

int wave_slices_resident(int bits, int rep) {
    int waves = 0;
    with_variant(bits, rep, [&](auto v) {
        using V = decltype(v);
        if constexpr (V::rep <= 4) waves = 4 * resident_wave_unit_workgroups<V::bits, V::rep, V::occ, false, true>();
    });
    return waves;
}

MfmaGeometry mfma_geometry(int bits, int rep) {
    MfmaGeometry g{0, 0};              // chunk_tiles 0: no matrix-core instantiation for this shape
    with_variant(bits, rep, [&](auto v) {
        using V = decltype(v);
        g.chunk_tiles = 4 * V::slots;
        g.resident_workgroups = resident_workgroups<V::bits, V::rep, V::slots, V::occ>();
    });
    return g;
}

}  // namespace kivi
