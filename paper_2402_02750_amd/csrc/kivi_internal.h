// Internal declarations shared by the library's translation units (host side only).
// Nothing here is part of the ABI; see include/kivi.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "kivi.h"

namespace kivi {

constexpr int kHeadDim = 128;
constexpr int kTileTokens = 32;        // tokens per code tile; a group of G = 32, 64 or 128 tokens covers 1, 2 or 4 tiles
constexpr int kMaxSplitTiles = 32;     // a context split covers at most 32 tiles (1024 tokens)
constexpr int kMfmaSplitTiles = 16;    // ... at most 16 tiles in the matrix-core family (4 per wavefront)
constexpr int kMaxRep = 8;             // query heads per kv-head handled by one launch
constexpr int kMaxRepTotal = 128;      // query heads per kv-head of a layout (wider groups take several launches)

// Source of fp16 rows for the quantise kernels: either a strided tensor or a ring buffer.
struct RowSource {
    const __half* base;   // element (b, h, t, c) at base[b*stride_b + h*stride_h + slot(t)*stride_t + c]
    int64_t stride_b, stride_h, stride_t;
    int32_t ring_start;   // slot(t) = (ring_start + t) % ring_cap when ring_cap > 0, else t
    int32_t ring_cap;
};

struct QuantKeyParams {
    RowSource src;
    uint32_t* codes;      // [b][h][cap_tiles][W]
    __half* scale;        // [b][h][cap_tiles][128]
    __half* zero;
    int32_t n_kv_heads, cap_tiles, bits;
    int32_t first_tile;   // destination tile index of source token 0
    int32_t n_tiles;
    int32_t batch;
    int32_t tiles_per_group;   // G / 32: 1, 2 or 4
};

struct QuantValueParams {
    RowSource src;
    uint32_t* codes;      // [b][h][cap_tiles][W]
    __half* scale;        // [b][h][cap_tokens][4]
    __half* zero;
    int32_t n_kv_heads, cap_tiles, bits;
    int32_t first_token;  // destination token index of source token 0 (any value)
    int32_t n_tokens;
    int32_t batch;
    int32_t group_blocks;      // G / 32: 32-channel blocks per group (1, 2 or 4)
};

// Copy fp16 rows of every (b, h) from strided tensors into residual rings: up to two (source,
// ring) pairs per launch (keys and values), the second is skipped when its n_tokens is 0.
struct CopyRowsParams {
    struct Job {
        const __half* src;    // element (b, h, t, c) at src[b*stride_b + h*stride_h + (src_t0 + t)*stride_t + c]
        int64_t stride_b, stride_h, stride_t;
        int32_t src_t0;
        __half* dst;          // [b][h][cap_r][128]
        int32_t dst_slot0;    // row t goes to slot (dst_slot0 + t) % cap_r
        int32_t n_tokens;
    } job[2];
    int32_t cap_r, n_kv_heads, batch;
};

// How the token axis [0, L) is cut into context splits (one workgroup each per (b, kv-head)).
// Region A = tiles [0, tiles_a): K and V both quantised.  Region B = tiles [tiles_a, tiles_total):
// at least one of K, V is fp16 there (5x the bytes per token), so its splits are shorter.
struct SplitPlan {
    int32_t tiles_a, tiles_total;
    int32_t tiles_per_split_a, tiles_per_split_b;
    int32_t n_splits_a, n_splits_b;
    __host__ __device__ int32_t n_splits() const { return n_splits_a + n_splits_b; }
};

struct DecodeParams {
    // cache
    const uint32_t* k_codes; const __half* k_scale; const __half* k_zero;
    const uint32_t* v_codes; const __half* v_scale; const __half* v_zero;
    const __half* k_resid; const __half* v_resid;
    // fused append (matrix-core family only; null otherwise): the rows of token length-1, [b][H_kv][128].
    // The kernel reads that token from here and writes it into the rings (which it may, then, modify).
    const __half* k_new; const __half* v_new;
    int32_t n_kq, n_vq, k_r_start, n_kr, v_r_start, n_vr;
    int32_t cap_tiles, cap_r;
    // problem
    const __half* q;        // [b][H_q][128]
    float* out;             // [b][H_q][128]
    int32_t* counters;      // workspace: [b][H_kv] finished-split counters (zero between calls)
    float* part_ml;         // workspace: [b][H_q][n_splits][2]  (max, sum)
    float* part_o;          // workspace: [b][H_q][n_splits][128]
    float softmax_scale;
    int32_t batch, n_q_heads, n_kv_heads, bits, length;
    // One launch serves query heads [q_head0, q_head0 + rep_here) of every kv-head's group, on the
    // kernel instantiation for rep_variant heads (>= rep_here; the surplus heads idle).  A group of
    // up to kMaxRep heads is one launch; a wider one (multi-query attention) takes several, all on
    // the kMaxRep instantiation so that they share one split plan.
    int32_t q_head0, rep_here, rep_variant;
    SplitPlan plan;
    // Persistent matrix-core kernel.  Work lies on a cost axis: unit u occupies [u * cost_unit,
    // (u + 1) * cost_unit): first its fp16-row chunks (cost_b each), then its all-quantised chunks
    // (cost 1 each).  Workgroup g of G owns the chunks that start in [g * T / G, (g + 1) * T / G),
    // T = units * cost_unit.
    int32_t total_chunks_a, total_chunks_b, cost_b, cost_unit;
    int64_t total_cost;
    // > 0: the matrix-core family runs as two launches (fp16 rows, then the all-quantised chunks); the
    // plan then has a single fp16-row split per unit (n_splits_b == 1).
    int32_t two_launches;
    // Batches whose sequences differ in length (two-launch form only; null otherwise): per batch entry
    // {n_q, n_r, k_r_start, v_r_start} in device memory (K and V split alike).  The scalar counters
    // and the plan above then describe the LONGEST sequence: every unit gets that many chunks on the
    // cost axis, and a shorter sequence's surplus chunks and tiles are masked.
    const int32_t* seq_state;
    int32_t kg_shift;           // log2(G / 32): scales and zero-points are stored once per group (keys: row tile >> kg_shift;
                                // values: 4 >> kg_shift entries per token); > 0 runs on instantiations of its own
    int32_t head_groups;        // > 1: runs of rep_here (4 or 8) query heads per kv-head served as units of one launch (matrix-core family)
    // Two-launch form, second launch as equally long slices of the unit-major axis of four-tile groups
    // (device arrays made by the host; null: not used): wave_desc[4 s] = {first unit, first group in it,
    // groups, 0} of slice s; unit_parts[2 u] = {first slice touching unit u, slices touching it}.
    const int32_t* wave_desc;
    const int32_t* unit_parts;
    int32_t n_slices;
    int32_t ragged_min_tiles;   // with seq_state: the fewest all-quantised tiles any sequence has (host knowledge)
    // Host side only (two-launch form): the residual flush of this decode step, to be carried out by
    // extra workgroups of the fp16-row launch instead of a launch of its own; null otherwise.
    const QuantKeyParams* flush_k;
    const QuantValueParams* flush_v;
    // k > 0 (single launch, 4, 6 or 8 query heads per kv-head, small batches): every kv-head's query
    // heads are served as 2^k equal parts, each a unit of its own on the instantiation for one part
    // (rep_variant 2 or 4, rep_here = heads of a part); the cache is read once per part.
    int32_t head_split;
};

// launchers (each defined next to its kernels); they return hipGetLastError() after the launch
hipError_t launch_quantize_keys(const QuantKeyParams& p, hipStream_t stream);
hipError_t launch_quantize_values(const QuantValueParams& p, hipStream_t stream);
// key groups and value tokens of one residual flush in a single launch (either part may be empty)
hipError_t launch_flush_quantize(const QuantKeyParams& kp, const QuantValueParams& vp, hipStream_t stream);
hipError_t launch_copy_rows(const CopyRowsParams& p, hipStream_t stream);
hipError_t launch_decode_valu(const DecodeParams& p, hipStream_t stream);
hipError_t launch_decode_mfma(const DecodeParams& p, hipStream_t stream);
hipError_t launch_residual_rows(const DecodeParams& p, hipStream_t stream);
// the same launch with extra workgroups that quantise the key group(s) and value tokens of a residual
// flush (G = 32 only: hipErrorNotSupported otherwise, nothing launched)
hipError_t launch_rows_and_flush(const DecodeParams& p, const QuantKeyParams& kp, const QuantValueParams& vp, hipStream_t stream);
// whether launch_residual_rows serves `tiles_b` tiles of fp16 rows on the instantiation for `rep_variant` heads
bool residual_rows_possible(int tiles_b, int rep_variant);
hipError_t launch_merge(const DecodeParams& p, hipStream_t stream);
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream);

// Chunk length (tiles) of all-quantised chunks and resident workgroups of the matrix-core instantiation
// that serves (bits, query heads per kv-head); the split planner and the kernel must agree on both.
struct MfmaGeometry { int chunk_tiles, resident_workgroups; };
MfmaGeometry mfma_geometry(int bits, int rep);
// wavefronts the device holds of the sliced form of decode_wave_units_kernel (0: no instantiation for the shape)
int wave_slices_resident(int bits, int rep);

}  // namespace kivi
