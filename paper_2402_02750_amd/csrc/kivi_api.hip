// Host side of the C ABI (include/kivi.h): argument validation, split planning, launches.
// No allocation, no synchronisation; the only state kept between calls is, per device, the address
// of the static scratch array below (and the occupancy answers next to the decode kernels).
#include "kivi_internal.h"

#include <algorithm>
#include <vector>
#include <atomic>

namespace kivi {
namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_layout(const kivi_layout_t* l) {
    if (!l) return KIVI_ERR_INVALID_ARG;
    if (l->batch < 1 || l->n_q_heads < 1 || l->n_kv_heads < 1) return KIVI_ERR_INVALID_ARG;
    if (l->batch > 65535 || l->n_kv_heads > 65535) return KIVI_ERR_INVALID_ARG;
    if (l->n_q_heads % l->n_kv_heads != 0) return KIVI_ERR_INVALID_ARG;
    if (l->residual < 0 || l->cap_q_tokens < 0 || l->cap_r_tokens < 0) return KIVI_ERR_INVALID_ARG;
    if (l->decode_path < KIVI_DECODE_AUTO || l->decode_path > KIVI_DECODE_MFMA_TWO) return KIVI_ERR_INVALID_ARG;
    if (l->head_dim != kHeadDim) return KIVI_ERR_UNSUPPORTED;
    if (l->bits != 2 && l->bits != 4) return KIVI_ERR_UNSUPPORTED;
    if (l->group != 32 && l->group != 64 && l->group != 128) return KIVI_ERR_UNSUPPORTED;
    if (l->residual % l->group != 0) return KIVI_ERR_INVALID_ARG;          // Section 3.3: G | R
    if (l->cap_q_tokens % l->group != 0 || l->cap_r_tokens % kTileTokens != 0) return KIVI_ERR_INVALID_ARG;
    if (l->cap_r_tokens < l->residual + l->group) return KIVI_ERR_INVALID_ARG;
    const int rep = l->n_q_heads / l->n_kv_heads;
    if (rep > kMaxRepTotal) return KIVI_ERR_UNSUPPORTED;
    return KIVI_OK;
}

int check_cache(const kivi_layout_t* l, const kivi_cache_t* c) {
    if (!c) return KIVI_ERR_INVALID_ARG;
    const void* ptrs[8] = {c->k_codes, c->k_scale, c->k_zero, c->v_codes,
                           c->v_scale, c->v_zero, c->k_resid, c->v_resid};
    for (const void* p : ptrs)
        if (!p || !aligned16(p)) return KIVI_ERR_INVALID_ARG;
    if (c->n_kq < 0 || c->n_vq < 0 || c->n_kr < 0 || c->n_vr < 0) return KIVI_ERR_INVALID_ARG;
    if (c->n_kq % l->group != 0) return KIVI_ERR_INVALID_ARG;
    if (c->n_kq > l->cap_q_tokens || c->n_vq > l->cap_q_tokens) return KIVI_ERR_INVALID_ARG;
    if (c->n_kr > l->cap_r_tokens || c->n_vr > l->cap_r_tokens) return KIVI_ERR_INVALID_ARG;
    if (c->k_r_start < 0 || c->k_r_start >= l->cap_r_tokens) return KIVI_ERR_INVALID_ARG;
    if (c->v_r_start < 0 || c->v_r_start >= l->cap_r_tokens) return KIVI_ERR_INVALID_ARG;
    return KIVI_OK;
}

int check_source(const void* x, int64_t sb, int64_t sh, int64_t st) {
    if (!x || !aligned16(x)) return KIVI_ERR_INVALID_ARG;
    if (sb < 0 || sh < 0 || st < kHeadDim) return KIVI_ERR_INVALID_ARG;
    if ((sb | sh | st) & 7) return KIVI_ERR_INVALID_ARG;          // keeps every row 16-byte aligned
    return KIVI_OK;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// The workspace starts with four finished-split counters per (batch, kv-head) -- one per quarter of
// the kv-head's query heads, should a launch serve parts of the group as units of their own -- padded
// to 256 bytes.
size_t counter_bytes(const kivi_layout_t* l) {
    // one counter per unit of the work axis: up to 4 parts of a kv-head's query heads (head split), or
    // one per run of 4 heads of a group wider than kMaxRep
    const int groups = std::max(4, ceil_div(l->n_q_heads / std::max(l->n_kv_heads, 1), 4));
    return ((size_t)l->batch * l->n_kv_heads * groups * sizeof(int32_t) + 255) / 256 * 256;
}

// Room for the per-sequence counters of a batch of different lengths (16 bytes per sequence, padded
// to 256 bytes); the ragged entry points keep them behind the split counters.
// Room for the tables of the sliced second launch of a batch of different lengths: 16 bytes per slice
// (at most kMaxSlices) and 8 bytes per (batch, kv-head) unit, behind the per-sequence counters.
constexpr int kMaxSlices = 4096;
constexpr int64_t kMaxSliceUnits = 65536;
size_t slice_table_bytes(const kivi_layout_t* l) {
    const int64_t units = std::min<int64_t>((int64_t)l->batch * l->n_kv_heads, kMaxSliceUnits);
    return ((size_t)kMaxSlices * 16 + (size_t)units * 8 + 255) / 256 * 256;
}

size_t seq_state_bytes(const kivi_layout_t* l) {
    return ((size_t)l->batch * 4 * sizeof(int32_t) + 255) / 256 * 256;
}

// Upper bound of the number of context splits for any cache state of this layout.
// Both planners below give every all-quantised split at least 4 tiles (the matrix-core family 8 or
// 16), and every split with fp16 rows at least one tile; enqueue_attention checks the actual count
// against the workspace before it launches.
int max_splits(const kivi_layout_t* l) {
    const int tiles_q = l->cap_q_tokens / kTileTokens, tiles_r = l->cap_r_tokens / kTileTokens;
    return (tiles_q + 3) / 4 + tiles_r + 2;
}

// `mfma`: plan for the persistent matrix-core kernel (fixed chunk length, resident workgroups known);
// otherwise for the vector-ALU family.
// `two_launches` (matrix-core family only): a single fp16-row split per unit, served by a launch of its own.
SplitPlan plan_splits(const kivi_layout_t* l, const kivi_cache_t* c, bool mfma, bool two_launches = false) {
    SplitPlan s{};
    const int length = c->n_kq + c->n_kr;
    s.tiles_a = std::min(c->n_kq, c->n_vq) / kTileTokens;
    s.tiles_total = ceil_div(length, kTileTokens);
    const int64_t units = (int64_t)l->batch * l->n_kv_heads;
    const int rep = std::min(l->n_q_heads / l->n_kv_heads, kMaxRep);      // heads per launch (wider groups: several launches)
    const int tiles_b = s.tiles_total - s.tiles_a;
    int tps_b_max;
    if (mfma) {
        // The kernel always walks full chunks (shorter ones would only re-read masked tiles).  The
        // natural fp16-row chunk is 4 tiles, one per wavefront; shorter ones when there would be
        // fewer chunks than resident workgroups.
        const MfmaGeometry g = mfma_geometry(l->bits, rep);
        s.tiles_per_split_a = g.chunk_tiles;
        tps_b_max = (int)std::max<int64_t>(1, std::min<int64_t>(4, units * tiles_b / g.resident_workgroups));
        if (two_launches) tps_b_max = std::max(tiles_b, 1);
    } else {
        // Aim at ~16 workgroups per compute unit in flight over the whole grid so the 256 CUs stay
        // busy through the tail, but keep splits long enough that the per-split partial results
        // (520 B per query head) stay a small fraction of the bytes a split streams.
        const int64_t target_wgs = 4096;
        int tps = (int)std::min<int64_t>(kMaxSplitTiles, ((int64_t)s.tiles_a * units + target_wgs - 1) / target_wgs);
        tps = std::max(tps, std::min(kMaxSplitTiles, 4 * rep));
        s.tiles_per_split_a = std::max(1, std::min(tps, kMaxSplitTiles));
        // fp16 rows cost 512 B per token against 96 B (2-bit) or 160 B (4-bit)
        const int packed_per_tile = kTileTokens * 2 * (kHeadDim * l->bits / 8 + 16);
        const int fp16_per_tile = kTileTokens * 2 * kHeadDim * 2;
        tps_b_max = std::max(1, std::min(8, s.tiles_per_split_a * packed_per_tile / fp16_per_tile));
    }
    s.n_splits_b = ceil_div(tiles_b, tps_b_max);
    s.tiles_per_split_b = s.n_splits_b ? ceil_div(tiles_b, s.n_splits_b) : 1;     // even out the pieces
    s.n_splits_a = ceil_div(s.tiles_a, s.tiles_per_split_a);
    return s;
}

int hip_status(hipError_t e) { return e == hipSuccess ? KIVI_OK : KIVI_ERR_HIP; }

QuantKeyParams key_quant_params(const kivi_layout_t* l, const kivi_cache_t* c, const RowSource& src, int n_tokens) {
    QuantKeyParams p{};
    p.src = src;
    p.codes = static_cast<uint32_t*>(c->k_codes);
    p.scale = static_cast<__half*>(c->k_scale);
    p.zero = static_cast<__half*>(c->k_zero);
    p.n_kv_heads = l->n_kv_heads; p.cap_tiles = l->cap_q_tokens / kTileTokens; p.bits = l->bits;
    p.first_tile = c->n_kq / kTileTokens; p.n_tiles = n_tokens / kTileTokens; p.batch = l->batch;
    p.tiles_per_group = l->group / kTileTokens;
    return p;
}

QuantValueParams value_quant_params(const kivi_layout_t* l, const kivi_cache_t* c, const RowSource& src, int n_tokens) {
    QuantValueParams p{};
    p.src = src;
    p.codes = static_cast<uint32_t*>(c->v_codes);
    p.scale = static_cast<__half*>(c->v_scale);
    p.zero = static_cast<__half*>(c->v_zero);
    p.n_kv_heads = l->n_kv_heads; p.cap_tiles = l->cap_q_tokens / kTileTokens; p.bits = l->bits;
    p.first_token = c->n_vq; p.n_tokens = n_tokens; p.batch = l->batch;
    p.group_blocks = l->group / kTileTokens;
    return p;
}

int enqueue_key_quant(const kivi_layout_t* l, const kivi_cache_t* c, const RowSource& src, int n_tokens,
                      hipStream_t hs) {
    return hip_status(launch_quantize_keys(key_quant_params(l, c, src, n_tokens), hs));
}

int enqueue_value_quant(const kivi_layout_t* l, const kivi_cache_t* c, const RowSource& src, int n_tokens,
                        hipStream_t hs) {
    return hip_status(launch_quantize_values(value_quant_params(l, c, src, n_tokens), hs));
}

}  // namespace
}  // namespace kivi

using namespace kivi;

namespace {

// How many of the oldest residual tokens each policy moves into the quantised part (host logic).
int plan_flush(const kivi_layout_t* l, const kivi_cache_t* c, int32_t policy, int* n_key, int* n_value) {
    const int G = l->group, R = l->residual;
    int nk = 0, nv = 0;
    if (policy == KIVI_FLUSH_WINDOW) {
        if (c->n_kr != c->n_vr || c->n_kq != c->n_vq) return KIVI_ERR_INVALID_ARG;   // symmetric policy
        while (c->n_kr - nk >= R + G) nk += G;
        nv = nk;
    } else {
        if (R > 0 && c->n_kr == R) nk = R;                 // Algorithm 1: len(X_Kr) == R
        if (c->n_vr > R) nv = c->n_vr - R;                 // Algorithm 1: len(X_Vr) > R
    }
    if ((int64_t)c->n_kq + nk > l->cap_q_tokens || (int64_t)c->n_vq + nv > l->cap_q_tokens)
        return KIVI_ERR_INVALID_ARG;
    *n_key = nk;
    *n_value = nv;
    return KIVI_OK;
}

// Quantise the oldest nk residual keys and nv residual values out of the rings (one launch; either
// count may be 0) and advance the cache counters (`launch` false: the counters only).
int enqueue_flush(const kivi_layout_t* l, kivi_cache_t* c, int nk, int nv, hipStream_t hs, bool launch = true) {
    const int64_t sh = (int64_t)l->cap_r_tokens * kHeadDim, sb = sh * l->n_kv_heads;
    if (launch && (nk > 0 || nv > 0)) {
        const RowSource ksrc{static_cast<const __half*>(c->k_resid), sb, sh, kHeadDim, c->k_r_start, l->cap_r_tokens};
        const RowSource vsrc{static_cast<const __half*>(c->v_resid), sb, sh, kHeadDim, c->v_r_start, l->cap_r_tokens};
        if (int s = hip_status(launch_flush_quantize(key_quant_params(l, c, ksrc, nk), value_quant_params(l, c, vsrc, nv), hs)))
            return s;
    }
    c->n_kq += nk; c->n_kr -= nk; c->k_r_start = (c->k_r_start + nk) % l->cap_r_tokens;
    c->n_vq += nv; c->n_vr -= nv; c->v_r_start = (c->v_r_start + nv) % l->cap_r_tokens;
    return KIVI_OK;
}

// Host checks shared by the attention entry points (the cache counts are those the kernel will see).
// any_state: the workspace must hold the parts of any cache state of the layout (the documented
// size); otherwise only a pointer check -- enqueue_attention checks the state's own need.
int check_attention_args(const kivi_layout_t* l, const kivi_cache_t* c, const void* q, const float* out,
                         const void* workspace, size_t workspace_bytes, bool any_state = true) {
    if (!q || !out || !aligned16(q) || !aligned16(out)) return KIVI_ERR_INVALID_ARG;
    const int length = c->n_kq + c->n_kr;
    if (length < 1 || length != c->n_vq + c->n_vr) return KIVI_ERR_INVALID_ARG;
    size_t need = 0;
    if (any_state) kivi_decode_workspace_bytes(l, &need);
    if (!workspace || !aligned16(workspace) || workspace_bytes < need) return KIVI_ERR_WORKSPACE;
    return KIVI_OK;
}

int decode_family(const kivi_layout_t* l) {
    // the matrix-core family unless the caller asks for the vector ALUs or it has no instantiation
    // for this (bits, query heads per kv-head)
    const int rep = std::min(l->n_q_heads / l->n_kv_heads, kMaxRep);
    if (l->decode_path == KIVI_DECODE_VALU) return KIVI_DECODE_VALU;
    return mfma_geometry(l->bits, rep).chunk_tiles == 0 ? KIVI_DECODE_VALU : KIVI_DECODE_MFMA;
}

// The matrix-core family as two launches (fp16 rows first, then the all-quantised chunks): possible
// when the cache has both parts and K and V are split at the same token; chosen when asked for, or
// by three measured rules.
//  (1) A workgroup of the persistent kernel would own several (batch, kv-head) units: their fp16-row
//      chunks would run one after the other, each a chain of dependent steps (32 heads, context 4096,
//      2 bits: equal at 1 unit per workgroup, 4-6 % faster from 1.5 on).
//  (2) Between half a unit and one unit per workgroup most workgroups straddle two units and run two
//      such chains: two launches are 2-12 % faster once the launch is long enough to carry the
//      second launch's fixed 8-12 us.
//  (3) Fewer units still, but 3 or more query heads per kv-head and at least two tiles of fp16 rows:
//      the rows kernel runs every tile of every unit at once where the persistent kernel gives each
//      fp16-row chunk to one workgroup (and its 4-bit instantiation for 5 to 8 heads spills
//      registers in the single-launch form only).  Two launches pay from a total amount of work
//      (units x tiles) and of fp16-row work (units x fp16 tiles) on.
// The thresholds are fitted to sweeps of both forms over 8-4096 units, contexts 1k-16k, windows
// 32-192, 1-8 heads per kv-head, 2 and 4 bits (730 shapes): against the better form of each shape
// these rules lose 0.1-1.2 % on average per instantiation, a single launch everywhere 1.3-7.6 %.
bool wants_two_launches(const kivi_layout_t* l, const kivi_cache_t* c, int path) {
    if (path != KIVI_DECODE_MFMA || l->decode_path == KIVI_DECODE_MFMA_ONE) return false;
    const int rep_launch = std::min(l->n_q_heads / l->n_kv_heads, kMaxRep);
    const int rep_variant = rep_launch <= 2 ? rep_launch : (rep_launch <= 4 ? 4 : 8);
    const int tiles_total = ceil_div(c->n_kq + c->n_kr, kTileTokens);
    const int tiles_b = tiles_total - c->n_kq / kTileTokens;
    const bool possible = c->n_kq == c->n_vq && c->n_kq >= kTileTokens && c->n_kr > 0 &&
                          residual_rows_possible(tiles_b, rep_variant);
    if (!possible) return false;
    if (l->decode_path == KIVI_DECODE_MFMA_TWO) return true;
    const int64_t units = (int64_t)l->batch * l->n_kv_heads;
    const int resident = mfma_geometry(l->bits, rep_launch).resident_workgroups;
    const int64_t work = units * tiles_total, row_work = units * tiles_b;
    if (units * 4 >= (int64_t)resident * 5) return true;                                             // (1)
    if (units * 2 > resident && units < resident && tiles_b >= 2 && work >= 24000) return true;      // (2)
    if (rep_variant < 4) return false;
    int64_t min_work, min_row_work;                                                                  // (3)
    int min_tiles_b = 2;
    if (rep_variant == 8) { min_work = 4000; min_row_work = 384; }
    else { min_work = l->bits == 4 ? 10000 : 16000; min_row_work = 512; min_tiles_b = 3; }
    return tiles_b >= min_tiles_b && work >= min_work && row_work >= min_row_work;
}

// With 4, 6 or 8 query heads per kv-head and few chunks per workgroup the single launch lasts about
// as long as its chunks, and a chunk takes longer the more heads it serves (8 kv-heads, context 4096,
// batch 1, one chunk per workgroup: 9.8 / 15.2 / 30.0 us with 1 / 4 / 8 heads per kv-head).  Then
// equal parts of every group run as units of their own on the instantiation for a part's heads:
// more workgroups, each shorter; the cache is read once per part, which such launches do not notice.
// Measured (8 kv-heads, batch 1-32, contexts 1k-32k) for limits from 1/2 to 16 chunks per resident
// workgroup.  Halves of 6 or 8 heads: faster wherever applied up to 4 chunks per workgroup at 2 bits
// (30.5 -> 18.3 us at batch 1 / context 4096, 69.6 -> 46.8 us at batch 2 / 32k; mixed beyond) and up to
// 16 at 4 bits, whose 8-head instantiation spills registers (29.5 -> 18.9, 98.5 -> 81.9 us).  Halves of
// 4 heads at 2 bits: 17.0 -> 13.8 us at batch 1 / 4096, 37.1 -> 24.6 us at batch 1 / 32k; from 128 units
// on 4 % slower.  Quarters of 8 heads at 2 bits, against halves: 18.3 -> 14.5 us at batch 1 / 4096,
// 29.7 -> 22.4 us at batch 1 / 16k, 20.4 -> 18.0 us at batch 2 / 4096; even or slower from 32 units on.
// log2 of the parts a kv-head's query heads are served in: 0 (whole group), 1 (halves), 2 (quarters)
int head_split_shift(const kivi_layout_t* l, const SplitPlan& plan, int path, bool two_launches) {
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    if (path != KIVI_DECODE_MFMA || two_launches || (rep_total != 4 && rep_total != 6 && rep_total != 8)) return 0;
    if (l->group != kTileTokens) return 0;            // G > 32 runs on instantiations of its own, which exist for whole groups only
    const int64_t units = (int64_t)l->batch * l->n_kv_heads, chunks = units * plan.n_splits();
    // parts of 2 heads run on the 2-head instantiation: 2 bits only (at 4 bits that instantiation's
    // chunks are not the length the plan was made for)
    const MfmaGeometry g2 = mfma_geometry(l->bits, 2);
    const bool two_heads_possible = g2.chunk_tiles == plan.tiles_per_split_a;
    if (rep_total == 8 && two_heads_possible && units <= 16 && chunks <= (int64_t)g2.resident_workgroups * 2) return 2;     // quarters
    if (rep_total == 4)     // 2 + 2: up to 64 units and 4 chunks per workgroup
        return two_heads_possible && units <= 64 && chunks <= (int64_t)g2.resident_workgroups * 4 ? 1 : 0;
    const int max_chunks_per_workgroup = l->bits == 4 ? 16 : 4;
    return chunks <= (int64_t)mfma_geometry(l->bits, 4).resident_workgroups * max_chunks_per_workgroup ? 1 : 0;
}

// Runs of kWideGroupRun query heads a kv-head's group is served in by ONE launch of the matrix-core
// family's single-launch form (1: the group fits one run, or the form is not the single launch:
// then a wider group takes one launch, or pair of launches, per run).
// Query heads per run when a wider group is served as units of one launch: 4 (measured against 8 on
// 71 : 1, 128 : 8 and 32 : 2 head shapes at 2 and 4 bits: 13-20 % faster everywhere -- the four-head
// instantiation's fp16-row phase and chunks are shorter and there are twice the units to spread).
constexpr int kWideGroupRun = 4;
int wide_group_width(const kivi_layout_t*) { return kWideGroupRun; }
int wide_group_runs(const kivi_layout_t* l, int path, bool two_launches) {
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    if (path != KIVI_DECODE_MFMA || two_launches || rep_total <= kMaxRep || l->group != kTileTokens) return 1;
    return ceil_div(rep_total, wide_group_width(l));
}

// Launch the attention of q over cache state `c` (already validated).  k_new / v_new non-null: the
// rows of token length-1 are not in the rings yet and the (matrix-core) kernel puts them there.
// flush_k / flush_v non-null (two-launch form only): the residual flush that produced state `c` has
// not been launched yet; the fp16-row launch carries it out with extra workgroups.
int enqueue_attention(const kivi_layout_t* l, const kivi_cache_t* c, const void* q, float softmax_scale,
                      float* out, void* workspace, size_t workspace_bytes, const void* k_new, const void* v_new,
                      void* stream, const QuantKeyParams* flush_k = nullptr, const QuantValueParams* flush_v = nullptr) {
    const int length = c->n_kq + c->n_kr;
    DecodeParams p{};
    p.k_codes = static_cast<const uint32_t*>(c->k_codes);
    p.k_scale = static_cast<const __half*>(c->k_scale);
    p.k_zero = static_cast<const __half*>(c->k_zero);
    p.v_codes = static_cast<const uint32_t*>(c->v_codes);
    p.v_scale = static_cast<const __half*>(c->v_scale);
    p.v_zero = static_cast<const __half*>(c->v_zero);
    p.k_resid = static_cast<const __half*>(c->k_resid);
    p.v_resid = static_cast<const __half*>(c->v_resid);
    p.n_kq = c->n_kq; p.n_vq = c->n_vq; p.k_r_start = c->k_r_start; p.n_kr = c->n_kr;
    p.v_r_start = c->v_r_start; p.n_vr = c->n_vr;
    p.cap_tiles = l->cap_q_tokens / kTileTokens; p.cap_r = l->cap_r_tokens;
    p.q = static_cast<const __half*>(q); p.out = out;
    p.softmax_scale = softmax_scale;
    p.batch = l->batch; p.n_q_heads = l->n_q_heads; p.n_kv_heads = l->n_kv_heads; p.bits = l->bits;
    p.kg_shift = l->group == 32 ? 0 : (l->group == 64 ? 1 : 2);
    p.length = length;
    const int path = decode_family(l);
    if ((k_new || v_new) && path != KIVI_DECODE_MFMA) return KIVI_ERR_UNSUPPORTED;
    p.k_new = static_cast<const __half*>(k_new); p.v_new = static_cast<const __half*>(v_new);
    const bool two = wants_two_launches(l, c, path);
    p.plan = plan_splits(l, c, path == KIVI_DECODE_MFMA, two);
    p.two_launches = two ? 1 : 0;
    p.head_groups = wide_group_runs(l, path, two);
    if ((flush_k || flush_v) && !(two && flush_k && flush_v)) return KIVI_ERR_INVALID_ARG;
    p.flush_k = flush_k;
    p.flush_v = flush_v;
    const size_t rows = (size_t)l->batch * l->n_q_heads * p.plan.n_splits();
    if (counter_bytes(l) + rows * (kHeadDim + 2) * sizeof(float) > workspace_bytes) return KIVI_ERR_WORKSPACE;
    p.counters = static_cast<int32_t*>(workspace);
    p.part_o = reinterpret_cast<float*>(static_cast<char*>(workspace) + counter_bytes(l));
    p.part_ml = p.part_o + rows * kHeadDim;

    hipStream_t hs = static_cast<hipStream_t>(stream);
    // Up to kMaxRep query heads per kv-head go through one launch.  A wider group (multi-query
    // attention: 71 heads on one kv-head) takes one launch per kMaxRep heads, each reading the cache
    // again; the launches share the plan and the workspace (their part rows are disjoint, and the
    // matrix-core kernel leaves its counters at zero).  Only the first one appends the new token.
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    p.rep_variant = std::min(rep_total, kMaxRep);
    if (p.head_groups > 1) {
        // a group wider than kMaxRep heads in the single-launch form: its runs of kWideGroupRun heads are
        // units of ONE launch (they read the same cache, which the caches serve after the first)
        p.q_head0 = 0;
        p.rep_here = wide_group_width(l);
        p.rep_variant = p.rep_here;
        return hip_status(launch_decode_mfma(p, hs));
    }
    if (const int shift = head_split_shift(l, p.plan, path, two)) {
        p.head_split = shift;
        p.q_head0 = 0;
        p.rep_here = rep_total >> shift;
        p.rep_variant = p.rep_here <= 2 ? 2 : 4;
        return hip_status(launch_decode_mfma(p, hs));
    }
    for (int h0 = 0; h0 < rep_total; h0 += kMaxRep) {
        p.q_head0 = h0;
        p.rep_here = std::min(kMaxRep, rep_total - h0);
        hipError_t e = path == KIVI_DECODE_MFMA ? launch_decode_mfma(p, hs) : launch_decode_valu(p, hs);
        if (e == hipErrorNotSupported) return KIVI_ERR_UNSUPPORTED;
        if (int s = hip_status(e)) return s;
        p.k_new = p.v_new = nullptr;
        p.flush_k = nullptr;
        p.flush_v = nullptr;
    }
    // the matrix-core kernel merges its splits itself; the vector-ALU family uses a second launch
    return path == KIVI_DECODE_MFMA ? KIVI_OK : hip_status(launch_merge(p, hs));
}

}  // namespace

namespace {

inline bool same_state(const kivi_seq_state_t& a, const kivi_seq_state_t& b) {
    return a.n_kq == b.n_kq && a.n_vq == b.n_vq && a.k_r_start == b.k_r_start && a.n_kr == b.n_kr &&
           a.v_r_start == b.v_r_start && a.n_vr == b.n_vr;
}

// Walk the batch in runs of equal state; `call(sub_layout, sub_cache, b0)` handles one run and may
// change the sub-cache's integer fields, which are then written back to the run's states.
template <class F>
int for_each_run(const kivi_layout_t* l, const kivi_cache_t* c, kivi_seq_state_t* states, bool write_back, F&& call) {
    if (int s = check_layout(l)) return s;
    if (!c || !states) return KIVI_ERR_INVALID_ARG;
    for (int b0 = 0; b0 < l->batch;) {
        int b1 = b0 + 1;
        while (b1 < l->batch && same_state(states[b0], states[b1])) ++b1;
        kivi_layout_t sl;
        kivi_cache_t sc;
        if (int s = kivi_batch_slice(l, c, b0, b1 - b0, &states[b0], &sl, &sc)) return s;
        if (int s = call(sl, sc, b0)) return s;
        if (write_back)
            for (int b = b0; b < b1; ++b)
                states[b] = kivi_seq_state_t{sc.n_kq, sc.n_vq, sc.k_r_start, sc.n_kr, sc.v_r_start, sc.n_vr};
        b0 = b1;
    }
    return KIVI_OK;
}

}  // namespace

// ---- batches of different lengths in one pair of launches ----
namespace {

constexpr int kNotApplicable = 1;       // (internal) the fast path does not serve this batch: use the run-by-run path

// Attention over a batch whose sequences differ in length as ONE pair of launches of the matrix-core
// family's two-launch form: the fp16 rows of every unit (which also append the new token when
// k_new / v_new are given), then the all-quantised chunks.  Both kernels read each sequence's
// counters from a device array; the split plan is the longest sequence's, a shorter one's surplus
// chunks and tiles are masked.  Served: K and V split alike in every sequence, at least one fp16
// row and at most 16 tiles of them per sequence, at least one quantised tile somewhere in the
// batch.  `st`: the states the attention sees (after append and flush).  Returns kNotApplicable
// (nothing launched) for any other batch.
int ragged_attention_fast(const kivi_layout_t* l, const kivi_cache_t* c, const kivi_seq_state_t* st, const void* q,
                          float softmax_scale, float* out, void* workspace, size_t workspace_bytes,
                          const void* k_new, const void* v_new, void* stream) {
    if (decode_family(l) != KIVI_DECODE_MFMA || l->decode_path == KIVI_DECODE_MFMA_ONE) return kNotApplicable;
    if (l->cap_q_tokens < kTileTokens || l->group != kTileTokens) return kNotApplicable;
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    const int rep_launch = std::min(rep_total, kMaxRep);
    const int rep_variant = rep_launch <= 2 ? rep_launch : (rep_launch <= 4 ? 4 : 8);
    int max_tiles_a = 0, max_tiles_b = 0, min_tiles_a = INT32_MAX;
    for (int b = 0; b < l->batch; ++b) {
        const kivi_seq_state_t& x = st[b];
        if (x.n_kq != x.n_vq || x.n_kr != x.n_vr || x.n_kr < 1 || x.n_kq % kTileTokens != 0) return kNotApplicable;
        const int tiles_a = x.n_kq / kTileTokens;
        max_tiles_a = std::max(max_tiles_a, tiles_a);
        min_tiles_a = std::min(min_tiles_a, tiles_a);
        max_tiles_b = std::max(max_tiles_b, ceil_div(x.n_kq + x.n_kr, kTileTokens) - tiles_a);
    }
    if (max_tiles_a < 1 || !residual_rows_possible(max_tiles_b, rep_variant)) return kNotApplicable;
    const MfmaGeometry g = mfma_geometry(l->bits, rep_launch);
    if (g.chunk_tiles == 0) return kNotApplicable;

    DecodeParams p{};
    p.k_codes = static_cast<const uint32_t*>(c->k_codes);
    p.k_scale = static_cast<const __half*>(c->k_scale);
    p.k_zero = static_cast<const __half*>(c->k_zero);
    p.v_codes = static_cast<const uint32_t*>(c->v_codes);
    p.v_scale = static_cast<const __half*>(c->v_scale);
    p.v_zero = static_cast<const __half*>(c->v_zero);
    p.k_resid = static_cast<const __half*>(c->k_resid);
    p.v_resid = static_cast<const __half*>(c->v_resid);
    p.k_new = static_cast<const __half*>(k_new); p.v_new = static_cast<const __half*>(v_new);
    // the scalar counters describe the longest sequence (the kernels take each sequence's own from seq_state)
    p.n_kq = p.n_vq = max_tiles_a * kTileTokens;
    p.n_kr = p.n_vr = max_tiles_b * kTileTokens;
    p.length = p.n_kq + p.n_kr;
    p.cap_tiles = l->cap_q_tokens / kTileTokens; p.cap_r = l->cap_r_tokens;
    p.q = static_cast<const __half*>(q); p.out = out;
    p.softmax_scale = softmax_scale;
    p.batch = l->batch; p.n_q_heads = l->n_q_heads; p.n_kv_heads = l->n_kv_heads; p.bits = l->bits;
    p.kg_shift = l->group == 32 ? 0 : (l->group == 64 ? 1 : 2);
    p.plan.tiles_a = max_tiles_a;
    p.plan.tiles_total = max_tiles_a + max_tiles_b;
    p.plan.tiles_per_split_a = g.chunk_tiles;
    p.plan.tiles_per_split_b = max_tiles_b;
    p.plan.n_splits_a = ceil_div(max_tiles_a, g.chunk_tiles);
    p.plan.n_splits_b = 1;
    p.two_launches = 1;
    char* ws = static_cast<char*>(workspace);
    const size_t parts_offset = counter_bytes(l) + seq_state_bytes(l) + slice_table_bytes(l);
    hipStream_t hs = static_cast<hipStream_t>(stream);

    // Fewer units than the chip holds wavefronts, every sequence with quantised tokens, at most 4 heads
    // per launch: the second launch runs as equally long slices of the unit-major axis of four-tile
    // groups, one per wavefront, so that no wavefront idles through a shorter sequence's share (with
    // more units than wavefronts every wavefront takes whole units instead, which balances by itself).
    const int64_t units = (int64_t)l->batch * l->n_kv_heads;
    const int slice_waves = (min_tiles_a >= 1 && rep_total <= 4) ? wave_slices_resident(l->bits, rep_launch) : 0;
    // Everything the kernels read per call goes to the device in ONE copy (a copy is an operation of its
    // own on the stream): the sequences' counters, then -- if used -- the slice table and the unit table.
    // (An asynchronous copy out of pageable memory has taken its source when the call returns.)
    static thread_local std::vector<int32_t> tables;
    const size_t state_ints = seq_state_bytes(l) / sizeof(int32_t);
    tables.assign(state_ints, 0);
    for (int b = 0; b < l->batch; ++b) {
        const kivi_seq_state_t& x = st[b];
        tables[4 * (size_t)b + 0] = x.n_kq; tables[4 * (size_t)b + 1] = x.n_kr;
        tables[4 * (size_t)b + 2] = x.k_r_start; tables[4 * (size_t)b + 3] = x.v_r_start;
    }
    int32_t* dev_state = reinterpret_cast<int32_t*>(ws + counter_bytes(l));
    int64_t total = 0;                                      // groups of four tiles over all units
    for (int b = 0; b < l->batch; ++b) total += (int64_t)ceil_div(st[b].n_kq / kTileTokens, 4) * l->n_kv_heads;
    // The slices cost a fixed ~18 us more than the padded plan (short slices, parts through memory for
    // every shared unit) and save the group steps the padded plan wastes on shorter sequences, ~3.7 us per
    // 2048 of them: they pay from about 14 000 wasted group steps on (sweep of 128-1600 units, 1, 2 and 4
    // heads per kv-head, length spreads from +-12 % to 1 : 80: 0.70-0.96 of the padded plan's time above the
    // threshold, 1.05-1.7 below it).
    const int64_t wasted = units * ceil_div(max_tiles_a, 4) - total;
    if (slice_waves > 0 && units < slice_waves && units <= kMaxSliceUnits && wasted >= 14000) {
        const int n_slices = (int)std::min<int64_t>(std::min(slice_waves, kMaxSlices), total);
        tables.resize(state_ints + (size_t)n_slices * 4 + (size_t)units * 2, 0);
        int32_t* desc = tables.data() + state_ints;
        int32_t* parts = desc + (size_t)n_slices * 4;
        // slice s covers the groups [s * total / n_slices, (s + 1) * total / n_slices) of the unit-major axis
        auto groups_of = [&](int64_t u) { return (int64_t)ceil_div(st[u / l->n_kv_heads].n_kq / kTileTokens, 4); };
        {
            int64_t u = 0, g_before = 0;                    // groups of the units before u
            for (int si = 0; si < n_slices; ++si) {
                const int64_t begin = (int64_t)si * total / n_slices, end = (int64_t)(si + 1) * total / n_slices;
                while (g_before + groups_of(u) <= begin) g_before += groups_of(u++);
                desc[4 * (size_t)si + 0] = (int32_t)u;
                desc[4 * (size_t)si + 1] = (int32_t)(begin - g_before);
                desc[4 * (size_t)si + 2] = (int32_t)(end - begin);
                desc[4 * (size_t)si + 3] = 0;
            }
        }
        // slices touching a unit: from the one that holds its first group to the one that holds its last
        // (group x lies in slice ((x + 1) * n_slices - 1) / total)
        int max_parts = 1;
        {
            int64_t g_before = 0;
            for (int64_t u = 0; u < units; ++u) {
                const int64_t groups = groups_of(u);
                const int first = (int)(((g_before + 1) * n_slices - 1) / total);
                const int last = (int)(((g_before + groups) * n_slices - 1) / total);
                parts[2 * (size_t)u + 0] = first;
                parts[2 * (size_t)u + 1] = last - first + 1;
                max_parts = std::max(max_parts, last - first + 1);
                g_before += groups;
            }
        }
        const size_t rows_s = (size_t)l->batch * l->n_q_heads * (max_parts + 1);
        if (parts_offset + rows_s * (kHeadDim + 2) * sizeof(float) <= workspace_bytes) {
            p.wave_desc = dev_state + state_ints;
            p.unit_parts = p.wave_desc + (size_t)n_slices * 4;
            p.n_slices = n_slices;
            p.plan.n_splits_a = max_parts;              // workspace rows per (batch, query head): the fp16-row part + one per slice
        } else {
            tables.resize(state_ints);
        }
    }
    const size_t rows = (size_t)l->batch * l->n_q_heads * p.plan.n_splits();
    if (parts_offset + rows * (kHeadDim + 2) * sizeof(float) > workspace_bytes) return KIVI_ERR_WORKSPACE;
    p.counters = reinterpret_cast<int32_t*>(ws);
    p.seq_state = dev_state;
    p.ragged_min_tiles = min_tiles_a;
    p.part_o = reinterpret_cast<float*>(ws + parts_offset);
    p.part_ml = p.part_o + rows * kHeadDim;
    if (hipMemcpyAsync(dev_state, tables.data(), (p.wave_desc ? tables.size() : (size_t)l->batch * 4) * sizeof(int32_t),
                       hipMemcpyHostToDevice, hs) != hipSuccess)
        return KIVI_ERR_HIP;
    p.rep_variant = rep_launch;
    for (int h0 = 0; h0 < rep_total; h0 += kMaxRep) {
        p.q_head0 = h0;
        p.rep_here = std::min(kMaxRep, rep_total - h0);
        const hipError_t e = launch_decode_mfma(p, hs);
        if (e == hipErrorNotSupported) return KIVI_ERR_UNSUPPORTED;
        if (int s2 = hip_status(e)) return s2;
        p.k_new = p.v_new = nullptr;
    }
    return KIVI_OK;
}

// One decoding step of every sequence of a batch of different lengths in one pair of attention
// launches (plus one flush launch per run of equal sequences that flush in this step, which is rare:
// a sequence flushes every G-th step).  Served when every sequence's flush leaves the new token in
// the window (then the flush can run out of the rings before the attention appends the token) and
// the states after the step suit ragged_attention_fast.  Returns kNotApplicable with nothing launched
// and nothing changed otherwise.
int ragged_step_fast(const kivi_layout_t* l, const kivi_cache_t* c, kivi_seq_state_t* states, const void* k_new,
                     const void* v_new, const void* q, float softmax_scale, int32_t policy, float* out,
                     void* workspace, size_t workspace_bytes, void* stream) {
    if (check_layout(l) != KIVI_OK || !c || !states) return kNotApplicable;        // the run-by-run path reports the error
    if (policy != KIVI_FLUSH_WINDOW && policy != KIVI_FLUSH_ALG1) return kNotApplicable;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(q) || !aligned16(out) || !workspace || !aligned16(workspace))
        return kNotApplicable;
    if (decode_family(l) != KIVI_DECODE_MFMA || l->batch > 4096) return kNotApplicable;
    // pass 1 (host only): every sequence's flush and its state after the step
    kivi_seq_state_t after[4096];
    int16_t nks[4096], nvs[4096];
    for (int b = 0; b < l->batch; ++b) {
        kivi_layout_t sl; kivi_cache_t sc;
        if (kivi_batch_slice(l, c, b, 1, &states[b], &sl, &sc) != KIVI_OK) return kNotApplicable;
        if (sc.n_kr >= l->cap_r_tokens || sc.n_vr >= l->cap_r_tokens) return kNotApplicable;
        kivi_cache_t ap = sc;
        ap.n_kr += 1; ap.n_vr += 1;
        int nk = 0, nv = 0;
        if (plan_flush(&sl, &ap, policy, &nk, &nv) != KIVI_OK) return kNotApplicable;
        if (nk > sc.n_kr || nv > sc.n_vr || nk > 32767 || nv > 32767) return kNotApplicable;
        nks[b] = (int16_t)nk; nvs[b] = (int16_t)nv;
        after[b] = kivi_seq_state_t{sc.n_kq + nk, sc.n_vq + nv, (sc.k_r_start + nk) % l->cap_r_tokens, sc.n_kr - nk + 1,
                                    (sc.v_r_start + nv) % l->cap_r_tokens, sc.n_vr - nv + 1};
    }
    // dry run of the attention's own conditions (no launch): the same checks it will make
    {
        const int rep_launch = std::min(l->n_q_heads / l->n_kv_heads, kMaxRep);
        const int rep_variant = rep_launch <= 2 ? rep_launch : (rep_launch <= 4 ? 4 : 8);
        if (l->decode_path == KIVI_DECODE_MFMA_ONE || l->cap_q_tokens < kTileTokens || l->group != kTileTokens) return kNotApplicable;
        int max_tiles_a = 0, max_tiles_b = 0;
        for (int b = 0; b < l->batch; ++b) {
            const kivi_seq_state_t& x = after[b];
            if (x.n_kq != x.n_vq || x.n_kr != x.n_vr || x.n_kr < 1 || x.n_kq % kTileTokens != 0) return kNotApplicable;
            max_tiles_a = std::max(max_tiles_a, x.n_kq / kTileTokens);
            max_tiles_b = std::max(max_tiles_b, ceil_div(x.n_kq + x.n_kr, kTileTokens) - x.n_kq / kTileTokens);
        }
        if (max_tiles_a < 1 || !residual_rows_possible(max_tiles_b, rep_variant)) return kNotApplicable;
        const size_t rows = (size_t)l->batch * l->n_q_heads * (ceil_div(max_tiles_a, mfma_geometry(l->bits, rep_launch).chunk_tiles) + 1);
        if (counter_bytes(l) + seq_state_bytes(l) + slice_table_bytes(l) + rows * (kHeadDim + 2) * sizeof(float) > workspace_bytes) return KIVI_ERR_WORKSPACE;
    }
    // pass 2: the flushes, one launch per run of consecutive sequences with equal state that flush
    hipStream_t hs = static_cast<hipStream_t>(stream);
    for (int b0 = 0; b0 < l->batch;) {
        int b1 = b0 + 1;
        while (b1 < l->batch && same_state(states[b0], states[b1])) ++b1;
        if (nks[b0] > 0 || nvs[b0] > 0) {
            kivi_layout_t sl; kivi_cache_t sc;
            if (int s = kivi_batch_slice(l, c, b0, b1 - b0, &states[b0], &sl, &sc)) return s;
            if (int s = enqueue_flush(&sl, &sc, nks[b0], nvs[b0], hs)) return s;
        }
        b0 = b1;
    }
    if (int s = ragged_attention_fast(l, c, after, q, softmax_scale, out, workspace, workspace_bytes, k_new, v_new, stream))
        return s == kNotApplicable ? KIVI_ERR_UNSUPPORTED : s;       // cannot happen after the dry run
    for (int b = 0; b < l->batch; ++b) states[b] = after[b];
    return KIVI_OK;
}

}  // namespace

// ---- kivi_decode_attention_static: the attention workspace as an array inside the library ----
// For callers that cannot allocate.  Every device the library runs on holds its own copy of the
// array at its own address; in host code the array's name is only a handle for
// hipGetSymbolAddress, the kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[KIVI_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxScratchDevices = 64;
std::atomic<void*> scratch_ptr[kMaxScratchDevices];

// Address of `scratch` on the current device: resolved once per device (with that device
// current), kept afterwards.
int static_scratch_address(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return KIVI_ERR_HIP;
    if (dev < 0 || dev >= kMaxScratchDevices) return KIVI_ERR_UNSUPPORTED;
    void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KIVI_ERR_HIP;
        scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return KIVI_OK;
}

__global__ void zero_words_kernel(uint32_t* dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0u;
}

}  // namespace

extern "C" {

const char* kivi_status_string(int status) {
    switch (status) {
        case KIVI_OK: return "KIVI_OK";
        case KIVI_ERR_INVALID_ARG: return "KIVI_ERR_INVALID_ARG";
        case KIVI_ERR_UNSUPPORTED: return "KIVI_ERR_UNSUPPORTED";
        case KIVI_ERR_WORKSPACE: return "KIVI_ERR_WORKSPACE";
        case KIVI_ERR_HIP: return "KIVI_ERR_HIP";
        default: return "KIVI_ERR_UNKNOWN";
    }
}

int kivi_cache_sizes(const kivi_layout_t* l, kivi_cache_sizes_t* out) {
    if (int st = check_layout(l)) return st;
    if (!out) return KIVI_ERR_INVALID_ARG;
    const size_t units = (size_t)l->batch * l->n_kv_heads;
    const size_t tiles = (size_t)l->cap_q_tokens / kTileTokens;
    const size_t words = (size_t)kTileTokens * kHeadDim * l->bits / 32;
    out->k_codes = out->v_codes = units * tiles * words * 4;
    // one scale / zero-point per group: keys per (G tokens, channel), values per (token, G channels)
    out->k_scale = out->k_zero = units * ((size_t)l->cap_q_tokens / l->group) * kHeadDim * 2;
    out->v_scale = out->v_zero = units * (size_t)l->cap_q_tokens * (kHeadDim / l->group) * 2;
    out->k_resid = out->v_resid = units * (size_t)l->cap_r_tokens * kHeadDim * 2;
    return KIVI_OK;
}

int kivi_decode_plan(const kivi_layout_t* l, const kivi_cache_t* c, kivi_decode_plan_t* out) {
    if (int st = check_layout(l)) return st;
    if (int st = check_cache(l, c)) return st;
    if (!out) return KIVI_ERR_INVALID_ARG;
    const int path = decode_family(l);
    const bool two = wants_two_launches(l, c, path);
    const SplitPlan plan = plan_splits(l, c, path == KIVI_DECODE_MFMA, two);
    out->family = path;
    // launches: a group wider than kMaxRep heads takes one pass per run of kMaxRep heads, except in the
    // matrix-core family's single-launch form, where the runs are units of one launch
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    const int runs = wide_group_runs(l, path, two);
    const int passes = runs > 1 ? 1 : ceil_div(rep_total, kMaxRep);
    out->launches = path == KIVI_DECODE_MFMA ? (two ? 2 : 1) * passes : passes + 1;      // vector-ALU family: decodes + merge
    out->units_per_kv_head = runs > 1 ? runs : 1 << head_split_shift(l, plan, path, two);
    out->splits_quantised = plan.n_splits_a;
    out->splits_fp16 = plan.n_splits_b;
    out->tiles_per_split_quantised = plan.tiles_per_split_a;
    out->tiles_per_split_fp16 = plan.tiles_per_split_b;
    return KIVI_OK;
}

int kivi_decode_workspace_bytes(const kivi_layout_t* l, size_t* bytes) {
    if (int st = check_layout(l)) return st;
    if (!bytes) return KIVI_ERR_INVALID_ARG;
    const size_t rows = (size_t)l->batch * l->n_q_heads * max_splits(l);
    *bytes = counter_bytes(l) + seq_state_bytes(l) + slice_table_bytes(l) + rows * (kHeadDim + 2) * sizeof(float);
    return KIVI_OK;
}

int kivi_quantize_key_groups(const kivi_layout_t* l, const void* k, int64_t sb, int64_t sh, int64_t st,
                             int32_t n_tokens, kivi_cache_t* c, void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (int s = check_source(k, sb, sh, st)) return s;
    if (n_tokens < 0 || n_tokens % l->group != 0) return KIVI_ERR_INVALID_ARG;
    if ((int64_t)c->n_kq + n_tokens > l->cap_q_tokens) return KIVI_ERR_INVALID_ARG;
    if (n_tokens == 0) return KIVI_OK;
    const RowSource src{static_cast<const __half*>(k), sb, sh, st, 0, 0};
    if (int s = enqueue_key_quant(l, c, src, n_tokens, static_cast<hipStream_t>(stream))) return s;
    c->n_kq += n_tokens;
    return KIVI_OK;
}

int kivi_quantize_value_tokens(const kivi_layout_t* l, const void* v, int64_t sb, int64_t sh, int64_t st,
                               int32_t n_tokens, kivi_cache_t* c, void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (int s = check_source(v, sb, sh, st)) return s;
    if (n_tokens < 0) return KIVI_ERR_INVALID_ARG;
    if ((int64_t)c->n_vq + n_tokens > l->cap_q_tokens) return KIVI_ERR_INVALID_ARG;
    if (n_tokens == 0) return KIVI_OK;
    const RowSource src{static_cast<const __half*>(v), sb, sh, st, 0, 0};
    if (int s = enqueue_value_quant(l, c, src, n_tokens, static_cast<hipStream_t>(stream))) return s;
    c->n_vq += n_tokens;
    return KIVI_OK;
}

int kivi_append_residual(const kivi_layout_t* l, kivi_cache_t* c, const void* k_new, const void* v_new,
                         void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return KIVI_ERR_INVALID_ARG;
    if (c->n_kr >= l->cap_r_tokens || c->n_vr >= l->cap_r_tokens) return KIVI_ERR_INVALID_ARG;
    const int64_t sh = kHeadDim, sb = sh * l->n_kv_heads;
    CopyRowsParams p{};
    p.cap_r = l->cap_r_tokens; p.n_kv_heads = l->n_kv_heads; p.batch = l->batch;
    p.job[0] = {static_cast<const __half*>(k_new), sb, sh, kHeadDim, 0, static_cast<__half*>(c->k_resid),
                (c->k_r_start + c->n_kr) % l->cap_r_tokens, 1};
    p.job[1] = {static_cast<const __half*>(v_new), sb, sh, kHeadDim, 0, static_cast<__half*>(c->v_resid),
                (c->v_r_start + c->n_vr) % l->cap_r_tokens, 1};
    if (int s = hip_status(launch_copy_rows(p, static_cast<hipStream_t>(stream)))) return s;
    c->n_kr += 1;
    c->n_vr += 1;
    return KIVI_OK;
}

int kivi_flush_residual(const kivi_layout_t* l, kivi_cache_t* c, int32_t policy, int32_t* n_key_flushed,
                        int32_t* n_value_flushed, void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (policy != KIVI_FLUSH_WINDOW && policy != KIVI_FLUSH_ALG1) return KIVI_ERR_INVALID_ARG;
    int nk = 0, nv = 0;
    if (int s = plan_flush(l, c, policy, &nk, &nv)) return s;
    if (int s = enqueue_flush(l, c, nk, nv, static_cast<hipStream_t>(stream))) return s;
    if (n_key_flushed) *n_key_flushed = nk;
    if (n_value_flushed) *n_value_flushed = nv;
    return KIVI_OK;
}

int kivi_prefill(const kivi_layout_t* l, const void* k, int64_t ksb, int64_t ksh, int64_t kst, const void* v,
                 int64_t vsb, int64_t vsh, int64_t vst, int32_t n_tokens, int32_t policy, kivi_cache_t* c,
                 void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (int s = check_source(k, ksb, ksh, kst)) return s;
    if (int s = check_source(v, vsb, vsh, vst)) return s;
    if (policy != KIVI_FLUSH_WINDOW && policy != KIVI_FLUSH_ALG1) return KIVI_ERR_INVALID_ARG;
    if (n_tokens < 0 || c->n_kq || c->n_vq || c->n_kr || c->n_vr) return KIVI_ERR_INVALID_ARG;
    const int G = l->group, R = l->residual;
    int nkq, nvq;
    if (policy == KIVI_FLUSH_WINDOW) {
        nkq = nvq = std::max(n_tokens - R, 0) / G * G;
    } else {
        nkq = R > 0 ? n_tokens - n_tokens % R : n_tokens / G * G;   // KeyQuant: r = l % R
        nvq = std::max(n_tokens - R, 0);                            // X_Vg = X_V[:l - R]
    }
    const int nkr = n_tokens - nkq, nvr = n_tokens - nvq;
    if (nkq > l->cap_q_tokens || nvq > l->cap_q_tokens || nkr > l->cap_r_tokens || nvr > l->cap_r_tokens)
        return KIVI_ERR_INVALID_ARG;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (nkq > 0) {
        const RowSource src{static_cast<const __half*>(k), ksb, ksh, kst, 0, 0};
        if (int s = enqueue_key_quant(l, c, src, nkq, hs)) return s;
    }
    if (nvq > 0) {
        const RowSource src{static_cast<const __half*>(v), vsb, vsh, vst, 0, 0};
        if (int s = enqueue_value_quant(l, c, src, nvq, hs)) return s;
    }
    CopyRowsParams p{};
    p.cap_r = l->cap_r_tokens; p.n_kv_heads = l->n_kv_heads; p.batch = l->batch;
    p.job[0] = {static_cast<const __half*>(k), ksb, ksh, kst, nkq, static_cast<__half*>(c->k_resid), 0, nkr};
    p.job[1] = {static_cast<const __half*>(v), vsb, vsh, vst, nvq, static_cast<__half*>(c->v_resid), 0, nvr};
    if (int s = hip_status(launch_copy_rows(p, hs))) return s;
    c->n_kq = nkq; c->n_vq = nvq; c->n_kr = nkr; c->n_vr = nvr; c->k_r_start = 0; c->v_r_start = 0;
    return KIVI_OK;
}

int kivi_decode_attention(const kivi_layout_t* l, const kivi_cache_t* c, const void* q, float softmax_scale,
                          float* out, void* workspace, size_t workspace_bytes, void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (int s = check_attention_args(l, c, q, out, workspace, workspace_bytes)) return s;
    return enqueue_attention(l, c, q, softmax_scale, out, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int kivi_decode_attention_static(const kivi_layout_t* l, const kivi_cache_t* c, const void* q,
                                 float softmax_scale, float* out, void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    // argument checks first (they need no device); the workspace pointer is not known yet, an aligned
    // dummy stands in for it
    if (int s = check_attention_args(l, c, q, out, reinterpret_cast<const void*>(uintptr_t{256}),
                                     KIVI_STATIC_WORKSPACE_BYTES, false)) return s;
    void* ws = nullptr;
    if (int s = static_scratch_address(&ws)) return s;
    // The array keeps what the last call on this device left.  The parts are written before they are
    // read; the counters at its start must be zero: a completed call leaves them so, a fill kernel
    // (not a memset, so that the call can be captured into a graph) makes sure.
    if (counter_bytes(l) > KIVI_STATIC_WORKSPACE_BYTES) return KIVI_ERR_WORKSPACE;
    const int n_words = (int)(counter_bytes(l) / sizeof(uint32_t));
    zero_words_kernel<<<(n_words + 255) / 256, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<uint32_t*>(ws), n_words);
    if (int s = hip_status(hipGetLastError())) return s;
    // enqueue_attention refuses (KIVI_ERR_WORKSPACE, nothing launched) a state whose counters and parts pass the limit
    return enqueue_attention(l, c, q, softmax_scale, out, ws, KIVI_STATIC_WORKSPACE_BYTES, nullptr, nullptr, stream);
}

int kivi_decode_step(const kivi_layout_t* l, kivi_cache_t* c, const void* k_new, const void* v_new, const void* q,
                     float softmax_scale, int32_t policy, float* out, void* workspace, size_t workspace_bytes,
                     void* stream) {
    if (int s = check_layout(l)) return s;
    if (int s = check_cache(l, c)) return s;
    if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return KIVI_ERR_INVALID_ARG;
    if (policy != KIVI_FLUSH_WINDOW && policy != KIVI_FLUSH_ALG1) return KIVI_ERR_INVALID_ARG;
    if (c->n_kr >= l->cap_r_tokens || c->n_vr >= l->cap_r_tokens) return KIVI_ERR_INVALID_ARG;
    // the cache as it will be after the append and the flush: everything is checked against it
    // before anything is launched
    kivi_cache_t after = *c;
    after.n_kr += 1;
    after.n_vr += 1;
    int nk = 0, nv = 0;
    if (int s = plan_flush(l, &after, policy, &nk, &nv)) return s;
    {
        kivi_cache_t fl = after;
        fl.n_kq += nk; fl.n_kr -= nk; fl.n_vq += nv; fl.n_vr -= nv;
        if (int s = check_attention_args(l, &fl, q, out, workspace, workspace_bytes)) return s;
    }
    if (decode_family(l) == KIVI_DECODE_MFMA && nk <= c->n_kr && nv <= c->n_vr) {
        // The tokens to flush were all in the rings before this step: quantise them first (one
        // launch, none on the steps without a flush), then let the attention read the new token from
        // k_new / v_new and store it in the rings itself.  The ring slot of the new token and the
        // cache state seen by the attention are the same as with append -> flush -> attention.
        kivi_cache_t flushed = *c;                       // the counters after the flush, nothing launched yet
        if (int s = enqueue_flush(l, &flushed, nk, nv, nullptr, false)) return s;
        after = flushed;
        after.n_kr += 1;
        after.n_vr += 1;
        // In the two-launch form (G = 32) the fp16-row launch quantises the flushed tokens with extra
        // workgroups: a flush step then takes two launches like any other step.
        if ((nk > 0 || nv > 0) && l->group == kTileTokens && wants_two_launches(l, &after, KIVI_DECODE_MFMA)) {
            const int64_t sh = (int64_t)l->cap_r_tokens * kHeadDim, sb = sh * l->n_kv_heads;
            const RowSource ksrc{static_cast<const __half*>(c->k_resid), sb, sh, kHeadDim, c->k_r_start, l->cap_r_tokens};
            const RowSource vsrc{static_cast<const __half*>(c->v_resid), sb, sh, kHeadDim, c->v_r_start, l->cap_r_tokens};
            const QuantKeyParams kp = key_quant_params(l, c, ksrc, nk);
            const QuantValueParams vp = value_quant_params(l, c, vsrc, nv);
            if (int s = enqueue_attention(l, &after, q, softmax_scale, out, workspace, workspace_bytes, k_new, v_new, stream, &kp, &vp))
                return s;
            *c = after;
            return KIVI_OK;
        }
        if (int s = enqueue_flush(l, c, nk, nv, static_cast<hipStream_t>(stream))) return s;
        if (int s = enqueue_attention(l, &after, q, softmax_scale, out, workspace, workspace_bytes, k_new, v_new, stream)) return s;
        *c = after;
        return KIVI_OK;
    }
    // the flush takes the new token itself (Algorithm 1's key flush, or no residual window): append first
    if (int s = kivi_append_residual(l, c, k_new, v_new, stream)) return s;
    if (int s = kivi_flush_residual(l, c, policy, nullptr, nullptr, stream)) return s;
    return enqueue_attention(l, c, q, softmax_scale, out, workspace, workspace_bytes, nullptr, nullptr, stream);
}

int kivi_batch_slice(const kivi_layout_t* l, const kivi_cache_t* c, int32_t b0, int32_t nb,
                     const kivi_seq_state_t* state, kivi_layout_t* sub_layout, kivi_cache_t* sub_cache) {
    if (int s = check_layout(l)) return s;
    if (!c || !sub_layout || !sub_cache || b0 < 0 || nb < 1 || (int64_t)b0 + nb > l->batch) return KIVI_ERR_INVALID_ARG;
    kivi_cache_sizes_t sz;
    if (int s = kivi_cache_sizes(l, &sz)) return s;
    *sub_layout = *l;
    sub_layout->batch = nb;
    *sub_cache = *c;
    // every array is dense [b][h][...]: one sequence takes 1/batch of it
    auto move = [&](void* base, size_t total) -> void* {
        return base ? static_cast<char*>(base) + total / l->batch * b0 : nullptr;
    };
    sub_cache->k_codes = move(c->k_codes, sz.k_codes); sub_cache->k_scale = move(c->k_scale, sz.k_scale);
    sub_cache->k_zero = move(c->k_zero, sz.k_zero);    sub_cache->v_codes = move(c->v_codes, sz.v_codes);
    sub_cache->v_scale = move(c->v_scale, sz.v_scale); sub_cache->v_zero = move(c->v_zero, sz.v_zero);
    sub_cache->k_resid = move(c->k_resid, sz.k_resid); sub_cache->v_resid = move(c->v_resid, sz.v_resid);
    if (state) {
        sub_cache->n_kq = state->n_kq; sub_cache->n_vq = state->n_vq; sub_cache->k_r_start = state->k_r_start;
        sub_cache->n_kr = state->n_kr; sub_cache->v_r_start = state->v_r_start; sub_cache->n_vr = state->n_vr;
    }
    return check_cache(sub_layout, sub_cache);
}

int kivi_decode_step_ragged(const kivi_layout_t* l, const kivi_cache_t* c, kivi_seq_state_t* states,
                            const void* k_new, const void* v_new, const void* q, float softmax_scale,
                            int32_t policy, float* out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!k_new || !v_new || !q || !out) return KIVI_ERR_INVALID_ARG;
    if (int s = ragged_step_fast(l, c, states, k_new, v_new, q, softmax_scale, policy, out, workspace, workspace_bytes, stream);
        s != kNotApplicable)
        return s;
    return for_each_run(l, c, states, true, [&](kivi_layout_t& sl, kivi_cache_t& sc, int b0) {
        const size_t kv_row = (size_t)l->n_kv_heads * kHeadDim, q_row = (size_t)l->n_q_heads * kHeadDim;
        return kivi_decode_step(&sl, &sc, static_cast<const __half*>(k_new) + b0 * kv_row,
                                static_cast<const __half*>(v_new) + b0 * kv_row,
                                static_cast<const __half*>(q) + b0 * q_row, softmax_scale, policy,
                                out + b0 * q_row, workspace, workspace_bytes, stream);
    });
}

int kivi_decode_launches_ragged(const kivi_layout_t* l, const kivi_seq_state_t* states, int32_t* launches) {
    if (int s = check_layout(l)) return s;
    if (!states || !launches) return KIVI_ERR_INVALID_ARG;
    const int path = decode_family(l);
    const int rep_total = l->n_q_heads / l->n_kv_heads;
    const int head_groups = ceil_div(rep_total, kMaxRep);
    // the conditions of ragged_attention_fast
    bool fast = path == KIVI_DECODE_MFMA && l->decode_path != KIVI_DECODE_MFMA_ONE && l->cap_q_tokens >= kTileTokens &&
                l->group == kTileTokens;
    int max_tiles_a = 0, max_tiles_b = 0;
    for (int b = 0; b < l->batch; ++b) {
        const kivi_seq_state_t& x = states[b];
        if (x.n_kq < 0 || x.n_vq < 0 || x.n_kr < 0 || x.n_vr < 0 || x.n_kq + x.n_kr != x.n_vq + x.n_vr) return KIVI_ERR_INVALID_ARG;
        if (x.n_kq != x.n_vq || x.n_kr < 1 || x.n_kq % kTileTokens != 0) fast = false;
        max_tiles_a = std::max(max_tiles_a, x.n_kq / kTileTokens);
        max_tiles_b = std::max(max_tiles_b, ceil_div(x.n_kq + x.n_kr, kTileTokens) - x.n_kq / kTileTokens);
    }
    const int rep_launch = std::min(rep_total, kMaxRep);
    if (fast && max_tiles_a >= 1 && residual_rows_possible(max_tiles_b, rep_launch <= 2 ? rep_launch : (rep_launch <= 4 ? 4 : 8))) {
        *launches = 2 * head_groups;
        return KIVI_OK;
    }
    // run by run
    int total = 0;
    for (int b0 = 0; b0 < l->batch;) {
        int b1 = b0 + 1;
        while (b1 < l->batch && same_state(states[b0], states[b1])) ++b1;
        const kivi_seq_state_t& x = states[b0];
        if (x.n_kq + x.n_kr > 0) {
            kivi_layout_t sl = *l;
            sl.batch = b1 - b0;
            kivi_cache_t sc{};
            sc.n_kq = x.n_kq; sc.n_vq = x.n_vq; sc.n_kr = x.n_kr; sc.n_vr = x.n_vr;
            const bool two = wants_two_launches(&sl, &sc, path);
            const bool split = head_split_shift(&sl, plan_splits(&sl, &sc, path == KIVI_DECODE_MFMA, two), path, two) > 0;
            total += path == KIVI_DECODE_MFMA ? (split ? 1 : head_groups * (two ? 2 : 1)) : head_groups + 1;
        }
        b0 = b1;
    }
    *launches = total;
    return KIVI_OK;
}

int kivi_decode_attention_ragged(const kivi_layout_t* l, const kivi_cache_t* c, const kivi_seq_state_t* states,
                                 const void* q, float softmax_scale, float* out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (!q || !out) return KIVI_ERR_INVALID_ARG;
    if (check_layout(l) == KIVI_OK && c && states && aligned16(q) && aligned16(out) && workspace && aligned16(workspace)) {
        bool ok = true;
        for (int b = 0; b < l->batch && ok; ++b) {
            kivi_layout_t sl; kivi_cache_t sc;
            ok = kivi_batch_slice(l, c, b, 1, &states[b], &sl, &sc) == KIVI_OK;     // validates the sequence's counters
        }
        if (ok) {
            const int s = ragged_attention_fast(l, c, states, q, softmax_scale, out, workspace, workspace_bytes, nullptr, nullptr, stream);
            if (s != kNotApplicable) return s;
        }
    }
    return for_each_run(l, c, const_cast<kivi_seq_state_t*>(states), false,
                        [&](kivi_layout_t& sl, kivi_cache_t& sc, int b0) {
        if (sc.n_kq + sc.n_kr == 0 && sc.n_vq + sc.n_vr == 0) return (int)KIVI_OK;      // empty slots of the batch
        const size_t q_row = (size_t)l->n_q_heads * kHeadDim;
        return kivi_decode_attention(&sl, &sc, static_cast<const __half*>(q) + b0 * q_row, softmax_scale,
                                     out + b0 * q_row, workspace, workspace_bytes, stream);
    });
}

int kivi_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || !aligned16(src) || !aligned16(sink) || (bytes & 15)) return KIVI_ERR_INVALID_ARG;
    return hip_status(launch_stream_read(src, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream)));
}

}  // extern "C"
