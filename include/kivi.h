/*
 * kivi.h -- C ABI of the MI355X (gfx950) KIVI decode-attention library.
 *
 * The library implements the hot path of KIVI (arXiv 2402.02750): decode-step attention over
 * a tuning-free asymmetric low-bit KV cache.  Keys are quantised per channel in groups of G
 * consecutive tokens, values per token in groups of G consecutive channels (Section 3.3), with
 * zero-point = min and scale = (max - min) / (2^B - 1) (Section 3.1); the most recent tokens stay
 * in an fp16 residual part (Section 3.3, Algorithm 1).
 *
 * Conventions for every entry point
 *   - returns an int status: KIVI_OK (0) or a negative KIVI_ERR_* code;
 *   - arguments are validated on the host before anything is enqueued; on error nothing is
 *     launched and no cache field is changed;
 *   - work is enqueued on the caller's HIP stream (`stream` is a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns without synchronising;
 *   - the library never allocates or frees device memory: all buffers, including the attention
 *     workspace, belong to the caller (kivi_decode_attention_static is the one exception: its
 *     workspace is an array inside the library).  The only state it keeps between calls is, per
 *     device, the answer of one occupancy query per kernel instantiation and that array's address,
 *     and, per host thread, a small staging buffer (host memory) from which the ragged entry points
 *     copy their per-sequence tables to the workspace;
 *   - pointers inside kivi_cache_t, `q`, `out`, `workspace` and the fp16 source tensors are DEVICE
 *     pointers, 16-byte aligned; the structs themselves and all counts live on the host;
 *   - the uniform entry points work on batches of equal length; kivi_decode_step_ragged /
 *     kivi_decode_attention_ragged serve batches whose sequences differ in length.
 *
 * Arithmetic contract of the quantiser (bit-exact between implementations)
 *   z = min over the group (an fp16 value, stored as is)
 *   s = fp16_round_nearest_even( (float(max) - float(min)) / float(2^B - 1) )   [fp32 arithmetic]
 *   code = clamp( round_half_even( (float(x) - float(z)) / float(s) ), 0, 2^B - 1 )   [fp32
 *          subtract, IEEE fp32 division];  all codes are 0 when s == 0.
 *   x' = code * s + z.
 *
 * Memory layout (all arrays dense, index order as written, b = batch entry, h = kv-head)
 *   k_codes  uint32 [b][h][cap_q/32][W]   one "key tile" per block of 32 tokens, W = 32*128*B/32
 *   k_scale  fp16   [b][h][cap_q/G][128]   per (group of G tokens, channel)
 *   k_zero   fp16   [b][h][cap_q/G][128]
 *   v_codes  uint32 [b][h][cap_q/32][W]   one "value tile" per block of 32 tokens
 *   v_scale  fp16   [b][h][cap_q][128/G]   per (token, group of G channels)
 *   v_zero   fp16   [b][h][cap_q][128/G]
 *   One scale / zero-point pair per group, whatever G is (32, 64 or 128): a larger G stores, and the
 *   decode kernels read, proportionally fewer of them (Table 5 / Appendix C's group sizes).
 *   k_resid  fp16   [b][h][cap_r][128]     ring buffer: the i-th oldest residual token is in slot
 *   v_resid  fp16   [b][h][cap_r][128]     (r_start + i) % cap_r
 *   q        fp16   [b][n_q_heads][128]
 *   out      fp32   [b][n_q_heads][128]
 *
 *   A code tile covers 32 tokens x 128 channels and is addressed by (u, lane, e), u in [0,8),
 *   lane in [0,64), e in [0,8):
 *     key tile  : token   = (u & 1) * 16 + (lane & 15),  channel = (u >> 1) * 32 + (lane >> 4) * 8 + e
 *     value tile: channel = u * 16 + (lane & 15),         token   = (lane >> 4) * 8 + e
 *     B = 2 : word = lane*4 + (u >> 1),                         bit = (e & 1)*16 + 2*((u & 1)*4 + (e >> 1))
 *     B = 4 : i = (u >> 1)*2 + (e >> 2), word = (i >> 2)*256 + lane*4 + (i & 3),
 *                                                               bit = (e & 1)*16 + 4*((u & 1)*2 + ((e >> 1) & 1))
 *   (little-endian uint32 words).  The layout hands wavefront lane `lane` one 16-byte piece per
 *   256-word plane that already is its operand fragment of a 16x16x32 matrix instruction.
 */
#ifndef KIVI_H
#define KIVI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KIVI_OK                 0
#define KIVI_ERR_INVALID_ARG   -1   /* null/misaligned pointer, inconsistent counts, capacity exceeded */
#define KIVI_ERR_UNSUPPORTED   -2   /* a shape or mode this build has no kernel for                   */
#define KIVI_ERR_WORKSPACE     -3   /* workspace missing or smaller than kivi_decode_workspace_bytes  */
#define KIVI_ERR_HIP           -4   /* the HIP runtime reported a launch error                        */

/* residual-flush policies for kivi_flush_residual */
#define KIVI_FLUSH_WINDOW       0   /* quantise the oldest G tokens of K and V while the fp16 window
                                       holds >= R + G tokens: the most recent R tokens stay fp16      */
#define KIVI_FLUSH_ALG1         1   /* Algorithm 1 (Decoding) literally: the whole key residual when it
                                       holds exactly R tokens; the oldest value tokens beyond R       */

/* decode kernel families (kivi_layout_t.decode_path) */
#define KIVI_DECODE_AUTO        0
#define KIVI_DECODE_VALU        1   /* vector-ALU dot products + cross-lane reductions               */
#define KIVI_DECODE_MFMA        2   /* codes fed to the matrix cores as exact fp16                   */
#define KIVI_DECODE_MFMA_ONE    3   /* ... always as one launch                                      */
#define KIVI_DECODE_MFMA_TWO    4   /* ... as two launches where the cache has both quantised tokens */
                                    /* and fp16 rows: the fp16 rows first, then the quantised part   */
                                    /* (KIVI_DECODE_MFMA and AUTO pick the form from the shape: two  */
                                    /* launches when a workgroup would otherwise own parts of several*/
                                    /* (batch, kv-head) units, or with 3 or more query heads per     */
                                    /* kv-head and enough fp16 rows; kivi_decode_plan tells which)   */

/* Static description of one attention layer's cache (host struct). */
typedef struct kivi_layout {
    int32_t batch;          /* b                                                          */
    int32_t n_q_heads;      /* query heads; a multiple (1x to 128x) of n_kv_heads: up to  */
                            /* 8 query heads per kv-head share one pass over the cache,   */
                            /* wider groups (multi-query attention) run as units of one   */
                            /* launch (runs of 4 heads) in the matrix-core family's       */
                            /* single-launch form, one launch per 8 heads otherwise       */
    int32_t n_kv_heads;     /* key/value heads                                            */
    int32_t head_dim;       /* D; this build supports 128                                 */
    int32_t bits;           /* B: 2 or 4                                                  */
    int32_t group;          /* G: 32, 64 or 128 (tokens per key group, channels per value group) */
    int32_t residual;       /* R: residual length, a multiple of G (Section 3.3)          */
    int32_t cap_q_tokens;   /* capacity of the quantised part in tokens, multiple of G    */
    int32_t cap_r_tokens;   /* capacity of each fp16 ring in tokens, multiple of 32, >= R + G */
    int32_t decode_path;    /* KIVI_DECODE_*                                              */
} kivi_layout_t;

/* One layer's cache: the 4-tuple (Q(X_Kg), X_Kr, Q(X_Vg), X_Vr) of Algorithm 1.
 * The pointers are the caller's device buffers (sizes: kivi_cache_sizes); the integers are host
 * state that the library reads and advances. */
typedef struct kivi_cache {
    void *k_codes, *k_scale, *k_zero;
    void *v_codes, *v_scale, *v_zero;
    void *k_resid, *v_resid;
    int32_t n_kq;        /* quantised key tokens, multiple of G        */
    int32_t n_vq;        /* quantised value tokens                     */
    int32_t k_r_start;   /* ring slot of the oldest residual key       */
    int32_t n_kr;        /* residual key tokens                        */
    int32_t v_r_start;   /* ring slot of the oldest residual value     */
    int32_t n_vr;        /* residual value tokens                      */
} kivi_cache_t;

/* Byte sizes of the eight cache buffers for a layout. */
typedef struct kivi_cache_sizes {
    size_t k_codes, k_scale, k_zero, v_codes, v_scale, v_zero, k_resid, v_resid;
} kivi_cache_sizes_t;

/* Human-readable name of a status code (static storage, never NULL). */
const char* kivi_status_string(int status);

/* Host helper: buffer sizes for `layout`.  Errors: INVALID_ARG, UNSUPPORTED. */
int kivi_cache_sizes(const kivi_layout_t* layout, kivi_cache_sizes_t* sizes);

/* How kivi_decode_attention would serve a cache state: which kernel family, how many launches per
 * group of up to 8 query heads per kv-head, and how the token axis is cut. */
typedef struct kivi_decode_plan {
    int32_t family;             /* KIVI_DECODE_VALU or KIVI_DECODE_MFMA                              */
    int32_t launches;           /* kernel launches of one attention call                            */
    int32_t splits_quantised;   /* pieces of the all-quantised token range per (batch, kv-head)     */
    int32_t splits_fp16;        /* pieces of the range that holds fp16 rows                         */
    int32_t tiles_per_split_quantised, tiles_per_split_fp16;   /* in 32-token tiles                */
    int32_t units_per_kv_head;  /* 1; 2 or 4 when the query heads of every kv-head are served as    */
                                /* halves or quarters that read the cache independently (4, 6 or 8  */
                                /* heads per kv-head, small batches); ceil(heads per kv-head / 4)   */
                                /* when a wider group (multi-query attention) runs as ONE launch    */
                                /* whose units are runs of 4 query heads                            */
} kivi_decode_plan_t;

/* Host helper: the plan for `cache`'s current state (no launch).  Errors: INVALID_ARG, UNSUPPORTED. */
int kivi_decode_plan(const kivi_layout_t* layout, const kivi_cache_t* cache, kivi_decode_plan_t* plan);

/* Host helper: bytes of workspace kivi_decode_attention needs for ANY cache state that fits
 * `layout` (partial softmax statistics and outputs of the context splits). */
int kivi_decode_workspace_bytes(const kivi_layout_t* layout, size_t* bytes);

/*
 * Key quantisation, per channel in groups of G tokens -- Section 3.3 "Algorithm" and
 * Algorithm 1 (KeyQuant: GroupQuant(X_Kg, dim=channel)); formula of Section 3.1.
 *   k_fp16     device, fp16, element (b, h, t, c) at k_fp16[b*stride_b + h*stride_h + t*stride_t + c]
 *              (strides in elements, multiples of 8)
 *   n_tokens   number of tokens to quantise, a multiple of G; they become groups
 *              n_kq/G ... of the cache, and cache->n_kq advances by n_tokens.
 * Errors: INVALID_ARG (null, misaligned, n_tokens % G != 0, capacity), UNSUPPORTED, HIP.
 */
int kivi_quantize_key_groups(const kivi_layout_t* layout, const void* k_fp16, int64_t stride_b,
                             int64_t stride_h, int64_t stride_t, int32_t n_tokens,
                             kivi_cache_t* cache, void* stream);

/*
 * Value quantisation, per token in groups of G channels -- Section 3.3 and Algorithm 1
 * (GroupQuant(X_Vg, dim=token, numGroup=d//G)); formula of Section 3.1.
 * Same argument meaning as above; the tokens are appended at cache->n_vq, which advances.
 * n_tokens need not be a multiple of 32: a partly filled value tile is completed by later calls.
 */
int kivi_quantize_value_tokens(const kivi_layout_t* layout, const void* v_fp16, int64_t stride_b,
                               int64_t stride_h, int64_t stride_t, int32_t n_tokens,
                               kivi_cache_t* cache, void* stream);

/*
 * Prefill -- Algorithm 1 (Prefill): split the prompt's keys and values into the grouped part,
 * which is quantised, and the fp16 residual part, which is copied into the rings.  The cache must
 * be empty (all counters 0).  `policy` selects the split:
 *   KIVI_FLUSH_WINDOW  K and V alike: the first floor(max(l - R, 0) / G) * G tokens are quantised;
 *   KIVI_FLUSH_ALG1    keys: l - l % R tokens (KeyQuant); values: max(l - R, 0) tokens.
 * Source tensors as for kivi_quantize_key_groups (separate strides for K and V).
 */
int kivi_prefill(const kivi_layout_t* layout, const void* k_fp16, int64_t k_stride_b, int64_t k_stride_h,
                 int64_t k_stride_t, const void* v_fp16, int64_t v_stride_b, int64_t v_stride_h,
                 int64_t v_stride_t, int32_t n_tokens, int32_t policy, kivi_cache_t* cache, void* stream);

/*
 * Append the new token's key and value to the fp16 residual parts -- Algorithm 1 (Decoding):
 * X_Kr <- Concat(X_Kr, t_K), X_Vr <- Concat(X_Vr, t_V).
 *   k_new, v_new   device, fp16 [b][n_kv_heads][128]
 * Errors: INVALID_ARG (null, a ring is full: flush first).
 */
int kivi_append_residual(const kivi_layout_t* layout, kivi_cache_t* cache, const void* k_new,
                         const void* v_new, void* stream);

/*
 * Move the oldest residual tokens into the quantised part -- Section 3.3 (the key residual is
 * quantised as a whole when it is full; the value residual is a queue of R tokens) and
 * Algorithm 1 (Decoding).
 * `policy` is KIVI_FLUSH_WINDOW or KIVI_FLUSH_ALG1 (see above).  A call that finds nothing to
 * flush enqueues nothing.  On return the cache counters describe the new split.
 * Optional outputs (host, may be NULL): number of key / value tokens quantised by this call.
 */
int kivi_flush_residual(const kivi_layout_t* layout, kivi_cache_t* cache, int32_t policy,
                        int32_t* n_key_flushed, int32_t* n_value_flushed, void* stream);

/*
 * Decode-step attention over the mixed-precision cache -- Equation 4 (tiled logits over the
 * quantised and the residual keys), Equation 1 / Algorithm 1 (Decoding): softmax over the
 * concatenated logits, t_O = A_g Q(X_Vg) + A_r X_Vr.
 *   q              device, fp16 [b][n_q_heads][128]; query head j reads kv-head
 *                  j / (n_q_heads / n_kv_heads)
 *   softmax_scale  multiplies the logits before the softmax (1/sqrt(D) for the usual attention)
 *   out            device, fp32 [b][n_q_heads][128]
 *   workspace      device scratch of at least kivi_decode_workspace_bytes(layout) bytes.  It must be
 *                  zero-filled once before its first use; every completed call leaves it ready
 *                  for the next one (it starts with per-(batch, kv-head) counters that the
 *                  kernel returns to zero).  Calls that share a workspace must not overlap.
 * Requires n_kq + n_kr == n_vq + n_vr >= 1.  The K and V splits may differ (Algorithm 1 splits
 * them differently).
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.
 */
int kivi_decode_attention(const kivi_layout_t* layout, const kivi_cache_t* cache, const void* q,
                          float softmax_scale, float* out, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * kivi_decode_attention for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and result as kivi_decode_attention, but the partial results of the context splits and
 * their counters live in a static device array of KIVI_STATIC_WORKSPACE_BYTES inside the library
 * (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 *   - A cache state whose counters and parts need more than the array holds is refused with
 *     KIVI_ERR_WORKSPACE and nothing is launched.  The need of a state is
 *     round_up(16 * batch * n_kv_heads, 256) + 520 * batch * n_q_heads * (splits_quantised + splits_fp16)
 *     bytes with the splits kivi_decode_plan reports (configurations of up to 2048 query-head rows
 *     with a 4096-token context, or 128 rows with 32768 tokens, need 2.5 to 6.5 MB).
 *   - All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 *     threads) race.  Calls on one stream, or otherwise ordered, are fine; the array's contents from
 *     one call are not needed by the next (the counters at its start are cleared by a small fill
 *     kernel at the start of every call).
 *   - The first call on a device resolves the array's address there (hipGetSymbolAddress); make that
 *     call outside a graph capture.
 * Errors: as kivi_decode_attention; KIVI_ERR_UNSUPPORTED for a device ordinal of 64 or more.
 */
#define KIVI_STATIC_WORKSPACE_BYTES (8u << 20)
int kivi_decode_attention_static(const kivi_layout_t* layout, const kivi_cache_t* cache, const void* q,
                                 float softmax_scale, float* out, void* stream);

/*
 * One whole decoding step of Algorithm 1 (Decoding) -- append (t_K, t_V) to the fp16 residual
 * parts, flush them per `policy`, attention of t_Q over the updated cache -- in as few launches
 * as possible.  The result is the same as kivi_append_residual + kivi_flush_residual +
 * kivi_decode_attention.  On steps where nothing is flushed and the matrix-core family runs, the
 * append costs no launch of its own: the attention (one launch or two, see
 * kivi_decode_plan) reads the new token's rows from k_new / v_new and writes them into the
 * residual rings itself.  On the other steps it enqueues the separate kernels.
 *   k_new, v_new   device, fp16 [b][n_kv_heads][128]; they must stay valid until the launch has run
 *   other arguments as for kivi_decode_attention / kivi_flush_residual
 * Errors: INVALID_ARG (also: a ring is full, no capacity left for the flush), UNSUPPORTED,
 * WORKSPACE, HIP.  On an error the cache is unchanged unless a kernel launch itself failed (HIP).
 */
int kivi_decode_step(const kivi_layout_t* layout, kivi_cache_t* cache, const void* k_new, const void* v_new,
                     const void* q, float softmax_scale, int32_t policy, float* out, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * Batches whose sequences differ in length.  Entry b of a `kivi_seq_state_t` array (host memory,
 * one entry per batch entry) holds for sequence b what the integer fields of kivi_cache_t hold for
 * a batch of equal lengths; the buffers keep the dense [b][h][...] layout with the same capacities
 * for every sequence.
 */
typedef struct kivi_seq_state {
    int32_t n_kq, n_vq, k_r_start, n_kr, v_r_start, n_vr;
} kivi_seq_state_t;

/*
 * Host helper: batch entries [b0, b0 + nb) of `cache` as a cache of their own -- `sub_layout` is
 * `layout` with batch = nb, `sub_cache` points at the sub-batch's part of every buffer and takes
 * its integer fields from `state` (from `cache` if `state` is NULL).  Every entry point can then be
 * used on a part of the batch, e.g. kivi_prefill one sequence at a time.
 * Errors: INVALID_ARG (range outside the batch, bad layout or cache).
 */
int kivi_batch_slice(const kivi_layout_t* layout, const kivi_cache_t* cache, int32_t b0, int32_t nb,
                     const kivi_seq_state_t* state, kivi_layout_t* sub_layout, kivi_cache_t* sub_cache);

/*
 * kivi_decode_step / kivi_decode_attention for a batch whose sequences differ in length.  The
 * integer fields of `cache` are ignored; `states` (host, [batch]) is read and, by the step,
 * advanced.
 *   One pair of launches for the whole batch, whatever the lengths: when the matrix-core family
 * serves the layout (decode_path AUTO, MFMA or MFMA_TWO), every sequence has K and V split alike
 * (the WINDOW policy) with 1 to 512 fp16 rows (at most 16 tiles; fewer with many query heads per
 * kv-head), and at least one sequence has quantised tokens.  The fp16 rows of all sequences run in
 * one launch (which also appends the step's new tokens), the all-quantised parts in a second; both
 * read each sequence's counters from a copy in the workspace, and the shorter sequences' share of
 * the work partition is skipped (where that share is large, or the batch holds as many (batch,
 * kv-head) units as the chip holds wavefronts, the second launch divides the tokens that are there
 * evenly over the wavefronts instead).  A step adds one launch per run of equal sequences that flush
 * in it (a sequence flushes every G-th step).
 *   Otherwise (another policy or family, empty slots, sequences without fp16 rows) the batch is
 * walked in runs of consecutive entries with equal state and each run is one call of the uniform
 * entry point on that part of the batch (same stream, same workspace): B different lengths take B
 * calls.  Entries without any token (all counts 0) are skipped by kivi_decode_attention_ragged and
 * their `out` rows are left untouched.  kivi_decode_launches_ragged tells which applies.
 *   The one-pair form copies the sequences' counters from host memory into the workspace with an
 * asynchronous copy on `stream` at every call (16 bytes per sequence): do not record these two entry
 * points into a HIP graph -- a replay would copy from host memory that is gone, and the counters
 * change from step to step anyway.
 *   k_new, v_new, q, out   the whole batch's tensors, as for the uniform entry points
 * Errors: as for the uniform entry points; entries before the failing run have been processed.
 */
int kivi_decode_step_ragged(const kivi_layout_t* layout, const kivi_cache_t* cache, kivi_seq_state_t* states,
                            const void* k_new, const void* v_new, const void* q, float softmax_scale,
                            int32_t policy, float* out, void* workspace, size_t workspace_bytes, void* stream);
int kivi_decode_attention_ragged(const kivi_layout_t* layout, const kivi_cache_t* cache,
                                 const kivi_seq_state_t* states, const void* q, float softmax_scale, float* out,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Host helper: the number of kernel launches kivi_decode_attention_ragged enqueues for these
 * sequence states (no launch).  Two per group of up to 8 query heads per kv-head when the whole batch
 * goes through one pair of launches (see above); otherwise the sum over the runs of equal state.
 * Errors: INVALID_ARG, UNSUPPORTED.
 */
int kivi_decode_launches_ragged(const kivi_layout_t* layout, const kivi_seq_state_t* states, int32_t* launches);

/*
 * Measurement helper, not part of the method: a plain read-only stream over `bytes` bytes of
 * device memory (grid-stride 16-byte loads, every workgroup leaves one word in `sink`), the
 * yardstick the benchmark prices the decode kernel against besides the chip's published HBM peak
 * (the paper's Section 2 names the once-per-token load of the cache as what bounds decoding).
 *   src    device, 16-byte aligned, at least `bytes` bytes (a multiple of 16)
 *   sink   device, at least 4096 * 4 bytes
 * Errors: INVALID_ARG, HIP.
 */
int kivi_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KIVI_H */
