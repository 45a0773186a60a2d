/*
 * l2kv -- L2-norm KV-cache compression and decode attention for AMD MI355X
 * (CDNA4, gfx950).  C ABI of libl2kv.so.
 *
 * Method: arXiv 2406.11430, "A Simple and Effective L2 Norm-Based Strategy for
 * KV Cache Compression".  Its rule (Sec. 1, Sec. 3): per layer and head, keep
 * the cached keys with the lowest L2 norm together with their values and drop
 * the rest; decoding then runs ordinary scaled dot-product attention (Eq. 2,
 * in the decode form of Eq. 4) over the smaller cache.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - All tensor pointers are DEVICE pointers unless a parameter name starts
 *    with h_.  The caller owns every buffer; the library never allocates,
 *    frees, synchronises or copies to the host.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and returns.
 *  - Arguments are validated on the host BEFORE anything is enqueued; a
 *    negative status means nothing was launched and no device memory was
 *    touched.  L2KV_ERR_LAUNCH wraps a failed kernel launch.
 *  - "Head" means one (layer, sequence, KV head) triple.  The rule is
 *    independent per layer and head (Eq. 5: the dropped set D_{l,h}), so any
 *    number of layers / sequences can be flattened into n_heads.
 *  - A K or V row is D contiguous elements; head i starts `head_stride`
 *    ELEMENTS after head i-1 (head_stride >= T*D).  Supported:
 *    D in {64, 128} for fp32 and bf16, D = 256 for bf16 only (rows of at most
 *    512 bytes).  Base pointers of K, V, Kc, Vc, Q
 *    must be 16-byte aligned and head_stride*sizeof(elem) a multiple of 16;
 *    norms / index / O / workspace pointers 4-byte aligned (workspace 16).
 *  - Outputs must not alias inputs.
 *  - Placement (performance only, no entry point allocates): on MI355X the
 *    288 GiB of device memory behave as three regions of 96 GiB, and a launch
 *    that streams its K rows from one region and its V rows from another
 *    runs about 9 % slower than one whose two streams share a region.  Keep
 *    the K and the V cache of a layer in one allocation, made early.
 *  - Global state of the library: a per-device cache of the compute-unit
 *    count and, for l2kv_decode_attn_static only, the per-device address of
 *    its scratch array.  No call changes a kernel attribute or a device
 *    setting.  Calls are thread-safe as long as they do not share a workspace.
 */
#ifndef L2KV_H
#define L2KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { L2KV_F32 = 0, L2KV_BF16 = 1 } l2kv_dtype;

typedef enum {
    L2KV_OK = 0,
    L2KV_ERR_NULL = -1,      /* a required pointer is NULL                     */
    L2KV_ERR_SHAPE = -2,     /* a size is <= 0, too large, or D unsupported    */
    L2KV_ERR_DTYPE = -3,     /* dtype is not L2KV_F32 / L2KV_BF16              */
    L2KV_ERR_RATIO = -4,     /* keep_ratio outside (0, 1] or not finite        */
    L2KV_ERR_WORKSPACE = -5, /* workspace NULL or smaller than *_workspace_bytes */
    L2KV_ERR_ALIGN = -6,     /* pointer or stride alignment violated           */
    L2KV_ERR_LAUNCH = -7     /* the HIP runtime refused a launch               */
} l2kv_status;

/* Eviction strategy.  LOWEST is the paper's method; HIGHEST is the control of
 * Sec. 4 (the highest-norm tokens are the ones kept). */
typedef enum { L2KV_KEEP_LOWEST = 0, L2KV_KEEP_HIGHEST = 1 } l2kv_mode;

/*
 * Number of rows kept out of T at keep_ratio r: k = ceil(r*T), clamped to
 * [1, T]; a product r*T within 1e-9 relative of an integer counts as that
 * integer (so 0.55*100 -> 55).  The paper fixes only that the count is exact
 * (|D_{l,h}| = m, Eq. 5) and quotes "compression ratios" X (Sec. 4), which
 * are r = 1 - X.  Host function; returns 0 for T <= 0 or r outside (0,1].
 */
int64_t l2kv_keep_count(int64_t T, double keep_ratio);

/*
 * Squared L2 norm of every cached key (the quantity the rule of Sec. 1 /
 * Sec. 3 ranks by; the square keeps the order and needs no sqrt):
 *     norms[i][t] = sum_d K[i][t][d]^2          fp32
 * summed in a fixed order so the result is reproducible bit for bit: the row
 * is cut into 16 chunks of D/16 consecutive elements, each chunk is summed
 * left to right, and the 16 partial sums are added as a balanced binary tree
 * over neighbours; every product and sum is rounded to fp32 separately.
 *   K      in : n_heads slabs of T rows (layout above), read once
 *   norms  out: [n_heads][T] fp32, dense
 * Errors: NULL, SHAPE (n_heads, T <= 0; T > 2^31-1; D; head_stride < T*D),
 * DTYPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_norms(const void* K, l2kv_dtype dt, int64_t n_heads, int64_t T,
                       int32_t D, int64_t head_stride, float* norms, void* stream);

/*
 * Selection (the eviction rule of Sec. 1: the lowest-norm keys stay in the
 * cache; Eq. 5: exactly m pairs dropped per layer and head).  For every head, the
 * k = l2kv_keep_count(T, keep_ratio) positions that come first in the total
 * order (uint32 bit pattern of the fp32 squared norm, token index) -- ties go
 * to the lower token index -- written in ascending token order.
 *   norms      in : [n_heads][T] fp32 (>= +0; +Inf / NaN patterns sort last)
 *   kept_idx   out: [n_heads][k] int32, strictly ascending per head
 *   kept_count out: [n_heads] int32, every entry = k; may be NULL
 *   workspace     : l2kv_select_workspace_bytes(n_heads, T) bytes, 16-aligned;
 *                   contents need not be initialised and are undefined after.
 *                   This version keeps all selection state in registers and
 *                   LDS and never touches the buffer; the size query returns
 *                   a small constant (256).  The argument is part of the
 *                   signature for versions that select across workgroups.
 * Errors: NULL, SHAPE, RATIO, WORKSPACE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_select(const float* norms, int64_t n_heads, int64_t T,
                        double keep_ratio, int32_t* kept_idx, int32_t* kept_count,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Same with an explicit kept count k (1 <= k <= T) and strategy.  HIGHEST
 * orders by descending norm, ties again to the lower token index. */
l2kv_status l2kv_select_k(const float* norms, int64_t n_heads, int64_t T,
                          int64_t k, l2kv_mode mode, int32_t* kept_idx,
                          int32_t* kept_count, void* workspace,
                          size_t workspace_bytes, void* stream);

size_t l2kv_select_workspace_bytes(int64_t n_heads, int64_t T);

/*
 * Keys for the keep-random control of Sec. 4 (a random subset of the tokens
 * is kept):
 * keys[i][t] receives, as a 32-bit pattern stored in an fp32 array, the hash
 *     x = t*0x9E3779B1 + i*0x85EBCA77 + seed   (mod 2^32)
 *     x ^= x>>16; x *= 0x85EBCA6B; x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16
 * (the 32-bit finalizer of MurmurHash3).  l2kv_select_k orders by bit pattern,
 * so running it on these keys instead of norms keeps k pseudo-random tokens per
 * head, reproducibly.  keys out: [n_heads][T].  Errors: NULL, SHAPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_random_keys(int64_t n_heads, int64_t T, uint32_t seed, float* keys, void* stream);

/*
 * Compaction (Sec. 1: the values of the kept keys stay with them): the kept rows of K
 * and of V copied, byte for byte and in the order of kept_idx, into dense
 * caches:
 *     Kc[i][j][:] = K[i][kept_idx[i][j]][:],   Vc likewise.
 *   K, V     in : n_heads slabs of T rows (layout above); dropped rows are
 *                 never read.  V may be NULL together with Vc (K only).
 *   kept_idx in : [n_heads][k] int32, every entry in [0, T) (an entry outside
 *                 that range is forced into it on the device: a wrong row is
 *                 copied, nothing is read outside the head)
 *   Kc, Vc   out: [n_heads][k][D], dense
 * Errors: NULL, SHAPE (k <= 0, k > T, ...), DTYPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_compact(const void* K, const void* V, l2kv_dtype dt,
                         const int32_t* kept_idx, int64_t n_heads, int64_t T,
                         int64_t k, int32_t D, int64_t head_stride,
                         void* Kc, void* Vc, void* stream);

/*
 * The whole compression step (the rule of Sec. 1 as one operation: keep the
 * lowest-norm keys and their values) in one call: l2kv_norms, l2kv_select and
 * l2kv_compact enqueued back to back on `stream`, with the same results as the
 * three separate calls.
 *   slab_heads : 0 = all heads at once (three launches).  > 0 = the three
 *                steps are enqueued slab by slab of that many consecutive
 *                heads, and the norm pass reads K with ordinary instead of
 *                non-temporal loads, so that the compaction's second read of
 *                the kept K rows of a slab can be served by the caches while
 *                the slab still fits them.  On an MI355X this is SLOWER than
 *                slab_heads = 0 at the shapes measured (selection runs one
 *                workgroup per head, so a slab of a few heads leaves most of
 *                the chip idle during its selection); the mode exists so that
 *                the trade can be measured.
 *   norms      out: [n_heads][T] fp32 (needed as scratch; left filled)
 *   kept_idx   out: [n_heads][k], k = l2kv_keep_count(T, keep_ratio)
 *   Kc, Vc     out: [n_heads][k][D]
 *   workspace     : as l2kv_select
 * Errors: NULL, SHAPE, DTYPE, RATIO, WORKSPACE, ALIGN, LAUNCH (a launch failure
 * part-way leaves the earlier slabs done).
 */
l2kv_status l2kv_compress(const void* K, const void* V, l2kv_dtype dt, int64_t n_heads,
                          int64_t T, int32_t D, int64_t head_stride, double keep_ratio,
                          int64_t slab_heads, float* norms, int32_t* kept_idx, void* Kc,
                          void* Vc, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Decode attention (Eq. 2 for a single query row; Eq. 4: the query attends to
 * every row of the cache it is handed, the current token's row included by
 * the caller).  For each sequence b and query head hq, with KV head
 * hkv = hq / (Hq/Hkv) (consecutive query heads share a KV head):
 *     O[b][hq][:] = softmax_j( scale * Q[b][hq] . Kc[b][hkv][j] ) . Vc[b][hkv]
 * over j in [0, kv_len).  No mask.  Scores are never written to memory: the
 * cache is streamed once per KV head for all Hq/Hkv query heads, split over
 * row ranges with an online softmax, and the partial results are merged.
 *   Q   in : [B][Hq][D], dtype dt
 *   Kc,Vc in: (b,hkv) slab starts (b*Hkv+hkv)*kv_head_stride elements in;
 *             kv_len rows of D
 *   scale  : softmax scale; <= 0 selects 1/sqrt(D) (Eq. 2)
 *   O   out: [B][Hq][D] fp32
 *   workspace: l2kv_decode_workspace_bytes(B, Hq, kv_len, D) bytes,
 *              16-aligned.  It starts with one arrival counter per
 *              (sequence, KV head) followed by the split partials.  The
 *              counters must be ZERO before the first call that uses this
 *              buffer (zero-fill the whole buffer once); every call leaves
 *              them zero again, so the buffer can be reused call after call
 *              for any shape it is large enough for.  Two calls that share a
 *              workspace must not overlap in time.
 * The rows need not have been compacted: an uncompressed layer is attended to
 * in place by passing the original cache and kv_len = T.
 * Arithmetic: fp32 accumulation throughout; for bf16 caches q.k is formed with
 * the packed bf16 dot instruction (exact bf16 products, fp32 sum), for fp32
 * caches with fp32 FMAs; softmax and the value sum are fp32.
 * Errors: NULL, SHAPE (Hq % Hkv != 0, Hq/Hkv > 8 -- > 4 for D = 256 --,
 * kv_len <= 0, ...), DTYPE, WORKSPACE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_decode_attn(const void* Q, const void* Kc, const void* Vc,
                             l2kv_dtype dt, int32_t B, int32_t Hq, int32_t Hkv,
                             int64_t kv_len, int32_t D, int64_t kv_head_stride,
                             float scale, float* O, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Same with the element type of O chosen by the caller: L2KV_F32 (O is float*,
 * identical to l2kv_decode_attn) or L2KV_BF16 (O is [B][Hq][D] bf16, 2-byte
 * aligned: the fp32 result rounded to nearest even once, at the very end).
 * Errors: as l2kv_decode_attn; DTYPE also for an unknown out_dt. */
l2kv_status l2kv_decode_attn_out(const void* Q, const void* Kc, const void* Vc,
                                 l2kv_dtype dt, int32_t B, int32_t Hq, int32_t Hkv,
                                 int64_t kv_len, int32_t D, int64_t kv_head_stride,
                                 float scale, l2kv_dtype out_dt, void* O, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Same with the number of row ranges per KV head chosen by the caller
 * (1 <= n_splits <= l2kv_decode_max_splits(kv_len); 0 = library default).
 * The result does not depend on n_splits beyond fp32 rounding. */
l2kv_status l2kv_decode_attn_splits(const void* Q, const void* Kc, const void* Vc,
                                    l2kv_dtype dt, int32_t B, int32_t Hq, int32_t Hkv,
                                    int64_t kv_len, int32_t D, int64_t kv_head_stride,
                                    float scale, int32_t n_splits, float* O,
                                    void* workspace, size_t workspace_bytes,
                                    void* stream);

int32_t l2kv_decode_max_splits(int64_t kv_len);

/* Zero-fills a decode workspace with a small kernel on `stream` (the "zero
 * before first use" of l2kv_decode_attn; safe under graph capture, where a
 * memset node is not).  workspace_bytes: the size from
 * l2kv_decode_workspace_bytes (always a multiple of 16).
 * Errors: NULL, WORKSPACE (size 0 or not a multiple of 16), ALIGN, LAUNCH. */
l2kv_status l2kv_decode_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
size_t  l2kv_decode_workspace_bytes(int32_t B, int32_t Hq, int64_t kv_len, int32_t D);

/*
 * l2kv_decode_attn for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same result as
 * l2kv_decode_attn, but the arrival counters and split partials live in a
 * scratch array inside the library (L2KV_STATIC_SCRATCH_BYTES of device memory
 * per GPU, held until the process ends).  The call itself allocates and frees
 * nothing and records no memset.
 *   Limit: counters (4 bytes per (sequence, KV head), padded to 256) plus
 *   B*Hq*(workgroups per KV head)*(D+4)*4 bytes of partials must fit the
 *   scratch array; larger shapes return L2KV_ERR_WORKSPACE and launch nothing.
 *   (32k-context batch of 4 x 32 query heads: 0.4 MB.)
 *   All calls on one GPU share that GPU's array: two calls that may overlap in
 *   time (different streams without an ordering between them, or two host
 *   threads) race and give wrong results; calls ordered on one stream are fine.
 *   The first call on a device looks the array up and enqueues one small fill
 *   kernel on `stream`; make that first call outside graph capture.
 * Errors: as l2kv_decode_attn, L2KV_ERR_WORKSPACE for a shape beyond the limit,
 * L2KV_ERR_LAUNCH if the array cannot be located on the current device.
 */
#define L2KV_STATIC_SCRATCH_BYTES (4u << 20)
l2kv_status l2kv_decode_attn_static(const void* Q, const void* Kc, const void* Vc,
                                    l2kv_dtype dt, int32_t B, int32_t Hq, int32_t Hkv,
                                    int64_t kv_len, int32_t D, int64_t kv_head_stride,
                                    float scale, float* O, void* stream);

/* ------------------------------------------------------------------------
 * Ragged batches and streaming eviction.
 *
 * Sec. 4 ("Language Modelling Tasks"): the cache is allowed to grow to a
 * pre-defined length, after which the tokens with the highest key norm are
 * discarded.  A batch of sequences of different lengths is held ragged:
 *
 *   prompt tensors   K, V [n_planes][total_tokens][D], norms [n_planes][total_tokens];
 *                    sequence s = rows in_offsets[s] .. in_offsets[s+1]-1 of every plane
 *   slot cache       Kc, Vc [n_planes][total_slots][D], norms_c [n_planes][total_slots] fp32,
 *                    pos_c [n_planes][total_slots] int32 (original token id of each slot);
 *                    sequence s owns slots slot_offsets[s] .. slot_offsets[s+1]-1 of every
 *                    plane, of which the first lens[s] are occupied (same count in all planes)
 *
 * n_planes = layers x KV heads (plane = layer*Hkv + head).  All offset arrays
 * are DEVICE int64 [n_seq+1], ascending, first entry 0; lens / budgets /
 * token_ids are DEVICE int32 [n_seq].  Their contents cannot be checked on the
 * host: the kernels clamp what they read so that nothing is accessed outside
 * the buffers described by total_tokens / total_slots, but inconsistent
 * arrays give meaningless results.  Slot order inside a sequence carries no
 * meaning (attention is order-free); after l2kv_compact_ragged it is ascending
 * token order, evictions then move the last slot into the hole.
 * ------------------------------------------------------------------------ */

/*
 * Selection on a ragged batch: for every plane and sequence, the
 * k_s = out_offsets[s+1]-out_offsets[s] positions with the lowest (norm bits,
 * position) among its T_s = in_offsets[s+1]-in_offsets[s] tokens (k_s is capped
 * at T_s; the caller normally sets it with l2kv_keep_count(T_s, keep_ratio)).
 * Positions are relative to the sequence start, ascending.
 *   kept_idx out: [n_planes][total_kept] int32, sequence s at out_offsets[s]
 *   max_len     : an upper bound of all T_s (chooses the kernel variant; tokens
 *                 of a sequence beyond it would be ignored)
 * Errors: NULL, SHAPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_select_ragged(const float* norms, int32_t n_planes, int32_t n_seq,
                               int64_t total_tokens, const int64_t* in_offsets,
                               const int64_t* out_offsets, int64_t total_kept, int64_t max_len,
                               l2kv_mode mode, int32_t* kept_idx, void* stream);

/*
 * Compaction of a ragged batch into the slot cache: slot j of sequence s gets
 * row kept_idx[..][j] of that sequence (K, V, its norm, and the position as
 * token id).  Sets up the cache that l2kv_stream_* and l2kv_decode_attn_ragged
 * work on; lens[s] = k_s is the caller's to fill.  k_s is capped at the
 * sequence's slot capacity.  max_kept: an upper bound of all k_s (checked against
 * total_kept; the launch itself is sized by total_kept).
 * Errors: NULL, SHAPE, DTYPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_compact_ragged(const void* K, const void* V, const float* norms, l2kv_dtype dt,
                                const int32_t* kept_idx, int32_t n_planes, int32_t n_seq,
                                int64_t total_tokens, const int64_t* in_offsets,
                                const int64_t* out_offsets, int64_t total_kept, int64_t max_kept,
                                const int64_t* slot_offsets, int64_t total_slots, int32_t D,
                                void* Kc, void* Vc, float* norms_c, int32_t* pos_c, void* stream);

/*
 * Append the current token of every sequence (Eq. 4: its K_t, V_t join the
 * cache before the query attends): Knew, Vnew [n_layers][n_seq][Hkv][D] go to
 * slot lens_in[s] of sequence s in plane layer*Hkv+head, with the squared key
 * norm (same fixed summation order as l2kv_norms) and token_ids[s].
 * lens_out[s] = lens_in[s] + 1; a sequence whose slots are all occupied is left
 * unchanged (lens_out[s] = lens_in[s]).  lens_out must not be lens_in.
 * Errors: NULL, SHAPE, DTYPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_stream_append(const void* Knew, const void* Vnew, l2kv_dtype dt, int32_t n_layers,
                               int32_t n_seq, int32_t Hkv, int32_t D, const int32_t* token_ids,
                               const int64_t* slot_offsets, int64_t total_slots,
                               const int32_t* lens_in, int32_t* lens_out, void* Kc, void* Vc,
                               float* norms_c, int32_t* pos_c, void* stream);

/*
 * Evict down to the budget: in every plane, while sequence s holds more than
 * budgets[s] slots, the slot with the largest (norm bits, token id) is dropped
 * (among equal norms the later token goes first -- the reverse of the keep
 * order of l2kv_select) and the last slot is moved into its place.
 * lens_out[s] = min(lens_in[s], budgets[s]).  lens_out must not be lens_in.
 * With a fixed budget the kept token set equals l2kv_select over all tokens
 * seen; with budgets[s] = l2kv_keep_count(tokens seen, keep_ratio) it is the
 * keep_ratio "enforced incrementally".
 * Errors: NULL, SHAPE, DTYPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_stream_evict(l2kv_dtype dt, int32_t n_planes, int32_t n_seq, int32_t D,
                              const int64_t* slot_offsets, int64_t total_slots,
                              const int32_t* lens_in, const int32_t* budgets, int32_t* lens_out,
                              void* Kc, void* Vc, float* norms_c, int32_t* pos_c, void* stream);

/*
 * Decode attention over ONE layer of the slot cache: Q [n_seq][Hq][D]; Kc, Vc
 * point at that layer's Hkv planes ([Hkv][total_slots][D]); sequence s attends
 * to its lens[s] occupied slots (0 slots give a zero output row).
 *   seq_order: a DEVICE int32 [n_seq] permutation of 0..n_seq-1 giving
 *             the order in which the sequences are launched; with the longest
 *             sequence first (l2kv_length_order) the library hands whole
 *             (sequence, KV head) pairs, longest first, to one workgroup per
 *             compute unit, whichever is free next (a work list in the
 *             workspace), which is faster on batches of mixed lengths (bf16
 *             caches with heads of 128 elements; other row sizes are launched
 *             as a grid in the given order).  It only steers scheduling:
 *             outputs land at the sequence's own rows of O in any case.  An
 *             array that is not a permutation computes some sequences twice
 *             and others not at all (entries are forced into 0..n_seq-1).
 *             The order may be stale (lengths change from step to step).
 *             NULL: batches of 2..512 sequences whose longest has 2048 rows or
 *             more (bf16, D = 128) get a longest-first order worked out inside the call (one
 *             small extra kernel, about 7 us per call on an MI355X); all other
 *             batches are launched in batch order.  Either way the call is
 *             made of plain kernel launches and may be captured into a graph.
 *   max_len : an upper bound of all lens[s] (sizes the decomposition and the
 *             workspace; rows beyond it are still attended to)
 * A layer that is left uncompressed (Sec. 4 skips the first layers by default)
 * needs no copy at all: pass its prompt tensors as Kc, Vc with slot_offsets =
 * the prompt offsets, total_slots = total_tokens and lens[s] = T_s.  Per-head
 * keep counts (the outlook of Sec. 8) are the same call with every (sequence,
 * KV head) laid out as one "sequence" of a single plane (Hkv = 1, Hq = the
 * query group), as produced by l2kv_select_ragged / l2kv_compact_ragged with one
 * k per head.
 *   n_splits: 0 = library default
 *   workspace: l2kv_decode_ragged_workspace_bytes(n_seq, Hq, max_len, D) bytes
 *              (the uniform workspace plus room for that order), same
 *              zero-before-first-use contract as l2kv_decode_attn
 * Errors: as l2kv_decode_attn.
 */
l2kv_status l2kv_decode_attn_ragged(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt,
                                    int32_t n_seq, int32_t Hq, int32_t Hkv, int32_t D,
                                    const int32_t* lens, const int64_t* slot_offsets,
                                    const int32_t* seq_order, int64_t total_slots, int64_t max_len,
                                    float scale, int32_t n_splits, float* O, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * Longest-first order of a batch: order[r] = the sequence with the r-th largest
 * lens (equal lengths: lower index first).  lens, order: DEVICE int32 [n_seq],
 * distinct arrays; n_seq <= 65535.  A set-up call (one workgroup, quadratic in
 * n_seq); its result can serve many decode steps.
 * Errors: NULL, SHAPE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_length_order(const int32_t* lens, int32_t n_seq, int32_t* order, void* stream);

size_t l2kv_decode_ragged_workspace_bytes(int32_t n_seq, int32_t Hq, int64_t max_len, int32_t D);

/* ---------------------------------------------------------------------------
 * Attention-loss analysis (Sec. 3, Eq. 5-7)
 *
 * When m of the T cached pairs of a head are dropped, the attention loss L^m is
 * the sum of the attention scores a_p (softmax of Eq. 2 over the FULL cache) of
 * the dropped pairs (Eq. 5).  The norm rule drops the highest key norms; the
 * ideal rule, which would need the next query in advance, drops the lowest
 * scores and gives the reference loss L^{m,ref}.  Y^m = L^m - L^{m,ref} >= 0
 * (Eq. 6) and Y = sum over m = 1..T of Y^m (Eq. 7) measure how far the norm
 * order is from the ideal order for that head and query.
 * ------------------------------------------------------------------------ */

/*
 * Discard order of the norm rule.  drop_rank[h][t] = number of positions of
 * head h that are discarded before position t when pairs go highest norm
 * first and, among equal norms, later position first -- the exact reverse of
 * the keep order of l2kv_select, so l2kv_select(k) keeps the positions with
 * drop_rank >= T-k and the m dropped pairs of Eq. 5 are those with
 * drop_rank < m.  Each row of drop_rank is a permutation of 0..T-1.
 *   norms     in : [n_heads][T] fp32, dense (as written by l2kv_norms)
 *   drop_rank out: [n_heads][T] int32
 *   workspace    : l2kv_norm_ranks_workspace_bytes(n_heads, T) bytes of device
 *                  memory, 16-byte aligned; contents irrelevant before and after
 * n_heads <= 2^31-1, T <= 2^31-1.  Errors: NULL, SHAPE, WORKSPACE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_norm_ranks(const float* norms, int64_t n_heads, int64_t T, int32_t* drop_rank,
                            void* workspace, size_t workspace_bytes, void* stream);

size_t l2kv_norm_ranks_workspace_bytes(int64_t n_heads, int64_t T);

/*
 * Attention loss of one query per head over the uncompressed cache:
 *   a[b][hq][p]      = softmax_p( scale * Q[b][hq] . K[b][hq / (Hq/Hkv)][p] )       (Eq. 2)
 *   loss[b][hq]      = L^m      = sum of a_p over drop_rank[b][hkv][p] < m          (Eq. 5)
 *   loss_ref[b][hq]  = L^{m,ref} = sum of the m smallest a_p                        (Eq. 6)
 *   alr[b][hq]       = Y = sum_{m'=1..T} ( L^{m'} - L^{m',ref} )                    (Eq. 7)
 *   Q         in : [B][Hq][D], dense, dtype dt
 *   K         in : [B][Hkv] slabs of [T][D], k_head_stride elements apart, dtype dt
 *   drop_rank in : [B][Hkv][T] int32 from l2kv_norm_ranks (values outside 0..T-1
 *                  are not detected and give meaningless sums)
 *   m            : number of dropped pairs for loss / loss_ref, 0..T
 *                  (T - k for a cache compressed to k rows)
 *   scale        : softmax scale; <= 0 selects 1/sqrt(D)
 *   alr, loss, loss_ref out: [B][Hq] double each; loss and loss_ref may be NULL
 *   workspace    : l2kv_alr_workspace_bytes(B, Hq, T) bytes, 16-byte aligned;
 *                  contents irrelevant before and after
 * Scores are computed in fp32 and summed in fp64; Hq/Hkv <= 8, B*Hkv <= 65535.
 * All device pointers; enqueues on `stream` and returns.
 * Errors: NULL, DTYPE, SHAPE, WORKSPACE, ALIGN, LAUNCH.
 */
l2kv_status l2kv_alr(const void* Q, const void* K, l2kv_dtype dt, const int32_t* drop_rank, int32_t B,
                     int32_t Hq, int32_t Hkv, int64_t T, int32_t D, int64_t k_head_stride, float scale,
                     int64_t m, double* alr, double* loss, double* loss_ref, void* workspace,
                     size_t workspace_bytes, void* stream);

size_t l2kv_alr_workspace_bytes(int32_t B, int32_t Hq, int64_t T);

/*
 * Measurement aid: streams `bytes` bytes from `data` (rounded down to a
 * multiple of 8192) through the compute units with the loads of the norm
 * pass, computes nothing and stores nothing -- the rate this launch reaches is
 * the read-stream ceiling of the device for that buffer, against which the
 * kernels above can be judged (it depends on where the buffer lies in device
 * memory).  `sink`: 4 writable device bytes; written only if a block of the
 * data XORs to one particular 32-bit value, which keeps the loads alive.
 * Errors: NULL, ALIGN (data 16, sink 4), SHAPE (fewer than 8192 bytes, or
 * more than 2^31 - 1 blocks of 8192), LAUNCH.
 */
l2kv_status l2kv_read_probe(const void* data, size_t bytes, uint32_t* sink, void* stream);

/*
 * What the current HIP device reports about itself (host function, no kernel):
 * compute units, peak memory clock in kHz and memory bus width in bits, so
 * that a benchmark can print them next to the bandwidth peak it assumes.  Any
 * of the three pointers may be NULL.  Errors: LAUNCH if the runtime refuses
 * the query.
 */
l2kv_status l2kv_device_info(int32_t* h_compute_units, int32_t* h_memory_clock_khz,
                             int32_t* h_memory_bus_bits);

/* Static, NUL-terminated description of a status code. */
const char* l2kv_status_string(l2kv_status s);

/* Library version as major*10000 + minor*100 + patch. */
int32_t l2kv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* L2KV_H */
