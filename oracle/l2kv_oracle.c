/*
 * CPU oracle for the L2-norm KV-cache compression hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * definition the GPU library is checked against.  It shares no code, header,
 * table or helper with the HIP path, and nothing in the product may call it:
 * only tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * What it computes (arXiv 2406.11430):
 *   - the eviction rule of Sec. 1 / Sec. 3: keep the keys with the lowest L2
 *     norm, per layer and head, together with their values; the number of
 *     dropped pairs is exact (|D_{l,h}| = m, Eq. 5);
 *   - scaled dot-product attention of one query over the cached rows
 *     (Eq. 2 in its decode form, Eq. 4).
 *
 * Readings the paper leaves open (listed in full in the design document):
 *   - squared norm instead of norm (same order, no sqrt);
 *   - ties: the lower token index is kept; total order = (fp32 bits, index);
 *   - kept rows stay in ascending token order;
 *   - with grouped-query attention the "head" of the rule is the KV head, and
 *     query head hq reads KV head hq / (Hq/Hkv);
 *   - fp32 norms are summed in ONE fixed order (below), because the order of
 *     two nearly equal norms decides an integer (which row is kept) and both
 *     sides must take that decision in the same precision.
 *
 * Pins: every function here is pinned by the no-GPU tests against something other
 * than itself (hand-derived fixtures, brute force on small inputs, closed forms,
 * library routines, and for the keep-random hash its mathematical inverse); no
 * function is left parity-unpinned.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC.
 * Floating point: norms in fp32 exactly as written (no contraction); fp64
 * "truth" norms beside them; attention accumulates in fp64 and rounds once.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
static float widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static float load_elem(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16)
        return widen_bf16(((const uint16_t *)base)[i]);
    return ((const float *)base)[i];
}

static uint32_t float_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/*
 * Kept count k for T cached tokens at keep_ratio r: ceil(r*T), where a product
 * that misses an integer only by binary rounding of r (0.55*100 =
 * 55.000000000000007) counts as that integer; clamped to [1, T].
 * "Compressing X %" in the paper (Sec. 4) is r = 1 - X.
 */
int64_t l2kv_oracle_keep_count(int64_t T, double r)
{
    if (T <= 0)
        return 0;
    double x = r * (double)T;
    double nearest = nearbyint(x);
    double tol = 1e-9 * (x > 1.0 ? x : 1.0);
    double kd = (fabs(x - nearest) <= tol) ? nearest : ceil(x);
    if (kd < 1.0)
        kd = 1.0;
    if (kd > (double)T)
        kd = (double)T;
    return (int64_t)kd;
}

/*
 * Squared L2 norm of one key row in fp32, in the fixed order:
 *   1. cut the row into 16 chunks of D/16 consecutive elements;
 *   2. sum the squares of each chunk left to right;
 *   3. add the 16 partial sums as a balanced binary tree over neighbours:
 *      (p0+p1), (p2+p3), ... then pairs of those, and so on.
 * Each product and each sum is rounded to fp32 on its own.
 */
static float row_norm_f32(const void *row, int dtype, int32_t D)
{
    float p[16];
    int32_t c = D / 16;
    for (int i = 0; i < 16; ++i) {
        float x0 = load_elem(row, dtype, (int64_t)i * c);
        float acc = x0 * x0;
        for (int e = 1; e < c; ++e) {
            float x = load_elem(row, dtype, (int64_t)i * c + e);
            float sq = x * x;
            acc = acc + sq;
        }
        p[i] = acc;
    }
    for (int width = 1; width < 16; width *= 2)
        for (int i = 0; i < 16; i += 2 * width)
            p[i] = p[i] + p[i + width];
    return p[0];
}

/* The same sum in fp64, left to right: the reference value the fp32 order is
 * judged against (used for tolerance windows only, never for selection). */
static double row_norm_f64(const void *row, int dtype, int32_t D)
{
    double acc = 0.0;
    for (int32_t d = 0; d < D; ++d) {
        double x = (double)load_elem(row, dtype, d);
        acc += x * x;
    }
    return acc;
}

/*
 * K: n_heads slabs, head i starts at element i*head_stride, rows of D
 * contiguous elements.  n32 [n_heads][T] (required), n64 [n_heads][T] or NULL.
 * Returns 0, or -1 for an unsupported D / dtype.
 */
int l2kv_oracle_norms(const void *K, int dtype, int64_t n_heads, int64_t T,
                      int32_t D, int64_t head_stride, float *n32, double *n64)
{
    if (D <= 0 || D % 16 != 0 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return -1;
    size_t es = dtype == ORACLE_BF16 ? 2 : 4;
    for (int64_t h = 0; h < n_heads; ++h) {
        const char *head = (const char *)K + (size_t)h * (size_t)head_stride * es;
        for (int64_t t = 0; t < T; ++t) {
            const void *row = head + (size_t)t * (size_t)D * es;
            n32[h * T + t] = row_norm_f32(row, dtype, D);
            if (n64)
                n64[h * T + t] = row_norm_f64(row, dtype, D);
        }
    }
    return 0;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Selection for one head.  Order the T positions by (fp32 bit pattern of the
 * squared norm, token index) with a full sort, keep the first k, and return
 * those positions in ascending token order.  Norms are >= +0, so the unsigned
 * bit pattern orders like the value; +Inf and NaN patterns sort last and are
 * evicted first.
 *
 * mode 0: keep the LOWEST norms (the paper's method).
 * mode 1: keep the HIGHEST norms (the control of Sec. 4); ties still go to
 *         the lower token index.
 */
int l2kv_oracle_select(const float *n32, int64_t T, int64_t k, int mode,
                       int32_t *kept_idx)
{
    if (T <= 0 || k < 0 || k > T || T > INT32_MAX)
        return -1;
    uint64_t *keys = (uint64_t *)malloc((size_t)T * sizeof *keys);
    if (!keys)
        return -2;
    for (int64_t t = 0; t < T; ++t) {
        uint32_t b = float_bits(n32[t]);
        if (mode == 1)
            b = ~b;
        keys[t] = ((uint64_t)b << 32) | (uint64_t)(uint32_t)t;
    }
    qsort(keys, (size_t)T, sizeof *keys, cmp_u64);
    for (int64_t j = 0; j < k; ++j)
        kept_idx[j] = (int32_t)(keys[j] & 0xffffffffu);
    free(keys);
    qsort(kept_idx, (size_t)k, sizeof *kept_idx, cmp_i32);
    return 0;
}

/*
 * Compaction for one head of one tensor: dst row j = src row kept_idx[j],
 * copied byte for byte.  row_bytes = D * element size.
 */
void l2kv_oracle_compact(const void *src, const int32_t *kept_idx, int64_t k,
                         int64_t row_bytes, void *dst)
{
    for (int64_t j = 0; j < k; ++j)
        memcpy((char *)dst + (size_t)j * (size_t)row_bytes,
               (const char *)src + (size_t)kept_idx[j] * (size_t)row_bytes,
               (size_t)row_bytes);
}

/*
 * Single-query attention over the rows it is given (Eq. 2 / Eq. 4), written
 * as the definition in three passes:
 *   s_j = (q . K_j) / sqrt(D)     (or * scale when scale > 0)
 *   p_j = exp(s_j - max_j s_j)
 *   o   = sum_j p_j V_j / sum_j p_j
 * Q [B][Hq][D]; Kc, Vc: (b, hkv) slab starts at element
 * (b*Hkv + hkv)*kv_head_stride, kv_len rows of D; O [B][Hq][D] fp32.
 * All sums in fp64; O is rounded to fp32 once.  No mask: every cached row is
 * in the past of the query.
 */
int l2kv_oracle_decode_attn(const void *Q, const void *Kc, const void *Vc,
                            int dtype, int32_t B, int32_t Hq, int32_t Hkv,
                            int64_t kv_len, int32_t D, int64_t kv_head_stride,
                            double scale, float *O)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || kv_len <= 0 || D <= 0)
        return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -1;
    size_t es = dtype == ORACLE_BF16 ? 2 : 4;
    int32_t G = Hq / Hkv;
    double *s = (double *)malloc((size_t)kv_len * sizeof *s);
    double *acc = (double *)malloc((size_t)D * sizeof *acc);
    if (!s || !acc) {
        free(s);
        free(acc);
        return -2;
    }
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t hq = 0; hq < Hq; ++hq) {
            int32_t hkv = hq / G;
            const char *q = (const char *)Q + ((size_t)b * Hq + hq) * (size_t)D * es;
            size_t slab = ((size_t)b * Hkv + hkv) * (size_t)kv_head_stride * es;
            const char *Kh = (const char *)Kc + slab;
            const char *Vh = (const char *)Vc + slab;
            double m = -INFINITY;
            for (int64_t j = 0; j < kv_len; ++j) {
                const char *row = Kh + (size_t)j * (size_t)D * es;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d)
                    dot += (double)load_elem(q, dtype, d) *
                           (double)load_elem(row, dtype, d);
                s[j] = scale > 0.0 ? dot * scale : dot / sqrt((double)D);
                if (s[j] > m)
                    m = s[j];
            }
            double denom = 0.0;
            for (int32_t d = 0; d < D; ++d)
                acc[d] = 0.0;
            for (int64_t j = 0; j < kv_len; ++j) {
                double p = exp(s[j] - m);
                denom += p;
                const char *row = Vh + (size_t)j * (size_t)D * es;
                for (int32_t d = 0; d < D; ++d)
                    acc[d] += p * (double)load_elem(row, dtype, d);
            }
            float *o = O + ((size_t)b * Hq + hq) * (size_t)D;
            for (int32_t d = 0; d < D; ++d)
                o[d] = (float)(acc[d] / denom);
        }
    }
    free(s);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------------
 * Streaming eviction (Sec. 4, "Language Modelling Tasks": the cache grows to a
 * pre-defined length, after which the tokens with the highest L2 norm are
 * discarded).  One (sequence, head) at a time; the cache is a set of slots,
 * slot j holding the key/value rows, the fp32 squared norm (fixed summation
 * order above) and the original token id of one kept token.
 *
 * Eviction order is the reverse of the keep order of l2kv_oracle_select: the
 * slot with the LARGEST (norm bits, token id) goes first, so among equal norms
 * the later token is dropped and the kept set is always "the lowest-norm
 * tokens, ties to the lower token id".  The hole is filled with the last slot
 * (the slot order carries no meaning; tests compare token-id sets).
 * ------------------------------------------------------------------------ */

/* Append one token: rows copied to slot *len, norm and id recorded, *len += 1. */
int l2kv_oracle_stream_append(void *K, void *V, float *norms, int32_t *pos, int32_t *len,
                              int32_t capacity, int dtype, int32_t D, const void *k_new,
                              const void *v_new, int32_t token_id)
{
    if (*len >= capacity || D <= 0 || D % 16 != 0)
        return -1;
    size_t rb = (size_t)D * (dtype == ORACLE_BF16 ? 2 : 4);
    memcpy((char *)K + (size_t)*len * rb, k_new, rb);
    memcpy((char *)V + (size_t)*len * rb, v_new, rb);
    norms[*len] = row_norm_f32(k_new, dtype, D);
    pos[*len] = token_id;
    *len += 1;
    return 0;
}

/* While more than `budget` slots are occupied, drop the slot with the largest
 * (norm bits, token id) and move the last slot into its place.
 * Returns the number of evictions. */
int l2kv_oracle_stream_evict(void *K, void *V, float *norms, int32_t *pos, int32_t *len,
                             int32_t budget, int dtype, int32_t D)
{
    size_t rb = (size_t)D * (dtype == ORACLE_BF16 ? 2 : 4);
    int evicted = 0;
    if (budget < 0)
        budget = 0;
    while (*len > budget) {
        int32_t worst = 0;
        uint64_t worst_key = 0;
        for (int32_t j = 0; j < *len; ++j) {
            uint64_t key = ((uint64_t)float_bits(norms[j]) << 32) | (uint64_t)(uint32_t)pos[j];
            if (j == 0 || key > worst_key) {
                worst_key = key;
                worst = j;
            }
        }
        int32_t last = *len - 1;
        if (worst != last) {
            memcpy((char *)K + (size_t)worst * rb, (char *)K + (size_t)last * rb, rb);
            memcpy((char *)V + (size_t)worst * rb, (char *)V + (size_t)last * rb, rb);
            norms[worst] = norms[last];
            pos[worst] = pos[last];
        }
        *len = last;
        ++evicted;
    }
    return evicted;
}

/* ------------------------------------------------------------------------
 * Keep-random control of Sec. 4 (a random subset of the tokens is kept).  The random order is
 * a counter-based hash of (seed, head, token) so that it can be reproduced
 * anywhere: x = token*0x9E3779B1 + head*0x85EBCA77 + seed (mod 2^32), followed
 * by the 32-bit finalizer of MurmurHash3 (x ^= x>>16; x *= 0x85EBCA6B;
 * x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16).  The keys are written as bit
 * patterns into an fp32 array; selection orders by bit pattern, so
 * l2kv_oracle_select on them keeps the k tokens with the lowest hash.
 * ------------------------------------------------------------------------ */
void l2kv_oracle_random_keys(int64_t n_heads, int64_t T, uint32_t seed, float *keys)
{
    for (int64_t h = 0; h < n_heads; ++h) {
        for (int64_t t = 0; t < T; ++t) {
            uint32_t x = (uint32_t)t * 0x9E3779B1u + (uint32_t)h * 0x85EBCA77u + seed;
            x ^= x >> 16;
            x *= 0x85EBCA6Bu;
            x ^= x >> 13;
            x *= 0xC2B2AE35u;
            x ^= x >> 16;
            memcpy(&keys[h * T + t], &x, sizeof x);
        }
    }
}
