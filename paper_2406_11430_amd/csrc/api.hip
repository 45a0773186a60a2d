// C ABI of libl2kv.so: argument validation on the host, then the launchers.
// Nothing here allocates, synchronises or touches device memory; a negative
// status means no kernel was enqueued.
#include <atomic>
#include <cmath>

#include "l2kv_host.hpp"

namespace l2kv {

int device_compute_units() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return 256;
    }
    int cu = cached[dev].load(std::memory_order_relaxed);
    if (cu > 0) return cu;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) {
        (void)hipGetLastError();
        cu = 256;
    }
    cached[dev].store(cu, std::memory_order_relaxed);
    return cu;
}

namespace {

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool dtype_ok(l2kv_dtype dt) { return dt == L2KV_F32 || dt == L2KV_BF16; }
inline int elem_bytes(l2kv_dtype dt) { return dt == L2KV_F32 ? 4 : 2; }
// head sizes: 64 and 128 for both element types, 256 for bf16 (a row is then 512 bytes, as an
// fp32 row of 128 elements)
inline bool dim_ok(int32_t D, l2kv_dtype dt) { return D == 64 || D == 128 || (D == 256 && dt == L2KV_BF16); }
// query heads per KV head the decode kernels are built for
inline int32_t max_group(int32_t D) { return D == 256 ? 4 : 8; }
constexpr int64_t kMaxTokens = 0x7fffffffLL;          // token indices are int32
constexpr int64_t kMaxHeads = 0x7fffffffLL;

// Shared checks of a strided [n_heads][T][D] tensor description.
l2kv_status check_cache(l2kv_dtype dt, int64_t n_heads, int64_t T, int32_t D, int64_t head_stride) {
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (head_stride < T * (int64_t)D) return L2KV_ERR_SHAPE;
    if ((head_stride * elem_bytes(dt)) % 16 != 0) return L2KV_ERR_ALIGN;
    return L2KV_OK;
}

}  // namespace
}  // namespace l2kv

using namespace l2kv;

extern "C" {

int64_t l2kv_keep_count(int64_t T, double keep_ratio) {
    if (T <= 0 || !(keep_ratio > 0.0) || !(keep_ratio <= 1.0)) return 0;
    const double x = keep_ratio * static_cast<double>(T);
    const double whole = std::nearbyint(x);
    const double slack = 1e-9 * (x > 1.0 ? x : 1.0);
    double kd = std::fabs(x - whole) <= slack ? whole : std::ceil(x);
    if (kd < 1.0) kd = 1.0;
    if (kd > static_cast<double>(T)) kd = static_cast<double>(T);
    return static_cast<int64_t>(kd);
}

l2kv_status l2kv_norms(const void* K, l2kv_dtype dt, int64_t n_heads, int64_t T, int32_t D,
                       int64_t head_stride, float* norms, void* stream) {
    if (K == nullptr || norms == nullptr) return L2KV_ERR_NULL;
    if (l2kv_status st = check_cache(dt, n_heads, T, D, head_stride); st != L2KV_OK) return st;
    if (!aligned(K, 16) || !aligned(norms, 4)) return L2KV_ERR_ALIGN;
    return norms_dispatch(K, dt, n_heads, T, D, head_stride, norms, false, static_cast<hipStream_t>(stream));
}

size_t l2kv_select_workspace_bytes(int64_t n_heads, int64_t T) {
    // The kernels keep all selection state in registers and LDS and never touch
    // the workspace; the header says so.  A small fixed size keeps callers'
    // allocation code valid for a version that does need scratch.
    (void)n_heads;
    (void)T;
    return 256;
}

l2kv_status l2kv_select_k(const float* norms, int64_t n_heads, int64_t T, int64_t k, l2kv_mode mode,
                          int32_t* kept_idx, int32_t* kept_count, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (norms == nullptr || kept_idx == nullptr) return L2KV_ERR_NULL;
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens) return L2KV_ERR_SHAPE;
    if (k <= 0 || k > T) return L2KV_ERR_SHAPE;
    if (mode != L2KV_KEEP_LOWEST && mode != L2KV_KEEP_HIGHEST) return L2KV_ERR_SHAPE;
    if (workspace == nullptr || workspace_bytes < l2kv_select_workspace_bytes(n_heads, T))
        return L2KV_ERR_WORKSPACE;
    if (!aligned(norms, 4) || !aligned(kept_idx, 4) || !aligned(kept_count, 4) || !aligned(workspace, 16))
        return L2KV_ERR_ALIGN;
    return select_dispatch(norms, n_heads, T, k, mode, kept_idx, kept_count, workspace,
                           static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_select(const float* norms, int64_t n_heads, int64_t T, double keep_ratio,
                        int32_t* kept_idx, int32_t* kept_count, void* workspace,
                        size_t workspace_bytes, void* stream) {
    if (norms == nullptr || kept_idx == nullptr) return L2KV_ERR_NULL;
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens) return L2KV_ERR_SHAPE;
    if (!(keep_ratio > 0.0) || !(keep_ratio <= 1.0)) return L2KV_ERR_RATIO;   // also rejects NaN
    return l2kv_select_k(norms, n_heads, T, l2kv_keep_count(T, keep_ratio), L2KV_KEEP_LOWEST,
                         kept_idx, kept_count, workspace, workspace_bytes, stream);
}

l2kv_status l2kv_compact(const void* K, const void* V, l2kv_dtype dt, const int32_t* kept_idx,
                         int64_t n_heads, int64_t T, int64_t k, int32_t D, int64_t head_stride,
                         void* Kc, void* Vc, void* stream) {
    if (K == nullptr || Kc == nullptr || kept_idx == nullptr) return L2KV_ERR_NULL;
    if ((V == nullptr) != (Vc == nullptr)) return L2KV_ERR_NULL;
    if (l2kv_status st = check_cache(dt, n_heads, T, D, head_stride); st != L2KV_OK) return st;
    if (k <= 0 || k > T) return L2KV_ERR_SHAPE;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(kept_idx, 4))
        return L2KV_ERR_ALIGN;
    return compact_dispatch(K, V, dt, kept_idx, n_heads, T, k, D, head_stride, Kc, Vc,
                            static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_compress(const void* K, const void* V, l2kv_dtype dt, int64_t n_heads, int64_t T, int32_t D,
                          int64_t head_stride, double keep_ratio, int64_t slab_heads, float* norms,
                          int32_t* kept_idx, void* Kc, void* Vc, void* workspace, size_t workspace_bytes,
                          void* stream) {
    if (K == nullptr || V == nullptr || norms == nullptr || kept_idx == nullptr || Kc == nullptr || Vc == nullptr)
        return L2KV_ERR_NULL;
    if (l2kv_status st = check_cache(dt, n_heads, T, D, head_stride); st != L2KV_OK) return st;
    if (!(keep_ratio > 0.0) || !(keep_ratio <= 1.0)) return L2KV_ERR_RATIO;
    if (slab_heads < 0) return L2KV_ERR_SHAPE;
    if (workspace == nullptr || workspace_bytes < l2kv_select_workspace_bytes(n_heads, T)) return L2KV_ERR_WORKSPACE;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(norms, 4) ||
        !aligned(kept_idx, 4) || !aligned(workspace, 16))
        return L2KV_ERR_ALIGN;
    const int64_t k = l2kv_keep_count(T, keep_ratio);
    const int64_t slab = slab_heads == 0 || slab_heads > n_heads ? n_heads : slab_heads;
    const bool keep_in_cache = slab < n_heads;       // the slab's K rows are read again two launches later
    const size_t es = static_cast<size_t>(elem_bytes(dt));
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int64_t h0 = 0; h0 < n_heads; h0 += slab) {
        const int64_t nh = n_heads - h0 < slab ? n_heads - h0 : slab;
        const char* Ks = static_cast<const char*>(K) + static_cast<size_t>(h0) * static_cast<size_t>(head_stride) * es;
        const char* Vs = static_cast<const char*>(V) + static_cast<size_t>(h0) * static_cast<size_t>(head_stride) * es;
        float* ns = norms + h0 * T;
        int32_t* is = kept_idx + h0 * k;
        const size_t dense = static_cast<size_t>(h0) * static_cast<size_t>(k) * static_cast<size_t>(D) * es;
        l2kv_status st = norms_dispatch(Ks, dt, nh, T, D, head_stride, ns, keep_in_cache, s);
        if (st == L2KV_OK) st = select_dispatch(ns, nh, T, k, L2KV_KEEP_LOWEST, is, nullptr, workspace, s);
        if (st == L2KV_OK)
            st = compact_dispatch(Ks, Vs, dt, is, nh, T, k, D, head_stride, static_cast<char*>(Kc) + dense,
                                  static_cast<char*>(Vc) + dense, s);
        if (st != L2KV_OK) return st;
    }
    return L2KV_OK;
}

int32_t l2kv_decode_max_splits(int64_t kv_len) { return decode_max_splits(kv_len); }

l2kv_status l2kv_decode_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (workspace == nullptr) return L2KV_ERR_NULL;
    if (workspace_bytes < 16 || workspace_bytes % 16 != 0) return L2KV_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return L2KV_ERR_ALIGN;
    return workspace_init_dispatch(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t l2kv_decode_workspace_bytes(int32_t B, int32_t Hq, int64_t kv_len, int32_t D) {
    if (B <= 0 || Hq <= 0 || kv_len <= 0 || D <= 0) return 0;
    // counters (at most one per query head: Hkv <= Hq) + split partials
    const size_t raw = decode_counter_bytes(B, Hq) +
                       static_cast<size_t>(B) * static_cast<size_t>(Hq) *
                           static_cast<size_t>(decode_max_splits(kv_len)) * decode_partial_floats(D) *
                           sizeof(float);
    return (raw + 255) / 256 * 256;
}

// Argument checks shared by the uniform decode entry points (everything but the workspace).
static l2kv_status check_decode(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                                int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D, int64_t kv_head_stride,
                                float scale, int32_t n_splits, const void* O, uintptr_t o_align = 4) {
    if (Q == nullptr || Kc == nullptr || Vc == nullptr || O == nullptr) return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || kv_len <= 0 || kv_len > kMaxTokens || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (Hq % Hkv != 0 || Hq / Hkv > max_group(D)) return L2KV_ERR_SHAPE;
    if (static_cast<int64_t>(B) * Hkv > 65535 || static_cast<int64_t>(B) * Hq > 0x7fffffffLL)
        return L2KV_ERR_SHAPE;
    if (kv_head_stride < kv_len * static_cast<int64_t>(D)) return L2KV_ERR_SHAPE;
    if (n_splits < 0 || n_splits > decode_max_splits(kv_len)) return L2KV_ERR_SHAPE;
    if (!std::isfinite(scale)) return L2KV_ERR_SHAPE;
    if ((kv_head_stride * elem_bytes(dt)) % 16 != 0) return L2KV_ERR_ALIGN;
    if (!aligned(Q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(O, o_align)) return L2KV_ERR_ALIGN;
    return L2KV_OK;
}

l2kv_status l2kv_decode_attn_splits(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt,
                                    int32_t B, int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                                    int64_t kv_head_stride, float scale, int32_t n_splits, float* O,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    l2kv_status st = check_decode(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, scale, n_splits, O);
    // the workspace is checked in the place it always had among the checks: after the sizes,
    // before the alignments
    if (st != L2KV_OK && st != L2KV_ERR_ALIGN) return st;
    if (workspace == nullptr || workspace_bytes < l2kv_decode_workspace_bytes(B, Hq, kv_len, D))
        return L2KV_ERR_WORKSPACE;
    if (st != L2KV_OK) return st;
    if (!aligned(workspace, 16)) return L2KV_ERR_ALIGN;
    const float s = scale > 0.f ? scale : 1.0f / std::sqrt(static_cast<float>(D));
    const DecodePlan plan = decode_plan(B, Hkv, Hq / Hkv, kv_len, n_splits);
    return decode_dispatch(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, nullptr, nullptr, nullptr, s,
                           plan, O, workspace, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_decode_attn_out(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                                 int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D, int64_t kv_head_stride,
                                 float scale, l2kv_dtype out_dt, void* O, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (O != nullptr && !dtype_ok(out_dt)) return L2KV_ERR_DTYPE;
    l2kv_status st = check_decode(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, scale, 0, O,
                                  out_dt == L2KV_BF16 ? 2 : 4);
    if (st != L2KV_OK && st != L2KV_ERR_ALIGN) return st;
    if (workspace == nullptr || workspace_bytes < l2kv_decode_workspace_bytes(B, Hq, kv_len, D))
        return L2KV_ERR_WORKSPACE;
    if (st != L2KV_OK) return st;
    if (!aligned(workspace, 16)) return L2KV_ERR_ALIGN;
    const float s = scale > 0.f ? scale : 1.0f / std::sqrt(static_cast<float>(D));
    DecodePlan plan = decode_plan(B, Hkv, Hq / Hkv, kv_len, 0);
    plan.out_bf16 = out_dt == L2KV_BF16 ? 1 : 0;
    return decode_dispatch(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, nullptr, nullptr, nullptr, s,
                           plan, static_cast<float*>(O), workspace, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_decode_attn_static(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt,
                                    int32_t B, int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                                    int64_t kv_head_stride, float scale, float* O, void* stream) {
    if (l2kv_status st = check_decode(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, scale, 0, O);
        st != L2KV_OK)
        return st;
    const float s = scale > 0.f ? scale : 1.0f / std::sqrt(static_cast<float>(D));
    const DecodePlan plan = decode_plan(B, Hkv, Hq / Hkv, kv_len, 0);
    // counters + the partials of the workgroups this launch really has
    const size_t need = decode_counter_bytes(B, Hkv) +
                        static_cast<size_t>(B) * static_cast<size_t>(Hq) * static_cast<size_t>(plan.n_splits) *
                            decode_partial_floats(D) * sizeof(float);
    if (need > static_cast<size_t>(L2KV_STATIC_SCRATCH_BYTES)) return L2KV_ERR_WORKSPACE;
    l2kv_status st = L2KV_OK;
    void* scratch_ptr = decode_static_scratch(static_cast<hipStream_t>(stream), &st);
    if (scratch_ptr == nullptr) return st;
    return decode_dispatch(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, nullptr, nullptr, nullptr, s,
                           plan, O, scratch_ptr, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_decode_attn(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                             int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                             int64_t kv_head_stride, float scale, float* O, void* workspace,
                             size_t workspace_bytes, void* stream) {
    return l2kv_decode_attn_splits(Q, Kc, Vc, dt, B, Hq, Hkv, kv_len, D, kv_head_stride, scale, 0, O,
                                   workspace, workspace_bytes, stream);
}

l2kv_status l2kv_random_keys(int64_t n_heads, int64_t T, uint32_t seed, float* keys, void* stream) {
    if (keys == nullptr) return L2KV_ERR_NULL;
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens) return L2KV_ERR_SHAPE;
    if (n_heads > (int64_t{1} << 62) / T) return L2KV_ERR_SHAPE;
    if (!aligned(keys, 4)) return L2KV_ERR_ALIGN;
    return random_keys_dispatch(n_heads, T, seed, keys, static_cast<hipStream_t>(stream));
}

/* ---- ragged batches and the streaming slot cache ------------------------- */

l2kv_status l2kv_select_ragged(const float* norms, int32_t n_planes, int32_t n_seq,
                               int64_t total_tokens, const int64_t* in_offsets,
                               const int64_t* out_offsets, int64_t total_kept, int64_t max_len,
                               l2kv_mode mode, int32_t* kept_idx, void* stream) {
    if (norms == nullptr || in_offsets == nullptr || out_offsets == nullptr || kept_idx == nullptr)
        return L2KV_ERR_NULL;
    if (n_planes <= 0 || n_seq <= 0 || total_tokens <= 0 || total_tokens > kMaxTokens ||
        total_kept <= 0 || total_kept > total_tokens || max_len <= 0 || max_len > total_tokens)
        return L2KV_ERR_SHAPE;
    if (mode != L2KV_KEEP_LOWEST && mode != L2KV_KEEP_HIGHEST) return L2KV_ERR_SHAPE;
    if (!aligned(norms, 4) || !aligned(kept_idx, 4) || !aligned(in_offsets, 8) || !aligned(out_offsets, 8))
        return L2KV_ERR_ALIGN;
    return select_ragged_dispatch(norms, n_planes, n_seq, total_tokens, in_offsets, out_offsets,
                                  total_kept, max_len, mode, kept_idx, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_compact_ragged(const void* K, const void* V, const float* norms, l2kv_dtype dt,
                                const int32_t* kept_idx, int32_t n_planes, int32_t n_seq,
                                int64_t total_tokens, const int64_t* in_offsets,
                                const int64_t* out_offsets, int64_t total_kept, int64_t max_kept,
                                const int64_t* slot_offsets, int64_t total_slots, int32_t D, void* Kc,
                                void* Vc, float* norms_c, int32_t* pos_c, void* stream) {
    if (K == nullptr || V == nullptr || norms == nullptr || kept_idx == nullptr || in_offsets == nullptr ||
        out_offsets == nullptr || slot_offsets == nullptr || Kc == nullptr || Vc == nullptr ||
        norms_c == nullptr || pos_c == nullptr)
        return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (n_planes <= 0 || n_seq <= 0 || total_tokens <= 0 || total_tokens > kMaxTokens ||
        total_kept <= 0 || total_kept > total_tokens || max_kept <= 0 || max_kept > total_kept ||
        total_slots <= 0 || total_slots > kMaxTokens || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(norms, 4) ||
        !aligned(norms_c, 4) || !aligned(pos_c, 4) || !aligned(kept_idx, 4) || !aligned(in_offsets, 8) ||
        !aligned(out_offsets, 8) || !aligned(slot_offsets, 8))
        return L2KV_ERR_ALIGN;
    return compact_ragged_dispatch(K, V, norms, dt, kept_idx, n_planes, n_seq, total_tokens, in_offsets,
                                   out_offsets, total_kept, max_kept, slot_offsets, total_slots, D, Kc,
                                   Vc, norms_c, pos_c, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_stream_append(const void* Knew, const void* Vnew, l2kv_dtype dt, int32_t n_layers,
                               int32_t n_seq, int32_t Hkv, int32_t D, const int32_t* token_ids,
                               const int64_t* slot_offsets, int64_t total_slots, const int32_t* lens_in,
                               int32_t* lens_out, void* Kc, void* Vc, float* norms_c, int32_t* pos_c,
                               void* stream) {
    if (Knew == nullptr || Vnew == nullptr || token_ids == nullptr || slot_offsets == nullptr ||
        lens_in == nullptr || lens_out == nullptr || Kc == nullptr || Vc == nullptr ||
        norms_c == nullptr || pos_c == nullptr)
        return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (n_layers <= 0 || n_seq <= 0 || Hkv <= 0 || total_slots <= 0 || total_slots > kMaxTokens || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (lens_in == lens_out) return L2KV_ERR_SHAPE;           // workgroups read lens_in while one writes lens_out
    if (!aligned(Knew, 16) || !aligned(Vnew, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) ||
        !aligned(norms_c, 4) || !aligned(pos_c, 4) || !aligned(token_ids, 4) || !aligned(lens_in, 4) ||
        !aligned(lens_out, 4) || !aligned(slot_offsets, 8))
        return L2KV_ERR_ALIGN;
    return stream_append_dispatch(Knew, Vnew, dt, n_layers, n_seq, Hkv, D, token_ids, slot_offsets,
                                  total_slots, lens_in, lens_out, Kc, Vc, norms_c, pos_c,
                                  static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_stream_evict(l2kv_dtype dt, int32_t n_planes, int32_t n_seq, int32_t D,
                              const int64_t* slot_offsets, int64_t total_slots, const int32_t* lens_in,
                              const int32_t* budgets, int32_t* lens_out, void* Kc, void* Vc,
                              float* norms_c, int32_t* pos_c, void* stream) {
    if (slot_offsets == nullptr || lens_in == nullptr || budgets == nullptr || lens_out == nullptr ||
        Kc == nullptr || Vc == nullptr || norms_c == nullptr || pos_c == nullptr)
        return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (n_planes <= 0 || n_seq <= 0 || total_slots <= 0 || total_slots > kMaxTokens || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (lens_in == lens_out) return L2KV_ERR_SHAPE;
    if (!aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(norms_c, 4) || !aligned(pos_c, 4) ||
        !aligned(lens_in, 4) || !aligned(lens_out, 4) || !aligned(budgets, 4) || !aligned(slot_offsets, 8))
        return L2KV_ERR_ALIGN;
    return stream_evict_dispatch(dt, n_planes, n_seq, D, slot_offsets, total_slots, lens_in, budgets,
                                 lens_out, Kc, Vc, norms_c, pos_c, static_cast<hipStream_t>(stream));
}

// Ragged workspace = the uniform one (counters, partials) followed by room for a
// launch order of the sequences, which the library computes itself when the
// caller passes none (small batches of long sequences only, see below).
static size_t ragged_order_bytes(int32_t n_seq) {
    return (static_cast<size_t>(n_seq) * sizeof(int32_t) + 255) / 256 * 256;
}
// Row size on which ordered batches take the work list (every (sequence, KV head, share) drawn
// from a device counter): bf16 heads of 128 elements, the shape its tests and the streaming
// benchmark cover.  Other row sizes are launched as a grid in the order given.
static bool work_list_rows(l2kv_dtype dt, int32_t D) { return dt == L2KV_BF16 && D == 128; }
constexpr int32_t kSelfOrderMaxSeq = 512;     // the set-up kernel is quadratic in n_seq
constexpr int64_t kSelfOrderMinRows = 2048;   // below this the ordered plan is not used anyway

size_t l2kv_decode_ragged_workspace_bytes(int32_t n_seq, int32_t Hq, int64_t max_len, int32_t D) {
    const size_t base = l2kv_decode_workspace_bytes(n_seq, Hq, max_len, D);
    return base == 0 ? 0 : base + ragged_order_bytes(n_seq);
}

l2kv_status l2kv_decode_attn_ragged(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt,
                                    int32_t n_seq, int32_t Hq, int32_t Hkv, int32_t D,
                                    const int32_t* lens, const int64_t* slot_offsets,
                                    const int32_t* seq_order, int64_t total_slots, int64_t max_len,
                                    float scale, int32_t n_splits, float* O, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    if (Q == nullptr || Kc == nullptr || Vc == nullptr || O == nullptr || lens == nullptr ||
        slot_offsets == nullptr)
        return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (n_seq <= 0 || Hq <= 0 || Hkv <= 0 || max_len <= 0 || total_slots <= 0 ||
        total_slots > kMaxTokens || max_len > total_slots || !dim_ok(D, dt))
        return L2KV_ERR_SHAPE;
    if (Hq % Hkv != 0 || Hq / Hkv > max_group(D)) return L2KV_ERR_SHAPE;
    if (static_cast<int64_t>(n_seq) * Hkv > 65535 || static_cast<int64_t>(n_seq) * Hq > 0x7fffffffLL)
        return L2KV_ERR_SHAPE;
    if (n_splits < 0 || n_splits > decode_max_splits(max_len) || !std::isfinite(scale)) return L2KV_ERR_SHAPE;
    if (workspace == nullptr || workspace_bytes < l2kv_decode_ragged_workspace_bytes(n_seq, Hq, max_len, D))
        return L2KV_ERR_WORKSPACE;
    if (!aligned(Q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(O, 4) ||
        !aligned(workspace, 16) || !aligned(lens, 4) || !aligned(slot_offsets, 8) || !aligned(seq_order, 4))
        return L2KV_ERR_ALIGN;
    const float s = scale > 0.f ? scale : 1.0f / std::sqrt(static_cast<float>(D));
    if (seq_order == nullptr && n_splits == 0 && n_seq > 1 && n_seq <= kSelfOrderMaxSeq &&
        max_len >= kSelfOrderMinRows && work_list_rows(dt, D)) {
        // no order from the caller: a longest-first order is worked out here, per call, into the
        // tail of the workspace (a few microseconds; passing a stored order avoids them)
        int32_t* own_order = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) +
                                                        l2kv_decode_workspace_bytes(n_seq, Hq, max_len, D));
        if (l2kv_status st = length_order_dispatch(lens, n_seq, own_order, static_cast<hipStream_t>(stream));
            st != L2KV_OK)
            return st;
        seq_order = own_order;
    }
    const DecodePlan plan = decode_plan_ragged(n_seq, Hkv, max_len, n_splits,
                                               seq_order != nullptr && work_list_rows(dt, D));
    return decode_dispatch(Q, Kc, Vc, dt, n_seq, Hq, Hkv, max_len, D, total_slots * static_cast<int64_t>(D),
                           lens, slot_offsets, seq_order, s, plan, O, workspace,
                           static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_length_order(const int32_t* lens, int32_t n_seq, int32_t* order, void* stream) {
    if (lens == nullptr || order == nullptr) return L2KV_ERR_NULL;
    if (n_seq <= 0 || n_seq > 65535) return L2KV_ERR_SHAPE;
    if (lens == order) return L2KV_ERR_SHAPE;
    if (!aligned(lens, 4) || !aligned(order, 4)) return L2KV_ERR_ALIGN;
    return length_order_dispatch(lens, n_seq, order, static_cast<hipStream_t>(stream));
}

/* ---- attention-loss analysis ---------------------------------------------- */

size_t l2kv_norm_ranks_workspace_bytes(int64_t n_heads, int64_t T) {
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens) return 0;
    return norm_ranks_workspace_bytes(n_heads, T);
}

l2kv_status l2kv_norm_ranks(const float* norms, int64_t n_heads, int64_t T, int32_t* drop_rank,
                            void* workspace, size_t workspace_bytes, void* stream) {
    if (norms == nullptr || drop_rank == nullptr) return L2KV_ERR_NULL;
    if (n_heads <= 0 || n_heads > kMaxHeads || T <= 0 || T > kMaxTokens) return L2KV_ERR_SHAPE;
    if (n_heads > (int64_t{1} << 58) / T) return L2KV_ERR_SHAPE;
    if (workspace == nullptr || workspace_bytes < norm_ranks_workspace_bytes(n_heads, T))
        return L2KV_ERR_WORKSPACE;
    if (!aligned(norms, 4) || !aligned(drop_rank, 4) || !aligned(workspace, 16)) return L2KV_ERR_ALIGN;
    return norm_ranks_dispatch(norms, n_heads, T, drop_rank, workspace, static_cast<hipStream_t>(stream));
}

size_t l2kv_alr_workspace_bytes(int32_t B, int32_t Hq, int64_t T) {
    if (B <= 0 || Hq <= 0 || T <= 0 || T > kMaxTokens) return 0;
    return alr_workspace_bytes(B, Hq, T);
}

l2kv_status l2kv_alr(const void* Q, const void* K, l2kv_dtype dt, const int32_t* drop_rank, int32_t B,
                     int32_t Hq, int32_t Hkv, int64_t T, int32_t D, int64_t k_head_stride, float scale,
                     int64_t m, double* alr, double* loss, double* loss_ref, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (Q == nullptr || K == nullptr || drop_rank == nullptr || alr == nullptr) return L2KV_ERR_NULL;
    if (!dtype_ok(dt)) return L2KV_ERR_DTYPE;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || T <= 0 || T > kMaxTokens || !dim_ok(D, dt)) return L2KV_ERR_SHAPE;
    if (Hq % Hkv != 0 || Hq / Hkv > 8) return L2KV_ERR_SHAPE;
    if (static_cast<int64_t>(B) * Hkv > 65535 || static_cast<int64_t>(B) * Hq > 0x7fffffffLL)
        return L2KV_ERR_SHAPE;
    if (k_head_stride < T * static_cast<int64_t>(D)) return L2KV_ERR_SHAPE;
    if (m < 0 || m > T || !std::isfinite(scale)) return L2KV_ERR_SHAPE;
    if (workspace == nullptr || workspace_bytes < alr_workspace_bytes(B, Hq, T)) return L2KV_ERR_WORKSPACE;
    if ((k_head_stride * elem_bytes(dt)) % 16 != 0) return L2KV_ERR_ALIGN;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(drop_rank, 4) || !aligned(alr, 8) ||
        !aligned(loss, 8) || !aligned(loss_ref, 8) || !aligned(workspace, 16))
        return L2KV_ERR_ALIGN;
    return alr_dispatch(Q, K, dt, drop_rank, B, Hq, Hkv, T, D, k_head_stride, scale, m, alr, loss, loss_ref,
                        workspace, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_read_probe(const void* data, size_t bytes, uint32_t* sink, void* stream) {
    if (data == nullptr || sink == nullptr) return L2KV_ERR_NULL;
    if (!aligned(data, 16) || !aligned(sink, 4)) return L2KV_ERR_ALIGN;
    return read_probe_dispatch(data, bytes, sink, static_cast<hipStream_t>(stream));
}

l2kv_status l2kv_device_info(int32_t* h_compute_units, int32_t* h_memory_clock_khz, int32_t* h_memory_bus_bits) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return L2KV_ERR_LAUNCH;
    }
    const struct { int32_t* out; hipDeviceAttribute_t attr; } want[] = {
        {h_compute_units, hipDeviceAttributeMultiprocessorCount},
        {h_memory_clock_khz, hipDeviceAttributeMemoryClockRate},
        {h_memory_bus_bits, hipDeviceAttributeMemoryBusWidth},
    };
    for (const auto& w : want) {
        if (w.out == nullptr) continue;
        int v = 0;
        if (hipDeviceGetAttribute(&v, w.attr, dev) != hipSuccess) {
            (void)hipGetLastError();
            return L2KV_ERR_LAUNCH;
        }
        *w.out = v;
    }
    return L2KV_OK;
}

const char* l2kv_status_string(l2kv_status s) {
    switch (s) {
        case L2KV_OK: return "ok";
        case L2KV_ERR_NULL: return "a required pointer is NULL";
        case L2KV_ERR_SHAPE: return "unsupported or inconsistent size";
        case L2KV_ERR_DTYPE: return "unsupported dtype";
        case L2KV_ERR_RATIO: return "keep_ratio must be in (0, 1]";
        case L2KV_ERR_WORKSPACE: return "workspace missing or too small";
        case L2KV_ERR_ALIGN: return "pointer or stride alignment violated";
        case L2KV_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int32_t l2kv_version(void) { return 300; }

}  // extern "C"
