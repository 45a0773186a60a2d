// Host-side glue between the C ABI (api.hip) and the per-kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/l2kv.h"

namespace l2kv {

// Status of the launch just enqueued on the calling thread.
inline l2kv_status launch_status() {
    return hipGetLastError() == hipSuccess ? L2KV_OK : L2KV_ERR_LAUNCH;
}

// Compute units of the current device (cached per device id).
int device_compute_units();

l2kv_status read_probe_dispatch(const void* data, size_t bytes, uint32_t* sink, hipStream_t stream);
l2kv_status norms_dispatch(const void* K, l2kv_dtype dt, int64_t n_heads, int64_t T, int32_t D,
                           int64_t head_stride, float* norms, bool keep_in_cache, hipStream_t stream);

l2kv_status select_dispatch(const float* norms, int64_t n_heads, int64_t T, int64_t k,
                            l2kv_mode mode, int32_t* kept_idx, int32_t* kept_count,
                            void* workspace, hipStream_t stream);

l2kv_status random_keys_dispatch(int64_t n_heads, int64_t T, uint32_t seed, float* keys, hipStream_t stream);

l2kv_status compact_dispatch(const void* K, const void* V, l2kv_dtype dt, const int32_t* kept_idx,
                             int64_t n_heads, int64_t T, int64_t k, int32_t D, int64_t head_stride,
                             void* Kc, void* Vc, hipStream_t stream);

// Decomposition of decode attention over the kv_len rows of a KV head:
// n_splits workgroups take turns on consecutive 64-row blocks.
struct DecodePlan {
    int32_t n_splits;        // workgroups launched per KV head
    int32_t rows_per_wg;     // ragged batches: a sequence of n rows employs ceil(n / rows_per_wg) of them
    int32_t worklist_wgs;    // > 0: ordered ragged batch, this many workgroups draw items from a device-side list
    int32_t out_bf16;        // 1: O is written as bf16 (16-bit elements behind the float pointer), 0: fp32
};
constexpr int kDecodeMaxSplits = 256;
constexpr int kDecodeRowTile = 64;   // rows one workgroup consumes per step (4 waves x 16)
int32_t decode_max_splits(int64_t kv_len);
// The decode workspace starts with one arrival counter per (sequence, KV head)
// and the two words of the work queue of ordered ragged launches, padded to
// 256 bytes; the split partials follow.
inline size_t decode_counter_bytes(int32_t B, int32_t Hkv) {
    const size_t raw = (static_cast<size_t>(B) * static_cast<size_t>(Hkv) + 2) * sizeof(uint32_t);
    return (raw + 255) / 256 * 256;
}
// One split partial = D accumulator floats, the running maximum, the denominator and two floats
// of padding, so that every partial row starts on a 16-byte boundary and belongs to one workgroup.
inline size_t decode_partial_floats(int32_t D) { return static_cast<size_t>(D) + 4; }
l2kv_status workspace_init_dispatch(void* workspace, size_t bytes, hipStream_t stream);
// Device address of the library's own scratch array on the current device (set up on first use,
// which enqueues one fill kernel on `stream`); nullptr with *status set on failure.
void* decode_static_scratch(hipStream_t stream, l2kv_status* status);
DecodePlan decode_plan(int32_t B, int32_t Hkv, int32_t group, int64_t kv_len, int32_t requested_splits);
DecodePlan decode_plan_ragged(int32_t n_seq, int32_t Hkv, int64_t max_len, int32_t requested_splits,
                              bool ordered);

// lens / slot_off NULL: uniform batch (kv_len rows per slab, slabs kv_head_stride apart).
// Otherwise ragged: cache [Hkv][total_slots][D], kv_head_stride = total_slots * D,
// kv_len = longest sequence (sizes the decomposition only); seq_order (may be NULL): the
// order in which the sequences are launched.
l2kv_status decode_dispatch(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                            int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                            int64_t kv_head_stride, const int32_t* lens, const int64_t* slot_off,
                            const int32_t* seq_order, float scale, const DecodePlan& plan, float* O,
                            void* workspace, hipStream_t stream);

// Ragged selection / compaction and the streaming slot cache (stream.hip, select.hip).
l2kv_status select_ragged_dispatch(const float* norms, int32_t n_planes, int32_t n_seq,
                                   int64_t total_tokens, const int64_t* in_off, const int64_t* out_off,
                                   int64_t total_kept, int64_t max_len, l2kv_mode mode,
                                   int32_t* kept_idx, hipStream_t stream);
l2kv_status compact_ragged_dispatch(const void* K, const void* V, const float* norms, l2kv_dtype dt,
                                    const int32_t* kept_idx, int32_t n_planes, int32_t n_seq,
                                    int64_t total_tokens, const int64_t* in_off, const int64_t* out_off,
                                    int64_t total_kept, int64_t max_kept, const int64_t* slot_off,
                                    int64_t total_slots, int32_t D, void* Kc, void* Vc, float* norms_c,
                                    int32_t* pos_c, hipStream_t stream);
l2kv_status stream_append_dispatch(const void* Knew, const void* Vnew, l2kv_dtype dt, int32_t n_layers,
                                   int32_t n_seq, int32_t Hkv, int32_t D, const int32_t* token_ids,
                                   const int64_t* slot_off, int64_t total_slots, const int32_t* lens_in,
                                   int32_t* lens_out, void* Kc, void* Vc, float* norms_c, int32_t* pos_c,
                                   hipStream_t stream);
l2kv_status length_order_dispatch(const int32_t* lens, int32_t n_seq, int32_t* order, hipStream_t stream);
l2kv_status stream_evict_dispatch(l2kv_dtype dt, int32_t n_planes, int32_t n_seq, int32_t D,
                                  const int64_t* slot_off, int64_t total_slots, const int32_t* lens_in,
                                  const int32_t* budgets, int32_t* lens_out, void* Kc, void* Vc,
                                  float* norms_c, int32_t* pos_c, hipStream_t stream);

// Attention-loss analysis (alr.hip).
size_t norm_ranks_workspace_bytes(int64_t n_heads, int64_t T);
size_t alr_workspace_bytes(int32_t B, int32_t Hq, int64_t T);
l2kv_status norm_ranks_dispatch(const float* norms, int64_t n_heads, int64_t T, int32_t* drop_rank,
                                void* workspace, hipStream_t stream);
l2kv_status alr_dispatch(const void* Q, const void* K, l2kv_dtype dt, const int32_t* drop_rank, int32_t B,
                         int32_t Hq, int32_t Hkv, int64_t T, int32_t D, int64_t k_head_stride, float scale,
                         int64_t m, double* alr, double* loss, double* loss_ref, void* workspace,
                         hipStream_t stream);

}  // namespace l2kv
