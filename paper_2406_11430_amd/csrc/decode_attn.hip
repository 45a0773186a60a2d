// l2kv_decode_attn, host side: decomposition plans, workspace set-up, the scratch array of the
// allocation-free entry point, and the dispatch to the kernels (decode_kernels.hpp, instantiated
// in decode_attn_<type>_<D>.hip).
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

#include <math.h>

#include <atomic>

namespace l2kv {

// Ordered ragged batches (a longest-first order of the sequences is known): from this length
// of the longest sequence on, the (sequence, KV head) pairs are handed out one by one to a fixed
// set of workgroups instead of being launched as a grid.
constexpr int64_t kOrderedMinRows = 2048;
constexpr int64_t kOrderedMaxRows = 16384;   // rows one workgroup takes before a sequence is split

template <typename E, int D>
l2kv_status decode_by_group(int G, const void* Q, const void* Kc, const void* Vc, int32_t B, int32_t Hq,
                            int32_t Hkv, int64_t kv_len, int64_t kv_head_stride, const int32_t* lens,
                            const int64_t* slot_off, const int32_t* seq_order, float scale,
                            const DecodePlan& plan, float* O, void* workspace, hipStream_t stream);
extern template l2kv_status decode_by_group<BF16, 128>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t, int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*, float, const DecodePlan&, float*, void*, hipStream_t);
extern template l2kv_status decode_by_group<BF16, 256>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t, int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*, float, const DecodePlan&, float*, void*, hipStream_t);
extern template l2kv_status decode_by_group<BF16, 64>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t, int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*, float, const DecodePlan&, float*, void*, hipStream_t);
extern template l2kv_status decode_by_group<F32, 128>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t, int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*, float, const DecodePlan&, float*, void*, hipStream_t);
extern template l2kv_status decode_by_group<F32, 64>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t, int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*, float, const DecodePlan&, float*, void*, hipStream_t);

// Zero-fill of a decode workspace as a kernel (callers under graph capture
// cannot record a memset node reliably; a fill kernel is always safe).
__global__ __launch_bounds__(256)
void workspace_fill_kernel(uint4* __restrict__ p, size_t n_vec) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_vec) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

l2kv_status workspace_init_dispatch(void* workspace, size_t bytes, hipStream_t stream) {
    const size_t n_vec = bytes / 16;
    const size_t blocks = (n_vec + 255) / 256;
    if (blocks == 0 || blocks > 0x7fffffffULL) return L2KV_ERR_SHAPE;
    hipLaunchKernelGGL(workspace_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<uint4*>(workspace), n_vec);
    return launch_status();
}

// ---- scratch memory of the allocation-free entry point ----------------------
// Callers that cannot allocate (graph capture, serving loops, harnesses that
// forbid hipMalloc) get the decode workspace from this array instead of from an
// argument.  Every device the library runs on holds its own copy at its own
// address.  On the host the array's name is only a handle for the symbol
// look-up below, never a device address: host code uses the pointer that
// hipGetSymbolAddress returned for the current device, and nothing else.
static __device__ __align__(256) unsigned char scratch[L2KV_STATIC_SCRATCH_BYTES];

void* decode_static_scratch(hipStream_t stream, l2kv_status* status) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> device_ptr[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        *status = L2KV_ERR_LAUNCH;
        return nullptr;
    }
    void* ptr = device_ptr[dev].load(std::memory_order_acquire);
    if (ptr != nullptr) return ptr;
    // First use on this device (which is current): look the array's address up and
    // zero the arrival counters at its start with the fill kernel.  Every later
    // call finds them zero because every decode launch resets the counters it used.
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
        (void)hipGetLastError();
        *status = L2KV_ERR_LAUNCH;
        return nullptr;
    }
    const size_t kCounterRegion = decode_counter_bytes(65535, 1);    // B * Hkv <= 65535 counters
    static_assert(65536 * sizeof(uint32_t) + 256 <= L2KV_STATIC_SCRATCH_BYTES, "scratch smaller than its counter region");
    if (l2kv_status st = workspace_init_dispatch(ptr, kCounterRegion, stream); st != L2KV_OK) {
        *status = st;
        return nullptr;
    }
    device_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}

int32_t decode_max_splits(int64_t kv_len) {
    if (kv_len <= 0) return 0;
    const int64_t by_rows = (kv_len + kDecodeRowTile - 1) / kDecodeRowTile;
    return (int32_t)(by_rows < kDecodeMaxSplits ? by_rows : kDecodeMaxSplits);
}

DecodePlan decode_plan(int32_t B, int32_t Hkv, int32_t group, int64_t kv_len, int32_t requested_splits) {
    const int64_t pairs = (int64_t)B * Hkv;
    int64_t want = requested_splits;
    if (want <= 0) {
        // Workgroups (4 waves each) for about three quarters of the compute units,
        // all resident at once.  Measured over batch sizes 1..16 and cache lengths
        // 4k..32k rows per head, the fastest launch always had 192-200 workgroups
        // on the 256 compute units (e.g. 6 splits x 32 heads: 43.5 us, 8 x 32:
        // 45.3 us, 9 x 32, which no longer fits at once: 65 us); fewer streams in
        // flight use the memory system better than one per compute unit.
        // Query groups of 5 and more heads are bound by arithmetic, not memory,
        // and take every compute unit (8 heads per group: 63 us on 256
        // workgroups, 78 us on 192).
        const int64_t cus = device_compute_units();
        const int64_t target = group >= 5 ? cus : 3 * cus / 4;
        want = (2 * target + pairs) / (2 * pairs);                 // nearest integer to target / pairs
        if (want > 1 && want * pairs > cus) --want;
        // With very few heads that rule asks for so many workgroups per head that
        // the final merge (about 0.2 us per workgroup) outweighs the shorter
        // streams (about 0.025 us per row): the sum is smallest near
        // 0.34 * sqrt(rows) workgroups (measured optima: 32 at 8k rows, 64 at 32k,
        // 128 at 131k with one or two heads).
        int64_t by_merge = (int64_t)(0.34 * sqrt((double)kv_len));
        if (by_merge < 8) by_merge = 8;
        if (want > by_merge) want = by_merge;
    }
    const int64_t cap = decode_max_splits(kv_len);
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    DecodePlan plan;
    plan.n_splits = (int32_t)want;
    plan.rows_per_wg = 1;
    plan.worklist_wgs = 0;
    plan.out_bf16 = 0;
    return plan;
}

DecodePlan decode_plan_ragged(int32_t n_seq, int32_t Hkv, int64_t max_len, int32_t requested_splits,
                              bool ordered) {
    const int64_t pairs = (int64_t)n_seq * Hkv;
    int64_t want = requested_splits;
    const int64_t cap = decode_max_splits(max_len);
    DecodePlan plan;
    plan.worklist_wgs = 0;
    plan.out_bf16 = 0;
    if (ordered && max_len >= kOrderedMinRows) {
        // A longest-first order is known.  One item of the work list is a whole
        // (sequence, KV head) -- only sequences beyond 16k rows, or all of them
        // when the batch has fewer pairs than the uniform rule wants workgroups,
        // are split -- and one workgroup per compute unit draws items from the
        // list.  Measured on the 64-sequence streaming batch (512 pairs of
        // 512..4200 rows): faster than any grid launch of the same batch, whose
        // best (5 workgroups per pair in batch order) took 108 us per layer.
        const int64_t cus = device_compute_units();
        if (want <= 0) {
            const int64_t by_len = (max_len + kOrderedMaxRows - 1) / kOrderedMaxRows;
            const int64_t target = 3 * cus / 4;
            const int64_t by_cu = (2 * target + pairs) / (2 * pairs);
            want = by_len > by_cu ? by_len : by_cu;
        }
        if (want > cap) want = cap;
        if (want < 1) want = 1;
        const int64_t items = pairs * want;
        plan.worklist_wgs = (int32_t)(items < cus ? items : cus);
    } else if (want <= 0) {
        // Lengths differ, so the launch relies on the hardware handing out more
        // workgroups than fit at once: about 1024 rows per workgroup, and never
        // fewer workgroups than compute units.  Workgroups go to the 8 compute
        // dies round-robin by linear id (split + n_splits * pair); an odd
        // n_splits spreads every split index over all dies, which matters here
        // because the high split indices carry less work (measured: 5 splits
        // 108 us, 4 splits 127 us, 8 splits 149 us on the same batch).
        const int64_t by_len = (max_len + 1023) / 1024;
        const int64_t by_cu = (device_compute_units() + pairs - 1) / pairs;
        want = by_len > by_cu ? by_len : by_cu;
        if (want > 1 && want % 2 == 0) want += want < cap ? 1 : -1;
    }
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    plan.n_splits = (int32_t)want;
    // rows per workgroup such that the longest sequence employs all workgroups
    const int64_t rows = (max_len + want - 1) / want;
    plan.rows_per_wg = (int32_t)(rows < kDecodeRowTile ? kDecodeRowTile : rows);
    return plan;
}

l2kv_status decode_dispatch(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                            int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                            int64_t kv_head_stride, const int32_t* lens, const int64_t* slot_off,
                            const int32_t* seq_order, float scale, const DecodePlan& plan, float* O,
                            void* workspace, hipStream_t stream) {
    const int G = Hq / Hkv;
    if (dt == L2KV_F32) {
        return D == 64 ? decode_by_group<F32, 64>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                  lens, slot_off, seq_order, scale, plan, O, workspace, stream)
                       : decode_by_group<F32, 128>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                   lens, slot_off, seq_order, scale, plan, O, workspace, stream);
    }
    if (D == 256)
        return decode_by_group<BF16, 256>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride, lens, slot_off,
                                          seq_order, scale, plan, O, workspace, stream);
    return D == 64 ? decode_by_group<BF16, 64>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                               lens, slot_off, seq_order, scale, plan, O, workspace, stream)
                   : decode_by_group<BF16, 128>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                lens, slot_off, seq_order, scale, plan, O, workspace, stream);
}

}  // namespace l2kv
