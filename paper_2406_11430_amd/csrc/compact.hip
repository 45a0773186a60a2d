// l2kv_compact: gather of the kept K and V rows into dense caches (arXiv
// 2406.11430 Sec. 1: the lowest-norm keys are kept, each with its value).
//
// A byte copy of whole rows: 16 lanes move one row (16 bytes per lane and
// instruction: one piece of a 256-byte row, pieces c and c + 16 of a 512-byte
// row), a wavefront moves 4 rows per instruction, and each row group handles kUnroll consecutive output rows so
// all index loads, then all row loads of K and V, are in flight before the
// first store.  Loads and stores carry the non-temporal hint (every byte is
// touched once).  Dropped rows are never read.
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

namespace l2kv {

constexpr int kCompactThreads = 256;
constexpr int kCompactWaves = kCompactThreads / kWaveSize;
#ifndef L2KV_COMPACT_UNROLL
#define L2KV_COMPACT_UNROLL 4
#endif
constexpr int kCompactUnroll = L2KV_COMPACT_UNROLL;
constexpr int kCompactRowsPerBlock = kCompactWaves * kRowsPerWaveLoad * kCompactUnroll;  // 64

// W = 32-bit words per lane slice (row bytes = 16 lanes * 4W).
template <int W, bool HAS_V>
__global__ __launch_bounds__(kCompactThreads)
void compact_kernel(const char* __restrict__ K, const char* __restrict__ V,
                    const int32_t* __restrict__ kept_idx, int64_t T, int64_t k, int64_t head_stride_bytes,
                    int64_t blocks_per_head, char* __restrict__ Kc, char* __restrict__ Vc) {
    using P = Pieces<W>;
    constexpr int64_t kRowBytes = kRowLanes * 4 * W;
    const int64_t head = blockIdx.x / blocks_per_head;
    const int64_t chunk = blockIdx.x % blocks_per_head;
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    const int c = lane % kRowLanes;
    const int rg = lane / kRowLanes;

    const int64_t first = chunk * kCompactRowsPerBlock + (wave * kRowsPerWaveLoad + rg) * kCompactUnroll;
    const int32_t* idx = kept_idx + head * k;
    const int64_t src_head = head * head_stride_bytes;
    const int64_t dst_head = head * k * kRowBytes;

    int64_t src[kCompactUnroll];
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
        int64_t j = first + u;
        j = j < k ? j : k - 1;            // tail: duplicate the last row, store skipped
        int64_t t = idx[j];
        t = t < 0 ? 0 : (t < T ? t : T - 1);          // an index outside [0, T) cannot lead out of the head
        src[u] = src_head + t * kRowBytes + c * P::kBytes;
    }
    Words<W> kr[kCompactUnroll], vr[kCompactUnroll];
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) kr[u] = load_words_stream<W, P::kStride>(K + src[u]);
    if constexpr (HAS_V) {
#pragma unroll
        for (int u = 0; u < kCompactUnroll; ++u) vr[u] = load_words_stream<W, P::kStride>(V + src[u]);
    }
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
        const int64_t j = first + u;
        if (j < k) {
            const int64_t dst = dst_head + j * kRowBytes + c * P::kBytes;
            store_words_stream<W, P::kStride>(Kc + dst, kr[u]);
            if constexpr (HAS_V) store_words_stream<W, P::kStride>(Vc + dst, vr[u]);
        }
    }
}

template <int W>
static l2kv_status launch_compact(const void* K, const void* V, const int32_t* kept_idx,
                                  int64_t n_heads, int64_t T, int64_t k, int64_t head_stride_bytes,
                                  void* Kc, void* Vc, hipStream_t stream) {
    const int64_t bph = (k + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    const int64_t blocks = bph * n_heads;
    if (blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
    if (V != nullptr) {
        hipLaunchKernelGGL((compact_kernel<W, true>), dim3((unsigned)blocks), dim3(kCompactThreads), 0,
                           stream, static_cast<const char*>(K), static_cast<const char*>(V), kept_idx,
                           T, k, head_stride_bytes, bph, static_cast<char*>(Kc), static_cast<char*>(Vc));
    } else {
        hipLaunchKernelGGL((compact_kernel<W, false>), dim3((unsigned)blocks), dim3(kCompactThreads), 0,
                           stream, static_cast<const char*>(K), static_cast<const char*>(nullptr),
                           kept_idx, T, k, head_stride_bytes, bph, static_cast<char*>(Kc),
                           static_cast<char*>(nullptr));
    }
    return launch_status();
}

l2kv_status compact_dispatch(const void* K, const void* V, l2kv_dtype dt, const int32_t* kept_idx,
                             int64_t n_heads, int64_t T, int64_t k, int32_t D, int64_t head_stride,
                             void* Kc, void* Vc, hipStream_t stream) {
    const int es = dt == L2KV_F32 ? 4 : 2;
    const int row_bytes = D * es;                      // 128, 256 or 512
    const int64_t hs_bytes = head_stride * es;
    switch (row_bytes) {
        case 128: return launch_compact<2>(K, V, kept_idx, n_heads, T, k, hs_bytes, Kc, Vc, stream);
        case 256: return launch_compact<4>(K, V, kept_idx, n_heads, T, k, hs_bytes, Kc, Vc, stream);
        case 512: return launch_compact<8>(K, V, kept_idx, n_heads, T, k, hs_bytes, Kc, Vc, stream);
    }
    return L2KV_ERR_SHAPE;
}

}  // namespace l2kv
