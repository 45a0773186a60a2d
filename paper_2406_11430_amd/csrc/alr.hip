// Attention-loss analysis of Sec. 3 on the GPU: for every query head, the
// attention mass lost by dropping m pairs by key norm (Eq. 5), the loss of the
// ideal rule that drops the m lowest attention scores (reference of Eq. 6) and
// the sum over m = 1..T of their gap (Eq. 7).
//
// Sum over m in closed form.  With r(p) = number of pairs the norm rule discards
// before p, pair p is inside the dropped set for T - r(p) values of m, so
//     sum_m L^m     = sum_p a_p (T - r(p)),
//     sum_m L^m,ref = sum_j a_(j) (T - j)       (a_(0) <= a_(1) <= ... ascending),
//     Y             = sum_j a_(j) j - sum_p a_p r(p).
// r depends only on the key norms: it comes from one sort of (norm bits,
// position) per KV head (norm_ranks_kernel) and is shared by all queries.  The
// second term is then a dot product; the first needs the scores of one query in
// ascending order, i.e. one sort of T positive floats per query head.
//
// Both sorts are least-significant-digit radix sorts (4 passes of 8 bits) run by
// one 1024-lane workgroup per head.  Each wavefront owns a contiguous chunk of
// the input; a pass counts digits per wavefront in LDS, turns the 16 x 256 counts
// into start offsets (digit-major, wavefront-minor, which keeps the pass stable)
// and scatters in input order, ranking the 64 keys of a step against each other
// with wave ballots.  Data ping-pongs between two global buffers that stay in
// L2; all waves of a workgroup share one vector L1, so a workgroup barrier is all
// the ordering the passes need.
//
// Unnormalised scores e_p = 2^(s_p - max) are sorted and summed (double
// accumulators, fixed order), and the three results are divided by sum_p e_p at
// the end.
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

namespace l2kv {
namespace {

constexpr int kSortLanes = 1024;
constexpr int kSortWaves = kSortLanes / kWaveSize;
constexpr int kRadixBits = 8;
constexpr int kBins = 1 << kRadixBits;
constexpr int kBatch = 8;            // keys per lane fetched together

struct SortShared {
    uint32_t hist[kSortWaves][kBins];   // per-wave digit counts, then running output offsets
    uint32_t digit_base[kBins];         // first output position of each digit
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// What a pass reads as payload and what it writes.
enum PassKind {
    kKeysOnly,      // keys in, keys out
    kIotaIn,        // payload in = position; (key, payload) out
    kPairs,         // (key, payload) in and out
    kRankOut        // (key, payload) in; writes out_val[payload] = n - 1 - output position
};

// One stable counting pass on digit (key >> shift) & 255 over n keys.  Called by
// all 1024 lanes of the workgroup; leaves a barrier behind it.
template <PassKind KIND>
__device__ void radix_pass(const uint32_t* in_key, const uint32_t* in_val, uint32_t* out_key,
                           uint32_t* out_val, int64_t n, int shift, SortShared& sh) {
    const int lane = threadIdx.x % kWaveSize;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    // contiguous chunk of this wavefront, a multiple of 64 keys
    const int64_t chunk = ((n + kSortWaves - 1) / kSortWaves + kWaveSize - 1) / kWaveSize * kWaveSize;
    const int64_t lo = wave * chunk < n ? wave * chunk : n;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;

    for (int i = threadIdx.x; i < kSortWaves * kBins; i += kSortLanes) (&sh.hist[0][0])[i] = 0u;
    __syncthreads();
    // kBatch independent loads are issued before their first use, so a wavefront
    // pays the L2 latency once per kBatch x 64 keys
    for (int64_t base = lo; base < hi; base += kBatch * kWaveSize) {
        uint32_t key[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int64_t i = base + u * kWaveSize + lane;
            key[u] = i < hi ? in_key[i] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (base + u * kWaveSize + lane < hi) atomicAdd(&sh.hist[wave][(key[u] >> shift) & (kBins - 1)], 1u);
    }
    __syncthreads();

    // counts -> start offsets: within a digit the wavefronts follow each other in
    // input order; digits follow each other in value order
    if (threadIdx.x < kBins) {
        uint32_t run = 0;
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t c = sh.hist[w][threadIdx.x];
            sh.hist[w][threadIdx.x] = run;
            run += c;
        }
        sh.digit_base[threadIdx.x] = run;
    }
    __syncthreads();
    if (wave == 0) {
        uint32_t t[kBins / kWaveSize];
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < kBins / kWaveSize; ++i) {
            t[i] = sh.digit_base[lane * (kBins / kWaveSize) + i];
            sum += t[i];
        }
        uint32_t incl = sum;
#pragma unroll
        for (int off = 1; off < kWaveSize; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        uint32_t run = incl - sum;
#pragma unroll
        for (int i = 0; i < kBins / kWaveSize; ++i) {
            sh.digit_base[lane * (kBins / kWaveSize) + i] = run;
            run += t[i];
        }
    }
    __syncthreads();

    // scatter in input order; hist[wave][d] is private to this wavefront from here on
    volatile uint32_t* my_off = sh.hist[wave];
    for (int64_t base = lo; base < hi; base += kBatch * kWaveSize) {
        uint32_t keys[kBatch], vals[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int64_t i = base + u * kWaveSize + lane;
            const bool valid = i < hi;
            keys[u] = valid ? in_key[i] : 0u;
            vals[u] = 0u;
            if constexpr (KIND == kIotaIn) vals[u] = (uint32_t)i;
            if constexpr (KIND == kPairs || KIND == kRankOut) vals[u] = valid ? in_val[i] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (base + u * kWaveSize >= hi) break;              // same for all lanes of the wavefront
            const bool valid = base + u * kWaveSize + lane < hi;
            const uint32_t key = keys[u], val = vals[u];
            const uint32_t d = (key >> shift) & (kBins - 1);
            uint64_t same = __ballot(valid);                    // lanes holding my digit
#pragma unroll
            for (int b = 0; b < kRadixBits; ++b) {
                const bool bit = (d >> b) & 1u;
                const uint64_t has = __ballot(bit);
                same &= bit ? has : ~has;
            }
            const uint32_t before = lanes_below(same);          // same-digit lanes ahead of me
            const uint32_t count = (uint32_t)__popcll(same);
            const uint32_t off = my_off[d];
            const uint32_t pos = sh.digit_base[d] + off + before;
            if (valid && pos < n && val < n) {                  // counts add up to n, so this always holds
                if constexpr (KIND == kRankOut) {
                    out_val[val] = (uint32_t)(n - 1) - pos;
                } else {
                    out_key[pos] = key;
                    if constexpr (KIND != kKeysOnly) out_val[pos] = val;
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (valid && before + 1 == count) my_off[d] = off + count;   // last lane of the digit advances it
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();
}

// drop_rank[h][t] = T - 1 - (rank of (norm bits, t) in ascending order).
__global__ __launch_bounds__(kSortLanes)
void norm_ranks_kernel(const float* __restrict__ norms, int64_t T, uint32_t* __restrict__ scratch,
                       int32_t* __restrict__ drop_rank) {
    __shared__ SortShared sh;
    const int64_t h = blockIdx.x;
    const uint32_t* keys = reinterpret_cast<const uint32_t*>(norms) + h * T;
    uint32_t* a_key = scratch + h * 4 * T;
    uint32_t* a_val = a_key + T;
    uint32_t* b_key = a_val + T;
    uint32_t* b_val = b_key + T;
    uint32_t* rank = reinterpret_cast<uint32_t*>(drop_rank) + h * T;
    radix_pass<kIotaIn>(keys, nullptr, a_key, a_val, T, 0, sh);
    radix_pass<kPairs>(a_key, a_val, b_key, b_val, T, 8, sh);
    radix_pass<kPairs>(b_key, b_val, a_key, a_val, T, 16, sh);
    radix_pass<kRankOut>(a_key, a_val, nullptr, rank, T, 24, sh);
}

// Scaled logits of all G query heads of one KV head over a block of rows:
// scores[b*Hq + hkv*G + g][t] = (q_g . K_t) * scale * log2(e).
constexpr int kScoreWaves = 4;
constexpr int kScoreLoads = 8;                                        // row loads in flight per lane
constexpr int kScoreRowsPerWave = kScoreLoads * kRowsPerWaveLoad;     // 32
constexpr int kScoreRowsPerBlock = kScoreWaves * kScoreRowsPerWave;   // 128

template <typename E, int D, int G>
__global__ __launch_bounds__(kScoreWaves * kWaveSize)
void alr_scores_kernel(const void* __restrict__ Q, const void* __restrict__ K, int64_t T,
                       int64_t k_head_stride, float scale_log2e, float* __restrict__ scores) {
    using S = Slice<E, D>;
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    const int c = lane % kRowLanes;
    const int r = lane / kRowLanes;
    const int64_t head = blockIdx.y;                                   // b * Hkv + hkv
    const int64_t q_head0 = head * G;                                  // b * Hq + hkv * G
    // q and K rows are shared among the 16 lanes in the same 16-byte pieces (the dot product
    // does not care which lane holds which element)
    using P = Pieces<S::kWords>;
    const char* kbase = static_cast<const char*>(K) + head * k_head_stride * E::kBytes + c * P::kBytes;
    const char* qbase = static_cast<const char*>(Q) + q_head0 * S::kRowBytes + c * P::kBytes;

    float q[G][S::kElems];
#pragma unroll
    for (int g = 0; g < G; ++g) widen<E, D>(load_words<S::kWords, P::kStride>(qbase + (size_t)g * S::kRowBytes), q[g]);

    const int64_t row0 = (int64_t)blockIdx.x * kScoreRowsPerBlock + wave * kScoreRowsPerWave + r;
    Words<S::kWords> tile[kScoreLoads];
#pragma unroll
    for (int u = 0; u < kScoreLoads; ++u) {
        int64_t t = row0 + u * kRowsPerWaveLoad;
        t = t < T ? t : T - 1;                                         // clamped, never stored
        tile[u] = load_words_stream<S::kWords, P::kStride>(kbase + (size_t)t * S::kRowBytes);
    }
#pragma unroll
    for (int u = 0; u < kScoreLoads; ++u) {
        float x[S::kElems];
        widen<E, D>(tile[u], x);
        float mine = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float p = 0.f;
#pragma unroll
            for (int i = 0; i < S::kElems; ++i) p = fmaf(q[g][i], x[i], p);
            p = row16_tree_sum(p);
            mine = c == g ? p : mine;
        }
        const int64_t t = row0 + u * kRowsPerWaveLoad;
        if (c < G && t < T) scores[(q_head0 + c) * T + t] = mine * scale_log2e;
    }
}

// Fixed-order sum of one double per lane over the workgroup; result valid in thread 0.
template <int N>
__device__ void block_sum(double (&v)[N], double (*stage)[N]) {
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
#pragma unroll
    for (int i = 0; i < N; ++i) {
#pragma unroll
        for (int off = kWaveSize / 2; off > 0; off >>= 1) v[i] += __shfl_down(v[i], off);
    }
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) stage[wave][i] = v[i];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            double s = stage[0][i];
            for (int w = 1; w < kSortWaves; ++w) s += stage[w][i];
            v[i] = s;
        }
    }
    __syncthreads();
}

// One workgroup per query head: softmax statistics, rank-weighted sums, sort of
// the scores, and the three outputs.
__global__ __launch_bounds__(kSortLanes)
void alr_head_kernel(uint32_t* __restrict__ scratch, const int32_t* __restrict__ drop_rank, int64_t T,
                     int32_t G, int64_t m, double* __restrict__ alr, double* __restrict__ loss,
                     double* __restrict__ loss_ref) {
    __shared__ SortShared sh;
    __shared__ double stage[kSortWaves][3];
    __shared__ float wave_max[kSortWaves];
    const int64_t head = blockIdx.x;                                   // b * Hq + hq
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    // scratch: two arrays [n_heads][T]; the first holds the logits on entry
    uint32_t* buf0 = scratch + head * T;
    uint32_t* buf1 = scratch + ((int64_t)gridDim.x + head) * T;
    const int32_t* rank = drop_rank + (head / G) * T;

    float mx = -INFINITY;
    for (int64_t t = threadIdx.x; t < T; t += kSortLanes) mx = fmaxf(mx, __builtin_bit_cast(float, buf0[t]));
#pragma unroll
    for (int off = kWaveSize / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) wave_max[wave] = mx;
    __syncthreads();
    mx = wave_max[0];
    for (int w = 1; w < kSortWaves; ++w) mx = fmaxf(mx, wave_max[w]);

    // e_p, their sum, the rank-weighted sum and the mass of the m pairs dropped by norm
    double acc[3] = {0.0, 0.0, 0.0};
    for (int64_t t = threadIdx.x; t < T; t += kSortLanes) {
        const float e = __builtin_amdgcn_exp2f(__builtin_bit_cast(float, buf0[t]) - mx);
        buf0[t] = __builtin_bit_cast(uint32_t, e);
        const int32_t rk = rank[t];
        acc[0] += (double)e;
        acc[1] += (double)e * (double)rk;
        acc[2] += rk < m ? (double)e : 0.0;
    }
    block_sum<3>(acc, stage);           // also orders the e_p stores before the sort
    const double l = acc[0], by_norm = acc[1], lost = acc[2];

    // ascending sort of the e_p (non-negative floats order like their bit patterns)
    radix_pass<kKeysOnly>(buf0, nullptr, buf1, nullptr, T, 0, sh);
    radix_pass<kKeysOnly>(buf1, nullptr, buf0, nullptr, T, 8, sh);
    radix_pass<kKeysOnly>(buf0, nullptr, buf1, nullptr, T, 16, sh);
    radix_pass<kKeysOnly>(buf1, nullptr, buf0, nullptr, T, 24, sh);

    double ref[3] = {0.0, 0.0, 0.0};
    for (int64_t j = threadIdx.x; j < T; j += kSortLanes) {
        const double e = (double)__builtin_bit_cast(float, buf0[j]);
        ref[0] += e * (double)j;
        ref[1] += j < m ? e : 0.0;
    }
    block_sum<3>(ref, stage);
    if (threadIdx.x == 0) {
        alr[head] = (ref[0] - by_norm) / l;
        if (loss != nullptr) loss[head] = lost / l;
        if (loss_ref != nullptr) loss_ref[head] = ref[1] / l;
    }
}

template <typename E, int D>
l2kv_status launch_scores(const void* Q, const void* K, int32_t B, int32_t Hkv, int32_t G, int64_t T,
                          int64_t k_head_stride, float scale_log2e, float* scores, hipStream_t stream) {
    const dim3 grid((unsigned)((T + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock), (unsigned)(B * Hkv));
    const dim3 block(kScoreWaves * kWaveSize);
#define L2KV_SCORES(GG)                                                                             \
    case GG:                                                                                        \
        hipLaunchKernelGGL((alr_scores_kernel<E, D, GG>), grid, block, 0, stream, Q, K, T,          \
                           k_head_stride, scale_log2e, scores);                                     \
        break;
    switch (G) {
        L2KV_SCORES(1) L2KV_SCORES(2) L2KV_SCORES(3) L2KV_SCORES(4)
        L2KV_SCORES(5) L2KV_SCORES(6) L2KV_SCORES(7) L2KV_SCORES(8)
        default: return L2KV_ERR_SHAPE;
    }
#undef L2KV_SCORES
    return launch_status();
}

}  // namespace

size_t norm_ranks_workspace_bytes(int64_t n_heads, int64_t T) {
    const size_t raw = (size_t)n_heads * (size_t)T * 4 * sizeof(uint32_t);
    return (raw + 255) / 256 * 256;
}

size_t alr_workspace_bytes(int32_t B, int32_t Hq, int64_t T) {
    const size_t raw = (size_t)B * (size_t)Hq * (size_t)T * 2 * sizeof(uint32_t);
    return (raw + 255) / 256 * 256;
}

l2kv_status norm_ranks_dispatch(const float* norms, int64_t n_heads, int64_t T, int32_t* drop_rank,
                                void* workspace, hipStream_t stream) {
    hipLaunchKernelGGL(norm_ranks_kernel, dim3((unsigned)n_heads), dim3(kSortLanes), 0, stream, norms, T,
                       static_cast<uint32_t*>(workspace), drop_rank);
    return launch_status();
}

l2kv_status alr_dispatch(const void* Q, const void* K, l2kv_dtype dt, const int32_t* drop_rank, int32_t B,
                         int32_t Hq, int32_t Hkv, int64_t T, int32_t D, int64_t k_head_stride, float scale,
                         int64_t m, double* alr, double* loss, double* loss_ref, void* workspace,
                         hipStream_t stream) {
    const int32_t G = Hq / Hkv;
    const float s = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    const float scale_log2e = s * 1.44269504088896340736f;
    float* scores = static_cast<float*>(workspace);
    l2kv_status st;
    if (dt == L2KV_BF16 && D == 256)
        st = launch_scores<BF16, 256>(Q, K, B, Hkv, G, T, k_head_stride, scale_log2e, scores, stream);
    else if (dt == L2KV_BF16)
        st = D == 128 ? launch_scores<BF16, 128>(Q, K, B, Hkv, G, T, k_head_stride, scale_log2e, scores, stream)
                      : launch_scores<BF16, 64>(Q, K, B, Hkv, G, T, k_head_stride, scale_log2e, scores, stream);
    else
        st = D == 128 ? launch_scores<F32, 128>(Q, K, B, Hkv, G, T, k_head_stride, scale_log2e, scores, stream)
                      : launch_scores<F32, 64>(Q, K, B, Hkv, G, T, k_head_stride, scale_log2e, scores, stream);
    if (st != L2KV_OK) return st;
    hipLaunchKernelGGL(alr_head_kernel, dim3((unsigned)(B * Hq)), dim3(kSortLanes), 0, stream,
                       static_cast<uint32_t*>(workspace), drop_rank, T, G, m, alr, loss, loss_ref);
    return launch_status();
}

}  // namespace l2kv
