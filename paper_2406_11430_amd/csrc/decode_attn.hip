// l2kv_decode_attn: single-query attention over the compacted cache
// (arXiv 2406.11430, Eq. 2 in the decode form of Eq. 4).  This is the step the
// paper's motivation is about: every decode step re-reads the whole cache from
// HBM, so the kernel is a read stream of Kc and Vc with the arithmetic folded
// in, and the scores never touch memory.
//
// Decomposition: grid (row range, sequence x KV head).  A workgroup of 4 waves
// streams its row range once for all G = Hq/Hkv query heads of the KV head.
// 16 lanes share a row (16 bytes each), a wave covers 16 rows of K and of V
// per step (4 + 4 loads per lane) and prefetches the next step's rows before
// computing on the current ones.  Every 16-lane row group runs its own online
// softmax (running max m, denominator l, weighted value sum acc), so the only
// cross-lane traffic in the loop is the 4-step DPP tree of each dot product.
// At the end the 16 row groups of the workgroup are merged through LDS and one
// partial (acc[D], m, l) per query head is written; a second small kernel
// merges the partials of all row ranges and normalises.
//
// Scores are kept in the log2 domain: q is pre-multiplied by scale*log2(e) so
// the exponentials are bare v_exp_f32.
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

#include <math.h>

namespace l2kv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWaveSize;                 // 4
constexpr int kDecLoads = 4;                                        // row loads per lane per step
constexpr int kDecRowsPerStep = kDecLoads * kRowsPerWaveLoad;       // 16 rows per wave step
constexpr int kDecGroups = kDecWaves * kRowsPerWaveLoad;            // 16 row groups per workgroup
static_assert(kDecWaves * kDecRowsPerStep == kDecodeRowTile, "row tile mismatch");

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename E, int D>
struct Tile {
    Words<Slice<E, D>::kWords> k[kDecLoads];
    Words<Slice<E, D>::kWords> v[kDecLoads];
};

template <typename E, int D>
__device__ __forceinline__ void load_tile(Tile<E, D>& t, const char* Kh, const char* Vh,
                                          int64_t first_row, int64_t last_valid, int rg, int c) {
    using S = Slice<E, D>;
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) {
        int64_t row = first_row + u * kRowsPerWaveLoad + rg;
        row = row < last_valid ? row : last_valid;       // tail rows re-read the last row; masked later
        const int64_t off = row * S::kRowBytes + c * S::kBytes;
        t.k[u] = load_words<S::kWords>(Kh + off);
    }
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) {
        int64_t row = first_row + u * kRowsPerWaveLoad + rg;
        row = row < last_valid ? row : last_valid;
        const int64_t off = row * S::kRowBytes + c * S::kBytes;
        t.v[u] = load_words<S::kWords>(Vh + off);
    }
}

// partial layout: [B*Hq][n_splits][D + 2] floats: acc[0..D), m (log2 domain), l.
template <typename E, int D, int G>
__global__ __launch_bounds__(kDecThreads)
void decode_partial_kernel(const char* __restrict__ Q, const char* __restrict__ Kc,
                           const char* __restrict__ Vc, int Hkv, int64_t kv_len,
                           int64_t head_stride_bytes, int64_t rows_per_split, int n_splits,
                           float scale_log2e, float* __restrict__ partial) {
    using S = Slice<E, D>;
    constexpr int EPL = S::kElems;
    constexpr float kNegInf = -INFINITY;
    __shared__ float s_acc[kDecGroups][G][D];
    __shared__ float s_m[kDecGroups][G];
    __shared__ float s_l[kDecGroups][G];

    const int split = blockIdx.x;
    const int pair = blockIdx.y;                 // b * Hkv + hkv
    const int b = pair / Hkv;
    const int hkv = pair % Hkv;
    const int Hq = Hkv * G;
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    const int c = lane % kRowLanes;
    const int rg = lane / kRowLanes;

    // This lane's slice of the G query rows, pre-scaled into the log2 domain.
    float q[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int64_t hq = (int64_t)b * Hq + (int64_t)hkv * G + g;
        Words<S::kWords> raw = load_words<S::kWords>(Q + hq * S::kRowBytes + c * S::kBytes);
        widen<E, D>(raw, q[g]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) q[g][e] *= scale_log2e;
    }

    const int64_t r0 = (int64_t)split * rows_per_split;
    const int64_t r1 = (r0 + rows_per_split < kv_len) ? r0 + rows_per_split : kv_len;
    const int64_t n_steps = (r1 - r0 + kDecRowsPerStep - 1) / kDecRowsPerStep;
    const char* Kh = Kc + (int64_t)pair * head_stride_bytes;
    const char* Vh = Vc + (int64_t)pair * head_stride_bytes;

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegInf;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    auto consume = [&](const Tile<E, D>& t, int64_t first_row) {
        float s[G][kDecLoads];
#pragma unroll
        for (int u = 0; u < kDecLoads; ++u) {
            float kx[EPL];
            widen<E, D>(t.k[u], kx);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float a = q[g][0] * kx[0];
#pragma unroll
                for (int e = 1; e < EPL; ++e) a = fmaf(q[g][e], kx[e], a);
                s[g][u] = a;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) s[g][u] = row16_tree_sum(s[g][u]);
        if (first_row + kDecRowsPerStep > r1) {          // wave-uniform: only the ragged last step
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) {
                const bool valid = first_row + u * kRowsPerWaveLoad + rg < r1;
#pragma unroll
                for (int g = 0; g < G; ++g) s[g][u] = valid ? s[g][u] : kNegInf;
            }
        }
        float p[G][kDecLoads];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mn = m[g];
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) mn = fmaxf(mn, s[g][u]);
            const float ms = mn == kNegInf ? 0.f : mn;   // group has seen no valid row yet
            const float alpha = fast_exp2(m[g] - ms);
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) {
                p[g][u] = fast_exp2(s[g][u] - ms);
                psum += p[g][u];
            }
            l[g] = fmaf(l[g], alpha, psum);
            m[g] = mn;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < kDecLoads; ++u) {
            float vx[EPL];
            widen<E, D>(t.v[u], vx);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p[g][u], vx[e], acc[g][e]);
        }
    };

    // Software pipeline: the loads of step j+kDecWaves are issued before the
    // arithmetic of step j.
    if (wave < n_steps) {
        Tile<E, D> cur, nxt;
        int64_t j = wave;
        load_tile<E, D>(cur, Kh, Vh, r0 + j * kDecRowsPerStep, r1 - 1, rg, c);
        while (true) {
            const int64_t jn = j + kDecWaves;
            const bool more = jn < n_steps;
            if (more) load_tile<E, D>(nxt, Kh, Vh, r0 + jn * kDecRowsPerStep, r1 - 1, rg, c);
            consume(cur, r0 + j * kDecRowsPerStep);
            if (!more) break;
            cur = nxt;
            j = jn;
        }
    }

    // ---- merge the 16 row groups of the workgroup through LDS --------------
    const int grp = wave * kRowsPerWaveLoad + rg;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[grp][g][c * EPL + e] = acc[g][e];
        if (c == 0) {
            s_m[grp][g] = m[g];
            s_l[grp][g] = l[g];
        }
    }
    __syncthreads();
    for (int o = threadIdx.x; o < G * D; o += kDecThreads) {
        const int g = o / D;
        const int d = o % D;
        float mx = kNegInf;
#pragma unroll
        for (int i = 0; i < kDecGroups; ++i) mx = fmaxf(mx, s_m[i][g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int i = 0; i < kDecGroups; ++i) {
            const float mi = s_m[i][g];
            const float w = mi == kNegInf ? 0.f : fast_exp2(mi - mx);
            num = fmaf(w, s_acc[i][g][d], num);
            den = fmaf(w, s_l[i][g], den);
        }
        const int64_t hq = (int64_t)b * Hq + (int64_t)hkv * G + g;
        float* out = partial + (hq * n_splits + split) * (D + 2);
        out[d] = num;
        if (d == 0) {
            out[D] = mx;
            out[D + 1] = den;
        }
    }
}

template <int D>
__global__ __launch_bounds__(D)
void decode_merge_kernel(const float* __restrict__ partial, int n_splits, float* __restrict__ O) {
    const int64_t hq = blockIdx.x;               // b * Hq + hq
    const int d = threadIdx.x;
    const float* p = partial + hq * n_splits * (D + 2);
    float mx = -INFINITY;
    for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, p[s * (D + 2) + D]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float w = fast_exp2(p[s * (D + 2) + D] - mx);   // every launched range has >= 1 row
        num = fmaf(w, p[s * (D + 2) + d], num);
        den = fmaf(w, p[s * (D + 2) + D + 1], den);
    }
    O[hq * D + d] = num / den;
}

int32_t decode_max_splits(int64_t kv_len) {
    if (kv_len <= 0) return 0;
    const int64_t by_rows = (kv_len + kDecodeRowTile - 1) / kDecodeRowTile;
    return (int32_t)(by_rows < kDecodeMaxSplits ? by_rows : kDecodeMaxSplits);
}

DecodePlan decode_plan(int32_t B, int32_t Hkv, int64_t kv_len, int32_t requested_splits) {
    const int64_t pairs = (int64_t)B * Hkv;
    int64_t want = requested_splits;
    if (want <= 0) {
        // Two resident workgroups per compute unit, all started in one wave of
        // the grid so every range finishes at about the same time.
        const int64_t target = 2LL * device_compute_units();
        want = (target + pairs - 1) / pairs;
    }
    const int64_t cap = decode_max_splits(kv_len);
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    int64_t rps = (kv_len + want - 1) / want;
    rps = (rps + kDecodeRowTile - 1) / kDecodeRowTile * kDecodeRowTile;
    DecodePlan plan;
    plan.rows_per_split = rps;
    plan.n_splits = (int32_t)((kv_len + rps - 1) / rps);
    return plan;
}

template <typename E, int D, int G>
static l2kv_status launch_decode(const void* Q, const void* Kc, const void* Vc, int32_t B, int32_t Hq,
                                 int32_t Hkv, int64_t kv_len, int64_t kv_head_stride, float scale,
                                 const DecodePlan& plan, float* O, float* workspace,
                                 hipStream_t stream) {
    const float scale_log2e = scale * 1.4426950408889634f;
    dim3 grid((unsigned)plan.n_splits, (unsigned)(B * Hkv));
    hipLaunchKernelGGL((decode_partial_kernel<E, D, G>), grid, dim3(kDecThreads), 0, stream,
                       static_cast<const char*>(Q), static_cast<const char*>(Kc),
                       static_cast<const char*>(Vc), (int)Hkv, kv_len,
                       kv_head_stride * (int64_t)E::kBytes, plan.rows_per_split, (int)plan.n_splits,
                       scale_log2e, workspace);
    if (hipGetLastError() != hipSuccess) return L2KV_ERR_LAUNCH;
    hipLaunchKernelGGL((decode_merge_kernel<D>), dim3((unsigned)(B * Hq)), dim3(D), 0, stream,
                       workspace, (int)plan.n_splits, O);
    return launch_status();
}

template <typename E, int D>
static l2kv_status decode_by_group(int G, const void* Q, const void* Kc, const void* Vc, int32_t B,
                                   int32_t Hq, int32_t Hkv, int64_t kv_len, int64_t kv_head_stride,
                                   float scale, const DecodePlan& plan, float* O, float* workspace,
                                   hipStream_t stream) {
#define L2KV_G(N)                                                                                   \
    case N:                                                                                         \
        return launch_decode<E, D, N>(Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride, scale, plan, O, \
                                      workspace, stream)
    switch (G) {
        L2KV_G(1); L2KV_G(2); L2KV_G(3); L2KV_G(4); L2KV_G(5); L2KV_G(6); L2KV_G(7); L2KV_G(8);
    }
#undef L2KV_G
    return L2KV_ERR_SHAPE;
}

l2kv_status decode_dispatch(const void* Q, const void* Kc, const void* Vc, l2kv_dtype dt, int32_t B,
                            int32_t Hq, int32_t Hkv, int64_t kv_len, int32_t D,
                            int64_t kv_head_stride, float scale, const DecodePlan& plan, float* O,
                            float* workspace, hipStream_t stream) {
    const int G = Hq / Hkv;
    if (dt == L2KV_F32) {
        return D == 64 ? decode_by_group<F32, 64>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                  scale, plan, O, workspace, stream)
                       : decode_by_group<F32, 128>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                   scale, plan, O, workspace, stream);
    }
    return D == 64 ? decode_by_group<BF16, 64>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                               scale, plan, O, workspace, stream)
                   : decode_by_group<BF16, 128>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                scale, plan, O, workspace, stream);
}

}  // namespace l2kv
