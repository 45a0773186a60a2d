// l2kv_decode_attn: single-query attention over the compacted cache
// (arXiv 2406.11430, Eq. 2 in the decode form of Eq. 4).  This is the step the
// paper's motivation is about: every decode step re-reads the whole cache from
// HBM, so the kernel is a read stream of Kc and Vc with the arithmetic folded
// in, and the scores never touch memory.
//
// Decomposition: grid (split, sequence x KV head).  The n_splits workgroups of a
// KV head take turns on consecutive 64-row blocks of its cache and stream them
// once for all G = Hq/Hkv query heads.  16 lanes share a row (16 bytes each),
// a wave covers 16 rows of K and of V per step (4 + 4 non-temporal loads per
// lane) and always has its next tile in flight while it computes on the
// current one (two register tiles, ping-pong, no branch between a load and its
// use so the wait counters stay exact).  Every 16-lane row group runs its own
// online softmax (running max m, denominator l, weighted value sum acc), so the
// only cross-lane traffic in the loop is the 4-step DPP tree of each dot
// product.
//
// bf16 caches: q.k uses the packed bf16 dot instruction with fp32 accumulate
// (both operands are exact bf16 inputs); the softmax scale is applied to the
// fp32 score afterwards.  fp32 caches use plain fp32 FMAs.
//
// At the end the 16 row groups of the workgroup are merged through LDS and one
// partial (acc[D], m, l) per query head goes to the workspace.  The workgroup
// that finishes last for its KV head (device-scope counter in the workspace)
// merges the partials of all workgroups and writes O: one kernel per call.
//
// Scores are kept in the log2 domain so the exponentials are bare v_exp_f32.
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

#include <math.h>

#include <atomic>

namespace l2kv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWaveSize;                 // 4
constexpr int kDecLoads = 4;                                        // row loads per lane per step
constexpr int kDecRowsPerStep = kDecLoads * kRowsPerWaveLoad;       // 16 rows per wave step
constexpr int kDecGroups = kDecWaves * kRowsPerWaveLoad;            // 16 row groups per workgroup
// Ordered ragged batches: from this length of the longest sequence on, one workgroup per compute
// unit is kept resident by requesting this much unused LDS (more than half of the 160 KiB).
constexpr int64_t kOrderedMinRows = 2048;
constexpr int64_t kOrderedMaxRows = 16384;   // rows one workgroup takes before a sequence is split
constexpr int32_t kOrderedLdsPad = 80 * 1024;
static_assert(kDecWaves * kDecRowsPerStep == kDecodeRowTile, "row tile mismatch");

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// K and V are read once per call: streaming loads, nothing to keep in L2.
template <int W>
__device__ __forceinline__ Words<W> stream_words(const char* p) { return load_words_stream<W>(p); }

// s_waitcnt immediate for "vmcnt(0)" alone on gfx9-family encodings: vmcnt in bits
// [3:0] and [15:14] = 0, expcnt [6:4] and lgkmcnt [11:8] left at their maxima.
constexpr int kWaitVmcnt0 = 0x0F70;

// Device-scope (agent) relaxed store / load of one float.
__device__ __forceinline__ void publish(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float fetch(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename E, int D>
struct Tile {
    Words<Slice<E, D>::kWords> k[kDecLoads];
    Words<Slice<E, D>::kWords> v[kDecLoads];
};

// Loads the 16 rows [first_row, first_row+16) of K and V for this lane; all 16
// rows must exist.  lane_off = rg * row_bytes + c * slice_bytes.
template <typename E, int D>
__device__ __forceinline__ void load_tile(Tile<E, D>& t, const char* Kh, const char* Vh,
                                          int64_t first_row, int lane_off) {
    using S = Slice<E, D>;
    const int64_t off = first_row * S::kRowBytes + lane_off;
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u)
        t.k[u] = stream_words<S::kWords>(Kh + off + u * (kRowsPerWaveLoad * S::kRowBytes));
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u)
        t.v[u] = stream_words<S::kWords>(Vh + off + u * (kRowsPerWaveLoad * S::kRowBytes));
}

// Ragged last tile of a row range: rows past last_valid re-read row last_valid
// (in bounds); the caller masks their scores.
template <typename E, int D>
__device__ __forceinline__ void load_tile_clamped(Tile<E, D>& t, const char* Kh, const char* Vh,
                                                  int64_t first_row, int64_t last_valid, int rg, int c) {
    using S = Slice<E, D>;
    int64_t off[kDecLoads];
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) {
        int64_t row = first_row + u * kRowsPerWaveLoad + rg;
        row = row < last_valid ? row : last_valid;
        off[u] = row * S::kRowBytes + c * S::kBytes;
    }
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) t.k[u] = stream_words<S::kWords>(Kh + off[u]);
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) t.v[u] = stream_words<S::kWords>(Vh + off[u]);
}

// workspace layout: [counters: kDecodeCounterBytes] [partials]
// partials: [B*Hq][n_splits][D + 2] floats: acc[0..D), m (log2 domain), l.
template <typename E, int D, int G>
__global__ __launch_bounds__(kDecThreads)
void decode_kernel(const char* __restrict__ Q, const char* __restrict__ Kc,
                   const char* __restrict__ Vc, int Hkv, int64_t kv_len_uniform,
                   int64_t head_stride_bytes, const int32_t* __restrict__ lens,
                   const int64_t* __restrict__ slot_off, const int32_t* __restrict__ seq_order,
                   int n_splits_grid, int rows_per_wg,
                   float scale_log2e, uint32_t* __restrict__ counters,
                   float* __restrict__ partial, float* __restrict__ O) {
    using S = Slice<E, D>;
    constexpr int EPL = S::kElems;
    constexpr int W = S::kWords;
    constexpr bool kBf16 = E::kBytes == 2;
    constexpr float kNegInf = -INFINITY;
    __shared__ float s_acc[kDecGroups][G][D];
    __shared__ float s_m[kDecGroups][G];
    __shared__ float s_l[kDecGroups][G];
    __shared__ uint32_t s_ticket;

    const int split = blockIdx.x;
    const int pair = blockIdx.y;                 // b * Hkv + hkv
    const int hkv = pair % Hkv;
    // Ragged batches may come with a processing order (longest sequence first):
    // the launch index then names a position in that order, not the sequence.
    int b = pair / Hkv;
    if (seq_order != nullptr) {
        const int n_seq = (int)gridDim.y / Hkv;
        const int ob = seq_order[b];
        b = ob < 0 ? 0 : (ob < n_seq ? ob : n_seq - 1);
    }
    const int Hq = Hkv * G;
    const int lane = threadIdx.x % kWaveSize;
    // the wave index is the same in all 64 lanes: keep it in a scalar register
    // so every branch on row positions below is a scalar branch
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const int c = lane % kRowLanes;
    const int rg = lane / kRowLanes;
    const int64_t hq0 = (int64_t)b * Hq + (int64_t)hkv * G;   // first query head of the group

    // Uniform batch: every (sequence, KV head) slab has kv_len rows and starts
    // pair * head_stride in.  Ragged batch (lens != NULL): the cache is
    // [Hkv][total_slots][D], head_stride is the plane stride, sequence b owns the
    // slots slot_off[b] .. slot_off[b+1]-1 and lens[b] of them are occupied
    // (offsets and length are clamped into the plane, so inconsistent arrays
    // cannot lead outside the cache).  A sequence only employs as many of the
    // launched workgroups as it has blocks of rows_per_wg rows; the others
    // leave at once.
    int64_t kv_len = kv_len_uniform;
    int64_t slab = (int64_t)pair * head_stride_bytes;
    int n_splits = n_splits_grid;
    if (lens != nullptr) {
        const Range slots = clamped_range(slot_off, b, head_stride_bytes / S::kRowBytes);
        kv_len = lens[b];
        kv_len = kv_len < 0 ? 0 : (kv_len > slots.count ? slots.count : kv_len);
        slab = (int64_t)hkv * head_stride_bytes + slots.first * (int64_t)S::kRowBytes;
        const int64_t need = (kv_len + rows_per_wg - 1) / rows_per_wg;
        n_splits = need < 1 ? 1 : (need < n_splits_grid ? (int)need : n_splits_grid);
        if (split >= n_splits) return;
    }

    // This lane's slice of the G query rows: raw bf16 pairs for the packed dot,
    // fp32 values otherwise.  The scale is applied to the reduced score.
    uint32_t qw[G][W];
    float qf[kBf16 ? 1 : G][kBf16 ? 1 : EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        Words<W> raw = load_words<W>(Q + (hq0 + g) * S::kRowBytes + c * S::kBytes);
#pragma unroll
        for (int w = 0; w < W; ++w) qw[g][w] = raw.w[w];
        if constexpr (!kBf16) widen<E, D>(raw, qf[g]);
    }

    const int64_t r1 = kv_len;                   // rows at or past r1 do not exist
    const char* Kh = Kc + slab;
    const char* Vh = Vc + slab;
    const int lane_off = rg * S::kRowBytes + c * S::kBytes;

    float m[G], l[G], acc[G][EPL];    // m: running max of the RAW score (before scaling)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegInf;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    auto consume = [&](const Tile<E, D>& t, int64_t first_row, bool ragged) {
        float s[G][kDecLoads];
#pragma unroll
        for (int u = 0; u < kDecLoads; ++u) {
            if constexpr (kBf16) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float a = dot2_bf16(qw[g][0], t.k[u].w[0], 0.f);
#pragma unroll
                    for (int w = 1; w < W; ++w) a = dot2_bf16(qw[g][w], t.k[u].w[w], a);
                    s[g][u] = a;
                }
            } else {
                float kx[EPL];
                widen<E, D>(t.k[u], kx);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float a = qf[g][0] * kx[0];
#pragma unroll
                    for (int e = 1; e < EPL; ++e) a = fmaf(qf[g][e], kx[e], a);
                    s[g][u] = a;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) s[g][u] = row16_tree_sum(s[g][u]);
        if (ragged) {                                    // only the last, partial tile of a range
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
            // scaled max; 0 while the group has seen no valid row (avoids inf - inf)
            const float ms = mn == kNegInf ? 0.f : mn * scale_log2e;
            const float alpha = fast_exp2(fmaf(m[g], scale_log2e, -ms));
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) {
                p[g][u] = fast_exp2(fmaf(s[g][u], scale_log2e, -ms));
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

    // Work assignment.  The head's rows are cut into 16-row tiles; tile t goes to
    // workgroup (t / 4) % n_splits, wave t % 4: the workgroups of a KV head take
    // turns on consecutive 64-row blocks.  Every workgroup therefore sweeps the
    // whole address range of the head, which evens out the differences in
    // memory distance between compute dies and address ranges that a
    // contiguous range per workgroup would expose.
    //
    // The full tiles run through a ping-pong pipeline: tile i+1 is requested
    // before tile i is consumed, with no branch between a load and its use, so
    // the hardware wait counters stay exact.  The ragged last tile of the head
    // (if any) is handled by its owner afterwards with clamped loads and
    // masked scores.
    {
        const int64_t n_full = kv_len / kDecRowsPerStep;                       // full tiles in the head
        const int64_t first_tile = (int64_t)split * kDecWaves + wave;
        const int64_t tile_stride = (int64_t)n_splits * kDecWaves;
        const int64_t mine = n_full > first_tile ? (n_full - first_tile + tile_stride - 1) / tile_stride : 0;
        const int64_t kStride = tile_stride * kDecRowsPerStep;                 // rows between my tiles
        int64_t row = first_tile * kDecRowsPerStep;
        if (mine > 0) {
            Tile<E, D> ta, tb;
            // The scheduling barriers pin each batch of loads ahead of the
            // arithmetic on the other tile; without them the compiler sinks
            // the loads next to their first use and the prefetch is lost.
            load_tile<E, D>(ta, Kh, Vh, row, lane_off);
            __builtin_amdgcn_sched_barrier(0);
            int64_t left = mine;                       // tiles not yet consumed; ta holds the first
            while (left > 2) {
                load_tile<E, D>(tb, Kh, Vh, row + kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(ta, row, false);
                __builtin_amdgcn_sched_barrier(0);
                load_tile<E, D>(ta, Kh, Vh, row + 2 * kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(tb, row + kStride, false);
                __builtin_amdgcn_sched_barrier(0);
                row += 2 * kStride;
                left -= 2;
            }
            if (left == 2) {
                load_tile<E, D>(tb, Kh, Vh, row + kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(ta, row, false);
                consume(tb, row + kStride, false);
            } else {
                consume(ta, row, false);
            }
        }
        if (kv_len % kDecRowsPerStep != 0 && (n_full / kDecWaves) % n_splits == split &&
            n_full % kDecWaves == wave) {
            Tile<E, D> tt;
            const int64_t first = n_full * kDecRowsPerStep;
            load_tile_clamped<E, D>(tt, Kh, Vh, first, r1 - 1, rg, c);
            consume(tt, first, true);
        }
    }

    // ---- merge the 16 row groups of the workgroup through LDS --------------
    const int grp = wave * kRowsPerWaveLoad + rg;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[grp][g][c * EPL + e] = acc[g][e];
        if (c == 0) {
            s_m[grp][g] = m[g] * scale_log2e;     // -inf stays -inf (scale > 0)
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
        // Device-scope stores: written through to the level every compute unit
        // of the device reads from, so the merging workgroup below sees them
        // without any bulk cache write-back.
        float* out = partial + ((hq0 + g) * n_splits_grid + split) * (D + 2);
        publish(out + d, num);
        if (d == 0) {
            publish(out + D, mx);
            publish(out + D + 1, den);
        }
    }

    // ---- the last workgroup of this KV head merges all row ranges ---------
    // Hand-over protocol: every partial is written with a device-scope store;
    // every wave then waits until its own stores have been acknowledged
    // (vmcnt(0): a workgroup barrier alone does not wait for outstanding global
    // stores, and the ticket below travels to a different memory channel than
    // the partials, so without the wait it could overtake them); after the
    // barrier one lane takes a ticket with a device-scope atomic.  The
    // workgroup that draws the last ticket re-reads all partials with
    // device-scope loads.  No lane ever waits on another workgroup, so nothing
    // here can hang.
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __syncthreads();
    if (threadIdx.x == 0)
        s_ticket = __hip_atomic_fetch_add(&counters[pair], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != (uint32_t)(n_splits - 1)) return;
    // Each lane owns up to kOut output elements (g, d) and fetches, for a batch
    // of workgroups at a time, their accumulator element together with their
    // (m, l): all loads of a batch are independent, so the whole merge costs
    // about one memory round trip per batch (one batch up to 8 workgroups).
    constexpr int kOut = (G * D + kDecThreads - 1) / kDecThreads;
    constexpr int kMergeBatch = 8;
    float num[kOut], den[kOut], mx[kOut];
#pragma unroll
    for (int j = 0; j < kOut; ++j) {
        num[j] = 0.f;
        den[j] = 0.f;
        mx[j] = kNegInf;
    }
    for (int s0 = 0; s0 < n_splits; s0 += kMergeBatch) {
        float v[kOut][kMergeBatch], pm[kOut][kMergeBatch], pl[kOut][kMergeBatch];
#pragma unroll
        for (int j = 0; j < kOut; ++j) {
            const int o = threadIdx.x + j * kDecThreads;
            const int oo = o < G * D ? o : 0;                               // idle lanes re-read element 0
            const int g = oo / D;
            const int d = oo % D;
#pragma unroll
            for (int i = 0; i < kMergeBatch; ++i) {
                const int sp = s0 + i < n_splits ? s0 + i : n_splits - 1;   // clamp: in bounds, ignored below
                const float* p = partial + ((hq0 + g) * n_splits_grid + sp) * (D + 2);
                v[j][i] = fetch(p + d);
                pm[j][i] = fetch(p + D);
                pl[j][i] = fetch(p + D + 1);
            }
        }
#pragma unroll
        for (int j = 0; j < kOut; ++j) {
            float bm = mx[j];
#pragma unroll
            for (int i = 0; i < kMergeBatch; ++i)
                if (s0 + i < n_splits) bm = fmaxf(bm, pm[j][i]);
            const float keep = mx[j] == kNegInf ? 0.f : fast_exp2(mx[j] - bm);
            num[j] *= keep;
            den[j] *= keep;
#pragma unroll
            for (int i = 0; i < kMergeBatch; ++i) {
                if (s0 + i < n_splits) {
                    // -inf: that workgroup saw no row (cannot happen with the current
                    // assignment, where every workgroup owns at least one row)
                    const float w = pm[j][i] == kNegInf ? 0.f : fast_exp2(pm[j][i] - bm);
                    num[j] = fmaf(w, v[j][i], num[j]);
                    den[j] = fmaf(w, pl[j][i], den[j]);
                }
            }
            mx[j] = bm;
        }
    }
#pragma unroll
    for (int j = 0; j < kOut; ++j) {
        const int o = threadIdx.x + j * kDecThreads;
        if (o < G * D) O[hq0 * D + o] = den[j] > 0.f ? num[j] / den[j] : 0.f;   // 0 for an empty cache
    }
    // leave the counter ready for the next call on this workspace
    if (threadIdx.x == 0) __hip_atomic_store(&counters[pair], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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
    constexpr size_t kCounterRegion = 65536 * sizeof(uint32_t);      // B * Hkv <= 65535 counters
    static_assert(kCounterRegion <= L2KV_STATIC_SCRATCH_BYTES, "scratch smaller than its counter region");
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
    plan.lds_pad = 0;
    return plan;
}

DecodePlan decode_plan_ragged(int32_t n_seq, int32_t Hkv, int64_t max_len, int32_t requested_splits,
                              bool ordered) {
    const int64_t pairs = (int64_t)n_seq * Hkv;
    int64_t want = requested_splits;
    const int64_t cap = decode_max_splits(max_len);
    DecodePlan plan;
    plan.lds_pad = 0;
    if (ordered && max_len >= kOrderedMinRows) {
        // The caller supplied a longest-first order.  One workgroup then takes a
        // whole (sequence, KV head) -- only sequences beyond 16k rows, or all of
        // them when the batch has fewer pairs than the uniform rule wants
        // workgroups, are split -- and only one workgroup is resident per
        // compute unit, so the hardware hands the remaining ones out as compute
        // units become free: longest-processing-time-first scheduling by the
        // dispatcher.  Measured on the 64-sequence streaming batch (512 pairs of
        // 512..4200 rows): 97 us per layer against 108 us for the unordered
        // plan; splitting every sequence in two costs 115 us.
        if (want <= 0) {
            const int64_t by_len = (max_len + kOrderedMaxRows - 1) / kOrderedMaxRows;
            const int64_t target = 3 * (int64_t)device_compute_units() / 4;
            const int64_t by_cu = (2 * target + pairs) / (2 * pairs);
            want = by_len > by_cu ? by_len : by_cu;
        }
        plan.lds_pad = kOrderedLdsPad;
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

template <typename E, int D, int G>
static l2kv_status launch_decode(const void* Q, const void* Kc, const void* Vc, int32_t B, int32_t Hq,
                                 int32_t Hkv, int64_t kv_len, int64_t kv_head_stride,
                                 const int32_t* lens, const int64_t* slot_off,
                                 const int32_t* seq_order, float scale, const DecodePlan& plan,
                                 float* O, void* workspace, hipStream_t stream) {
    (void)Hq;
    const float scale_log2e = scale * 1.4426950408889634f;
    uint32_t* counters = static_cast<uint32_t*>(workspace);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + decode_counter_bytes(B, Hkv));
    dim3 grid((unsigned)plan.n_splits, (unsigned)(B * Hkv));
    if (plan.lds_pad > 0) {
        // Unused dynamic LDS, requested only to keep a second workgroup off the
        // compute unit.  Requests beyond 64 KiB need the attribute; it is set per
        // kernel instance and device, here every time the device changes.
        static std::atomic<int> attr_device{-1};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return L2KV_ERR_LAUNCH;
        if (attr_device.load(std::memory_order_relaxed) != dev) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<E, D, G>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, plan.lds_pad) != hipSuccess) {
                (void)hipGetLastError();
                return L2KV_ERR_LAUNCH;
            }
            attr_device.store(dev, std::memory_order_relaxed);
        }
    }
    hipLaunchKernelGGL((decode_kernel<E, D, G>), grid, dim3(kDecThreads), (size_t)plan.lds_pad, stream,
                       static_cast<const char*>(Q), static_cast<const char*>(Kc),
                       static_cast<const char*>(Vc), (int)Hkv, kv_len,
                       kv_head_stride * (int64_t)E::kBytes, lens, slot_off, seq_order, (int)plan.n_splits,
                       (int)plan.rows_per_wg, scale_log2e, counters, partial, O);
    return launch_status();
}

template <typename E, int D>
static l2kv_status decode_by_group(int G, const void* Q, const void* Kc, const void* Vc, int32_t B,
                                   int32_t Hq, int32_t Hkv, int64_t kv_len, int64_t kv_head_stride,
                                   const int32_t* lens, const int64_t* slot_off,
                                   const int32_t* seq_order, float scale, const DecodePlan& plan,
                                   float* O, void* workspace, hipStream_t stream) {
#define L2KV_G(N)                                                                                   \
    case N:                                                                                         \
        return launch_decode<E, D, N>(Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride, lens, slot_off, \
                                      seq_order, scale, plan, O, workspace, stream)
    switch (G) {
        L2KV_G(1); L2KV_G(2); L2KV_G(3); L2KV_G(4); L2KV_G(5); L2KV_G(6); L2KV_G(7); L2KV_G(8);
    }
#undef L2KV_G
    return L2KV_ERR_SHAPE;
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
    return D == 64 ? decode_by_group<BF16, 64>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                               lens, slot_off, seq_order, scale, plan, O, workspace, stream)
                   : decode_by_group<BF16, 128>(G, Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride,
                                                lens, slot_off, seq_order, scale, plan, O, workspace, stream);
}

}  // namespace l2kv
