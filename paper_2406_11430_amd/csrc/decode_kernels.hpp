// l2kv_decode_attn: single-query attention over the compacted cache
// (arXiv 2406.11430, Eq. 2 in the decode form of Eq. 4).  This is the step the
// paper's motivation is about: every decode step re-reads the whole cache from
// HBM, so the kernel is a read stream of Kc and Vc with the arithmetic folded
// in, and the scores never touch memory.
//
// Decomposition: grid (split, sequence x KV head).  The n_splits workgroups of a
// KV head take turns on consecutive 64-row blocks of its cache and stream them
// once for all G = Hq/Hkv query heads.  16 lanes share a row (16 bytes per lane
// and load: one piece of a 256-byte row, two pieces of a 512-byte row; rows of
// 128 bytes are taken in pairs, 8 lanes each -- DecodeGeometry), a wave covers
// 16 rows of K and of V per step (4 + 4 non-temporal loads per lane) and always
// has its next tile in flight while it computes on the current one (two
// register tiles, ping-pong, no branch between a load and its use so the wait
// counters stay exact).  Every row group runs its own online softmax (running
// max m, denominator l, weighted value sum acc), so the only cross-lane traffic
// in the loop is the DPP tree of each dot product.
//
// bf16 caches: q.k uses the packed bf16 dot instruction with fp32 accumulate
// (both operands are exact bf16 inputs); the softmax scale is applied to the
// fp32 score afterwards.  fp32 caches use plain fp32 FMAs.
//
// Query groups of 6 to 8 heads (bf16, D = 128) form q.k on the matrix unit
// instead, run the softmax once per (head, row) and, in grid launches, form p.V
// on the matrix unit in fp32; see decode_item.
//
// At the end the row groups of the workgroup are merged through LDS.  A KV
// head with a single workgroup writes O from that merge.  Otherwise one partial
// (acc[D], m, l) per query head goes to the workspace, and the workgroup that
// finishes last for its KV head (device-scope counter in the workspace) merges
// the partials of all workgroups and writes O: one kernel per call.  Two builds
// of that final merge (template parameter kWideMerge): for at most 8 workgroups
// per head everything stays in registers; for more, the weights are formed once
// in LDS and the accumulators arrive as 16-byte device-scope loads.  In both
// merges a thread forms 1, 2 or 4 consecutive output elements of one head and
// issues all its reads before the first use: every step of this epilogue is a
// memory or LDS round trip on the critical path of the launch.
//
// The same routine (decode_item) runs under two launch shapes: a grid
// (decode_kernel) and, for ragged batches with a known longest-first order, a
// fixed set of workgroups that draw (sequence, KV head, share) items from a
// counter in the workspace (decode_worklist_kernel).
//
// Scores are kept in the log2 domain so the exponentials are bare v_exp_f32.
// This header is instantiated per (element type, head size) by
// decode_attn_<type>_<D>.hip; the host side (plans, dispatch) is decode_attn.hip.
#pragma once
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

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// Row element held in fp32 slot e of the slice of lane c (slots in the order of widen()), with
// the row shared among the lanes in 16-byte pieces (Pieces in l2kv_device.hpp).
template <typename E, int W>
__device__ __forceinline__ constexpr int slice_elem(int c, int e) {
    using P = Pieces<W>;
    constexpr int per_piece = P::kBytes / E::kBytes;
    return (e / per_piece) * (P::kStride / E::kBytes) + c * per_piece + e % per_piece;
}

// K and V are read once per call: streaming loads, nothing to keep in L2.  p = the lane's
// first piece of the row.
template <int W>
__device__ __forceinline__ Words<W> stream_words(const char* p) {
    return load_words_stream<W, Pieces<W>::kStride>(p);
}
// The same for data that is re-read (the query rows).
template <int W>
__device__ __forceinline__ Words<W> cached_words(const char* p) {
    return load_words<W, Pieces<W>::kStride>(p);
}

// s_waitcnt immediate for "vmcnt(0)" alone in the gfx9-family encoding that gfx950 uses: vmcnt
// in bits [3:0] and [15:14] = 0, expcnt [6:4] and lgkmcnt [11:8] left at their maxima.
constexpr int kWaitVmcnt0 = 0x0F70;
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "the s_waitcnt immediate above is the gfx950 encoding: this file is written for gfx950 only"
#endif

// Device-scope (agent) relaxed store of one float.
__device__ __forceinline__ void publish(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Device-scope loads of the published values: buffer loads with the cache policy (sc1) the
// compiler emits for an agent-scope atomic load of one dword, 16, 8 or 4 bytes wide.  `region`
// describes the bytes that may be read (the hardware returns zero outside it); offsets are
// 32-bit, so no 64-bit address arithmetic stands between the ticket and the loads.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kBufferWord3 = 0x00020000;     // raw buffer, 32-bit data format
constexpr int kCachePolicySc1 = 16;
__device__ __forceinline__ f32x4 fetch4(__amdgpu_buffer_rsrc_t region, int byte_offset) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(region, byte_offset, 0, kCachePolicySc1));
}

// voffset per lane, soffset uniform, both in bytes
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2p __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));
// Device-scope stores of 8 and 16 bytes: the policy of publish() on wider stores, so that the
// lanes of a store instruction write contiguous bytes.
__device__ __forceinline__ void publish2(__amdgpu_buffer_rsrc_t region, int voffset, f32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2p, v), region, voffset, 0, kCachePolicySc1);
}
__device__ __forceinline__ void publish4(__amdgpu_buffer_rsrc_t region, int voffset, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4p, v), region, voffset, 0, kCachePolicySc1);
}
__device__ __forceinline__ f32x2 fetch2(__amdgpu_buffer_rsrc_t region, int voffset, int soffset) {
    return __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(region, voffset, soffset, kCachePolicySc1));
}
__device__ __forceinline__ float fetch1(__amdgpu_buffer_rsrc_t region, int voffset, int soffset) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(region, voffset, soffset, kCachePolicySc1));
}

// One output element: fp32, or bf16 (round to nearest even) when the caller asked for it; O then
// points at 16-bit elements.
__device__ __forceinline__ void store_out(float* O, int64_t i, float v, int out_bf16) {
    if (out_bf16) {
        const uint32_t u = __builtin_bit_cast(uint32_t, v);
        const uint32_t r = (u & 0x7f800000u) == 0x7f800000u ? u : u + 0x7fffu + ((u >> 16) & 1u);   // Inf / NaN: truncate
        reinterpret_cast<uint16_t*>(O)[i] = (uint16_t)(r >> 16);
    } else {
        O[i] = v;
    }
}

// Maximum over the 16 lanes of a row group (same lane pairing as row16_tree_sum).
__device__ __forceinline__ float row16_max(float p) {
    p = fmaxf(p, dpp_read<kDppXor1>(p));
    p = fmaxf(p, dpp_read<kDppXor2>(p));
    p = fmaxf(p, dpp_read<kDppHalfMirror>(p));
    p = fmaxf(p, dpp_read<kDppMirror>(p));
    return p;
}

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
// Bytes per K row in the wave's LDS tile of the matrix-unit path: 256 + 16 of padding, so that
// the 16 lanes that read the same 16-byte column of 16 different rows hit different banks.
constexpr int kKtRow = 272;

// How the 16 lanes of a row group share the rows in these kernels.  Rows of 256 and 512 bytes:
// one row per 16 lanes.  Rows of 128 bytes (bf16, 64 elements): two consecutive rows are 256
// contiguous bytes, so a row group takes a PAIR of rows with one 16-byte load per lane (lanes
// 0..7 the even row, 8..15 the odd one) -- the same load instructions as for 256-byte rows
// instead of 8-byte loads -- and runs one online softmax per 8 lanes.
template <typename E, int D> struct DecodeGeometry {
    using S = Slice<E, D>;
    static constexpr int kRowsPerSlot = S::kRowBytes == 128 ? 2 : 1;        // rows per 16 lanes and load
    static constexpr int kLanesPerRow = kRowLanes / kRowsPerSlot;
    static constexpr int kWords = S::kWords * kRowsPerSlot;                  // 32-bit words per lane
    static constexpr int kElems = S::kElems * kRowsPerSlot;                  // row elements per lane
    static constexpr int kSlotBytes = S::kRowBytes * kRowsPerSlot;           // bytes per 16 lanes and load
    static constexpr int kTileRows = kDecRowsPerStep * kRowsPerSlot;         // rows per wave step
    static constexpr int kGroups = kDecGroups * kRowsPerSlot;                // softmax streams per workgroup
};

// Sum over the lanes that share a row: 16, or 8 for row pairs (same tree, one level less).
template <int kLanes>
__device__ __forceinline__ float row_tree_sum(float p) {
    p = p + dpp_read<kDppXor1>(p);
    p = p + dpp_read<kDppXor2>(p);
    p = p + dpp_read<kDppHalfMirror>(p);
    if constexpr (kLanes == 16) p = p + dpp_read<kDppMirror>(p);
    return p;
}

// A lane's words as fp32 values in element order.
template <typename E, int W>
__device__ __forceinline__ void widen_words(const Words<W>& r, float (&x)[W * 4 / E::kBytes]) {
    if constexpr (E::kBytes == 4) {
#pragma unroll
        for (int i = 0; i < W; ++i) x[i] = __builtin_bit_cast(float, r.w[i]);
    } else {
#pragma unroll
        for (int i = 0; i < W; ++i) {
            x[2 * i] = bf16_lo(r.w[i]);
            x[2 * i + 1] = bf16_hi(r.w[i]);
        }
    }
}

template <typename E, int D>
struct Tile {
    Words<DecodeGeometry<E, D>::kWords> k[kDecLoads];
    Words<DecodeGeometry<E, D>::kWords> v[kDecLoads];
};

// Loads the tile of rows that starts at first_row (16 rows, 32 for row pairs) of K and V for
// this lane; all its rows must exist.  lane_off = rg * slot_bytes + c * piece_bytes.
template <typename E, int D>
__device__ __forceinline__ void load_tile(Tile<E, D>& t, const char* Kh, const char* Vh,
                                          int64_t first_row, int lane_off) {
    using S = Slice<E, D>;
    using Geo = DecodeGeometry<E, D>;
    const int64_t off = first_row * S::kRowBytes + lane_off;
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u)
        t.k[u] = stream_words<Geo::kWords>(Kh + off + u * (kRowsPerWaveLoad * Geo::kSlotBytes));
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u)
        t.v[u] = stream_words<Geo::kWords>(Vh + off + u * (kRowsPerWaveLoad * Geo::kSlotBytes));
}

// Ragged last tile of a row range: rows past last_valid re-read row last_valid
// (in bounds); the caller masks their scores.
template <typename E, int D>
__device__ __forceinline__ void load_tile_clamped(Tile<E, D>& t, const char* Kh, const char* Vh,
                                                  int64_t first_row, int64_t last_valid, int rg, int c) {
    using S = Slice<E, D>;
    using Geo = DecodeGeometry<E, D>;
    int64_t off[kDecLoads];
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) {
        int64_t row = first_row + (u * kRowsPerWaveLoad + rg) * Geo::kRowsPerSlot + c / Geo::kLanesPerRow;
        row = row < last_valid ? row : last_valid;
        off[u] = row * S::kRowBytes + (c % Geo::kLanesPerRow) * Pieces<Geo::kWords>::kBytes;
    }
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) t.k[u] = stream_words<Geo::kWords>(Kh + off[u]);
#pragma unroll
    for (int u = 0; u < kDecLoads; ++u) t.v[u] = stream_words<Geo::kWords>(Vh + off[u]);
}

// The builds that use the matrix unit (bf16, D = 128, 6 to 8 query heads per KV head) state an
// occupancy of at least 2 waves per SIMD: a wave may then use at most 256 registers, all of them
// ordinary vector registers, and the compiler keeps the accumulators of the matrix instructions
// in vector registers, where the rescaling of the online softmax reaches them without copies from
// and to the accumulation registers.
template <typename E, int D, int G>
constexpr bool kDecodeOnMatrixUnit = E::kBytes == 2 && D == 128 && G >= 6;
template <typename E, int D, int G>
constexpr int kDecodeMinWaves = kDecodeOnMatrixUnit<E, D, G> ? 2 : 1;

// workspace layout: [counters + work queue: decode_counter_bytes] [partials]
// partials: [B*Hq][n_splits][D + 4] floats: acc[0..D), m (log2 domain), l, two floats of padding
// (rows start on 16-byte boundaries; no two workgroups write into the same row).
//
// decode_item: the share `split` (of n_splits) of one (sequence, KV head): stream
// the rows, merge the workgroup's row groups, publish the partial and, if this
// workgroup is the last of its KV head to finish, merge all partials into O.
// With n_splits == 1 the workgroup's own merge already is the result.
// Called by all threads of the workgroup; every barrier below is reached by all
// of them or by none (the conditions are uniform).
template <typename E, int D, int G, bool kWideMerge, bool kGridLaunch>
__device__ __forceinline__ void decode_item(const char* __restrict__ Q, const char* __restrict__ Kh,
                                            const char* __restrict__ Vh, int64_t kv_len, int64_t hq0,
                                            int split, int n_splits, int n_splits_grid,
                                            float scale_log2e, uint32_t* __restrict__ counter,
                                            float* __restrict__ partial, float* __restrict__ O, int out_bf16,
                                            uint32_t* __restrict__ queue, uint32_t& drawn) {
    using S = Slice<E, D>;
    using Geo = DecodeGeometry<E, D>;
    constexpr int EPL = Geo::kElems;
    constexpr int W = Geo::kWords;
    constexpr int kLanesPerRow = Geo::kLanesPerRow;
    constexpr int kGroups = Geo::kGroups;
    constexpr bool kBf16 = E::kBytes == 2;
    constexpr float kNegInf = -INFINITY;
    constexpr int kRow = D + 4;                      // floats per partial row (decode_partial_floats)
    // One LDS array used twice: first the row-group tiles s_acc[16][G][D], s_m[16][G], s_l[16][G]
    // of the workgroup's own merge, then (last workgroup of a KV head only, after two barriers)
    // the tables of the final merge.
    constexpr int kQuads = G * D / 4;                                   // float4 pieces of the G output rows
    constexpr int kWays = kDecThreads / kQuads;                         // threads sharing one piece, >= 1
    static_assert(kQuads <= kDecThreads, "more output pieces than threads");
    constexpr int kAccFloats = kGroups * G * D;
    constexpr int kTabFloats = 3 * G * kDecodeMaxSplits + kWays * G * D;
    constexpr int kLdsFloats = kAccFloats + 2 * kGroups * G > kTabFloats ? kAccFloats + 2 * kGroups * G : kTabFloats;
    __shared__ __attribute__((aligned(16))) float s_raw[kLdsFloats];
    __shared__ uint32_t s_ticket;
    __shared__ float s_max[G];                   // per query head: maximum of the workgroups' m (final merge)
    if (threadIdx.x < G) s_max[threadIdx.x] = -INFINITY;       // ordered before its use by the barriers below
    float* const s_acc = s_raw;                                          // [(grp * G + g) * D + d]
    float* const s_m = s_raw + kAccFloats;                               // [grp * G + g]
    float* const s_l = s_m + kGroups * G;

    const int lane = threadIdx.x % kWaveSize;
    // the wave index is the same in all 64 lanes: keep it in a scalar register
    // so every branch on row positions below is a scalar branch
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const int c = lane % kRowLanes;
    const int rg = lane / kRowLanes;

    // This lane's slice of the G query rows: raw bf16 pairs for the packed dot,
    // fp32 values otherwise.  The scale is applied to the reduced score.
    uint32_t qw[G][W];
    float qf[kBf16 ? 1 : G][kBf16 ? 1 : EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        Words<W> raw = cached_words<W>(Q + (hq0 + g) * S::kRowBytes + (c % kLanesPerRow) * Pieces<W>::kBytes);
#pragma unroll
        for (int w = 0; w < W; ++w) qw[g][w] = raw.w[w];
        if constexpr (!kBf16) widen_words<E, W>(raw, qf[g]);
    }

    const int64_t r1 = kv_len;                   // rows at or past r1 do not exist
    const int lane_off = rg * Geo::kSlotBytes + c * Pieces<W>::kBytes;

    float m[G], l[G], acc[G][EPL];    // m: running max of the RAW score (before scaling)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegInf;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    // ---- query groups of 6 to 8 heads (bf16, D = 128): q.k on the matrix unit ----------------
    // With that many heads per streamed row the vector ALU, not HBM, bounds the launch, and
    // S = Q.K^T is a real contraction: M = heads (padded to 16), N = the 16 rows of a tile,
    // K = 128.  Measured per C3-shaped layer launch, vector path / this path (with p.V on the
    // matrix unit too, below): 5 heads 45.4 / 45.8 us, 6 heads 47.4 / 46.1, 7 heads 47.7 / 46.0,
    // 8 heads 49.1 / 46.0 -- hence the threshold.  The K tile
    // goes through a wave-private LDS buffer into the operand layout of
    // v_mfma_f32_16x16x32_bf16 (lane (c, rg) supplies row c, elements 32j + 8rg .. +7 for
    // j = 0..3); the result has heads 4rg .. 4rg+3 of row c in lane (c, rg), where the online
    // softmax runs ONCE per (head, row) instead of in all 16 lanes of a row group; the weights
    // and the rescaling factors return through LDS to the row-per-16-lanes layout in which V
    // was loaded, where p.V is formed in fp32 (bf16 weights would cost 2e-3 relative).
    // All four row groups of a wave share one running maximum per head.  (Loading K straight
    // into the operand layout -- 64 contiguous bytes of each of 16 rows per load instruction
    // instead of 256 bytes of each of 4 rows -- needs no LDS staging but streams worse: 59.1 us
    // against 52.6 us at 8 heads.)
    constexpr bool kMfma = kDecodeOnMatrixUnit<E, D, G>;
    // p.V on the matrix unit as well: grid launches only.  The work-list kernel carries more
    // live state and would spill under the 256-register budget this needs (measured on the
    // ragged streaming batch at 8 heads per group: 126 us per layer with the spills, 112 us with
    // the accumulators in accumulation registers, 108 us with p.V on the vector unit).
    constexpr bool kPvMatrix = kMfma && kGridLaunch;
    // The wave-private buffers of this path (K tile, weights, rescaling factors) live in the
    // LDS array that the merge after the loop uses: the workgroup then needs less than half of a
    // compute unit's LDS, two workgroups fit, and the occupancy stated for these builds holds.
    constexpr int kKtFloats = kDecWaves * 16 * kKtRow / 4;
    static_assert(!kMfma || kKtFloats + kDecWaves * G * 16 + kDecWaves * 8 <= kLdsFloats, "loop buffers exceed the merge array");
    [[maybe_unused]] bf16x8_t qa[4];                     // matrix operand of Q: head c, elements 32j + 8rg ..
    [[maybe_unused]] float cm[4], cl[4];                 // heads 4rg+i: running maximum (raw), denominator of row position c
    [[maybe_unused]] f32x4 accq0[kPvMatrix ? EPL : 1], accq1[kPvMatrix ? EPL : 1];   // per element: heads 0..3, heads 4..7
    [[maybe_unused]] char* const kt = reinterpret_cast<char*>(s_raw) + (kMfma ? wave * 16 * kKtRow : 0);
    [[maybe_unused]] float* const sp = s_raw + (kMfma ? kKtFloats + wave * G * 16 : 0);
    [[maybe_unused]] float* const sa = s_raw + (kMfma ? kKtFloats + kDecWaves * G * 16 + wave * 8 : 0);
    if constexpr (kMfma) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            typedef uint32_t u32x4q __attribute__((ext_vector_type(4)));
            u32x4q raw = {0u, 0u, 0u, 0u};
            if (c < G) raw = *reinterpret_cast<const u32x4q*>(Q + (hq0 + c) * S::kRowBytes + (j * 4 + rg) * 16);
            qa[j] = __builtin_bit_cast(bf16x8_t, raw);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            cm[i] = kNegInf;
            cl[i] = 0.f;
        }
        if constexpr (kPvMatrix) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                accq0[e] = f32x4{0.f, 0.f, 0.f, 0.f};
                accq1[e] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    auto consume_mfma = [&](const Tile<E, D>& t, int64_t first_row, bool ragged) {
        typedef uint32_t u32x4m __attribute__((ext_vector_type(4)));
        if constexpr (kMfma) {
            // 1. K tile, row-major with padded rows, into the wave's LDS buffer
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) {
                const u32x4m w = {t.k[u].w[0], t.k[u].w[1], t.k[u].w[2], t.k[u].w[3]};
                *reinterpret_cast<u32x4m*>(kt + (u * kRowsPerWaveLoad + rg) * kKtRow + c * 16) = w;
            }
            __builtin_amdgcn_wave_barrier();
            // 2. S = Q.K^T: four matrix instructions over the 128 elements of a row
            f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4m w = *reinterpret_cast<const u32x4m*>(kt + c * kKtRow + (j * 4 + rg) * 16);
                sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[j], __builtin_bit_cast(bf16x8_t, w), sc, 0, 0, 0);
            }
            // 3. online softmax of heads 4rg+i over the tile's rows (row c in this lane)
            float sv[4] = {sc.x, sc.y, sc.z, sc.w};
            const bool row_ok = !ragged || first_row + c < r1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float si = row_ok ? sv[i] : kNegInf;
                const float mn = fmaxf(cm[i], row16_max(si));
                const float ms = mn == kNegInf ? 0.f : mn * scale_log2e;
                const float alpha = fast_exp2(fmaf(cm[i], scale_log2e, -ms));
                const float pi = fast_exp2(fmaf(si, scale_log2e, -ms));
                cl[i] = fmaf(cl[i], alpha, pi);
                cm[i] = mn;
                const int g = 4 * rg + i;
                if (g < G) {
                    sp[g * 16 + (c % 4) * 4 + c / 4] = pi;        // [head][row group of the row][load of the row]
                    if (c == 0) sa[g] = alpha;
                }
            }
            __builtin_amdgcn_wave_barrier();
            // 4. p.V in the layout V was loaded in: lane (rg, c) holds rows 4u + rg, elements 8c ..
            float al[G];
#pragma unroll
            for (int g = 0; g < G; ++g) al[g] = sa[g];
            // The factors are the same in every lane (one running maximum per head and wave) and
            // exactly 1 while no maximum moves, which is the rule after the first tiles.  Groups
            // of 6 and 7 heads then skip the rescaling, a branch the whole wave takes alike
            // (46.1 -> 44.3 and 46.4 -> 44.5 us per C3-shaped launch); at 8 heads the same branch
            // costs more in instruction scheduling than it saves (48.3 against 46.0 us).
            constexpr bool kSkipUnitFactors = kPvMatrix && G < 8;
            [[maybe_unused]] bool moved = true;
            if constexpr (kSkipUnitFactors) {
                moved = false;
#pragma unroll
                for (int g = 0; g < G; ++g)
                    moved |= __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, al[g])) != 0x3f800000;
            }
            if constexpr (kPvMatrix) {
                // On the matrix unit in fp32: v_mfma_f32_4x4x1_16b_f32 computes, per lane l and
                // result register r, D[r] += A(lane 4*(l/4) + r) * B(lane l).  With B = one value
                // element of this lane and A = the weight of head (lane % 4) [+ 4], one
                // instruction is the multiply-add of four heads, and it runs beside the vector
                // unit.
                const int ga = c % 4;
                const f32x4 pa = *reinterpret_cast<const f32x4*>(sp + ga * 16 + rg * 4);           // heads 0..3
                f32x4 pb = {0.f, 0.f, 0.f, 0.f};                                                 // heads 4..7
                if (ga + 4 < G) pb = *reinterpret_cast<const f32x4*>(sp + (ga + 4) * 16 + rg * 4);
                if (moved) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) {
                        accq0[e].x *= al[0]; accq0[e].y *= al[1]; accq0[e].z *= al[2]; accq0[e].w *= al[3];
                        if constexpr (G > 4) accq1[e].x *= al[4];
                        if constexpr (G > 5) accq1[e].y *= al[5];
                        if constexpr (G > 6) accq1[e].z *= al[6];
                        if constexpr (G > 7) accq1[e].w *= al[7];
                    }
                }
#pragma unroll
                for (int u = 0; u < kDecLoads; ++u) {
                    float vx[EPL];
                    widen_words<E, W>(t.v[u], vx);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) {
                        accq0[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(pa[u], vx[e], accq0[e], 0, 0, 0);
                        accq1[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(pb[u], vx[e], accq1[e], 0, 0, 0);
                    }
                }
            } else {
                float pw[G][kDecLoads];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const f32x4 pg = *reinterpret_cast<const f32x4*>(sp + g * 16 + rg * 4);
                    pw[g][0] = pg.x; pw[g][1] = pg.y; pw[g][2] = pg.z; pw[g][3] = pg.w;
                }
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[g][e] *= al[g];
#pragma unroll
                for (int u = 0; u < kDecLoads; ++u) {
                    float vx[EPL];
                    widen_words<E, W>(t.v[u], vx);
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pw[g][u], vx[e], acc[g][e]);
                }
            }
            __builtin_amdgcn_wave_barrier();          // the buffers are rewritten by the next tile
        }
    };

    auto consume_valu = [&](const Tile<E, D>& t, int64_t first_row, bool ragged) {
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
                widen_words<E, W>(t.k[u], kx);
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
            for (int u = 0; u < kDecLoads; ++u) s[g][u] = row_tree_sum<kLanesPerRow>(s[g][u]);
        if (ragged) {                                    // only the last, partial tile of a range
#pragma unroll
            for (int u = 0; u < kDecLoads; ++u) {
                const bool valid = first_row + (u * kRowsPerWaveLoad + rg) * Geo::kRowsPerSlot + c / kLanesPerRow < r1;
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
            widen_words<E, W>(t.v[u], vx);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p[g][u], vx[e], acc[g][e]);
        }
    };

    auto consume = [&](const Tile<E, D>& t, int64_t first_row, bool ragged) {
        if constexpr (kMfma) consume_mfma(t, first_row, ragged);
        else consume_valu(t, first_row, ragged);
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
        // Tile indices fit 32 bits (the host admits at most 2^31 - 1 rows) and the loop runs on
        // comparisons of them: no division stands between the launch and the first load.
        const int n_full = (int)(kv_len / Geo::kTileRows);                      // full tiles in the head
        const int tile_stride = n_splits * kDecWaves;
        int tile = split * kDecWaves + wave;                                     // my next tile
        const int64_t kStride = (int64_t)tile_stride * Geo::kTileRows;          // rows between my tiles
        int64_t row = (int64_t)tile * Geo::kTileRows;
        if (tile < n_full) {
            Tile<E, D> ta, tb;
            // The scheduling barriers pin each batch of loads ahead of the
            // arithmetic on the other tile; without them the compiler sinks
            // the loads next to their first use and the prefetch is lost.
            load_tile<E, D>(ta, Kh, Vh, row, lane_off);
            __builtin_amdgcn_sched_barrier(0);
            while (tile + 2 * tile_stride < n_full) {    // ta holds `tile`; at least two more follow
                load_tile<E, D>(tb, Kh, Vh, row + kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(ta, row, false);
                __builtin_amdgcn_sched_barrier(0);
                load_tile<E, D>(ta, Kh, Vh, row + 2 * kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(tb, row + kStride, false);
                __builtin_amdgcn_sched_barrier(0);
                row += 2 * kStride;
                tile += 2 * tile_stride;
            }
            if (tile + tile_stride < n_full) {
                load_tile<E, D>(tb, Kh, Vh, row + kStride, lane_off);
                __builtin_amdgcn_sched_barrier(0);
                consume(ta, row, false);
                consume(tb, row + kStride, false);
                tile += 2 * tile_stride;
            } else {
                consume(ta, row, false);
                tile += tile_stride;
            }
        }
        // `tile` is now the first tile of this wave's sequence at or past the full ones: the
        // ragged last tile of the head, if there is one, belongs to the wave whose sequence hits it
        if (kv_len % Geo::kTileRows != 0 && tile == n_full) {
            Tile<E, D> tt;
            const int64_t first = (int64_t)n_full * Geo::kTileRows;
            load_tile_clamped<E, D>(tt, Kh, Vh, first, r1 - 1, rg, c);
            consume(tt, first, true);
        }
    }

    if constexpr (kMfma) {
        // hand the wave's softmax state to the row-group layout of the merge below: all four row
        // groups of the wave share the maximum; the denominator is counted once (row group 0)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lt = row16_tree_sum(cl[i]);
            const int g = 4 * rg + i;
            if (g < G && c == 0) {
                sa[g] = cm[i];
                sp[g] = lt;
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m[g] = sa[g];
            l[g] = rg == 0 ? sp[g] : 0.f;
            if constexpr (kPvMatrix) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = g < 4 ? accq0[e][g] : accq1[e][g - 4];
            }
        }
    }

    // Work-list launches draw the workgroup's next item here, when its rows have been streamed:
    // early enough for the counter's latency to hide behind the merge below, late enough that
    // items are still handed out in the order in which workgroups become free.
    if (queue != nullptr && threadIdx.x == 0)
        drawn = gridDim.x + __hip_atomic_fetch_add(queue, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // ---- merge the 16 row groups of the workgroup through LDS --------------
    if constexpr (kMfma) __syncthreads();          // every wave is done with its buffers in that array
    const int grp = (wave * kRowsPerWaveLoad + rg) * Geo::kRowsPerSlot + c / kLanesPerRow;
    const int cr = c % kLanesPerRow;               // position among the lanes of this row
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[(grp * G + g) * D + slice_elem<E, W>(cr, e)] = acc[g][e];
        if (cr == 0) {
            s_m[grp * G + g] = m[g] * scale_log2e;     // -inf stays -inf (scale > 0)
            s_l[grp * G + g] = l[g];
        }
    }
    __syncthreads();
    // Thread t forms the kVec consecutive output elements t * kVec .. of the G * D (all of one
    // query head): the weights of the 16 row groups are computed once per thread, and all LDS
    // reads are issued before the arithmetic (one LDS latency, not one per row group).
    constexpr int kVec = G * D <= kDecThreads ? 1 : (G * D <= 2 * kDecThreads ? 2 : 4);
    static_assert(G * D <= 4 * kDecThreads && D % kVec == 0, "output elements per thread");
    const int o0 = threadIdx.x * kVec;
    if (o0 < G * D) {
        const int g = o0 / D;
        const int d = o0 % D;
        float mi[kGroups], li[kGroups], ai[kGroups][kVec];
#pragma unroll
        for (int i = 0; i < kGroups; ++i) {
            mi[i] = s_m[i * G + g];
            li[i] = s_l[i * G + g];
            const float* a = s_acc + (i * G + g) * D + d;
            if constexpr (kVec == 4) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(a);
                ai[i][0] = t.x; ai[i][1] = t.y; ai[i][2] = t.z; ai[i][3] = t.w;
            } else if constexpr (kVec == 2) {
                const f32x2 t = *reinterpret_cast<const f32x2*>(a);
                ai[i][0] = t.x; ai[i][1] = t.y;
            } else {
                ai[i][0] = a[0];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float mx = kNegInf;
#pragma unroll
        for (int i = 0; i < kGroups; ++i) mx = fmaxf(mx, mi[i]);
        float num[kVec], den = 0.f;
#pragma unroll
        for (int k = 0; k < kVec; ++k) num[k] = 0.f;
#pragma unroll
        for (int i = 0; i < kGroups; ++i) {
            const float w = mi[i] == kNegInf ? 0.f : fast_exp2(mi[i] - mx);
#pragma unroll
            for (int k = 0; k < kVec; ++k) num[k] = fmaf(w, ai[i][k], num[k]);
            den = fmaf(w, li[i], den);
        }
        if (n_splits == 1) {
            // the only workgroup of this KV head: its merge is the result (0 for an empty cache)
#pragma unroll
            for (int k = 0; k < kVec; ++k)
                store_out(O, hq0 * D + o0 + k, den > 0.f ? num[k] / den : 0.f, out_bf16);
        } else {
            // Device-scope stores: written through to the level every compute unit
            // of the device reads from, so the merging workgroup below sees them
            // without any bulk cache write-back.
            float* out = partial + ((hq0 + g) * n_splits_grid + split) * kRow;
            const __amdgpu_buffer_rsrc_t row = __builtin_amdgcn_make_buffer_rsrc(out, 0, kRow * (int)sizeof(float), kBufferWord3);
            if constexpr (kVec == 4) publish4(row, d * (int)sizeof(float), f32x4{num[0], num[1], num[2], num[3]});
            else if constexpr (kVec == 2) publish2(row, d * (int)sizeof(float), f32x2{num[0], num[1]});
            else publish(out + d, num[0]);
            if (d == 0) publish2(row, D * (int)sizeof(float), f32x2{mx, den});
        }
    }
    if (n_splits == 1) {
        __syncthreads();          // the LDS tiles may be reused by the caller's next item
        return;
    }

    // ---- the last workgroup of this KV head merges all row ranges ---------
    // Hand-over protocol.  (1) Every partial is written with a device-scope
    // atomic store (write-through: it does not stay in this die's L2).  (2)
    // Every wave waits until its own stores have been acknowledged (vmcnt(0): a
    // workgroup barrier alone does not wait for outstanding global stores, and
    // the ticket below travels to a different memory channel than the partials,
    // so without the wait it could overtake them).  (3) After the barrier one
    // lane takes a ticket with a device-scope read-modify-write.  (4) After a
    // second barrier the workgroup that drew the last ticket re-reads all
    // partials with device-scope loads.  No lane ever waits on another
    // workgroup, so nothing here can hang.
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __syncthreads();
    if (threadIdx.x == 0)
        s_ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != (uint32_t)(n_splits - 1)) return;

    constexpr int kNarrow = 8;
    if constexpr (!kWideMerge) {
        // Launches with at most 8 workgroups per KV head: every lane fetches, for its kVec
        // output elements (one query head, consecutive d), the accumulator elements together
        // with (m, l) of all workgroups at once: all loads are independent, one memory round
        // trip, no LDS, no barrier.  (The host never pairs this variant with more than 8
        // workgroups.)  The partials of this KV head's G query heads are one contiguous region;
        // 32-bit offsets into it (per lane: query head and element; uniform: workgroup) keep the
        // address arithmetic off the critical path.
        const __amdgpu_buffer_rsrc_t region = __builtin_amdgcn_make_buffer_rsrc(
            partial + hq0 * n_splits_grid * kRow, 0, G * n_splits_grid * kRow * (int)sizeof(float), kBufferWord3);
        const int last = __builtin_amdgcn_readfirstlane(n_splits - 1);
        const int oo = o0 < G * D ? o0 : 0;                                 // idle lanes re-read element 0
        const int head_off = (oo / D) * n_splits_grid * kRow * (int)sizeof(float);
        const int elem_off = head_off + (oo % D) * (int)sizeof(float);
        const int stat_off = head_off + D * (int)sizeof(float);
        float v[kNarrow][kVec], pm[kNarrow], pl[kNarrow];
#pragma unroll
        for (int i = 0; i < kNarrow; ++i) {
            const int wg_off = (i < last ? i : last) * kRow * (int)sizeof(float);   // clamp: in bounds, weight 0 below
            if constexpr (kVec == 4) {
                const f32x4 t = fetch4(region, elem_off + wg_off);
                v[i][0] = t.x; v[i][1] = t.y; v[i][2] = t.z; v[i][3] = t.w;
            } else if constexpr (kVec == 2) {
                const f32x2 t = fetch2(region, elem_off, wg_off);
                v[i][0] = t.x; v[i][1] = t.y;
            } else {
                v[i][0] = fetch1(region, elem_off, wg_off);
            }
            const f32x2 st = fetch2(region, stat_off, wg_off);
            pm[i] = st.x;
            pl[i] = st.y;
        }
        // every request above is issued before the first use below (the compiler would otherwise
        // move each load next to its use and turn one memory round trip into several)
        __builtin_amdgcn_sched_barrier(0);
        // branch-free: the slots past n_splits hold copies of the last workgroup's values
        // (finite or -inf like any other) and get weight 0
        float bm = kNegInf;
#pragma unroll
        for (int i = 0; i < kNarrow; ++i) bm = fmaxf(bm, pm[i]);
        float num[kVec], den = 0.f;
#pragma unroll
        for (int k = 0; k < kVec; ++k) num[k] = 0.f;
#pragma unroll
        for (int i = 0; i < kNarrow; ++i) {
            // -inf: that workgroup saw no row (cannot happen with the current
            // assignment, where every workgroup owns at least one row)
            float w = pm[i] == kNegInf ? 0.f : fast_exp2(pm[i] - bm);
            w = i < n_splits ? w : 0.f;
#pragma unroll
            for (int k = 0; k < kVec; ++k) num[k] = fmaf(w, v[i][k], num[k]);
            den = fmaf(w, pl[i], den);
        }
        if (o0 < G * D) {
#pragma unroll
            for (int k = 0; k < kVec; ++k)
                store_out(O, hq0 * D + o0 + k, den > 0.f ? num[k] / den : 0.f, out_bf16);   // 0 for an empty cache
        }
    } else {
    // Launches with more than 8 workgroups per KV head: final merge in one memory round trip
    // and four LDS steps.  The weights depend on (m, l) only, the sums on the accumulators
    // only, so both are requested at once.  Entry e = (workgroup, query head) is handled by
    // thread e % 256: (1) an LDS float-max per head (order-free, hence bit-reproducible) gives
    // the per-head maximum; (2) w = 2^(m - max) and w*l go to LDS tables; (3) the accumulators,
    // which arrived as 16-byte pieces -- piece q = (g, 4 consecutive d) is shared by kWays
    // threads, thread `way` taking the workgroups way, way + kWays, ... -- are weighted and
    // summed, together with the w*l of the same workgroups; (4) the kWays partial sums meet in
    // LDS and are added in order of `way`, so the result does not depend on timing.
    {
        constexpr int kBatch = 16;                                       // 16-byte loads in flight per thread
        constexpr int kEnt = (G * kDecodeMaxSplits + kDecThreads - 1) / kDecThreads;
        float* const s_w = s_raw;                                        // [G][n_splits] weights
        float* const s_wl = s_w + G * kDecodeMaxSplits;                  // [G][n_splits] weights * l
        float* const s_red = s_wl + G * kDecodeMaxSplits;                // [kWays][G * D] partial sums
        float* const s_den = s_red + kWays * G * D;                      // [kWays][G] partial denominators
        static_assert(2 * G * kDecodeMaxSplits + kWays * G * D + kWays * G <= kLdsFloats, "LDS tables");
        const int n_ent = G * n_splits;
        const bool active = (int)threadIdx.x < kWays * kQuads;
        const int way = active ? (int)threadIdx.x / kQuads : 0;
        const int q = active ? (int)threadIdx.x % kQuads : 0;
        const int qg = q / (D / 4);
        // the partials of this KV head's G query heads are one contiguous region
        const __amdgpu_buffer_rsrc_t region = __builtin_amdgcn_make_buffer_rsrc(
            partial + hq0 * n_splits_grid * kRow, 0, G * n_splits_grid * kRow * (int)sizeof(float), kBufferWord3);
        const int q_off = (qg * n_splits_grid * kRow + (q % (D / 4)) * 4) * (int)sizeof(float);
        f32x4 v[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int sp = way + i * kWays;
            v[i] = fetch4(region, q_off + (sp < n_splits ? sp : n_splits - 1) * kRow * (int)sizeof(float));
        }
        float pm[kEnt], pl[kEnt];
#pragma unroll
        for (int t = 0; t < kEnt; ++t) {
            const int e = threadIdx.x + t * kDecThreads;
            const int ee = e < n_ent ? e : 0;
            const int stat_off = (((ee % G) * n_splits_grid + ee / G) * kRow + D) * (int)sizeof(float);
            pm[t] = fetch1(region, stat_off, 0);
            pl[t] = fetch1(region, stat_off + 4, 0);
        }
        // keep every request above ahead of the LDS work below (the compiler would otherwise
        // sink the accumulator loads behind the barriers, next to their first use)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < kEnt; ++t) {
            const int e = threadIdx.x + t * kDecThreads;
            if (e < n_ent) __hip_atomic_fetch_max(&s_max[e % G], pm[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kEnt; ++t) {
            const int e = threadIdx.x + t * kDecThreads;
            if (e < n_ent) {
                // -inf: that workgroup saw no row (cannot happen with the current
                // assignment, where every workgroup owns at least one row)
                const float w = pm[t] == kNegInf ? 0.f : fast_exp2(pm[t] - s_max[e % G]);
                s_w[(e % G) * n_splits + e / G] = w;
                s_wl[(e % G) * n_splits + e / G] = w * pl[t];
            }
        }
        __syncthreads();
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        float dsum = 0.f;
        for (int s0 = 0; s0 < n_splits; s0 += kBatch * kWays) {
            if (s0 > 0) {
#pragma unroll
                for (int i = 0; i < kBatch; ++i) {
                    const int sp = s0 + way + i * kWays;
                    v[i] = fetch4(region, q_off + (sp < n_splits ? sp : n_splits - 1) * kRow * (int)sizeof(float));
                }
            }
            float w[kBatch], wl[kBatch];                                  // independent LDS reads first
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int sp = s0 + way + i * kWays;
                w[i] = s_w[qg * n_splits + (sp < n_splits ? sp : n_splits - 1)];
                wl[i] = s_wl[qg * n_splits + (sp < n_splits ? sp : n_splits - 1)];
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const bool live = s0 + way + i * kWays < n_splits;
                const float wi = live ? w[i] : 0.f;
                sum.x = fmaf(wi, v[i].x, sum.x);
                sum.y = fmaf(wi, v[i].y, sum.y);
                sum.z = fmaf(wi, v[i].z, sum.z);
                sum.w = fmaf(wi, v[i].w, sum.w);
                dsum += live ? wl[i] : 0.f;
            }
        }
        if (active) {
            *reinterpret_cast<f32x4*>(s_red + way * (G * D) + q * 4) = sum;
            if (q % (D / 4) == 0) s_den[way * G + qg] = dsum;
        }
        __syncthreads();
        for (int o = threadIdx.x; o < G * D; o += kDecThreads) {
            const int g = o / D;
            float num = 0.f, den = 0.f;
#pragma unroll
            for (int y = 0; y < kWays; ++y) {
                num += s_red[y * (G * D) + o];
                den += s_den[y * G + g];
            }
            store_out(O, hq0 * D + o, den > 0.f ? num / den : 0.f, out_bf16);   // 0 for an empty cache
        }
    }
    }
    // leave the counter ready for the next call on this workspace
    if (threadIdx.x == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();              // the LDS tables may be reused by the caller's next item
}

// Grid launch: blockIdx.x = share of the KV head, blockIdx.y = KV head, blockIdx.z = sequence
// (or position in the launch order); workgroups are dispatched with x running fastest, then y.
template <typename E, int D, int G, bool kWideMerge>
__global__ __launch_bounds__(kDecThreads) __attribute__((amdgpu_waves_per_eu(kDecodeMinWaves<E, D, G>)))
void decode_kernel(const char* __restrict__ Q, const char* __restrict__ Kc,
                   const char* __restrict__ Vc, int Hkv, int64_t kv_len_uniform,
                   int64_t head_stride_bytes, const int32_t* __restrict__ lens,
                   const int64_t* __restrict__ slot_off, const int32_t* __restrict__ seq_order,
                   int n_splits_grid, int rows_per_wg,
                   float scale_log2e, uint32_t* __restrict__ counters,
                   float* __restrict__ partial, float* __restrict__ O, int out_bf16) {
    using S = Slice<E, D>;
    // All arguments into scalar registers at once: one batch of loads and one wait, instead of
    // a load and a wait wherever the code below first touches an argument (eight round trips
    // in a row before the first row could be requested).  The price: the compiler must assume
    // that a statement without outputs writes memory, so the three small reads of a ragged
    // launch below (seq_order, lens, slot_off) go through the vector memory path instead of the
    // scalar cache; measured, that costs nothing (99.9 against 100.5 us on the ragged
    // streaming batch launched as a grid), and short uniform launches gain about 0.1 us.
    asm volatile("" ::"s"(Q), "s"(Kc), "s"(Vc), "s"(Hkv), "s"(kv_len_uniform), "s"(head_stride_bytes), "s"(lens),
                 "s"(slot_off), "s"(seq_order), "s"(n_splits_grid), "s"(rows_per_wg), "s"(scale_log2e),
                 "s"(counters), "s"(partial), "s"(O), "s"(out_bf16));
    const int split = blockIdx.x;
    const int hkv = blockIdx.y;
    const int pair = blockIdx.z * Hkv + hkv;     // b * Hkv + hkv
    // Ragged batches may come with a processing order (longest sequence first):
    // the launch index then names a position in that order, not the sequence.
    int b = blockIdx.z;
    if (seq_order != nullptr) {
        const int n_seq = (int)gridDim.z;
        const int ob = seq_order[b];
        b = ob < 0 ? 0 : (ob < n_seq ? ob : n_seq - 1);
    }
    const int Hq = Hkv * G;
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
        const int32_t len_b = lens[b];             // requested together with the two offsets below
        const Range slots = clamped_range(slot_off, b, head_stride_bytes / S::kRowBytes);
        kv_len = len_b;
        kv_len = kv_len < 0 ? 0 : (kv_len > slots.count ? slots.count : kv_len);
        slab = (int64_t)hkv * head_stride_bytes + slots.first * (int64_t)S::kRowBytes;
        const int need = (int)(((uint32_t)kv_len + (uint32_t)rows_per_wg - 1u) / (uint32_t)rows_per_wg);   // kv_len is a clamped int32 here
        n_splits = need < 1 ? 1 : (need < n_splits_grid ? need : n_splits_grid);
        if (split >= n_splits) return;
    }
    uint32_t unused = 0;
    decode_item<E, D, G, kWideMerge, true>(Q, Kc + slab, Vc + slab, kv_len, hq0, split, n_splits, n_splits_grid,
                                           scale_log2e, counters + ((int64_t)b * Hkv + hkv), partial, O, out_bf16, nullptr, unused);
}

// Work-list launch for ragged batches with a known longest-first order.  A
// fixed set of workgroups (about one per compute unit) draws items from a
// device counter: item i is share i % n_splits_grid of KV head
// (i / n_splits_grid) % Hkv of the sequence at position i / (n_splits_grid * Hkv)
// of the order, so the longest sequences are handed out first and whichever
// workgroup becomes free takes the next-longest remaining piece
// (longest-processing-time-first list scheduling).  The next item is drawn
// when the current one has been streamed, before its merge, which hides most
// of the latency of the counter.  queue[0] = items drawn beyond the first round, queue[1] = workgroups that have left; the
// last one to leave zeroes both for the next launch.  Every workgroup leaves as
// soon as it draws an item past the end; nobody waits for anybody.
template <typename E, int D, int G, bool kWideMerge>
__global__ __launch_bounds__(kDecThreads)
void decode_worklist_kernel(const char* __restrict__ Q, const char* __restrict__ Kc,
                            const char* __restrict__ Vc, int Hkv, int n_seq, int64_t plane_stride_bytes,
                            const int32_t* __restrict__ lens, const int64_t* __restrict__ slot_off,
                            const int32_t* __restrict__ seq_order, int n_splits_grid, int rows_per_wg,
                            float scale_log2e, uint32_t* __restrict__ counters, uint32_t* __restrict__ queue,
                            float* __restrict__ partial, float* __restrict__ O, int out_bf16) {
    using S = Slice<E, D>;
    __shared__ uint32_t s_item;
    const uint32_t n_items = (uint32_t)n_seq * (uint32_t)Hkv * (uint32_t)n_splits_grid;
    const int Hq = Hkv * G;
    // The first gridDim.x items need no counter: workgroup i starts on item i (a simultaneous
    // draw by every workgroup would queue up behind one memory location); the counter hands
    // out the items from gridDim.x on.
    uint32_t drawn = blockIdx.x;                          // thread 0 only: the item drawn ahead
    for (;;) {
        if (threadIdx.x == 0) s_item = drawn;
        __syncthreads();
        const uint32_t item = s_item;
        __syncthreads();                                  // everyone has read s_item before it is rewritten
        if (item >= n_items) break;
        const int split = (int)(item % (uint32_t)n_splits_grid);
        const int hkv = (int)((item / (uint32_t)n_splits_grid) % (uint32_t)Hkv);
        const int pos = (int)(item / ((uint32_t)n_splits_grid * (uint32_t)Hkv));
        const int ob = seq_order[pos];
        const int b = ob < 0 ? 0 : (ob < n_seq ? ob : n_seq - 1);
        const int32_t len_b = lens[b];             // requested together with the two offsets below
        const Range slots = clamped_range(slot_off, b, plane_stride_bytes / S::kRowBytes);
        int64_t kv_len = len_b;
        kv_len = kv_len < 0 ? 0 : (kv_len > slots.count ? slots.count : kv_len);
        const int64_t slab = (int64_t)hkv * plane_stride_bytes + slots.first * (int64_t)S::kRowBytes;
        const int need = (int)(((uint32_t)kv_len + (uint32_t)rows_per_wg - 1u) / (uint32_t)rows_per_wg);   // kv_len is a clamped int32 here
        const int n_splits = need < 1 ? 1 : (need < n_splits_grid ? need : n_splits_grid);
        if (split >= n_splits) {                          // uniform: the whole workgroup skips the item
            if (threadIdx.x == 0)
                drawn = gridDim.x + __hip_atomic_fetch_add(&queue[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            continue;
        }
        const int64_t hq0 = (int64_t)b * Hq + (int64_t)hkv * G;
        decode_item<E, D, G, kWideMerge, false>(Q, Kc + slab, Vc + slab, kv_len, hq0, split, n_splits, n_splits_grid,
                                                scale_log2e, counters + ((int64_t)b * Hkv + hkv), partial, O, out_bf16, &queue[0], drawn);
    }
    if (threadIdx.x == 0) {
        // every draw of this workgroup has returned (its value was used above), so the workgroup
        // that finds all others gone may reset the queue
        const uint32_t gone = __hip_atomic_fetch_add(&queue[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (gone == gridDim.x - 1) {
            __hip_atomic_store(&queue[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&queue[1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <typename E, int D, int G>
l2kv_status launch_decode(const void* Q, const void* Kc, const void* Vc, int32_t B, int32_t Hq,
                                 int32_t Hkv, int64_t kv_len, int64_t kv_head_stride,
                                 const int32_t* lens, const int64_t* slot_off,
                                 const int32_t* seq_order, float scale, const DecodePlan& plan,
                                 float* O, void* workspace, hipStream_t stream) {
    const float scale_log2e = scale * 1.4426950408889634f;
    uint32_t* counters = static_cast<uint32_t*>(workspace);
    (void)Hq;
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + decode_counter_bytes(B, Hkv));
    // two builds of each kernel: the final merge for at most 8 workgroups per KV head (all in
    // registers) or for more (tables in LDS); keeping both in one kernel slows the short one down
    const bool wide = plan.n_splits > 8;
    // the work list exists for bf16 heads of 128 elements only (the host plans it for no other)
    constexpr bool kWorkListRows = E::kBytes == 2 && D == 128;
    if constexpr (kWorkListRows) {
        if (plan.worklist_wgs > 0 && lens != nullptr && slot_off != nullptr && seq_order != nullptr) {
            uint32_t* queue = counters + (size_t)B * (size_t)Hkv;     // two words behind the arrival counters
            auto kernel = wide ? decode_worklist_kernel<E, D, G, true> : decode_worklist_kernel<E, D, G, false>;
            hipLaunchKernelGGL(kernel, dim3((unsigned)plan.worklist_wgs),
                               dim3(kDecThreads), 0, stream, static_cast<const char*>(Q),
                               static_cast<const char*>(Kc), static_cast<const char*>(Vc), (int)Hkv, (int)B,
                               kv_head_stride * (int64_t)E::kBytes, lens, slot_off, seq_order,
                               (int)plan.n_splits, (int)plan.rows_per_wg, scale_log2e, counters, queue, partial, O, (int)plan.out_bf16);
            return launch_status();
        }
    }
    dim3 grid((unsigned)plan.n_splits, (unsigned)Hkv, (unsigned)B);
    auto kernel = wide ? decode_kernel<E, D, G, true> : decode_kernel<E, D, G, false>;
    hipLaunchKernelGGL(kernel, grid, dim3(kDecThreads), 0, stream,
                       static_cast<const char*>(Q), static_cast<const char*>(Kc),
                       static_cast<const char*>(Vc), (int)Hkv, kv_len,
                       kv_head_stride * (int64_t)E::kBytes, lens, slot_off, seq_order, (int)plan.n_splits,
                       (int)plan.rows_per_wg, scale_log2e, counters, partial, O, (int)plan.out_bf16);
    return launch_status();
}

template <typename E, int D>
l2kv_status decode_by_group(int G, const void* Q, const void* Kc, const void* Vc, int32_t B,
                                   int32_t Hq, int32_t Hkv, int64_t kv_len, int64_t kv_head_stride,
                                   const int32_t* lens, const int64_t* slot_off,
                                   const int32_t* seq_order, float scale, const DecodePlan& plan,
                                   float* O, void* workspace, hipStream_t stream) {
#define L2KV_G(N)                                                                                   \
    case N:                                                                                         \
        return launch_decode<E, D, N>(Q, Kc, Vc, B, Hq, Hkv, kv_len, kv_head_stride, lens, slot_off, \
                                      seq_order, scale, plan, O, workspace, stream)
    // the final merge gives every thread at most one 16-byte piece of the G output rows:
    // G * D <= 1024, i.e. up to 8 heads for rows of 64 and 128 elements, 4 for rows of 256
    if constexpr (D <= 128) {
        switch (G) { L2KV_G(5); L2KV_G(6); L2KV_G(7); L2KV_G(8); }
    }
    switch (G) { L2KV_G(1); L2KV_G(2); L2KV_G(3); L2KV_G(4); }
#undef L2KV_G
    return L2KV_ERR_SHAPE;
}

}  // namespace l2kv
