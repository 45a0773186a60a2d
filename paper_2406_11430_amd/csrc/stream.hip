// Ragged batches and the streaming slot cache.
//
// arXiv 2406.11430, Sec. 4 ("Language Modelling Tasks"): the cache grows up to a
// pre-defined length, after which the tokens with the highest key norm are
// discarded.  Here every sequence owns a fixed range of slots in each head
// plane; a slot holds the K and V rows, the fp32 squared key norm and the
// original token id of one kept token:
//
//   Kc, Vc  [n_planes][total_slots][D]      n_planes = layers x KV heads
//   norms_c [n_planes][total_slots] fp32    pos_c [n_planes][total_slots] int32
//   sequence s: slots slot_off[s] .. slot_off[s+1]-1, the first lens[s] occupied
//
// Three kernels:
//   compact_ragged : kept rows of a ragged prompt batch -> slot cache (with norms, ids)
//   stream_append  : one new token per sequence -> next free slot, norm computed here
//                    (fixed summation order), so no separate norm pass is ever needed
//   stream_evict   : while a sequence holds more than its budget, drop the slot
//                    with the largest (norm bits, token id) and move the last
//                    slot into the hole -- the reverse of the keep order of
//                    l2kv_select, so the kept set is always "lowest norms, ties
//                    to the lower token id"
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

namespace l2kv {

// ------------------------------------------------------------ compact_ragged
constexpr int kRagThreads = 256;
constexpr int kRagWaves = kRagThreads / kWaveSize;
constexpr int kRagUnroll = 4;
constexpr int kRagRowsPerBlock = kRagWaves * kRowsPerWaveLoad * kRagUnroll;   // 64

// Index of the sequence whose output range holds flat kept row j of a plane: the last s in
// [0, n_seq) with out_off[s] <= j (binary search; offsets ascend in a consistent batch, and
// whatever they hold the result is a valid sequence index).
__device__ __forceinline__ int64_t owner_of_row(const int64_t* __restrict__ out_off, int64_t n_seq, int64_t j) {
    int64_t lo = 0, hi = n_seq - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (out_off[mid] <= j) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// grid.x = chunks_per_plane * n_planes: the kept rows of a plane, all sequences back to back
// (as kept_idx holds them), are cut into chunks of 64 consecutive rows, so every workgroup has
// a full chunk whatever the lengths of the sequences are (a launch sized by the longest
// sequence would leave almost half of its workgroups without work on a batch of mixed lengths).
// A row group takes 4 consecutive flat rows, which may belong to different sequences.
template <int W>
__global__ __launch_bounds__(kRagThreads)
void compact_ragged_kernel(const char* __restrict__ K, const char* __restrict__ V,
                           const float* __restrict__ norms, const int32_t* __restrict__ kept_idx,
                           int64_t n_seq, int64_t total_tokens, const int64_t* __restrict__ in_off,
                           const int64_t* __restrict__ out_off, int64_t total_kept,
                           int64_t chunks_per_plane, const int64_t* __restrict__ slot_off,
                           int64_t total_slots, char* __restrict__ Kc, char* __restrict__ Vc,
                           float* __restrict__ norms_c, int32_t* __restrict__ pos_c) {
    using P = Pieces<W>;                               // byte copy: rows shared among lanes in 16-byte pieces
    constexpr int64_t kRowBytes = kRowLanes * 4 * W;
    const int64_t chunk = blockIdx.x % chunks_per_plane;
    const int64_t plane = blockIdx.x / chunks_per_plane;
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    const int c = lane % kRowLanes;
    const int rg = lane / kRowLanes;

    const int64_t first = chunk * kRagRowsPerBlock + (wave * kRowsPerWaveLoad + rg) * kRagUnroll;
    if (first >= total_kept) return;
    const int32_t* idx = kept_idx + plane * total_kept;

    // per row: its sequence, source row and destination slot; a row that the (possibly
    // inconsistent) offset arrays do not place inside its sequence's ranges is skipped
    int64_t src[kRagUnroll], dst[kRagUnroll];
    int32_t tok[kRagUnroll];
    bool live[kRagUnroll];
    int64_t seq = owner_of_row(out_off, n_seq, first);
#pragma unroll
    for (int u = 0; u < kRagUnroll; ++u) {
        const int64_t j = first + u < total_kept ? first + u : total_kept - 1;
        while (seq + 1 < n_seq && out_off[seq + 1] <= j) ++seq;
        const Range in = clamped_range(in_off, seq, total_tokens);
        const Range outr = clamped_range(out_off, seq, total_kept);
        const Range slots = clamped_range(slot_off, seq, total_slots);
        const int64_t k = outr.count < slots.count ? outr.count : slots.count;   // never write past the sequence's slots
        const int64_t local = j - outr.first;
        live[u] = first + u < total_kept && local >= 0 && local < k && in.count > 0;
        int32_t t = idx[j];
        const int64_t T = in.count > 0 ? in.count : 1;
        t = t < 0 ? 0 : (t < T ? t : (int32_t)(T - 1));      // stay inside the sequence whatever idx holds
        tok[u] = t;
        // a skipped row still gets an in-bounds source (row 0 of the plane) so the loads below need no branch
        src[u] = plane * total_tokens + (live[u] ? in.first + t : 0);
        dst[u] = plane * total_slots + slots.first + (live[u] ? local : 0);
    }
    Words<W> kr[kRagUnroll], vr[kRagUnroll];
#pragma unroll
    for (int u = 0; u < kRagUnroll; ++u) kr[u] = load_words_stream<W, P::kStride>(K + src[u] * kRowBytes + c * P::kBytes);
#pragma unroll
    for (int u = 0; u < kRagUnroll; ++u) vr[u] = load_words_stream<W, P::kStride>(V + src[u] * kRowBytes + c * P::kBytes);
#pragma unroll
    for (int u = 0; u < kRagUnroll; ++u) {
        if (live[u]) {
            store_words_stream<W, P::kStride>(Kc + dst[u] * kRowBytes + c * P::kBytes, kr[u]);
            store_words_stream<W, P::kStride>(Vc + dst[u] * kRowBytes + c * P::kBytes, vr[u]);
            if (c == 0) {
                norms_c[dst[u]] = norms[src[u]];
                pos_c[dst[u]] = tok[u];
            }
        }
    }
}

l2kv_status compact_ragged_dispatch(const void* K, const void* V, const float* norms, l2kv_dtype dt,
                                    const int32_t* kept_idx, int32_t n_planes, int32_t n_seq,
                                    int64_t total_tokens, const int64_t* in_off, const int64_t* out_off,
                                    int64_t total_kept, int64_t max_kept, const int64_t* slot_off,
                                    int64_t total_slots, int32_t D, void* Kc, void* Vc, float* norms_c,
                                    int32_t* pos_c, hipStream_t stream) {
    (void)max_kept;                                    // the launch is sized by total_kept
    const int row_bytes = D * (dt == L2KV_F32 ? 4 : 2);
    const int64_t cpp = (total_kept + kRagRowsPerBlock - 1) / kRagRowsPerBlock;
    const int64_t blocks = cpp * n_planes;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
#define L2KV_RAG(WW)                                                                               \
    hipLaunchKernelGGL((compact_ragged_kernel<WW>), dim3((unsigned)blocks), dim3(kRagThreads), 0,  \
                       stream, static_cast<const char*>(K), static_cast<const char*>(V), norms,   \
                       kept_idx, (int64_t)n_seq, total_tokens, in_off, out_off, total_kept, cpp,   \
                       slot_off, total_slots, static_cast<char*>(Kc), static_cast<char*>(Vc),      \
                       norms_c, pos_c)
    switch (row_bytes) {
        case 128: L2KV_RAG(2); break;
        case 256: L2KV_RAG(4); break;
        case 512: L2KV_RAG(8); break;
        default: return L2KV_ERR_SHAPE;
    }
#undef L2KV_RAG
    return launch_status();
}

// -------------------------------------------------------------- stream_append
// One 16-lane row group per (layer, sequence, KV head).  Knew, Vnew are
// [n_layers][n_seq][Hkv][D]; the plane of (layer, head) is layer*Hkv + head.
template <typename E, int D>
__global__ __launch_bounds__(256)
void stream_append_kernel(const char* __restrict__ Knew, const char* __restrict__ Vnew, int64_t n_rows,
                          int64_t n_seq, int64_t Hkv, const int32_t* __restrict__ token_ids,
                          const int64_t* __restrict__ slot_off, int64_t total_slots,
                          const int32_t* __restrict__ lens_in, int32_t* __restrict__ lens_out,
                          char* __restrict__ Kc, char* __restrict__ Vc, float* __restrict__ norms_c,
                          int32_t* __restrict__ pos_c) {
#pragma clang fp contract(off)
    using S = Slice<E, D>;
    const int c = threadIdx.x % kRowLanes;
    int64_t r = (int64_t)blockIdx.x * (256 / kRowLanes) + threadIdx.x / kRowLanes;   // (layer, seq, head) row
    const bool live = r < n_rows;
    r = live ? r : n_rows - 1;                    // idle groups shadow the last row, stores skipped
    const int64_t head = r % Hkv;
    const int64_t seq = (r / Hkv) % n_seq;
    const int64_t layer = r / (Hkv * n_seq);
    const int64_t plane = layer * Hkv + head;

    const int32_t len = lens_in[seq];
    const Range slots = clamped_range(slot_off, seq, total_slots);
    const bool room = len >= 0 && len < slots.count;   // a full sequence is left untouched
    const Words<S::kWords> kr = load_words<S::kWords>(Knew + r * S::kRowBytes + c * S::kBytes);
    const Words<S::kWords> vr = load_words<S::kWords>(Vnew + r * S::kRowBytes + c * S::kBytes);

    // squared norm in the library's fixed order (chunk left to right, neighbour tree)
    float x[S::kElems];
    widen<E, D>(kr, x);
    float acc = x[0] * x[0];
#pragma unroll
    for (int e = 1; e < S::kElems; ++e) {
        const float sq = x[e] * x[e];
        acc = acc + sq;
    }
    const float norm = row16_tree_sum(acc);

    if (live && room) {
        const int64_t slot = plane * total_slots + slots.first + len;
        store_words<S::kWords>(Kc + slot * S::kRowBytes + c * S::kBytes, kr);
        store_words<S::kWords>(Vc + slot * S::kRowBytes + c * S::kBytes, vr);
        if (c == 0) {
            norms_c[slot] = norm;
            pos_c[slot] = token_ids[seq];
        }
    }
    if (live && plane == 0 && c == 0) lens_out[seq] = room ? len + 1 : len;
}

l2kv_status stream_append_dispatch(const void* Knew, const void* Vnew, l2kv_dtype dt, int32_t n_layers,
                                   int32_t n_seq, int32_t Hkv, int32_t D, const int32_t* token_ids,
                                   const int64_t* slot_off, int64_t total_slots, const int32_t* lens_in,
                                   int32_t* lens_out, void* Kc, void* Vc, float* norms_c, int32_t* pos_c,
                                   hipStream_t stream) {
    const int64_t n_rows = (int64_t)n_layers * n_seq * Hkv;
    const int64_t blocks = (n_rows + 15) / 16;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
#define L2KV_APP(EE, DD)                                                                           \
    hipLaunchKernelGGL((stream_append_kernel<EE, DD>), dim3((unsigned)blocks), dim3(256), 0, stream, \
                       static_cast<const char*>(Knew), static_cast<const char*>(Vnew), n_rows,     \
                       (int64_t)n_seq, (int64_t)Hkv, token_ids, slot_off, total_slots, lens_in,     \
                       lens_out, static_cast<char*>(Kc), static_cast<char*>(Vc), norms_c, pos_c)
    if (dt == L2KV_F32) {
        if (D == 64) L2KV_APP(F32, 64); else L2KV_APP(F32, 128);
    } else {
        if (D == 64) L2KV_APP(BF16, 64); else if (D == 128) L2KV_APP(BF16, 128); else L2KV_APP(BF16, 256);
    }
#undef L2KV_APP
    return launch_status();
}

// --------------------------------------------------------------- stream_evict
constexpr int kEvictThreads = 256;
constexpr int kEvictWaves = kEvictThreads / kWaveSize;

// One team of lanes per (plane, sequence): a whole workgroup (kTeam = 256), or one wave of a
// workgroup that serves four of them (kTeam = 64, for batches whose sequences are short: the
// work of a team is a chain of dependent loads, so more and smaller teams keep more of them in
// flight; no LDS and no barrier then).  Every eviction is one arg-max over the occupied slots
// of key = (norm bits << 32 | token id): per-lane scan, wave reduction with shuffles, and for
// workgroup teams 4 wave results through LDS.  In the steady state of a growing budget at most
// one slot goes per step.
template <int W, int kTeam>
__global__ __launch_bounds__(kEvictThreads)
void stream_evict_kernel(int64_t n_seq, int64_t n_teams, const int64_t* __restrict__ slot_off, int64_t total_slots,
                         const int32_t* __restrict__ lens_in, const int32_t* __restrict__ budgets,
                         int32_t* __restrict__ lens_out, char* __restrict__ Kc, char* __restrict__ Vc,
                         float* __restrict__ norms_c, int32_t* __restrict__ pos_c) {
    constexpr int64_t kSliceBytes = 4 * W;
    constexpr int64_t kRowBytes = kRowLanes * kSliceBytes;
    __shared__ unsigned long long s_key[kEvictWaves];
    __shared__ int32_t s_slot[kEvictWaves];
    const int64_t team = (int64_t)blockIdx.x * (kEvictThreads / kTeam) + threadIdx.x / kTeam;
    if (team >= n_teams) return;                   // a whole wave (teams are waves or workgroups)
    const int tid = threadIdx.x % kTeam;           // position in the team
    const int64_t seq = team % n_seq;
    const int64_t plane = team / n_seq;
    const int lane = threadIdx.x % kWaveSize;
    [[maybe_unused]] const int wave = threadIdx.x / kWaveSize;

    const Range slots = clamped_range(slot_off, seq, total_slots);
    const int64_t cap = slots.count;
    int32_t len = lens_in[seq];
    len = len < 0 ? 0 : (len < cap ? len : (int32_t)cap);
    int32_t budget = budgets[seq];
    budget = budget < 0 ? 0 : budget;
    const int64_t base = plane * total_slots + slots.first;
    const uint32_t* nb = reinterpret_cast<const uint32_t*>(norms_c) + base;
    float* nw = norms_c + base;
    int32_t* pw = pos_c + base;

    while (len > budget) {                         // uniform over the workgroup
        // Per-lane scan over the NORMS only (half of the bytes a scan of norms and token ids would
        // read): eight slots per lane and step, their loads issued before the first compare
        // (positions past the end re-read the last slot, which cannot beat itself).  Token ids
        // are fetched only where they decide: when two norms tie, and once per lane at the end.
        uint32_t best_norm = 0;
        int32_t best_slot = -1, best_id = 0;
        bool have_id = false;
        constexpr int kScan = 8;
        for (int32_t j0 = tid; j0 < len; j0 += kScan * kTeam) {
            uint32_t nv[kScan];
            int32_t js[kScan];
#pragma unroll
            for (int u = 0; u < kScan; ++u) {
                const int32_t j = j0 + u * kTeam;
                js[u] = j < len ? j : len - 1;
                nv[u] = nb[js[u]];
            }
#pragma unroll
            for (int u = 0; u < kScan; ++u) {
                if (best_slot < 0 || nv[u] > best_norm) {
                    best_norm = nv[u];
                    best_slot = js[u];
                    have_id = false;
                } else if (nv[u] == best_norm && js[u] != best_slot) {        // rare: equal norms
                    if (!have_id) best_id = pw[best_slot];
                    have_id = true;
                    const int32_t id = pw[js[u]];
                    if ((uint32_t)id > (uint32_t)best_id) {
                        best_id = id;
                        best_slot = js[u];
                    }
                }
            }
        }
        if (best_slot >= 0 && !have_id) best_id = pw[best_slot];
        unsigned long long best = ((unsigned long long)best_norm << 32) | (uint32_t)best_id;
        // keys are distinct (token ids are), so "larger key" is a total order; -1 marks "none"
#pragma unroll
        for (int off = kWaveSize / 2; off > 0; off >>= 1) {
            const unsigned long long ok = __shfl_xor(best, off);
            const int32_t os = __shfl_xor(best_slot, off);
            if (os >= 0 && (best_slot < 0 || ok > best)) {
                best = ok;
                best_slot = os;
            }
        }
        if constexpr (kTeam == kEvictThreads) {
            if (lane == 0) {
                s_key[wave] = best;
                s_slot[wave] = best_slot;
            }
            __syncthreads();
            best = s_key[0];
            best_slot = s_slot[0];
#pragma unroll
            for (int w = 1; w < kEvictWaves; ++w) {
                if (s_slot[w] >= 0 && (best_slot < 0 || s_key[w] > best)) {
                    best = s_key[w];
                    best_slot = s_slot[w];
                }
            }
        }
        const int32_t last = len - 1;
        if (best_slot != last) {
            // move the last slot into the hole: first 16 lanes K, next 16 lanes V
            if (tid < 2 * kRowLanes) {
                char* buf = tid < kRowLanes ? Kc : Vc;
                const int c = tid % kRowLanes;
                const Words<W> row = load_words<W>(buf + (base + last) * kRowBytes + c * kSliceBytes);
                store_words<W>(buf + (base + best_slot) * kRowBytes + c * kSliceBytes, row);
            } else if (tid == 2 * kRowLanes) {
                nw[best_slot] = nw[last];
                pw[best_slot] = pw[last];
            }
        }
        len = last;
        // moves visible to the team before its next scan (and the LDS reusable)
        if constexpr (kTeam == kEvictThreads) __syncthreads();
        else __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    }
    if (plane == 0 && tid == 0) lens_out[seq] = len;
}

l2kv_status stream_evict_dispatch(l2kv_dtype dt, int32_t n_planes, int32_t n_seq, int32_t D,
                                  const int64_t* slot_off, int64_t total_slots, const int32_t* lens_in,
                                  const int32_t* budgets, int32_t* lens_out, void* Kc, void* Vc,
                                  float* norms_c, int32_t* pos_c, hipStream_t stream) {
    const int row_bytes = D * (dt == L2KV_F32 ? 4 : 2);
    const int64_t teams = (int64_t)n_planes * n_seq;
    // sequences of a few thousand slots on average: one wave per (plane, sequence)
    const bool waves = total_slots / n_seq <= 8192;
    const int64_t blocks = waves ? (teams + kEvictWaves - 1) / kEvictWaves : teams;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
#define L2KV_EV(WW)                                                                               \
    hipLaunchKernelGGL((waves ? stream_evict_kernel<WW, kWaveSize> : stream_evict_kernel<WW, kEvictThreads>), \
                       dim3((unsigned)blocks), dim3(kEvictThreads), 0,                            \
                       stream, (int64_t)n_seq, teams, slot_off, total_slots, lens_in, budgets, lens_out,  \
                       static_cast<char*>(Kc), static_cast<char*>(Vc), norms_c, pos_c)
    switch (row_bytes) {
        case 128: L2KV_EV(2); break;
        case 256: L2KV_EV(4); break;
        case 512: L2KV_EV(8); break;
        default: return L2KV_ERR_SHAPE;
    }
#undef L2KV_EV
    return launch_status();
}

// ---------------------------------------------------------------- length order
// order[r] = the sequence with the r-th largest length (equal lengths: lower
// index first), by rank counting in one workgroup: a permutation of 0..n_seq-1
// whatever lens holds.  Meant for batch set-up, not for the decode loop.
constexpr int kOrderLdsSeqs = 8192;    // batches up to this size are ranked out of LDS

__global__ __launch_bounds__(1024)
void length_order_kernel(const int32_t* __restrict__ lens, int32_t n_seq, int32_t* __restrict__ order) {
    __shared__ int32_t s_len[kOrderLdsSeqs];
    const bool in_lds = n_seq <= kOrderLdsSeqs;
    if (in_lds) {
        for (int32_t s = threadIdx.x; s < n_seq; s += (int32_t)blockDim.x) s_len[s] = lens[s];
        __syncthreads();
    }
    for (int32_t s = threadIdx.x; s < n_seq; s += (int32_t)blockDim.x) {
        const int32_t mine = in_lds ? s_len[s] : lens[s];
        int32_t rank = 0;
        if (in_lds) {
            for (int32_t t = 0; t < n_seq; ++t) {
                const int32_t other = s_len[t];
                rank += (other > mine || (other == mine && t < s)) ? 1 : 0;
            }
        } else {
            for (int32_t t = 0; t < n_seq; ++t) {
                const int32_t other = lens[t];
                rank += (other > mine || (other == mine && t < s)) ? 1 : 0;
            }
        }
        order[rank] = s;
    }
}

l2kv_status length_order_dispatch(const int32_t* lens, int32_t n_seq, int32_t* order, hipStream_t stream) {
    // small batches need only as many lanes as sequences (fewer waves to start and retire)
    const unsigned threads = n_seq <= 64 ? 64u : (n_seq <= 256 ? 256u : 1024u);
    hipLaunchKernelGGL(length_order_kernel, dim3(1), dim3(threads), 0, stream, lens, n_seq, order);
    return launch_status();
}

}  // namespace l2kv
