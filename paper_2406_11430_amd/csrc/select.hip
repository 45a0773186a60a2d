// l2kv_select: per head, the k positions that come first in the total order
// (bit pattern of the fp32 squared norm, token index), written in ascending
// token order.  This is the eviction rule of arXiv 2406.11430 (Sec. 1: keep
// the lowest-norm keys; Eq. 5: exactly m pairs dropped per layer and head)
// with ties resolved towards the lower token index.
//
// One workgroup of 1024 lanes per head (512 for the packed variant below).
// The keys (norm bits, complemented for the keep-highest control) sit in
// registers -- 32 per lane covers 32k tokens -- so nothing is re-read from
// memory.  The k-th smallest key tau is found
// exactly by a 32-step binary search on its bits: step b counts the keys below
// (prefix | 1<<b) with wave ballots + popcounts (scalar unit), one LDS atomic
// per wave and one barrier.  No histogram, no data-dependent contention.
// Heads of up to 131072 tokens use the same search on packed halves: the upper
// 16 bits of all keys fit the registers two to a word (16 steps), then the
// lower 16 bits of the keys that tie on the upper half are packed the same way
// (16 more steps); the keys are read three more times from L2 (repack, count,
// emit) instead of 32.  Longer heads fall back to re-reading the keys in every
// step.
// The emit is ordered: every wave owns a contiguous token range, so a prefix
// over the 16 wave totals plus a running ballot prefix gives each kept token
// its output slot; keys equal to tau are admitted in token order until the
// budget k is met.
#include "l2kv_device.hpp"
#include "l2kv_host.hpp"

namespace l2kv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWaveSize;   // 16
constexpr int kSelMaxRegKeys = 32;                   // keys per lane held in registers

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The packed variant runs 512 lanes with twice the register budget per lane:
// 128 words of two 16-bit halves = 256 keys per lane, 131072 per workgroup.
constexpr int kSelPackedThreads = 512;
constexpr int kSelPackedRegs = 128;

// E > 0 : keys of the head fit E per lane and are cached in registers.
// E == 0: streaming variant, keys are re-read from memory (L2) in every pass.
// E == -1: packed variant, 256 keys per lane as 16-bit halves (T <= 131072).
// Ragged batches: [n_planes][total_in] norms, sequence s at in_off[s]..in_off[s+1];
// its kept positions (relative to the sequence start) go to
// [n_planes][total_out] at out_off[s]..out_off[s+1].  in_off == NULL: uniform.
struct RaggedSelect {
    const int64_t* in_off;
    const int64_t* out_off;
    int64_t n_seq, total_in, total_out;
};

template <int E>
__global__ __launch_bounds__(E == -1 ? kSelPackedThreads : kSelThreads)
void select_kernel(const uint32_t* __restrict__ norm_bits, int64_t T, uint32_t k, uint32_t flip,
                   int32_t* __restrict__ kept_idx, int32_t* __restrict__ kept_count,
                   RaggedSelect rag) {
    constexpr bool kInRegs = E > 0;
    constexpr bool kPacked = E == -1;
    constexpr int kWaves = (kPacked ? kSelPackedThreads : kSelThreads) / kWaveSize;
    __shared__ uint32_t s_count[32];
    __shared__ uint32_t s_lt[kSelWaves];
    __shared__ uint32_t s_eq[kSelWaves];

    const int64_t head = blockIdx.x;
    const int lane = threadIdx.x % kWaveSize;
    const int wave = threadIdx.x / kWaveSize;
    const uint32_t* src = norm_bits + head * T;
    int32_t* out = kept_idx + head * (int64_t)k;
    if (rag.in_off != nullptr) {
        // ragged batch: block = (plane, sequence); sizes and places come from the offset arrays
        const int64_t plane = head / rag.n_seq;
        const int64_t seq = head % rag.n_seq;
        const Range in = clamped_range(rag.in_off, seq, rag.total_in);
        const Range outr = clamped_range(rag.out_off, seq, rag.total_out);
        T = in.count;
        const int64_t kk = outr.count;
        if (T <= 0 || kk <= 0) return;                       // whole workgroup: nothing to select
        k = (uint32_t)(kk < T ? kk : T);                     // never more than there are
        src = norm_bits + plane * rag.total_in + in.first;
        out = kept_idx + plane * rag.total_out + outr.first;
    }

    // Wave w owns tokens [w*span, (w+1)*span), span a multiple of 64; iteration
    // e of lane l looks at token w*span + e*64 + l.
    const int64_t iters = kInRegs ? E
                          : kPacked ? 2 * kSelPackedRegs
                                    : (((T + kWaves - 1) / kWaves + kWaveSize - 1) / kWaveSize);
    const int64_t span = iters * kWaveSize;
    // Token positions fit 32 bits: T < 2^31 and the padded range ends below T + 2^17.
    const uint32_t t0 = (uint32_t)(wave * span + lane);
    const uint32_t T32 = (uint32_t)T;

    // Branch-free: positions past the end re-read the last key (in bounds) and
    // are replaced by the largest key, which is never "below" anything.  Such
    // padding sits after every real token, so in the ordered emit it is reached
    // only after all real keys equal to tau, when the budget is already met.
    // `base` is this lane's first position, passed through launder() by every
    // pass that re-reads the keys: otherwise the compiler keeps all addresses
    // and bounds predicates of one pass alive for the next and spills them.
    auto launder = [](uint32_t x) -> uint32_t {
        asm volatile("" : "+v"(x));
        return x;
    };
    auto fetch_at = [&](uint32_t base, int64_t e) -> uint32_t {
        const uint32_t t = base + (uint32_t)e * kWaveSize;
        const uint32_t v = src[t < T32 ? t : T32 - 1] ^ flip;
        return t < T32 ? v : 0xffffffffu;
    };
    auto fetch = [&](int64_t e) -> uint32_t { return fetch_at(t0, e); };

    uint32_t regs[kInRegs ? E : 1];
    if constexpr (kInRegs) {
#pragma unroll
        for (int e = 0; e < E; ++e) regs[e] = fetch(e);
    }
    if (threadIdx.x < 32) s_count[threadIdx.x] = 0;
    __syncthreads();

    // ---- k-th smallest key by binary search on its bits (MSB first) -------
    uint32_t prefix = 0;     // tau so far
    uint32_t less = 0;       // number of keys < prefix
    if constexpr (kPacked) {
        uint32_t pk[kSelPackedRegs];
        // one 16-step search over the packed halves in pk; `want` keys are sought
        auto search16 = [&](int count_slot, uint32_t want, uint32_t& found, uint32_t& below_found) {
            uint32_t pre = 0, lo = 0;
            for (int bit = 15; bit >= 0; --bit) {
                const uint32_t cand = pre | (1u << bit);
                // per-lane counters here (compare + add-with-carry): 128 wave ballots
                // per step would need more scalar registers than there are
                uint32_t mine = 0;
#pragma unroll
                for (int r = 0; r < kSelPackedRegs; ++r) {
                    mine += (pk[r] & 0xffffu) < cand ? 1u : 0u;
                    mine += (pk[r] >> 16) < cand ? 1u : 0u;
                }
                uint32_t cnt = mine;
#pragma unroll
                for (int off = kWaveSize / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
                if (lane == 0 && cnt) atomicAdd(&s_count[count_slot + bit], cnt);
                __syncthreads();
                const uint32_t below = s_count[count_slot + bit];
                if (below < want) {
                    pre = cand;
                    lo = below;
                }
            }
            found = pre;
            below_found = lo;
        };
        // upper halves of all keys (padding reads as 0xffff and is never "below")
        // (batches of 4 words, fenced for the scheduler: issuing all 128 loads and
        // their bounds predicates at once would not fit the register files)
        const uint32_t base1 = launder(t0);
#pragma unroll
        for (int r0 = 0; r0 < kSelPackedRegs; r0 += 4) {
#pragma unroll
            for (int r = r0; r < r0 + 4; ++r)
                pk[r] = (fetch_at(base1, 2 * r) >> 16) | (fetch_at(base1, 2 * r + 1) & 0xffff0000u);
            __builtin_amdgcn_sched_barrier(0);
        }
        uint32_t tau_hi, less_hi;
        search16(16, k, tau_hi, less_hi);
        // lower halves of the keys that tie on the upper half; every other key
        // is parked at 0xffff, which no candidate value exceeds
        const uint32_t base2 = launder(t0);
#pragma unroll
        for (int r0 = 0; r0 < kSelPackedRegs; r0 += 4) {
#pragma unroll
            for (int r = r0; r < r0 + 4; ++r) {
                const uint32_t a = fetch_at(base2, 2 * r), b = fetch_at(base2, 2 * r + 1);
                const uint32_t la = (a >> 16) == tau_hi ? (a & 0xffffu) : 0xffffu;
                const uint32_t lb = (b >> 16) == tau_hi ? (b & 0xffffu) : 0xffffu;
                pk[r] = la | (lb << 16);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        uint32_t tau_lo, less_lo;
        search16(0, k - less_hi, tau_lo, less_lo);
        prefix = (tau_hi << 16) | tau_lo;
        less = less_hi + less_lo;
    } else {
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand = prefix | (1u << bit);
            uint32_t cnt = 0;
            if constexpr (kInRegs) {
#pragma unroll
                for (int e = 0; e < E; ++e) cnt += __popcll(__ballot(regs[e] < cand));
            } else {
                for (int64_t e = 0; e < iters; ++e) cnt += __popcll(__ballot(fetch(e) < cand));
            }
            if (lane == 0 && cnt) atomicAdd(&s_count[bit], cnt);
            __syncthreads();
            const uint32_t below = s_count[bit];
            if (below < k) {     // the k-th smallest is >= cand
                prefix = cand;
                less = below;
            }
        }
    }
    const uint32_t tau = prefix;
    const uint32_t need_eq = k - less;   // >= 1 keys equal to tau are kept, lowest tokens first

    // ---- per-wave totals, then ordered emit ---------------------------------
    uint32_t lt_w = 0, eq_w = 0;
    auto tally = [&](uint32_t key, int64_t) {
        lt_w += __popcll(__ballot(key < tau));
        eq_w += __popcll(__ballot(key == tau));
    };
    if constexpr (kInRegs) {
#pragma unroll
        for (int e = 0; e < E; ++e) tally(regs[e], e);
    } else {
        for (int64_t e = 0; e < iters; ++e) tally(fetch(e), e);
    }
    if (lane == 0) {
        s_lt[wave] = lt_w;
        s_eq[wave] = eq_w;
    }
    __syncthreads();
    uint32_t lt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) {
        lt_before += s_lt[w];
        eq_before += s_eq[w];
    }
    uint32_t out_base = lt_before + (eq_before < need_eq ? eq_before : need_eq);
    uint32_t eq_base = eq_before;

    auto emit = [&](uint32_t key, int64_t e) {
        const uint32_t t = t0 + (uint32_t)e * kWaveSize;
        const bool is_lt = key < tau;
        const bool is_eq = key == tau;
        const uint64_t eq_mask = __ballot(is_eq);
        const bool keep = is_lt || (is_eq && (eq_base + lanes_below(eq_mask)) < need_eq);
        const uint64_t keep_mask = __ballot(keep);
        if (keep) out[out_base + lanes_below(keep_mask)] = (int32_t)t;
        out_base += __popcll(keep_mask);
        eq_base += __popcll(eq_mask);
    };
    if constexpr (kInRegs) {
#pragma unroll
        for (int e = 0; e < E; ++e) emit(regs[e], e);
    } else {
        for (int64_t e = 0; e < iters; ++e) emit(fetch(e), e);
    }
    if (kept_count != nullptr && threadIdx.x == 0) kept_count[head] = (int32_t)k;
}

template <int E>
static void launch_select(const float* norms, int64_t n_heads, int64_t T, int64_t k, uint32_t flip,
                          int32_t* kept_idx, int32_t* kept_count, hipStream_t stream,
                          RaggedSelect rag = RaggedSelect{nullptr, nullptr, 0, 0, 0}) {
    hipLaunchKernelGGL((select_kernel<E>), dim3((unsigned)n_heads),
                       dim3(E == -1 ? kSelPackedThreads : kSelThreads), 0, stream,
                       reinterpret_cast<const uint32_t*>(norms), T, (uint32_t)k, flip, kept_idx,
                       kept_count, rag);
}

// Picks the kernel variant from the (longest) head length and launches it.
static void launch_select_for_length(int64_t longest, const float* norms, int64_t n_heads, int64_t T,
                                     int64_t k, uint32_t flip, int32_t* kept_idx, int32_t* kept_count,
                                     hipStream_t stream, RaggedSelect rag) {
    const int64_t per_lane = (longest + kSelThreads - 1) / kSelThreads;
    if (per_lane <= 1)       launch_select<1>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (per_lane <= 2)  launch_select<2>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (per_lane <= 4)  launch_select<4>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (per_lane <= 8)  launch_select<8>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (per_lane <= 16) launch_select<16>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (per_lane <= kSelMaxRegKeys)
        launch_select<32>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else if (longest <= (int64_t)kSelPackedThreads * 2 * kSelPackedRegs)
        launch_select<-1>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
    else
        launch_select<0>(norms, n_heads, T, k, flip, kept_idx, kept_count, stream, rag);
}

// Keys of the keep-random control (arXiv 2406.11430 Sec. 4, where a random
// subset of the tokens is kept): a counter-based hash of (seed, head, token) written as bit patterns
// into an fp32 array, on which l2kv_select_k then keeps the k lowest.  The hash
// is x = token*0x9E3779B1 + head*0x85EBCA77 + seed followed by the 32-bit
// finalizer of MurmurHash3.
__global__ __launch_bounds__(256)
void random_keys_kernel(int64_t total, int64_t T, uint32_t seed, uint32_t* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const uint32_t head = (uint32_t)(i / T), t = (uint32_t)(i % T);
    uint32_t x = t * 0x9E3779B1u + head * 0x85EBCA77u + seed;
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    keys[i] = x;
}

l2kv_status random_keys_dispatch(int64_t n_heads, int64_t T, uint32_t seed, float* keys, hipStream_t stream) {
    const int64_t total = n_heads * T;
    const int64_t blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
    hipLaunchKernelGGL(random_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, total, T, seed,
                       reinterpret_cast<uint32_t*>(keys));
    return launch_status();
}

l2kv_status select_dispatch(const float* norms, int64_t n_heads, int64_t T, int64_t k,
                            l2kv_mode mode, int32_t* kept_idx, int32_t* kept_count,
                            void* workspace, hipStream_t stream) {
    (void)workspace;
    if (n_heads > 0x7fffffffLL) return L2KV_ERR_SHAPE;
    const uint32_t flip = mode == L2KV_KEEP_HIGHEST ? 0xffffffffu : 0u;
    launch_select_for_length(T, norms, n_heads, T, k, flip, kept_idx, kept_count, stream,
                             RaggedSelect{nullptr, nullptr, 0, 0, 0});
    return launch_status();
}

l2kv_status select_ragged_dispatch(const float* norms, int32_t n_planes, int32_t n_seq,
                                   int64_t total_tokens, const int64_t* in_off, const int64_t* out_off,
                                   int64_t total_kept, int64_t max_len, l2kv_mode mode,
                                   int32_t* kept_idx, hipStream_t stream) {
    const int64_t blocks = (int64_t)n_planes * n_seq;
    if (blocks > 0x7fffffffLL) return L2KV_ERR_SHAPE;
    const uint32_t flip = mode == L2KV_KEEP_HIGHEST ? 0xffffffffu : 0u;
    launch_select_for_length(max_len, norms, blocks, 0, 0, flip, kept_idx, nullptr, stream,
                             RaggedSelect{in_off, out_off, n_seq, total_tokens, total_kept});
    return launch_status();
}

}  // namespace l2kv
