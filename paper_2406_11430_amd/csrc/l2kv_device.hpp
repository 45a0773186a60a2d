// Device-side helpers shared by the l2kv kernels (gfx950, wave64).
//
// Layout convention used by every streaming kernel: a K or V row is split over
// a "row group" of 16 consecutive lanes, lane c of the group owning the c-th
// sixteenth of the row (D/16 consecutive elements).  A wavefront therefore
// holds 4 rows per load instruction, and a DPP row (16 lanes) is exactly one
// cache row, so per-row reductions never leave the DPP row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace l2kv {

constexpr int kWaveSize = 64;
constexpr int kRowLanes = 16;   // lanes cooperating on one cache row
constexpr int kRowsPerWaveLoad = kWaveSize / kRowLanes;

// DPP control words (cross-lane operand swizzles inside a 16-lane row).
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppQuadEven = 0xA0;    // quad_perm [0,0,2,2]: every lane reads the even lane of its pair
constexpr int kDppQuadOdd = 0xF5;     // quad_perm [1,1,3,3]: every lane reads the odd lane of its pair
constexpr int kDppHalfMirror = 0x141; // lane i <- lane 7-i within 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <- lane 15-i within 16 lanes

template <int CTRL>
__device__ __forceinline__ float dpp_read(float v) {
    // Full row/bank masks with bound_ctrl: every lane reads a live lane, and the
    // compiler may fold the swizzle into the consuming VALU instruction.
    int iv = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, iv, CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a row group as a balanced binary tree over
// neighbouring lanes: (0+1),(2+3),... then pairs of those, etc.  After the two
// quad steps every lane of a quad holds the same value, so the mirror swizzles
// pair quad q with quad q^1 and then half h with half h^1.  IEEE addition is
// commutative, hence all 16 lanes end with the identical bit pattern.
__device__ __forceinline__ float row16_tree_sum(float p) {
    p = p + dpp_read<kDppXor1>(p);
    p = p + dpp_read<kDppXor2>(p);
    p = p + dpp_read<kDppHalfMirror>(p);
    p = p + dpp_read<kDppMirror>(p);
    return p;
}

// bf16 -> fp32 widening is a 16-bit shift (exact).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// A lane's slice of a row as W 32-bit words (W = 2, 4 or 8).
template <int W> struct Words { uint32_t w[W]; };

// How the 16 lanes of a row group share a row in the kernels whose result does not depend on
// which lane holds which element (row copies, dot products with both operands laid out alike):
// lane c takes the 16-byte pieces c, c + 16, ... of the row -- one piece of a 256-byte row, two
// of a 512-byte row, one 8-byte piece of a 128-byte row -- so that every load or store
// instruction of a row group covers contiguous bytes.  (Consecutive 32 bytes per lane make each
// instruction touch every second 16 bytes of a 512-byte row; measured on decode attention over
// such rows: 57 us against 43 us per launch.)  The loads and stores below take the byte distance
// between a lane's 16-byte pieces as kPieceStride: 16 = consecutive, Pieces<W>::kStride = shared
// as described, with p = row + c * Pieces<W>::kBytes.
template <int W> struct Pieces {
    static constexpr int kCount = W >= 4 ? W / 4 : 1;
    static constexpr int kBytes = 4 * W / kCount;                // bytes per piece
    static constexpr int kStride = kRowLanes * kBytes;           // bytes between a lane's pieces
};

template <int W, int kPieceStride = 16>
__device__ __forceinline__ Words<W> load_words(const void* p) {
    Words<W> r;
    if constexpr (W == 2) {
        uint2 v = *reinterpret_cast<const uint2*>(p);
        r.w[0] = v.x; r.w[1] = v.y;
    } else {
        static_assert(W % 4 == 0, "slice must be 8 bytes or a multiple of 16");
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            uint4 v = *reinterpret_cast<const uint4*>(static_cast<const char*>(p) + i * kPieceStride);
            r.w[4 * i + 0] = v.x; r.w[4 * i + 1] = v.y;
            r.w[4 * i + 2] = v.z; r.w[4 * i + 3] = v.w;
        }
    }
    return r;
}

// Streaming variants: data that is read or written exactly once per call and
// should not displace anything in the caches (non-temporal hint).
template <int W, int kPieceStride = 16>
__device__ __forceinline__ Words<W> load_words_stream(const void* p) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    Words<W> r;
    if constexpr (W == 2) {
        u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
        r.w[0] = v.x; r.w[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            u32x4 v = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4*>(static_cast<const char*>(p) + i * kPieceStride));
            r.w[4 * i + 0] = v.x; r.w[4 * i + 1] = v.y; r.w[4 * i + 2] = v.z; r.w[4 * i + 3] = v.w;
        }
    }
    return r;
}

// The same loads through a buffer descriptor (raw buffer, 32-bit data format): `byte_offset` is
// a 32-bit per-lane offset from the descriptor's base, bytes outside its range read as zero.
// Policy: plain, or the non-temporal hint of the streaming loads above.
constexpr int kRawBufferWord3 = 0x00020000;
constexpr int kBufferPolicyPlain = 0;
constexpr int kBufferPolicyStream = 2;
template <int W, int kPieceStride, int kPolicy>
__device__ __forceinline__ Words<W> buffer_load_words(__amdgpu_buffer_rsrc_t rsrc, int byte_offset) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    Words<W> r;
    if constexpr (W == 2) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_offset, 0, kPolicy);
        r.w[0] = v.x; r.w[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_offset + i * kPieceStride, 0, kPolicy);
            r.w[4 * i + 0] = v.x; r.w[4 * i + 1] = v.y; r.w[4 * i + 2] = v.z; r.w[4 * i + 3] = v.w;
        }
    }
    return r;
}

template <int W, int kPieceStride = 16>
__device__ __forceinline__ void store_words_stream(void* p, const Words<W>& r) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    if constexpr (W == 2) {
        u32x2 v = {r.w[0], r.w[1]};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
    } else {
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            u32x4 v = {r.w[4 * i + 0], r.w[4 * i + 1], r.w[4 * i + 2], r.w[4 * i + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<char*>(p) + i * kPieceStride));
        }
    }
}

template <int W, int kPieceStride = 16>
__device__ __forceinline__ void store_words(void* p, const Words<W>& r) {
    if constexpr (W == 2) {
        *reinterpret_cast<uint2*>(p) = make_uint2(r.w[0], r.w[1]);
    } else {
#pragma unroll
        for (int i = 0; i < W / 4; ++i)
            *reinterpret_cast<uint4*>(static_cast<char*>(p) + i * kPieceStride) =
                make_uint4(r.w[4 * i + 0], r.w[4 * i + 1], r.w[4 * i + 2], r.w[4 * i + 3]);
    }
}

// Range of sequence `seq` in a device-side offset array (off[seq] .. off[seq+1]),
// forced into [0, total]: whatever the array holds, first + count <= total, so a
// caller's inconsistent offsets give meaningless results but no access outside
// the tensor the offsets describe.
struct Range { int64_t first, count; };
__device__ __forceinline__ Range clamped_range(const int64_t* off, int64_t seq, int64_t total) {
    int64_t a = off[seq], b = off[seq + 1];
    a = a < 0 ? 0 : (a > total ? total : a);
    b = b < a ? a : (b > total ? total : b);
    return Range{a, b - a};
}

// Element type tags.
struct F32 { static constexpr int kBytes = 4; };
struct BF16 { static constexpr int kBytes = 2; };

// Slice geometry for element type E and head_dim D.
template <typename E, int D> struct Slice {
    static constexpr int kElems = D / kRowLanes;               // elements per lane
    static constexpr int kWords = kElems * E::kBytes / 4;      // 32-bit words per lane
    static constexpr int kBytes = kElems * E::kBytes;          // bytes per lane
    static constexpr int kRowBytes = D * E::kBytes;
};

// Widen a lane's slice to fp32 values in element order.
template <typename E, int D>
__device__ __forceinline__ void widen(const Words<Slice<E, D>::kWords>& r, float (&x)[Slice<E, D>::kElems]) {
    if constexpr (E::kBytes == 4) {
#pragma unroll
        for (int i = 0; i < Slice<E, D>::kElems; ++i) x[i] = __builtin_bit_cast(float, r.w[i]);
    } else {
#pragma unroll
        for (int i = 0; i < Slice<E, D>::kWords; ++i) {
            x[2 * i] = bf16_lo(r.w[i]);
            x[2 * i + 1] = bf16_hi(r.w[i]);
        }
    }
}

}  // namespace l2kv
