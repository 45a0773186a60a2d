// Decode-attention kernels for bf16 caches with 256-element rows (query groups of 1..4 heads):
// one translation unit per (element type, head size) so that the units compile in parallel.
#include "decode_kernels.hpp"

namespace l2kv {
template l2kv_status decode_by_group<BF16, 256>(int, const void*, const void*, const void*, int32_t, int32_t, int32_t,
                                             int64_t, int64_t, const int32_t*, const int64_t*, const int32_t*,
                                             float, const DecodePlan&, float*, void*, hipStream_t);
}  // namespace l2kv
