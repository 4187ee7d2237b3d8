// The two library primitives of the work-list construction (rocPRIM through hipCUB): an exclusive
// sum and a stable least-significant-digit radix sort of (word, task id) pairs.  Kept in their own
// translation unit: these templates take most of the library's compile time.
#include <hip/hip_runtime.h>
#include <hipcub/hipcub.hpp>
#include <stdint.h>

namespace same {

size_t wl_exclusive_sum_bytes(size_t n)
{
    size_t bytes = 0;
    (void)hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, (const uint32_t*)nullptr, (uint32_t*)nullptr, n);
    return bytes;
}

hipError_t wl_exclusive_sum(void* tmp, size_t tmp_bytes, const uint32_t* in, uint32_t* out, size_t n, hipStream_t st)
{
    return hipcub::DeviceScan::ExclusiveSum(tmp, tmp_bytes, in, out, n, st);
}

size_t wl_sort_pairs_bytes(size_t n, int end_bit)
{
    size_t bytes = 0;
    (void)hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, (const int32_t*)nullptr, (int32_t*)nullptr,
                                             (const int32_t*)nullptr, (int32_t*)nullptr, n, 0, end_bit);
    return bytes;
}

hipError_t wl_sort_pairs(void* tmp, size_t tmp_bytes, const int32_t* keys_in, int32_t* keys_out,
                         const int32_t* vals_in, int32_t* vals_out, size_t n, int end_bit, hipStream_t st)
{
    return hipcub::DeviceRadixSort::SortPairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, vals_out, n, 0, end_bit, st);
}

}  // namespace same
