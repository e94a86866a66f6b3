// Device-wide radix sort of 64-bit edge keys (rocPRIM primitive), kept in its own translation unit.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "ctx.h"

namespace reinc {

size_t sort_keys_tmp_bytes(int64_t n)
{
    size_t bytes = 0;
    (void)rocprim::radix_sort_keys(nullptr, bytes, static_cast<uint64_t *>(nullptr), static_cast<uint64_t *>(nullptr),
                                   size_t(n > 0 ? n : 1), 0u, 64u, hipStream_t(nullptr));
    return bytes;
}

hipError_t sort_keys(void *tmp, size_t tmp_bytes, const uint64_t *in, uint64_t *out, int64_t n, unsigned begin_bit, unsigned end_bit,
                     hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    return rocprim::radix_sort_keys(tmp, tmp_bytes, in, out, size_t(n), begin_bit, end_bit, s);
}

}  // namespace reinc
