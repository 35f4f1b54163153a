// Upload-time helper: stable radix sort of (user id, upload position) pairs on the
// device, used once per index to turn user ids into dense ranks (the tie-break of the
// k-selection).  Kept in its own translation unit because the sort library's headers
// dominate compile time.  Not part of the search path.
#include <cstring>
#include <hip/hip_runtime.h>
#include <rocprim/rocprim.hpp>
#include <cstdint>

extern "C" int ivf_internal_sort_pairs(const int64_t* keys_in, int64_t* keys_out,
                                       const uint32_t* vals_in, uint32_t* vals_out, size_t n,
                                       hipStream_t stream) {
    if (n == 0) return 0;
    size_t tmp_bytes = 0;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys_in, keys_out, vals_in,
                                             vals_out, n, 0, 64, stream);
    if (e != hipSuccess) return (int)e;
    void* tmp = nullptr;
    e = hipMalloc(&tmp, tmp_bytes ? tmp_bytes : 16);
    if (e != hipSuccess) return (int)e;
    e = rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, vals_out, n, 0, 64,
                                  stream);
    hipError_t e2 = hipStreamSynchronize(stream);
    hipFree(tmp);
    return (int)(e != hipSuccess ? e : e2);
}
