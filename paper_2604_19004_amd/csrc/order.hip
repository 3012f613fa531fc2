// Order of the rows inside the launch of the heavy-row kernel.  Its persistent
// workgroups take rows one by one from the end of the list; a row of a
// power-law matrix can hold a hundred times the work of the median row of its
// bin, and one that is handed out late keeps a single CU busy long after all
// others have finished.  Sorting the list by the product count (a radix sort
// of a few hundred thousand keys, a library primitive) hands out the longest
// rows first.
#include <hipcub/hipcub.hpp>

#include "ocean_internal.hpp"

namespace ocean {

namespace {
constexpr size_t SORT_ALIGN = 256;
inline size_t sort_up(size_t b) { return (b + SORT_ALIGN - 1) / SORT_ALIGN * SORT_ALIGN; }

__global__ void k_product_keys(const int64_t *__restrict__ prod, const int32_t *__restrict__ rows, int64_t count,
                               uint32_t *__restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) {
        const int64_t p = prod[rows[i]];
        keys[i] = p > 0xffffffffLL ? 0xffffffffu : (uint32_t)p;
    }
}

size_t cub_bytes(int64_t count)
{
    size_t bytes = 0;
    (void)hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, (const uint32_t *)nullptr, (uint32_t *)nullptr,
                                             (const int32_t *)nullptr, (int32_t *)nullptr, (int)count);
    return bytes;
}
}  // namespace

size_t sort_rows_scratch_bytes(int64_t count)
{
    if (count <= 1 || count > 0x7fffffffLL) return 0;
    return 3 * sort_up((size_t)count * 4) + sort_up(cub_bytes(count));
}

// rows[0..count) reordered in place by ascending product count.  scratch: sort_rows_scratch_bytes(count) bytes.
hipError_t launch_sort_rows_by_products(const int64_t *prod, int32_t *rows, int64_t count, void *scratch, hipStream_t s)
{
    if (count <= 1 || count > 0x7fffffffLL) return hipSuccess;
    char *base = static_cast<char *>(scratch);
    const size_t arr = sort_up((size_t)count * 4);
    uint32_t *keys_in = reinterpret_cast<uint32_t *>(base);
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(base + arr);
    int32_t *rows_out = reinterpret_cast<int32_t *>(base + 2 * arr);
    void *tmp = base + 3 * arr;
    size_t tmp_bytes = cub_bytes(count);
    hipLaunchKernelGGL(k_product_keys, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, prod, rows, count, keys_in);
    hipError_t e = hipcub::DeviceRadixSort::SortPairs(tmp, tmp_bytes, keys_in, keys_out, rows, rows_out, (int)count, 0, 32, s);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(rows, rows_out, (size_t)count * 4, hipMemcpyDeviceToDevice, s);
}

}  // namespace ocean
