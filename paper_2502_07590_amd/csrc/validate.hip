// Optional debug check of an index tensor against the idx contract of the stage-2 calls: values in
// [0, L), distinct within a row, and strictly ascending when the caller promises sorted rows (the
// L2-blocked kernels cut every row into contiguous segments by binary search, which is only correct
// for ascending rows).  Every kernel here exits normally whatever the index holds; the verdict goes to
// a small report in the caller's workspace that the host reads back.
#include <algorithm>

#include "common.h"

namespace dsv {

// report[0] = number of offending rows; report[1] = smallest (slot-independent) id bh * L + row of one.
__device__ __forceinline__ void flag_row(unsigned long long *report, int bh, int L, int64_t row)
{
    atomicAdd(&report[0], 1ull);
    atomicMin(&report[1], (unsigned long long)((int64_t)bh * L + row));
}

// One block walks rows blockIdx.x, blockIdx.x + gridDim.x, ... of one head.
//   SORTED: every entry in range and larger than its predecessor (which implies distinct).
//   else:   every entry in range, and no key twice: a bitmap of L bits in LDS, set with atomicOr; the
//           row's own words are cleared again afterwards, so the bitmap is all-zero between rows.
template <bool SORTED>
__global__ __launch_bounds__(256) void idx_validate_kernel(const int32_t *__restrict__ idx, int L, HeadTable tab,
                                                           unsigned long long *__restrict__ report)
{
    extern __shared__ uint32_t bitmap[];  // [(L + 31) / 32] when !SORTED
    __shared__ int bad;
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int32_t *base = idx + tab.off[slot];
    if (!SORTED) {
        for (int w = threadIdx.x; w < (L + 31) / 32; w += 256) bitmap[w] = 0u;
    }
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    for (int64_t i = blockIdx.x; i < L; i += gridDim.x) {
        const int32_t *row = base + i * k;
        int mine = 0;
        for (int t = threadIdx.x; t < k; t += 256) {
            const int v = row[t];
            if (v < 0 || v >= L) { mine = 1; continue; }
            if (SORTED) {
                if (t > 0 && row[t - 1] >= v) mine = 1;
            } else {
                const uint32_t bit = 1u << (v & 31);
                if (atomicOr(&bitmap[v >> 5], bit) & bit) mine = 1;
            }
        }
        if (mine) bad = 1;  // benign race: every writer stores 1
        __syncthreads();
        if (!SORTED) {
            for (int t = threadIdx.x; t < k; t += 256) {
                const int v = row[t];
                if (v >= 0 && v < L) bitmap[v >> 5] = 0u;
            }
        }
        if (threadIdx.x == 0 && bad) flag_row(report, bh, L, i);
        __syncthreads();
        if (threadIdx.x == 0) bad = 0;
        __syncthreads();
    }
}

__global__ void validate_reset_kernel(unsigned long long *report)
{
    report[0] = 0ull;
    report[1] = ~0ull;
}

dsv_status launch_idx_validate(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const int32_t *idx,
                               unsigned long long *report_dev, int64_t *report_host, hipStream_t st)
{
    const bool sorted = (p.flags & DSV_FLAG_SORTED_INDEX) != 0;
    const size_t lds = sorted ? 0 : (size_t)((p.L + 31) / 32) * 4;
    if (lds > (64u << 10)) return DSV_EUNSUPPORTED;
    hipLaunchKernelGGL(validate_reset_kernel, dim3(1), dim3(1), 0, st, report_dev);
    DSV_LAUNCH_CHECK();
    const int row_blocks = std::min(p.L, 2048);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid(row_blocks, tabs[t].n);
        if (sorted)
            hipLaunchKernelGGL(idx_validate_kernel<true>, grid, dim3(256), 0, st, idx, p.L, tabs[t], report_dev);
        else
            hipLaunchKernelGGL(idx_validate_kernel<false>, grid, dim3(256), lds, st, idx, p.L, tabs[t], report_dev);
        DSV_LAUNCH_CHECK();
    }
    unsigned long long host[2] = {0ull, ~0ull};
    DSV_HIP_CHECK(hipMemcpyAsync(host, report_dev, sizeof(host), hipMemcpyDeviceToHost, st));
    DSV_HIP_CHECK(hipStreamSynchronize(st));
    if (report_host) {
        report_host[0] = (int64_t)host[0];
        report_host[1] = host[0] ? (int64_t)(host[1] / (unsigned long long)p.L) : -1;
        report_host[2] = host[0] ? (int64_t)(host[1] % (unsigned long long)p.L) : -1;
    }
    return host[0] ? DSV_EINVAL : DSV_OK;
}

}  // namespace dsv
