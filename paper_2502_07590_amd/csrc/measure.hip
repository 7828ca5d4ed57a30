// Measurement aid (not an operation of the method): how fast can the chip gather 256-byte rows from an
// L2-resident range through the vector memory path, with the forward sweep's lane layout, index staging
// and XCD-aware block order, but no arithmetic?  That rate is the practical ceiling the stage-2 sweeps are
// measured against (the derived peak of the path is 64 bytes per clock per CU).
#include "stage2_core.h"

namespace dsv {

// One block = 64 query rows (4 lanes per row, 16 rows per wave) of one range; block b runs on XCD b % 8 and
// every XCD walks its ranges one after the other, as the L2-blocked sweeps do.  Every row gathers, for each
// of its k index entries, one K row and one V row of the range (2 x 256 bytes, bf16 d = 128).
__global__ __launch_bounds__(256) void gather_ceiling_kernel(const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
                                                             const int32_t *__restrict__ idx, int k, int nq,
                                                             int idx_rows, int range_rows, int n_ranges,
                                                             uint32_t *__restrict__ out)
{
    constexpr int D = 128, LPR = 4, CH = D / LPR;
    typedef LaneLayout<bf16_t, D, LPR> LL;
    const int nqb = (nq + 63) / 64;
    const int64_t b = blockIdx.x;
    const int xcd = (int)(b & 7);
    const int64_t local = b >> 3;
    const int t = (int)(local / nqb), qb = (int)(local % nqb);
    const int range = t * 8 + xcd;
    if (range >= n_ranges) return;
    const int lane = threadIdx.x & 63;
    const int s = lane % LPR;
    const int q = min(qb * 64 + (int)threadIdx.x / LPR, nq - 1);
    const int32_t *row = idx + ((int64_t)range * idx_rows + q % idx_rows) * k;
    const bf16_t *Kb = K + (int64_t)range * range_rows * D;
    const bf16_t *Vb = V + (int64_t)range * range_rows * D;
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];
    int32_t *stage = stage_all[threadIdx.x / LPR];
    uint32_t sink = 0;
    StagedIndex<LPR> si;
    si.request(row, 0, k, s);
    for (int c0 = 0; c0 < k; c0 += kStage) {
        si.park(stage, s);
        if (c0 + kStage < k) si.request(row, c0 + kStage, k, s);
        const int n = min(kStage, k - c0);
        for (int it = 0; it + 4 <= n; it += 4) {
            RowChunk<bf16_t, CH> kc[4], vc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t j = (uint32_t)stage[it + u];
                kc[u] = gather_chunk<bf16_t, D, LPR>(Kb, j, (uint32_t)LL::off(s));
                vc[u] = gather_chunk<bf16_t, D, LPR>(Vb, j, (uint32_t)LL::off(s));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // every loaded word is "used" (so that the loads stay whole) without costing an instruction
#pragma unroll
                for (int w = 0; w < RowChunk<bf16_t, CH>::NW; ++w) asm volatile("" ::"v"(kc[u].w[w]), "v"(vc[u].w[w]));
                sink ^= kc[u].w[0] ^ vc[u].w[0];
            }
        }
    }
    if (s == 0 && qb * 64 + (int)threadIdx.x / LPR < nq) out[(int64_t)range * nq + q] = sink;
}

}  // namespace dsv

using namespace dsv;

extern "C" dsv_status dsv_measure_gather_ceiling(int32_t n_ranges, int32_t range_rows, int32_t nq, int32_t k,
                                                 int32_t idx_rows, const void *K, const void *V, const int32_t *idx,
                                                 void *out, int32_t reps, float *ms, void *hip_stream)
{
    if (!K || !V || !idx || !out || !ms) return DSV_EINVAL;
    if (n_ranges < 1 || range_rows < 1 || nq < 1 || k < 1 || k % 4 || idx_rows < 1 || idx_rows > nq || reps < 1) return DSV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0, e1;
    DSV_HIP_CHECK(hipEventCreate(&e0));
    DSV_HIP_CHECK(hipEventCreate(&e1));
    const int64_t blocks = (int64_t)((n_ranges + 7) / 8 * 8) * ((nq + 63) / 64);
    if (blocks > 0x7FFFFFFF) return DSV_EINVAL;
    dsv_status rc = DSV_OK;
    for (int rep = 0; rep <= reps; ++rep) {  // rep 0 warms the caches and is not timed
        if (rep == 1 && hipEventRecord(e0, st) != hipSuccess) rc = DSV_EHIP;
        hipLaunchKernelGGL(gather_ceiling_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)K,
                           (const bf16_t *)V, idx, k, nq, idx_rows, range_rows, n_ranges, (uint32_t *)out);
        if (hipGetLastError() != hipSuccess) rc = DSV_EHIP;
    }
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) rc = DSV_EHIP;
    float total = 0.f;
    if (rc == DSV_OK && hipEventElapsedTime(&total, e0, e1) != hipSuccess) rc = DSV_EHIP;
    *ms = total / reps;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
