// Analysis instrument of Sec. 2.3 (H1): the strict head-level hit rate.  A head scores 1 only
// if, at every decoding step, the candidates it selected hold the golden answer position of
// that step.  One launch folds one step's index lists into the running per-head flags.
#include "common.h"

namespace rs {

// one wave per (batch, head): lanes sweep the list, a ballot says whether the golden candidate is in it
__global__ __launch_bounds__(256) void selection_hit_kernel(const int32_t *__restrict__ idx, int BH, int K,
                                                            const int32_t *__restrict__ gold, int unit,
                                                            uint8_t *__restrict__ hit)
{
    const int w = (int)((blockIdx.x * (long)blockDim.x + threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    if (w >= BH) return;
    const int g = gold[w];
    if (g < 0) return;  // no golden position at this step for this head
    const int want = g / unit;
    const int32_t *row = idx + (long)w * K;
    bool found = false;
    for (int j = lane; j < K; j += 64) found |= (row[j] == want);
    if (__ballot(found) == 0ull && lane == 0) hit[w] = 0;
}

}  // namespace rs

using namespace rs;

extern "C" int32_t selection_hit_update(const int32_t *idx, int32_t B, int32_t H, int32_t K, const int32_t *gold,
                                        int32_t unit, uint8_t *hit, void *stream)
{
    if (!idx || !gold || !hit) return RS_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(idx) & 3u) || (reinterpret_cast<uintptr_t>(gold) & 3u)) return RS_INVALID_ARG;
    if (B <= 0 || H <= 0 || K <= 0 || unit <= 0) return RS_INVALID_ARG;
    const long BH = (long)B * H;
    if (BH > (1L << 24)) return RS_UNSUPPORTED;
    const unsigned blocks = (unsigned)((BH + 3) / 4);
    selection_hit_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>(idx, (int)BH, K, gold, unit, hit);
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}
