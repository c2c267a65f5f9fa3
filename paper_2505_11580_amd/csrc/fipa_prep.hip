// Per-batch preparation (fp32 path, backward, and the bf16 forward with a generic head shape; the
// AlphaFold2-shape pack kernel does this work itself): centroid of the valid translations and
// the key-loop bound.  One workgroup per batch element.  The launch also clears the arrival
// counters of the attention kernel's key-range split, when there are any.  `cu` (or null): row
// offsets of a packed batch, chain b at rows cu[b] .. cu[b+1] - 1 instead of b L .. b L + L - 1.
#include "fipa_internal.h"

namespace fipa {

__global__ __launch_bounds__(256) void fipa_prep_kernel(const float *__restrict__ trans,
                                                        const uint8_t *__restrict__ mask, int L,
                                                        const int *__restrict__ cu,
                                                        float *__restrict__ cen,
                                                        int *__restrict__ kvlen,
                                                        int *__restrict__ counters, int n_counters)
{
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    for (int i = b * 256 + tid; i < n_counters; i += gridDim.x * 256) counters[i] = 0;
    float sx = 0.f, sy = 0.f, sz = 0.f;
    int cnt = 0, last = 0;
    const size_t row0 = cu ? (size_t)cu[b] : (size_t)b * L;
    const int len = cu ? cu[b + 1] - cu[b] : L;
    for (int i = tid; i < len; i += 256) {
        const bool ok = mask ? (mask[row0 + i] != 0) : true;
        if (ok) {
            const float *t = trans + (row0 + i) * 3;
            sx += t[0];
            sy += t[1];
            sz += t[2];
            cnt += 1;
            last = i + 1;
        }
    }
    __shared__ float red[4][256];
    __shared__ int redl[256];
    red[0][tid] = sx;
    red[1][tid] = sy;
    red[2][tid] = sz;
    red[3][tid] = (float)cnt;
    redl[tid] = last;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) {
            for (int a = 0; a < 4; ++a) red[a][tid] += red[a][tid + s];
            redl[tid] = max(redl[tid], redl[tid + s]);
        }
        __syncthreads();
    }
    if (tid == 0) {
        const float n = red[3][0] > 0.f ? red[3][0] : 1.f;
        cen[4 * b + 0] = red[0][0] / n;
        cen[4 * b + 1] = red[1][0] / n;
        cen[4 * b + 2] = red[2][0] / n;
        cen[4 * b + 3] = 0.f;
        kvlen[b] = redl[0];
    }
}

hipError_t launch_prep(const fipa_desc &d, const float *trans, const uint8_t *mask, const int *cu, float *cen,
                       int *kvlen, int *counters, int n_counters, hipStream_t stream)
{
    hipLaunchKernelGGL(fipa_prep_kernel, dim3(d.B), dim3(256), 0, stream, trans, mask, d.L, cu, cen,
                       kvlen, counters, n_counters);
    return hipGetLastError();
}

}  // namespace fipa
