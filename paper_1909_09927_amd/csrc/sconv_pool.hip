// Stand-alone ReLU + max pooling of a stored convolution result: the second kernel of the unfused
// path (Section 5.5 stores the convolution tensor, a pooling layer then reads it back), kept to
// measure what the fused kernel of Section 6 saves.  One thread per pooled result, lanes along the
// pooled row; bound by HBM traffic: the convolution tensor read once, the pooled tensor written once.
#include "sconv_internal.h"

namespace sconv {

namespace {

__global__ __launch_bounds__(256) void maxpool_kernel(Problem p, long long total,
                                                      const float* __restrict__ conv, float* __restrict__ y)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const int pwi = (int)(i % p.PW);
        long long q = i / p.PW;
        const int phi = (int)(q % p.PH);
        const long long nk = q / p.PH;
        const float* src = conv + (nk * p.OH + (long long)phi * p.ps) * p.OW + (long long)pwi * p.ps;
        float m = 0.0f;   // ReLU: the maximum is taken over max(value, 0)
        for (int py = 0; py < p.ph; ++py)
            for (int px = 0; px < p.pw; ++px) m = fmaxf(m, src[py * p.OW + px]);
        y[i] = m;
    }
}

}  // namespace

int launch_maxpool(const Problem& p, const float* conv, float* y, hipStream_t stream)
{
    const long long total = (long long)p.N * p.K * p.PH * p.PW;
    long long blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;   // grid-stride beyond 64 workgroups per compute unit
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, total, conv, y);
    return launch_status();
}

}  // namespace sconv
