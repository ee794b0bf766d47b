// Density probe: how many elements of a feature map are nonzero (the test of Algorithm 1's scan,
// x != 0), so that the choice between the per-element vector kernel and the group-skipping matrix
// kernels can follow the zero ratio (Section 8.3 reports the method's time against the ratio; the first
// layers of a network are much denser than the deep ones, Section 8.2).  Reads at most 4 Mi elements:
// the whole map when it is smaller, else whole 256-element runs spread evenly over the tensor.
#include "sconv_internal.h"

namespace sconv {

namespace {

__global__ void probe_clear_kernel(unsigned long long* counts)
{
    counts[0] = 0;
    counts[1] = 0;
}

// run r of the sample starts at element r * run_stride; a run is 256 consecutive elements (one per thread)
__global__ __launch_bounds__(256) void probe_kernel(const float* __restrict__ x, long long total, long long runs,
                                                    long long run_stride, unsigned long long* counts)
{
    unsigned long long seen = 0, nonzero = 0;
    for (long long r = blockIdx.x; r < runs; r += gridDim.x) {
        const long long i = r * run_stride + threadIdx.x;
        const bool in = i < total;
        const float v = in ? x[i] : 0.0f;
        seen += __popcll(__ballot(in));
        nonzero += __popcll(__ballot(in && v != 0.0f));
    }
    if ((threadIdx.x & 63) == 0) {   // every wavefront counted its own lanes
        atomicAdd(&counts[0], seen);
        atomicAdd(&counts[1], nonzero);
    }
}

}  // namespace

int launch_density_probe(const Problem& p, const float* x, unsigned long long* counts, hipStream_t stream)
{
    const long long total = (long long)p.N * p.C * p.H * p.W;
    const long long all_runs = (total + 255) / 256;
    const long long max_runs = (4LL << 20) / 256;
    const long long runs = all_runs < max_runs ? all_runs : max_runs;
    const long long run_stride = runs == all_runs ? 256 : (total / runs) / 256 * 256;
    hipLaunchKernelGGL(probe_clear_kernel, dim3(1), dim3(1), 0, stream, counts);
    const unsigned blocks = (unsigned)(runs < 2048 ? runs : 2048);
    hipLaunchKernelGGL(probe_kernel, dim3(blocks), dim3(256), 0, stream, x, total, runs, run_stride, counts);
    return launch_status();
}

}  // namespace sconv
