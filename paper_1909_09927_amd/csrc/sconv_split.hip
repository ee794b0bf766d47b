// Channel split across workgroups, for launches too small to fill the chip.
//
// A deep layer at batch 1 (512 channels on a 7x7 or 14x14 map) has a handful of spatial tiles and
// a few filter blocks: a dozen workgroups, each walking all the channels with one staged filter
// chunk in flight, so the whole launch waits on memory latency, chunk after chunk, on a few compute
// units.  Splitting the channel range over NSS workgroups per tile multiplies the workgroups (and
// the filter fetches in flight) by NSS.  The sums of Section 5.4 are associative, so each
// workgroup stores the raw partial sums of its channel range - the plain convolution layout,
// no ReLU, no pooling - into slice number ss of a workspace, and the small kernel below adds
// the slices in a fixed order (slice 0 first: results do not depend on scheduling) and applies the
// epilogue of Sections 5.5 / 6: ReLU, and the max over the pooling window when fused.
//
// The workspace is the caller's: lent per device and stream with sconv_set_workspace and looked up
// for every launch.  Without one no launch is split; the library allocates nothing.
#include <map>
#include <utility>

#include "sconv_internal.h"

namespace sconv {

namespace {

__global__ __launch_bounds__(256) void split_sum_kernel(const float* __restrict__ part, float* __restrict__ y,
                                                        int nss, long long slice, long long total, int relu,
                                                        const float* __restrict__ bias, int K, int plane)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float v = part[i];
    for (int s = 1; s < nss; ++s) v += part[s * slice + i];
    if (bias) v += bias[(i / plane) % K];
    if (relu) v = fmaxf(v, 0.0f);
    y[i] = v;
}

// one thread per pooled result; the window's convolution results are summed over the slices first
__global__ __launch_bounds__(256) void split_pool_kernel(Problem p, const float* __restrict__ part,
                                                         float* __restrict__ y, int nss, long long slice,
                                                         long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int pwi = (int)(i % p.PW);
    long long q = i / p.PW;
    const int phi = (int)(q % p.PH);
    const long long nk = q / p.PH;
    const float* src = part + (nk * p.OH + (long long)phi * p.ps) * p.OW + (long long)pwi * p.ps;
    float m = -INFINITY;
    for (int py = 0; py < p.ph; ++py)
        for (int px = 0; px < p.pw; ++px) {
            const float* e = src + py * p.OW + px;
            float v = e[0];
            for (int s = 1; s < nss; ++s) v += e[s * slice];
            m = fmaxf(m, v);
        }
    y[i] = fmaxf(m + bias_of(p, (size_t)(nk % p.K)), 0.0f);   // bias, ReLU: both commute with the maximum
}

struct Lent {
    float* ptr;
    size_t bytes;
};
std::map<std::pair<int, hipStream_t>, Lent> g_lent;   // under the dispatcher's lock
thread_local Lent g_cur = {nullptr, 0};                 // the workspace of the launch being planned
thread_local Lent g_given = {nullptr, 0};               // the workspace passed with the call in progress
thread_local bool g_given_on = false;

}  // namespace

int split_workspace_set(void* ws, size_t bytes, hipStream_t stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SCONV_ELAUNCH;
    const auto key = std::make_pair(dev, stream);
    if (!ws)
        g_lent.erase(key);
    else
        g_lent[key] = Lent{static_cast<float*>(ws), bytes};
    return SCONV_OK;
}

void split_workspace_clear() { g_lent.clear(); }

bool split_workspace_lent(hipStream_t stream, bool any_stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (!any_stream) return g_lent.count(std::make_pair(dev, stream)) != 0;
    for (const auto& kv : g_lent)
        if (kv.first.first == dev) return true;
    return false;
}

void split_scratch_given(void* ws, size_t bytes, bool on)
{
    g_given = Lent{static_cast<float*>(ws), bytes};
    g_given_on = on;
}

bool split_scratch_is_given() { return g_given_on; }

void split_scratch_select(hipStream_t stream)
{
    if (g_given_on) {   // a call that brought its own workspace (or none) does not look at the lent ones
        g_cur = g_given;
        return;
    }
    g_cur = Lent{nullptr, 0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    auto it = g_lent.find(std::make_pair(dev, stream));
    if (it != g_lent.end()) g_cur = it->second;
}

bool split_scratch_possible(hipStream_t) { return g_cur.ptr != nullptr; }
float* split_scratch(hipStream_t) { return g_cur.ptr; }
size_t split_scratch_bytes() { return g_cur.bytes; }

// Scratch of the entry point that may not allocate (sconv_forward_static): partial sums of a split
// launch, in device memory that is part of the loaded code object.  Every device the library runs on
// holds its own copy, at its own address, until the process ends.  In host code the array's name is
// only a handle for the symbol lookup below; kernels get the looked-up address as an argument.
__device__ __align__(256) static float scratch[kStaticScratchBytes / sizeof(float)];

namespace {
constexpr int kMaxDevices = 64;
float* g_static_ptr[kMaxDevices];   // per device, under the dispatcher's lock
}

int split_static_scratch(float** ptr, size_t* bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCONV_ELAUNCH;
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SCONV_ELAUNCH;
        g_static_ptr[dev] = static_cast<float*>(p);
    }
    *ptr = g_static_ptr[dev];
    *bytes = kStaticScratchBytes;
    return SCONV_OK;
}

int launch_split_reduce(const Problem& p, bool pooled, const float* part, int nss, float* y, hipStream_t stream)
{
    const long long slice = (long long)p.N * p.K * p.OH * p.OW;
    if (!pooled) {
        hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)((slice + 255) / 256)), dim3(256), 0, stream, part, y,
                           nss, slice, slice, p.relu, p.bias, p.K, p.OH * p.OW);
    } else {
        const long long total = (long long)p.N * p.K * p.PH * p.PW;
        hipLaunchKernelGGL(split_pool_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p, part,
                           y, nss, slice, total);
    }
    return launch_status();
}

}  // namespace sconv
