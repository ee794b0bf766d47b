// Internal declarations shared by the translation units of libsconv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sconv.h"

namespace sconv {

// Problem description with every derived size filled in by the host (see fill_problem).
struct Problem {
    int N, C, H, W, K, R, S, stride, pad, G;
    int Cg, Kg;          // channels / filters per group
    int OH, OW;          // convolution output
    int ph, pw, ps;      // pooling window and stride (0 when not pooling)
    int PH, PW;          // pooled output (0 when not pooling)
    int L;               // slots per window row = Cg*R*S
    int relu;            // apply max(.,0) before the store
    float zhint;         // the map's zero ratio as the caller reported it in the descriptor; negative: unknown
    const float* bias;   // device, [K]: added to every result of filter k before the ReLU; null = none
    const float* wprep;  // device: the filters in the transposed layout (filter_prep_bytes), written by the
                         // caller beforehand with sconv_filter_prep; null = none (a kernel that wants the layout
                         // writes it into the workspace before its launch)
};

// The bias of filter kglob (0 when the call carries none).
__device__ __forceinline__ float bias_of(const Problem& p, size_t kglob) { return p.bias ? p.bias[kglob] : 0.0f; }

// Validates a descriptor (pure host code) and fills a Problem.  pooled: the pooling fields
// are required and checked.  Returns SCONV_OK / SCONV_EINVAL / SCONV_EUNSUPPORTED.
int fill_problem(const sconv_desc_t* d, bool pooled, Problem* out);

// Kernel launchers.  Each returns SCONV_OK, SCONV_EUNSUPPORTED (shape outside what the variant
// covers; nothing was launched) or SCONV_ELAUNCH.
int launch_encode(const Problem& p, int fmt, const float* x, float* values, int32_t* index,
                  int32_t* count, hipStream_t stream);

// Two layers in one launch, one workgroup per image, the first layer's output kept in LDS (and copied to
// mid_out when that is not null).  SCONV_EUNSUPPORTED when the pair does not fit a workgroup's LDS or
// is grouped; SCONV_EINVAL when the second layer's input is not the first layer's output.
int launch_pair(const Problem& p1, bool pooled1, const Problem& p2, bool pooled2, const float* x, const float* w1,
                const float* w2, float* mid_out, float* y, hipStream_t stream);

// Counts examined and nonzero elements of x into counts[0], counts[1] (device); at most 4 Mi elements.
int launch_density_probe(const Problem& p, const float* x, unsigned long long* counts, hipStream_t stream);

// ReLU + max pooling of a stored convolution tensor [N][K][OH][OW] -> [N][K][PH][PW].
int launch_maxpool(const Problem& p, const float* conv, float* y, hipStream_t stream);

// General window-row kernel: any R, S, stride, pad, groups, pooling window of up to 64 results.
int launch_rows(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream);

// Element-stationary 3x3 / stride 1 / pad 1 kernel.  tap_supported tells whether it covers p.
bool tap_supported(const Problem& p, bool pooled);
int launch_tap(const Problem& p, bool pooled, const float* x, const float* w, float* y,
               hipStream_t stream);

// "geometry/WxS[xP]" of the plan launch_tap would take on this stream (after split_scratch_select).
bool describe_tap(const Problem& p, bool pooled, hipStream_t stream, char* out, size_t out_size);

// Matrix-core variant of the same kernel (3x3 / stride 1 / pad 1): four inputs per instruction.
bool quad_supported(const Problem& p, bool pooled);
int launch_quad(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream);

// Wide-granule matrix-core kernel: 3x3, any stride and padding, 16 window rows per instruction.
bool wide_supported(const Problem& p, bool pooled);
int launch_wide(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream);

// General matrix-core kernel: kernels up to 15x15, any stride, padding, grouping and channel count;
// 16 window rows per instruction, columns walked linearly.
bool gen_supported(const Problem& p, bool pooled);
int launch_gen(const Problem& p, bool pooled, const float* x, const float* w, float* y,
               hipStream_t stream);

// Matrix-core kernel for 1x1 / stride 1 / pad 0 convolutions (optional 2x2 / stride 2 pooling).
bool pw_supported(const Problem& p, bool pooled);
int launch_pointwise(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                     hipStream_t stream);

// A fixed decomposition in place of the cost models' choice: candidate geometry inside a kernel
// variant, wavefronts per workgroup, channel slices.  Set by the dispatcher (under its lock) around
// one launch - from the tuning cache or while sconv_tune tries the candidates; without one, the
// tuning-aid environment variables apply.
struct PlanPin {
    char geom[16];       // "" = any geometry
    int nwv, ncs;        // 0 = the model's choice
    int nss;             // workgroups splitting the channels of a tile (with nwv, ncs); 0 or 1 = none
};
const PlanPin* current_pin();

// Value of one of the library's tuning-aid environment variables as it was when the library first
// looked (or when sconv_env_refresh last ran); null when unset.
const char* env_value(const char* name);

// Geometry pin for a launcher: the dispatcher's, else the named environment variable's.
const char* pinned_geom(const char* env_name);
// Split pin "nwv,ncs" or "nwv,ncs,nss" likewise; all 0 when there is none.
void pinned_split(const char* env_name, int* nwv, int* ncs, int* nss = nullptr);

// Channel split across workgroups: every workgroup stores the raw partial sums of its channel
// range into slice ss of a workspace laid out [nss][N][K][OH][OW]; launch_split_reduce adds the
// slices in order and applies ReLU and, when pooled, the max over the pooling window.  The
// workspace is lent by the caller per device and stream (split_workspace_set, behind
// sconv_set_workspace).  The dispatcher selects the stream's workspace before every launch
// (split_scratch_select, under its lock); the launchers then ask whether there is one, for its
// address and for its size.  Without one they plan without a split.
constexpr size_t kSplitWorkspaceCap = size_t(64) << 20;   // more than this is never asked for
int split_workspace_set(void* ws, size_t bytes, hipStream_t stream);
void split_workspace_clear();
// whether a workspace is lent for this stream of the current device (any_stream: for any of its streams)
bool split_workspace_lent(hipStream_t stream, bool any_stream);
void split_scratch_select(hipStream_t stream);
// A workspace that comes with one call (the ..._ws entry points) instead of the stream's lent one:
// set before the call's launches are planned and cleared (on = false) after them; per calling thread.
// ws may be null: that call then plans without a split.
void split_scratch_given(void* ws, size_t bytes, bool on);
bool split_scratch_is_given();
bool split_scratch_possible(hipStream_t stream);
float* split_scratch(hipStream_t stream);
size_t split_scratch_bytes();
int launch_split_reduce(const Problem& p, bool pooled, const float* part, int nss, float* y,
                        hipStream_t stream);
// The library's own scratch for callers that may not allocate: a fixed array in device memory, one
// copy per device.  Looks its address up on the current device at the first call there.
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
int split_static_scratch(float** ptr, size_t* bytes);

// Transposed layout of 3x3 filters for kernels whose 64 lanes read 64 consecutive filters of one (channel,
// tap) in one load: w[K][Cg][9] -> wt[group][block of 64 filters][channel * 9 + tap][64], the blocks of a
// group padded with zeros to an even count (so that a lane pair of filters k, k + 64 always has both blocks).
// filter_prep_bytes: size of the copy, a multiple of 256; launch_filter_prep enqueues the kernel that writes it.
size_t filter_prep_bytes(const Problem& p);
int launch_filter_prep(const Problem& p, const float* w, float* wt, hipStream_t stream);

// Candidate geometry names of the variants (for sconv_tune); null-terminated arrays.
const char* const* pw_geoms();
const char* const* tap_geoms();
const char* const* quad_geoms();
const char* const* wide_geoms();
const char* const* gen_geoms();

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? SCONV_OK : SCONV_ELAUNCH;
}

}  // namespace sconv
