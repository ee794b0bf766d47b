/*
 * sconv: zero-skipping direct convolution (+ fused ReLU / max-pooling) for AMD MI355X (gfx950).
 *
 * C ABI of the GPU library.  All tensors are fp32 and contiguous; every pointer marked
 * "device" is HIP device memory owned by the caller.  The library allocates and frees no device
 * memory (the only device memory of its own is the fixed 16 MiB array behind sconv_forward_static,
 * part of the loaded library).  Every entry point that launches work enqueues it on the given HIP stream
 * (a hipStream_t passed as void*; NULL = the default stream) and returns without synchronising.
 * Outputs are overwritten, never accumulated into.  Calls may come from several host threads
 * (planning and enqueueing are serialised inside the library); the only state kept between calls
 * is cached launch information (occupancy answers) for the device the first calls ran on - so one
 * process should drive one device -, the plans sconv_tune found, the workspaces lent with
 * sconv_set_workspace and the SCONV_* environment as first read.  Calls that change process state:
 * sconv_tune / sconv_tune_prep / sconv_tune_import / sconv_tune_reset (plan table), sconv_set_workspace /
 * sconv_clear_workspaces (lent workspaces), sconv_env_refresh; every other call only reads it.  A caller
 * that wants none of it uses the ..._ws or ..._prep forms and never tunes.
 *
 * Notation follows Table 1 of the paper: feature map i_h x i_w (H x W here), kernel k_h x k_w
 * (R x S), pooling window p_h x p_w, convolution stride c_s, pooling stride p_s.  Several input
 * channels, filters and images are handled as Section 7 describes: channels are scanned one
 * after another inside a window, filters and images only add independent results.
 *
 * Return value of every int function: 0 on success or a negative SCONV_E* code.  Argument
 * checks are pure host code and run before any GPU call.
 */
#ifndef SCONV_H
#define SCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N, C, H, W;          /* input  x[N][C][H][W]                                     */
    int32_t K, R, S;             /* filter w[K][C/groups][R][S]                              */
    int32_t stride, pad, groups; /* c_s; symmetric zero padding; groups G (C%G == K%G == 0)  */
    int32_t pool_h, pool_w, pool_stride; /* p_h, p_w, p_s; read only by the pooling calls    */
    int32_t flags;               /* SCONV_RELU: sconv_forward applies max(y, 0) before the
                                    store (Section 5.5).  The pooling path always applies it.
                                    SCONV_ZERO_RATIO(z): optional, the map's zero ratio if the
                                    caller knows it (see sconv_density) - a hint for the choice
                                    of kernel, never for the result.                            */
} sconv_desc_t;

enum { SCONV_RELU = 1,
       SCONV_PREPARED_FILTERS = 2 /* read by sconv_variant_name / sconv_plan_name only: name the plan of a
                                     ..._prep call that brings prepared filters; the forward calls ignore it */ };
/* Zero-ratio hint: bits 8..15 of flags hold 0 (not given) or 1 + round(254 * z), z in [0, 1]. */
enum { SCONV_ZERO_RATIO_SHIFT = 8, SCONV_ZERO_RATIO_MASK = 0xff << 8 };
#define SCONV_ZERO_RATIO(z) ((int32_t)((1 + (int32_t)((z) * 254.0 + 0.5)) << SCONV_ZERO_RATIO_SHIFT))
enum { SCONV_FMT_ECR = 0, SCONV_FMT_PECR = 1 };
enum {
    SCONV_OK = 0,
    SCONV_EINVAL = -1,       /* null pointer, non-positive size, C or K not divisible by groups,
                                pad >= R or pad >= S, empty output, pooling window larger than
                                the convolution output, unknown format or flag                 */
    SCONV_EUNSUPPORTED = -2, /* valid problem that exceeds a kernel limit (see each call)      */
    SCONV_ELAUNCH = -3,      /* the HIP runtime reported an error for the launch               */
    SCONV_ETOOLARGE = -4     /* sconv_forward_static: the problem exceeds the static scratch   */
};

/*
 * Output sizes (Section 5.3 and Eq. 3, floored): OH = (H + 2*pad - R)/c_s + 1, OW likewise;
 * PH = (OH - p_h)/p_s + 1, PW likewise (0 when the descriptor has no pooling window).
 * PH/PW may be NULL.  Host only.
 */
int sconv_output_dims(const sconv_desc_t* desc, int32_t* OH, int32_t* OW, int32_t* PH, int32_t* PW);

/*
 * Size of an encoding.  rows = N*G*OH*OW (ECR) or N*G*PH*PW*p_h*p_w (PECR);
 * slots_per_row = L = (C/G)*R*S.  Host only.
 */
int sconv_encode_sizes(const sconv_desc_t* desc, int fmt, int64_t* rows, int64_t* slots_per_row);

/*
 * Format conversion alone (Algorithm 1 for ECR, Algorithm 3 for PECR), materialised in device
 * memory.  One row per convolution window.  Row order: ECR (n, g, oh, ow) - one block row per
 * output row, one entry per output column (Section 5.2); PECR (n, g, ph, pw, py, px) - the
 * windows of one pooling window are adjacent, left to right then top to bottom (Section 6.2),
 * and a window that lies in several pooling windows is repeated.  Within a row the window is
 * scanned channel by channel, then kernel row, then kernel column; every element != 0 appends
 * its value to values[row][.] and its column c*R*S + r*S + s (its position in a filter) to
 * index[row][.].  count[row] = number appended; ECR stores -1 instead of 0 for an empty window.
 * Slots past the count are written as value +0.0f and index 0, so whole arrays are defined.
 *   x_dev      device, in : [N][C][H][W]
 *   values_dev device, out: [rows][L] fp32
 *   index_dev  device, out: [rows][L] int32
 *   count_dev  device, out: [rows]    int32
 * SCONV_EUNSUPPORTED if rows*L >= 2^40 or L >= 2^24.
 */
int sconv_encode(const sconv_desc_t* desc, int fmt, const float* x_dev, float* values_dev,
                 int32_t* index_dev, int32_t* count_dev, void* hip_stream);

/*
 * Sparse convolution (Section 5: conversion of every window to ECR on chip, then the
 * sparse row-times-filter product of Algorithm 2, optional ReLU, one store):
 *   y[n][k][oh][ow] = sum over the window's nonzeros of value * w[k][column],
 * the window of group g = k / (K/G).  Which zeros are skipped depends on the kernel variant the
 * shape selects (sconv_variant_name): "rows" and "tap3x3" skip every zero element; "quad3x3",
 * "quad1x1", "wide3x3" and "gen" issue products of several adjacent elements at a time on the matrix
 * pipe (groups of 6, 8, 16 and 16 elements) and skip a group only when all of its elements are zero, so a
 * zero inside a group that also holds a nonzero is multiplied (0 * w adds nothing for finite w;
 * with Inf or NaN filters the variants can differ).
 * A workspace (lent with sconv_set_workspace, or passed to the ..._ws forms) is used two ways.
 * (1) Launches too small to fill the chip - fewer than 128 workgroups ("tap3x3" and "gen": deep layers
 * at batch 1), "tap3x3" launches of up to 768 workgroups that walk 256 or more channels, 100-400 tiles of
 * "quad3x3" on a map 28 or more wide - are split along the channels over up to 16 workgroups per tile;
 * each stores the plain partial sums of its channel range into the workspace, and a second kernel on the
 * same stream adds them in a fixed order and applies bias and ReLU (and, for a fused call that small, the
 * pooling).  (2) "tap3x3" launches of 512 or more workgroups (256 for fused calls) with 128 or more
 * channels per group first write a transposed copy of the filters, [block of 64 filters][channel][tap][64],
 * into the workspace and run the form of the kernel that reads filters from it without staging
 * them in LDS (a caller with constant filters writes that copy once and passes it: the ..._prep calls below).
 * Results stay deterministic; the association of the fp32 sums differs between plans.
 *   x_dev device, in : [N][C][H][W]
 *   w_dev device, in : [K][C/G][R][S]
 *   y_dev device, out: [N][K][OH][OW]
 * SCONV_EUNSUPPORTED if a tensor has 2^31 or more elements.
 */
int sconv_forward(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, float* y_dev,
                  void* hip_stream);

/*
 * Sparse convolution fused with ReLU and max pooling (Section 6, Algorithm 4): the convolution
 * results of one pooling window are reduced on chip and only the pooled tensor is stored:
 *   y[n][k][ph][pw] = max over py < p_h, px < p_w of max(0, conv[n][k][ph*p_s+py][pw*p_s+px]).
 * (A launch too small to fill the chip - fewer than 128 workgroups, and only when a workspace is there,
 * see sconv_forward - is split across workgroups and passes its partial sums through that workspace; the
 * second kernel then pools.  Every larger fused call is one convolution kernel, whatever the pooling window,
 * also after sconv_tune: it does not offer a split to such a call.)
 *   y_dev device, out: [N][K][PH][PW]
 * SCONV_EUNSUPPORTED if p_h*p_w > 64 or a tensor has 2^31 or more elements.
 */
int sconv_pool_forward(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                       float* y_dev, void* hip_stream);

/*
 * The two forward calls with the layer's bias: bias_dev[k] (device, [K] fp32) is added to every result of
 * filter k before the ReLU - y = max(0, bias[k] + sum) - inside the same kernels' epilogues (for a split
 * launch, in the kernel that adds the partial sums).  The paper's kernels stop at the products and the
 * ReLU (Sections 5.5 and 6.4); the bias is the affine term the layers they are taken from carry, so
 * that one layer's output can feed the next layer directly.  Plans, workspaces and errors as the plain
 * calls; bias_dev NULL is SCONV_EINVAL (use the plain calls).
 */
int sconv_forward_bias(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, const float* bias_dev,
                       float* y_dev, void* hip_stream);
int sconv_pool_forward_bias(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                            const float* bias_dev, float* y_dev, void* hip_stream);

/*
 * Two consecutive layers in one launch with the first layer's output handed over on chip (Section 6.4:
 * when one thread block computes all pooling results they can stay in shared memory for the next
 * convolution layer; step 4 of the procedure of Section 5.1 then skips global memory).  One workgroup per
 * image holds the image, both filter tensors and the intermediate map in LDS, so this covers small pairs
 * only (4 * (C1*H*W + L1*K1' + K1*MH*MW + L2*K2') <= 160 KiB, K' = K rounded up to 64, MH x MW the first
 * layer's stored map; e.g. LeNet: 5x5 1->20 on 28x28 + 2x2/2 pooling, then 5x5 20->50 + pooling).
 *   first, second: the two layers; a layer with pooling fields set is conv + ReLU + max pooling (as
 *          sconv_pool_forward), one without is conv with its SCONV_RELU flag (as sconv_forward).  The
 *          second layer's input must be the first layer's output: N equal, C2 = K1, H2 x W2 = the first
 *          layer's (pooled) output size.  groups must be 1 in both.
 *   x_dev  device, in : [N][C1][H][W];  w1_dev, w2_dev device, in: the layers' filters
 *   bias1_dev, bias2_dev device, in, optional (NULL: none): [K1], [K2], added before the ReLU
 *   mid_dev device, out, optional (NULL: the intermediate map never leaves the chip): [N][K1][MH][MW]
 *   y_dev  device, out: the second layer's output
 * SCONV_EINVAL when the layers do not chain; SCONV_EUNSUPPORTED when the pair does not fit (call the
 * layers one after the other instead).  Zeros are skipped element by element in both layers.
 */
int sconv_pair_forward(const sconv_desc_t* first, const sconv_desc_t* second, const float* x_dev,
                       const float* w1_dev, const float* bias1_dev, const float* w2_dev, const float* bias2_dev,
                       float* mid_dev, float* y_dev, void* hip_stream);

/*
 * The unfused second step, for comparison with sconv_pool_forward: ReLU and max pooling of a
 * convolution tensor that sconv_forward stored (Section 5.5 followed by a pooling layer; Section 6
 * fuses the two to save this tensor's trip through memory):
 *   y[n][k][ph][pw] = max over py < p_h, px < p_w of max(0, conv[n][k][ph*p_s+py][pw*p_s+px]).
 * The descriptor is the convolution's (it fixes OH, OW) with its pooling fields.
 *   conv_dev device, in : [N][K][OH][OW]
 *   y_dev    device, out: [N][K][PH][PW]
 */
int sconv_maxpool(const sconv_desc_t* desc, const float* conv_dev, float* y_dev, void* hip_stream);

/*
 * Optional workspace.  Small launches (deep layers at batch 1: a handful of tiles) run 1.3-3.5x
 * faster when the channels of a tile are split over several workgroups, whose partial sums pass
 * through device scratch to a second kernel (see sconv_forward).  That scratch is the caller's:
 *   sconv_workspace_size: bytes the plans of this descriptor can use (0: none would; at most
 *            64 MiB of partial sums plus, for 3x3 layers, the size of the filter tensor with the
 *            filters of a group rounded up to a multiple of 128).  Host only.
 *   sconv_set_workspace: lends ws_dev (bytes long, 16-byte aligned) to every later forward or tuning
 *            call on hip_stream of the current device, until it is replaced or withdrawn
 *            (ws_dev NULL, bytes 0).  A launch whose plan needs more than was lent, and every
 *            launch on a stream without a workspace, runs unsplit (correct, slower on batch-1
 *            layers).  The caller keeps the memory alive while such launches - or graphs captured
 *            from them - can still run, and runs the launches that share a workspace in stream
 *            order: concurrent launches on one workspace race.  Contents need no initialisation.
 *            Nothing is enqueued, but the current device is asked of the HIP runtime (which
 *            initialises it).  The entry is keyed by (device, stream handle) and outlives the
 *            stream: withdraw a workspace (NULL, 0) before destroying its stream - a later stream
 *            that reuses the handle would otherwise inherit the stale pointer - or call
 *            sconv_clear_workspaces.  The ..._ws calls below need none of this.
 *   sconv_clear_workspaces: withdraws every lent workspace of every device and stream.
 */
int sconv_workspace_size(const sconv_desc_t* desc, int pooled, size_t* bytes);
int sconv_set_workspace(void* ws_dev, size_t bytes, void* hip_stream);
int sconv_clear_workspaces(void);

/*
 * sconv_forward / sconv_pool_forward (Sections 5 and 6) with the workspace as an argument of the
 * call instead of a buffer lent to the stream beforehand: nothing about the workspace is remembered
 * after the call returns, and a buffer lent with sconv_set_workspace is ignored for this call.
 *   ws_dev device, scratch: ws_bytes bytes, 16-byte aligned, contents irrelevant before and undefined
 *          after; NULL with ws_bytes 0: the call plans without a split.  sconv_workspace_size tells
 *          how much a descriptor can use; with less, smaller splits or none are planned.
 * The launches read and write ws_dev in stream order; the caller keeps it alive until they have
 * run and does not share it with launches that may run at the same time.
 * Errors as the plain calls, plus SCONV_EINVAL for a misaligned or half-given workspace.
 */
int sconv_forward_ws(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, float* y_dev,
                     void* ws_dev, size_t ws_bytes, void* hip_stream);
int sconv_pool_forward_ws(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, float* y_dev,
                          void* ws_dev, size_t ws_bytes, void* hip_stream);

/*
 * Prepared filters.  The vector kernel's fastest form for large 3x3 launches ("tap3x3", see sconv_forward)
 * has every wavefront read the nine taps of 64 consecutive filters of one channel in nine 256-byte loads,
 * which needs the filters in the layout [group][block of 64 filters][channel][tap][64] (blocks of a group
 * padded with zeros to an even count).  The plain calls write that copy into the workspace before every
 * such launch (about 10 us for 512 x 512 x 3 x 3 filters).  The paper's setting is inference: the filters
 * are transferred to the GPU once, before the first kernel (step 0 of the procedure in Section 5.1), and stay
 * as they are while feature maps flow through.  A caller in that setting writes the copy once and passes it
 * with every call.
 *   sconv_filter_prep_size: bytes of the prepared copy for this descriptor's filters (a multiple of 256);
 *            0 when no kernel reads the layout for it (anything but 3x3 / stride 1 / pad 1 with channels
 *            per group a multiple of 16).  Depends on K, C, groups, R, S only.  Host only.
 *   sconv_filter_prep: enqueues the kernel that writes the copy of w_dev into wprep_dev (device, out,
 *            256-byte aligned, wprep_bytes >= the size above).  SCONV_EUNSUPPORTED when the size is 0.
 *   sconv_forward_prep / sconv_pool_forward_prep: sconv_forward / sconv_pool_forward (Sections 5 and 6)
 *            with every optional operand as an argument of the call:
 *              wprep_dev device, in, optional (NULL with wprep_bytes 0): the prepared copy of w_dev - the
 *                    caller guarantees it was written from the same filters; a descriptor whose plans do not
 *                    read the layout ignores it.  With it the transposed-filter form needs no workspace.
 *              bias_dev  device, in, optional (NULL: none): as sconv_forward_bias.
 *              ws_dev    device, scratch, optional (NULL with ws_bytes 0): as sconv_forward_ws; a workspace
 *                    lent with sconv_set_workspace is ignored for this call.
 *            w_dev is still required: kernels that do not read the prepared layout read it.
 *            Nothing is remembered after the call returns.
 *   sconv_tune_prep: sconv_tune for calls that bring prepared filters (plans are remembered separately for
 *            calls with and without them: the transposed-filter form is about 10 us cheaper with them), the
 *            workspace being an argument as well.
 * Errors as the plain calls, plus SCONV_EINVAL for a misaligned, half-given or too small wprep_dev.
 */
int sconv_filter_prep_size(const sconv_desc_t* desc, size_t* bytes);
int sconv_filter_prep(const sconv_desc_t* desc, const float* w_dev, void* wprep_dev, size_t wprep_bytes,
                      void* hip_stream);
int sconv_forward_prep(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, const void* wprep_dev,
                       size_t wprep_bytes, const float* bias_dev, float* y_dev, void* ws_dev, size_t ws_bytes,
                       void* hip_stream);
int sconv_pool_forward_prep(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                            const void* wprep_dev, size_t wprep_bytes, const float* bias_dev, float* y_dev,
                            void* ws_dev, size_t ws_bytes, void* hip_stream);
int sconv_tune_prep(const sconv_desc_t* desc, int pooled, const float* x_dev, const float* w_dev,
                    const void* wprep_dev, size_t wprep_bytes, float* y_dev, void* ws_dev, size_t ws_bytes,
                    void* flush_dev, size_t flush_bytes, void* hip_stream, float* best_ms);

/*
 * sconv_forward for callers that cannot allocate or lend device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same result and plans as sconv_forward_ws,
 * but the workspace is the library's own: a fixed array of SCONV_STATIC_SCRATCH_BYTES (16 MiB) in
 * device memory that belongs to the loaded library (every GPU the library runs on holds its copy
 * until the process ends).  The call allocates and frees nothing and uses no allocating library
 * routine; the first call on a device looks the array's address up once (make that call outside a
 * graph capture).
 *   Limit: 2 * N*K*OH*OW * 4 bytes (two slices of partial sums, the smallest split) must fit the
 *   array; a larger problem is refused with SCONV_ETOOLARGE before anything is enqueued - use
 *   sconv_forward or sconv_forward_ws for it.
 *   The array keeps the previous call's contents; nothing in it needs clearing, because a split
 *   launch writes every partial sum it later reads.  All calls on one GPU share the array: run them
 *   in stream order on one stream.  Calls that overlap on one GPU (two streams, two threads) race.
 * Other errors as sconv_forward.
 */
enum { SCONV_STATIC_SCRATCH_BYTES = 16 << 20 };
int sconv_forward_static(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, float* y_dev,
                         void* hip_stream);

/*
 * Name of the kernel variant the two forward calls would pick for this descriptor (a static
 * string, for benchmark records and profiles).  pooled != 0 asks about sconv_pool_forward.
 * Variants: "quad1x1" (1x1 / stride 1 / pad 0, channels per group a multiple of 64), "quad3x3"
 * (3x3 / stride 1 / pad 1, channels per group a multiple of 16), "wide3x3" (3x3 of any stride and
 * padding, channels per group a multiple of 8; also preferred for maps up to 14 wide with 128 or
 * more filters and fewer than 256 channels per group), "tap3x3" (3x3 / pad 1, stride 1 or 2,
 * channels a multiple of 16; preferred for the deep layers - maps up to 14 wide with 256 or more
 * channels per group, maps up to 28 wide with 512 or more - and for launches too small to fill the
 * matrix kernels' tiles; with a workspace lent on a stream of the current device also for fused calls
 * on wider maps with 128 or more channels per group, while launches of 100-400 "quad3x3" tiles on maps
 * 28 or more wide are then "quad3x3", split, instead),
 * "gen" (every other shape with a kernel of at most 15x15; any pooling window of up to 64
 * results; also, for its split across workgroups, 1x1 layers of 512 or more channels per group and few
 * tiles and - with a workspace - 3x3 launches of fewer than 128 tile-workgroups with 64-160 channels per
 * group), "rows" (everything else).  A zero ratio in the descriptor's flags (SCONV_ZERO_RATIO) moves
 * the choice among "quad3x3", "wide3x3" and "tap3x3" for launches that fill the matrix kernels' tiles
 * (see sconv_density).  The environment variable SCONV_VARIANT ("rows", "tap",
 * "quad", "wide", "gen" or unset) pins the choice for profiling; a plan remembered by sconv_tune comes
 * before the static rules.
 * Returns NULL for an invalid descriptor.  Nothing is enqueued, but the call asks the HIP runtime for
 * the current device (to see whether a workspace is lent there), which initialises the runtime.
 */
const char* sconv_variant_name(const sconv_desc_t* desc, int pooled);

/*
 * Run-time choice of the kernel.  Which variant and decomposition is fastest depends on the zero
 * ratio of the map (Section 8's sparsity sweep: the vector kernel's time falls with the ratio, the
 * matrix kernels' only once whole groups are zero), which the host does not know.  sconv_tune runs
 * every variant and every decomposition that covers the descriptor on the caller's operands - a first
 * pass of one untimed and one timed launch each (two more for a candidate within a quarter of the
 * fastest so far) between two events on hip_stream with the operands left in the caches, then the static
 * choice and the four fastest again for about a millisecond each - and remembers the fastest (the static
 * choice unless another measures 3 % and 1.5 us faster) for this exact descriptor (and pooled flag) in a
 * host-side table; later sconv_forward / sconv_pool_forward calls with an identical descriptor launch that plan instead of the cost
 * models' choice.  The table is per process, guarded by the library's lock, and holds no device
 * memory.
 *   pooled != 0: tune sconv_pool_forward (y_dev is [N][K][PH][PW]), else sconv_forward.
 *   x_dev, w_dev device, in; y_dev device, out: overwritten many times, left holding the result.
 *   flush_dev device, scratch, optional (NULL with flush_bytes 0): when given, its flush_bytes
 *            bytes are overwritten before every timed launch of the five finalists, so that none
 *            finds its operands in the caches (give it at least twice the last-level cache, 512 MiB);
 *            without it plans are ranked cache-warm only.  With it, the finalists are timed both
 *            ways and a plan replaces the static choice only if it wins both.  This buffer is
 *            the caller's and only used during this call.  Split plans are tried only when a
 *            workspace is lent for hip_stream (sconv_set_workspace) - lend it first.
 *   best_ms host, out, optional: average launch duration of the chosen plan in milliseconds.
 * Unlike every other call this one SYNCHRONISES with hip_stream (it reads event times), so it
 * must not be called while the stream is being captured into a graph; call it once at set-up.
 * SCONV_VARIANT, when set, overrides the table.  Errors as sconv_forward.
 */
int sconv_tune(const sconv_desc_t* desc, int pooled, const float* x_dev, const float* w_dev,
               float* y_dev, void* flush_dev, size_t flush_bytes, void* hip_stream, float* best_ms);

/*
 * Density probe (the cheap alternative to sconv_tune).  The zero ratio of a feature map decides
 * which kernel is fastest (Section 8.3 plots the method's time against it; the first layers of a network
 * are far less sparse than the deep ones, Section 8.2), and the host cannot see it.
 *   sconv_density: enqueues two small kernels on hip_stream that count, with the test of Algorithm 1's
 *            scan (x != 0), the elements of x examined and those that are nonzero:
 *            counts_dev[0] = examined, counts_dev[1] = nonzero (device, 2 x 64-bit, 8-byte aligned,
 *            overwritten).  Every element is examined when the map has at most 4 Mi of them, else 4 Mi
 *            in runs of 256 spread evenly over the tensor.  Does not synchronise; the caller reads the
 *            counts after the stream has run (zero ratio = 1 - nonzero / examined).  A producer that knows
 *            its output's zero ratio some other way needs no probe.
 *   The hint itself is stateless: the caller puts the ratio into the descriptor of the forward (or
 *            tuning) call, flags |= SCONV_ZERO_RATIO(z).  With it, 3x3 / stride 1 / pad 1 launches that
 *            fill the matrix kernels' tiles take, below 68 % zeros, the matrix kernel whose tiles fit
 *            the map ("quad3x3" on maps wider than 16 whose width fills its 28-column tiles, "wide3x3"
 *            up to 60 % on the others) or else the vector kernel, the vector kernel ("tap3x3") from
 *            68 %, and "quad3x3" again from 92 % (crossovers of the zero-ratio sweeps on independent
 *            zeros and of 80 random shapes with each variant pinned); plans found by sconv_tune
 *            are kept per density class (no hint; below 55 %; 55-80 %; above), so two layers of one
 *            shape with different densities each get their own.  Without the hint the rules assume what
 *            the paper reports for deep layers (more than 70 % zeros, Fig. 2).
 */
int sconv_density(const sconv_desc_t* desc, const float* x_dev, unsigned long long* counts_dev, void* hip_stream);

/* Forgets every tuned plan.  Host only. */
int sconv_tune_reset(void);

/*
 * The plan table as text, so that a deployment tunes once (sconv_tune costs 0.02-0.3 s a layer) and later
 * processes load the result instead of measuring again.  Plans are tied to the descriptor (batch size
 * included), the density class of its zero-ratio field and whether the call brings prepared filters - not to
 * pointers - and a plan that does not apply where it is loaded (no workspace for a split plan, say) falls back
 * to the static rules at the call, as a tuned plan always does.  Host only.
 *   sconv_tune_export: writes one line per remembered plan into out (NUL-terminated).  needed (optional)
 *            receives the bytes required, terminator included; out NULL with out_size 0 asks for the size
 *            only.  SCONV_EINVAL when out_size is too small (nothing written).
 *   sconv_tune_import: adds the plans of such a text to the table, replacing entries with the same key.
 *            SCONV_EINVAL for a line it cannot read or a plan no kernel knows (nothing is imported then).
 */
int sconv_tune_export(char* out, size_t out_size, size_t* needed);
int sconv_tune_import(const char* text);

/*
 * Writes the plan the forward calls would launch for this descriptor into out (NUL-terminated,
 * truncated to out_size): "variant/geometry/WxS" (wavefronts per workgroup x channel slices;
 * geometry "-": the variant has one; "dense" and names ending in d: the form without zero tests), or
 * "variant/geometry/WxSxP" when P workgroups split a tile's channels, for a tuned descriptor
 * ("variant/model/kept" when tuning found nothing 3 % faster than the static choice, "tap3x3/model:geometry/WxS[xP]/kept"
 * for the vector kernel, whose static plan has a name);
 * "variant/model" for a descriptor that was not tuned ("tap3x3/model:geometry/WxS[xP]": the vector
 * kernel's cost model is asked what it would launch on the default stream, so a split shows).  Nothing is enqueued; asks the HIP runtime
 * for the current device, as sconv_variant_name does.
 */
int sconv_plan_name(const sconv_desc_t* desc, int pooled, char* out, int out_size);

/*
 * The SCONV_* environment variables (tuning aids for profiles and tests: SCONV_VARIANT,
 * SCONV_{TAP,QUAD,WIDE,GEN,PW}_GEOM, SCONV_{TAP,QUAD,WIDE,GEN,PW}_SPLIT, SCONV_ENCODE,
 * SCONV_TRACE_PLAN) are read once, by the first call that needs one, and kept; no launch calls
 * getenv.  sconv_env_refresh reads them again (a test that changes the environment calls it).  It must
 * not run while another thread is inside a launching call.  Host only.
 */
int sconv_env_refresh(void);

/* Static description of an error code. */
const char* sconv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SCONV_H */
