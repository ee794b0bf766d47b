// Issue-rate microbenchmarks for gfx950: how long a SIMD takes for the instruction patterns the
// zero-skipping kernels are built from - vector multiply-adds with a scalar operand, scalar tests,
// conditional branches taken and not taken, computed jumps, lane broadcasts - at 1 to 8 resident
// wavefronts per SIMD.  A library of its own (libsconv_micro.so); nothing in libsconv uses it.
//
// Every kernel runs `iters` rounds of one inline-assembly block that repeats its pattern 64 times;
// the host divides the event time by iters * 64.  One workgroup is 256 threads (one wavefront per
// SIMD of a compute unit); `blocks` workgroups are launched, so blocks / 256 wavefronts share a SIMD.
#include <hip/hip_runtime.h>
#include <stdint.h>

extern "C" {
enum {
    MICRO_FMA = 0,            // 8 independent v_fmac with a scalar operand per repeat (8 instructions)
    MICRO_SALU_DEP = 1,       // 8 dependent s_add_u32 per repeat
    MICRO_TEST_NOT_TAKEN = 2, // s_bitcmp1 + s_cbranch (not taken) per repeat
    MICRO_TEST_TAKEN = 3,     // s_bitcmp1 + s_cbranch taken to the next instruction
    MICRO_SKIP5_NOT_TAKEN = 4,// test + branch not taken over 5 v_fmac (they run)
    MICRO_SKIP5_TAKEN = 5,    // test + branch taken over 5 v_fmac (they are skipped)
    MICRO_SETPC = 6,          // s_getpc + s_add + s_addc + s_setpc to the next instruction
    MICRO_READLANE_FMA5 = 7,  // v_readlane + s_nop 1 + 5 v_fmac reading the broadcast value
    MICRO_FAR_TAKEN = 8,      // branch out of line (about 3 KB away), 5 v_fmac there, branch back
    MICRO_FF1_SETPC = 9,      // s_ff1 + s_bitset0 + s_lshl + s_add + s_addc + s_setpc (threaded dispatch)
    MICRO_MFMA_4X4X1 = 10,    // 8 independent v_mfma_f32_4x4x1 (16 blocks, 256 multiply-adds each) per repeat
    MICRO_MFMA_16X16X1 = 11,  // 4 independent v_mfma_f32_16x16x1 (4 blocks, 1024 multiply-adds each) per repeat
    MICRO_VSKIP5_ON = 12,     // s_setvskip (skip mode on) + 5 v_fmac, which are then not issued
    MICRO_VSKIP5_OFF = 13,    // s_setvskip (skip mode off) + 5 v_fmac, which run
    MICRO_VSKIP_POS_ON = 14,  // s_setvskip on + v_readlane + 5 v_fmac: a zero position of the vector kernel, no branch
    MICRO_VSKIP_POS_OFF = 15, // the same with skip mode off: a nonzero position
    MICRO_MODES = 16
};
}

namespace {

typedef float mv4f __attribute__((ext_vector_type(4)));
typedef float mv16f __attribute__((ext_vector_type(16)));

// Matrix-pipe issue rate: independent accumulators, operands that change with the lane (not zeros).
template <int MODE>
__global__ __launch_bounds__(256) void micro_mfma_kernel(int iters, float* out)
{
    const float a = 1.0f + threadIdx.x * 0.001f, b = 0.5f + threadIdx.x * 0.002f;
    float r = 0.0f;
    if constexpr (MODE == MICRO_MFMA_4X4X1) {
        mv4f acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = mv4f{0.f, 0.f, 0.f, 0.f};
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int rep = 0; rep < 64; ++rep)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) r += acc[j][0] + acc[j][3];
    } else {
        mv16f acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
        for (int i = 0; i < iters; ++i)
#pragma unroll
            for (int rep = 0; rep < 64; ++rep)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, acc[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) r += acc[j][0] + acc[j][15];
    }
    if (out) out[blockIdx.x * 256 + threadIdx.x] = r;
}

// Streaming read: every thread sums 16-byte loads, `unroll` of them in flight, over a buffer of `n16` 16-byte
// words; one result per thread so that nothing is optimised away.
__global__ __launch_bounds__(256) void micro_read_kernel(const mv4f* __restrict__ src, long long n16, float* out)
{
    const long long stride = (long long)gridDim.x * 256;
    mv4f s0 = {0, 0, 0, 0}, s1 = s0, s2 = s0, s3 = s0;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const mv4f a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        s0 += a; s1 += b; s2 += c; s3 += d;
    }
    for (; i < n16; i += stride) s0 += src[i];
    const mv4f s = s0 + s1 + s2 + s3;
    out[blockIdx.x * 256 + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

template <int MODE>
__global__ __launch_bounds__(256) void micro_kernel(int iters, unsigned m, float* out)
{
    float a0 = threadIdx.x, a1 = 1.f, a2 = 2.f, a3 = 3.f, a4 = 4.f, a5 = 5.f, a6 = 6.f, a7 = 7.f;
    const float w = out ? 1.0009765625f : 0.f;
    unsigned t = m;
    for (int i = 0; i < iters; ++i) {
        if constexpr (MODE == MICRO_FMA) {
            asm volatile(".rept 64\n"
                         "v_fmac_f32 %0, %8, %9\n v_fmac_f32 %1, %8, %9\n v_fmac_f32 %2, %8, %9\n v_fmac_f32 %3, %8, %9\n"
                         "v_fmac_f32 %4, %8, %9\n v_fmac_f32 %5, %8, %9\n v_fmac_f32 %6, %8, %9\n v_fmac_f32 %7, %8, %9\n"
                         ".endr\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "s"(m), "v"(w));
        } else if constexpr (MODE == MICRO_SALU_DEP) {
            asm volatile(".rept 64\n"
                         "s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n"
                         "s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n s_add_u32 %0, %0, 1\n"
                         ".endr\n"
                         : "+s"(t) : : "scc");
        } else if constexpr (MODE == MICRO_TEST_NOT_TAKEN || MODE == MICRO_TEST_TAKEN) {
            asm volatile(".rept 64\n"
                         "s_bitcmp1_b32 %0, 0\n s_cbranch_scc1 1f\n 1:\n"
                         ".endr\n"
                         : : "s"(m) : "scc");
        } else if constexpr (MODE == MICRO_SKIP5_NOT_TAKEN || MODE == MICRO_SKIP5_TAKEN) {
            asm volatile(".rept 64\n"
                         "s_bitcmp1_b32 %5, 0\n s_cbranch_scc1 1f\n"
                         "v_fmac_f32 %0, %5, %6\n v_fmac_f32 %1, %5, %6\n v_fmac_f32 %2, %5, %6\n v_fmac_f32 %3, %5, %6\n"
                         "v_fmac_f32 %4, %5, %6\n 1:\n"
                         ".endr\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4)
                         : "s"(m), "v"(w) : "scc");
        } else if constexpr (MODE == MICRO_SETPC) {
            // s_getpc returns the address of the instruction after it; the three that follow are 4 bytes each
            asm volatile(".rept 64\n"
                         "s_getpc_b64 s[40:41]\n s_add_u32 s40, s40, 12\n s_addc_u32 s41, s41, 0\n s_setpc_b64 s[40:41]\n"
                         ".endr\n"
                         : : : "s40", "s41", "scc");
        } else if constexpr (MODE == MICRO_READLANE_FMA5) {
            asm volatile(".rept 64\n"
                         "v_readlane_b32 s40, %5, 7\n s_nop 1\n"
                         "v_fmac_f32 %0, s40, %5\n v_fmac_f32 %1, s40, %5\n v_fmac_f32 %2, s40, %5\n v_fmac_f32 %3, s40, %5\n"
                         "v_fmac_f32 %4, s40, %5\n"
                         ".endr\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4)
                         : "v"(w) : "s40");
        } else if constexpr (MODE == MICRO_FAR_TAKEN) {
            // 64 branches in line; their blocks follow the in-line code (each 5 v_fmac + a branch back)
#define MICRO_FAR_BR(i) "s_cbranch_scc1 1" #i "f\n 2" #i ":\n"
#define MICRO_FAR_BLK(i)                                                                                   \
    "1" #i ":\n v_fmac_f32 %0, %5, %6\n v_fmac_f32 %1, %5, %6\n v_fmac_f32 %2, %5, %6\n v_fmac_f32 %3, %5, %6\n" \
    "v_fmac_f32 %4, %5, %6\n s_branch 2" #i "b\n"
#define MICRO_R8(m, a) m(a##0) m(a##1) m(a##2) m(a##3) m(a##4) m(a##5) m(a##6) m(a##7)
#define MICRO_R64(m) MICRO_R8(m, 0) MICRO_R8(m, 1) MICRO_R8(m, 2) MICRO_R8(m, 3) MICRO_R8(m, 4) MICRO_R8(m, 5) \
    MICRO_R8(m, 6) MICRO_R8(m, 7)
            asm volatile("s_bitcmp1_b32 %5, 0\n"
                         MICRO_R64(MICRO_FAR_BR)
                         "s_branch 3f\n"
                         MICRO_R64(MICRO_FAR_BLK)
                         "3:\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4)
                         : "s"(m), "v"(w) : "scc");
        } else if constexpr (MODE == MICRO_VSKIP5_ON || MODE == MICRO_VSKIP5_OFF) {
            // s_setvskip S0, S1: the wavefront's vector-skip mode := bit S1 of S0.  While it is set, vector ALU,
            // vector memory and LDS instructions are not issued.  Cleared again before the block ends.
            asm volatile(".rept 64\n"
                         "s_setvskip %5, 0\n"
                         "v_fmac_f32 %0, %5, %6\n v_fmac_f32 %1, %5, %6\n v_fmac_f32 %2, %5, %6\n v_fmac_f32 %3, %5, %6\n"
                         "v_fmac_f32 %4, %5, %6\n"
                         ".endr\n"
                         "s_setvskip 0, 0\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4)
                         : "s"(m), "v"(w));
        } else if constexpr (MODE == MICRO_VSKIP_POS_ON || MODE == MICRO_VSKIP_POS_OFF) {
            asm volatile(".rept 64\n"
                         "s_setvskip %5, 0\n"
                         "v_readlane_b32 s40, %6, 7\n s_nop 1\n"
                         "v_fmac_f32 %0, s40, %6\n v_fmac_f32 %1, s40, %6\n v_fmac_f32 %2, s40, %6\n v_fmac_f32 %3, s40, %6\n"
                         "v_fmac_f32 %4, s40, %6\n"
                         ".endr\n"
                         "s_setvskip 0, 0\n"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4)
                         : "s"(m), "v"(w) : "s40");
        } else if constexpr (MODE == MICRO_FF1_SETPC) {
            // the dispatch sequence of a threaded position loop; the target is the next instruction
            asm volatile("s_mov_b64 s[42:43], -1\n"
                         ".rept 64\n"
                         "s_ff1_i32_b64 s44, s[42:43]\n s_bitset0_b64 s[42:43], s44\n s_lshl_b32 s44, s44, 0\n"
                         "s_getpc_b64 s[40:41]\n s_add_u32 s40, s40, 12\n s_addc_u32 s41, s41, 0\n s_setpc_b64 s[40:41]\n"
                         ".endr\n"
                         : : : "s40", "s41", "s42", "s43", "s44", "scc");
        }
    }
    if (out) out[blockIdx.x * 256 + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + (float)t;
}

template <int MODE>
int launch(int iters, unsigned m, int blocks, float* out, hipStream_t s)
{
    hipLaunchKernelGGL(micro_kernel<MODE>, dim3(blocks), dim3(256), 0, s, iters, m, out);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // namespace

// Enqueues one microbenchmark kernel: `blocks` workgroups of 256 threads, `iters` rounds of 64 repeats.
// out_dev: device, blocks * 256 floats (written once at the end, so that nothing is optimised away).
// Returns 0, -1 (bad argument) or -3 (launch failed).
extern "C" int sconv_micro_launch(int mode, int iters, int blocks, float* out_dev, void* hip_stream)
{
    if (iters <= 0 || blocks <= 0 || !out_dev) return -1;
    hipStream_t s = (hipStream_t)hip_stream;
    switch (mode) {
    case MICRO_FMA: return launch<MICRO_FMA>(iters, 0x3f800000u, blocks, out_dev, s);
    case MICRO_SALU_DEP: return launch<MICRO_SALU_DEP>(iters, 0, blocks, out_dev, s);
    case MICRO_TEST_NOT_TAKEN: return launch<MICRO_TEST_NOT_TAKEN>(iters, 0, blocks, out_dev, s);
    case MICRO_TEST_TAKEN: return launch<MICRO_TEST_TAKEN>(iters, 1, blocks, out_dev, s);
    case MICRO_SKIP5_NOT_TAKEN: return launch<MICRO_SKIP5_NOT_TAKEN>(iters, 0x3f800000u, blocks, out_dev, s);
    case MICRO_SKIP5_TAKEN: return launch<MICRO_SKIP5_TAKEN>(iters, 0x3f800001u, blocks, out_dev, s);
    case MICRO_SETPC: return launch<MICRO_SETPC>(iters, 0, blocks, out_dev, s);
    case MICRO_READLANE_FMA5: return launch<MICRO_READLANE_FMA5>(iters, 0, blocks, out_dev, s);
    case MICRO_FAR_TAKEN: return launch<MICRO_FAR_TAKEN>(iters, 1, blocks, out_dev, s);
    case MICRO_FF1_SETPC: return launch<MICRO_FF1_SETPC>(iters, 0, blocks, out_dev, s);
    case MICRO_VSKIP5_ON: return launch<MICRO_VSKIP5_ON>(iters, 0x3f800001u, blocks, out_dev, s);
    case MICRO_VSKIP5_OFF: return launch<MICRO_VSKIP5_OFF>(iters, 0x3f800000u, blocks, out_dev, s);
    case MICRO_VSKIP_POS_ON: return launch<MICRO_VSKIP_POS_ON>(iters, 1, blocks, out_dev, s);
    case MICRO_VSKIP_POS_OFF: return launch<MICRO_VSKIP_POS_OFF>(iters, 0, blocks, out_dev, s);
    case MICRO_MFMA_4X4X1:
        hipLaunchKernelGGL(micro_mfma_kernel<MICRO_MFMA_4X4X1>, dim3(blocks), dim3(256), 0, s, iters, out_dev);
        return hipGetLastError() == hipSuccess ? 0 : -3;
    case MICRO_MFMA_16X16X1:
        hipLaunchKernelGGL(micro_mfma_kernel<MICRO_MFMA_16X16X1>, dim3(blocks), dim3(256), 0, s, iters, out_dev);
        return hipGetLastError() == hipSuccess ? 0 : -3;
    default: return -1;
    }
}

// Enqueues a streaming read of `bytes` bytes (a multiple of 16) at src_dev by `blocks` workgroups of 256
// threads; out_dev: blocks * 256 floats.  Returns 0, -1 or -3.
extern "C" int sconv_micro_read(const float* src_dev, size_t bytes, int blocks, float* out_dev, void* hip_stream)
{
    if (!src_dev || !out_dev || blocks <= 0 || bytes < 16 || bytes % 16) return -1;
    hipLaunchKernelGGL(micro_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       reinterpret_cast<const mv4f*>(src_dev), (long long)(bytes / 16), out_dev);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}
