// Pieces shared by the matrix-core kernels that work on tiles of 64 window rows (sconv_wide.hip,
// sconv_gen.hip): the launch configuration, the four guarded 16x16x1 matrix instructions of one
// tap, and the reduction / epilogue of a tile.
#pragma once

#include "sconv_internal.h"

namespace sconv {
namespace wide {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct WideCfg {
    int NT, NCS;        // wavefronts per workgroup = NT row tiles x NCS channel slices
    int CPW;            // channels per wavefront per chunk = CCH / NCS
    int ntiles;         // tiles of 64 window rows
    int npos;           // window rows: N*OH*OW, or N*PH*PW*4 in PECR order
    int vec4;           // plain epilogue may store four rows with one 16-byte store
};

// One tap of one channel: xv holds the 64 rows' elements, m their nonzero mask, wt the lane's
// filter values.  Four blocks of 16 rows, each guarded by one scalar test (DENSE: no tests, for maps
// with so few zeros that hardly a 16-row block is empty).
template <int KPL, bool DENSE = false>
__device__ __forceinline__ void tap_blocks(const float xv, const unsigned long long m,
                                           const float (&wt)[KPL], v16f (&acc)[KPL][4])
{
    unsigned lo = (unsigned)m, hi = (unsigned)(m >> 32);
    asm volatile("" : "+s"(lo), "+s"(hi));   // keep the four tests 32-bit scalar compares
    if (DENSE || (lo & 0xFFFFu)) {
#pragma unroll
        for (int i = 0; i < KPL; ++i)
            acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x1f32(xv, wt[i], acc[i][0], 2, 0, 0);
    }
    if (DENSE || (lo & 0xFFFF0000u)) {
#pragma unroll
        for (int i = 0; i < KPL; ++i)
            acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x1f32(xv, wt[i], acc[i][1], 2, 1, 0);
    }
    if (DENSE || (hi & 0xFFFFu)) {
#pragma unroll
        for (int i = 0; i < KPL; ++i)
            acc[i][2] = __builtin_amdgcn_mfma_f32_16x16x1f32(xv, wt[i], acc[i][2], 2, 2, 0);
    }
    if (DENSE || (hi & 0xFFFF0000u)) {
#pragma unroll
        for (int i = 0; i < KPL; ++i)
            acc[i][3] = __builtin_amdgcn_mfma_f32_16x16x1f32(xv, wt[i], acc[i][3], 2, 3, 0);
    }
}

// Reduction of the channel slices and epilogue of one 64-row tile, shared by the kernels of this
// file.  acc[i][q][v]: filter register i, 16-row block q, element v (filter 16*(v/4) + lane%16, row
// 4*(lane/16) + v%4 of the block).
// Reduction of the channel slices (NCS is 1, 2 or 4).  The four 16-row blocks of the tile are dealt
// out to the slices: a slice writes the partial sums of the blocks it does not own to LDS, then
// adds what the others wrote for its own blocks (block q belongs to slice q / (4 / NCS)).
template <int KPL>
__device__ __forceinline__ void reduce_slices(const WideCfg& cfg, float* lds, v16f (&acc)[KPL][4], int lane,
                                              int ts, int cs)
{
    const int bps = 4 / cfg.NCS;                   // blocks per slice
    if (cfg.NCS > 1) {
        float* red = lds;  // [NT][4 blocks][NCS - 1 writers][KPL * 16][64]
        __syncthreads();   // every wavefront is done with the filter buffers
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int owner = q / bps;
            if (cs == owner) continue;
            const int slot = cs - (cs > owner ? 1 : 0);
            float* dst = red + (size_t)(((ts * 4 + q) * (cfg.NCS - 1) + slot) * (KPL * 16)) * 64 + lane;
#pragma unroll
            for (int i = 0; i < KPL; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[(i * 16 + v) * 64] = acc[i][q][v];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (cs != q / bps) continue;
            for (int slot = 0; slot < cfg.NCS - 1; ++slot) {
                const float* src = red + (size_t)(((ts * 4 + q) * (cfg.NCS - 1) + slot) * (KPL * 16)) * 64 + lane;
#pragma unroll
                for (int i = 0; i < KPL; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][q][v] += src[(i * 16 + v) * 64];
            }
        }
    }
}

template <int KPL, bool POOL>
__device__ __forceinline__ void finish_tile(const Problem& p, const WideCfg& cfg, float* lds,
                                            v16f (&acc)[KPL][4], int lane, int ts, int cs, int tile,
                                            bool tile_ok, int g, int kb0, int kvalid, int plane,
                                            float* __restrict__ y)
{
    reduce_slices<KPL>(cfg, lds, acc, lane, ts, cs);
    const int bps = 4 / cfg.NCS;                   // blocks per slice
    if (!tile_ok) return;

    // epilogue: element (q, 4*b + e) of the lane = filter 16*b + lane%16, window row
    // 64*tile + 16*q + 4*(lane/16) + e
    const int kf = lane & 15, rg = lane >> 4;
    if (p.bias) {   // (a branch of its own: without a bias the epilogue is exactly the plain one)
#pragma unroll
        for (int i = 0; i < KPL; ++i)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int k = 64 * i + 16 * b + kf;
                const float bk = k < kvalid ? p.bias[(size_t)g * p.Kg + kb0 + k] : 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][q][4 * b + e] += bk;
            }
    }
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = 64 * i + 16 * b + kf;
            if (k >= kvalid) continue;
            const size_t kglob = (size_t)g * p.Kg + kb0 + k;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int P0 = tile * 64 + 16 * q + 4 * rg;
                if (cs != q / bps || P0 >= cfg.npos) continue;
                float v0 = acc[i][q][4 * b], v1 = acc[i][q][4 * b + 1], v2 = acc[i][q][4 * b + 2],
                      v3 = acc[i][q][4 * b + 3];
                if (POOL) {
                    // four rows of one pooling window: ReLU, maximum, one pooled result
                    const int pp = P0 >> 2;
                    const int nn = pp / plane;
                    const float mx = fmaxf(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)), 0.0f);
                    y[((size_t)nn * p.K + kglob) * plane + (pp - nn * plane)] = mx;
                } else {
                    if (p.relu) {
                        v0 = fmaxf(v0, 0.0f); v1 = fmaxf(v1, 0.0f); v2 = fmaxf(v2, 0.0f); v3 = fmaxf(v3, 0.0f);
                    }
                    if (cfg.vec4) {
                        // plane % 4 == 0: the four rows lie in one image, 16-byte aligned
                        const int nn = P0 / plane;
                        float* dst = y + ((size_t)nn * p.K + kglob) * plane + (P0 - nn * plane);
                        *reinterpret_cast<v4f*>(dst) = v4f{v0, v1, v2, v3};
                    } else {
                        const float vs[4] = {v0, v1, v2, v3};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int Pe = P0 + e;
                            if (Pe < cfg.npos) {
                                const int nn = Pe / plane;
                                y[((size_t)nn * p.K + kglob) * plane + (Pe - nn * plane)] = vs[e];
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace wide
}  // namespace sconv
