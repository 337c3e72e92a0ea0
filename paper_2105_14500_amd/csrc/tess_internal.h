// Internal declarations shared by the host dispatcher and the HIP kernels of the
// Tesseract per-processor linear library.  Not part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tesseract.h"

namespace tess {

constexpr int BK_HOST = 64;   // K extent of one LDS stage of the MFMA path

// One launch computes  OUT[M,N] = epilogue( sum_{t<q} Aop_t * Bop_t ), where the
// contraction length per panel is Kp and the operands of step t are the t-th
// panels.  An operand is "K-contiguous" (KC) when the contracted index is the
// fastest one in memory and "MN-contiguous" (MC) otherwise:
//   forward (Alg. 3)   A = A_{i,t,k} [M,Kp]  KC      B = B_{t,j}   [Kp,N]  MC
//   dX (C = A B^T)     A = dY_{i,t,k} [M,Kp] KC      B = W_{j,t}   [N,Kp]  KC
//   dW (C = A^T B)     A = X_{t,i,k} [Kp,M]  MC      B = dY_{t,j,k} [Kp,N] MC
struct GemmArgs {
    const void* a[TESS_MAX_Q];
    const void* b[TESS_MAX_Q];
    int32_t q;
    int32_t M, N, Kp;
    int64_t lda, ldb;       // elements
    void* out;              // [M,N], ldo
    void* preact;           // optional second output (pre-activation)
    const void* bias;       // [N] or null, input dtype
    int64_t ldo;
    int32_t act;            // tess_act
    int32_t out_f32;        // 1: out / preact are fp32, 0: bf16
    int32_t accumulate;     // 1: out (fp32) += result
    int32_t a_kc, b_kc;     // operand orientation
    int32_t in_f32;         // 1: inputs fp32, 0: bf16
    // optional: multiply the result by dact'(zin[row, col]) before the store (zin in the
    // input dtype, leading dimension ldz)
    const void* zin;
    int64_t ldz;
    int32_t dact;           // tess_act whose derivative is applied
    // optional: column sums of the B operand over the whole contraction, [N] fp32,
    // overwritten or added to according to `accumulate`
    float* colsum;
    // split of the K loop over gridDim.z; partials go to ws in the accumulator layout,
    // followed by splits x N partial column sums
    int32_t splits;
    float* ws;
    unsigned long long* stamps;      // diagnostic builds only (TESS_STAMPS): 16 time stamps per workgroup
};

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Position of block
// `bid` in an order that lists XCD 0's blocks first, then XCD 1's, ...: blocks that run on
// one XCD get a contiguous run of indices.  A bijection on [0, n).
__host__ __device__ inline int xcd_major_index(int bid, int n)
{
    const int per = n >> 3, rem = n & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// Index in the tile order -> output tile.  The order walks bands of GM tile rows column by
// column, so that a run of `conc` consecutive indices (the tiles one XCD has in flight) is a
// compact patch that shares row and column panels in that XCD's L2.  GM is the band height
// (1..8) that needs the fewest panels, GM + conc / GM, preferring heights that divide the
// grid: 8 x 4 for 32 tiles (12 panels), 4 x 2 for 8 (6 panels where an 8 x 1 strip needs 9).
// A bijection from [0, tiles_m*tiles_n) onto the tile grid for every grid size.
__host__ __device__ inline void tile_of_index(int lid, int tiles_m, int tiles_n, int conc, int& tm, int& tn)
{
    int GM = 1, best = 1 << 30;
    for (int gm = 1; gm <= 8 && gm <= tiles_m; ++gm) {
        // panels x gm, so that the comparison stays in integers; ragged bands cost one more
        const int cost = gm * gm + conc + (tiles_m % gm ? gm : 0);
        if (cost * GM <= best * gm) { best = cost; GM = gm; }   // cost/gm <= best/GM, ties -> taller
    }
    const int band = lid / (GM * tiles_n);
    const int first = band * GM;
    const int rows = tiles_m - first < GM ? tiles_m - first : GM;
    const int in_band = lid - band * GM * tiles_n;
    tm = first + in_band % rows;
    tn = in_band / rows;
}

// Block -> output tile of a launch with one workgroup per tile: the block ids that land on
// one XCD are relabelled to a contiguous run of tile indices (at most 32 of them in flight).
__host__ __device__ inline void tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int nb = tiles_m * tiles_n;
    const int per = nb >> 3;
    const int conc = per >= 32 ? 32 : (per >= 1 ? per : 1);   // tiles of one XCD in flight
    tile_of_index(xcd_major_index(bid, nb), tiles_m, tiles_n, conc, tm, tn);
}

// Kernel families.
enum class Path : int32_t { Generic = 0, Mfma = 1 };

struct Plan {
    Path path;
    int32_t bm, bn;     // macro tile of the MFMA path
    int32_t splits;     // K splits (1 = none): equal parts over gridDim.z + reduction kernel
    int32_t direct;     // 1: global->LDS direct loads (needs Kp % 64 == 0)
    size_t ws_bytes;
};

// Enqueue; returns hipSuccess or the launch error.
hipError_t launch_generic(const GemmArgs& g, hipStream_t s);
hipError_t launch_mfma(const GemmArgs& g, const Plan& p, hipStream_t s);
hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, int real_data, hipStream_t s);
hipError_t launch_row_sums(const void* x, int64_t m, int64_t w, int64_t ldx, int in_f32,
                           int accumulate, float* out, hipStream_t s);
hipError_t launch_row_sums_bwd(const void* xhat, const void* g, int64_t m, int64_t w, int64_t ldx,
                               int64_t ldg, int in_f32, int accumulate, float* out, hipStream_t s);
hipError_t launch_layernorm_bwd(const void* xhat, const void* g, int64_t m, int64_t w, int64_t ldx,
                                int64_t ldg, int in_f32, const float* sums_bwd, const float* sums_fwd,
                                float inv_n, float eps, void* out, int64_t ldo, hipStream_t s);
hipError_t launch_normalize(const void* x, int64_t m, int64_t w, int64_t ldx, int in_f32,
                            const float* sums, float inv_n, float eps, void* out, int64_t ldo,
                            hipStream_t s);

}  // namespace tess
