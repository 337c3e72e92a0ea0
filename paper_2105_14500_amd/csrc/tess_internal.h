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
    // split of the K loop over gridDim.z; partials go to ws in the accumulator layout
    int32_t splits;
    float* ws;
};

// Kernel families.
enum class Path : int32_t { Generic = 0, Mfma = 1 };

struct Plan {
    Path path;
    int32_t bm, bn;     // macro tile of the MFMA path
    int32_t bk;         // K extent of one LDS stage (64, or 32 with a deeper ring)
    int32_t waves;      // wavefronts per workgroup of the 256 x 256 tile (8 or 4)
    int32_t splits;     // K splits (1 = none)
    int32_t direct;     // 1: global->LDS direct loads (needs Kp % 64 == 0)
    size_t ws_bytes;
};

// Chooses kernel family, tile and split for a launch; pure host arithmetic.
Plan make_plan(const GemmArgs& g);

// Enqueue; returns hipSuccess or the launch error.
hipError_t launch_generic(const GemmArgs& g, hipStream_t s);
hipError_t launch_mfma(const GemmArgs& g, const Plan& p, hipStream_t s);
hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, hipStream_t s);

}  // namespace tess
