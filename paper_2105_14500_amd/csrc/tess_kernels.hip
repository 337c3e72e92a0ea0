// HIP kernels (gfx950 / CDNA4) for the per-processor compute of a Tesseract
// [q,q,d]-partitioned linear layer: the q-step block accumulation of Alg. 3 and
// its two transposed variants (Section 3.1), with the bias/activation epilogue.
//
// Two kernel families:
//   * tess_mfma_kernel   bf16 inputs, v_mfma_f32_32x32x16_bf16, fp32 accumulators
//     that stay in registers over all q steps; operand tiles go through LDS.
//   * tess_generic_kernel  any shape / alignment / fp32 inputs, fp32 FMA.
#include "tess_internal.h"

#include <type_traits>

namespace tess {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLB_PTR(T) __attribute__((address_space(1))) T*

constexpr int NTHREADS = 256;   // 4 wavefronts, arranged 2 x 2 over the macro tile

// ---------------------------------------------------------------------------
// epilogue helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_erf_f(float x)
{
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_tanh_f(float x)
{
    const float c = 0.79788456080286535588f;
    return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float apply_act(float z, int act)
{
    if (act == TESS_ACT_GELU_ERF) return gelu_erf_f(z);
    if (act == TESS_ACT_GELU_TANH) return gelu_tanh_f(z);
    return z;
}
// fp32 -> bf16 bits, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b)
{
    return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ float load_in(const void* p, int64_t idx, int in_f32)
{
    return in_f32 ? ((const float*)p)[idx] : bf16_bits_to_f32(((const uint16_t*)p)[idx]);
}

// value `acc` of output element (row, col): bias, optional pre-activation copy,
// activation, accumulate, down-cast, store.
__device__ __forceinline__ void store_out(const GemmArgs& g, int row, int col, float acc,
                                          float bias_v)
{
    float z = acc + bias_v;
    const int64_t o = (int64_t)row * g.ldo + col;
    if (g.preact) {
        if (g.out_f32) ((float*)g.preact)[o] = z;
        else ((uint16_t*)g.preact)[o] = f32_to_bf16_bits(z);
    }
    float y = apply_act(z, g.act);
    if (g.out_f32) {
        float* op = (float*)g.out + o;
        *op = g.accumulate ? (*op + y) : y;
    } else {
        ((uint16_t*)g.out)[o] = f32_to_bf16_bits(y);
    }
}

// ---------------------------------------------------------------------------
// generic kernel: 64 x 64 output tile per 256 threads, 4 x 4 outputs per thread,
// any shape, strides and alignment; inputs fp32 or bf16; fp32 FMA, contracted
// index ascending within a panel and panels in ascending step order.
// ---------------------------------------------------------------------------
constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // K step

__global__ __launch_bounds__(256) void tess_generic_kernel(GemmArgs g)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int row0 = blockIdx.y * GT, col0 = blockIdx.x * GT;
    // element (row, kk) of the A operand: a_kc ? [row*lda + kk] : [kk*lda + row]
    const int64_t a_rs = g.a_kc ? g.lda : 1, a_ks = g.a_kc ? 1 : g.lda;
    // element (kk, col) of the B operand: b_kc ? [col*ldb + kk] : [kk*ldb + col]
    const int64_t b_cs = g.b_kc ? g.ldb : 1, b_ks = g.b_kc ? 1 : g.ldb;
    float acc[4][4] = {};
    for (int t = 0; t < g.q; ++t) {
        const void* Ap = g.a[t];
        const void* Bp = g.b[t];
        for (int k0 = 0; k0 < g.Kp; k0 += GK) {
            for (int e = tid; e < GK * GT; e += 256) {
                int kk, rr;
                if (g.a_kc) { kk = e % GK; rr = e / GK; } else { rr = e % GT; kk = e / GT; }
                const int row = row0 + rr, kidx = k0 + kk;
                As[kk][rr] = (row < g.M && kidx < g.Kp)
                                 ? load_in(Ap, row * a_rs + kidx * a_ks, g.in_f32) : 0.0f;
                int kb, cc;
                if (g.b_kc) { kb = e % GK; cc = e / GK; } else { cc = e % GT; kb = e / GT; }
                const int col = col0 + cc, kidb = k0 + kb;
                Bs[kb][cc] = (col < g.N && kidb < g.Kp)
                                 ? load_in(Bp, kidb * b_ks + col * b_cs, g.in_f32) : 0.0f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < GK; ++kk) {
                float av[4], bv[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) { av[x] = As[kk][ty * 4 + x]; bv[x] = Bs[kk][tx * 4 + x]; }
#pragma unroll
                for (int x = 0; x < 4; ++x)
#pragma unroll
                    for (int y = 0; y < 4; ++y) acc[x][y] = fmaf(av[x], bv[y], acc[x][y]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int row = row0 + ty * 4 + x;
        if (row >= g.M) continue;
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const int col = col0 + tx * 4 + y;
            if (col >= g.N) continue;
            const float bv = g.bias ? load_in(g.bias, col, g.in_f32) : 0.0f;
            store_out(g, row, col, acc[x][y], bv);
        }
    }
}

hipError_t launch_generic(const GemmArgs& g, hipStream_t s)
{
    dim3 grid((g.N + GT - 1) / GT, (g.M + GT - 1) / GT, 1);
    hipLaunchKernelGGL(tess_generic_kernel, grid, dim3(256), 0, s, g);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// MFMA path
// ---------------------------------------------------------------------------
// LDS tile formats, in 16-byte granules (8 bf16), for a stage of BK contracted
// elements (CH = BK/8 granules along k):
//  KC operand, R rows x BK k:  granule (r, pc) at index r*CH + pc holds k-chunk
//      c = pc ^ swz_kc(r) of row r.  A 32x32x16 fragment read (lane -> row l%32,
//      chunk 2*kk + l/32, one 128-bit read) then touches every bank once per
//      16 consecutive rows.
//  MC operand, BK k-rows x R elements: granule (kr, pg) at index kr*(R/8) + pg
//      holds elements 8g..8g+7, g = pg ^ swz_mc(kr), of k-row kr.  Fragments are
//      read with the transposing 64-bit LDS read, which hands lane s of a 16-lane
//      group the 4 k-values of column s from 4 k-rows.
// Tiles are always written linearly (granule index = it*256 + thread), so the
// swizzle is applied on the global-memory side of the copy.
template <int BK>
__device__ __forceinline__ int swz_kc(int r)
{
    constexpr int CH = BK / 8, RPL = 128 / BK;   // chunks per row, rows per 256-byte bank line
    return (r / RPL) % CH;
}
__device__ __forceinline__ int swz_mc(int kr) { return ((kr & 3) << 2) ^ (((kr >> 3) & 1) << 1); }

// Compile-time loop: the body sees the index as an integral constant, so every
// accumulator index is static and the accumulators stay in registers.
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that orders LDS traffic only: global loads into LDS that are
// still in flight for later stages are not waited for.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wavefront
// fills bytes [16*l, 16*l+16) behind the wave-uniform LDS address `lds_dst` (M0).
// Written as inline assembly on purpose: the compiler then does not track these
// loads, so it inserts no "wait for every outstanding load" before LDS reads of
// other ring slots; completion is enforced by the explicit vmcnt waits in front of
// the workgroup barriers instead.
__device__ __forceinline__ void lds_dma16(const char* src, char* lds_dst)
{
    const uint32_t m0 = (uint32_t)(uintptr_t)(LDS_PTR(char))lds_dst;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(m0)
                 : "memory", "m0");
}

template <int R, int BK, bool KC, bool DIRECT>
struct TileLoader {
    static constexpr int CH = BK / 8;            // granules per row (KC)
    static constexpr int NG = R * CH;            // granules per stage
    static constexpr int ITERS = NG / NTHREADS;
    static constexpr int RG = R / 8;             // granules per k-row (MC)
    uint32_t off[ITERS];    // byte offset of this thread's granule inside a panel at k0 = 0
    uint32_t kpos[DIRECT ? 1 : ITERS];   // k index (within the stage) that the granule starts at
    u32x4 stage[DIRECT ? 1 : ITERS];

    // origin: first row (KC) / first element along R (MC) of this block's tile;
    // extent: total rows / elements of the operand along R; ld in elements.
    __device__ __forceinline__ void init(int tid, int origin, int extent, int64_t ld)
    {
        static_for<ITERS>([&](auto it) {
            const int G = it * NTHREADS + tid;
            if (KC) {
                const int r = G / CH, pc = G % CH;
                const int c = pc ^ swz_kc<BK>(r);
                int row = origin + r;
                row = row < extent ? row : extent - 1;
                off[it] = (uint32_t)(((int64_t)row * ld + 8 * c) * 2);
                if (!DIRECT) kpos[it] = 8 * c;
            } else {
                const int kr = G / RG, pg = G % RG;
                const int gidx = pg ^ swz_mc(kr);
                int col = origin + 8 * gidx;
                col = col + 8 <= extent ? col : extent - 8;
                off[it] = (uint32_t)(((int64_t)kr * ld + col) * 2);
                if (!DIRECT) kpos[it] = kr;
            }
        });
    }

    // base: panel pointer advanced to the stage's first k (uniform); krem: number of
    // valid k from there (only used by the staged variant, for the zero-filled tail).
    // wave_u: wavefront index as a wave-uniform value (the LDS address of a direct
    // load is a scalar: base of the 64 granules that the wavefront's lanes fill).
    template <typename IT>
    __device__ __forceinline__ void issue_one(const char* base, char* lds_tile, int wave_u, int tid,
                                              int krem, IT it)
    {
        if (DIRECT) {
            const int wave_first = (it * NTHREADS + wave_u * 64) * 16;
            lds_dma16(base + off[it], lds_tile + wave_first);
        } else {
            u32x4 v = {0u, 0u, 0u, 0u};
            if ((int)kpos[it] < krem) v = *(const u32x4*)(base + off[it]);
            stage[it] = v;
        }
    }
    __device__ __forceinline__ void issue(const char* base, char* lds_tile, int wave_u, int tid,
                                          int krem)
    {
        static_for<ITERS>([&](auto it) { issue_one(base, lds_tile, wave_u, tid, krem, it); });
    }
    __device__ __forceinline__ void commit(char* lds_tile, int tid)
    {
        if (!DIRECT) {
            static_for<ITERS>([&](auto it) {
                *(u32x4*)(lds_tile + (it * NTHREADS + tid) * 16) = stage[it];
            });
        }
    }
};

// Fragment reader: 32 (rows along R) x 16 (k) bf16 operand fragment for
// v_mfma_f32_32x32x16_bf16: lane l gets row l%32, k = 8*(l/32) .. +7.
template <int R, int BK, bool KC>
struct FragReader {
    static constexpr int KSTEPS = BK / 16;
    uint32_t lane_off;          // per-lane byte offset, fragment 0
    uint32_t kcol[KC ? KSTEPS : 2];   // KC: byte offset of the k-chunk for each k16 step
    __device__ __forceinline__ void init(int lane, int wave_origin)
    {
        if (KC) {
            const int r = wave_origin + (lane & 31);
            lane_off = (uint32_t)r * (uint32_t)(BK * 2);
            static_for<KSTEPS>([&](auto kk) {
                kcol[kk] = (uint32_t)(((2 * kk + (lane >> 5)) ^ swz_kc<BK>(r)) * 16);
            });
        } else {
            const int s = lane & 15, bl = lane >> 4;
            const int kr = 8 * (bl >> 1) + (s >> 2);           // k-row inside a k16 step, first read
            lane_off = (uint32_t)(kr * (R / 8) * 16 + (s & 1) * 8);
            kcol[0] = (uint32_t)swz_mc(kr);
            kcol[1] = (uint32_t)(wave_origin + 16 * (bl & 1) + 4 * (s & 3)) >> 3;  // granule, frag 0
        }
    }
    // f: fragment index along R inside the wave tile, kk: k16 step of the stage
    __device__ __forceinline__ bf16x8 read(const char* lds_tile, int f, int kk) const
    {
        if (KC) {
            return *(const bf16x8*)(lds_tile + lane_off + f * (32 * BK * 2) + kcol[kk]);
        } else {
            const uint32_t gsw = ((kcol[1] + 4u * f) ^ kcol[0]) * 16u;
            const char* p = lds_tile + lane_off + gsw + kk * (16 * (R / 8) * 16);
            bf16x4 lo = __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                                       (LDS_PTR(short4v))(p)));
            bf16x4 hi = __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                                       (LDS_PTR(short4v))(p + 4 * (R / 8) * 16)));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
};

// Stores one 32x32 accumulator fragment.  Accumulator layout: lane l, register r ->
//   row = 8*(r/4) + 4*(l/32) + r%4,  col = l%32.
// frow0: first row of the fragment + 4*(l/32); col: this lane's column.
__device__ __forceinline__ void store_fragment(const GemmArgs& g, const floatx16& v, int frow0,
                                               int col, float bias_v)
{
    if (col >= g.N) return;
    float z[16];
    static_for<16>([&](auto r) { z[r] = v[r()] + bias_v; });
    if (g.preact) {
        static_for<16>([&](auto r) {
            const int row = frow0 + 8 * (r / 4) + (r % 4);
            if (row < g.M) {
                const int64_t o = (int64_t)row * g.ldo + col;
                if (g.out_f32) ((float*)g.preact)[o] = z[r];
                else ((uint16_t*)g.preact)[o] = f32_to_bf16_bits(z[r]);
            }
        });
    }
    if (g.act == TESS_ACT_GELU_ERF) static_for<16>([&](auto r) { z[r] = gelu_erf_f(z[r]); });
    else if (g.act == TESS_ACT_GELU_TANH) static_for<16>([&](auto r) { z[r] = gelu_tanh_f(z[r]); });
    if (g.out_f32) {
        float* out = (float*)g.out;
        if (g.accumulate) {
            static_for<16>([&](auto r) {
                const int row = frow0 + 8 * (r / 4) + (r % 4);
                if (row < g.M) out[(int64_t)row * g.ldo + col] += z[r];
            });
        } else {
            static_for<16>([&](auto r) {
                const int row = frow0 + 8 * (r / 4) + (r % 4);
                if (row < g.M) out[(int64_t)row * g.ldo + col] = z[r];
            });
        }
    } else {
        uint16_t* out = (uint16_t*)g.out;
        static_for<16>([&](auto r) {
            const int row = frow0 + 8 * (r / 4) + (r % 4);
            if (row < g.M) out[(int64_t)row * g.ldo + col] = f32_to_bf16_bits(z[r]);
        });
    }
}

// Block -> output tile.  Workgroups are dealt round-robin to the 8 XCDs, each with
// its own L2: relabel so that one XCD gets a contiguous run of tile ids, and walk the
// tiles in bands of 8 tile-rows so that a run shares A and B panels.
__device__ __forceinline__ void block_to_tile(int bid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int nb = tiles_m * tiles_n;
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    const int lid = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    constexpr int GM = 8;
    const int band = lid / (GM * tiles_n);
    const int first = band * GM;
    const int rows = tiles_m - first < GM ? tiles_m - first : GM;
    const int in_band = lid - band * GM * tiles_n;
    tm = first + in_band % rows;
    tn = in_band / rows;
}


template <int BM, int BN, int BK, int NSTAGE, bool A_KC, bool B_KC, bool DIRECT>
__global__ __launch_bounds__(NTHREADS) void tess_mfma_kernel(GemmArgs g)
{
    constexpr int FM = BM / 64, FN = BN / 64;          // fragments per wave tile
    constexpr int KSTEPS = BK / 16;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static_assert(DIRECT || NSTAGE == 2, "the register-staged loader is double-buffered");
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int nb = tiles_m * tiles_n;
    int tm, tn;
    block_to_tile(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int row0 = tm * BM, col0 = tn * BN;

    // ---- K range of this block (split over gridDim.z in whole stages)
    const int kt_per_panel = (g.Kp + BK - 1) / BK;
    const int kt_total = g.q * kt_per_panel;
    int kt_begin = 0, kt_end = kt_total;
    if (g.splits > 1) {
        const int z = blockIdx.z;
        const int base = kt_total / g.splits, extra = kt_total % g.splits;
        kt_begin = z * base + (z < extra ? z : extra);
        kt_end = kt_begin + base + (z < extra ? 1 : 0);
    }
    const int nkt = kt_end - kt_begin;

    typedef TileLoader<BM, BK, A_KC, DIRECT> LA;
    typedef TileLoader<BN, BK, B_KC, DIRECT> LB;
    constexpr int LOADS = LA::ITERS + LB::ITERS;       // global loads per thread per stage
    LA la;
    LB lb;
    la.init(tid, row0, g.M, g.lda);
    lb.init(tid, col0, g.N, g.ldb);
    FragReader<BM, BK, A_KC> ra;
    FragReader<BN, BK, B_KC> rb;
    ra.init(lane, wm * (BM / 2));
    rb.init(lane, wn * (BN / 2));

    floatx16 acc[FM * FN];
    static_for<FM * FN>([&](auto f) {
        static_for<16>([&](auto r) { acc[f][r()] = 0.0f; });
    });

    // byte advance of one stage along K for each operand
    const int64_t a_kstep = A_KC ? (int64_t)BK * 2 : (int64_t)BK * g.lda * 2;
    const int64_t b_kstep = B_KC ? (int64_t)BK * 2 : (int64_t)BK * g.ldb * 2;

    // Panel pointers are fetched from the kernel-argument segment (constant address
    // space, scalar loads) with the uniform step index; indexing the by-value copy
    // of the argument struct dynamically would move it to scratch memory.
    typedef __attribute__((address_space(4))) const GemmArgs* KernArgs;
    const KernArgs ka = (KernArgs)__builtin_amdgcn_kernarg_segment_ptr();
    // (panel, stage-in-panel) of the next stage to fetch and its operand pointers,
    // advanced incrementally; the pointers are re-read only when the panel changes
    int ld_t = kt_begin / kt_per_panel, ld_ks = kt_begin - ld_t * kt_per_panel;
    const char* ld_ap = (const char*)ka->a[ld_t < g.q ? ld_t : 0] + ld_ks * a_kstep;
    const char* ld_bp = (const char*)ka->b[ld_t < g.q ? ld_t : 0] + ld_ks * b_kstep;
    auto issue = [&](int stage) {
        char* sa = lds + stage * STAGE_BYTES;
        const int krem = g.Kp - ld_ks * BK;
        la.issue(ld_ap, sa, wave_u, tid, krem);
        lb.issue(ld_bp, sa + A_BYTES, wave_u, tid, krem);
    };
    auto advance = [&]() {
        ld_ap += a_kstep;
        ld_bp += b_kstep;
        if (++ld_ks == kt_per_panel) {
            ld_ks = 0;
            ++ld_t;
            const int t = ld_t < g.q ? ld_t : g.q - 1;
            ld_ap = (const char*)ka->a[t];
            ld_bp = (const char*)ka->b[t];
        }
    };

    bf16x8 af[2][FM], bfr[2][FN];
    // Fragment u of a k16 step: the FN fragments of B first, then the FM of A (the
    // first MFMAs of a step need af[0] and every bfr[j]).
    auto load_frag = [&](auto buf, int stage, auto kk, auto u) {
        const char* sa = lds + stage * STAGE_BYTES;
        if constexpr (u < FN) bfr[buf][u] = rb.read(sa + A_BYTES, u, kk);
        else af[buf][u - FN] = ra.read(sa, u - FN, kk);
    };
    auto load_frags = [&](auto buf, int stage, auto kk) {
        static_for<FM + FN>([&](auto u) { load_frag(buf, stage, kk, u); });
    };
    // One k16 step written out in issue order: MFMA x is followed by the side work
    // side(x) (LDS reads of the next step, requests for a later tile), and a
    // scheduling fence keeps the compiler from regrouping them, so the matrix pipe
    // is fed while the reads and requests are in flight.
    auto mfma_step = [&](auto buf, auto&& side) {
        static_for<FM * FN>([&](auto x) {
            constexpr int i = x / FN, j = x % FN;
            acc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[x], 0, 0, 0);
            side(x);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // all k16 steps of a stage except the last: fetch the next step's fragments with
    // the first MFMAs of the current one
    auto body_steps = [&](int stage) {
        static_for<KSTEPS - 1>([&](auto kk) {
            mfma_step(std::integral_constant<int, kk & 1>{}, [&](auto x) {
                if constexpr (x < FM + FN)
                    load_frag(std::integral_constant<int, (kk + 1) & 1>{}, stage,
                              std::integral_constant<int, kk + 1>{}, x);
            });
        });
    };
    constexpr int LASTBUF = (KSTEPS - 1) & 1;
    static_assert(FM + FN <= FM * FN, "one fragment read per MFMA slot");
    auto no_side = [](auto) {};

    if constexpr (DIRECT) {
        // Ring of NSTAGE LDS slots; tile r lives in slot r % NSTAGE.  All slots are
        // requested up front; tile r+NSTAGE is requested into slot r % NSTAGE as soon
        // as every wave has finished reading tile r, so NSTAGE-1 tiles are in flight
        // or ready while one is being consumed.
        static_for<NSTAGE>([&](auto s) {
            if (s < nkt) { issue(s); advance(); }
        });
        // tile 0 must have landed; the later ones may still be in flight
        if (nkt >= NSTAGE) wait_vmcnt<(NSTAGE - 1) * LOADS>();
        else wait_vmcnt<0>();
        lds_barrier();
        if (nkt > 0) load_frags(std::integral_constant<int, 0>{}, 0, std::integral_constant<int, 0>{});
        int stage = 0;
        int r = 0;
        constexpr int LPS = (LOADS + FM * FN - 1) / (FM * FN);   // requests per MFMA slot
        // steady state: a tile to request at every step
        for (; r + NSTAGE < nkt; ++r) {
            body_steps(stage);
            const int next = stage + 1 == NSTAGE ? 0 : stage + 1;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of this slot are done
            wait_vmcnt<(NSTAGE - 2) * LOADS>();                    // tile r+1 has landed
            lds_barrier();
            // last k16 step of tile r, carrying the first fragments of tile r+1 and
            // the requests for tile r+NSTAGE into the slot that was just freed
            char* sa = lds + stage * STAGE_BYTES;
            const int krem = g.Kp - ld_ks * BK;
            mfma_step(std::integral_constant<int, LASTBUF>{}, [&](auto x) {
                if constexpr (x < FM + FN)
                    load_frag(std::integral_constant<int, (LASTBUF ^ 1)>{}, next,
                              std::integral_constant<int, 0>{}, x);
                static_for<LPS>([&](auto l) {
                    constexpr int it = x * LPS + l;
                    if constexpr (it < LA::ITERS) la.issue_one(ld_ap, sa, wave_u, tid, krem, std::integral_constant<int, it>{});
                    else if constexpr (it < LOADS) lb.issue_one(ld_bp, sa + A_BYTES, wave_u, tid, krem, std::integral_constant<int, it - LA::ITERS>{});
                });
            });
            advance();
            stage = next;
        }
        // drain: nothing left to request
        for (; r < nkt; ++r) {
            body_steps(stage);
            const int next = stage + 1 == NSTAGE ? 0 : stage + 1;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            wait_vmcnt<0>();
            lds_barrier();
            if (r + 1 < nkt)
                load_frags(std::integral_constant<int, (LASTBUF ^ 1)>{}, next, std::integral_constant<int, 0>{});
            mfma_step(std::integral_constant<int, LASTBUF>{}, no_side);
            stage = next;
        }
    } else {
        // register-staged double buffer with a zero-filled K tail
        auto commit = [&](int stage) {
            char* sa = lds + stage * STAGE_BYTES;
            la.commit(sa, tid);
            lb.commit(sa + A_BYTES, tid);
        };
        if (nkt > 0) {
            issue(0);
            advance();
            commit(0);
            __syncthreads();
        }
        for (int r = 0; r < nkt; ++r) {
            const int cur = r & 1;
            const bool more = r + 1 < nkt;
            if (more) { issue(cur ^ 1); advance(); }
            load_frags(std::integral_constant<int, 0>{}, cur, std::integral_constant<int, 0>{});
            body_steps(cur);
            mfma_step(std::integral_constant<int, LASTBUF>{}, no_side);
            if (more) commit(cur ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue
    if (g.splits > 1) {
        // partial sums in accumulator order: [(z*nb + tile)][wave][frag][reg][lane]
        float* w = g.ws + ((size_t)blockIdx.z * nb + (size_t)(tm * tiles_n + tn)) * (BM * BN) +
                   (size_t)wave * (FM * FN * 16 * 64) + lane;
        static_for<FM * FN>([&](auto f) {
            static_for<16>([&](auto r) { w[(f * 16 + r) * 64] = acc[f][r()]; });
        });
        return;
    }
    static_for<FN>([&](auto j) {
        const int col = col0 + wn * (BN / 2) + j * 32 + (lane & 31);
        const float bv = (g.bias && col < g.N) ? bf16_bits_to_f32(((const uint16_t*)g.bias)[col]) : 0.0f;
        static_for<FM>([&](auto i) {
            const int frow0 = row0 + wm * (BM / 2) + i * 32 + 4 * (lane >> 5);
            store_fragment(g, acc[i * FN + j], frow0, col, bv);
        });
    });
}

// Sums the K-split partials in ascending split order and applies the epilogue.
template <int BM, int BN>
__global__ __launch_bounds__(NTHREADS) void tess_splitk_reduce_kernel(GemmArgs g)
{
    constexpr int FM = BM / 64, FN = BN / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_n = (g.N + BN - 1) / BN, tiles_m = (g.M + BM - 1) / BM;
    const int nb = tiles_m * tiles_n;
    const int tile = blockIdx.x;
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int row0 = tm * BM, col0 = tn * BN;
    const float* w0 = g.ws + (size_t)tile * (BM * BN) + (size_t)wave * (FM * FN * 16 * 64) + lane;
    for (int j = 0; j < FN; ++j) {
        const int col = col0 + wn * (BN / 2) + j * 32 + (lane & 31);
        const float bv = (g.bias && col < g.N) ? bf16_bits_to_f32(((const uint16_t*)g.bias)[col]) : 0.0f;
        for (int i = 0; i < FM; ++i) {
#pragma unroll 4
            for (int r = 0; r < 16; ++r) {
                float sum = 0.0f;
                for (int z = 0; z < g.splits; ++z)
                    sum += w0[(size_t)z * nb * (BM * BN) + ((i * FN + j) * 16 + r) * 64];
                const int row = row0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < g.M && col < g.N) store_out(g, row, col, sum, bv);
            }
        }
    }
}

template <int BM, int BN, int BK, int NSTAGE, bool A_KC, bool B_KC, bool DIRECT>
static hipError_t launch_one(const GemmArgs& g, const Plan& p, hipStream_t s)
{
    constexpr int lds_bytes = NSTAGE * (BM + BN) * BK * 2;
    auto kern = tess_mfma_kernel<BM, BN, BK, NSTAGE, A_KC, B_KC, DIRECT>;
    static bool attr_set = false;   // per instantiation; the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    GemmArgs a = g;
    a.splits = p.splits;
    hipLaunchKernelGGL(kern, dim3(tiles, 1, p.splits), dim3(NTHREADS), lds_bytes, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.splits > 1) {
        hipLaunchKernelGGL((tess_splitk_reduce_kernel<BM, BN>), dim3(tiles), dim3(NTHREADS), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

template <int BM, int BN, int BK, int NSTAGE, bool DIRECT>
static hipError_t launch_layout(const GemmArgs& g, const Plan& p, hipStream_t s)
{
    if (g.a_kc && !g.b_kc) return launch_one<BM, BN, BK, NSTAGE, true, false, DIRECT>(g, p, s);
    if (g.a_kc && g.b_kc) return launch_one<BM, BN, BK, NSTAGE, true, true, DIRECT>(g, p, s);
    if (!g.a_kc && !g.b_kc) return launch_one<BM, BN, BK, NSTAGE, false, false, DIRECT>(g, p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_mfma(const GemmArgs& g, const Plan& p, hipStream_t s)
{
    if (p.bm == 256 && p.bn == 256) {
        if (!p.direct) return hipErrorInvalidValue;
        if (p.bk == 32) return launch_layout<256, 256, 32, 4, true>(g, p, s);
        return launch_layout<256, 256, 64, 2, true>(g, p, s);
    }
    if (p.bm == 128 && p.bn == 128) {
        if (!p.direct) return launch_layout<128, 128, 64, 2, false>(g, p, s);
        if (p.bk == 32) return launch_layout<128, 128, 32, 4, true>(g, p, s);
        return launch_layout<128, 128, 64, 4, true>(g, p, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace tess
