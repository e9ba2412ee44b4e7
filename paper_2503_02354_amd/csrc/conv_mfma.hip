// bf16 implicit-GEMM convolution on the gfx950 matrix cores.
//
// GEMM view: out[m][k] = sum_{r,s,c} x[n][p*stride-pad+r][q*stride-pad+s][c] * w[k][r][s][c], m = (n,p,q) flattened.
// NHWC activations and [K][R][S][C] weights make the reduction index contiguous in c for both operands, so a
// reduction step is one (r,s) position and a run of 32 channels: 64 bytes per output pixel and per filter.
// A workgroup (4 wavefronts of 64) owns a BM x BN output tile; every step stages a BM x 32 activation slab and a
// BN x 32 weight slab in LDS (two stages, global loads of step i+1 in flight while step i runs on the matrix
// cores), and each wavefront feeds v_mfma_f32_32x32x16_bf16 from LDS with 16-byte reads.
// Epilogue in fp32: + bias (+ residual), activation, one round-to-nearest-even to bf16.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace coe {
namespace k {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBK = 32;              // reduction elements per step
constexpr int kLdsStride = 40;       // elements per LDS row: 64 data bytes + 16 pad bytes -> conflict-free 16-byte reads
constexpr int kXcds = 8;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float act_fn(float v, int act)
{
    if (act == 1) return v > 0.f ? v : 0.f;
    if (act == 2) return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f));
    return v;
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(kThreads) void conv_igemm_bf16_kernel(const uint16_t* __restrict__ x,
                                                                    const uint16_t* __restrict__ w,
                                                                    const float* __restrict__ bias,
                                                                    const uint16_t* __restrict__ res,
                                                                    uint16_t* __restrict__ y, ConvShape s, int M,
                                                                    int tiles_n)
{
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int MB = WM / 32, NB = WN / 32;
    static_assert(MB >= 1 && NB >= 1, "wave tile");
    constexpr int A_CHUNKS = BM * 4, B_CHUNKS = BN * 4;          // 16-byte chunks per slab
    constexpr int A_LOADS = (A_CHUNKS + kThreads - 1) / kThreads;
    constexpr int B_LOADS = (B_CHUNKS + kThreads - 1) / kThreads;
    constexpr int STAGE = (BM + BN) * kLdsStride;                // elements

    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * STAGE];

    // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give each XCD a contiguous range
    // of tiles (filter tiles fastest) and the slabs shared by neighbouring tiles stay in one XCD's L2.
    int tile;
    {
        int L = blockIdx.x, total = gridDim.x;
        int xcd = L % kXcds, slot = L / kXcds;
        int base = total / kXcds, rem = total % kXcds;
        tile = xcd * base + (xcd < rem ? xcd : rem) + slot;
    }
    const int tile_n = tile % tiles_n, tile_m = tile / tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int wm = wid / WAVES_N, wn = wid % WAVES_N;
    const int chunk = tid & 3;               // which 16-byte piece of the 64-byte run
    const int row0 = tid >> 2;               // 0..63

    // per-thread description of the activation rows it fetches
    const int PQ = s.P * s.Q;
    int a_ih0[A_LOADS], a_iw0[A_LOADS];
    size_t a_base[A_LOADS];
    bool a_ok[A_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        int row = row0 + 64 * j;
        int m = m0 + row;
        a_ok[j] = (row < BM) && (m < M);
        int mm = a_ok[j] ? m : 0;
        int n = mm / PQ, pq = mm % PQ;
        int p = pq / s.Q, q = pq % s.Q;
        a_ih0[j] = p * s.stride - s.pad;
        a_iw0[j] = q * s.stride - s.pad;
        a_base[j] = (size_t)n * s.H * s.W * s.C;
    }
    const size_t w_row = (size_t)s.R * s.S * s.C;   // elements per filter

    const int cblocks = s.C / kBK;
    const int nsteps = s.R * s.S * cblocks;

    uint4 a_reg[A_LOADS], b_reg[B_LOADS];
    int r = 0, t = 0, cb = 0;                       // position of the step being fetched

    auto fetch = [&]() {
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            int ih = a_ih0[j] + r, iw = a_iw0[j] + t;
            bool ok = a_ok[j] && (unsigned)ih < (unsigned)s.H && (unsigned)iw < (unsigned)s.W;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (ok) v = *(const uint4*)(x + a_base[j] + ((size_t)ih * s.W + iw) * s.C + cb * kBK + chunk * 8);
            a_reg[j] = v;
        }
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) {
            int row = row0 + 64 * j;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < BN) v = *(const uint4*)(w + (size_t)(n0 + row) * w_row + ((size_t)r * s.S + t) * s.C + cb * kBK + chunk * 8);
            b_reg[j] = v;
        }
        if (++cb == cblocks) { cb = 0; if (++t == s.S) { t = 0; ++r; } }
    };
    auto stash = [&](int stage) {
        uint16_t* a_lds = lds + stage * STAGE;
        uint16_t* b_lds = a_lds + BM * kLdsStride;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            int row = row0 + 64 * j;
            if (row < BM) *(uint4*)(a_lds + row * kLdsStride + chunk * 8) = a_reg[j];
        }
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) {
            int row = row0 + 64 * j;
            if (row < BN) *(uint4*)(b_lds + row * kLdsStride + chunk * 8) = b_reg[j];
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    fetch();
    stash(0);
    __syncthreads();

    const int frag_row = lane & 31;          // row (A) / filter (B) inside a 32-wide block
    const int frag_k = (lane >> 5) * 8;      // which 8 of the 16 reduction elements this lane supplies

    for (int step = 0; step < nsteps; ++step) {
        const bool more = step + 1 < nsteps;
        if (more) fetch();
        const uint16_t* a_lds = lds + (step & 1) * STAGE;
        const uint16_t* b_lds = a_lds + BM * kLdsStride;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 af[MB], bfr[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i)
                af[i] = *(const bf16x8*)(a_lds + (wm * WM + i * 32 + frag_row) * kLdsStride + ks * 16 + frag_k);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                bfr[j] = *(const bf16x8*)(b_lds + (wn * WN + j * 32 + frag_row) * kLdsStride + ks * 16 + frag_k);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) stash((step + 1) & 1);
        __syncthreads();
    }

    // epilogue.  Accumulator element v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the 32x32 block.
    const int col_in = lane & 31, row_hi = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int col = n0 + wn * WN + j * 32 + col_in;
        const float bv = bias[col];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = wm * WM + i * 32 + 8 * (v >> 2) + row_hi + (v & 3);
                int m = m0 + row;
                if (m < M) {
                    size_t o = (size_t)m * s.K + col;
                    float val = acc[i][j][v] + bv;
                    if (res) val += bf16_to_f32(res[o]);
                    y[o] = f32_to_bf16(act_fn(val, s.act));
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch(const void* x, const void* w, const float* bias, const void* res, void* y, const ConvShape& s,
                  hipStream_t stream)
{
    long long M = (long long)s.N * s.P * s.Q;
    if (M <= 0) return hipSuccess;
    if (M > 0x7FFFFFFFll - BM) return hipErrorInvalidValue;
    int tiles_m = (int)((M + BM - 1) / BM), tiles_n = s.K / BN;
    long long total = (long long)tiles_m * tiles_n;
    if (total > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_igemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N>), dim3((unsigned)total), dim3(kThreads), 0, stream,
                       (const uint16_t*)x, (const uint16_t*)w, bias, (const uint16_t*)res, (uint16_t*)y, s, (int)M, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_supported(const ConvShape& s) { return s.C % kBK == 0 && s.K % 32 == 0 && s.C > 0 && s.K > 0; }

hipError_t conv_mfma(const void* x, const void* w, const float* bias, const void* res, void* y, const ConvShape& s,
                     hipStream_t stream)
{
    if (!conv_mfma_supported(s)) return hipErrorInvalidValue;
    if (s.K % 128 == 0) return launch<128, 128, 2, 2>(x, w, bias, res, y, s, stream);
    if (s.K % 64 == 0) return launch<256, 64, 4, 1>(x, w, bias, res, y, s, stream);
    return launch<256, 32, 4, 1>(x, w, bias, res, y, s, stream);
}

}  // namespace k
}  // namespace coe
