// bf16 convolution for few input channels (the 7x7/2, C=3 stem) on the gfx950 matrix cores.
//
// With C=3 the reduction run that is contiguous in memory is one window row: S*C elements (21 for 7x7x3).  A workgroup
// stages the input patch of a 16x16 output tile in LDS once, and every lane builds its matrix-core operand straight
// from that patch: the reduction is cut into 8-element chunks (ceil(S*C/8) per window row, zero weights where a chunk
// overhangs the row), and one v_mfma_f32_32x32x16_bf16 consumes two chunks (lanes 0-31 one, lanes 32-63 the next).
// The filters are repacked into the same chunk order in LDS once per workgroup, which then loops over many tiles.
// Epilogue in fp32: + bias, activation, one round-to-nearest-even to bf16.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace coe {
namespace k {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kTile = 16;     // output tile is kTile x kTile pixels = 256 GEMM rows, 64 per wavefront

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
    if (act == 2) return 0.5f * v * erfcf(-v * 0.70710678118654752440f);
    return v;
}

struct StemGeom {
    int tiles_p, tiles_q, total_tiles;
    int patch_rows, patch_cols;   // patch_cols = elements of one patch row that are loaded ((tile-1)*stride+S)*C
    int patch_stride;             // elements per LDS patch row (even, covers the furthest chunk read)
    int cpr;                      // 8-element chunks per window row
    int ksteps;                   // matrix-core steps = ceil(R*cpr / 2)
    int wstride;                  // elements per LDS filter row
};

template <int NB>
__global__ __launch_bounds__(kThreads) void conv_smallc_bf16_kernel(const uint16_t* __restrict__ x,
                                                                     const uint16_t* __restrict__ w,
                                                                     const float* __restrict__ bias,
                                                                     uint16_t* __restrict__ y, ConvShape s, StemGeom g)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* wpack = smem;                               // [32*NB][wstride]
    uint16_t* patch = smem + 32 * NB * g.wstride;         // [patch_rows][patch_stride]
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int SC = s.S * s.C;

    // filters into chunk order; zero where a chunk overhangs its window row or the step count is padded
    for (int idx = tid; idx < 32 * NB * g.ksteps * 16; idx += kThreads) {
        int kk = idx / (g.ksteps * 16), e = idx % (g.ksteps * 16);
        int chunk = e >> 3, i = e & 7;
        int r = chunk / g.cpr, sc = (chunk % g.cpr) * 8 + i;
        uint16_t v = 0;
        if (r < s.R && sc < SC) v = w[((size_t)kk * s.R + r) * SC + sc];
        wpack[kk * g.wstride + e] = v;
    }
    for (int idx = tid; idx < g.patch_rows * g.patch_stride; idx += kThreads) patch[idx] = 0;
    __syncthreads();

    const int half = lane >> 5, l32 = lane & 31;
    for (int tile = blockIdx.x; tile < g.total_tiles; tile += gridDim.x) {
        const int n = tile / (g.tiles_p * g.tiles_q);
        const int tp = (tile / g.tiles_q) % g.tiles_p, tq = tile % g.tiles_q;
        const int p0 = tp * kTile, q0 = tq * kTile;
        const int ih_base = p0 * s.stride - s.pad;
        const int g_base = (q0 * s.stride - s.pad) * s.C;         // element offset inside an input row, may be negative
        const int WC = s.W * s.C;
        for (int idx = tid; idx < g.patch_rows * g.patch_cols; idx += kThreads) {
            int pr = idx / g.patch_cols, ce = idx % g.patch_cols;
            int ih = ih_base + pr, ge = g_base + ce;
            uint16_t v = 0;
            if ((unsigned)ih < (unsigned)s.H && ge >= 0 && ge < WC) v = x[((size_t)n * s.H + ih) * WC + ge];
            patch[pr * g.patch_stride + ce] = v;
        }
        __syncthreads();

        f32x16 acc[2][NB];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        int a_off[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int ml = wid * 64 + i * 32 + l32;
            a_off[i] = (ml / kTile) * s.stride * g.patch_stride + (ml % kTile) * s.stride * s.C;
        }
        for (int j = 0; j < g.ksteps; ++j) {
            int chunk = 2 * j + half;
            int r = chunk / g.cpr, part = chunk % g.cpr;
            if (r >= s.R) { r = s.R - 1; }                         // padded step: filters are zero, any finite data will do
            const int koff = r * g.patch_stride + part * 8;
            bf16x8 af[2], bfr[NB];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t* p32 = (const uint32_t*)(patch + a_off[i] + koff);      // 4-byte aligned by construction
                uint4 v = make_uint4(p32[0], p32[1], p32[2], p32[3]);
                af[i] = __builtin_bit_cast(bf16x8, v);
            }
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
                bfr[jn] = *(const bf16x8*)(wpack + (jn * 32 + l32) * g.wstride + chunk * 8);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jn = 0; jn < NB; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[jn], acc[i][jn], 0, 0, 0);
        }

        // accumulator element v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the 32x32 block
#pragma unroll
        for (int jn = 0; jn < NB; ++jn) {
            const int col = jn * 32 + l32;
            const float bv = bias[col];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int ml = wid * 64 + i * 32 + 8 * (v >> 2) + half * 4 + (v & 3);
                    int p = p0 + ml / kTile, q = q0 + ml % kTile;
                    if (p < s.P && q < s.Q)
                        y[(((size_t)n * s.P + p) * s.Q + q) * s.K + col] = f32_to_bf16(act_fn(acc[i][jn][v] + bv, s.act));
                }
        }
        __syncthreads();      // the patch is rewritten by the next tile
    }
}

bool geometry(const ConvShape& s, StemGeom& g, size_t& smem)
{
    if (s.K != 32 && s.K != 64) return false;
    if (s.C <= 0 || s.C % 32 == 0) return false;
    if ((s.stride * s.C) % 2) return false;                        // chunk reads must stay 4-byte aligned
    int SC = s.S * s.C;
    g.cpr = (SC + 7) / 8;
    g.ksteps = (s.R * g.cpr + 1) / 2;
    g.wstride = g.ksteps * 16 + 8;
    g.patch_rows = (kTile - 1) * s.stride + s.R;
    g.patch_cols = ((kTile - 1) * s.stride + s.S) * s.C;
    int furthest = (kTile - 1) * s.stride * s.C + g.cpr * 8;       // one past the last element any chunk read touches
    int ps = g.patch_cols > furthest ? g.patch_cols : furthest;
    g.patch_stride = (ps + 1) / 2 * 2 + 2;
    g.tiles_p = (s.P + kTile - 1) / kTile;
    g.tiles_q = (s.Q + kTile - 1) / kTile;
    long long total = (long long)s.N * g.tiles_p * g.tiles_q;
    if (total > 0x7FFFFFFFll) return false;
    g.total_tiles = (int)total;
    smem = sizeof(uint16_t) * ((size_t)s.K * g.wstride + (size_t)g.patch_rows * g.patch_stride);
    return smem <= 64 * 1024;
}

}  // namespace

bool conv_smallc_supported(const ConvShape& s, bool has_res)
{
    StemGeom g;
    size_t smem;
    return !has_res && geometry(s, g, smem);
}

hipError_t conv_smallc(const void* x, const void* w, const float* bias, void* y, const ConvShape& s, hipStream_t stream)
{
    StemGeom g;
    size_t smem = 0;
    if (!geometry(s, g, smem)) return hipErrorInvalidValue;
    if (g.total_tiles == 0) return hipSuccess;
    int grid = g.total_tiles < 1024 ? g.total_tiles : 1024;
    if (s.K == 64)
        hipLaunchKernelGGL(conv_smallc_bf16_kernel<2>, dim3(grid), dim3(kThreads), smem, stream, (const uint16_t*)x,
                           (const uint16_t*)w, bias, (uint16_t*)y, s, g);
    else
        hipLaunchKernelGGL(conv_smallc_bf16_kernel<1>, dim3(grid), dim3(kThreads), smem, stream, (const uint16_t*)x,
                           (const uint16_t*)w, bias, (uint16_t*)y, s, g);
    return hipGetLastError();
}

}  // namespace k
}  // namespace coe
