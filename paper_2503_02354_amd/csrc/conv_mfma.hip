// bf16 implicit-GEMM convolution on the gfx950 matrix cores.
//
// GEMM view: out[m][k] = sum_{r,s,c} x[n][p*stride-pad+r][q*stride-pad+s][c] * w[k][r][s][c], m = (n,p,q) flattened.
// NHWC activations make the reduction index contiguous in c, so a reduction step is one (r,s) position and a run
// of 32 channels.  A workgroup of four wavefronts owns a BM x BN output tile.  Three kernels, picked by conv_mfma():
//   1. conv3x3_slab_kernel   3x3, stride 1, pad 1, filter count a multiple of 64: the activation rows a tile needs are
//                            DMA'd into LDS once per 32-channel block and serve all nine window positions;
//   2. conv_igemm_dma_kernel any other shape with a filter count that is a multiple of 64: both operands DMA'd
//                            global -> LDS per reduction step;
//   3. conv_igemm_bf16_kernel (below) the rest: operands staged through registers.
// Common to all three:
//   * Filters are repacked once, when an expert is registered, into matrix-core fragment order (pack_filters_mfma),
//     so a filter slab is contiguous in memory and in LDS and an operand read is one linear 1 KiB access.
//   * v_mfma_f32_32x32x16_bf16 is issued with the filter fragment as the first operand, so a lane ends up holding 4
//     consecutive output channels of one pixel per accumulator quad.
//   * Epilogue in fp32: + bias (+ residual), activation, one round-to-nearest-even to bf16 (v_cvt_pk_bf16_f32).
//   * Zero padding of the convolution and rows past the end of a tile come from buffer loads whose out-of-range
//     offsets return zero; which window positions fall inside the image is a per-row bit mask computed once.
// The register-staged kernel:
//   * Loads run kDepth steps ahead: each step's activation slab (BM x BK) and filter slab (BN x BK) travel
//     global -> registers (kDepth register stages) -> LDS (two stages) -> matrix-core operands.  Every step issues
//     the same loads unconditionally, so the wait before a register stage is moved to LDS can leave the younger
//     stages in flight.
//   * A wave64 vector instruction occupies a SIMD for 4 cycles and a step has only 16 matrix-core instructions per
//     wavefront, so per-step address arithmetic is kept to a few instructions per load (the position inside the
//     window is a scalar offset shared by all lanes).
//   * Activation rows are padded by 16 bytes in LDS so the 16-byte operand reads are bank-conflict free.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.h"

namespace coe {
namespace k {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPad = 8;              // elements of padding per LDS activation row (16 bytes)
constexpr int kXcds = 8;
constexpr int kDepth = 3;            // register stages = how many steps ahead the global loads run
constexpr uint32_t kOutOfRange = 0x80000000u;   // buffer offset beyond any tensor: the load returns zeros

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // round to nearest even
}
__device__ __forceinline__ float act_fn(float v, int act)
{
    if (act == 1) return v > 0.f ? v : 0.f;
    if (act == 2) return 0.5f * v * erfcf(-v * 0.70710678118654752440f);
    if (act == 3) return v / (1.f + expf(-v));
    return v;
}
// The activation is a launch parameter, but an epilogue that tests it per element compiles into hundreds of
// branches: dispatch ONCE per wave to a body specialised for the activation.
template <typename F> __device__ __forceinline__ void with_activation(int act, F&& body)
{
    if (act == 1) body(std::integral_constant<int, 1>{});
    else if (act == 2) body(std::integral_constant<int, 2>{});
    else if (act == 3) body(std::integral_constant<int, 3>{});
    else body(std::integral_constant<int, 0>{});
}
// raw buffer descriptor over [p, p + bytes): offsets at or beyond `bytes` read as zero
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void conv_igemm_bf16_kernel(const uint16_t* __restrict__ x,
                                                                    const uint16_t* __restrict__ wp,
                                                                    const float* __restrict__ bias,
                                                                    const uint16_t* __restrict__ res,
                                                                    uint16_t* __restrict__ y, ConvShape s, int M,
                                                                    int tiles_n)
{
    constexpr int kThreads = 64 * WAVES_M * WAVES_N;
    static_assert(kThreads == 256 || kThreads == 512, "four or eight wavefronts per workgroup");
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int MB = WM / 32, NB = WN / 32;
    static_assert(MB >= 1 && NB >= 1, "wave tile");
    constexpr int CH = BK / 8;                       // 16-byte chunks per activation slab row
    constexpr int ROWS_PER_PASS = kThreads / CH;
    constexpr int A_LOADS = BM / ROWS_PER_PASS;
    constexpr int KS = BK / 16;                      // matrix-core steps per slab
    constexpr int A_STRIDE = BK + kPad;
    constexpr int A_STAGE = BM * A_STRIDE;           // elements
    constexpr int B_STAGE = BN * BK;                 // elements, fragment order: [BN/32][KS][64 lanes][8]
    constexpr int B_CHUNKS = B_STAGE / 8;
    constexpr int B_LOADS = (B_CHUNKS + kThreads - 1) / kThreads;
    constexpr int B_PER_BLOCK = KS * 64;             // chunks per 32-filter block and step
    constexpr int STAGE = A_STAGE + B_STAGE;

    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // 2 * STAGE elements

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
    const int chunk = tid % CH;
    const int row0 = tid / CH;

    const int cblocks = s.C / BK;
    const int RS = s.R * s.S;
    const int nsteps = RS * cblocks;
    const int ks16_total = nsteps * KS;               // 16-channel steps per filter

    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(x, (uint32_t)s.N * (uint32_t)(s.H * s.W * s.C) * 2u);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wp, (uint32_t)s.K * (uint32_t)(RS * s.C) * 2u);

    // Per activation row this thread fetches: byte offset of window position (0,0), channel 0 (+ its 16-byte chunk),
    // and a mask with bit r*S+s set when that window position lies inside the image.  Rows past M have mask 0.
    int32_t a_off[A_LOADS];
    uint64_t a_mask[A_LOADS];
    {
        const int PQ = s.P * s.Q;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            int m = m0 + row0 + ROWS_PER_PASS * j;
            bool ok = m < M;
            int mm = ok ? m : 0;
            int n = mm / PQ, pq = mm % PQ;
            int p = pq / s.Q, q = pq % s.Q;
            int ih0 = p * s.stride - s.pad, iw0 = q * s.stride - s.pad;
            a_off[j] = ((n * s.H + ih0) * s.W + iw0) * s.C * 2 + chunk * 16;
            uint64_t mask = 0;
            for (int rr = 0; rr < s.R; ++rr)
                for (int tt = 0; tt < s.S; ++tt)
                    if (ok && (unsigned)(ih0 + rr) < (unsigned)s.H && (unsigned)(iw0 + tt) < (unsigned)s.W)
                        mask |= 1ull << (rr * s.S + tt);
            a_mask[j] = mask;
        }
    }
    // filter slab: chunk c of a step lives at block (c / B_PER_BLOCK), offset (c % B_PER_BLOCK) inside the step's
    // KS fragments of that block; LDS keeps the same linear order
    uint32_t b_off[B_LOADS];
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
        int c = tid + kThreads * j;
        b_off[j] = c < B_CHUNKS
                       ? (uint32_t)((((n0 / 32 + c / B_PER_BLOCK) * ks16_total) * 512 + (c % B_PER_BLOCK) * 8) * 2)
                       : kOutOfRange;
    }

    // One register stage: the loads of one reduction step while they are in flight.
    struct RegStage {
        u32x4 a[A_LOADS];
        u32x4 b[B_LOADS];
    };
    RegStage st0, st1, st2;
    static_assert(kDepth == 3, "three named register stages");
    int r = 0, t = 0, cb = 0, f_step = 0;             // (r, s, channel block) and index of the step being fetched

    auto fetch = [&](RegStage& st) {
        const int rs = r * s.S + t;
        const int32_t win = ((r * s.W + t) * s.C + cb * BK) * 2;      // scalar: same for every lane
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
            uint32_t off = ((a_mask[j] >> rs) & 1ull) ? (uint32_t)(a_off[j] + win) : kOutOfRange;
            st.a[j] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off, 0, 0);
        }
        const uint32_t wstep = (uint32_t)f_step * (KS * 512 * 2);     // scalar
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j) st.b[j] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, b_off[j], wstep, 0);
        // advance; past the last step the fetch position stays put, so a fetch issued beyond the end re-reads the
        // last step (never used) and every step issues the same number of loads
        if (f_step + 1 < nsteps) {
            ++f_step;
            if (++cb == cblocks) { cb = 0; if (++t == s.S) { t = 0; ++r; } }
        }
    };
    uint16_t* const a_dst = lds + row0 * A_STRIDE + chunk * 8;
    uint16_t* const b_dst = lds + A_STAGE + tid * 8;
    auto stash = [&](int stage, const RegStage& st) {
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j)
            *(u32x4*)(a_dst + stage * STAGE + ROWS_PER_PASS * j * A_STRIDE) = st.a[j];
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j)
            if (B_CHUNKS % kThreads == 0 || tid + kThreads * j < B_CHUNKS)
                *(u32x4*)(b_dst + stage * STAGE + kThreads * j * 8) = st.b[j];
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int frag_row = lane & 31;          // pixel row inside a 32-row block
    const int frag_k = (lane >> 5) * 8;      // which 8 of the 16 reduction elements this lane supplies

    // Operand fragments are read one matrix-core step ahead of their use, so the LDS latency of step ks+1 hides behind
    // the matrix-core work of step ks.
    const uint16_t* const a_src = lds + (wm * WM + frag_row) * A_STRIDE + frag_k;
    const uint16_t* const b_src = lds + A_STAGE + (wn * NB) * (KS * 512) + lane * 8;
    auto compute = [&](int stage) {
        const uint16_t* a_lds = a_src + stage * STAGE;
        const uint16_t* b_lds = b_src + stage * STAGE;
        bf16x8 af[2][MB], bfr[2][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i) af[0][i] = *(const bf16x8*)(a_lds + i * 32 * A_STRIDE);
#pragma unroll
        for (int j = 0; j < NB; ++j) bfr[0][j] = *(const bf16x8*)(b_lds + (j * KS) * 512);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) {
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    af[(ks + 1) & 1][i] = *(const bf16x8*)(a_lds + i * 32 * A_STRIDE + (ks + 1) * 16);
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    bfr[(ks + 1) & 1][j] = *(const bf16x8*)(b_lds + (j * KS + ks + 1) * 512);
            }
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
        }
    };

    // prologue: three steps in flight, the first one staged
    fetch(st0);
    fetch(st1);
    fetch(st2);
    stash(0, st0);
    __syncthreads();

    // Step u: the register stage that held step u is free -> refill it with step u + 3; compute step u from LDS
    // stage u & 1; move step u + 1 (loads issued two steps ago) from its register stage to the other LDS stage.
    // Fetch and staging are unconditional (past the end they move data nobody reads): the number of loads in flight
    // at every wait is then a compile-time constant and the wait can leave the younger two stages outstanding.
    auto step = [&](int u, RegStage& refill, const RegStage& next) {
        fetch(refill);
        if (u < nsteps) compute(u & 1);
        stash((u + 1) & 1, next);
        __syncthreads();
    };
    for (int u0 = 0; u0 < nsteps; u0 += kDepth) {
        step(u0, st0, st1);
        step(u0 + 1, st1, st2);
        step(u0 + 2, st2, st0);
    }

    // Epilogue.  With the filter fragment as the first operand, accumulator element v of lane l belongs to pixel l%32
    // and filter 8*(v/4) + 4*(l/32) + v%4 of the 32x32 block: a quad of v is 4 consecutive channels of one pixel.
    const int f_hi = (lane >> 5) * 4;
    with_activation(s.act, [&](auto act_c) {
    constexpr int ACT = decltype(act_c)::value;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int m = m0 + wm * WM + i * 32 + frag_row;
        if (m >= M) continue;
        const size_t orow = (size_t)m * s.K;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * WN + j * 32 + 8 * g + f_hi;
                const float4 bv = *(const float4*)(bias + n);
                float v0 = acc[i][j][4 * g + 0] + bv.x, v1 = acc[i][j][4 * g + 1] + bv.y;
                float v2 = acc[i][j][4 * g + 2] + bv.z, v3 = acc[i][j][4 * g + 3] + bv.w;
                if (res) {
                    uint2 rv = *(const uint2*)(res + orow + n);
                    v0 += bf16_to_f32(rv.x & 0xFFFFu); v1 += bf16_to_f32(rv.x >> 16);
                    v2 += bf16_to_f32(rv.y & 0xFFFFu); v3 += bf16_to_f32(rv.y >> 16);
                }
                uint2 o;
                o.x = pack_bf16(act_fn(v0, ACT), act_fn(v1, ACT));
                o.y = pack_bf16(act_fn(v2, ACT), act_fn(v3, ACT));
                *(uint2*)(y + orow + n) = o;
            }
        }
    }
    });
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N>
hipError_t launch(const void* x, const void* wp, const float* bias, const void* res, void* y, const ConvShape& s,
                  hipStream_t stream)
{
    long long M = (long long)s.N * s.P * s.Q;
    int tiles_m = (int)((M + BM - 1) / BM), tiles_n = s.K / BN;
    long long total = (long long)tiles_m * tiles_n;
    if (total > 0x7FFFFFFFll) return hipErrorInvalidValue;
    constexpr size_t kLdsBytes = 2 * (size_t)(BM * (BK + kPad) + BN * BK) * sizeof(uint16_t);
    constexpr int kThreads = 64 * WAVES_M * WAVES_N;
    static bool configured = false;
    if (!configured) {   // more than the default 64 KiB of LDS per workgroup needs an explicit opt-in
        hipError_t e = hipFuncSetAttribute((const void*)conv_igemm_bf16_kernel<BM, BN, BK, WAVES_M, WAVES_N>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL((conv_igemm_bf16_kernel<BM, BN, BK, WAVES_M, WAVES_N>), dim3((unsigned)total), dim3(kThreads), kLdsBytes,
                       stream, (const uint16_t*)x, (const uint16_t*)wp, bias, (const uint16_t*)res, (uint16_t*)y, s, (int)M,
                       tiles_n);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------------
// Direct-to-LDS kernel.  Both operands of a reduction step are DMA'd from global memory straight into LDS (buffer
// loads with the LDS bit: lane i of a load lands at base + 16 i, one instruction fills 1 KiB).  No register staging
// and no LDS store instructions (an LDS store instruction moves 64 bytes per clock, half the read rate, and the
// staging registers cost occupancy).
//   * Filters: one load = one fragment of the repacked filter tensor, read back linearly.
//   * Activations: one load = 16 pixel rows x 64 bytes (a 32-channel run), four adjacent lanes per row so the global
//     access stays 64 bytes contiguous.  Inside the 1 KiB block the 16-byte chunk c of row r sits in slot
//     4 r + (c ^ f(r)), f(r) = ((r >> 1) & 3) ^ (r >> 3): the later operand read (lane = pixel row, fixed chunk) then
//     touches every LDS bank equally, whether the hardware resolves conflicts per 8 or per 16 lanes.  The lane that
//     fills slot i simply fetches the chunk that belongs there.
// Three LDS stages, loads two steps ahead, one barrier per step:
//     wait until this wave's loads of step u have landed | barrier | issue loads of step u+2 into the stage that
//     step u-1 was computed from (every wave is past that, it is behind the barrier) | compute step u.
// ---------------------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void;

// Which group a tile belongs to in a grouped launch, and what that means for the tile: its first output pixel, the end of
// the group's pixels, its position among the filter tiles, the group's filters and bias.  Tiles are numbered group by
// group, filter tiles fastest; every group starts a fresh row of tiles, so no tile mixes two experts' weights.
struct TileOrigin {
    int m0, m_end, tile_n;
    const uint16_t* wp;
    const float* bias;
};
template <int BM>
__device__ __forceinline__ TileOrigin locate_tile(int tile, int tiles_n, int PQ, int M, const uint16_t* wp, const float* bias,
                                                  const GroupTable& gt, uint32_t off_w, uint32_t off_b)
{
    TileOrigin o;
    if (gt.n == 0) {
        o.tile_n = tile % tiles_n;
        o.m0 = (tile / tiles_n) * BM;
        o.m_end = M;
        o.wp = wp;
        o.bias = bias;
        return o;
    }
    int g = 0, t = tile;
    for (;; ++g) {                                            // the launch has exactly sum-of-tiles workgroups
        const int rows = (gt.first_row[g + 1] - gt.first_row[g]) * PQ;
        const int tiles_g = ((rows + BM - 1) / BM) * tiles_n;
        if (t < tiles_g || g + 1 >= gt.n) break;
        t -= tiles_g;
    }
    o.tile_n = t % tiles_n;
    o.m0 = gt.first_row[g] * PQ + (t / tiles_n) * BM;
    o.m_end = gt.first_row[g + 1] * PQ;
    const char* base = (const char*)gt.weights[g];
    o.wp = (const uint16_t*)(base + off_w);
    o.bias = (const float*)(base + off_b);
    return o;
}


// Epilogue of the direct-to-LDS kernels: + bias (+ residual), activation, round to bf16 in the accumulator layout (a
// lane holds 4 consecutive channels of one pixel per accumulator quad), then through a wave-private LDS buffer of
// 32 rows so that the global stores are 16 bytes per lane and cover whole rows of the wave tile (full cache lines
// instead of 8-byte pieces of 32 different lines per instruction).  LDS operations of one wave execute in program
// order, so the wave-private buffer needs no barrier between its writes and reads.
template <int MB, int NB, int ACT, bool RES>
__device__ __forceinline__ void store_tile_via_lds_act(f32x16 (&acc)[MB][NB], uint16_t* stage, const float* __restrict__ bias,
                                                   const uint16_t* __restrict__ res, uint16_t* __restrict__ y, int m_wave,
                                                   int n_wave, int M, int K, int lane)
{
    constexpr int WN = NB * 32, ROW = WN + 8;             // elements; 16 bytes of padding per staged row
    constexpr int CPR = WN / 8;                            // 16-byte chunks per row
    constexpr int T = 32 * CPR / 64;                       // chunks per lane and 32-row block
    const int frag_row = lane & 31, f_hi = (lane >> 5) * 4;
    // the residual takes the same road in the other direction: row-contiguous 16-byte loads (all issued up front),
    // staged in LDS, picked up in the accumulator layout
    u32x4 rres[MB][T];
    if (RES) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int idx = lane + 64 * t;
                const int mo = m_wave + i * 32 + idx / CPR;
                rres[i][t] = mo < M ? *(const u32x4*)(res + (size_t)mo * K + n_wave + (idx % CPR) * 8) : u32x4{0u, 0u, 0u, 0u};
            }
    }
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        if (RES) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int idx = lane + 64 * t;
                *(u32x4*)(stage + (idx / CPR) * ROW + (idx % CPR) * 8) = rres[i][t];
            }
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nl = j * 32 + 8 * g + f_hi;
                uint2* cell = (uint2*)(stage + frag_row * ROW + nl);
                const float4 bv = *(const float4*)(bias + n_wave + nl);
                float v0 = acc[i][j][4 * g + 0] + bv.x, v1 = acc[i][j][4 * g + 1] + bv.y;
                float v2 = acc[i][j][4 * g + 2] + bv.z, v3 = acc[i][j][4 * g + 3] + bv.w;
                if (RES) {
                    const uint2 rv = *cell;
                    v0 += bf16_to_f32(rv.x & 0xFFFFu); v1 += bf16_to_f32(rv.x >> 16);
                    v2 += bf16_to_f32(rv.y & 0xFFFFu); v3 += bf16_to_f32(rv.y >> 16);
                }
                uint2 o;
                o.x = pack_bf16(act_fn(v0, ACT), act_fn(v1, ACT));
                o.y = pack_bf16(act_fn(v2, ACT), act_fn(v3, ACT));
                *cell = o;
            }
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int idx = lane + 64 * t;
            const int row = idx / CPR, ch = idx % CPR;
            const int mo = m_wave + i * 32 + row;
            const u32x4 v = *(const u32x4*)(stage + row * ROW + ch * 8);
            if (mo < M) *(u32x4*)(y + (size_t)mo * K + n_wave + ch * 8) = v;
        }
    }
}

template <int MB, int NB>
__device__ __forceinline__ void store_tile_via_lds(f32x16 (&acc)[MB][NB], uint16_t* stage, const float* __restrict__ bias,
                                                   const uint16_t* __restrict__ res, uint16_t* __restrict__ y, int m_wave,
                                                   int n_wave, int M, int K, int act, int lane)
{
    with_activation(act, [&](auto a) {
        if (res) store_tile_via_lds_act<MB, NB, decltype(a)::value, true>(acc, stage, bias, res, y, m_wave, n_wave, M, K, lane);
        else store_tile_via_lds_act<MB, NB, decltype(a)::value, false>(acc, stage, bias, res, y, m_wave, n_wave, M, K, lane);
    });
}

// host side of a grouped launch: the table and where a layer's filters and bias sit inside every group's blob
struct Grouping {
    GroupTable table{};              // table.n == 0: plain launch
    uint32_t off_w = 0, off_b = 0;
};
inline long long count_tiles(long long M, long long PQ, int BM, int tiles_n, const GroupTable& gt)
{
    if (gt.n == 0) return (M + BM - 1) / BM * tiles_n;
    long long total = 0;
    for (int g = 0; g < gt.n; ++g) total += ((gt.first_row[g + 1] - gt.first_row[g]) * PQ + BM - 1) / BM * tiles_n;
    return total;
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    // s_waitcnt with only the vector-memory counter armed (expcnt and lgkmcnt fields at their maxima)
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// The wait in front of a step's barrier.  Besides the wave's own loads of the step (all but the newest N vector-memory
// operations) it also drains the wave's LDS reads: the compiler is free to sink the last matrix-core instructions of a
// step below the barrier, and with them the wait for their operand reads, so a wave could pass the barrier with reads of
// the previous step still queued while another wave's DMA of a later step already targets the same LDS stage.
template <int N> __device__ __forceinline__ void wait_before_barrier()
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void conv_igemm_dma_kernel(const uint16_t* __restrict__ x,
                                                                   const uint16_t* __restrict__ wp_all,
                                                                   const float* __restrict__ bias_all,
                                                                   const uint16_t* __restrict__ res,
                                                                   uint16_t* __restrict__ y, ConvShape s, int M,
                                                                   int tiles_n, GroupTable gt, uint32_t off_w, uint32_t off_b)
{
#if defined(__HIP_DEVICE_COMPILE__)      // the host pass only needs the launch stub (LDS address-space casts do not exist there)
    constexpr int BK = 32, KS = 2, kStages = 3;
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int MB = WM / 32, NB = WN / 32;
    constexpr int FA = BM / 16, FB = BN / 32 * KS;           // 1 KiB blocks per step: 16-row activation blocks, filter fragments
    static_assert(FA % NW == 0 && FB % NW == 0, "every wave issues the same number of loads");
    constexpr int A_PER_WAVE = FA / NW, B_PER_WAVE = FB / NW;
    constexpr int LOADS = A_PER_WAVE + B_PER_WAVE;
    constexpr int FRAG = 512;                                 // elements per 1 KiB block
    constexpr int STAGE = (FA + FB) * FRAG;                   // elements

    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // kStages * STAGE elements

    int tile;
    {
        int L = blockIdx.x, total = gridDim.x;
        int xcd = L % kXcds, slot = L / kXcds;
        int base = total / kXcds, rem = total % kXcds;
        tile = xcd * base + (xcd < rem ? xcd : rem) + slot;
    }
    const TileOrigin org = locate_tile<BM>(tile, tiles_n, s.P * s.Q, M, wp_all, bias_all, gt, off_w, off_b);
    const int m0 = org.m0, n0 = org.tile_n * BN;
    M = org.m_end;                                            // rows of this tile's group end here
    const uint16_t* const wp = org.wp;
    const float* const bias = org.bias;
    const int tid = threadIdx.x, lane = tid & 63, wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wid / WAVES_N, wn = wid % WAVES_N;

    const int cblocks = s.C / BK;
    const int RS = s.R * s.S;
    const int nsteps = RS * cblocks;
    const int ks16_total = nsteps * KS;

    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(x, (uint32_t)s.N * (uint32_t)(s.H * s.W * s.C) * 2u);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wp, (uint32_t)s.K * (uint32_t)(RS * s.C) * 2u);

    // rows this lane fetches: block (wid * A_PER_WAVE + j), row lane / 4 of the block; which 16-byte chunk of the
    // 32-channel run follows from the slot the lane fills
    auto swz = [](int r16) { return ((r16 >> 1) & 3) ^ (r16 >> 3); };
    int32_t a_off[A_PER_WAVE];
    uint64_t a_mask[A_PER_WAVE];
    {
        const int PQ = s.P * s.Q;
        const int chunk = (lane & 3) ^ swz(lane >> 2);
#pragma unroll
        for (int j = 0; j < A_PER_WAVE; ++j) {
            int m = m0 + (wid * A_PER_WAVE + j) * 16 + (lane >> 2);
            bool ok = m < M;
            int mm = ok ? m : 0;
            int n = mm / PQ, pq = mm % PQ;
            int p = pq / s.Q, q = pq % s.Q;
            int ih0 = p * s.stride - s.pad, iw0 = q * s.stride - s.pad;
            a_off[j] = ((n * s.H + ih0) * s.W + iw0) * s.C * 2 + chunk * 16;
            uint64_t mask = 0;
            for (int rr = 0; rr < s.R; ++rr)
                for (int tt = 0; tt < s.S; ++tt)
                    if (ok && (unsigned)(ih0 + rr) < (unsigned)s.H && (unsigned)(iw0 + tt) < (unsigned)s.W)
                        mask |= 1ull << (rr * s.S + tt);
            a_mask[j] = mask;
        }
    }
    // filter fragments of this wave: (wid * B_PER_WAVE + j) = nb * KS + ks
    uint32_t b_off[B_PER_WAVE];
#pragma unroll
    for (int j = 0; j < B_PER_WAVE; ++j) {
        int fb = wid * B_PER_WAVE + j;
        b_off[j] = (uint32_t)((((n0 / 32 + fb / KS) * ks16_total + fb % KS) * FRAG + lane * 8) * 2);
    }

    int r = 0, t = 0, cb = 0, f_step = 0;
    auto issue = [&](int stage) {
        uint16_t* const st = lds + stage * STAGE;
        const int rs = r * s.S + t;
        const int32_t win = ((r * s.W + t) * s.C + cb * BK) * 2;
#pragma unroll
        for (int j = 0; j < A_PER_WAVE; ++j) {
            uint32_t off = ((a_mask[j] >> rs) & 1ull) ? (uint32_t)(a_off[j] + win) : kOutOfRange;
            // (the immediate offset of such a load would also shift the LDS destination: keep it 0)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (lds_void*)(st + (wid * A_PER_WAVE + j) * FRAG), 16, off, 0, 0, 0);
        }
        const uint32_t wstep = (uint32_t)f_step * (KS * FRAG * 2);
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lds_void*)(st + (FA + wid * B_PER_WAVE + j) * FRAG), 16, b_off[j],
                                                     wstep, 0, 0);
        if (f_step + 1 < nsteps) {
            ++f_step;
            if (++cb == cblocks) { cb = 0; if (++t == s.S) { t = 0; ++r; } }
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand read: pixel row lane % 32 of a 32-row block, chunk 2 ks + lane / 32 -> element offset inside the
    // two 1 KiB blocks; the chunk of ks = 1 is the one of ks = 0 with bit 1 flipped (32 bytes = 16 elements)
    static_assert(KS == 2, "two 16-channel halves per step");
    const int rd_row = lane & 31;
    const int rd0 = (rd_row >> 4) * FRAG + ((rd_row & 15) * 4 + ((lane >> 5) ^ swz(rd_row & 15))) * 8;
    auto compute = [&](int stage) {
        const uint16_t* a_lds = lds + stage * STAGE + (wm * MB * 2) * FRAG;
        const uint16_t* b_lds = lds + stage * STAGE + (FA + wn * NB * KS) * FRAG + lane * 8;
        bf16x8 af[KS][MB], bfr[KS][NB];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < MB; ++i) af[ks][i] = *(const bf16x8*)(a_lds + i * 2 * FRAG + (rd0 ^ (ks * 16)));
#pragma unroll
            for (int j = 0; j < NB; ++j) bfr[ks][j] = *(const bf16x8*)(b_lds + (j * KS + ks) * FRAG);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks][j], af[ks][i], acc[i][j], 0, 0, 0);
    };

    issue(0);
    issue(1);
    int stage_c = 0, stage_l = 2;
    for (int u = 0; u < nsteps; ++u) {
        wait_before_barrier<LOADS>();        // step u has landed; step u + 1 may still be in flight
        __builtin_amdgcn_s_barrier();
        issue(stage_l);
        compute(stage_c);
        stage_c = stage_c == kStages - 1 ? 0 : stage_c + 1;
        stage_l = stage_l == kStages - 1 ? 0 : stage_l + 1;
    }
    wait_before_barrier<0>();
    __builtin_amdgcn_s_barrier();        // every wave is done with the operand stages: LDS is free for the epilogue
    store_tile_via_lds<MB, NB>(acc, lds + wid * (32 * (WN + 8)), bias, res, y, m0 + wm * WM, n0 + wn * WN, M, s.K, s.act, lane);
#endif
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_dma(const void* x, const void* wp, const float* bias, const void* res, void* y, const ConvShape& s,
                      hipStream_t stream, const Grouping& grp = Grouping())
{
    long long M = (long long)s.N * s.P * s.Q;
    int tiles_n = s.K / BN;
    long long total = count_tiles(M, (long long)s.P * s.Q, BM, tiles_n, grp.table);
    if (total > 0x7FFFFFFFll) return hipErrorInvalidValue;
    if (total == 0) return hipSuccess;
    constexpr size_t kLdsBytes = 3 * (size_t)(BM + BN) * 32 * sizeof(uint16_t);
    constexpr int kThreads = 64 * WAVES_M * WAVES_N;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)conv_igemm_dma_kernel<BM, BN, WAVES_M, WAVES_N>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL((conv_igemm_dma_kernel<BM, BN, WAVES_M, WAVES_N>), dim3((unsigned)total), dim3(kThreads), kLdsBytes, stream,
                       (const uint16_t*)x, (const uint16_t*)wp, bias, (const uint16_t*)res, (uint16_t*)y, s, (int)M, tiles_n,
                       grp.table, grp.off_w, grp.off_b);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------------
// 3x3, stride 1, pad 1: the activation slab is loaded ONCE per 32-channel block and shared by the nine window
// positions.  Output pixels are numbered m = (n, p, q) flattened and, with "same" padding, input pixel (n, h, w) has
// the same number; window position (r, s) of output pixel m reads input pixel m + (r-1) W + (s-1) whenever that
// position is inside the image.  A tile of BM consecutive output pixels therefore needs the BM + 2W + 2 consecutive
// input pixels starting at m0 - W - 1: they are DMA'd into LDS as 16-row blocks (same swizzle as above) while the
// previous channel block is being computed, one block per wave and step.  Window positions outside the image are
// redirected to a 64-byte row of zeros; every lane keeps its nine LDS addresses per 32-row block in registers, so the
// inner loop has no address arithmetic beyond adding the slab buffer's base.  Filters: as above, three stages.
// ---------------------------------------------------------------------------------------------------------------
constexpr int kSlabMaxW = 56;

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void conv3x3_slab_kernel(const uint16_t* __restrict__ x,
                                                                    const uint16_t* __restrict__ wp_all,
                                                                    const float* __restrict__ bias_all,
                                                                    const uint16_t* __restrict__ res,
                                                                    uint16_t* __restrict__ y, ConvShape s, int M,
                                                                    int tiles_n, GroupTable gt, uint32_t off_w, uint32_t off_b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int BK = 32, KS = 2, kTaps = 9;
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int MB = WM / 32, NB = WN / 32;
    constexpr int FRAG = 512;                                             // elements per 1 KiB block
    constexpr int SB_CAP = (BM + 2 * kSlabMaxW + 2 + 15) / 16;            // slab blocks per channel block (capacity)
    static_assert(SB_CAP <= 8 * NW, "the slab must be complete one step before it is used");
    constexpr int SLAB = SB_CAP * FRAG + 64;                              // + the row of zeros (32 elements) + padding
    constexpr int ZERO_OFF = SB_CAP * FRAG;                               // elements, inside either slab buffer
    constexpr int FB = BN / 32 * KS;
    static_assert(FB % NW == 0, "every wave issues the same number of loads");
    constexpr int B_PER_WAVE = FB / NW;
    constexpr int B_STAGE = FB * FRAG;
    constexpr int SPARE = 2 * SLAB;                                       // 1 KiB that absorbs the padding loads
    constexpr int B_BASE = SPARE + FRAG;
    // 64-row wave tiles have registers for two sets of operands: ALL operands of step u + 1 (filters too) are read while
    // step u is multiplied, so after a step's barrier the matrix cores start at once instead of waiting for the filter
    // reads.  A wave then keeps its SIMD's matrix core busy on its own, which matters whenever the other workgroup of the
    // compute unit is in its epilogue.  The filters then have to be in LDS one step earlier: four stages, loads three
    // steps ahead.
    constexpr bool kDeep = MB <= 2;
    constexpr int kStagesB = kDeep ? 4 : 3;

    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // 2 slabs | spare block | 3 or 4 filter stages

    int tile;
    {
        int L = blockIdx.x, total = gridDim.x;
        int xcd = L % kXcds, slot = L / kXcds;
        int base = total / kXcds, rem = total % kXcds;
        tile = xcd * base + (xcd < rem ? xcd : rem) + slot;
    }
    const TileOrigin org = locate_tile<BM>(tile, tiles_n, s.H * s.W, M, wp_all, bias_all, gt, off_w, off_b);
    const int m0 = org.m0, n0 = org.tile_n * BN;
    M = org.m_end;                                            // rows of this tile's group end here
    const uint16_t* const wp = org.wp;
    const float* const bias = org.bias;
    const int tid = threadIdx.x, lane = tid & 63, wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wid / WAVES_N, wn = wid % WAVES_N;
    const int W = s.W, H = s.H;
    const int cblocks = s.C / BK;
    const int ks16_total = kTaps * cblocks * KS;
    const int total_px = s.N * H * W;
    const int slab_rows = BM + 2 * W + 2;

    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(x, (uint32_t)total_px * (uint32_t)s.C * 2u);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wp, (uint32_t)s.K * (uint32_t)(kTaps * s.C) * 2u);

    auto swz = [](int r16) { return ((r16 >> 1) & 3) ^ (r16 >> 3); };

    // the rows of zeros
    if (tid < 8) {
        *(u32x4*)(lds + ZERO_OFF + (tid & 3) * 8 + (tid >> 2) * SLAB) = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();

    // slab loader: row lane / 4 of a block, chunk chosen by the slot this lane fills
    const int ld_row = lane >> 2;
    const int ld_chunk = (lane & 3) ^ swz(ld_row);
    const int g_base = m0 - (W + 1) + ld_row;                 // input pixel of slab row ld_row
    auto issue_slab = [&](int cb, int tap, int parity) {
        const int sb = tap * NW + wid;                        // wave-uniform
        const int rho = sb * 16 + ld_row;
        const int g = g_base + sb * 16;
        const bool ok = sb < SB_CAP && cb < cblocks && rho < slab_rows && (unsigned)g < (unsigned)total_px;
        const uint32_t off = ok ? (uint32_t)((g * s.C + cb * BK + ld_chunk * 8) * 2) : kOutOfRange;
        uint16_t* dst = sb < SB_CAP ? lds + parity * SLAB + sb * FRAG : lds + SPARE;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (lds_void*)dst, 16, off, 0, 0, 0);
    };
    uint32_t b_off[B_PER_WAVE];
#pragma unroll
    for (int j = 0; j < B_PER_WAVE; ++j) {
        int fb = wid * B_PER_WAVE + j;
        b_off[j] = (uint32_t)((((n0 / 32 + fb / KS) * ks16_total + fb % KS) * FRAG + lane * 8) * 2);
    }
    auto issue_b = [&](int cb, int tap, int stage) {
        if (tap >= kTaps) { tap -= kTaps; ++cb; }
        if (cb >= cblocks) { cb = cblocks - 1; tap = kTaps - 1; }          // past the end: re-read the last step
        const uint32_t wstep = (uint32_t)((tap * cblocks + cb) * KS) * (FRAG * 2);
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lds_void*)(lds + B_BASE + stage * B_STAGE + (wid * B_PER_WAVE + j) * FRAG),
                                                     16, b_off[j], wstep, 0, 0);
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // prologue: the whole first slab, then filters of steps 0 and 1 (and 2) with one padding load between them so that
    // the order of outstanding loads is the steady-state one (slab piece, filters, slab piece, filters)
#pragma unroll
    for (int t = 0; t < (SB_CAP + NW - 1) / NW; ++t) issue_slab(0, t, 0);
    issue_b(0, 0, 0);
    issue_slab(cblocks, 8, 0);                                              // lands in the spare block
    issue_b(0, 1, 1);
    if (kDeep) {
        issue_slab(cblocks, 8, 0);
        issue_b(0, 2, 2);
    }

    // (built while the first loads are in flight)
    // operand addresses (elements, relative to a slab buffer) of this lane's pixel rows for the nine positions.
    // Slab row rho, chunk c sits at element 32 rho + 8 (c ^ f(rho & 15)) (16-row blocks of 512 elements are contiguous).
    // Kept free of branches and integer divisions: this runs once per tile and a 64-channel layer has only 18 steps
    // to amortise it over.  Pixel coordinates come from the tile's first pixel (one wave-uniform division) plus small
    // exact float divisions (numerators below 2^13, divisors up to 56^2).
    int32_t a_addr[MB][kTaps];
    {
        const int HW = H * W;
        const int pq0 = __builtin_amdgcn_readfirstlane(m0 % HW);
        const float inv_hw = 1.0f / (float)HW, inv_w = 1.0f / (float)W;
        const int khalf = lane >> 5;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const int ml = wm * WM + i * 32 + (lane & 31);
            const int ok = (m0 + ml) < M;
            const int t0 = pq0 + ml;                                       // < H*W + BM
            const int pq = t0 - (int)(((float)t0 + 0.5f) * inv_hw) * HW;
            const int p = (int)(((float)pq + 0.5f) * inv_w), q = pq - p * W;
            const int row_in[3] = {ok & (p > 0), ok, ok & (p < H - 1)};
            const int col_in[3] = {q > 0, 1, q < W - 1};
#pragma unroll
            for (int rr = 0; rr < 3; ++rr)
#pragma unroll
                for (int tt = 0; tt < 3; ++tt) {
                    const int rho = ml + rr * W + tt;                      // = ml + (W + 1) + (rr - 1) W + (tt - 1)
                    const int chunk = (khalf ^ (rho >> 1) ^ ((rho >> 3) & 1)) & 3;
                    const int a = rho * 32 + chunk * 8;
                    a_addr[i][rr * 3 + tt] = (row_in[rr] & col_in[tt]) ? a : ZERO_OFF + khalf * 8;
                }
        }
    }

    // Activation operands of position tap+1 are read while position tap is multiplied: the slab does not change
    // inside a channel block, so only the filter operands have to wait for the step's barrier.  (With 128-row wave
    // tiles there are no registers left for that; there the reads of the second 16-channel half are slipped between
    // the matrix-core instructions of the first.)
    constexpr bool kAhead = MB <= 2;
    if constexpr (kDeep) {
        bf16x8 af[2][KS][MB], bfr[2][KS][NB];   // [step parity]
        auto read_a = [&](int par, const uint16_t* slab, int tap) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int i = 0; i < MB; ++i) af[par][ks][i] = *(const bf16x8*)(slab + (a_addr[i][tap] ^ (ks * 16)));
        };
        auto read_b = [&](int par, int stage) {
            const uint16_t* b_lds = lds + B_BASE + stage * B_STAGE + (wn * NB * KS) * FRAG + lane * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int j = 0; j < NB; ++j) bfr[par][ks][j] = *(const bf16x8*)(b_lds + (j * KS + ks) * FRAG);
        };
        // operands of step 0: its filters and the first slab have landed when all but the newest two steps' loads have
        wait_before_barrier<2 * (1 + B_PER_WAVE)>();
        __builtin_amdgcn_s_barrier();
        read_a(0, lds, 0);
        read_b(0, 0);
        static_assert(SB_CAP <= 7 * NW, "the next slab is complete one step before its first operands are read ahead");
        int stage_rd = 1, stage_ld = 3;          // stage of the NEXT step's filters; stage the loads three steps ahead go to
        // one step; TAP and the register set CUR of its operands are compile-time (a channel block has nine positions, so
        // the sets swap roles from one block to the next: blocks are walked in pairs)
        auto step = [&](auto tap_c, auto cur_c, int cb) {
            constexpr int tap = decltype(tap_c)::value, cur = decltype(cur_c)::value, nxt = cur ^ 1;
            constexpr int kReads = KS * MB + KS * NB, kMfma = KS * MB * NB;
            const bool more = cb + 1 < cblocks;
            // the filters of the next step (and, at a channel block's last position, the whole next slab: its last piece
            // was issued at least two steps ago) have landed; only this wave's newest loads may still be in flight
            wait_before_barrier<1 + B_PER_WAVE>();
            __builtin_amdgcn_s_barrier();
            issue_slab(cb + 1, tap, (cb + 1) & 1);
            issue_b(cb, tap + 3, stage_ld);
            // operands of the next step: next position of this channel block, or position 0 of the next block
            if (tap + 1 < kTaps) { read_a(nxt, lds + (cb & 1) * SLAB, tap + 1); read_b(nxt, stage_rd); }
            else if (more) { read_a(nxt, lds + ((cb + 1) & 1) * SLAB, 0); read_b(nxt, stage_rd); }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ks][j], af[cur][ks][i], acc[i][j], 0, 0, 0);
            // issue order inside the step (0x100 = LDS read, 0x008 = matrix core): matrix-core instructions from the start,
            // the next step's operand reads slipped in between them one by one
            if (tap + 1 < kTaps || more) {
#pragma unroll
                for (int t = 0; t < (kReads < kMfma ? kReads : kMfma); ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                if (kReads > kMfma) __builtin_amdgcn_sched_group_barrier(0x100, kReads - kMfma, 0);
                if (kReads < kMfma) __builtin_amdgcn_sched_group_barrier(0x008, kMfma - kReads, 0);
            } else {
                __builtin_amdgcn_sched_group_barrier(0x008, kMfma, 0);
            }
            stage_rd = (stage_rd + 1) & 3;
            stage_ld = (stage_ld + 1) & 3;
        };
        auto block = [&](auto first_c, int cb) {        // the nine positions of channel block cb, starting in register set FIRST
            constexpr int f = decltype(first_c)::value;
            step(std::integral_constant<int, 0>{}, std::integral_constant<int, f>{}, cb);
            step(std::integral_constant<int, 1>{}, std::integral_constant<int, f ^ 1>{}, cb);
            step(std::integral_constant<int, 2>{}, std::integral_constant<int, f>{}, cb);
            step(std::integral_constant<int, 3>{}, std::integral_constant<int, f ^ 1>{}, cb);
            step(std::integral_constant<int, 4>{}, std::integral_constant<int, f>{}, cb);
            step(std::integral_constant<int, 5>{}, std::integral_constant<int, f ^ 1>{}, cb);
            step(std::integral_constant<int, 6>{}, std::integral_constant<int, f>{}, cb);
            step(std::integral_constant<int, 7>{}, std::integral_constant<int, f ^ 1>{}, cb);
            step(std::integral_constant<int, 8>{}, std::integral_constant<int, f>{}, cb);
        };
        for (int cb = 0; cb < cblocks; cb += 2) {
            block(std::integral_constant<int, 0>{}, cb);
            if (cb + 1 < cblocks) block(std::integral_constant<int, 1>{}, cb + 1);
        }
    } else
    for (int cb = 0; cb < cblocks; ++cb) {
        const uint16_t* slab = lds + (cb & 1) * SLAB;
        bf16x8 af[2][KS][MB];               // [tap parity]
#pragma unroll
        for (int tap = 0; tap < kTaps; ++tap) {
            wait_before_barrier<1 + B_PER_WAVE>();      // everything up to this step's filters has landed
            __builtin_amdgcn_s_barrier();
            issue_slab(cb + 1, tap, (cb + 1) & 1);
            issue_b(tap + 2 < kTaps ? cb : cb + 1, (tap + 2) % kTaps, (tap + 2) % 3);
            const uint16_t* b_lds = lds + B_BASE + (tap % 3) * B_STAGE + (wn * NB * KS) * FRAG + lane * 8;
            bf16x8 bfr[KS][NB];
            if (!kAhead || tap == 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int i = 0; i < MB; ++i) af[tap & 1][ks][i] = *(const bf16x8*)(slab + (a_addr[i][tap] ^ (ks * 16)));
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int j = 0; j < NB; ++j) bfr[ks][j] = *(const bf16x8*)(b_lds + (j * KS + ks) * FRAG);
            if (kAhead && tap + 1 < kTaps) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int i = 0; i < MB; ++i)
                        af[(tap + 1) & 1][ks][i] = *(const bf16x8*)(slab + (a_addr[i][tap + 1] ^ (ks * 16)));
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks][j], af[tap & 1][ks][i], acc[i][j], 0, 0, 0);
            // issue order inside the step (0x100 = LDS read, 0x008 = matrix core)
            if (kAhead) {
                // this step's operands first (filters; at position 0 also the activations), then the matrix-core
                // instructions with the next position's activation reads slipped in between
                if (tap == 0) __builtin_amdgcn_sched_group_barrier(0x100, KS * NB + KS * MB, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, KS * NB, 0);
                if (tap + 1 < kTaps) {
#pragma unroll
                    for (int t = 0; t < KS * MB; ++t) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, KS * MB * NB - KS * MB, 0);
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x008, KS * MB * NB, 0);
                }
            } else {
                // the operands of the first 16-channel half, then matrix-core instructions with the reads of the second
                // half slipped in between them
                __builtin_amdgcn_sched_group_barrier(0x100, MB + NB, 0);
#pragma unroll
                for (int t = 0; t < MB + NB; ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, KS * MB * NB - (MB + NB), 0);
            }
        }
    }
    wait_before_barrier<0>();
    __builtin_amdgcn_s_barrier();        // every wave is done with the operand stages: LDS is free for the epilogue
    store_tile_via_lds<MB, NB>(acc, lds + wid * (32 * (WN + 8)), bias, res, y, m0 + wm * WM, n0 + wn * WN, M, s.K, s.act, lane);
#endif
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_slab(const void* x, const void* wp, const float* bias, const void* res, void* y, const ConvShape& s,
                       hipStream_t stream, const Grouping& grp = Grouping())
{
    long long M = (long long)s.N * s.P * s.Q;
    int tiles_n = s.K / BN;
    long long total = count_tiles(M, (long long)s.P * s.Q, BM, tiles_n, grp.table);
    if (total > 0x7FFFFFFFll) return hipErrorInvalidValue;
    if (total == 0) return hipSuccess;
    constexpr int kSbCap = (BM + 2 * kSlabMaxW + 2 + 15) / 16;
    constexpr int kStagesB = (BM / WAVES_M) / 32 <= 2 ? 4 : 3;             // as in the kernel: 64-row wave tiles read one step ahead
    constexpr size_t kLdsBytes = (2 * (size_t)(kSbCap * 512 + 64) + 512 + kStagesB * (size_t)BN * 32) * sizeof(uint16_t);
    constexpr int kThreads = 64 * WAVES_M * WAVES_N;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)conv3x3_slab_kernel<BM, BN, WAVES_M, WAVES_N>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL((conv3x3_slab_kernel<BM, BN, WAVES_M, WAVES_N>), dim3((unsigned)total), dim3(kThreads), kLdsBytes, stream,
                       (const uint16_t*)x, (const uint16_t*)wp, bias, (const uint16_t*)res, (uint16_t*)y, s, (int)M, tiles_n,
                       grp.table, grp.off_w, grp.off_b);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_uses_slab(const ConvShape& s)
{
    return s.R == 3 && s.S == 3 && s.stride == 1 && s.pad == 1 && s.W <= kSlabMaxW && s.C % 32 == 0 && s.K % 64 == 0;
}

namespace {

template <int BK>
hipError_t pick_tile(const void* x, const void* wp, const float* bias, const void* res, void* y, const ConvShape& s,
                     hipStream_t stream)
{
    if (s.K % 128 == 0) return launch<128, 128, BK, 2, 2>(x, wp, bias, res, y, s, stream);
    if (s.K % 64 == 0) return launch<128, 64, BK, 2, 2>(x, wp, bias, res, y, s, stream);
    return launch<128, 32, BK, 4, 1>(x, wp, bias, res, y, s, stream);
}

}  // namespace

bool conv_mfma_supported(const ConvShape& s)
{
    return s.C > 0 && s.K > 0 && s.C % 32 == 0 && s.K % 32 == 0 && s.R * s.S <= 64;
}

void pack_filters_mfma(const uint16_t* w, uint16_t* out, int K, int red)
{
    // out[((nb * red/16 + ks) * 64 + lane) * 8 + i] = w[nb*32 + lane%32][ks*16 + (lane/32)*8 + i]
    const int ks_total = red / 16;
    for (int nb = 0; nb < K / 32; ++nb)
        for (int ks = 0; ks < ks_total; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const uint16_t* src = w + (size_t)(nb * 32 + lane % 32) * red + ks * 16 + (lane / 32) * 8;
                uint16_t* dst = out + (((size_t)nb * ks_total + ks) * 64 + lane) * 8;
                for (int i = 0; i < 8; ++i) dst[i] = src[i];
            }
}

hipError_t conv_mfma(const void* x, const void* wp, const float* bias, const void* res, void* y, const ConvShape& s,
                     hipStream_t stream)
{
    if (!conv_mfma_supported(s)) return hipErrorInvalidValue;
    long long M = (long long)s.N * s.P * s.Q;
    if (M <= 0) return hipSuccess;
    // 31-bit byte offsets inside the kernel (buffer offsets; bit 31 marks "out of range")
    if ((long long)s.N * s.H * s.W * s.C * 2 >= 0x7FFFFFFFll || (long long)s.K * s.R * s.S * s.C * 2 >= 0x7FFFFFFFll ||
        M >= 0x7FFFFFFFll - 256)
        return hipErrorInvalidValue;
    // 32-channel steps everywhere: measured equal or better than 64-channel steps on every ResNet layer shape
    if (conv_mfma_uses_slab(s)) {
        // 256-row and 128-row tiles measured within a few percent of each other on every ResNet-18 layer shape
        if (s.K % 128 == 0) return launch_slab<256, 128, 2, 2>(x, wp, bias, res, y, s, stream);
        return launch_slab<256, 64, 4, 1>(x, wp, bias, res, y, s, stream);
    }
    // 128-row tiles: three workgroups per compute unit; measured ahead of 256-row tiles on the ResNet layer shapes
    if (s.K % 128 == 0) return launch_dma<128, 128, 2, 2>(x, wp, bias, res, y, s, stream);
    if (s.K % 64 == 0) return launch_dma<128, 64, 2, 2>(x, wp, bias, res, y, s, stream);
    // filter counts that are not a multiple of 64: the register-staged kernel
    return pick_tile<32>(x, wp, bias, res, y, s, stream);
}

bool conv_mfma_groupable(const ConvShape& s)
{
    return conv_mfma_supported(s) && s.K % 64 == 0;
}

hipError_t conv_mfma_grouped(const void* x, const GroupTable& groups, size_t off_w, size_t off_b, const void* res, void* y,
                             const ConvShape& s, hipStream_t stream)
{
    if (!conv_mfma_groupable(s) || groups.n <= 0 || groups.n > kMaxGroups || groups.first_row[0] != 0 ||
        groups.first_row[groups.n] != s.N || off_w > 0x7FFFFFFFull || off_b > 0x7FFFFFFFull)
        return hipErrorInvalidValue;
    for (int g = 0; g < groups.n; ++g)
        if (groups.first_row[g + 1] < groups.first_row[g] || !groups.weights[g]) return hipErrorInvalidValue;
    long long M = (long long)s.N * s.P * s.Q;
    if (M <= 0) return hipSuccess;
    if ((long long)s.N * s.H * s.W * s.C * 2 >= 0x7FFFFFFFll || (long long)s.K * s.R * s.S * s.C * 2 >= 0x7FFFFFFFll ||
        M >= 0x7FFFFFFFll - 256)
        return hipErrorInvalidValue;
    Grouping grp;
    grp.table = groups;
    grp.off_w = (uint32_t)off_w;
    grp.off_b = (uint32_t)off_b;
    // every group starts a fresh row of tiles: 128-row tiles waste fewer rows past the end of a small group, 256-row
    // tiles (twice the accumulator rows per wave and operand read) are the faster ones where that waste stays small
    if (conv_mfma_uses_slab(s)) {
        const long long PQ = (long long)s.P * s.Q;
        const bool tall = 256 * count_tiles(M, PQ, 256, 1, groups) * 100 <= 128 * count_tiles(M, PQ, 128, 1, groups) * 104;
        if (s.K % 128 == 0)
            return tall ? launch_slab<256, 128, 2, 2>(x, nullptr, nullptr, res, y, s, stream, grp)
                        : launch_slab<128, 128, 2, 2>(x, nullptr, nullptr, res, y, s, stream, grp);
        return tall ? launch_slab<256, 64, 4, 1>(x, nullptr, nullptr, res, y, s, stream, grp)
                    : launch_slab<128, 64, 4, 1>(x, nullptr, nullptr, res, y, s, stream, grp);
    }
    if (s.K % 128 == 0) return launch_dma<128, 128, 2, 2>(x, nullptr, nullptr, res, y, s, stream, grp);
    return launch_dma<128, 64, 2, 2>(x, nullptr, nullptr, res, y, s, stream, grp);
}

}  // namespace k
}  // namespace coe
