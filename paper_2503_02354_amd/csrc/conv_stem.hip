// bf16 convolution for few input channels (the 7x7/2, C=3 stem) on the gfx950 matrix cores, optionally fused with
// the 3x3/2 max pool that follows it.
//
// With C=3 the reduction run that is contiguous in memory is one window row: S*C elements (21 for 7x7x3).  A workgroup
// stages the input patch of a 16x16 tile of conv outputs in LDS once, and every lane builds its matrix-core operand
// straight from that patch: the reduction is cut into 8-element chunks (ceil(S*C/8) per window row, zero weights where a
// chunk overhangs the row), and one v_mfma_f32_32x32x16_bf16 consumes two chunks (lanes 0-31 one, lanes 32-63 the next).
// The filters are repacked into the same chunk order in LDS once per workgroup, which then loops over many tiles.
// The patch is fetched row by row with 2-byte buffer loads through a per-row descriptor, so both image edges and
// rows outside the image read as zero without any per-element bounds arithmetic.
// Epilogue in fp32: + bias, activation, one round-to-nearest-even to bf16.
//
// Fused pool: the stem output is 1.6 MB per 224x224 image and the pool reads it straight back to keep a quarter of
// it.  In the fused form a 16x16 conv tile starts at (14t-1, 14u-1), its rounded outputs go to LDS, and the workgroup
// writes the 7x7 pooled pixels whose 3x3 windows lie inside the tile.  Rounding is monotonic, so the max of the rounded
// values equals what a separate pool kernel would produce from the stored conv output.
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
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;       // eight wavefronts per workgroup, two workgroups per compute unit (LDS): every phase of a
                                // tile (patch staging, products, epilogue, pool) is latency-bound, more waves overlap them;
                                // measured 17 % faster than four
constexpr int kThreads = 64 * kWaves;
constexpr int kRowsPerWave = 256 / kWaves;
constexpr int kMB = kRowsPerWave / 32;      // 32-row blocks per wavefront
constexpr int kTile = 16;        // conv-output tile is kTile x kTile pixels = 256 GEMM rows, 32 per wavefront
constexpr int kPoolTile = 7;     // pooled pixels per tile side in the fused form (3x3/2 windows inside 16 rows)
constexpr int kOutPad = 8;       // elements of padding per LDS row of the conv-output tile
constexpr int kMaxRowsPerWave = 48 / kWaves;   // patch rows one wavefront fetches (patch_rows <= 48)
constexpr int kMaxDwordsPerLane = 1;  // aligned dwords one lane fetches per patch row (patch_cols + 1 <= 128 elements)

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
template <typename F> __device__ __forceinline__ void with_activation(int act, F&& body)
{
    if (act == 1) body(std::integral_constant<int, 1>{});
    else if (act == 2) body(std::integral_constant<int, 2>{});
    else if (act == 3) body(std::integral_constant<int, 3>{});
    else body(std::integral_constant<int, 0>{});
}

struct StemGeom {
    int tiles_p, tiles_q, total_tiles;
    int patch_rows, patch_cols;   // patch_cols = elements of one patch row that are loaded ((tile-1)*stride+S)*C
    int patch_stride;             // elements per LDS patch row (even, covers the furthest chunk read)
    int cpr;                      // 8-element chunks per window row
    int ksteps;                   // matrix-core steps = ceil(R*cpr / 2)
    int wstride;                  // elements per LDS filter row
    int PP, PQ;                   // pooled output size (fused form)
};

// CPR_, R_: chunks per window row and window rows when known at compile time (the 7x7x3 stem: 3, 7), else 0: the
// reduction loop is then unrolled with constant offsets instead of running a counted loop with a carried (row, chunk).
template <int NB, bool POOL, int CPR_, int R_>
__global__ __launch_bounds__(kThreads, 4) void conv_smallc_bf16_kernel(const uint16_t* __restrict__ x,
                                                                     const uint16_t* __restrict__ w,
                                                                     const float* __restrict__ bias,
                                                                     uint16_t* __restrict__ y, ConvShape s, StemGeom g,
                                                                     const int32_t* __restrict__ rows)
{
    constexpr int K = 32 * NB;
    constexpr int OUT_STRIDE = K + kOutPad;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* wpack = smem;                               // [K][wstride]
    uint16_t* patch = smem + K * g.wstride;               // [patch_rows][patch_stride]
    uint16_t* otile = patch + g.patch_rows * g.patch_stride;   // [256][OUT_STRIDE], fused form only (16-byte aligned)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int SC = s.S * s.C;
    const int WC = s.W * s.C;

    // filters into chunk order; zero where a chunk overhangs its window row or the step count is padded
    for (int idx = tid; idx < K * g.ksteps * 16; idx += kThreads) {
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
    const int tile_step = POOL ? 2 * kPoolTile : kTile;   // conv rows/cols between tile origins
    const int tile_org = POOL ? -1 : 0;

    // The patch of the NEXT tile is fetched into registers while the current tile is computed: patch rows round-robin
    // over wavefronts, lanes along the row, one aligned dword (two elements) per lane and load.  A patch row starts at
    // element g_base of its image row, which may be odd: the loads start at the even element below it and the staging
    // step shifts by one element where needed (neighbour lane's dword + one v_alignbit), so that the LDS copy starts
    // exactly at g_base and the operand reads stay 4-byte aligned.  W*C is even, so no dword straddles a row's end.
    uint32_t pre[kMaxRowsPerWave][kMaxDwordsPerLane];
    int pre_shift = 0;
    auto prefetch = [&](int tile) {
        const int n = tile / (g.tiles_p * g.tiles_q);
        const int tp = (tile / g.tiles_q) % g.tiles_p, tq = tile % g.tiles_q;
        const int ih_base = (tp * tile_step + tile_org) * s.stride - s.pad;
        const int g_base = ((tq * tile_step + tile_org) * s.stride - s.pad) * s.C;   // may be negative
        const int e0 = g_base & ~1;                                                  // even element at or below g_base
        pre_shift = g_base - e0;
        // one descriptor per image; a dword outside its row (left or right of the image) or in a row outside the image
        // gets an offset beyond the descriptor's range and reads as zero
        // (with a row table, image n of the launch is image rows[n] of the array at x: request arranging's gather of
        // the inputs happens here instead of in a copy of its own)
        const int n_src = rows ? __builtin_amdgcn_readfirstlane(rows[n]) : n;
        const __amdgpu_buffer_rsrc_t rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x + (size_t)n_src * s.H * WC), 0, s.H * WC * 2, 0x00020000);
#pragma unroll
        for (int j = 0; j < kMaxDwordsPerLane; ++j) {
            const int e = e0 + 2 * (lane + 64 * j);
            const bool col_ok = (unsigned)e < (unsigned)WC;                          // WC is even: e + 1 < WC as well
#pragma unroll
            for (int i = 0; i < kMaxRowsPerWave; ++i) {
                const int pr = wid + i * (kThreads / 64);
                const int ih = ih_base + pr;
                const bool ok = col_ok && pr < g.patch_rows && (unsigned)ih < (unsigned)s.H;
                pre[i][j] = __builtin_amdgcn_raw_buffer_load_b32(rs, ok ? (ih * WC + e) * 2 : (int)0x80000000, 0, 0);
            }
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < kMaxRowsPerWave; ++i) {
            const int pr = wid + i * (kThreads / 64);
            if (pr < g.patch_rows) {
#pragma unroll
                for (int j = 0; j < kMaxDwordsPerLane; ++j) {
                    uint32_t v = pre[i][j];
                    if (pre_shift) {
                        // the dword one position further along the row: the next lane's, or lane 0's of the next load
                        uint32_t nb = __shfl_down(v, 1);
                        if (j + 1 < kMaxDwordsPerLane) {
                            const uint32_t first_of_next = __builtin_amdgcn_readfirstlane(pre[i][j + 1 < kMaxDwordsPerLane ? j + 1 : j]);
                            if (lane == 63) nb = first_of_next;
                        }
                        v = __builtin_amdgcn_alignbit(nb, v, 16);
                    }
                    const int col = 2 * (lane + 64 * j);
                    if (col + 1 >= g.patch_cols) v &= 0xFFFFu;            // nothing beyond the patch reaches LDS
                    if (col < g.patch_cols) *(uint32_t*)(patch + pr * g.patch_stride + col) = v;
                }
            }
        }
    };

    if ((int)blockIdx.x < g.total_tiles) prefetch(blockIdx.x);
    for (int tile = blockIdx.x; tile < g.total_tiles; tile += gridDim.x) {
        const int n = tile / (g.tiles_p * g.tiles_q);
        const int tp = (tile / g.tiles_q) % g.tiles_p, tq = tile % g.tiles_q;
        const int p0 = tp * tile_step + tile_org, q0 = tq * tile_step + tile_org;     // conv-output origin of the tile
        commit();
        __syncthreads();
        if (tile + (int)gridDim.x < g.total_tiles) prefetch(tile + gridDim.x);

        f32x16 acc[kMB][NB];
#pragma unroll
        for (int i = 0; i < kMB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        int a_off[kMB];
#pragma unroll
        for (int i = 0; i < kMB; ++i) {
            int ml = wid * kRowsPerWave + i * 32 + l32;
            a_off[i] = (ml / kTile) * s.stride * g.patch_stride + (ml % kTile) * s.stride * s.C;
        }
        auto kstep = [&](int koff, int chunk) {
            bf16x8 af[kMB], bfr[NB];
#pragma unroll
            for (int i = 0; i < kMB; ++i) {
                const uint32_t* p32 = (const uint32_t*)(patch + a_off[i] + koff);      // 4-byte aligned by construction
                uint4 v = make_uint4(p32[0], p32[1], p32[2], p32[3]);
                af[i] = __builtin_bit_cast(bf16x8, v);
            }
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
                bfr[jn] = *(const bf16x8*)(wpack + (jn * 32 + l32) * g.wstride + chunk * 8);
            // filter fragment first: a lane then holds 4 consecutive output channels of one pixel per accumulator quad
#pragma unroll
            for (int i = 0; i < kMB; ++i)
#pragma unroll
                for (int jn = 0; jn < NB; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[jn], af[i], acc[i][jn], 0, 0, 0);
        };
        if constexpr (CPR_ > 0) {
            constexpr int KSTEPS = (R_ * CPR_ + 1) / 2;
#pragma unroll
            for (int j = 0; j < KSTEPS; ++j) {
                // chunk 2j (lanes 0-31) and 2j+1 (lanes 32-63): window row and chunk inside it are constants; a padded
                // last chunk reads the last window row again (its filters are zero, any finite data will do)
                const int c0 = 2 * j, c1 = 2 * j + 1;
                const int r0 = c0 / CPR_ < R_ ? c0 / CPR_ : R_ - 1, r1 = c1 / CPR_ < R_ ? c1 / CPR_ : R_ - 1;
                const int off0 = r0 * g.patch_stride + (c0 % CPR_) * 8, off1 = r1 * g.patch_stride + (c1 % CPR_) * 8;
                kstep(half ? off1 : off0, 2 * j + half);
            }
        } else {
            int kr = half / g.cpr, kpart = half % g.cpr;          // window row and chunk inside it of this lane's chunk
            for (int j = 0; j < g.ksteps; ++j) {
                const int r = kr < s.R ? kr : s.R - 1;             // padded step: filters are zero, any finite data will do
                kstep(r * g.patch_stride + kpart * 8, 2 * j + half);
                kpart += 2;                                        // next step: two chunks on, without a division
                while (kpart >= g.cpr) { kpart -= g.cpr; ++kr; }
            }
        }

        // (dispatched once on the activation: a per-element test compiles into hundreds of branches)
        with_activation(s.act, [&](auto act_c) {
        constexpr int ACT = decltype(act_c)::value;
        // accumulator element v of lane l: pixel l%32 of the 32-pixel block, filter 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
        for (int i = 0; i < kMB; ++i) {
            const int ml = wid * kRowsPerWave + i * 32 + l32;
            const int p = p0 + ml / kTile, q = q0 + ml % kTile;
            const bool inside = (unsigned)p < (unsigned)s.P && (unsigned)q < (unsigned)s.Q;
#pragma unroll
            for (int jn = 0; jn < NB; ++jn)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int ch = jn * 32 + 8 * gq + half * 4;
                    const float4 bv = *(const float4*)(bias + ch);
                    uint2 o;
                    o.x = pack_bf16(act_fn(acc[i][jn][4 * gq + 0] + bv.x, ACT), act_fn(acc[i][jn][4 * gq + 1] + bv.y, ACT));
                    o.y = pack_bf16(act_fn(acc[i][jn][4 * gq + 2] + bv.z, ACT), act_fn(acc[i][jn][4 * gq + 3] + bv.w, ACT));
                    if (POOL) {
                        // outside the conv output: -inf (or 0 after ReLU, see the pool below) never wins the max
                        if (!inside) o = ACT == 1 ? make_uint2(0u, 0u) : make_uint2(0xFF80FF80u, 0xFF80FF80u);
                        *(uint2*)(otile + ml * OUT_STRIDE + ch) = o;
                    } else if (inside) {
                        *(uint2*)(y + (((size_t)n * s.P + p) * s.Q + q) * K + ch) = o;
                    }
                }
        }
        });
        if (POOL) {
            __syncthreads();
            // 7x7 pooled pixels x K/8 channel groups; window of pooled (a, b) = tile rows 2a..2a+2, cols 2b..2b+2
            for (int item = tid; item < kPoolTile * kPoolTile * (K / 8); item += kThreads) {
                const int c8 = item % (K / 8), pix = item / (K / 8);
                const int a = pix / kPoolTile, b = pix % kPoolTile;
                const int pi = tp * kPoolTile + a, pj = tq * kPoolTile + b;
                if (pi >= g.PP || pj >= g.PQ) continue;
                if (s.act == 1) {
                    // after ReLU every value is >= +0, and non-negative bf16 order like their bit patterns: the max is
                    // a packed 16-bit integer max, two channels per instruction (tile pixels outside the conv output
                    // hold 0 here, which never beats a real value)
                    u16x2 m[4] = {u16x2{0, 0}, u16x2{0, 0}, u16x2{0, 0}, u16x2{0, 0}};
#pragma unroll
                    for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                        for (int dc = 0; dc < 3; ++dc) {
                            const uint4 v = *(const uint4*)(otile + ((2 * a + dr) * kTile + 2 * b + dc) * OUT_STRIDE + c8 * 8);
                            m[0] = __builtin_elementwise_max(m[0], __builtin_bit_cast(u16x2, v.x));
                            m[1] = __builtin_elementwise_max(m[1], __builtin_bit_cast(u16x2, v.y));
                            m[2] = __builtin_elementwise_max(m[2], __builtin_bit_cast(u16x2, v.z));
                            m[3] = __builtin_elementwise_max(m[3], __builtin_bit_cast(u16x2, v.w));
                        }
                    uint4 o;
                    o.x = __builtin_bit_cast(uint32_t, m[0]); o.y = __builtin_bit_cast(uint32_t, m[1]);
                    o.z = __builtin_bit_cast(uint32_t, m[2]); o.w = __builtin_bit_cast(uint32_t, m[3]);
                    *(uint4*)(y + (((size_t)n * g.PP + pi) * g.PQ + pj) * K + c8 * 8) = o;
                    continue;
                }
                float best[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
                for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                    for (int dc = 0; dc < 3; ++dc) {
                        const uint4 v = *(const uint4*)(otile + ((2 * a + dr) * kTile + 2 * b + dc) * OUT_STRIDE + c8 * 8);
                        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            best[2 * e] = fmaxf(best[2 * e], __uint_as_float(wds[e] << 16));
                            best[2 * e + 1] = fmaxf(best[2 * e + 1], __uint_as_float(wds[e] & 0xFFFF0000u));
                        }
                    }
                uint4 o;
                o.x = (__float_as_uint(best[0]) >> 16) | (__float_as_uint(best[1]) & 0xFFFF0000u);
                o.y = (__float_as_uint(best[2]) >> 16) | (__float_as_uint(best[3]) & 0xFFFF0000u);
                o.z = (__float_as_uint(best[4]) >> 16) | (__float_as_uint(best[5]) & 0xFFFF0000u);
                o.w = (__float_as_uint(best[6]) >> 16) | (__float_as_uint(best[7]) & 0xFFFF0000u);
                *(uint4*)(y + (((size_t)n * g.PP + pi) * g.PQ + pj) * K + c8 * 8) = o;
            }
        }
        __syncthreads();      // patch (and the conv-output tile) are rewritten by the next tile
    }
}

bool geometry(const ConvShape& s, bool pool, StemGeom& g, size_t& smem)
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
    g.patch_stride = (ps + 7) / 8 * 8 + 8;                         // multiple of 8: the regions after it stay 16-byte aligned
    // The 32 lanes of an operand read cover two rows of the conv tile, 16 pixels each, stride * C elements apart inside a row:
    // dword 3 l for lane l of a row with the 7x7x3 stem's 6 elements per pixel.  Two tile rows are stride * patch_stride
    // elements apart; when that is a multiple of 32 dwords both rows hit the same 16 banks.  Shift it to 16 dwords mod 32:
    // the second row's banks (3 l + 16 mod 32) then fall between the first row's.
    for (int extra = 0; extra < 64; extra += 8)
        if ((s.stride * (g.patch_stride + extra) / 2) % 32 == 16) { g.patch_stride += extra; break; }
    if ((long long)s.H * s.W * s.C * 2 >= 0x7FFFFFFFll) return false;    // byte offsets inside one image are 31-bit
    if (g.patch_rows > kMaxRowsPerWave * (kThreads / 64) || g.patch_cols + 1 > kMaxDwordsPerLane * 128) return false;
    if ((s.W * s.C) % 2) return false;                             // aligned dwords must not straddle the end of an image row
    g.PP = (s.P + 2 - 3) / 2 + 1;
    g.PQ = (s.Q + 2 - 3) / 2 + 1;
    if (pool) {
        if (s.P < 2 || s.Q < 2) return false;
        g.tiles_p = (g.PP + kPoolTile - 1) / kPoolTile;
        g.tiles_q = (g.PQ + kPoolTile - 1) / kPoolTile;
    } else {
        g.tiles_p = (s.P + kTile - 1) / kTile;
        g.tiles_q = (s.Q + kTile - 1) / kTile;
    }
    long long total = (long long)s.N * g.tiles_p * g.tiles_q;
    if (total > 0x7FFFFFFFll) return false;
    g.total_tiles = (int)total;
    smem = sizeof(uint16_t) * ((size_t)s.K * g.wstride + (size_t)g.patch_rows * g.patch_stride +
                               (pool ? (size_t)kTile * kTile * (s.K + kOutPad) : 0));
    return smem <= 96 * 1024;
}

template <int NB, bool POOL, int CPR_, int R_>
hipError_t launch(const void* x, const void* w, const float* bias, void* y, const ConvShape& s, const StemGeom& g, size_t smem,
                  hipStream_t stream, const int32_t* rows)
{
    static bool configured = false;
    if (!configured) {   // more than the default 64 KiB of LDS per workgroup needs an explicit opt-in
        hipError_t e = hipFuncSetAttribute((const void*)conv_smallc_bf16_kernel<NB, POOL, CPR_, R_>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    int grid = g.total_tiles < 1024 ? g.total_tiles : 1024;
    hipLaunchKernelGGL((conv_smallc_bf16_kernel<NB, POOL, CPR_, R_>), dim3(grid), dim3(kThreads), smem, stream, (const uint16_t*)x,
                       (const uint16_t*)w, bias, (uint16_t*)y, s, g, rows);
    return hipGetLastError();
}

}  // namespace

bool conv_smallc_supported(const ConvShape& s, bool has_res, bool fused_pool)
{
    StemGeom g;
    size_t smem;
    return !has_res && geometry(s, fused_pool, g, smem);
}

hipError_t conv_smallc(const void* x, const void* w, const float* bias, void* y, const ConvShape& s, bool fused_pool,
                       hipStream_t stream, const int32_t* rows)
{
    StemGeom g;
    size_t smem = 0;
    if (!geometry(s, fused_pool, g, smem)) return hipErrorInvalidValue;
    if (g.total_tiles == 0) return hipSuccess;
    if (s.K == 64) {
        if (fused_pool && g.cpr == 3 && s.R == 7)         // the ResNet stem: reduction loop unrolled with constant offsets
            return launch<2, true, 3, 7>(x, w, bias, y, s, g, smem, stream, rows);
        return fused_pool ? launch<2, true, 0, 0>(x, w, bias, y, s, g, smem, stream, rows)
                          : launch<2, false, 0, 0>(x, w, bias, y, s, g, smem, stream, rows);
    }
    return fused_pool ? launch<1, true, 0, 0>(x, w, bias, y, s, g, smem, stream, rows)
                      : launch<1, false, 0, 0>(x, w, bias, y, s, g, smem, stream, rows);
}

}  // namespace k
}  // namespace coe
