// gfx950 kernels for transformer-shaped experts (bf16): patch gathering, class token + positions, layer norm,
// multi-head attention on the matrix cores.  Token tensors are [N][T][D], D contiguous.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace coe {
namespace k {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // round to nearest even
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// ---- patches of a non-overlapping convolution laid out as GEMM rows -------------------------------------------
// x [N][H][W][C] -> out [N][H/R][W/S][R][S*C]: one 16-byte chunk per thread; S*C*2 bytes is a multiple of 16.
__global__ __launch_bounds__(256) void patchify_kernel(const uint4* __restrict__ x, uint4* __restrict__ out, int N, int H, int W,
                                                       int R, int gh, int gw, int run_chunks)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)N * gh * gw * R * run_chunks;
    if (idx >= total) return;
    int ch = (int)(idx % run_chunks);
    size_t t = idx / run_chunks;
    int r = (int)(t % R); t /= R;
    int pw = (int)(t % gw); t /= gw;
    int ph = (int)(t % gh);
    int n = (int)(t / gh);
    // a source row holds W*C elements = gw * run_chunks chunks
    size_t src = (((size_t)n * H + (size_t)ph * R + r) * gw + pw) * run_chunks + ch;
    out[idx] = x[src];
}

// ---- class token + position embedding: out[n][0] = cls + pos[0]; out[n][1+i] = x[n][i] + pos[1+i] -----------------
__global__ __launch_bounds__(256) void tokens_kernel(const uint4* __restrict__ x, const uint4* __restrict__ cls,
                                                     const uint4* __restrict__ pos, uint4* __restrict__ out, int N, int T, int D8)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)N * T * D8;
    if (idx >= total) return;
    int c = (int)(idx % D8);
    size_t r = idx / D8;
    int t = (int)(r % T);
    int n = (int)(r / T);
    uint4 a = t == 0 ? cls[c] : x[((size_t)n * (T - 1) + (t - 1)) * D8 + c];
    uint4 p = pos[(size_t)t * D8 + c];
    uint4 o;
    o.x = pack_bf16(bf16_lo(a.x) + bf16_lo(p.x), bf16_hi(a.x) + bf16_hi(p.x));
    o.y = pack_bf16(bf16_lo(a.y) + bf16_lo(p.y), bf16_hi(a.y) + bf16_hi(p.y));
    o.z = pack_bf16(bf16_lo(a.z) + bf16_lo(p.z), bf16_hi(a.z) + bf16_hi(p.z));
    o.w = pack_bf16(bf16_lo(a.w) + bf16_lo(p.w), bf16_hi(a.w) + bf16_hi(p.w));
    out[idx] = o;
}

// ---- layer norm over channels, one wavefront per token, the token held in registers ---------------------------------
constexpr int kLnMaxPairs = 16;     // D <= 64 lanes * 2 * 16 = 2048
__global__ __launch_bounds__(256) void layernorm_kernel(const uint32_t* __restrict__ x, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, uint32_t* __restrict__ y, int rows,
                                                        int D2 /* pairs per token */)
{
    int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    int lane = threadIdx.x & 63;
    const uint32_t* xp = x + (size_t)row * D2;
    float v[2 * kLnMaxPairs];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < kLnMaxPairs; ++j) {
        int c = lane + 64 * j;
        uint32_t w = c < D2 ? xp[c] : 0u;
        v[2 * j] = bf16_lo(w);
        v[2 * j + 1] = bf16_hi(w);
        sum += v[2 * j] + v[2 * j + 1];
    }
    const float inv_d = 1.f / (float)(2 * D2);
    const float mean = wave_sum(sum) * inv_d;
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < kLnMaxPairs; ++j) {
        if (lane + 64 * j < D2) {
            float a = v[2 * j] - mean, b = v[2 * j + 1] - mean;
            sq += a * a + b * b;
        }
    }
    const float rstd = rsqrtf(wave_sum(sq) * inv_d + 1e-6f);
#pragma unroll
    for (int j = 0; j < kLnMaxPairs; ++j) {
        int c = lane + 64 * j;
        if (c < D2) {
            float2 g = *(const float2*)(gamma + 2 * c), b = *(const float2*)(beta + 2 * c);
            y[(size_t)row * D2 + c] = pack_bf16((v[2 * j] - mean) * rstd * g.x + b.x, (v[2 * j + 1] - mean) * rstd * g.y + b.y);
        }
    }
}

// ---- attention, one workgroup per (head, request), head width 64, up to 224 tokens --------------------------------
// Scores are computed transposed, S^T = K Q^T, with the key fragment as the first matrix-core operand: a lane then
// owns ONE query (column l%32) and, per 32-key block, the keys 8*(v/4) + 4*(l/32) + v%4.  Softmax statistics of a
// query therefore live in two lanes (l and l^32), and the exponentials, rounded to bf16, are already laid out as the
// second operand of the next product O^T = V^T P^T (keys may be visited in any order as long as V^T uses the same
// one), so the probabilities never leave registers.  A lane ends with 4 consecutive head channels of its query per
// accumulator quad and stores 8 bytes at a time.
// Numerics: scores in fp32, e = exp(s - max), probabilities p = e / sum(e) rounded to bf16 (they are a tensor of their
// own in storage precision), output = sum_j p_j v_j accumulated in fp32 and rounded to bf16.
constexpr int kDh = 64;
constexpr int kMaxKeyBlocks = 7;
constexpr int kKStride = kDh + 8;                 // K tile row stride (elements): conflict-free 16-byte reads
constexpr int kVStride = kMaxKeyBlocks * 32 + 8;  // V^T row stride
__global__ __launch_bounds__(256) void attention_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ out, int T,
                                                        int D, float scale)
{
    __shared__ __attribute__((aligned(16))) uint16_t Kl[kMaxKeyBlocks * 32 * kKStride];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[kDh * kVStride];
    const int head = blockIdx.x, n = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int TB = (T + 31) / 32;
    const size_t row_stride = (size_t)3 * D;
    const uint16_t* base = qkv + (size_t)n * T * row_stride + (size_t)head * kDh;

    // K as it is, V transposed; two tokens per thread so that the transposed stores are 4 bytes (token pairs)
    for (int c = tid; c < TB * 16 * 8; c += 256) {
        const int t = (c >> 3) * 2, part = c & 7;
        uint4 kv[2], vv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            kv[j] = make_uint4(0, 0, 0, 0);
            vv[j] = make_uint4(0, 0, 0, 0);
            if (t + j < T) {
                kv[j] = *(const uint4*)(base + (size_t)(t + j) * row_stride + D + part * 8);
                vv[j] = *(const uint4*)(base + (size_t)(t + j) * row_stride + 2 * D + part * 8);
            }
            *(uint4*)(Kl + (t + j) * kKStride + part * 8) = kv[j];
        }
        const uint32_t w0[4] = {vv[0].x, vv[0].y, vv[0].z, vv[0].w}, w1[4] = {vv[1].x, vv[1].y, vv[1].z, vv[1].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(uint32_t*)(Vt + (part * 8 + 2 * i) * kVStride + t) = (w0[i] & 0xFFFFu) | (w1[i] << 16);
            *(uint32_t*)(Vt + (part * 8 + 2 * i + 1) * kVStride + t) = (w0[i] >> 16) | (w1[i] & 0xFFFF0000u);
        }
    }
    __syncthreads();

    const int l32 = lane & 31, half = lane >> 5;
    const float scale2 = scale * 1.44269504088896340736f;
    for (int qb = wid; qb < TB; qb += 4) {
        const int query = qb * 32 + l32;
        bf16x8 qf[kDh / 16];
#pragma unroll
        for (int ks = 0; ks < kDh / 16; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (query < T) v = *(const uint4*)(base + (size_t)query * row_stride + ks * 16 + half * 8);
            qf[ks] = __builtin_bit_cast(bf16x8, v);
        }
        f32x16 sc[kMaxKeyBlocks];
        float m = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < kMaxKeyBlocks; ++kb) {
            if (kb < TB) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[kb][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < kDh / 16; ++ks) {
                    bf16x8 kf = *(const bf16x8*)(Kl + (kb * 32 + l32) * kKStride + ks * 16 + half * 8);
                    sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc[kb], 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int key = kb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    float s = key < T ? sc[kb][v] * scale2 : -INFINITY;       // scores in units of ln 2
                    sc[kb][v] = s;
                    m = fmaxf(m, s);
                }
            }
        }
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        float lsum = 0.f;
        uint32_t pw[kMaxKeyBlocks][8];          // bf16 pairs: [kb][2*g + j/2] = keys 8g + 4*half + (j, j+1)
#pragma unroll
        for (int kb = 0; kb < kMaxKeyBlocks; ++kb) {
            if (kb < TB) {
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    // 2^x on the transcendental unit (one instruction; exp(s - max) = 2^((s - max) / ln 2))
                    float e0 = __builtin_amdgcn_exp2f(sc[kb][v] - m), e1 = __builtin_amdgcn_exp2f(sc[kb][v + 1] - m);
                    lsum += e0 + e1;
                    sc[kb][v] = e0;
                    sc[kb][v + 1] = e1;
                }
            }
        }
        lsum += __shfl_xor(lsum, 32, 64);
        const float inv = 1.f / lsum;
#pragma unroll
        for (int kb = 0; kb < kMaxKeyBlocks; ++kb) {
            if (kb < TB) {
#pragma unroll
                for (int v = 0; v < 16; v += 2) pw[kb][v >> 1] = pack_bf16(sc[kb][v] * inv, sc[kb][v + 1] * inv);
            }
        }

        f32x16 oacc[kDh / 32];
#pragma unroll
        for (int db = 0; db < kDh / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
#pragma unroll
        for (int kb = 0; kb < kMaxKeyBlocks; ++kb) {
            if (kb < TB) {
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {          // 16 keys per matrix-core step: quads g = 2*t2 and 2*t2 + 1
                    const int g = 2 * t2;
                    uint4 pv = make_uint4(pw[kb][2 * g], pw[kb][2 * g + 1], pw[kb][2 * g + 2], pw[kb][2 * g + 3]);
                    bf16x8 pf = __builtin_bit_cast(bf16x8, pv);
#pragma unroll
                    for (int db = 0; db < kDh / 32; ++db) {
                        const uint16_t* vp = Vt + (db * 32 + l32) * kVStride + kb * 32 + 4 * half;
                        uint2 a = *(const uint2*)(vp + 8 * g), b = *(const uint2*)(vp + 8 * (g + 1));
                        bf16x8 vf = __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[db], 0, 0, 0);
                    }
                }
            }
        }
        if (query < T) {
            uint16_t* op = out + ((size_t)n * T + query) * D + (size_t)head * kDh;
#pragma unroll
            for (int db = 0; db < kDh / 32; ++db)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    uint2 o;
                    o.x = pack_bf16(oacc[db][4 * gq], oacc[db][4 * gq + 1]);
                    o.y = pack_bf16(oacc[db][4 * gq + 2], oacc[db][4 * gq + 3]);
                    *(uint2*)(op + db * 32 + 8 * gq + 4 * half) = o;
                }
        }
    }
}

}  // namespace

hipError_t patchify(const void* x, void* out, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, hipStream_t stream)
{
    if (R <= 0 || S <= 0 || H % R || W % S || (S * C * 2) % 16) return hipErrorInvalidValue;
    int gh = H / R, gw = W / S, run_chunks = S * C * 2 / 16;
    size_t total = (size_t)N * gh * gw * R * run_chunks;
    if (total == 0) return hipSuccess;
    size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(patchify_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)x, (uint4*)out, N, H, W, R, gh,
                       gw, run_chunks);
    return hipGetLastError();
}

hipError_t tokens(const void* x, const void* cls, const void* pos, void* out, int32_t N, int32_t T, int32_t D, hipStream_t stream)
{
    if (D % 8) return hipErrorInvalidValue;
    size_t total = (size_t)N * T * (D / 8);
    if (total == 0) return hipSuccess;
    size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tokens_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)x, (const uint4*)cls,
                       (const uint4*)pos, (uint4*)out, N, T, D / 8);
    return hipGetLastError();
}

hipError_t layernorm(const void* x, const float* gamma, const float* beta, void* y, int64_t rows, int32_t D, hipStream_t stream)
{
    if (D % 2 || D > 128 * kLnMaxPairs) return hipErrorInvalidValue;
    if (rows == 0) return hipSuccess;
    int64_t blocks = (rows + 3) / 4;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layernorm_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint32_t*)x, gamma, beta,
                       (uint32_t*)y, (int)rows, D / 2);
    return hipGetLastError();
}

bool attention_supported(int32_t T, int32_t D, int32_t heads)
{
    return heads > 0 && D == heads * kDh && T > 0 && T <= kMaxKeyBlocks * 32;
}

hipError_t attention(const void* qkv, void* out, int32_t N, int32_t T, int32_t D, int32_t heads, hipStream_t stream)
{
    if (!attention_supported(T, D, heads)) return hipErrorInvalidValue;
    if (N == 0) return hipSuccess;
    if (N > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attention_kernel, dim3(heads, N), dim3(256), 0, stream, (const uint16_t*)qkv, (uint16_t*)out, T, D,
                       1.0f / sqrtf((float)kDh));
    return hipGetLastError();
}

}  // namespace k
}  // namespace coe
