// gfx950 kernels: request arranging (regroup), plain convolution, max pool, routing head.
// Wavefronts are 64 lanes wide throughout.
#include <hip/hip_runtime.h>

#include <mutex>

#include "kernels.h"

namespace coe {
namespace k {

namespace {

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest even; NaN becomes a quiet NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float apply_act(float v, int act)
{
    if (act == 1) return v > 0.f ? v : 0.f;
    if (act == 2) return 0.5f * v * erfcf(-v * 0.70710678118654752440f);
    if (act == 3) return v / (1.f + expf(-v));
    return v;
}

// -------------------------------------------------------------------------------------------------------------
// regroup, index part
// -------------------------------------------------------------------------------------------------------------
// Pass 1: per-workgroup histogram of the pending requests' expert ids.
__global__ __launch_bounds__(kRegroupTile) void regroup_count_kernel(const int32_t* __restrict__ cur, int32_t n,
                                                                     int32_t E, int32_t* __restrict__ blockhist)
{
    extern __shared__ int32_t hist[];
    for (int e = threadIdx.x; e < E; e += kRegroupTile) hist[e] = 0;
    __syncthreads();
    int i = blockIdx.x * kRegroupTile + threadIdx.x;
    if (i < n) {
        int key = cur[i];
        if (key >= 0 && key < E) atomicAdd(&hist[key], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kRegroupTile) blockhist[(size_t)blockIdx.x * E + e] = hist[e];
}

// inclusive prefix sum across one wavefront
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// Pass 2 (one workgroup): column sums of blockhist -> cnt; blockhist becomes the exclusive prefix down each column;
// exclusive scan of cnt over experts -> off.
constexpr int kScanThreads = 1024;
__global__ __launch_bounds__(kScanThreads) void regroup_scan_kernel(int32_t* __restrict__ blockhist, int32_t nblocks,
                                                                    int32_t E, int32_t* __restrict__ cnt,
                                                                    int32_t* __restrict__ off)
{
    __shared__ int32_t wave_tot[kScanThreads / kWave];
    __shared__ int32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    for (int base = 0; base < E; base += kScanThreads) {
        int e = base + threadIdx.x;
        int total = 0;
        if (e < E) {
            for (int b = 0; b < nblocks; ++b) {
                int t = blockhist[(size_t)b * E + e];
                blockhist[(size_t)b * E + e] = total;
                total += t;
            }
            cnt[e] = total;
        }
        int incl = wave_inclusive_scan(total);
        if (lane == kWave - 1) wave_tot[wid] = incl;
        __syncthreads();
        if (wid == 0) {
            int t = lane < kScanThreads / kWave ? wave_tot[lane] : 0;
            int s = wave_inclusive_scan(t);
            if (lane < kScanThreads / kWave) wave_tot[lane] = s - t;   // exclusive offset of each wave
        }
        __syncthreads();
        int c = carry;
        int excl = c + wave_tot[wid] + incl - total;
        if (e < E) off[e] = excl;
        __syncthreads();
        if (threadIdx.x == kScanThreads - 1) carry = excl + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) off[E] = carry;
}

// Pass 3: stable scatter.  Position of request i = off[key] + (requests with that key in earlier workgroups)
// + (in earlier wavefronts of this workgroup) + (in lower lanes of this wavefront).
__global__ __launch_bounds__(kRegroupTile) void regroup_scatter_kernel(const int32_t* __restrict__ cur, int32_t n,
                                                                       int32_t E, const int32_t* __restrict__ blockhist,
                                                                       const int32_t* __restrict__ off,
                                                                       int32_t* __restrict__ perm,
                                                                       int32_t* __restrict__ inv)
{
    extern __shared__ int32_t wcount[];   // [waves][E]
    constexpr int kWaves = kRegroupTile / kWave;
    for (int j = threadIdx.x; j < kWaves * E; j += kRegroupTile) wcount[j] = 0;
    __syncthreads();
    int i = blockIdx.x * kRegroupTile + threadIdx.x;
    int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    int key = -1;
    if (i < n) {
        key = cur[i];
        if (key < 0 || key >= E) key = -1;
    }
    unsigned long long lt_mask = lane == 0 ? 0ull : (~0ull >> (kWave - lane));
    unsigned long long remaining = __ballot(key >= 0);
    int rank = 0;
    while (remaining) {
        int leader = __ffsll((long long)remaining) - 1;
        int lk = __shfl(key, leader, kWave);
        unsigned long long peers = __ballot(key == lk);
        if (key == lk) {
            rank = __popcll(peers & lt_mask);
            if (lane == leader) wcount[wid * E + lk] = __popcll(peers);
        }
        remaining &= ~peers;
    }
    __syncthreads();
    if (key >= 0) {
        int before = 0;
        for (int w = 0; w < wid; ++w) before += wcount[w * E + key];
        int pos = off[key] + blockhist[(size_t)blockIdx.x * E + key] + before + rank;
        perm[pos] = i;
        inv[i] = pos;
    } else if (i < n) {
        inv[i] = -1;
    }
}

// -------------------------------------------------------------------------------------------------------------
// regroup, activation part: coalesced row gather, 16 bytes per lane
// -------------------------------------------------------------------------------------------------------------
constexpr int kGatherThreads = 256;
template <typename V>
__global__ __launch_bounds__(kGatherThreads) void gather_rows_kernel(const V* __restrict__ src,
                                                                     const int32_t* __restrict__ perm,
                                                                     size_t row_vecs, V* __restrict__ dst)
{
    int row = blockIdx.x;
    const V* s = src + (size_t)perm[row] * row_vecs;
    V* d = dst + (size_t)row * row_vecs;
    for (size_t j = (size_t)blockIdx.y * kGatherThreads + threadIdx.x; j < row_vecs; j += (size_t)gridDim.y * kGatherThreads)
        d[j] = s[j];
}

// -------------------------------------------------------------------------------------------------------------
// plain convolution: one thread per output element, channels fastest
// -------------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void conv_direct_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                          const float* __restrict__ bias, const T* __restrict__ res,
                                                          T* __restrict__ y, ConvShape s)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)s.N * s.P * s.Q * s.K;
    if (idx >= total) return;
    int k = (int)(idx % s.K);
    size_t m = idx / s.K;
    int q = (int)(m % s.Q);
    int p = (int)((m / s.Q) % s.P);
    int n = (int)(m / ((size_t)s.Q * s.P));
    float acc = 0.f;
    for (int r = 0; r < s.R; ++r) {
        int ih = p * s.stride - s.pad + r;
        if (ih < 0 || ih >= s.H) continue;
        for (int t = 0; t < s.S; ++t) {
            int iw = q * s.stride - s.pad + t;
            if (iw < 0 || iw >= s.W) continue;
            const T* xp = x + (((size_t)n * s.H + ih) * s.W + iw) * s.C;
            const T* wp = w + (((size_t)k * s.R + r) * s.S + t) * s.C;
            for (int c = 0; c < s.C; ++c) acc = fmaf(Elem<T>::load(xp + c), Elem<T>::load(wp + c), acc);
        }
    }
    float v = acc + bias[k];
    if (res) v += Elem<T>::load(res + idx);
    Elem<T>::store(y + idx, apply_act(v, s.act));
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const T* __restrict__ x, T* __restrict__ y, int N, int H, int W,
                                                      int C, int R, int S, int stride, int pad, int P, int Q)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)N * P * Q * C;
    if (idx >= total) return;
    int c = (int)(idx % C);
    size_t m = idx / C;
    int q = (int)(m % Q);
    int p = (int)((m / Q) % P);
    int n = (int)(m / ((size_t)Q * P));
    float best = -INFINITY;
    for (int r = 0; r < R; ++r) {
        int ih = p * stride - pad + r;
        if (ih < 0 || ih >= H) continue;
        for (int t = 0; t < S; ++t) {
            int iw = q * stride - pad + t;
            if (iw < 0 || iw >= W) continue;
            best = fmaxf(best, Elem<T>::load(x + (((size_t)n * H + ih) * W + iw) * C + c));
        }
    }
    Elem<T>::store(y + idx, best);
}

// bf16 max pool, 8 channels (16 bytes) per lane.  bf16 order equals the order of the fp32 values, so the max is taken
// on the widened values and the winning pattern is stored unchanged.
__global__ __launch_bounds__(256) void maxpool_bf16x8_kernel(const uint4* __restrict__ x, uint4* __restrict__ y, int N, int H,
                                                             int W, int C8, int R, int S, int stride, int pad, int P, int Q)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)N * P * Q * C8;
    if (idx >= total) return;
    int c8 = (int)(idx % C8);
    size_t m = idx / C8;
    int q = (int)(m % Q);
    int p = (int)((m / Q) % P);
    int n = (int)(m / ((size_t)Q * P));
    float best[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) best[i] = -INFINITY;
    for (int r = 0; r < R; ++r) {
        int ih = p * stride - pad + r;
        if (ih < 0 || ih >= H) continue;
        for (int t = 0; t < S; ++t) {
            int iw = q * stride - pad + t;
            if (iw < 0 || iw >= W) continue;
            uint4 v = x[(((size_t)n * H + ih) * W + iw) * C8 + c8];
            uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                best[2 * i] = fmaxf(best[2 * i], __uint_as_float(wds[i] << 16));
                best[2 * i + 1] = fmaxf(best[2 * i + 1], __uint_as_float(wds[i] & 0xFFFF0000u));
            }
        }
    }
    uint4 o;
    o.x = (__float_as_uint(best[0]) >> 16) | (__float_as_uint(best[1]) & 0xFFFF0000u);
    o.y = (__float_as_uint(best[2]) >> 16) | (__float_as_uint(best[3]) & 0xFFFF0000u);
    o.z = (__float_as_uint(best[4]) >> 16) | (__float_as_uint(best[5]) & 0xFFFF0000u);
    o.w = (__float_as_uint(best[6]) >> 16) | (__float_as_uint(best[7]) & 0xFFFF0000u);
    y[idx] = o;
}

// -------------------------------------------------------------------------------------------------------------
// routing head: global average pool, FC, argmax over the routed classes, successor lookup
// -------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

constexpr int kHeadThreads = 256;

// logits of one request are in LDS: write them out, take the argmax over the routed classes (lowest index wins
// ties), look the successor up, append the expert to the request's path
__device__ __forceinline__ void route_tail(const float* logit, int ncls, int row, const RouteArgs& r)
{
    int slot = r.slot ? r.slot[row] : row;
    for (int j = threadIdx.x; j < r.logits_stride; j += kHeadThreads)
        r.logits[(size_t)slot * r.logits_stride + j] = j < ncls ? logit[j] : 0.f;
    if (threadIdx.x == 0 && r.cur) {
        int nxt = -1;
        if (r.n_route > 0) {
            int best = 0;
            for (int j = 1; j < r.n_route; ++j)
                if (logit[j] > logit[best]) best = j;      // strict: the lowest index wins ties
            nxt = r.succ[best];
        }
        int d = r.depth[slot];
        if (d < r.max_stages) r.path[(size_t)slot * r.max_stages + d] = r.expert;
        r.depth[slot] = d + 1;
        r.cur[slot] = nxt;
    }
}

// 16-byte loads in the pooling phase: bf16 tensors whose channel count is a multiple of 8 with C/8 dividing the block
template <typename T> __host__ __device__ inline bool head_vector_path(int C)
{
    return sizeof(T) == 2 && C >= 64 && C % 8 == 0 && kHeadThreads % (C / 8) == 0;
}

template <typename T>
__global__ __launch_bounds__(kHeadThreads) void head_gap_fc_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                                   const float* __restrict__ b, int HW, int C, int ncls,
                                                                   RouteArgs r, GroupTable gt, GroupRoutes gr, uint32_t off_w,
                                                                   uint32_t off_b)
{
    extern __shared__ float smem[];          // feat[C] | part[groups][C] | logit[ncls]
    int row = blockIdx.x;
    if (gt.n > 0) {
        // grouped launch: this request's group decides the FC weights and the routing rule
        int g = 0;
        while (g + 1 < gt.n && row >= gt.first_row[g + 1]) ++g;
        const char* base = (const char*)gt.weights[g];
        w = (const T*)(base + off_w);
        b = (const float*)(base + off_b);
        r.expert = gr.expert[g];
        r.succ = r.succ + gr.succ_off[g];
        r.n_route = gr.n_route[g];
        if (r.slot) r.slot = r.slot + (gr.slot_off[g] - gt.first_row[g]);
    }
    const T* xp = x + (size_t)row * HW * C;
    int groups = C < kHeadThreads ? kHeadThreads / C : 1;      // position groups when there are few channels
    if (head_vector_path<T>(C)) groups = kHeadThreads / (C / 8);
    float* feat = smem;
    float* part = smem + C;
    float* logit = part + (size_t)groups * C;
    // phase 1: per-channel sums, lanes run along channels (contiguous in NHWC)
    if (head_vector_path<T>(C)) {
        // bf16, C a multiple of 8 with C/8 dividing the block: 16-byte loads, 8 channels per thread, the positions
        // dealt round-robin to 256 / (C/8) thread groups whose partial sums meet in LDS
        const int cpb = C / 8, G = kHeadThreads / cpb;
        const int chunk = threadIdx.x % cpb, pg = threadIdx.x / cpb;
        float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int i = pg; i < HW; i += G) {
            const uint4 v = *(const uint4*)((const uint16_t*)xp + (size_t)i * C + chunk * 8);
            const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a8[2 * e] += __uint_as_float(wds[e] << 16);
                a8[2 * e + 1] += __uint_as_float(wds[e] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[pg * C + chunk * 8 + e] = a8[e];
        __syncthreads();
        for (int c2 = threadIdx.x; c2 < C; c2 += kHeadThreads) {
            float a = 0.f;
            for (int g2 = 0; g2 < G; ++g2) a += part[g2 * C + c2];
            feat[c2] = a / (float)HW;
        }
    } else if (groups > 1) {
        int g = threadIdx.x / C, c = threadIdx.x % C;
        if (g < groups) {
            float a = 0.f;
            for (int i = g; i < HW; i += groups) a += Elem<T>::load(xp + (size_t)i * C + c);
            part[g * C + c] = a;
        }
        __syncthreads();
        for (int c2 = threadIdx.x; c2 < C; c2 += kHeadThreads) {
            float a = 0.f;
            for (int g2 = 0; g2 < groups; ++g2) a += part[g2 * C + c2];
            feat[c2] = a / (float)HW;
        }
    } else {
        for (int c = threadIdx.x; c < C; c += kHeadThreads) {
            float a = 0.f;
            for (int i = 0; i < HW; ++i) a += Elem<T>::load(xp + (size_t)i * C + c);
            feat[c] = a / (float)HW;
        }
    }
    __syncthreads();
    // phase 2: one wavefront per class, lanes along the feature dimension, wavefront reduction
    int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    if (head_vector_path<T>(C)) {
        // 16-byte weight loads, four classes per wavefront in flight: with one 2-byte load per multiply-add the loop is
        // a chain of ~C/64 * classes/4 global-load latencies per wavefront (200 us for a 2048 x 64 head)
        constexpr int kWaves = kHeadThreads / kWave;
        const uint16_t* wq = (const uint16_t*)w;
        const int cpb = C / 8;
        for (int j0 = wid; j0 < ncls; j0 += 4 * kWaves) {
            float a[4] = {0.f, 0.f, 0.f, 0.f};
            for (int ch = lane; ch < cpb; ch += kWave) {
                uint4 wv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = j0 + u * kWaves;
                    wv[u] = j < ncls ? *(const uint4*)(wq + (size_t)j * C + ch * 8) : make_uint4(0, 0, 0, 0);
                }
                const float4 f0 = *(const float4*)(feat + ch * 8), f1 = *(const float4*)(feat + ch * 8 + 4);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = fmaf(f0.x, __uint_as_float(wv[u].x << 16), a[u]);
                    a[u] = fmaf(f0.y, __uint_as_float(wv[u].x & 0xFFFF0000u), a[u]);
                    a[u] = fmaf(f0.z, __uint_as_float(wv[u].y << 16), a[u]);
                    a[u] = fmaf(f0.w, __uint_as_float(wv[u].y & 0xFFFF0000u), a[u]);
                    a[u] = fmaf(f1.x, __uint_as_float(wv[u].z << 16), a[u]);
                    a[u] = fmaf(f1.y, __uint_as_float(wv[u].z & 0xFFFF0000u), a[u]);
                    a[u] = fmaf(f1.z, __uint_as_float(wv[u].w << 16), a[u]);
                    a[u] = fmaf(f1.w, __uint_as_float(wv[u].w & 0xFFFF0000u), a[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * kWaves;
                const float t = wave_sum(a[u]);
                if (lane == 0 && j < ncls) logit[j] = t + b[j];
            }
        }
    } else {
        for (int j = wid; j < ncls; j += kHeadThreads / kWave) {
            float a = 0.f;
            for (int c = lane; c < C; c += kWave) a = fmaf(feat[c], Elem<T>::load(w + (size_t)j * C + c), a);
            a = wave_sum(a);
            if (lane == 0) logit[j] = a + b[j];
        }
    }
    __syncthreads();
    // phase 3: write logits, pick the route
    route_tail(logit, ncls, row, r);
}

// class-token head: layer norm of token 0 (rounded to bf16 like every stored activation), FC, routing
__global__ __launch_bounds__(kHeadThreads) void head_cls_kernel(const uint16_t* __restrict__ x, const float* __restrict__ gamma,
                                                                const float* __restrict__ beta, const uint16_t* __restrict__ w,
                                                                const float* __restrict__ b, int T, int D, int ncls, RouteArgs r)
{
    extern __shared__ float smem[];          // feat[D] | red[8] | logit[ncls]
    float* feat = smem;
    float* red = smem + D;
    float* logit = red + 8;
    const int row = blockIdx.x;
    const uint16_t* xp = x + (size_t)row * T * D;     // token 0
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    float sum = 0.f;
    for (int c = threadIdx.x; c < D; c += kHeadThreads) { float v = bf16_to_f32(xp[c]); feat[c] = v; sum += v; }
    sum = wave_sum(sum);
    if (lane == 0) red[wid] = sum;
    __syncthreads();
    const float mean = (red[0] + red[1] + red[2] + red[3]) / (float)D;
    float sq = 0.f;
    for (int c = threadIdx.x; c < D; c += kHeadThreads) { float d = feat[c] - mean; sq += d * d; }
    sq = wave_sum(sq);
    if (lane == 0) red[4 + wid] = sq;
    __syncthreads();
    const float rstd = rsqrtf((red[4] + red[5] + red[6] + red[7]) / (float)D + 1e-6f);
    for (int c = threadIdx.x; c < D; c += kHeadThreads)
        feat[c] = bf16_to_f32(f32_to_bf16((feat[c] - mean) * rstd * gamma[c] + beta[c]));
    __syncthreads();
    for (int j = wid; j < ncls; j += kHeadThreads / kWave) {
        float a = 0.f;
        for (int c = lane; c < D; c += kWave) a = fmaf(feat[c], bf16_to_f32(w[(size_t)j * D + c]), a);
        a = wave_sum(a);
        if (lane == 0) logit[j] = a + b[j];
    }
    __syncthreads();
    route_tail(logit, ncls, row, r);
}

// -------------------------------------------------------------------------------------------------------------
// detector-shaped experts: channel concatenation, nearest-neighbour upsampling, detection read-out
// -------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void concat_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b, uint4* __restrict__ out,
                                                     size_t rows, int A8, int B8)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int C8 = A8 + B8;
    if (idx >= rows * C8) return;
    const size_t r = idx / C8;
    const int c = (int)(idx % C8);
    out[idx] = c < A8 ? a[r * A8 + c] : b[r * B8 + (c - A8)];
}

__global__ __launch_bounds__(256) void upsample2_kernel(const uint4* __restrict__ x, uint4* __restrict__ out, int N, int H, int W, int C8)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)N * 4 * H * W * C8;
    if (idx >= total) return;
    const int c = (int)(idx % C8);
    size_t m = idx / C8;
    const int w = (int)(m % (2 * W)); m /= 2 * W;
    const int h = (int)(m % (2 * H));
    const int n = (int)(m / (2 * H));
    out[idx] = x[(((size_t)n * H + h / 2) * W + w / 2) * C8 + c];
}

__device__ __forceinline__ float sigmoid_f(float v) { return 1.f / (1.f + expf(-v)); }

// one workgroup per request.  A box is box_len = 5 + classes consecutive elements; thread t owns element t % box_len of
// boxes t / box_len, + per_iter, ... (per_iter = boxes the workgroup covers at once), so consecutive threads read consecutive
// elements and a thread's class never changes: it keeps its best score in a register.  The per_iter partial maxima of a
// class meet in LDS at the end.  Scores are products of two sigmoids, hence positive, and the maximum does not depend on
// the order it is taken in.
constexpr int kDetMaxClasses = 251;            // box_len <= kHeadThreads
__global__ __launch_bounds__(kHeadThreads) void head_det_kernel(const uint16_t* __restrict__ m0, int hw0, const uint16_t* __restrict__ m1,
                                                                int hw1, int anchors, int ncls, RouteArgs r)
{
    __shared__ float part[kHeadThreads];
    __shared__ float logit[kHeadThreads];
    const int row = blockIdx.x;
    const int box_len = 5 + ncls, stride = anchors * box_len;
    const int per_iter = kHeadThreads / box_len;
    const int j = threadIdx.x % box_len, b0 = threadIdx.x / box_len;
    float best = 0.f;
    if (b0 < per_iter && j >= 5) {
        for (int map = 0; map < 2; ++map) {
            const uint16_t* mp = map == 0 ? m0 : m1;
            const int hw = map == 0 ? hw0 : hw1;
            if (!mp) continue;
            const uint16_t* base = mp + (size_t)row * hw * stride;
            const int nbox = hw * anchors;                           // boxes of one position are consecutive
            // four boxes per trip: eight loads in flight per thread (a launch may hold only a few workgroups per compute unit)
            int bx = b0;
            for (; bx + 3 * per_iter < nbox; bx += 4 * per_iter) {
                uint16_t o[4], v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint16_t* box = base + (size_t)(bx + u * per_iter) * box_len;
                    o[u] = box[4];
                    v[u] = box[j];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) best = fmaxf(best, sigmoid_f(bf16_to_f32(o[u])) * sigmoid_f(bf16_to_f32(v[u])));
            }
            for (; bx < nbox; bx += per_iter) {
                const uint16_t* box = base + (size_t)bx * box_len;
                best = fmaxf(best, sigmoid_f(bf16_to_f32(box[4])) * sigmoid_f(bf16_to_f32(box[j])));
            }
        }
    }
    part[threadIdx.x] = best;
    __syncthreads();
    for (int c = threadIdx.x; c < ncls; c += kHeadThreads) {
        float m = 0.f;
        for (int b = 0; b < per_iter; ++b) m = fmaxf(m, part[b * box_len + 5 + c]);
        logit[c] = m;
    }
    __syncthreads();
    route_tail(logit, ncls, row, r);
}

}  // namespace

// -------------------------------------------------------------------------------------------------------------
// launchers
// -------------------------------------------------------------------------------------------------------------
hipError_t regroup_index(const int32_t* cur, int32_t n, int32_t E, int32_t* cnt, int32_t* off, int32_t* perm,
                         int32_t* inv, int32_t* blockhist, hipStream_t stream)
{
    if (n < 0 || E <= 0 || E > kRegroupMaxExperts) return hipErrorInvalidValue;
    int nblocks = (n + kRegroupTile - 1) / kRegroupTile;
    if (nblocks > 0)
        hipLaunchKernelGGL(regroup_count_kernel, dim3(nblocks), dim3(kRegroupTile), sizeof(int32_t) * E, stream, cur, n, E,
                           blockhist);
    hipLaunchKernelGGL(regroup_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, blockhist, nblocks, E, cnt, off);
    if (nblocks > 0)
        hipLaunchKernelGGL(regroup_scatter_kernel, dim3(nblocks), dim3(kRegroupTile),
                           sizeof(int32_t) * E * (kRegroupTile / kWave), stream, cur, n, E, blockhist, off, perm, inv);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------------------------
// regroup for callers that cannot allocate: the per-workgroup histograms live in a static device array instead of a
// buffer the caller or a context owns.  Every GPU the library runs on holds its own copy of the array (4 MiB) until the
// process ends; in host code the array's name is only a handle for hipGetSymbolAddress, the address a kernel can use is
// looked up once per device and kept.
// -------------------------------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[kRegroupStaticInts];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {nullptr};
}  // namespace

hipError_t regroup_index_static(const int32_t* cur, int32_t n, int32_t E, int32_t* cnt, int32_t* off, int32_t* perm,
                                int32_t* inv, hipStream_t stream)
{
    if (n < 0 || E <= 0 || E > kRegroupMaxExperts) return hipErrorInvalidValue;
    const long long nblocks = ((long long)n + kRegroupTile - 1) / kRegroupTile;
    if (nblocks * E > (long long)kRegroupStaticInts) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int32_t* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // this device's copy of the array
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = (int32_t*)p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // every histogram entry the scan and the scatter read is written by the count kernel of the same call: nothing has to
    // start at zero
    return regroup_index(cur, n, E, cnt, off, perm, inv, ptr, stream);
}

__global__ void group_heads_kernel(const int32_t* __restrict__ perm, const int32_t* __restrict__ off,
                                   const int32_t* __restrict__ cnt, int32_t E, int32_t* __restrict__ heads)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) heads[e] = cnt[e] > 0 ? perm[off[e]] : -1;
}

hipError_t group_heads(const int32_t* perm, const int32_t* off, const int32_t* cnt, int32_t E, int32_t* heads,
                       hipStream_t stream)
{
    if (E <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(group_heads_kernel, dim3((E + 255) / 256), dim3(256), 0, stream, perm, off, cnt, E, heads);
    return hipGetLastError();
}

hipError_t gather_rows(const void* src, const int32_t* perm, int32_t n_rows, size_t row_bytes, void* dst,
                       hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    if (row_bytes % 4) return hipErrorInvalidValue;
    if (row_bytes % 16 == 0) {
        size_t vecs = row_bytes / 16;
        int gy = (int)((vecs + kGatherThreads * 8 - 1) / (kGatherThreads * 8));
        if (gy < 1) gy = 1;
        if (gy > 64) gy = 64;
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(n_rows, gy), dim3(kGatherThreads), 0, stream,
                           (const uint4*)src, perm, vecs, (uint4*)dst);
    } else {
        size_t vecs = row_bytes / 4;
        int gy = (int)((vecs + kGatherThreads * 8 - 1) / (kGatherThreads * 8));
        if (gy < 1) gy = 1;
        if (gy > 64) gy = 64;
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(n_rows, gy), dim3(kGatherThreads), 0, stream,
                           (const uint32_t*)src, perm, vecs, (uint32_t*)dst);
    }
    return hipGetLastError();
}

hipError_t conv_direct(int dtype, const void* x, const void* w, const float* bias, const void* res, void* y,
                       const ConvShape& s, hipStream_t stream)
{
    size_t total = (size_t)s.N * s.P * s.Q * s.K;
    if (total == 0) return hipSuccess;
    size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (dtype == 1)
        hipLaunchKernelGGL(conv_direct_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)x,
                           (const uint16_t*)w, bias, (const uint16_t*)res, (uint16_t*)y, s);
    else
        hipLaunchKernelGGL(conv_direct_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)x,
                           (const float*)w, bias, (const float*)res, (float*)y, s);
    return hipGetLastError();
}

hipError_t maxpool(int dtype, const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S,
                   int32_t stride, int32_t pad, int32_t P, int32_t Q, hipStream_t stream)
{
    size_t total = (size_t)N * P * Q * C;
    if (total == 0) return hipSuccess;
    if (dtype == 1 && C % 8 == 0) {
        size_t blocks8 = (total / 8 + 255) / 256;
        if (blocks8 > 0x7FFFFFFFull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(maxpool_bf16x8_kernel, dim3((unsigned)blocks8), dim3(256), 0, stream, (const uint4*)x, (uint4*)y, N,
                           H, W, C / 8, R, S, stride, pad, P, Q);
        return hipGetLastError();
    }
    size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (dtype == 1)
        hipLaunchKernelGGL(maxpool_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)x,
                           (uint16_t*)y, N, H, W, C, R, S, stride, pad, P, Q);
    else
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)x, (float*)y,
                           N, H, W, C, R, S, stride, pad, P, Q);
    return hipGetLastError();
}

hipError_t head_gap_fc(int dtype, const void* x, const void* w, const float* b, int32_t N, int32_t HW, int32_t C,
                       int32_t ncls, const RouteArgs& r, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    int groups = C < kHeadThreads ? kHeadThreads / C : 1;
    if (dtype == 1 && head_vector_path<uint16_t>(C)) groups = kHeadThreads / (C / 8);      // partial sums of the 16-byte path
    size_t smem = sizeof(float) * ((size_t)C + (size_t)groups * C + (size_t)ncls);
    if (smem > 60 * 1024) return hipErrorInvalidValue;
    const GroupTable gt{};
    const GroupRoutes gr{};
    if (dtype == 1)
        hipLaunchKernelGGL(head_gap_fc_kernel<uint16_t>, dim3(N), dim3(kHeadThreads), smem, stream, (const uint16_t*)x,
                           (const uint16_t*)w, b, HW, C, ncls, r, gt, gr, 0u, 0u);
    else
        hipLaunchKernelGGL(head_gap_fc_kernel<float>, dim3(N), dim3(kHeadThreads), smem, stream, (const float*)x,
                           (const float*)w, b, HW, C, ncls, r, gt, gr, 0u, 0u);
    return hipGetLastError();
}

hipError_t head_gap_fc_grouped(int dtype, const void* x, const GroupTable& groups, size_t off_w, size_t off_b, int32_t N,
                               int32_t HW, int32_t C, int32_t ncls, const RouteArgs& r, const GroupRoutes& routes,
                               hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    if (groups.n <= 0 || groups.n > kMaxGroups || groups.first_row[0] != 0 || groups.first_row[groups.n] != N ||
        off_w > 0x7FFFFFFFull || off_b > 0x7FFFFFFFull)
        return hipErrorInvalidValue;
    int pgroups = C < kHeadThreads ? kHeadThreads / C : 1;
    if (dtype == 1 && head_vector_path<uint16_t>(C)) pgroups = kHeadThreads / (C / 8);
    size_t smem = sizeof(float) * ((size_t)C + (size_t)pgroups * C + (size_t)ncls);
    if (smem > 60 * 1024) return hipErrorInvalidValue;
    if (dtype == 1)
        hipLaunchKernelGGL(head_gap_fc_kernel<uint16_t>, dim3(N), dim3(kHeadThreads), smem, stream, (const uint16_t*)x,
                           (const uint16_t*)nullptr, (const float*)nullptr, HW, C, ncls, r, groups, routes, (uint32_t)off_w,
                           (uint32_t)off_b);
    else
        hipLaunchKernelGGL(head_gap_fc_kernel<float>, dim3(N), dim3(kHeadThreads), smem, stream, (const float*)x,
                           (const float*)nullptr, (const float*)nullptr, HW, C, ncls, r, groups, routes, (uint32_t)off_w,
                           (uint32_t)off_b);
    return hipGetLastError();
}

hipError_t concat_channels(const void* a, const void* b, void* out, int64_t rows, int32_t Ca, int32_t Cb, hipStream_t stream)
{
    if (Ca <= 0 || Cb <= 0 || Ca % 8 || Cb % 8 || rows < 0) return hipErrorInvalidValue;
    const size_t total = (size_t)rows * ((Ca + Cb) / 8);
    if (total == 0) return hipSuccess;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(concat_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)a, (const uint4*)b, (uint4*)out,
                       (size_t)rows, Ca / 8, Cb / 8);
    return hipGetLastError();
}

hipError_t upsample2(const void* x, void* out, int32_t N, int32_t H, int32_t W, int32_t C, hipStream_t stream)
{
    if (C <= 0 || C % 8 || H <= 0 || W <= 0 || N < 0) return hipErrorInvalidValue;
    const size_t total = (size_t)N * 4 * H * W * (C / 8);
    if (total == 0) return hipSuccess;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(upsample2_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)x, (uint4*)out, N, H, W, C / 8);
    return hipGetLastError();
}

hipError_t head_det(const void* m0, int32_t hw0, const void* m1, int32_t hw1, int32_t N, int32_t anchors, int32_t ncls,
                    const RouteArgs& r, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    if (!m0 || hw0 <= 0 || anchors <= 0 || ncls <= 0 || ncls > kDetMaxClasses || (m1 && hw1 <= 0)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(head_det_kernel, dim3(N), dim3(kHeadThreads), 0, stream, (const uint16_t*)m0, hw0, (const uint16_t*)m1, hw1,
                       anchors, ncls, r);
    return hipGetLastError();
}

hipError_t head_cls(const void* x, const float* gamma, const float* beta, const void* w, const float* b, int32_t N, int32_t T,
                    int32_t D, int32_t ncls, const RouteArgs& r, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    size_t smem = sizeof(float) * ((size_t)D + 8 + (size_t)ncls);
    if (smem > 60 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(head_cls_kernel, dim3(N), dim3(kHeadThreads), smem, stream, (const uint16_t*)x, gamma, beta,
                       (const uint16_t*)w, b, T, D, ncls, r);
    return hipGetLastError();
}

}  // namespace k
}  // namespace coe
