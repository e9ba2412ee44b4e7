// Launch interface of the gfx950 kernels.  Every function enqueues on `stream` and returns the launch status;
// shapes are validated by the caller (the stage driver), which owns all buffers.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

namespace coe {
namespace k {

constexpr int kRegroupTile = 256;     // requests per workgroup in the regroup kernels
constexpr int kRegroupMaxExperts = 2048;

// Routing epilogue arguments.  slot == nullptr: row i writes logits row i and nothing else (plain forward).
struct RouteArgs {
    const int32_t* slot;   // [n] request-store slot of each row of this batch (device)
    int32_t expert;        // expert that ran
    const int32_t* succ;   // device successor list of that expert
    int32_t n_route;       // its length (0: every request is final)
    int32_t* cur;          // [slots] next expert per request, -1 = final
    int32_t* depth;        // [slots] stages executed so far
    int32_t* path;         // [slots][max_stages]
    int32_t max_stages;
    float* logits;         // [slots or n][logits_stride]
    int32_t logits_stride;
};

// Request arranging, index part: per-expert histogram, prefix scan, stable scatter of request indices.
// cur[n]: expert id in [0,E) = pending, anything else = not pending.  cnt[E], off[E+1], perm[<=n], inv[n].
// blockhist: scratch of ceil(n/kRegroupTile)*E int32.
hipError_t regroup_index(const int32_t* cur, int32_t n, int32_t E, int32_t* cnt, int32_t* off, int32_t* perm,
                         int32_t* inv, int32_t* blockhist, hipStream_t stream);

// The same with the histogram scratch in a static device array of kRegroupStaticInts int32 (no allocation anywhere on the
// path): hipErrorInvalidValue when ceil(n / kRegroupTile) * E exceeds it.  Runs on the current device; calls on one device
// share the array, so calls that overlap there race.
constexpr int kRegroupStaticInts = 1 << 20;
hipError_t regroup_index_static(const int32_t* cur, int32_t n, int32_t E, int32_t* cnt, int32_t* off, int32_t* perm,
                                int32_t* inv, hipStream_t stream);

// Request arranging, activation part: dst row i = src row perm[i]; rows of row_bytes (multiple of 4) bytes.
// heads[e] = perm[off[e]] (the oldest queued request of expert e: the regroup is stable) or -1 for an empty group
hipError_t group_heads(const int32_t* perm, const int32_t* off, const int32_t* cnt, int32_t E, int32_t* heads,
                       hipStream_t stream);
hipError_t gather_rows(const void* src, const int32_t* perm, int32_t n_rows, size_t row_bytes, void* dst,
                       hipStream_t stream);

struct ConvShape {
    int32_t N, H, W, C, K, R, S, stride, pad, P, Q, act;
};

// Several groups of requests in ONE launch, each group with the weights of its own expert; the experts share an
// architecture, so only the weight base differs (request arranging leaves many groups of a handful of requests, and a
// launch per layer and group would be all launch latency).  The requests of the groups are consecutive rows of the
// batch.  The table travels as a kernel argument: no device copy per launch.
constexpr int kMaxGroups = 32;
struct GroupTable {
    int32_t n;                            // groups; 0 = plain launch with one set of weights
    int32_t first_row[kMaxGroups + 1];    // requests [first_row[g], first_row[g + 1]) of the batch belong to group g
    const void* weights[kMaxGroups];      // device blob of group g's expert
};
// per-group routing data for the head kernel
struct GroupRoutes {
    int32_t expert[kMaxGroups];           // expert id
    int32_t succ_off[kMaxGroups];         // offset of its successor list in RouteArgs::succ
    int32_t n_route[kMaxGroups];
    int32_t slot_off[kMaxGroups];         // offset of the group's first request in RouteArgs::slot
};

// Plain convolution kernel for any shape, fp32 or bf16 storage, fp32 FMA accumulation.
hipError_t conv_direct(int dtype, const void* x, const void* w, const float* bias, const void* res, void* y,
                       const ConvShape& s, hipStream_t stream);

// bf16 implicit-GEMM convolution on the matrix cores.  Requires C % 32 == 0 and K % 32 == 0 (N is not looked at).
// The filters must have been repacked with pack_filters_mfma (host): w is [K][red] with red = R*S*C, out has the
// same number of elements, ordered so that a wavefront reads a 32-filter x 16-element operand as 1 KiB contiguous.
bool conv_mfma_supported(const ConvShape& s);
// true when conv_mfma runs this shape with the 3x3 kernel that keeps the activation slab in LDS for all nine positions
bool conv_mfma_uses_slab(const ConvShape& s);
void pack_filters_mfma(const uint16_t* w, uint16_t* out, int K, int red);
hipError_t conv_mfma(const void* x, const void* w, const float* bias, const void* res, void* y, const ConvShape& s,
                     hipStream_t stream);
// Grouped form: s.N = requests of all groups; group g's (repacked) filters sit at weights[g] + off_w, its bias at
// weights[g] + off_b.  Output tiles never straddle two groups.  Only shapes with K % 64 == 0 (conv_mfma_groupable).
bool conv_mfma_groupable(const ConvShape& s);
hipError_t conv_mfma_grouped(const void* x, const GroupTable& groups, size_t off_w, size_t off_b, const void* res, void* y,
                             const ConvShape& s, hipStream_t stream);

// bf16 convolution with few input channels (C not a multiple of 32, e.g. the C=3 stem) on the matrix cores.
// Requires K in {32, 64}, stride*C even, no residual.  fused_pool: the 3x3 / stride 2 / pad 1 max pool that follows is
// applied in the same kernel and y receives the pooled tensor [N][(P-1)/2+1][(Q-1)/2+1][K] instead of the conv output.
// rows != nullptr: image n of the launch is image rows[n] of the array at x (the gather of request arranging, done
// while the patches are fetched instead of in a copy of its own).
bool conv_smallc_supported(const ConvShape& s, bool has_res, bool fused_pool);
hipError_t conv_smallc(const void* x, const void* w, const float* bias, void* y, const ConvShape& s, bool fused_pool,
                       hipStream_t stream, const int32_t* rows = nullptr);

hipError_t maxpool(int dtype, const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S,
                   int32_t stride, int32_t pad, int32_t P, int32_t Q, hipStream_t stream);

// Global average pool + FC + argmax routing.  x: [N][HW][C]; w: [ncls][C] in dtype; b: [ncls] fp32.
hipError_t head_gap_fc(int dtype, const void* x, const void* w, const float* b, int32_t N, int32_t HW, int32_t C,
                       int32_t ncls, const RouteArgs& r, hipStream_t stream);
// Grouped form: FC weights at weights[g] + off_w, bias at + off_b; r.succ is the base of all successor lists and r.slot
// the base of the slot array, both indexed through `routes`; r.expert and r.n_route are ignored.
hipError_t head_gap_fc_grouped(int dtype, const void* x, const GroupTable& groups, size_t off_w, size_t off_b, int32_t N,
                               int32_t HW, int32_t C, int32_t ncls, const RouteArgs& r, const GroupRoutes& routes,
                               hipStream_t stream);

// ---- detector-shaped experts (bf16 only) -----------------------------------------------------------------------
// out[n][i] = [a[n][i] (Ca channels) | b[n][i] (Cb channels)] for the HW positions of every image; Ca, Cb multiples of 8.
hipError_t concat_channels(const void* a, const void* b, void* out, int64_t rows, int32_t Ca, int32_t Cb, hipStream_t stream);
// nearest-neighbour upsampling by two: out[n][h][w] = x[n][h/2][w/2]; C a multiple of 8.
hipError_t upsample2(const void* x, void* out, int32_t N, int32_t H, int32_t W, int32_t C, hipStream_t stream);
// Detection read-out: maps m0 [N][hw0][anchors*(5+ncls)] and (optional) m1 [N][hw1][...]; logits[c] = max over maps, positions
// and anchors of sigmoid(objectness) * sigmoid(class c); then routing like head_gap_fc.  ncls <= 256.
hipError_t head_det(const void* m0, int32_t hw0, const void* m1, int32_t hw1, int32_t N, int32_t anchors, int32_t ncls,
                    const RouteArgs& r, hipStream_t stream);

// ---- transformer-shaped experts (bf16 only) --------------------------------------------------------------------
// Patches of a non-overlapping convolution (stride == window, no padding) as GEMM rows:
// x [N][H][W][C] -> out [N * (H/R) * (W/S)][R*S*C].  S*C*2 bytes must be a multiple of 16.
hipError_t patchify(const void* x, void* out, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, hipStream_t stream);
// out[n][0] = cls + pos[0]; out[n][1+i] = x[n][i] + pos[1+i]; T = tokens of out; D % 8 == 0.
hipError_t tokens(const void* x, const void* cls, const void* pos, void* out, int32_t N, int32_t T, int32_t D, hipStream_t stream);
// layer norm over D channels of `rows` tokens, eps 1e-6, D even and <= 2048.
hipError_t layernorm(const void* x, const float* gamma, const float* beta, void* y, int64_t rows, int32_t D, hipStream_t stream);
// qkv [N][T][3D] (q | k | v) -> out [N][T][D]; head width must be 64, T <= 224.
bool attention_supported(int32_t T, int32_t D, int32_t heads);
hipError_t attention(const void* qkv, void* out, int32_t N, int32_t T, int32_t D, int32_t heads, hipStream_t stream);
// logits = FC(layer norm(token 0 of x [N][T][D])), then routing like head_gap_fc.
hipError_t head_cls(const void* x, const float* gamma, const float* beta, const void* w, const float* b, int32_t N, int32_t T,
                    int32_t D, int32_t ncls, const RouteArgs& r, hipStream_t stream);

}  // namespace k
}  // namespace coe
