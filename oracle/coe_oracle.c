/*
 * CPU oracle for dependency-routed batched expert inference (CoE serving).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, direct-loop statement of what the
 * GPU hot path must compute.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the product path never does.  It shares no code with the HIP library.
 *
 * What it follows (CoServe paper):
 *   - Section 2.1 "CoE Model and Its Use Cases": an input picks a first expert; the expert's
 *     output either selects the next expert or is the final result; several upstream experts
 *     may share one downstream expert.  -> orc_run_chain
 *   - Section 4.2 "Request arranging": requests using the same expert are placed behind each
 *     other so an expert is loaded at most once per group.  -> orc_regroup
 *   - Section 4.2 "Request splitting": a group is cut into batches no larger than the maximum
 *     executable batch size.  -> orc_split
 *   - Section 4.1 "System initialization" + Section 4.3 "Dependency-aware Expert Management":
 *     initial fill by descending usage probability; on a miss, two-stage eviction (first
 *     dependent experts none of whose predecessors is around, largest first; then ascending
 *     usage probability), each stage stopping as soon as the new expert fits.  -> orc_cache_*
 *
 * The paper fixes no layer numerics (its experts are stock PyTorch models).  The reading used
 * here: convolution is cross-correlation with zero padding; accumulation in fp64 over the
 * exactly representable products; epilogue acc + bias (+ residual), activation, one cast to
 * fp32, then (bf16 experts) round-to-nearest-even to bf16 at every stored activation;
 * global-average-pool and FC accumulate in fp64 from the stored features; logits are fp32;
 * argmax takes the lowest index among equal maxima and is taken on the fp32 logits.
 *
 * Pins (see tests): brute-force im2col convolution, delta / constant / linearity / stride
 * closed forms, exhaustive bf16 rounding checks, exhaustive regroup on tiny inputs, planted
 * one-hot routing, hand-made eviction cases.  Cache switch-log parity has no printed example
 * in the paper (the eviction figure's numbers are not in the text): beyond the hand cases it is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OP_CONV = 1, OP_MAXPOOL = 2, OP_HEAD = 3, OP_TOKENS = 4, OP_LAYERNORM = 5, OP_ATTENTION = 6, OP_HEAD_CLS = 7,
       OP_CONCAT = 8, OP_UPSAMPLE = 9, OP_HEAD_DET = 10 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2, ACT_SILU = 3 };
enum { DT_F32 = 0, DT_BF16 = 1 };
#define LAYER_WORDS 12
#define BLOB_ALIGN 256
#define MAX_BUFS 8

/* ------------------------------------------------------------------------------------------
 * bf16 helpers
 * ---------------------------------------------------------------------------------------- */
/* fp32 -> nearest bf16 (ties to even), returned as the fp32 value it represents. */
float orc_bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) { /* inf / nan: keep class, quiet the nan */
        if (u & 0x007FFFFFu) u |= 0x00400000u;
        u &= 0xFFFF0000u;
    } else {
        uint32_t keep = u & 0xFFFF0000u, rest = u & 0x0000FFFFu;
        if (rest > 0x8000u || (rest == 0x8000u && (keep & 0x00010000u))) keep += 0x00010000u;
        u = keep;
    }
    memcpy(&f, &u, 4);
    return f;
}

static float bf16_bits_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* value -> storage precision of the expert (fp32, or bf16 after the fp32 cast) */
static float store_val(double v, int dtype)
{
    float f = (float)v;
    return dtype == DT_BF16 ? orc_bf16_round(f) : f;
}

static double apply_act(double v, int act)
{
    if (act == ACT_RELU) return v > 0.0 ? v : 0.0;
    if (act == ACT_GELU) return 0.5 * v * (1.0 + erf(v * 0.70710678118654752440));
    if (act == ACT_SILU) return v / (1.0 + exp(-v));
    return v;
}

/* ------------------------------------------------------------------------------------------
 * layers (single image, NHWC, activations held as fp32 values already in storage precision)
 * ---------------------------------------------------------------------------------------- */
/* y[p][q][k] = act( sum_{r,s,c} x[p*stride-pad+r][q*stride-pad+s][c] * w[k][r][s][c] + bias[k] (+ res[p][q][k]) ) */
void orc_conv2d(const float* x, int H, int W, int C, const float* w, const float* bias, const float* res,
                int K, int R, int S, int stride, int pad, int act, int dtype, float* y)
{
    int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    /* weights copied to [r][s][c][k] so the innermost loop runs over independent accumulators */
    double* wt = (double*)malloc(sizeof(double) * (size_t)R * S * C * K);
    double* acc = (double*)malloc(sizeof(double) * (size_t)K);
    for (int k = 0; k < K; ++k)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s)
                for (int c = 0; c < C; ++c)
                    wt[(((size_t)r * S + s) * C + c) * K + k] = (double)w[(((size_t)k * R + r) * S + s) * C + c];
    for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
            for (int k = 0; k < K; ++k) acc[k] = 0.0;
            for (int r = 0; r < R; ++r) {
                int ih = p * stride - pad + r;
                if (ih < 0 || ih >= H) continue;
                for (int s = 0; s < S; ++s) {
                    int iw = q * stride - pad + s;
                    if (iw < 0 || iw >= W) continue;
                    const float* xp = x + ((size_t)ih * W + iw) * C;
                    const double* wp = wt + ((size_t)r * S + s) * C * K;
                    for (int c = 0; c < C; ++c) {
                        double xv = (double)xp[c];
                        const double* wk = wp + (size_t)c * K;
                        for (int k = 0; k < K; ++k) acc[k] += xv * wk[k];
                    }
                }
            }
            float* yp = y + ((size_t)p * Q + q) * K;
            const float* rp = res ? res + ((size_t)p * Q + q) * K : 0;
            for (int k = 0; k < K; ++k) {
                double v = acc[k] + (double)bias[k];
                if (rp) v += (double)rp[k];
                yp[k] = store_val(apply_act(v, act), dtype);
            }
        }
    free(acc);
    free(wt);
}

/* window max; padded positions never win (as if -inf) */
void orc_maxpool(const float* x, int H, int W, int C, int R, int S, int stride, int pad, float* y)
{
    int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q)
            for (int c = 0; c < C; ++c) {
                float m = -INFINITY;
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        int ih = p * stride - pad + r, iw = q * stride - pad + s;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                        float v = x[((size_t)ih * W + iw) * C + c];
                        if (v > m) m = v;
                    }
                y[((size_t)p * Q + q) * C + c] = m;
            }
}

/* logits[j] = sum_c mean_{h,w}(x[h][w][c]) * w[j][c] + b[j]   (fp64 throughout, one cast to fp32) */
void orc_gap_fc(const float* x, int H, int W, int C, const float* w, const float* b, int ncls, float* logits)
{
    double* feat = (double*)malloc(sizeof(double) * (size_t)C);
    for (int c = 0; c < C; ++c) feat[c] = 0.0;
    for (int i = 0; i < H * W; ++i)
        for (int c = 0; c < C; ++c) feat[c] += (double)x[(size_t)i * C + c];
    for (int c = 0; c < C; ++c) feat[c] /= (double)(H * W);
    for (int j = 0; j < ncls; ++j) {
        double a = 0.0;
        for (int c = 0; c < C; ++c) a += feat[c] * (double)w[(size_t)j * C + c];
        logits[j] = (float)(a + (double)b[j]);
    }
    free(feat);
}

/* out[0] = cls + pos[0]; out[1+i] = x[i] + pos[1+i] */
void orc_tokens(const float* x, int T0, int C, const float* cls, const float* pos, int dtype, float* y)
{
    for (int c = 0; c < C; ++c) y[c] = store_val((double)cls[c] + (double)pos[c], dtype);
    for (int i = 0; i < T0; ++i)
        for (int c = 0; c < C; ++c)
            y[(size_t)(i + 1) * C + c] = store_val((double)x[(size_t)i * C + c] + (double)pos[(size_t)(i + 1) * C + c], dtype);
}

/* per token: (x - mean) / sqrt(var + 1e-6) * gamma + beta, biased variance */
void orc_layernorm(const float* x, int T, int C, const float* gamma, const float* beta, int dtype, float* y)
{
    for (int t = 0; t < T; ++t) {
        const float* xp = x + (size_t)t * C;
        double mean = 0.0, var = 0.0;
        for (int c = 0; c < C; ++c) mean += (double)xp[c];
        mean /= C;
        for (int c = 0; c < C; ++c) { double d = (double)xp[c] - mean; var += d * d; }
        var /= C;
        double rstd = 1.0 / sqrt(var + 1e-6);
        for (int c = 0; c < C; ++c)
            y[(size_t)t * C + c] = store_val(((double)xp[c] - mean) * rstd * (double)gamma[c] + (double)beta[c], dtype);
    }
}

/* qkv[t] = [q(D) | k(D) | v(D)], head h owns channels [h*dh, (h+1)*dh).
 * Scaled dot-product attention as it is defined: s_ij = q_i.k_j / sqrt(dh); p_ij = exp(s_ij - max_j s_ij) / sum_j exp(...)
 * (the softmax, fp64); the probabilities are a tensor of their own and take the storage precision of the expert like every
 * other tensor (bf16 experts: one cast to fp32, one round to bf16 per probability); out_i = sum_j p_ij v_j, accumulated in
 * fp64 over the rounded probabilities and stored in storage precision.  Nothing is divided after the rounding. */
void orc_attention(const float* qkv, int T, int D, int heads, int dtype, float* y)
{
    int dh = D / heads;
    double scale = 1.0 / sqrt((double)dh);
    double* s = (double*)malloc(sizeof(double) * (size_t)T);
    for (int h = 0; h < heads; ++h)
        for (int i = 0; i < T; ++i) {
            const float* q = qkv + (size_t)i * 3 * D + h * dh;
            double m = -INFINITY;
            for (int j = 0; j < T; ++j) {
                const float* k = qkv + (size_t)j * 3 * D + D + h * dh;
                double a = 0.0;
                for (int d = 0; d < dh; ++d) a += (double)q[d] * (double)k[d];
                s[j] = a * scale;
                if (s[j] > m) m = s[j];
            }
            double l = 0.0;
            for (int j = 0; j < T; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
            for (int j = 0; j < T; ++j) s[j] = (double)store_val(s[j] / l, dtype);
            for (int d = 0; d < dh; ++d) {
                double a = 0.0;
                for (int j = 0; j < T; ++j) a += s[j] * (double)qkv[(size_t)j * 3 * D + 2 * D + h * dh + d];
                y[(size_t)i * D + h * dh + d] = store_val(a, dtype);
            }
        }
    free(s);
}

/* ---- detector-shaped experts (the paper's object-detection experts, Section 5.1: a multi-scale backbone whose feature maps
 * are concatenated, upsampled and read out by per-position detection outputs) ---- */
/* y[h][w] = [a[h][w] (Ca channels) | b[h][w] (Cb channels)] */
void orc_concat(const float* a, const float* b, int HW, int Ca, int Cb, float* y)
{
    for (int i = 0; i < HW; ++i) {
        for (int c = 0; c < Ca; ++c) y[(size_t)i * (Ca + Cb) + c] = a[(size_t)i * Ca + c];
        for (int c = 0; c < Cb; ++c) y[(size_t)i * (Ca + Cb) + Ca + c] = b[(size_t)i * Cb + c];
    }
}

/* nearest-neighbour upsampling by two: y[h][w] = x[h / 2][w / 2] */
void orc_upsample2(const float* x, int H, int W, int C, float* y)
{
    for (int h = 0; h < 2 * H; ++h)
        for (int w = 0; w < 2 * W; ++w)
            for (int c = 0; c < C; ++c) y[((size_t)h * 2 * W + w) * C + c] = x[((size_t)(h / 2) * W + w / 2) * C + c];
}

/* Detection read-out.  A detection map holds, per position, `anchors` boxes of (5 + ncls) values: 4 box terms, one
 * objectness logit, ncls class logits.  The expert's output for class c is its best detection of that class anywhere:
 * logits[c] = max over maps, positions and anchors of sigmoid(objectness) * sigmoid(class c), computed in fp64 from the
 * stored map values and cast to fp32 once.  (A maximum has no accumulation order: the value is exact on any device.) */
void orc_det_head(const float* const* maps, const int* map_hw, int n_maps, int anchors, int ncls, float* logits)
{
    int stride = anchors * (5 + ncls);
    for (int c = 0; c < ncls; ++c) {
        double best = 0.0;
        for (int m = 0; m < n_maps; ++m)
            for (int i = 0; i < map_hw[m]; ++i)
                for (int a = 0; a < anchors; ++a) {
                    const float* box = maps[m] + (size_t)i * stride + (size_t)a * (5 + ncls);
                    double sc = 1.0 / (1.0 + exp(-(double)box[4])) * (1.0 / (1.0 + exp(-(double)box[5 + c])));
                    if (sc > best) best = sc;
                }
        logits[c] = (float)best;
    }
}

/* ------------------------------------------------------------------------------------------
 * expert forward from an architecture descriptor and a weight blob
 * ---------------------------------------------------------------------------------------- */
typedef struct { int h, w, c; float* data; size_t cap; } obuf;

static size_t align_up(size_t x) { return (x + BLOB_ALIGN - 1) / BLOB_ALIGN * BLOB_ALIGN; }

/* read n parameters from the blob at *off (aligned first) into a fresh fp32 array */
static float* take(const uint8_t* blob, size_t* off, size_t n, int as_dtype)
{
    float* out = (float*)malloc(sizeof(float) * (n ? n : 1));
    *off = align_up(*off);
    if (as_dtype == DT_BF16) {
        const uint16_t* p = (const uint16_t*)(blob + *off);
        for (size_t i = 0; i < n; ++i) out[i] = bf16_bits_to_f32(p[i]);
        *off += 2 * n;
    } else {
        memcpy(out, blob + *off, 4 * n);
        *off += 4 * n;
    }
    return out;
}

static void ensure(obuf* b, size_t n)
{
    if (b->cap < n) { free(b->data); b->data = (float*)malloc(sizeof(float) * n); b->cap = n; }
}

/* One request through one expert.  input: in_h*in_w*in_c elements in the expert's dtype (bf16 bits or fp32).
 * Returns 0, or a negative number for a malformed descriptor. */
static int forward_impl(int dtype, int in_h, int in_w, int in_c, int n_layers, const int32_t* layers, const uint8_t* blob,
                        const void* input, float* logits, int stop_after, float* layer_out, int64_t layer_cap, int32_t* layer_shape);

int orc_forward(int dtype, int in_h, int in_w, int in_c, int n_layers, const int32_t* layers, const uint8_t* blob,
                const void* input, float* logits)
{
    return forward_impl(dtype, in_h, in_w, in_c, n_layers, layers, blob, input, logits, -1, 0, 0, 0);
}

/* The same program stopped after layer `stop_after` (not a head): that layer's output tensor [h][w][c], as fp32 values in
 * storage precision, goes to layer_out (at most layer_cap elements) and its shape to layer_shape[3].  For looking at where two
 * implementations of an expert drift apart.  Returns 0, a negative error, or -20 when layer_cap is too small. */
int orc_forward_layer(int dtype, int in_h, int in_w, int in_c, int n_layers, const int32_t* layers, const uint8_t* blob,
                      const void* input, int stop_after, float* layer_out, int64_t layer_cap, int32_t* layer_shape)
{
    float dummy[1024];
    if (stop_after < 0 || stop_after >= n_layers) return -21;
    return forward_impl(dtype, in_h, in_w, in_c, n_layers, layers, blob, input, dummy, stop_after, layer_out, layer_cap, layer_shape);
}

static int forward_impl(int dtype, int in_h, int in_w, int in_c, int n_layers, const int32_t* layers, const uint8_t* blob,
                        const void* input, float* logits, int stop_after, float* layer_out, int64_t layer_cap, int32_t* layer_shape)
{
    obuf buf[MAX_BUFS];
    memset(buf, 0, sizeof(buf));
    size_t n_in = (size_t)in_h * in_w * in_c;
    ensure(&buf[0], n_in);
    buf[0].h = in_h; buf[0].w = in_w; buf[0].c = in_c;
    if (dtype == DT_BF16) for (size_t i = 0; i < n_in; ++i) buf[0].data[i] = bf16_bits_to_f32(((const uint16_t*)input)[i]);
    else memcpy(buf[0].data, input, 4 * n_in);
    size_t off = 0;
    int rc = 0;
    for (int li = 0; li < n_layers && rc == 0; ++li) {
        const int32_t* L = layers + (size_t)li * LAYER_WORDS;
        int op = L[0], src = L[1], dst = L[2], res = L[3], K = L[4], R = L[5], S = L[6], stride = L[7], pad = L[8], act = L[9];
        if (src < 0 || src >= MAX_BUFS || !buf[src].data) { rc = -1; break; }
        obuf* x = &buf[src];
        if (op == OP_CONV || op == OP_MAXPOOL) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src) { rc = -2; break; }
            int P = (x->h + 2 * pad - R) / stride + 1, Q = (x->w + 2 * pad - S) / stride + 1;
            ensure(&buf[dst], (size_t)P * Q * K);
            if (op == OP_CONV) {
                float* w = take(blob, &off, (size_t)K * R * S * x->c, dtype);
                float* b = take(blob, &off, (size_t)K, DT_F32);
                const float* rp = 0;
                if (res >= 0) {
                    if (res >= MAX_BUFS || !buf[res].data || buf[res].h != P || buf[res].w != Q || buf[res].c != K || res == dst) rc = -3;
                    else rp = buf[res].data;
                }
                if (rc == 0) orc_conv2d(x->data, x->h, x->w, x->c, w, b, rp, K, R, S, stride, pad, act, dtype, buf[dst].data);
                free(w); free(b);
            } else {
                if (K != x->c) rc = -4;
                else orc_maxpool(x->data, x->h, x->w, x->c, R, S, stride, pad, buf[dst].data);
            }
            buf[dst].h = P; buf[dst].w = Q; buf[dst].c = K;
        } else if (op == OP_HEAD) {
            float* w = take(blob, &off, (size_t)K * x->c, dtype);
            float* b = take(blob, &off, (size_t)K, DT_F32);
            orc_gap_fc(x->data, x->h, x->w, x->c, w, b, K, logits);
            free(w); free(b);
        } else if (op == OP_TOKENS) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src) { rc = -2; break; }
            int T0 = x->h * x->w;
            float* cls = take(blob, &off, (size_t)x->c, dtype);
            float* pos = take(blob, &off, (size_t)(T0 + 1) * x->c, dtype);
            ensure(&buf[dst], (size_t)(T0 + 1) * x->c);
            orc_tokens(x->data, T0, x->c, cls, pos, dtype, buf[dst].data);
            buf[dst].h = T0 + 1; buf[dst].w = 1; buf[dst].c = x->c;
            free(cls); free(pos);
        } else if (op == OP_LAYERNORM) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src) { rc = -2; break; }
            float* g = take(blob, &off, (size_t)x->c, DT_F32);
            float* b = take(blob, &off, (size_t)x->c, DT_F32);
            ensure(&buf[dst], (size_t)x->h * x->w * x->c);
            orc_layernorm(x->data, x->h * x->w, x->c, g, b, dtype, buf[dst].data);
            buf[dst].h = x->h; buf[dst].w = x->w; buf[dst].c = x->c;
            free(g); free(b);
        } else if (op == OP_ATTENTION) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src) { rc = -2; break; }
            int D = x->c / 3, heads = L[10];
            if (heads <= 0 || D % heads) { rc = -5; break; }
            ensure(&buf[dst], (size_t)x->h * x->w * D);
            orc_attention(x->data, x->h * x->w, D, heads, dtype, buf[dst].data);
            buf[dst].h = x->h; buf[dst].w = x->w; buf[dst].c = D;
        } else if (op == OP_CONCAT) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src || dst == res) { rc = -2; break; }
            if (res < 0 || res >= MAX_BUFS || !buf[res].data || buf[res].h != x->h || buf[res].w != x->w) { rc = -3; break; }
            int Cc = x->c + buf[res].c;
            ensure(&buf[dst], (size_t)x->h * x->w * Cc);
            orc_concat(x->data, buf[res].data, x->h * x->w, x->c, buf[res].c, buf[dst].data);
            buf[dst].h = x->h; buf[dst].w = x->w; buf[dst].c = Cc;
        } else if (op == OP_UPSAMPLE) {
            if (dst <= 0 || dst >= MAX_BUFS || dst == src) { rc = -2; break; }
            ensure(&buf[dst], (size_t)4 * x->h * x->w * x->c);
            orc_upsample2(x->data, x->h, x->w, x->c, buf[dst].data);
            buf[dst].h = 2 * x->h; buf[dst].w = 2 * x->w; buf[dst].c = x->c;
        } else if (op == OP_HEAD_DET) {
            /* src (and res, if >= 0) are detection maps; K classes; aux0 anchors */
            int anchors = L[10];
            const float* maps[2]; int hw[2]; int nm = 0;
            if (anchors <= 0 || x->c != anchors * (5 + K)) { rc = -6; break; }
            maps[nm] = x->data; hw[nm] = x->h * x->w; ++nm;
            if (res >= 0) {
                if (res >= MAX_BUFS || !buf[res].data || buf[res].c != x->c) { rc = -3; break; }
                maps[nm] = buf[res].data; hw[nm] = buf[res].h * buf[res].w; ++nm;
            }
            orc_det_head(maps, hw, nm, anchors, K, logits);
        } else if (op == OP_HEAD_CLS) {
            float* g = take(blob, &off, (size_t)x->c, DT_F32);
            float* b = take(blob, &off, (size_t)x->c, DT_F32);
            float* w = take(blob, &off, (size_t)K * x->c, dtype);
            float* fb = take(blob, &off, (size_t)K, DT_F32);
            float* n = (float*)malloc(sizeof(float) * (size_t)x->c);
            orc_layernorm(x->data, 1, x->c, g, b, dtype, n);          /* token 0 only */
            for (int j = 0; j < K; ++j) {
                double a = 0.0;
                for (int c = 0; c < x->c; ++c) a += (double)n[c] * (double)w[(size_t)j * x->c + c];
                logits[j] = (float)(a + (double)fb[j]);
            }
            free(g); free(b); free(w); free(fb); free(n);
        } else rc = -9;
        if (rc == 0 && li == stop_after) {
            if (op == OP_HEAD || op == OP_HEAD_CLS || op == OP_HEAD_DET) rc = -22;
            else {
                int64_t n = (int64_t)buf[dst].h * buf[dst].w * buf[dst].c;
                if (n > layer_cap) rc = -20;
                else {
                    memcpy(layer_out, buf[dst].data, sizeof(float) * (size_t)n);
                    layer_shape[0] = buf[dst].h; layer_shape[1] = buf[dst].w; layer_shape[2] = buf[dst].c;
                }
            }
            break;
        }
    }
    for (int i = 0; i < MAX_BUFS; ++i) free(buf[i].data);
    return rc;
}

/* lowest index among equal maxima */
int orc_argmax(const float* v, int n)
{
    int best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/* ------------------------------------------------------------------------------------------
 * the CoE chain, one request at a time (no batching, no cache): the plain definition
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int32_t dtype, in_h, in_w, in_c, n_classes, n_layers;
    const int32_t* layers;
} orc_arch;

/* For every request r: e = first_expert[r] (or 0); repeat { run expert e on the request's ORIGINAL input;
 * k = number of successors of e; if k == 0 stop; c = argmax over the first k logits; e = succ[e][c]; if e == -1 stop }.
 * Outputs: logits[r][max_classes] of the last expert (zero padded), path[r][max_stages] (-1 padded),
 * all_logits (nullable) [r][max_stages][max_classes] logits of every visited stage,
 * margin (nullable) [r][max_stages]: (top1 - top2) / max|logit| over the routed classes at each routing stage, else -1.
 * Returns 0 or a negative error.  Requests run in parallel over `threads` OpenMP threads (<=0: all). */
int orc_run_chain(int n_archs, const orc_arch* archs, int n_experts, const int32_t* expert_arch,
                  const uint8_t* const* blobs, const int32_t* succ_off, const int32_t* succ,
                  int n_req, const void* inputs, const int32_t* first_expert, int max_stages, int max_classes,
                  float* logits, int32_t* path, float* all_logits, float* margin, int threads)
{
    if (n_archs <= 0) return -1;
    size_t in_elems = (size_t)archs[0].in_h * archs[0].in_w * archs[0].in_c;
    size_t in_bytes = in_elems * (archs[0].dtype == DT_BF16 ? 2 : 4);
    int err = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_req; ++r) {
        float* lg = (float*)calloc((size_t)max_classes, sizeof(float));
        int e = first_expert ? first_expert[r] : 0;
        for (int s = 0; s < max_stages; ++s) { path[(size_t)r * max_stages + s] = -1; if (margin) margin[(size_t)r * max_stages + s] = -1.f; }
        for (int s = 0; s < max_stages; ++s) {
            if (e < 0 || e >= n_experts) { err = -2; break; }
            const orc_arch* a = &archs[expert_arch[e]];
            path[(size_t)r * max_stages + s] = e;
            memset(lg, 0, sizeof(float) * (size_t)max_classes);
            int rc = orc_forward(a->dtype, a->in_h, a->in_w, a->in_c, a->n_layers, a->layers, blobs[e],
                                 (const uint8_t*)inputs + (size_t)r * in_bytes, lg);
            if (rc) { err = rc; break; }
            if (all_logits) memcpy(all_logits + ((size_t)r * max_stages + s) * max_classes, lg, sizeof(float) * (size_t)max_classes);
            int k = succ_off[e + 1] - succ_off[e];
            if (k == 0) break;
            if (k > a->n_classes) { err = -3; break; }
            int c = orc_argmax(lg, k);
            if (margin) {
                float top2 = -INFINITY, amax = 0.f;
                for (int j = 0; j < k; ++j) { if (j != c && lg[j] > top2) top2 = lg[j]; if (fabsf(lg[j]) > amax) amax = fabsf(lg[j]); }
                margin[(size_t)r * max_stages + s] = k > 1 ? (lg[c] - top2) / (amax > 1e-30f ? amax : 1e-30f) : 1.f;
            }
            int nxt = succ[succ_off[e] + c];
            if (nxt == -1) break;
            if (s == max_stages - 1) { err = -4; break; } /* graph deeper than max_stages */
            e = nxt;
        }
        memcpy(logits + (size_t)r * max_classes, lg, sizeof(float) * (size_t)max_classes);
        free(lg);
    }
    return err;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * request arranging: stable order of the pending requests by the expert they need
 * ---------------------------------------------------------------------------------------- */
typedef struct { int32_t key, idx; } kv;
static int kv_cmp(const void* a, const void* b)
{
    const kv* x = (const kv*)a; const kv* y = (const kv*)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx);
}

/* cur[r] in [0,E) = expert request r waits for; anything else = not pending.
 * perm lists the pending requests ordered by (expert, request index); cnt[e] requests per expert;
 * off[e] = start of expert e's group in perm (off[E] = number pending); inv[r] = position of r in perm or -1.
 * Returns the number of pending requests. */
int orc_regroup(const int32_t* cur, int n, int E, int32_t* cnt, int32_t* off, int32_t* perm, int32_t* inv)
{
    kv* a = (kv*)malloc(sizeof(kv) * (size_t)(n ? n : 1));
    int m = 0;
    for (int e = 0; e < E; ++e) cnt[e] = 0;
    for (int r = 0; r < n; ++r) {
        inv[r] = -1;
        if (cur[r] >= 0 && cur[r] < E) { a[m].key = cur[r]; a[m].idx = r; ++m; cnt[cur[r]]++; }
    }
    qsort(a, (size_t)m, sizeof(kv), kv_cmp);
    for (int i = 0; i < m; ++i) { perm[i] = a[i].idx; inv[a[i].idx] = i; }
    off[0] = 0;
    for (int e = 0; e < E; ++e) off[e + 1] = off[e] + cnt[e];
    free(a);
    return m;
}

/* Request splitting (Section 4.2): no batch may exceed the maximum executable batch size.  The paper fixes only that bound;
 * the reading taken here: a group of n requests becomes the FEWEST batches the bound allows, ceil(n / max_batch), and those
 * are made as even as consecutive cutting allows - every batch holds ceil(n / batches) requests and the last one the rest -
 * because a short last batch is the least efficient one (latency per request falls with the batch size, Section 4.5).
 * Groups are taken in the given expert order.  chunks[i] = {expert, start in perm, count}.  Returns the number of chunks
 * (<= cap) or -1. */
int orc_split(const int32_t* off, int n_order, const int32_t* order, int max_batch, int32_t* chunks, int cap)
{
    int n = 0;
    for (int i = 0; i < n_order; ++i) {
        int e = order[i];
        int cnt = off[e + 1] - off[e];
        if (cnt <= 0) continue;
        int batches = (cnt + max_batch - 1) / max_batch;
        int size = (cnt + batches - 1) / batches;
        for (int s = off[e]; s < off[e + 1]; s += size) {
            if (n >= cap) return -1;
            int c = off[e + 1] - s; if (c > size) c = size;
            chunks[3 * n] = e; chunks[3 * n + 1] = s; chunks[3 * n + 2] = c; ++n;
        }
    }
    return n;
}

/* ------------------------------------------------------------------------------------------
 * expert cache policy simulator
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int E;
    const int64_t* bytes;     /* memory footprint per expert */
    const float* prob;        /* usage probability per expert */
    const int32_t* succ_off; const int32_t* succ;
    int cap_experts;          /* 0 = unlimited */
    int64_t cap_bytes;        /* 0 = unlimited */
    uint8_t* resident;        /* [E] */
    int n_res; int64_t res_bytes;
    int rule;                 /* 0 = two-stage (Section 4.3); 1 = least recently used; 2 = first in, first out */
    int in_use;               /* a load is started while the groups before it in the plan still run (Section 4.2: an
                                 expert can be loaded during the processing of a preceding request): the experts of this
                                 many preceding groups cannot be its victims */
    int64_t now;              /* event counter: every load and every executed group is one event */
    int64_t* t_load;          /* [E] event of the last load */
    int64_t* t_use;           /* [E] event of the last use (a load counts as a use) */
} orc_cache;

orc_cache* orc_cache_new(int E, const int64_t* bytes, const float* prob, const int32_t* succ_off, const int32_t* succ,
                         int cap_experts, int64_t cap_bytes)
{
    orc_cache* c = (orc_cache*)calloc(1, sizeof(orc_cache));
    c->E = E; c->bytes = bytes; c->prob = prob; c->succ_off = succ_off; c->succ = succ;
    c->cap_experts = cap_experts; c->cap_bytes = cap_bytes;
    c->resident = (uint8_t*)calloc((size_t)E, 1);
    c->t_load = (int64_t*)calloc((size_t)E, sizeof(int64_t));
    c->t_use = (int64_t*)calloc((size_t)E, sizeof(int64_t));
    return c;
}
void orc_cache_free(orc_cache* c) { if (c) { free(c->resident); free(c->t_load); free(c->t_use); free(c); } }
/* Replacement rule of the comparison systems (Section 5.1: LRU, FIFO) instead of the two-stage rule; the textbook
 * definitions: the victim is the resident expert used (LRU) / loaded (FIFO) longest ago.  As under the two-stage rule,
 * an expert whose group has not run yet in the stage is not a candidate. */
int orc_cache_set_rule(orc_cache* c, int rule) { if (rule < 0 || rule > 2) return -1; c->rule = rule; return 0; }
int orc_cache_set_in_use(orc_cache* c, int depth) { if (depth < 0) return -1; c->in_use = depth; return 0; }

/* is expert x one of the `depth` plan entries right before position i? */
static int runs_just_before(const int32_t* order, int i, int depth, int x)
{
    for (int q = i - 1; q >= 0 && q >= i - depth; --q)
        if (order[q] == x) return 1;
    return 0;
}
int orc_cache_resident(const orc_cache* c, uint8_t* out) { memcpy(out, c->resident, (size_t)c->E); return c->n_res; }

static int fits(const orc_cache* c, int e)
{
    if (c->cap_experts > 0 && c->n_res + 1 > c->cap_experts) return 0;
    if (c->cap_bytes > 0 && c->res_bytes + c->bytes[e] > c->cap_bytes) return 0;
    return 1;
}

/* initial fill: experts in descending usage probability (ties: lower id first) until the first that does not fit.
 * loaded[] receives the ids in load order; returns how many. */
int orc_cache_init_fill(orc_cache* c, int32_t* loaded)
{
    int n = 0;
    uint8_t* done = (uint8_t*)calloc((size_t)c->E, 1);
    for (;;) {
        int best = -1;
        for (int e = 0; e < c->E; ++e)
            if (!done[e] && (best < 0 || c->prob[e] > c->prob[best])) best = e;
        if (best < 0 || !fits(c, best)) break;
        done[best] = 1; c->resident[best] = 1; c->n_res++; c->res_bytes += c->bytes[best];
        c->t_load[best] = c->t_use[best] = ++c->now;
        loaded[n++] = best;
    }
    free(done);
    return n;
}

/* One stage.  has_group[e] != 0 marks the experts some pending request needs.
 * order[] receives the execution order: resident experts first (ascending id), then missing ones (ascending id).
 * For every miss, log receives: expert, n_victims, victim ids... (flat int32).  Victims: stage 1 = resident experts
 * that have predecessors, none of which is resident or has a group this stage, and that have no group themselves,
 * by descending bytes (ties: lower id); stage 2 = the remaining resident experts by ascending (probability, id);
 * experts whose group has not run yet in this stage, and the one being loaded, are never evicted.  Each stage stops
 * as soon as the new expert fits.  Returns the number of log words, or -1 if an expert cannot be made to fit. */
int orc_cache_stage(orc_cache* c, const uint8_t* has_group, int32_t* order, int* n_order, int32_t* log, int log_cap)
{
    int E = c->E, no = 0, nl = 0;
    for (int e = 0; e < E; ++e) if (has_group[e] && c->resident[e]) order[no++] = e;
    for (int e = 0; e < E; ++e) if (has_group[e] && !c->resident[e]) order[no++] = e;
    *n_order = no;
    uint8_t* todo = (uint8_t*)calloc((size_t)E, 1);   /* group not yet executed */
    for (int e = 0; e < E; ++e) todo[e] = has_group[e] ? 1 : 0;
    for (int i = 0; i < no; ++i) {
        int e = order[i];
        if (!c->resident[e]) {
            if (nl + 2 > log_cap) { free(todo); return -1; }
            int head = nl; log[nl++] = e; log[nl++] = 0;
            if (c->rule != 0) {
                const int64_t* t = c->rule == 1 ? c->t_use : c->t_load;
                while (!fits(c, e)) {
                    int v = -1;
                    for (int x = 0; x < E; ++x) {
                        if (!c->resident[x] || todo[x] || runs_just_before(order, i, c->in_use, x)) continue;
                        if (v < 0 || t[x] < t[v]) v = x;
                    }
                    if (v < 0) { free(todo); return -1; }
                    c->resident[v] = 0; c->n_res--; c->res_bytes -= c->bytes[v];
                    if (nl >= log_cap) { free(todo); return -1; }
                    log[nl++] = v; log[head + 1]++;
                }
            }
            /* stage 1: the candidate set is fixed when the miss occurs, then evicted largest first */
            uint8_t* cand = (uint8_t*)calloc((size_t)E, 1);
            for (int x = 0; x < E; ++x) {
                if (!c->resident[x] || todo[x] || has_group[x]) continue;
                int has_pred = 0, pred_around = 0;
                for (int p = 0; p < E; ++p)
                    for (int j = c->succ_off[p]; j < c->succ_off[p + 1]; ++j)
                        if (c->succ[j] == x) { has_pred = 1; if (c->resident[p] || has_group[p]) pred_around = 1; }
                cand[x] = (uint8_t)(has_pred && !pred_around);
            }
            while (!fits(c, e)) {
                int v = -1;
                for (int x = 0; x < E; ++x)
                    if (cand[x] && (v < 0 || c->bytes[x] > c->bytes[v])) v = x;
                if (v < 0) break;
                cand[v] = 0;
                c->resident[v] = 0; c->n_res--; c->res_bytes -= c->bytes[v];
                if (nl >= log_cap) { free(cand); free(todo); return -1; }
                log[nl++] = v; log[head + 1]++;
            }
            free(cand);
            /* stage 2 */
            while (!fits(c, e)) {
                int v = -1;
                for (int x = 0; x < E; ++x) {
                    if (!c->resident[x] || todo[x] || runs_just_before(order, i, c->in_use, x)) continue;
                    if (v < 0 || c->prob[x] < c->prob[v]) v = x;
                }
                if (v < 0) { free(todo); return -1; }
                c->resident[v] = 0; c->n_res--; c->res_bytes -= c->bytes[v];
                if (nl >= log_cap) { free(todo); return -1; }
                log[nl++] = v; log[head + 1]++;
            }
            c->resident[e] = 1; c->n_res++; c->res_bytes += c->bytes[e];
            c->t_load[e] = ++c->now;
        }
        c->t_use[e] = ++c->now;
        todo[e] = 0;
    }
    free(todo);
    return nl;
}
