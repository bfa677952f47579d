// Shape-agnostic scalar kernels of the KVCapsule hot path (any n, m, d <= 256, fp32 or
// bf16 storage, fp32 arithmetic).  They evaluate the decode step in the score-space
// order of Alg. 1 of the paper, generalised to a softmax that is joint over vision and
// text keys (Sec. 3.2):
//     S = sigma q Kc^T  ->  L = S theta  ->  P = softmax([L ; text logits])
//     W = P_vis U^T     ->  out = sum_blocks W Vc + (sum P_vis) mu + P_txt V_text
// The fp32 configuration and every shape outside the matrix-core kernels runs here.
#include "kvc_internal.h"

namespace kvc {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// ---- append the new token's k, v to the text cache (Sec. 3.2: text KV unchanged) ----
// per-sequence counts of a ragged call (null pointers: the uniform values); clamped to what the buffers hold
__device__ inline int seq_images(const int32_t *n_img, int b, int I) { return n_img ? min(max(n_img[b], 0), I) : I; }
__device__ inline int seq_text(const int32_t *tlen, int b, int t_uniform, int t_max) { return tlen ? min(max(tlen[b], 0), t_max) : t_uniform; }

template <class T>
__global__ void g_append(T *Kt, T *Vt, const T *k_new, const T *v_new, int d, int cap, int row_uniform, int Hkv,
                         const int32_t *tlen)
{
    size_t bh = blockIdx.x;
    const int row = seq_text(tlen, static_cast<int>(bh / Hkv), row_uniform, cap - 1);
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        Kt[(bh * cap + row) * d + c] = k_new[bh * d + c];
        Vt[(bh * cap + row) * d + c] = v_new[bh * d + c];
    }
}

// ---- Alg. 1 step 1: scores on the compressed keys, plus the text logits ----------------
// one wavefront per key row; grid.y = (b, kv head)
template <class T>
__global__ void g_scores(const T *__restrict__ q, const T *__restrict__ Kc,
                         const T *__restrict__ Kt, float *__restrict__ Svis,
                         float *__restrict__ Stxt, int Hq, int Hkv, int d, int Im, int t, int cap,
                         int tstride, float scale, int m, const int32_t *n_img, const int32_t *tlen, int append)
{
    const int G = Hq / Hkv;
    const size_t bh = blockIdx.y;
    const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rows = Im + t;                                   // t: the longest text of the call
    const int Imb = seq_images(n_img, b, Im / max(m, 1)) * m;  // this sequence's compressed rows
    const int tb = tlen ? seq_text(tlen, b, 0, cap - append) + append : t;
    for (int r = blockIdx.x * kWaves + wave; r < rows; r += gridDim.x * kWaves) {
        const bool live = r < Im ? r < Imb : r - Im < tb;      // rows the sequence does not have score -inf
        const T *k = r < Im ? Kc + (bh * Im + r) * d : Kt + (bh * cap + (r - Im)) * d;
        for (int g = 0; g < G; ++g) {
            const size_t bg = static_cast<size_t>(b) * Hq + h * G + g;
            const T *qr = q + bg * d;
            float acc = 0.f;
            if (live)
                for (int c = lane; c < d; c += 64) acc += to_f(qr[c]) * to_f(k[c]);
            acc = live ? wave_sum(acc) * scale : -INFINITY;
            if (lane == 0) {
                if (r < Im) Svis[bg * Im + r] = acc;
                else Stxt[bg * tstride + (r - Im)] = acc;
            }
        }
    }
}

// ---- Alg. 1 step 2: expand the compressed scores to the n positions of a block --------
// L[b,g,i,p] = sum_j S[b,g,i,j] theta[h,j,p];  grid = (p chunks, I, B*Hq)
template <class T>
__global__ void g_expand(const float *__restrict__ Svis, const T *__restrict__ theta,
                         float *__restrict__ L, int Hq, int Hkv, int n, int m, int I, const int32_t *n_img)
{
    extern __shared__ float sS[];
    const size_t bg = blockIdx.z;
    const int g = static_cast<int>(bg % Hq), h = g / (Hq / Hkv), i = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= seq_images(n_img, static_cast<int>(bg / Hq), I)) {      // a block the sequence does not have
        if (p < n) L[(bg * I + i) * n + p] = -INFINITY;
        return;
    }
    const float *Srow = Svis + (bg * I + i) * m;
    for (int j = threadIdx.x; j < m; j += blockDim.x) sS[j] = Srow[j];
    __syncthreads();
    if (p < n) {
        const T *th = theta + static_cast<size_t>(h) * m * n + p;
        float acc = 0.f;
        for (int j = 0; j < m; ++j) acc += sS[j] * to_f(th[static_cast<size_t>(j) * n]);
        L[(bg * I + i) * n + p] = acc;
    }
}

// ---- static variant: the compressed scores are the vision logits; their probabilities are the weights ----
__global__ void g_static_weights(const float *__restrict__ Svis, const float *__restrict__ stats,
                                 float *__restrict__ W, int Im)
{
    const size_t bg = blockIdx.y;
    const float mx = stats[bg * 4 + 0], inv = 1.f / stats[bg * 4 + 1];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < Im) W[bg * Im + r] = __expf(Svis[bg * Im + r] - mx) * inv;
}

// ---- joint softmax statistics per (b, query head): max, denominator, vision mass ----
__global__ void g_stats(const float *__restrict__ L, const float *__restrict__ Stxt,
                        float *__restrict__ stats, int Nvis, int t, int tstride)
{
    __shared__ float red[2 * kWaves];
    const size_t bg = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float mx = -INFINITY;
    for (int x = threadIdx.x; x < Nvis; x += blockDim.x) mx = fmaxf(mx, L[bg * Nvis + x]);
    for (int x = threadIdx.x; x < t; x += blockDim.x) mx = fmaxf(mx, Stxt[bg * tstride + x]);
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = red[0];
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, red[w]);
    __syncthreads();
    float sv = 0.f, st = 0.f;
    for (int x = threadIdx.x; x < Nvis; x += blockDim.x) sv += __expf(L[bg * Nvis + x] - mx);
    for (int x = threadIdx.x; x < t; x += blockDim.x) st += __expf(Stxt[bg * tstride + x] - mx);
    sv = wave_sum(sv);
    st = wave_sum(st);
    if (lane == 0) { red[wave] = sv; red[kWaves + wave] = st; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f, c = 0.f;
        for (int w = 0; w < kWaves; ++w) { a += red[w]; c += red[kWaves + w]; }
        stats[bg * 4 + 0] = mx;
        stats[bg * 4 + 1] = a + c;
        stats[bg * 4 + 2] = a / (a + c);
        stats[bg * 4 + 3] = 0.f;
    }
}

// ---- Alg. 1 step 3: fold the vision probabilities through U^T -----------------------------
// W[b,g,i,j] = sum_p P[b,g,i,p] U[h,j,p];  grid = (j groups of kJB, I, B*Hq)
constexpr int kJB = 32;
template <class T>
__global__ void g_project(const float *__restrict__ L, const float *__restrict__ stats,
                          const T *__restrict__ U, float *__restrict__ W, int Hq, int Hkv, int n,
                          int m, int I)
{
    extern __shared__ float sP[];
    const size_t bg = blockIdx.z;
    const int g = static_cast<int>(bg % Hq), h = g / (Hq / Hkv), i = blockIdx.y;
    const float mx = stats[bg * 4 + 0], inv = 1.f / stats[bg * 4 + 1];
    const float *Lrow = L + (bg * I + i) * n;
    for (int p = threadIdx.x; p < n; p += blockDim.x) sP[p] = __expf(Lrow[p] - mx) * inv;
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int jend = min(m, (static_cast<int>(blockIdx.x) + 1) * kJB);
    for (int j = blockIdx.x * kJB + wave; j < jend; j += kWaves) {
        const T *u = U + (static_cast<size_t>(h) * m + j) * n;
        float acc = 0.f;
        for (int p = lane; p < n; p += 64) acc += sP[p] * to_f(u[p]);
        acc = wave_sum(acc);
        if (lane == 0) W[(bg * I + i) * m + j] = acc;
    }
}

// ---- Alg. 1 step 4 plus the text part: out = W Vc + (sum P_vis) mu + P_txt V_text ---------
// one workgroup per (b, query head)
template <class T>
__global__ void g_output(const float *__restrict__ W, const float *__restrict__ Stxt,
                         const float *__restrict__ stats, const T *__restrict__ Vc,
                         const T *__restrict__ Vt, const T *__restrict__ mu, T *__restrict__ out,
                         float *__restrict__ lse, int Hq, int Hkv, int d, int Im, int m, int t,
                         int cap, int tstride, const int32_t *n_img, const int32_t *tlen, int append,
                         int with_mu)
{
    __shared__ float red[kThreads];
    const size_t bg = blockIdx.x;
    const int b = static_cast<int>(bg / Hq), g = static_cast<int>(bg % Hq), h = g / (Hq / Hkv);
    const size_t bh = static_cast<size_t>(b) * Hkv + h;
    const int slices = kThreads / d;          // d <= 256
    const int c = threadIdx.x % d, sl = threadIdx.x / d;
    const float mx = stats[bg * 4 + 0], inv = 1.f / stats[bg * 4 + 1];
    const int Imb = seq_images(n_img, b, Im / m) * m;
    const int tb = tlen ? seq_text(tlen, b, 0, cap - append) + append : t;
    float acc = 0.f;
    if (sl < slices) {
        for (int r = sl; r < Imb; r += slices) {
            const int i = r / m, j = r - i * m;
            acc += W[bg * Im + r] * to_f(Vc[(bh * Im + static_cast<size_t>(i) * m) * d + vc_offset(j, c, m, d)]);
        }
        for (int x = sl; x < tb; x += slices)
            acc += __expf(Stxt[bg * tstride + x] - mx) * inv * to_f(Vt[(bh * cap + x) * d + c]);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < d) {
        float y = 0.f;
        for (int s2 = 0; s2 < slices; ++s2) y += red[s2 * d + c];
        if (with_mu) y += stats[bg * 4 + 2] * to_f(mu[static_cast<size_t>(h) * d + c]);
        out[bg * d + c] = from_f<T>(y);
    }
    if (threadIdx.x == 0 && lse) lse[bg] = mx + __logf(stats[bg * 4 + 1]);
}

// ---- compress: key rows by the mask (Sec. 3.1, Keys) ----------------------------------------
template <class T>
__global__ void g_gather(const T *__restrict__ K, const int32_t *__restrict__ idx,
                         T *__restrict__ Kc, int64_t sb, int64_t sh, int64_t ss, int Hkv, int d,
                         int n, int m, int I, int vis0)
{
    const size_t bh = blockIdx.z;
    const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
    const int i = blockIdx.y, j = blockIdx.x;
    const int row = min(max(idx[j], 0), n - 1);              // an index outside the block must not leave it
    const T *src = K + b * sb + h * sh + (static_cast<int64_t>(vis0) + static_cast<int64_t>(i) * n + row) * ss;
    T *dst = Kc + ((bh * I + i) * m + j) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = src[c];
}

// ---- compress: centred values onto the PCA basis (Sec. 3.1, Values) -------------------------
// Vc[b,h,i,j,c] = sum_p U[h,j,p] (V[p,c] - mu[h,c]);  grid = (j groups of kJV, I, B*Hkv)
constexpr int kJV = 8;
template <class T>
__global__ void g_vproject(const T *__restrict__ V, const T *__restrict__ U,
                           const T *__restrict__ mu, T *__restrict__ Vc, int64_t sb, int64_t sh,
                           int64_t ss, int Hkv, int d, int n, int m, int I, int vis0)
{
    const size_t bh = blockIdx.z;
    const int b = static_cast<int>(bh / Hkv), h = static_cast<int>(bh % Hkv);
    const int i = blockIdx.y, j0 = blockIdx.x * kJV;
    const int c = threadIdx.x;
    if (c >= d) return;
    const T *Vb = V + b * sb + h * sh + (static_cast<int64_t>(vis0) + static_cast<int64_t>(i) * n) * ss + c;
    const T *Ub = U + (static_cast<size_t>(h) * m + j0) * n;
    const float muc = to_f(mu[static_cast<size_t>(h) * d + c]);
    const int jn = min(kJV, m - j0);
    float acc[kJV];
#pragma unroll
    for (int jj = 0; jj < kJV; ++jj) acc[jj] = 0.f;
    for (int p = 0; p < n; ++p) {
        const float v = to_f(Vb[static_cast<int64_t>(p) * ss]) - muc;
#pragma unroll
        for (int jj = 0; jj < kJV; ++jj)
            if (jj < jn) acc[jj] += to_f(Ub[static_cast<size_t>(jj) * n + p]) * v;
    }
    for (int jj = 0; jj < jn; ++jj)
        Vc[(bh * I + i) * m * d + vc_offset(j0 + jj, c, m, d)] = from_f<T>(acc[jj]);
}

// ---- first layer of the two-layer key reconstructor (Sec. 3.1, Keys) --------------------------------
// H[b,h,i,r,c] = act(sum_j W1[h,j,r] Kc[b,h,i,j,c]);  grid = (r groups of kRH, I, B*Hkv), a thread per channel
constexpr int kRH = 8;
__device__ inline float act_apply(float x, int act)
{
    if (act == 1) return fmaxf(x, 0.f);
    if (act == 2) return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));     // GELU, erf form
    return x;
}
template <class T>
__global__ void g_mlp_hidden(const T *__restrict__ Kc, const T *__restrict__ W1, T *__restrict__ H, int Hkv, int d,
                             int m, int I, int act)
{
    const size_t bh = blockIdx.z;
    const int h = static_cast<int>(bh % Hkv), i = blockIdx.y, r0 = blockIdx.x * kRH;
    const int c = threadIdx.x;
    if (c >= d) return;
    const T *Kb = Kc + (bh * I + i) * static_cast<size_t>(m) * d + c;
    const T *Wb = W1 + static_cast<size_t>(h) * m * m + r0;
    const int rn = min(kRH, m - r0);
    float acc[kRH];
#pragma unroll
    for (int rr = 0; rr < kRH; ++rr) acc[rr] = 0.f;
    for (int j = 0; j < m; ++j) {
        const float k = to_f(Kb[static_cast<size_t>(j) * d]);
#pragma unroll
        for (int rr = 0; rr < kRH; ++rr)
            if (rr < rn) acc[rr] += to_f(Wb[static_cast<size_t>(j) * m + rr]) * k;
    }
    for (int rr = 0; rr < rn; ++rr)
        H[((bh * I + i) * static_cast<size_t>(m) + r0 + rr) * d + c] = from_f<T>(act_apply(acc[rr], act));
}

struct GenericWs {
    float *Svis, *Stxt, *L, *stats, *W;
    size_t bytes;
};

GenericWs carve(const kvc_shape &s, int32_t max_text, void *base)
{
    const size_t rows = static_cast<size_t>(s.batch) * s.n_q_heads;
    const size_t Im = static_cast<size_t>(s.n_images) * s.m;
    const size_t In = static_cast<size_t>(s.n_images) * s.n_img_tokens;
    size_t off = 0;
    auto take = [&](size_t floats) {
        size_t o = off;
        off += align_up(floats * sizeof(float), 256);
        return reinterpret_cast<float *>(static_cast<char *>(base) + o);
    };
    GenericWs w;
    w.Svis = take(rows * Im);
    w.Stxt = take(rows * static_cast<size_t>(max_text > 0 ? max_text : 1));
    w.L = take(rows * In);
    w.stats = take(rows * 4);
    w.W = take(rows * Im);
    w.bytes = off;
    return w;
}

template <class T> kvc_status decode_t(const DecodeCall &c)
{
    const kvc_shape &s = c.s;
    const int B = s.batch, Hq = s.n_q_heads, Hkv = s.n_kv_heads, d = s.head_dim;
    const int n = s.n_img_tokens, I = s.n_images, m = s.m;
    const int Im = I * m, t = c.t;
    GenericWs w = carve(s, c.cap, c.ws);
    const int tstride = c.cap > 0 ? c.cap : 1;
    const int append = c.k_new ? 1 : 0;
    if (c.k_new)
        g_append<T><<<B * Hkv, 64, 0, c.stream>>>(static_cast<T *>(c.Kt), static_cast<T *>(c.Vt),
                                                  static_cast<const T *>(c.k_new),
                                                  static_cast<const T *>(c.v_new), d, c.cap, c.t_in, Hkv, c.text_len_dev);
    const int rows = Im + t;
    int gx = (rows + kWaves - 1) / kWaves;
    if (gx > 4096) gx = 4096;
    g_scores<T><<<dim3(gx, B * Hkv), kThreads, 0, c.stream>>>(
        static_cast<const T *>(c.q), static_cast<const T *>(c.Kc), static_cast<const T *>(c.Kt),
        w.Svis, w.Stxt, Hq, Hkv, d, Im, t, c.cap, tstride, c.scale, m, c.n_images_dev, c.text_len_dev, append);
    if (c.static_variant) {
        // the compressed rows are the vision keys and values themselves: softmax over [Svis ; Stxt]
        g_stats<<<B * Hq, kThreads, 0, c.stream>>>(w.Svis, w.Stxt, w.stats, Im, t, tstride);
        if (Im > 0)
            g_static_weights<<<dim3((Im + kThreads - 1) / kThreads, B * Hq), kThreads, 0, c.stream>>>(w.Svis, w.stats, w.W, Im);
    } else {
        if (I > 0) {
            g_expand<T><<<dim3((n + kThreads - 1) / kThreads, I, B * Hq), kThreads, m * sizeof(float),
                          c.stream>>>(w.Svis, static_cast<const T *>(c.theta), w.L, Hq, Hkv, n, m, I, c.n_images_dev);
        }
        g_stats<<<B * Hq, kThreads, 0, c.stream>>>(w.L, w.Stxt, w.stats, I * n, t, tstride);
        if (I > 0) {
            g_project<T><<<dim3((m + kJB - 1) / kJB, I, B * Hq), kThreads, n * sizeof(float), c.stream>>>(
                w.L, w.stats, static_cast<const T *>(c.U), w.W, Hq, Hkv, n, m, I);
        }
    }
    g_output<T><<<B * Hq, kThreads, 0, c.stream>>>(
        w.W, w.Stxt, w.stats, static_cast<const T *>(c.Vc), static_cast<const T *>(c.Vt),
        static_cast<const T *>(c.mu), static_cast<T *>(c.out), c.lse, Hq, Hkv, d, Im, m, t, c.cap,
        tstride, c.n_images_dev, c.text_len_dev, append, c.static_variant ? 0 : 1);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

template <class T> kvc_status compress_t(const CompressCall &c)
{
    const kvc_shape &s = c.s;
    if (s.n_images == 0) return KVC_OK;
    const int B = s.batch, Hkv = s.n_kv_heads, d = s.head_dim;
    const int n = s.n_img_tokens, I = s.n_images, m = s.m;
    g_gather<T><<<dim3(m, I, B * Hkv), 64, 0, c.stream>>>(
        static_cast<const T *>(c.K), c.key_idx, static_cast<T *>(c.Kc), c.stride_b, c.stride_h,
        c.stride_s, Hkv, d, n, m, I, c.vis_start);
    g_vproject<T><<<dim3((m + kJV - 1) / kJV, I, B * Hkv), ((d + 63) / 64) * 64, 0, c.stream>>>(
        static_cast<const T *>(c.V), static_cast<const T *>(c.U), static_cast<const T *>(c.mu),
        static_cast<T *>(c.Vc), c.stride_b, c.stride_h, c.stride_s, Hkv, d, n, m, I, c.vis_start);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace

size_t generic_decode_ws_bytes(const kvc_shape &s, int32_t max_text)
{
    return carve(s, max_text, nullptr).bytes;
}

kvc_status generic_decode(const DecodeCall &c)
{
    // dynamic LDS of g_expand / g_project holds one row of m / n floats
    if (static_cast<size_t>(c.s.n_img_tokens) * sizeof(float) > 64 * 1024) return KVC_ERR_UNSUPPORTED;
    if (carve(c.s, c.cap, nullptr).bytes > c.ws_bytes) return KVC_ERR_WORKSPACE;
    return c.s.dtype == KVC_F32 ? decode_t<float>(c) : decode_t<bf16_t>(c);
}

kvc_status generic_mlp_hidden(const kvc_shape &s, const void *W1, int act, const void *Kc, void *H, hipStream_t stream)
{
    if (s.n_images == 0) return KVC_OK;
    const dim3 grid((s.m + kRH - 1) / kRH, s.n_images, s.batch * s.n_kv_heads);
    const int threads = ((s.head_dim + 63) / 64) * 64;
    if (s.dtype == KVC_F32)
        g_mlp_hidden<float><<<grid, threads, 0, stream>>>(static_cast<const float *>(Kc), static_cast<const float *>(W1),
                                                          static_cast<float *>(H), s.n_kv_heads, s.head_dim, s.m, s.n_images, act);
    else
        g_mlp_hidden<bf16_t><<<grid, threads, 0, stream>>>(static_cast<const bf16_t *>(Kc), static_cast<const bf16_t *>(W1),
                                                           static_cast<bf16_t *>(H), s.n_kv_heads, s.head_dim, s.m, s.n_images, act);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

kvc_status generic_compress(const CompressCall &c)
{
    return c.s.dtype == KVC_F32 ? compress_t<float>(c) : compress_t<bf16_t>(c);
}

}  // namespace kvc
