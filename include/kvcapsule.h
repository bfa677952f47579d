/*
 * kvcapsule.h -- C ABI of the KVCapsule hot path on AMD MI355X (gfx950).
 *
 * KVCapsule (arxiv 2605.16439) keeps, per transformer layer, the vision-token
 * part of the KV cache in a compact "capsule": keys by row selection with a
 * learned mask M, values by a projection onto a sequence-axis PCA basis U after
 * centring with mu (Sec. 3.1).  At every decode step the full-length vision K/V
 * is reconstructed (keys with the reconstructor theta, values with U^T and mu)
 * and the unmodified softmax attention runs over [vision ; text] (Sec. 3.2).
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    never allocates, frees or keeps them; scratch memory comes in through the
 *    `workspace` argument (size from kvc_workspace_bytes).
 *  - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and return without synchronising.  Calls that share a
 *    workspace must be ordered on one stream.
 *  - The first call for a kernel variant on a device also sets a function
 *    attribute (dynamic LDS limit) and asks the runtime for the variant's
 *    occupancy; every later call consists of kernel launches only.  No call
 *    allocates, copies, sets memory or synchronises, so every call, the first
 *    included, may be captured into a HIP graph.
 *  - The library keeps no state between calls: what a call needs beyond its arguments lives in the
 *    workspace (its first 64 KB hold arrival counters of the decode kernels; their contents need not be
 *    initialised and may be overwritten between calls).  Calls that share a workspace must not overlap:
 *    order them on one stream -- this includes replays of captured calls.  Calls with workspaces of their
 *    own may run concurrently on any number of streams.
 *  - Tensors are dense row-major with head_dim fastest unless strides are
 *    passed.  Every pointer must be 16-byte aligned.
 *  - The return value is a kvc_status.  Argument errors (every negative status but KVC_ERR_HIP) are
 *    found before anything touches the device: nothing was launched.  KVC_ERR_HIP reports a failed
 *    launch; kernels of the same call that were launched before it still run, and the outputs are then
 *    undefined.  No exception crosses the boundary.
 *  - Notation follows the paper: B batch, H_q query heads, H_kv KV heads,
 *    G = H_q / H_kv (query head g reads KV head g / G), d = head_dim, n vision
 *    tokens per image block, I image blocks (the vision span is I*n contiguous
 *    tokens; the same per-layer parameters serve every block and every batch
 *    element), m = ceil((1 - c) n) compressed length for compression ratio c,
 *    t text tokens in the cache.
 *  - The matrix-core (MFMA) kernels cover bf16 with d = 128: compression for n a multiple of 64;
 *    decode for n in {256, 576, 1024}, G in {1, 2, 4, 6, 7, 8} and at most 256 partial results per
 *    (batch element, KV head).  Other shapes, and fp32, run shape-agnostic scalar kernels: same results
 *    within rounding, far lower speed; their decode is limited to n <= 16384 (KVC_ERR_UNSUPPORTED beyond).
 */
#ifndef KVCAPSULE_H
#define KVCAPSULE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVC_OK = 0,
    KVC_ERR_NULL = -1,        /* a required pointer is NULL                          */
    KVC_ERR_SHAPE = -2,       /* a size or index is out of range or inconsistent     */
    KVC_ERR_DTYPE = -3,       /* unknown element type                                */
    KVC_ERR_ALIGN = -4,       /* a pointer or stride breaks the 16-byte rule         */
    KVC_ERR_WORKSPACE = -5,   /* workspace missing or smaller than required          */
    KVC_ERR_UNSUPPORTED = -6, /* valid but not implemented (e.g. head_dim > 256)     */
    KVC_ERR_HIP = -7          /* the HIP runtime reported a launch error             */
} kvc_status;

typedef enum { KVC_F32 = 0, KVC_BF16 = 1 } kvc_dtype;

/* One LAYER's problem. */
typedef struct {
    int32_t batch;         /* B >= 1                                                 */
    int32_t n_q_heads;     /* H_q, a multiple of n_kv_heads                          */
    int32_t n_kv_heads;    /* H_kv >= 1                                              */
    int32_t head_dim;      /* d, a multiple of 8, at most 256                        */
    int32_t n_img_tokens;  /* n >= 1: vision tokens of one image block               */
    int32_t n_images;      /* I >= 0: number of blocks in the vision span            */
    int32_t m;             /* compressed length, 1 <= m <= n (per layer, so a        */
                           /* pyramid schedule is a sequence of calls with own m)    */
    int32_t dtype;         /* kvc_dtype of K, V, q, out, capsule and parameters;     */
                           /* accumulation is always fp32                            */
} kvc_shape;

/* Per-layer learned parameters, fixed at inference (Sec. 3.2). */
typedef struct {
    const int32_t *key_idx; /* M : [m] strictly ascending indices in [0, n); shared  */
                            /* by heads, blocks and batch (Sec. 3.1, Keys).  Lives   */
                            /* in device memory, so it is not validated: an entry    */
                            /* outside [0, n) is the caller's error and is read as   */
                            /* the nearest row of the block.  Unused by decode.      */
    const void *theta;      /* theta : [H_kv][m][n] key / score reconstructor        */
                            /* (App. C; applied to scores in Alg. 1 step 2)          */
    const void *U;          /* U : [H_kv][m][n] value PCA basis (Sec. 3.1, Values)   */
    const void *mu;         /* mu : [H_kv][d] value centre (Sec. 3.1, Values)        */
    const void *theta_packed; /* optional (may be NULL): theta re-tiled once by      */
                            /* kvc_pack_theta, same size; decode calls whose shape   */
                            /* has a one-pass kernel use it (together with U_packed),*/
                            /* all others read theta.                                */
                            /* Unused by compress.                                   */
    const void *U_packed;   /* optional (may be NULL): U re-tiled once by kvc_pack_u */
                            /* for the decode side, same size.  The one-pass decode  */
                            /* kernel runs when BOTH packed forms are given; U       */
                            /* itself stays required (compress and the other decode  */
                            /* kernels read it), so a caller who opts in keeps       */
                            /* H_kv m n more elements per layer.                     */
} kvc_params;

/* |M| = ceil(l_r n) with retention l_r = 1 - compression_ratio (Sec. 3.1, Keys),
 * clamped to [1, n]; products that are integers in exact arithmetic do not round
 * up.  Host arithmetic only.  Returns 0 for n <= 0. */
int32_t kvc_compressed_len(int32_t n, double compression_ratio);

/* Bytes of scratch that kvc_compress and kvc_reconstruct_attend_decode need for
 * this shape with up to max_text_len cached text rows (new token included).
 * Host arithmetic only.  Returns 0 if the shape is invalid. */
size_t kvc_workspace_bytes(const kvc_shape *shape, int32_t max_text_len);

/* Persistent bytes of one layer, App. C eq. (1) (full cache) and eq. (2) (capsule
 * + parameter overhead), for c_prompt + t text rows around the I*n vision tokens.
 * Host arithmetic only; either output pointer may be NULL. */
kvc_status kvc_memory_footprint(const kvc_shape *shape, int64_t c_prompt, int64_t t,
                                int64_t *bytes_full_cache, int64_t *bytes_capsule);

/* Compress one layer's vision K/V into the capsule (Sec. 3.1; Sec. 3.2
 * "Prefilling Stage"):
 *     Kc[b,h,i,j,:] = K[b,h, vis_start + i n + M[j], :]            (bit-exact copy)
 *     Vc[b,h,i,j,:] = sum_p U[h,j,p] (V[b,h, vis_start + i n + p, :] - mu[h,:])
 * with fp32 accumulation and one round-to-nearest-even to the storage type.
 *  K, V  in : [B][H_kv][S][d], S = seq_len, with element strides stride_b / stride_h /
 *             stride_s (d contiguous; strides multiples of 8 elements); rows outside the
 *             span [vis_start, vis_start + I n) are not touched -- text K/V stays
 *             where the backbone keeps it.  The span must lie inside the S rows.
 *  Kc out  : [B][H_kv][I][m][d] dense.
 *  Vc out  : [B][H_kv][I] records of m*d elements (no padding).  Inside a record the m rows
 *            are grouped in blocks of 8 and a block is stored channel-major, [d][w] with
 *            w = 8 (w = m % 8 for a shorter last block): element (row j, channel c) sits at
 *            (j/8)*8*d + c*w + j%8.  Eight consecutive rows of one channel are then 16
 *            contiguous bytes, which is the matrix-core operand of the decode kernel.
 * Errors: NULL pointers, bad shape/dtype, vis_start < 0, vis_start + I n > seq_len,
 * misalignment. */
kvc_status kvc_compress(const kvc_shape *shape, const kvc_params *params,
                        const void *K, const void *V,
                        int64_t stride_b, int64_t stride_h, int64_t stride_s,
                        int32_t vis_start, int32_t seq_len,
                        void *Kc, void *Vc,
                        void *workspace, size_t workspace_bytes, void *stream);

/* One decode step of one layer (Sec. 3.2 "Decoding Stage"): attention of one new
 * query token per sequence over the reconstructed vision K/V and the text cache,
 *     K_hat[b,h,i] = theta[h]^T Kc[b,h,i]            V_hat[b,h,i] = U[h]^T Vc[b,h,i] + 1 mu[h]^T
 *     out[b,g,:]   = softmax(scale * q[b,g] . [K_hat[b,g/G] ; K_text[b,g/G]]^T) [V_hat ; V_text]
 * evaluated in the score-space order of Alg. 1 (scores on the compressed keys,
 * expanded with theta, probabilities folded through U^T), which never forms
 * K_hat / V_hat in memory; the softmax is joint over vision and text keys.
 *  q        in : [B][H_q][d]
 *  Kc, Vc   in : capsule written by kvc_compress (Vc in its blocked layout)
 *  K_text, V_text in/out: [B][H_kv][text_cap][d], first text_len rows valid; may
 *             be NULL when text_cap == 0
 *  k_new, v_new in (optional, both or neither): [B][H_kv][d]; if given they are
 *             stored at row text_len of the text cache and attended, which needs
 *             text_len + 1 <= text_cap
 *  softmax_scale: sigma of Alg. 1; 0 selects 1/sqrt(d)
 *  out      out: [B][H_q][d]
 *  lse_out  out (optional): [B][H_q] float, log of the softmax denominator -- what a
 *             caller needs to merge partial results of a sequence split
 * Errors: NULL pointers, bad shape/dtype, text_len outside [0, text_cap], no key at
 * all (I == 0 and no text row), misalignment, workspace too small. */
kvc_status kvc_reconstruct_attend_decode(const kvc_shape *shape, const kvc_params *params,
                                         const void *q, const void *Kc, const void *Vc,
                                         void *K_text, void *V_text,
                                         int32_t text_len, int32_t text_cap,
                                         const void *k_new, const void *v_new,
                                         float softmax_scale,
                                         void *out, float *lse_out,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* theta re-tiled for the matrix cores, once at load time (the survey of the method allows a packed
 * copy of the parameters that is no larger than the original; App. C counts theta as H_kv m n
 * elements, and so does this form).  Alg. 1 step 2 contracts the scores with theta over its ROW index
 * j, which is the slow index of [H_kv][m][n]; the packed form makes 8 consecutive rows of one position
 * 16 contiguous bytes, so that a matrix-core operand is one load:
 *   per KV head one record of exactly m n elements; rows in blocks of 8, each block position-major
 *   [n][w] with w = 8 (w = m mod 8 for the last, shorter block); element (j, pos) sits at
 *   kvc_capsule_value_offset(j, pos, m, n) within the record (the layout of the compressed values
 *   with positions in place of channels).
 *  theta in: [H_kv][m][n]; packed out: same size, a different buffer; both device memory, element type
 *  of the shape.  Pass the result as kvc_params.theta_packed (theta itself stays required: shapes
 *  without a one-pass kernel read it).
 * Errors: NULL pointers, bad shape, theta == packed, misalignment. */
kvc_status kvc_pack_theta(const kvc_shape *shape, const void *theta, void *packed, void *stream);

/* The same for U on the decode side.  Alg. 1 step 3 contracts the probabilities with U over the POSITION
 * index; a matrix-core operand (8 consecutive positions of one row j) is 16 contiguous bytes of [H_kv][m][n]
 * already, but the 16 rows of a tile are n elements apart, and loads of that shape run at a fifth of the
 * rate of whole lines.  The packed form puts the 16-byte pieces of consecutive ROWS next to each other:
 *   per KV head one record of m n elements; positions in blocks of 8, each block row-major [m][8];
 *   element (j, pos) sits at kvc_capsule_value_offset(pos, j, n, m) (the layout of kvc_pack_theta with the
 *   roles of rows and positions exchanged).  n must be a multiple of 8.
 * Pass the result as kvc_params.U_packed.  Errors: as kvc_pack_theta; n % 8 != 0 is KVC_ERR_UNSUPPORTED. */
kvc_status kvc_pack_u(const kvc_shape *shape, const void *U, void *packed, void *stream);

/* Ragged batch: the decode step for sequences with their own numbers of image blocks and text rows.
 * Sequence b attends the first n_images[b] of its I = shape->n_images capsule slots and text_len[b]
 * text rows; with k_new / v_new its new token is stored at row text_len[b] first.  The paper states
 * the method per image "with size n" and is silent on batching; the same per-layer parameters serve
 * every block as in the uniform call.
 *  n_images, text_len in: DEVICE arrays [B] of int32; the host cannot see their values, so they are
 *             clamped on the device to [0, I] and [0, text_cap] ([0, text_cap - 1] with a new token).
 *             A sequence left with no key at all gets NaNs.
 * Everything else as in kvc_reconstruct_attend_decode, the kernels included (matrix cores for the shapes
 * that have them, the one-pass kernel with kvc_params.theta_packed; a uniform batch gives the uniform call's result bit for bit).  Capsule slots beyond
 * n_images[b] may be read but never reach the result, whatever they hold (NaNs included); text rows
 * beyond the sequence's own are not read.
 * Errors: as kvc_reconstruct_attend_decode, plus NULL / misaligned count arrays, text_cap < 1. */
kvc_status kvc_reconstruct_attend_decode_ragged(const kvc_shape *shape, const kvc_params *params,
                                                const void *q, const void *Kc, const void *Vc,
                                                void *K_text, void *V_text,
                                                const int32_t *n_images, const int32_t *text_len,
                                                int32_t text_cap,
                                                const void *k_new, const void *v_new, float softmax_scale,
                                                void *out, float *lse_out,
                                                void *workspace, size_t workspace_bytes, void *stream);

/* Two-layer form of the key reconstructor (Sec. 3.1, Keys: f_theta "implemented as a two-layer MLP"),
 * read as acting along the sequence axis per KV head with hidden width m and no bias:
 *     K_hat = W2^T act(W1^T K_tilde).
 * The first layer depends on the compressed keys only, not on the decode step, so it is applied once,
 * after kvc_compress, and its result is kept in place of K_tilde (same size):
 *     H[b,h,i,r,:] = act( sum_j W1[h,j,r] Kc[b,h,i,j,:] ),   r < m,   rounded once to the storage type.
 * The decode step is then kvc_reconstruct_attend_decode with Kc = H and theta = W2 (the second layer is
 * the linear reconstruction).  With KVC_ACT_IDENTITY this is the linear form with theta = W1 W2.
 *  W1 in : [H_kv][m][m] (row j, column r), element type of the shape;  Kc in, H out: [B][H_kv][I][m][d],
 *          different buffers.
 * Runs on a scalar kernel (a one-off step of the prefill).
 * Errors: NULL pointers, bad shape / activation, Kc == H, misalignment. */
typedef enum { KVC_ACT_IDENTITY = 0, KVC_ACT_RELU = 1, KVC_ACT_GELU = 2 /* 0.5 x (1 + erf(x / sqrt 2)) */ } kvc_activation;
kvc_status kvc_mlp_hidden(const kvc_shape *shape, const void *W1, int32_t activation,
                          const void *Kc, void *H, void *stream);

/* Static variant of the paper's ablation (App. "Static Compression vs. Reconstruction-before-Attention":
 * reconstruction disabled, the compressed KV used directly throughout decoding): plain attention over
 * the I*m compressed rows of each (batch element, KV head) and the text rows,
 *     out[b,g,:] = softmax(scale * q[b,g] . [Kc[b,g/G] ; K_text]^T) [Vc[b,g/G] ; V_text],
 * no theta, no U^T, no mu.  Arguments as in kvc_reconstruct_attend_decode (Vc in its blocked layout;
 * shape->n_img_tokens is not used).  Runs on the shape-agnostic scalar kernels. */
kvc_status kvc_static_attend_decode(const kvc_shape *shape, const void *q, const void *Kc, const void *Vc,
                                    void *K_text, void *V_text, int32_t text_len, int32_t text_cap,
                                    const void *k_new, const void *v_new, float softmax_scale,
                                    void *out, float *lse_out,
                                    void *workspace, size_t workspace_bytes, void *stream);

/* The blocked layout of the compressed values (see kvc_compress), for code that has to read or build a
 * capsule: offset, in elements from the start of an image block's record of m*d elements, of (row j,
 * channel c).  Host arithmetic only; returns -1 if an argument is out of range. */
int64_t kvc_capsule_value_offset(int32_t j, int32_t c, int32_t m, int32_t d);

/* Compressed values of `records` image blocks (B*H_kv*I of them, as kvc_compress wrote them) -> dense
 * row-major [records][m][d], same element type.  Index shuffling only; asynchronous on `stream`.
 * Errors: NULL pointers, bad sizes, unknown dtype, misalignment. */
kvc_status kvc_unpack_values(const void *Vc, void *dense, int64_t records, int32_t m, int32_t d,
                             int32_t dtype, void *stream);

/* For callers that cannot allocate or hand over device memory at call time (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): kvc_reconstruct_attend_decode
 * without the workspace arguments.  Same operation, same kernels, same results; the scratch lives in a
 * device array inside the library, kvc_static_scratch_bytes() = 32 MiB per GPU, held until the process
 * ends.  The call allocates nothing and frees nothing.  A shape whose kvc_workspace_bytes(shape,
 * text_cap) exceeds that size is refused with KVC_ERR_WORKSPACE before anything is launched (the five
 * benchmark configurations fit).  Every call on a GPU shares that GPU's one array: calls that overlap
 * on one GPU (two streams, overlapping graph replays) race on it and must be ordered by the caller;
 * the array keeps the previous call's contents, none of which a later call relies on. */
size_t kvc_static_scratch_bytes(void);
kvc_status kvc_reconstruct_attend_decode_static(const kvc_shape *shape, const kvc_params *params,
                                                const void *q, const void *Kc, const void *Vc,
                                                void *K_text, void *V_text,
                                                int32_t text_len, int32_t text_cap,
                                                const void *k_new, const void *v_new,
                                                float softmax_scale,
                                                void *out, float *lse_out, void *stream);

/* Full-cache ("All KV") decode attention: the comparison point of the paper's efficiency analysis
 * (Sec. 4; "All KV" rows of Fig. 5) -- the same decode step without KVCapsule.  One new query token
 * per sequence attends every row of the uncompressed cache (vision and text alike),
 *     out[b,g,:] = softmax(scale * q[b,g] . K[b,g/G,:t]^T) V[b,g/G,:t]      (Sec. 3.1, attention equation)
 * after the new token's k, v have been stored at row kv_len (t = kv_len + 1 then; t = kv_len when
 * k_new / v_new are NULL).
 *  q        in : [B][H_q][d]
 *  K, V  in/out: [B][H_kv][kv_cap][d] with element strides stride_b / stride_h / stride_s (d
 *             contiguous; strides multiples of 8 elements), first kv_len rows valid
 *  k_new, v_new in (optional, both or neither): [B][H_kv][d], needs kv_len + 1 <= kv_cap
 *  softmax_scale: 0 selects 1/sqrt(d)
 *  out      out: [B][H_q][d];  lse_out out (optional): [B][H_q] float
 *  workspace : kvc_attend_full_workspace_bytes(...) bytes, 256-byte aligned
 * bf16 with d = 128 and G <= 16 runs a split-KV matrix-core kernel (any strides); other shapes run
 * the scalar kernels and need a dense cache (KVC_ERR_UNSUPPORTED otherwise).
 * Errors: NULL pointers, bad sizes, kv_len outside [0, kv_cap], no key at all, misalignment,
 * workspace too small. */
size_t kvc_attend_full_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                       int32_t head_dim, int32_t dtype, int32_t max_kv_len);
kvc_status kvc_attend_full_decode(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                  int32_t dtype, const void *q, void *K, void *V,
                                  int64_t stride_b, int64_t stride_h, int64_t stride_s,
                                  int32_t kv_len, int32_t kv_cap,
                                  const void *k_new, const void *v_new, float softmax_scale,
                                  void *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Static string for a status code. */
const char *kvc_status_string(int32_t status);

/* Library version, "major.minor". */
const char *kvc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVCAPSULE_H */
