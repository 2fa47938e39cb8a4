/*
 * dab.h - C ABI of the MI355X (gfx950) hot path of distribution-aware
 * binarization, after "Distribution-Aware Binarization of Neural Networks for
 * Sketch Recognition" (arXiv 1804.02941).
 *
 * The path: a layer's real-valued filters W_f (n = c*w*h weights each) are
 * replaced by W~_f = alpha_f*e_f + beta_f*(1 - e_f) with a 0/1 mask e_f
 * (Section 4.1, Theorem 2); the mask comes from a split of the sorted weights
 * found with prefix sums (Section 4.3.1, Algorithm 1); inputs of the layer are
 * binary, +1 / -1 (Section 4); the layer output is the ordinary convolution of
 * the binary input with W~ (Section 4.3.2).  Since W~ takes two values,
 *     y = alpha*s1 + beta*s2,  s1 = sum a_i e_i,  s2 = sum a_i (1 - e_i),
 * over the taps inside the image, with s1 + s2 = sA = sum a_i.  One bit per
 * weight and per activation is what crosses this interface; s1 is an exact
 * integer contraction of the two bit tensors and the two scalars recombine it
 * with the per-pixel sum sA.
 *
 * General rules
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *     The caller owns every buffer; the library allocates nothing and never
 *     frees or retains a pointer.  Its only state is a one-time set-up per
 *     device (dab_init), which every entry point that needs it performs on
 *     its first call on that device.
 *   - "stream" is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued on it and the call returns without synchronising.
 *   - Every call returns a dab_status.  Arguments are validated on the host
 *     before anything is enqueued: on DAB_ERR_NULL, _SHAPE, _ALIGN, _WORKSPACE
 *     and _UNSUPPORTED nothing was launched.  A failing launch gives
 *     DAB_ERR_HIP (the status of that launch call, kept for
 *     dab_last_hip_error()); kernels of the same call enqueued before it
 *     stay enqueued and only write the call's own outputs and workspace.
 *     Faults inside a kernel surface at the caller's next synchronisation,
 *     as with any HIP work.
 *   - Float buffers are fp32, 4-byte aligned; packed buffers and Y are
 *     16-byte aligned (DAB_ERR_ALIGN otherwise).
 *   - Inputs must be finite.  A NaN activation binarizes to -1 (x >= tau is
 *     false); NaN weights give unspecified masks.
 *
 * Packed layouts (bit k of a word = (word >> k) & 1, least significant first)
 *   Activations  uint32 [B][H][W][Cw], Cw = ceil(C/32).  Bit (c mod 32) of
 *                word (c div 32) of pixel (b,h,w) is 1 iff a[b,c,h,w] = +1.
 *                Bits past C are 0.  A fully-connected input is H = W = 1.
 *   Weights      uint32 [R][Fp], R = kh*kw*Cw, Fp = 64*ceil(F/64).  Row
 *                r = (ky*kw + kx)*Cw + (c div 32), column f, bit (c mod 32) is
 *                e[f,c,ky,kx].  Bits past C and columns past F are 0.
 *                (Word-major: the word of one reduction position is contiguous
 *                over the filters, which is how both packing and expansion walk it.)
 *   Tap counts   uint32 [F][kh*kw]: ecnt[f][ky*kw+kx] = sum_c e[f,c,ky,kx]; their sum
 *                over the taps is K_f.  They describe the mask (and check it); the
 *                layer kernels do not need them.
 */
#ifndef DAB_H
#define DAB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dab_status {
    DAB_OK = 0,
    DAB_ERR_NULL = 1,        /* a required pointer is NULL                          */
    DAB_ERR_SHAPE = 2,       /* a size is non-positive, n < 2, or the output empty  */
    DAB_ERR_ALIGN = 3,       /* a buffer is not aligned as stated above             */
    DAB_ERR_WORKSPACE = 4,   /* ws is NULL or smaller than the *_workspace_bytes    */
    DAB_ERR_UNSUPPORTED = 5, /* valid problem outside what the kernels cover        */
    DAB_ERR_HIP = 6          /* a HIP call failed; see dab_last_hip_error()         */
} dab_status;

typedef enum dab_layout {
    DAB_LAYOUT_NHWC = 0,     /* X[b][h][w][c], the native layout                    */
    DAB_LAYOUT_NCHW = 1      /* X[b][c][h][w], packed through a transposing kernel  */
} dab_layout;

/* One binarized convolution.  Output size Ho = (H + 2*pad_h - kh)/stride_h + 1,
 * Wo likewise; both must be >= 1. */
typedef struct dab_conv_desc {
    int32_t B, C, H, W;                 /* input: batch, channels, height, width */
    int32_t F, kh, kw;                  /* filters and their spatial extent      */
    int32_t pad_h, pad_w;               /* zero padding on each side             */
    int32_t stride_h, stride_w;
} dab_conv_desc;

/* Text for a status code (static storage, never NULL). */
const char* dab_strerror(int status);

/* hipError_t of the last failed HIP call made by this thread (0 if none). */
int dab_last_hip_error(void);

/*
 * dab_init - one-time set-up of the current device: raises the dynamic-LDS limit of the kernels
 * that stage more than the default 48 KB and looks up the address of the library's own device
 * memory.  Optional: entry points that depend on it do the same on their first call on a device.
 * Callers that capture a stream into a graph call it before the capture begins, so that no
 * attribute call falls inside it.  Thread-safe; later calls return at once.
 */
int dab_init(void);

/*
 * dab_estimate_alpha_beta - optimal alpha, beta, K and split of every filter.
 * Section 4.1 (Theorem 2) and Section 4.3.1 / Algorithm 1: sort the n weights
 * of a filter, form prefix sums P_i, score every split i = 1..n-1 with
 * D_i = P_i^2/i + (T - P_i)^2/(n - i), take the largest i of maximal D.  The
 * lower group is the i smallest weights (ties by original index), the upper
 * group the rest; alpha is the mean of the group whose mean has the greater
 * magnitude (the upper group if equal), beta the other mean, K the size of
 * the alpha group.  Sums and scores are accumulated in fp64; alpha and beta
 * are rounded to fp32 at the end.
 *
 *   W              [F][n] fp32, row f = filter f flattened in (c,ky,kx) order
 *   alpha, beta    [F] fp32 out
 *   K              [F] int32 out, 1 <= K <= n-1
 *   thr_val        [F] fp32 out: value of the largest element of the lower group
 *   thr_idx        [F] int32 out: its index in the row; element i is in the lower
 *                  group iff w_i < thr_val or (w_i == thr_val and i <= thr_idx)
 *   alpha_is_upper [F] uint8 out: 1 if the alpha group is the upper group
 *   ws, ws_bytes   scratch of at least dab_estimate_workspace_bytes(F, n) bytes (one flag per
 *                  filter for rows of 4096 weights and more, nothing for shorter rows).
 *                  Rows of more than 256 weights are estimated without a full sort: value
 *                  buckets with exact integer sums give D at every bucket end and an
 *                  upper bound inside every bucket, and only the few elements of the
 *                  buckets that can hold the arg-max are ranked exactly; rows where that
 *                  does not apply (many equal values) are sorted, the long ones through
 *                  their flag in ws by a second kernel.  The result is the same split.
 *                  ws may be NULL (or too small): then every long row is sorted.
 * Errors: NULL pointers, F < 1 or n < 2 (a filter needs both groups non-empty)
 * -> DAB_ERR_SHAPE; n above the largest supported row (dab_estimate_max_n())
 * -> DAB_ERR_UNSUPPORTED.
 */
int dab_estimate_alpha_beta(const float* W, int32_t F, int32_t n,
                            float* alpha, float* beta, int32_t* K,
                            float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper,
                            void* ws, size_t ws_bytes, void* stream);
size_t dab_estimate_workspace_bytes(int32_t F, int32_t n);
int32_t dab_estimate_max_n(void);

/*
 * dab_estimate_alpha_beta_noalloc - dab_estimate_alpha_beta for callers that cannot allocate
 * device memory or bring a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The per-row hand-over flags live in a device array that is part of the
 * library (dab_estimate_noalloc_max_filters() bytes, held by every GPU the library runs on until
 * the process ends), so the call takes no workspace and makes no allocating call (its address is
 * looked up once per device, by dab_init or by the first call).  Same kernels, same outputs, bit
 * for bit, as dab_estimate_alpha_beta with a workspace.
 *
 *   arguments as for dab_estimate_alpha_beta, without ws / ws_bytes
 * Errors: as dab_estimate_alpha_beta; F above dab_estimate_noalloc_max_filters()
 * -> DAB_ERR_UNSUPPORTED.  All calls on one GPU share the one array (every flag a call reads it
 * has written itself, so nothing needs clearing between calls): two such calls whose work may
 * overlap on the same GPU (different streams) race; calls on one stream are safe.
 */
int dab_estimate_alpha_beta_noalloc(const float* W, int32_t F, int32_t n,
                                    float* alpha, float* beta, int32_t* K,
                                    float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* stream);
int32_t dab_estimate_noalloc_max_filters(void);

/*
 * dab_estimate_alpha_beta_bounded - the same estimate with the split kept near the previous
 * iteration's.  Section 5 remarks that on natural images the algorithm needs K restricted to
 * change by slight amounts only and gives no rule; here the partition may move by at most
 * max_change elements: with i_prev the previous size of the lower group (K_prev if the alpha group
 * was the lower one, n - K_prev otherwise, pulled into 1 .. n-1), the best split is searched over
 * max(1, i_prev - max_change) .. min(n-1, i_prev + max_change) only.  Ties, labelling and outputs
 * are as above; max_change >= n gives dab_estimate_alpha_beta's result, max_change = 0 keeps the
 * previous partition sizes and refreshes alpha, beta and the descriptor for the new weights.
 *
 *   K_prev              [F] int32, alpha_is_upper_prev [F] uint8: the previous call's outputs; they
 *                       may be the very buffers passed as K and alpha_is_upper
 * Errors as above; max_change < 0 -> DAB_ERR_SHAPE.
 */
int dab_estimate_alpha_beta_bounded(const float* W, int32_t F, int32_t n, const int32_t* K_prev,
                                    const uint8_t* alpha_is_upper_prev, int32_t max_change, float* alpha,
                                    float* beta, int32_t* K, float* thr_val, int32_t* thr_idx,
                                    uint8_t* alpha_is_upper, void* ws, size_t ws_bytes, void* stream);

/*
 * dab_estimate_sign_split - the baseline the paper compares with, in the estimator's output form.
 * Section 4.1 notes that XNOR-Net / binary-weight networks are the special case that ignores the
 * weight distribution: e = [w >= 0], alpha = mean |w| over the filter, beta = -alpha.  The outputs
 * can be passed to dab_pack_weights and to the layer calls unchanged, which gives the comparison
 * axis of the paper's tables on the same kernels.
 *
 *   W, alpha, beta, thr_val, thr_idx, alpha_is_upper   as for dab_estimate_alpha_beta
 *   K              [F] int32 out: number of non-negative weights, 0 <= K <= n
 * The lower group is the negative weights: thr_val is the largest negative weight and thr_idx the
 * last index holding it (thr_val = -inf and thr_idx = 0 for a filter without negative weights);
 * alpha_is_upper is 1.  n >= 1; any row length is supported.
 */
int dab_estimate_sign_split(const float* W, int32_t F, int32_t n,
                            float* alpha, float* beta, int32_t* K,
                            float* thr_val, int32_t* thr_idx, uint8_t* alpha_is_upper, void* stream);

/*
 * dab_pack_weights - the mask e of Corollary 1 as bits, plus per-tap counts.
 * e[f,i] = 1 iff weight i of filter f belongs to the alpha group, decided from
 * the split descriptor of dab_estimate_alpha_beta (so the mask is defined by
 * stable rank, not by the sign of the kept values).
 *
 *   W          [F][C][kh][kw] fp32 (kh = kw = 1, C = n for a fully-connected layer)
 *   thr_val, thr_idx, alpha_is_upper   [F], as returned by the estimator
 *   E_packed   uint32 [kh*kw*Cw][Fp] out, every word written (layout above)
 *   ecnt       uint32 [F][kh*kw] out
 * Kernels of up to 384 taps (kh*kw; more -> DAB_ERR_UNSUPPORTED).
 */
int dab_pack_weights(const float* W, int32_t F, int32_t C, int32_t kh, int32_t kw,
                     const float* thr_val, const int32_t* thr_idx, const uint8_t* alpha_is_upper,
                     uint32_t* E_packed, uint32_t* ecnt, void* stream);

/*
 * dab_binarize_weights_multi - the whole weight side of several layers in a few launches (one per
 * class of row length present: up to 2304 weights, up to 4608, up to 9216, longer; plus one behind them
 * for the rows handed to the sort):
 * for every job, dab_estimate_alpha_beta (or, with K_prev, dab_estimate_alpha_beta_bounded) of its
 * filters followed by dab_pack_weights of the resulting masks.  Section 4.3.1 handles all filters of
 * a layer together; filters of different layers are just as independent, so they share the
 * launches (a workgroup looks up its job), and a filter's mask (Corollary 1) is packed by the
 * workgroup that has just found its split, while the row is still in cache.  Results are, bit
 * for bit, those of the separate calls, with one exception: for a row in which several splits have
 * scores that are equal to the last bit or differ only by the rounding of the float64 sums (a
 * constant row is the extreme case), the two may return different ones of those splits, because
 * their sort kernels cut such a row into different per-thread pieces.
 *
 *   jobs      host array of n_jobs descriptors (read during the call only); every pointer inside is a
 *             device pointer with the meaning it has in dab_estimate_alpha_beta / dab_pack_weights.
 *             E_packed and ecnt may both be NULL (estimation only); K_prev and alpha_is_upper_prev
 *             may both be NULL (unrestricted search), else max_change >= 0 bounds the split's move.
 *   ws        scratch of dab_binarize_weights_multi_workspace_bytes(jobs, n_jobs) bytes, 8-byte aligned
 *             (one flag per filter of the jobs whose unfinished rows go to the sort kernel; 0 for a
 *             few layers with rows of at most 4608 weights, which are finished in their own launch)
 * Errors: per job as in the separate calls (rows above dab_estimate_max_n(), more than 128 taps with
 * packing -> DAB_ERR_UNSUPPORTED: such a layer takes the separate calls); more than 16 jobs -> DAB_ERR_UNSUPPORTED; ws missing or too
 * small -> DAB_ERR_WORKSPACE; ws not 8-byte aligned -> DAB_ERR_ALIGN.
 */
typedef struct dab_weight_job {
    const float* W;                       /* [F][C][kh][kw] fp32 */
    int32_t F, C, kh, kw;
    float* alpha; float* beta; int32_t* K; float* thr_val; int32_t* thr_idx; uint8_t* alpha_is_upper;   /* [F] out */
    uint32_t* E_packed; uint32_t* ecnt;   /* out, or both NULL */
    const int32_t* K_prev; const uint8_t* alpha_is_upper_prev; int32_t max_change;   /* previous split, or both NULL */
} dab_weight_job;
size_t dab_binarize_weights_multi_workspace_bytes(const dab_weight_job* jobs /* host */, int32_t n_jobs);
int dab_binarize_weights_multi(const dab_weight_job* jobs /* host */, int32_t n_jobs, void* ws, size_t ws_bytes, void* stream);

/*
 * dab_pack_activations - sign binarization of a layer input (Section 4: inputs
 * are +1 / -1) into bits along the channel dimension: bit = [x >= tau_c],
 * tau = 0 when tau is NULL (sign(0) = +1).
 *
 *   X          fp32, NHWC [B][H][W][C] or NCHW [B][C][H][W] according to layout
 *   tau        [C] fp32 per-channel thresholds, or NULL
 *   A_packed   uint32 [B][H][W][Cw] out, every word written
 */
int dab_pack_activations(const float* X, int32_t layout, int32_t B, int32_t C, int32_t H, int32_t W,
                         const float* tau, uint32_t* A_packed, void* stream);

/*
 * dab_pack_activations_multi - dab_pack_activations for several tensors in one launch: the inputs
 * of all binarized layers of a network that are resident together (Section 4: every binarized
 * layer's input is +1 / -1).  Each job is one NHWC tensor with its own thresholds and output; the
 * results are those of n_jobs separate calls.
 *
 *   jobs      host array of n_jobs descriptors (read during the call only); pointers inside are device pointers
 * Errors: as dab_pack_activations per job; more than 16 jobs -> DAB_ERR_UNSUPPORTED.
 */
typedef struct dab_pack_job {
    const float* X;              /* fp32 NHWC [B][H][W][C] */
    const float* tau;            /* [C] or NULL */
    uint32_t* A_packed;          /* uint32 [B][H][W][ceil(C/32)] out */
    int32_t B, C, H, W;
} dab_pack_job;
int dab_pack_activations_multi(const dab_pack_job* jobs /* host */, int32_t n_jobs, void* stream);

/*
 * dab_prepare_layers - everything that precedes the binary products of a set of resident layers:
 * dab_binarize_weights_multi(wjobs) and dab_pack_activations_multi(pjobs) in the launches of the
 * former.  The weight side (Section 4.3.1, Corollary 1) and the binarization of the inputs (Section 4)
 * do not depend on each other and load different parts of the chip (vector instructions and LDS
 * against memory), so every workgroup of the weight-side launches also packs a share of the
 * activations, and the two overlap inside one launch.  Results are, bit for bit, those of the two
 * separate calls; arguments, workspace and errors are theirs.  In addition: fewer filters in all
 * wjobs together than tensors in pjobs -> DAB_ERR_UNSUPPORTED (call the two separately).
 */
int dab_prepare_layers(const dab_weight_job* wjobs /* host */, int32_t n_wjobs, const dab_pack_job* pjobs /* host */,
                       int32_t n_pjobs, void* ws, size_t ws_bytes, void* stream);

/*
 * dab_binconv2d - binarized convolution, Section 4.3.2's I (*) W~ on packed
 * operands: cross-correlation, zero padding (a padded tap contributes 0),
 * no bias.  For every output pixel p and filter f, over the taps inside the image,
 *     s1 = sum a_i e_i   (exact integer; a = +1/-1 from the activation bits, e from the weight bits),
 *     sA = sum a_i = 2*popc(A) - C * (number of those taps),
 *     Y[p][f] = alpha_f*s1 + beta_f*(sA - s1), evaluated in fp32 as
 *               (alpha_f - beta_f)*s1 + beta_f*sA  (|beta| <= |alpha|, so the rounding
 *               error stays within a few ulp of |alpha||s1| + |beta||s2|).
 *
 *   A_packed   uint32 [B][H][W][Cw]
 *   E_packed   uint32 [kh*kw*Cw][Fp]
 *   alpha,beta [F] fp32
 *   Y          fp32 NHWC [B][Ho][Wo][F] out
 *   dbg_s1     optional int32 [B][Ho][Wo][F] out: the integer s1 of every output
 *              (NULL to skip); this is what bit-exact tests compare
 *   ws         scratch of at least dab_binconv2d_workspace_bytes(d) bytes, 256-byte
 *              aligned (0 bytes for most layers: the kernels then read the packed bits
 *              directly; long reductions over many rows expand their operands into it);
 *              dead when the call's work has completed (DAB_ERR_WORKSPACE if NULL,
 *              too small or misaligned)
 * Padding may reach or exceed the kernel extent (windows entirely in the border give 0).
 * Errors: |s1| can reach C*kh*kw, which must stay below 2^24 -> DAB_ERR_UNSUPPORTED
 * beyond (also for tensors past 2^31 bytes expanded).
 */
int dab_binconv2d(const dab_conv_desc* d /* host */, const uint32_t* A_packed, const uint32_t* E_packed,
                  const float* alpha, const float* beta,
                  float* Y, int32_t* dbg_s1, void* ws, size_t ws_bytes, void* stream);
size_t dab_binconv2d_workspace_bytes(const dab_conv_desc* d /* host */);

/*
 * dab_binfc - binarized fully-connected layer: the same product with a 1x1
 * spatial extent.  Y[b][f] = alpha_f*s1 + beta_f*s2 over the Kin inputs.
 *
 *   A_packed   uint32 [B][ceil(Kin/32)],  E_packed uint32 [ceil(Kin/32)][Fp]
 *   Y          fp32 [B][F] out;  dbg_s1 optional int32 [B][F]
 *   ws         as for dab_binconv2d, sized by dab_binfc_workspace_bytes
 */
int dab_binfc(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
              const float* alpha, const float* beta,
              float* Y, int32_t* dbg_s1, void* ws, size_t ws_bytes, void* stream);
size_t dab_binfc_workspace_bytes(int32_t B, int32_t Kin, int32_t F);

/*
 * dab_binconv2d_bits / dab_binfc_bits - the same products with a re-binarizing epilogue: when
 * the next layer is binarized as well (Section 4: its inputs are +1 / -1; the appendix's block
 * puts the sign right after the previous binarized layer), the fp32 output is never needed, only
 *     A_next bit f of pixel p = [ Y[p][f] >= tau_out[f] ],
 * with Y[p][f] evaluated in fp32 exactly as dab_binconv2d evaluates it, so the result is identical,
 * bit for bit, to dab_pack_activations applied to dab_binconv2d's output.  1/32 of the output
 * bytes are written.
 *
 *   tau_out    [F] fp32 thresholds of the next layer's sign, or NULL for 0
 *   A_next     uint32 [B][Ho][Wo][ceil(F/32)] out (dab_binfc_bits: [B][ceil(F/32)]), every word
 *              written, bits past F are 0; this is the packed activation layout above with C = F
 *   other arguments, workspace and errors as for dab_binconv2d / dab_binfc
 */
int dab_binconv2d_bits(const dab_conv_desc* d /* host */, const uint32_t* A_packed, const uint32_t* E_packed,
                       const float* alpha, const float* beta, const float* tau_out, uint32_t* A_next,
                       void* ws, size_t ws_bytes, void* stream);
int dab_binfc_bits(int32_t B, int32_t Kin, int32_t F, const uint32_t* A_packed, const uint32_t* E_packed,
                   const float* alpha, const float* beta, const float* tau_out, uint32_t* A_next,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * dab_pool_bits - max-pooling between two binarized layers, on the packed signs.  The sign of a
 * window's maximum is +1 iff any element's sign is +1 (one threshold per channel), so
 * sign(maxpool(y) - tau) is the bitwise OR of the window's packed words.  Windows lie inside the
 * image (no padding): Ho = (H - kh)/stride_h + 1, Wo likewise.  The Sketch-A-Net architecture that
 * Section 5.1 trains (the network of the work it cites) pools 3x3 with stride 2 between binarized
 * layers.
 *
 *   A_packed   uint32 [B][H][W][ceil(C/32)];  A_pooled uint32 [B][Ho][Wo][ceil(C/32)] out
 * Errors: a window larger than the image -> DAB_ERR_SHAPE.
 */
int dab_pool_bits(const uint32_t* A_packed, int32_t B, int32_t C, int32_t H, int32_t W, int32_t kh, int32_t kw,
                  int32_t stride_h, int32_t stride_w, uint32_t* A_pooled, void* stream);

/*
 * dab_wbin_conv2d / dab_wbin_fc - the weights-only binarized layer (Section 5.1's WBin: the
 * convolutional weights binarized, the inputs left real): y = x (*) W~ with
 * W~ = alpha e + beta (1 - e) (Sections 4.1, 4.3.2), evaluated as
 *     y[p][f] = beta[f] * sum_i x_i + (alpha[f] - beta[f]) * sum_i x_i e_i
 * over the taps inside the image (zero padding, cross-correlation, no bias).  The second sum is a
 * dense contraction and runs on the matrix cores: each fp32 input is split exactly into three bf16
 * pieces, the mask is bf16 0 / 1, so every product is exact and only the fp32 accumulation rounds.
 *
 *   X          fp32 NHWC [B][H][W][C] (dab_wbin_fc: [B][Kin]), finite, 16-byte aligned
 *   E_packed, alpha, beta   as for dab_binconv2d (the outputs of dab_pack_weights / the estimator)
 *   Y          fp32 NHWC [B][Ho][Wo][F] out (dab_wbin_fc: [B][F])
 *   ws         workspace of dab_wbin_conv2d_workspace_bytes(d) bytes (dab_wbin_fc_workspace_bytes),
 *              256-byte aligned: the bf16 pieces (6 bytes per input element, with the padding
 *              halo), the expanded masks, per-pixel input sums
 * Accuracy: fp32 accumulation of exact terms; the error is bounded by about (3*n/16 + T) * 2^-24
 * times sum_i |x_i| |w~_i| (n = C*kh*kw, T = kh*kw) and is typically a few 1e-7 of that scale.
 * Errors as for dab_binconv2d.
 */
size_t dab_wbin_conv2d_workspace_bytes(const dab_conv_desc* d /* host */);
size_t dab_wbin_fc_workspace_bytes(int32_t B, int32_t Kin, int32_t F);
int dab_wbin_conv2d(const dab_conv_desc* d /* host */, const float* X, const uint32_t* E_packed, const float* alpha,
                    const float* beta, float* Y, void* ws, size_t ws_bytes, void* stream);
int dab_wbin_fc(int32_t B, int32_t Kin, int32_t F, const float* X, const uint32_t* E_packed, const float* alpha,
                const float* beta, float* Y, void* ws, size_t ws_bytes, void* stream);

/*
 * Weight-side steps of one training iteration (Algorithm 2).  The real weights are mean-centred
 * and clamped, every filter is binarized (dab_estimate_alpha_beta on the result), W~ is formed for
 * the forward and backward pass, and the gradient with respect to W~ is turned into the gradient
 * applied to the real weights (Theorem 4).  All buffers are device memory; W is [F][C][kh][kw]
 * fp32, seen as F rows of n = C*kh*kw.
 */
typedef enum {
    DAB_CENTER_FILTER = 0,   /* subtract the mean of the filter's n weights                    */
    DAB_CENTER_CHANNEL = 1   /* subtract, per filter and tap, the mean over the C channels     */
} dab_center_axis;

/*
 * dab_mean_center_clamp - MeanCenter, then Clamp(lo, hi) (Algorithm 2 lists them in this order
 * and does not name the axis of the mean; both conventions above are provided).  The mean is
 * accumulated in double, the centred value is rounded once to fp32.
 *
 *   W      [F][C][T] fp32 in (T = kh*kw);  W_out the same shape, may be W itself (in place)
 * Errors: lo > hi or a non-positive size -> DAB_ERR_SHAPE; another axis -> DAB_ERR_UNSUPPORTED.
 */
int dab_mean_center_clamp(const float* W, int32_t F, int32_t C, int32_t T, int32_t axis, float lo, float hi,
                          float* W_out, void* stream);

/*
 * dab_binarized_weights - W~ = alpha e + beta (1 - e) as fp32 (the last line of Algorithm 2's
 * binarization loop), with e taken from the split descriptor exactly as dab_pack_weights takes it.
 *
 *   W, alpha, beta, thr_val, thr_idx, alpha_is_upper   as for dab_estimate_alpha_beta
 *   W_tilde  [F][n] fp32 out, every element alpha[f] or beta[f]; must not overlap W
 */
int dab_binarized_weights(const float* W, int32_t F, int32_t n, const float* alpha, const float* beta,
                          const float* thr_val, const int32_t* thr_idx, const uint8_t* alpha_is_upper,
                          float* W_tilde, void* stream);

/*
 * dab_weight_gradient - Theorem 4 (derived in the appendix): G~ = G~1 + G~2, element-wise.  With e
 * the mask of the split descriptor, K its number of ones, T_k = W o e and R = W - T_k,
 *     G~_i = e_i/K + (||T_k||_1 / K) T_k^i [|W_i| <= 1] + (1-e_i)/(n-K) + (||R||_1 / (n-K)) R^i [|W_i| <= 1]
 * (the theorem's sgn(T_k) and sgn(W - T_k) are the masks e and 1 - e, as its derivation
 * substitutes them; STE passes the value where |W_i| <= 1).  With an upstream gradient dC/dW~ the
 * output is its element-wise product with G~, the gradient applied to the real weights.
 *
 *   W         [F][n] fp32, the mean-centred, clamped weights that were binarized (n >= 2)
 *   upstream  [F][n] fp32 or NULL
 *   G_out     [F][n] fp32 out; must not overlap W
 * K and the two l1 norms are recomputed from W and the descriptor (double accumulation).  A
 * descriptor whose mask is empty or full is outside the theorem; that group's terms are 0.
 */
int dab_weight_gradient(const float* W, int32_t F, int32_t n, const float* thr_val, const int32_t* thr_idx,
                        const uint8_t* alpha_is_upper, const float* upstream, float* G_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DAB_H */
