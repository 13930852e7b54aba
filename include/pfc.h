/*
 * pfc.h -- C ABI of libpfc.so: one Partial FC (PFC) training step on one MI355X (gfx950).
 *
 * The method is "Partial FC" (An et al., CVPR 2022, arXiv 2203.15565), Sec. 3.2: all N class
 * centers W (N x D) are kept, but in an iteration the margin-based softmax loss is evaluated
 * over a sampled set S only -- every class present in the batch plus random negatives,
 * |S| = r*N -- and only the rows of W in S are updated.
 *
 * Conventions
 *   - Every matrix is row-major; a row is one sample (features) or one class center (weight).
 *   - "dev" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library never frees or keeps a caller pointer after a call returns,
 *     and allocates device memory only inside pfc_create (scratch owned by the context).
 *   - All work is enqueued on the stream given to pfc_create; calls return without waiting
 *     for the GPU unless stated.  One context must not be used from two threads at once.
 *   - Every function returns PFC_OK (0) or a negative error code; nothing aborts or throws.
 *     On PFC_EINVAL nothing has been launched and no caller buffer has been written.
 *   - Same inputs give bit-identical outputs on every run (no floating-point atomics).
 */
#ifndef PFC_H_
#define PFC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PFC_OK       0
#define PFC_EINVAL  (-1)  /* bad argument: null pointer, size out of range, r outside (0,1], ... */
#define PFC_ELABEL  (-2)  /* a label / index on the device was out of range (seen by pfc_check) */
#define PFC_EHIP    (-3)  /* a HIP runtime call failed; pfc_last_hip_error() has the text        */
#define PFC_ENOMEM  (-4)  /* scratch allocation failed in pfc_create                              */

#define PFC_PRECISION_FP32 0  /* GEMM operands fp32 (fp32 MFMA)                                   */
#define PFC_PRECISION_BF16 1  /* GEMM operands rounded to bf16 (RNE), fp32 accumulate; W, v fp32 */

typedef struct pfc_ctx pfc_ctx;

/* Create a context holding the scratch for problems up to (N classes, D, B_max samples, ratio
 * r_max).  D must be a multiple of 64, 64 <= D <= 1024 (the GEMMs work on rows padded to the next
 * multiple of 256 inside the library: D = 256, 512, 768, 1024 waste nothing; the one-kernel form
 * of pfc_forward_backward_update exists for D = 512, other D take its two-kernel form);
 * 1 <= N < 2^31; 0 < r_max <= 1; the largest sampled set, pfc_num_sampled(N, B_max, r_max), must stay below 2^25 classes (bf16
 * operands) or 2^24 (fp32 operands): PFC_EINVAL otherwise.
 * `hip_stream` is a hipStream_t (NULL = the default stream).  Allocates device memory. */
int pfc_create(pfc_ctx** out, int64_t N, int32_t D, int32_t B_max, double r_max,
               int32_t precision, void* hip_stream);
int pfc_destroy(pfc_ctx* ctx);

/* Upper bound on |S| that needs no knowledge of the labels: max(B, ceil(r*N)), the product
 * taken in IEEE binary64.  (|S| = C*r, text after Eq. 4; Sec. 3.3: never fewer than the classes
 * present in the batch.)  Returns -1 on bad arguments. */
int64_t pfc_num_sampled(int64_t N, int32_t B, double r);

/*
 * pfc_sample -- choose the class set S of one iteration (Sec. 3.2: positive centers are picked
 * through the labels and put in the buffer first, random negatives fill the rest; Fig. 4).
 *
 *   labels            dev, int64[B], each in [0, N)
 *   r                 sampling ratio in (0, 1];  k = max(U, ceil(r*N)), U = #distinct labels
 *   seed, step        the random negatives are a pure function of (seed, step, class id):
 *                     class j scores word (j mod 4) of Philox4x32-10 with counter
 *                     (lo32(j/4), hi32(j/4), lo32(step), hi32(step)) and key (lo32(seed),
 *                     hi32(seed)); the k - U non-positive classes with the largest scores are
 *                     taken, equal scores resolved towards the smaller class id.
 *   idx_out           dev, int32[capacity >= pfc_num_sampled(N,B,r)]; receives the k chosen
 *                     class ids in ascending order (entries past k are not written)
 *   labels_local_out  dev, int32[B]; position of labels[i] inside idx_out (-1 for a bad label)
 *   k_out             host, exact k.  When ceil(r*N) >= B it is known without looking at the
 *                     labels and the call does not wait for the GPU; otherwise (the
 *                     "within-batch classes only" regime of Sec. 3.3) the call synchronises the
 *                     stream once to read U back.
 * A label outside [0, N) is skipped and recorded; pfc_check reports it as PFC_ELABEL.
 */
int pfc_sample(pfc_ctx* ctx, const int64_t* labels, int32_t B, double r,
               uint64_t seed, uint64_t step,
               int32_t* idx_out, int32_t* labels_local_out, int64_t* k_out);

/* Same as pfc_sample with every score ANDed with `score_mask` first (0xFFFFFFFF gives
 * pfc_sample).  Exists so that the tie rule can be exercised: a mask of 0 makes all scores
 * equal and the smallest class ids must win. */
int pfc_sample_masked(pfc_ctx* ctx, const int64_t* labels, int32_t B, double r,
                      uint64_t seed, uint64_t step, uint32_t score_mask,
                      int32_t* idx_out, int32_t* labels_local_out, int64_t* k_out);

/*
 * pfc_sample_noalloc -- pfc_sample for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  It needs no context: the
 * sampler's scratch (bitmap of batch classes, radix histograms, block counts; 2.2 MB) is a
 * file-scope device array of the library, one copy per GPU, held until the process ends.  The
 * call allocates nothing, frees nothing, never waits for the GPU and records no memset: it only
 * launches the kernels of pfc_sample on `hip_stream` (a hipStream_t, NULL = the default stream)
 * of the current device.  Results are those of pfc_sample, bit for bit.
 *   N                 number of classes, 1 <= N <= 16,777,216 (2^24); more is PFC_EINVAL
 *   B, r              1 <= B <= 2^20, 0 < r <= 1, and ceil(r*N) >= B so that k = ceil(r*N) is
 *                     known without reading the labels back (otherwise PFC_EINVAL: that regime
 *                     needs the synchronising pfc_sample)
 *   labels, idx_out, labels_local_out (dev), k_out (host), seed, step: as for pfc_sample
 * A label outside [0, N) is skipped and its labels_local_out entry is -1; there is no context
 * to report it through.  All calls on one GPU share that GPU's scratch array, which every call
 * leaves cleared for the next: two calls that overlap in time on one GPU (different streams or
 * threads) race and give undefined results; calls on one stream, or ordered by events, are fine.
 */
int pfc_sample_noalloc(const int64_t* labels, int32_t B, int64_t N, double r,
                       uint64_t seed, uint64_t step,
                       int32_t* idx_out, int32_t* labels_local_out, int64_t* k_out,
                       void* hip_stream);

/*
 * pfc_forward_backward -- loss and gradients of the margin-based softmax over S.
 * Eq. 1 (mean over the batch) with cosine logits, the sum running over j in S only (Eq. 4);
 * the label logit carries the additive angular margin:  z_ij = s*cos_ij for j != y_i,
 * z_iy = s*cos(theta_iy + m);  cos_ij = <x_i/|x_i|, W_j/|W_j|> clamped to [-1,1], norms bounded
 * below by 1e-12.  There is no special case for theta + m > pi.  Gradients follow Eq. 2 / Eq. 4
 * (features) and the bracket of Eq. 3 (centers), carried through scale and margin.
 *
 *   features       dev, fp32[B x D]
 *   weight         dev, fp32[N x D], read only
 *   idx            dev, int32[k], ascending class ids (as written by pfc_sample)
 *   labels_local   dev, int32[B], each in [0, k)
 *   s, m           scale (0 < s <= 65536) and margin (0 <= m < pi)
 *   loss_out       dev, fp32[1]
 *   dfeatures_out  dev, fp32[B x D]: dL/dx_i w.r.t. the RAW feature rows
 *   dweight_out    dev, fp32[k x D]: row j is dL/d wn_j, the gradient w.r.t. the L2-NORMALISED
 *                  center idx[j].  pfc_update turns it into the raw-row gradient
 *                  (g - <g,wn> wn)/|W_j| while it has W_j in registers anyway.
 * An out-of-range idx / labels_local entry is skipped and recorded (pfc_check -> PFC_ELABEL).
 * Up to s = 64 the softmax needs no running maximum (z lies in [-s, s] by construction, so exp(z)
 * and its sums are representable in fp32/bf16); above, one more pass of the logit GEMM finds each
 * sample's largest logit first and the softmax runs relative to it (about a fifth more time).
 */
int pfc_forward_backward(pfc_ctx* ctx, const float* features, const float* weight,
                         const int32_t* idx, int64_t k, const int32_t* labels_local, int32_t B,
                         float s, float m,
                         float* loss_out, float* dfeatures_out, float* dweight_out);

/*
 * pfc_forward_backward_ex -- pfc_forward_backward with the variants the paper also trains with.
 *   margin_type       PFC_MARGIN_ARCFACE: label logit s*cos(theta + m) (as pfc_forward_backward);
 *                     PFC_MARGIN_COSFACE: label logit s*(cos(theta) - m).  Sec. 4.1 uses the
 *                     hyper-parameters of both margin-based losses.
 *   filter_threshold  the PFC* variant (Sec. 3.3, Fig. 4 caption): a negative center whose clamped
 *                     cosine to sample i is greater than this value (0.4 in the paper) is left out
 *                     of sample i's softmax, in the loss and in every gradient.  The label center
 *                     is never filtered.  Any value >= 1 switches the filter off; values below -1
 *                     are rejected.
 *   stats_out         dev, fp32[2] or NULL: {APCS, AMNCS} of Sec. 3.3 -- the batch mean of the label
 *                     cosine, and the batch mean of the largest cosine between a sample and a
 *                     sampled center other than its label's (taken before filtering; needs k >= 2).
 * Everything else is as for pfc_forward_backward, which is this call with PFC_MARGIN_ARCFACE, the
 * filter off and stats_out = NULL.
 */
#define PFC_MARGIN_ARCFACE 0
#define PFC_MARGIN_COSFACE 1
int pfc_forward_backward_ex(pfc_ctx* ctx, const float* features, const float* weight,
                            const int32_t* idx, int64_t k, const int32_t* labels_local, int32_t B,
                            float s, float m, int32_t margin_type, float filter_threshold,
                            float* loss_out, float* dfeatures_out, float* dweight_out,
                            float* stats_out);

/*
 * pfc_update -- SGD with momentum on the sampled rows only (Eq. 3; text after Eq. 4: only the
 * sampled centers are updated in an iteration).  For every j < k, with W_j = weight[idx[j]]:
 *     wn = W_j/|W_j|;  g = (dweight[j] - <dweight[j], wn> wn)/|W_j|
 *     v_j <- mu*v_j + g;   W_j <- W_j - lr*v_j
 * Rows of weight and momentum that are not in idx are neither read nor written.
 *   weight, momentum  dev, fp32[N x D], updated in place
 *   idx               dev, int32[k], distinct class ids
 *   dweight           dev, fp32[k x D], as written by pfc_forward_backward
 */
int pfc_update(pfc_ctx* ctx, float* weight, float* momentum, const int32_t* idx, int64_t k,
               const float* dweight, float lr, float mu);

/*
 * pfc_forward_backward_update -- pfc_forward_backward_ex followed by pfc_update in one call
 * (Eq. 1-4 as above): loss and feature gradients come out, the sampled rows of weight and
 * momentum are updated in place, and the center gradient is consumed where it is produced
 * instead of crossing the boundary.  The results are those of the two calls in a row (the
 * feature gradient and the loss are taken before any row changes).  With D = 512 the backward
 * GEMM for the centers applies the update in its own epilogue and the k x D gradient never
 * reaches memory; otherwise it passes through a buffer of the context.
 *   weight, momentum  dev, fp32[N x D], updated in place on the rows in idx only
 *   lr, mu            learning rate and momentum of pfc_update
 *   the other arguments are those of pfc_forward_backward_ex (there is no dweight_out).
 */
int pfc_forward_backward_update(pfc_ctx* ctx, const float* features, float* weight,
                                float* momentum, const int32_t* idx, int64_t k,
                                const int32_t* labels_local, int32_t B, float s, float m,
                                int32_t margin_type, float filter_threshold, float lr, float mu,
                                float* loss_out, float* dfeatures_out, float* stats_out);

/* Wait for the stream and report: PFC_ELABEL if any kernel since the last pfc_check saw an
 * out-of-range label or index (the flag is cleared), PFC_EHIP on a HIP error, else PFC_OK. */
int pfc_check(pfc_ctx* ctx);

/* Timing hooks for benchmarks: per-kernel durations of the most recent pfc_sample /
 * pfc_forward_backward / pfc_update calls, measured with HIP events on the context's stream.
 * pfc_set_timing(ctx, 1) turns the events on (off by default; they cost a few microseconds per
 * kernel).  pfc_get_timing waits for the stream, then copies up to `cap` entries: names_out[i]
 * points to a static string, ms_out[i] is that kernel's duration in milliseconds for its last
 * launch.  Returns the number of entries, or a negative error code. */
int pfc_set_timing(pfc_ctx* ctx, int32_t enabled);
int pfc_get_timing(pfc_ctx* ctx, const char** names_out, float* ms_out, int32_t cap);

const char* pfc_strerror(int code);
const char* pfc_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PFC_H_ */
