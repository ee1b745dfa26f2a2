/*
 * pex.h -- C ABI of libpex: per-example gradient statistics of a dense layer in a
 * sequence model, and the optimizer updates that consume them, for AMD MI355X (gfx950).
 *
 * Problem (Sec. 2.3, "Dense layers in sequence-level architectures"; paper -> here:
 * H -> X, Lambda -> G, L -> T, D -> din, F -> dout):
 *     X[B,T,din]  activations entering the layer,
 *     G[B,T,dout] cotangents (d loss / d layer output),
 *     M_b = X_b^T G_b   the per-example weight gradient (din x dout), never stored,
 *     S   = sum_b phi(M_b),  phi in {identity, elementwise square, sign}.
 *
 * Conventions common to every entry point
 *   - Every pointer is DEVICE memory owned by the caller, dense, row-major, last
 *     dimension contiguous, no strides.  The library never allocates, frees or
 *     keeps a pointer.  X and G must be 16-byte aligned, fp32 buffers 16-byte aligned.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  No entry point synchronises the device or reads results back.
 *   - Arguments are validated on the host first; a call that returns anything but
 *     PEX_OK has launched nothing.
 *   - Outputs are overwritten, not accumulated into.  Inputs are read-only.
 *   - No exceptions cross this boundary; errors are return codes only.
 *   - Results are run-to-run deterministic (no floating-point atomics).
 */
#ifndef PEX_H
#define PEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PEX_OK = 0,
    PEX_ERR_NULL = 1,       /* a required pointer is NULL */
    PEX_ERR_SHAPE = 2,      /* a dimension is < 1, too large for the kernels' 32-bit row indexing, or B < 2 where B >= 2 is needed */
    PEX_ERR_DTYPE = 3,      /* unknown pex_dtype */
    PEX_ERR_PHI = 4,        /* unknown pex_phi / pex_adam_variant */
    PEX_ERR_ALIGN = 5,      /* a pointer is not 16-byte aligned */
    PEX_ERR_WORKSPACE = 6,  /* workspace is NULL or smaller than the matching *_workspace_bytes() */
    PEX_ERR_HIP = 7,        /* the HIP runtime reported an error at launch */
    PEX_ERR_TOO_LARGE = 8   /* pex_stat_noalloc: the call needs more than PEX_NOALLOC_SCRATCH_BYTES of scratch */
} pex_status;

typedef enum { PEX_F32 = 0, PEX_BF16 = 1 } pex_dtype;                          /* storage type of X and of G (same for both) */
typedef enum { PEX_PHI_IDENTITY = 0, PEX_PHI_SQUARE = 1, PEX_PHI_SIGN = 2 } pex_phi;
typedef enum { PEX_ADAM = 0, PEX_MICROADAM = 1, PEX_MICROADAM_VAR = 2, PEX_MICROADAM_MSQ = 3 } pex_adam_variant;

typedef void *pex_stream_t; /* a hipStream_t */

/* Human-readable name of a status code (static storage, never NULL). */
const char *pex_status_string(pex_status s);

/* Library version, major*10000 + minor*100 + patch. */
int pex_version(void);

/*
 * Planner options.  Each starts from an environment variable that is read once per process (on the first call that
 * plans anything) and is changed afterwards only by pex_set_option; both calls are safe from any host thread.
 *   PEX_OPT_MAX_SPLIT        1 .. 32 (default 32; environment PEX_MAX_SPLIT, clamped to that range): the largest
 *                            number of groups the batch is split into when a layer has too few tiles to fill the
 *                            chip; it bounds the workspace at max_split * din*dout*4 bytes.
 *   PEX_OPT_TOKEN_PRESQUARE  0 = pex_token_sq always squares inside the contraction, 1 = chosen by a cost model
 *                            (default), 2 = always through bf16 copies of the squares (environment
 *                            PEX_TOKEN_PRESQUARE).  Both routes round alike and give the same bits.
 *   PEX_OPT_WIDE_BLOCKS      pex_stat(square), pex_weighted_sum and pex_stat_power on bf16 layers keep two fp32
 *                            register tiles and have two block shapes, 256 x 128 and 256 x 192.  0 = the narrow one
 *                            only, 1 = the first columns of S on the wide shape where a cost model says so
 *                            (default: layers whose wide blocks fill whole rounds of the 256 compute units),
 *                            2 = as many columns as fit on the wide shape, always (environment PEX_WIDE_BLOCKS).
 *                            The result is the same bits under every value.
 *   PEX_OPT_GRAM_NORMS       pex_example_norms on bf16 layers has two routes: the per-example contraction, and the T x T
 *                            Gram matrices of the "ghost" norm (Sec. 2.3), N_b = <X_b X_b^T, G_b G_b^T>, on blocks of
 *                            128 x 128 or, with 256 KiB of workspace per block and example, of 256 x 256.  0 = the
 *                            contraction only, 1 = chosen by a cost model (default: a Gram route for sequences that
 *                            are short for the layer), 2 = the Gram route on 128 x 128 blocks wherever it applies (rows
 *                            that are multiples of 16 bytes, B <= 65535), 3 = on 256 x 256 blocks wherever that applies
 *                            (its workspace at most 256 MiB), else as 2 (environment PEX_GRAM_NORMS).  The routes agree
 *                            to fp32 rounding, not bit for bit.
 *   PEX_OPT_MEMORY_FOLD      the same three calls have a third route on bf16 layers: the 256 x 256 block with one register
 *                            tile, phi(M_b) being added to S in memory at the end of every example (by the one lane
 *                            that owns the entry, examples in ascending order: as reproducible as a register).  Each
 *                            such fold moves the whole of S once, so it pays for few, long examples only.  0 = never,
 *                            1 = chosen by a cost model (default), 2 = wherever it applies (dout < 2^20) (environment
 *                            PEX_MEMORY_FOLD).  It rounds the square before adding it where the register tiles use a
 *                            fused multiply-add: the routes agree to fp32 rounding, not bit for bit.
 * An option changes the plan and with it the *_workspace_bytes of later calls: query again after setting one.  A
 * call whose workspace was sized under another value returns PEX_ERR_WORKSPACE if it is too small.
 * pex_set_option: PEX_ERR_PHI for an unknown option, PEX_ERR_SHAPE for a value out of range.  pex_get_option: the
 * current value, -1 for an unknown option.
 */
typedef enum { PEX_OPT_MAX_SPLIT = 0, PEX_OPT_TOKEN_PRESQUARE = 1, PEX_OPT_WIDE_BLOCKS = 2, PEX_OPT_GRAM_NORMS = 3,
               PEX_OPT_MEMORY_FOLD = 4 } pex_option;
pex_status pex_set_option(pex_option opt, int32_t value);
int32_t pex_get_option(pex_option opt);

/*
 * pex_stat -- S = sum_b phi(X_b^T G_b)  (Sec. 2.3: M = einsum(BLD,BLF->BDF), phi, reduce over B;
 * phi = identity is the ordinary batch weight gradient, phi = square is B * nu_micro of Eq. (nu_defs),
 * phi = sign is B * (avg o sign) of Sec. 3.1).
 *
 *   X  [B,T,din], G [B,T,dout]  device, dtype `dt` (bf16 payloads are multiplied exactly and summed in
 *                               fp32; fp32 payloads use true fp32 products), read-only.
 *   S  [din,dout] fp32 device, overwritten.  For phi = sign the entries are integers in [-B, B]
 *                               (sgn(0) = 0) stored as fp32, exact for B < 2^24.
 *   workspace / workspace_bytes device scratch of at least pex_stat_workspace_bytes(...) bytes with the
 *                               same (B,T,din,dout,dt,phi); may be NULL when that query returns 0.  It
 *                               holds partial sums over groups of examples when the batch is split over
 *                               workgroups; it never holds a per-example gradient, and its size is at most
 *                               32 * din*dout*4 bytes, whatever B (reached by small layers only, where
 *                               many groups are needed to occupy the chip; at the 1B-scale shapes identity
 *                               and sign need none, and square splits only the columns its wider block
 *                               shape leaves over, in two groups: half the size of S).  Partial sign counts
 *                               of bf16 layers are held as bytes while a group has at most 127 examples.
 *   The contraction over T of one example is never split across workgroups (phi is applied to the complete
 *   sum over the sequence), the sum over b is taken in a fixed order.
 *   Any B,T,din,dout >= 1 is accepted with B*T, din, dout each < 2^31; fp32 inputs and bf16 layers whose rows are
 *   not multiples of 16 bytes additionally need din <= 65535*128 resp. 65535*64 (PEX_ERR_SHAPE beyond).
 */
size_t pex_stat_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, pex_phi phi);
pex_status pex_stat(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                    pex_dtype dt, pex_phi phi, float *S, void *workspace, size_t workspace_bytes,
                    pex_stream_t stream);

/*
 * pex_stat_noalloc -- pex_stat for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels, results (bit
 * for bit) and error codes as pex_stat, but the partial sums over groups of examples go to a buffer of
 * PEX_NOALLOC_SCRATCH_BYTES that is part of the library's device image (one copy per GPU, held until the process
 * ends) instead of a caller's workspace.  The call allocates and frees nothing.
 *   - A call whose pex_stat_workspace_bytes(...) exceeds PEX_NOALLOC_SCRATCH_BYTES returns PEX_ERR_TOO_LARGE and
 *     launches nothing (small layers with many groups: e.g. 768 x 768 in 28 groups needs 63 MiB).
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different streams,
 *     different host threads) race on it; calls on one stream, or otherwise ordered, are safe.  Nothing in the
 *     buffer needs to start at zero and nothing is kept in it between calls.
 *   - The buffer's address is looked up on the first call on each device (no allocation, but make that first
 *     call outside graph capture).
 */
#define PEX_NOALLOC_SCRATCH_BYTES (32u << 20)
pex_status pex_stat_noalloc(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                            pex_dtype dt, pex_phi phi, float *S, pex_stream_t stream);

/*
 * pex_stat_multi -- several of the statistics of pex_stat from one pass over X and G.  MicroAdam needs the mean
 * gradient and the mean square of the same step (Algorithm 1, App. E; nu_micro and nu_adam of Eq. (nu_defs));
 * the per-example gradient tile M_b is the same for every phi, so one contraction can feed them all.
 *   want     bit set of PEX_WANT_IDENTITY, PEX_WANT_SQUARE, PEX_WANT_SIGN (at least one).
 *   S_id, S_sq, S_sign  [din,dout] fp32 device outputs, each required iff its bit is set (ignored otherwise);
 *                       same definitions, layout and error bounds as pex_stat with the matching phi.
 *   On bf16 layers the MFMA kernel produces all wanted statistics from one contraction (for all three this needs
 *   at most 127 examples per group of the batch; beyond that identity and square share one and sign runs alone);
 *   other inputs are served one statistic at a time.  Workspace as for pex_stat, sized by the query below.
 */
#define PEX_WANT_IDENTITY 1u
#define PEX_WANT_SQUARE 2u
#define PEX_WANT_SIGN 4u
size_t pex_stat_multi_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, uint32_t want);
pex_status pex_stat_multi(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                          pex_dtype dt, uint32_t want, float *S_id, float *S_sq, float *S_sign, void *workspace,
                          size_t workspace_bytes, pex_stream_t stream);

/*
 * pex_vec_stat -- the same statistics for a vector parameter (App. B, "Affine operations": an offset is a
 * contraction of the cotangents with a vector of ones, so its per-example gradient is the reduction over the
 * length axis).
 *   v_b[j] = sum_t A[b,t,j] * C[b,t,j]      (C == NULL: an offset, v_b[j] = sum_t A[b,t,j];
 *                                            C given: an elementwise scale applied to the activation C)
 *   s      = sum_b phi(v_b)                 for every phi in `want` (bits as for pex_stat_multi)
 *   A, C   [B,T,d] device, dtype `dt`, read-only; products are exact for bf16 and summed in fp32.
 *   s_id, s_sq, s_sign  [d] fp32 device outputs, each required iff its bit is set.
 *   workspace  at least pex_vec_stat_workspace_bytes(...) bytes (never 0): fp32 partial sums over ranges of the
 *              length axis, B * ranges * d floats, summed in a fixed order.  These partial sums are the per-example
 *              gradients of the vector themselves (B*d floats per range): for a vector, unlike for a weight
 *              matrix, staging them is cheap (B*d against B*T*d input values).
 *   Bound by HBM bandwidth: every input byte is read once.  B,T,d >= 1 with B*T, d < 2^31 and B * ranges < 65536
 *   (there are at most max(1, 2048/B) ranges, so this is B < 65536); PEX_ERR_SHAPE beyond.
 */
size_t pex_vec_stat_workspace_bytes(int64_t B, int64_t T, int64_t d, pex_dtype dt);
pex_status pex_vec_stat(const void *A, const void *C, int64_t B, int64_t T, int64_t d, pex_dtype dt, uint32_t want,
                        float *s_id, float *s_sq, float *s_sign, void *workspace, size_t workspace_bytes,
                        pex_stream_t stream);

/*
 * pex_stat_power -- S = sum_b |X_b^T G_b|^alpha elementwise, 0 < alpha <= 64 (PEX_ERR_PHI otherwise): the power
 * nonlinearities phi(s) = s^alpha that Sec. 2.3 names beside square and sign (alpha = 2 is phi = square, alpha = 1
 * the mean absolute gradient).  Each term is 2^(alpha * log2 |m|) through the hardware log2 / exp2 instructions:
 * relative error of a term about 1e-6 * alpha * |log2 m|; all terms are >= 0.  Buffers as for pex_stat.
 */
size_t pex_stat_power_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt);
pex_status pex_stat_power(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                          pex_dtype dt, float alpha, float *S, void *workspace, size_t workspace_bytes,
                          pex_stream_t stream);

/*
 * Norms and clipping (Sec. 2.1 names clipping among the statistics of interest; Sec. 2.3 the squared norms).
 *
 * pex_example_norms -- N[b] = || X_b^T G_b ||_F^2, the squared norm of every per-example gradient of the layer.
 *   N [B] fp32 device, overwritten.  One per-example contraction; M_b stays in registers, each workgroup adds its
 *   tile's share of the norm to a small partial-sum buffer in the workspace ([tiles * 8][B] floats), a second kernel
 *   sums the shares in a fixed order.
 * pex_weighted_sum -- S = sum_b w[b] * X_b^T G_b with one weight per example (w [B] fp32 device, read-only).  With
 *   w[b] = min(1, c / ||g_b||), ||g_b||^2 the sum of N[b] over the layers of the model, this is the clipped gradient
 *   sum; with w = 1 it is pex_stat(identity).  Workspace as for pex_stat.
 * pex_token_norms -- N_tok[b*T + t] = || x_bt ||^2 * || g_bt ||^2, the per-sample per-token norms of Sec. 2.3 (the
 *   squared norm of the rank-one term x_bt g_bt^T).  N_tok [B*T] fp32 device, overwritten; no workspace; bound by
 *   HBM bandwidth (X and G read once).
 * Same input conventions, limits and error codes as pex_stat.
 * pex_clip_weights -- the clip nonlinearity of Sec. 2.1, phi(g_b) = min(1, c / ||g_b||) g_b, for a model of several
 *   layers: the gradient of example b is the concatenation of its per-layer gradients, so
 *   w[b] = min(1, max_norm / sqrt(sum_l N[l*B + b])), N [nlayers][B] fp32 device holding the pex_example_norms output
 *   of every layer (let layer l write to N + l*B), summed in ascending l in fp64.  An example whose gradient is
 *   zero keeps w = 1.  w [B] fp32 device, overwritten; feed it to pex_weighted_sum of every layer for the sum of the
 *   clipped per-example gradients.  Everything stays on the device and on `stream`: no host round trip, so a clipped
 *   step can be captured as a whole.  nlayers >= 1, max_norm > 0 (PEX_ERR_SHAPE otherwise).
 */
size_t pex_example_norms_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt);
pex_status pex_example_norms(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                             pex_dtype dt, float *N, void *workspace, size_t workspace_bytes, pex_stream_t stream);
size_t pex_weighted_sum_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt);
pex_status pex_weighted_sum(const void *X, const void *G, const float *w, int64_t B, int64_t T, int64_t din,
                            int64_t dout, pex_dtype dt, float *S, void *workspace, size_t workspace_bytes,
                            pex_stream_t stream);
pex_status pex_token_norms(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                           pex_dtype dt, float *N_tok, pex_stream_t stream);
pex_status pex_clip_weights(const float *N, int64_t B, int32_t nlayers, float max_norm, float *w, pex_stream_t stream);

/*
 * pex_token_sq -- S_tok = (X o X)^T (G o G) = sum_{b,t} (x_bt o x_bt)(g_bt o g_bt)^T  (Sec. 2.3,
 * "per-token second moments").  A proxy statistic: tokens are not independent computational paths in a
 * transformer, so this is not a per-token gradient second moment.
 *   Same buffers and conventions as pex_stat.  For bf16 inputs each squared operand is formed in fp32 and
 *   rounded to bf16 (round to nearest even) before the contraction; all terms are >= 0, so every entry
 *   carries a relative error of at most about 2^-7.  fp32 inputs are squared and multiplied in fp32.
 *   Workspace: besides partial sums, for large bf16 layers (din*dout/(din+dout) beyond roughly 800) the
 *   workspace holds bf16 copies of the squared operands, 2*B*T*(din+dout) bytes: squaring once at HBM speed
 *   is cheaper there than squaring every slab inside the contraction.  The query returns the total.
 */
size_t pex_token_sq_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt);
pex_status pex_token_sq(const void *X, const void *G, int64_t B, int64_t T, int64_t din, int64_t dout,
                        pex_dtype dt, float *S_tok, void *workspace, size_t workspace_bytes,
                        pex_stream_t stream);

/*
 * pex_adam_update -- one elementwise step of Algorithm 1 (App. E) over n parameters, in place.
 *   mu_t   = grad_scale * S_id                      (mean gradient)
 *   nu_mic = sq_scale   * S_sq                      (nu_micro of Eq. (nu_defs); unused and may be NULL for PEX_ADAM)
 *   m  <- beta1*m + (1-beta1)*mu_t
 *   nu_t = mu_t^2                                   PEX_ADAM
 *        = nu_mic                                   PEX_MICROADAM
 *        = (nu_mic - mu_t^2) / (1 - 1/B)            PEX_MICROADAM_VAR   (sigma^2-hat, Eq. (musq_sigsq_est))
 *        = (mu_t^2 - nu_mic/B) / (1 - 1/B)          PEX_MICROADAM_MSQ   (mu^2-hat,    Eq. (musq_sigsq_est))
 *   v  <- beta2*v + (1-beta2)*nu_t                  (stored unclamped; may be negative for MSQ)
 *   mh = m/(1-beta1^step), vh = v/(1-beta2^step);   VAR and MSQ: vh <- max(0, vh)  (Sec. 3.2.3)
 *   theta <- theta - lr * mh/(sqrt(vh + eps_root) + eps) - weight_decay*theta
 * theta, m, v, S_id, S_sq: fp32 device arrays of n elements, 16-byte aligned.  step >= 1.
 * VAR and MSQ need B >= 2 (PEX_ERR_SHAPE otherwise).  With cotangents of the summed loss use
 * grad_scale = sq_scale = 1/B; with cotangents of the mean loss use grad_scale = 1, sq_scale = B.
 */
typedef struct {
    float lr, beta1, beta2, eps, eps_root, weight_decay, grad_scale, sq_scale;
    int64_t step;
    int32_t B;
} pex_adam_params;
pex_status pex_adam_update(float *theta, float *m, float *v, const float *S_id, const float *S_sq,
                           int64_t n, pex_adam_variant variant, const pex_adam_params *p /* host */,
                           pex_stream_t stream);

/*
 * pex_signsgd_update -- MicroSignSGD = EMA o avg o sign (Sec. 3.1), in place over n parameters:
 *   m <- beta*m + (1-beta) * S_sign/B ;  d = debias ? m/(1-beta^step) : m ;
 *   theta <- theta - lr*d - weight_decay*theta
 * theta, m, S_sign: fp32 device arrays of n elements, 16-byte aligned.  B >= 1, step >= 1.
 */
pex_status pex_signsgd_update(float *theta, float *m, const float *S_sign, int64_t n, float lr,
                              float beta, float weight_decay, int32_t B, int32_t debias, int64_t step,
                              pex_stream_t stream);

/*
 * pex_sign_update -- the three placements of sign in SignSGD with momentum that Sec. 3.1 compares, in place:
 *   PEX_MICROSIGNSGD  EMA o avg o sign : S = sum_b sgn(g_b) (pex_stat phi = sign);  m <- beta*m + (1-beta)*S/B;
 *                                        theta <- theta - lr*d - weight_decay*theta, d = debias ? m/(1-beta^step) : m
 *   PEX_SIGNSGD       EMA o sign o avg : S = sum_b g_b (phi = identity);            m <- beta*m + (1-beta)*sgn(S); same step
 *   PEX_SIGNEMA       sign o EMA o avg : S = sum_b g_b;                             m <- beta*m + (1-beta)*S/B;
 *                                        theta <- theta - lr*sgn(m) - weight_decay*theta  (debias cannot change a sign)
 * sgn(0) = 0.  theta, m, S: fp32 device arrays of n elements, 16-byte aligned.  B >= 1, step >= 1.
 * pex_signsgd_update is this call with PEX_MICROSIGNSGD.
 */
typedef enum { PEX_MICROSIGNSGD = 0, PEX_SIGNSGD = 1, PEX_SIGNEMA = 2 } pex_sign_variant;
pex_status pex_sign_update(float *theta, float *m, const float *S, int64_t n, pex_sign_variant variant, float lr,
                           float beta, float weight_decay, int32_t B, int32_t debias, int64_t step,
                           pex_stream_t stream);

/*
 * Gradient clipping by the global norm (Sec. 3.2.3 and App. C stabilise MicroAdam, MicroAdamVar and MicroAdamMSQ with
 * it; read as: every per-example gradient is multiplied by kappa = min(1, max_norm / ||mu_t||), the norm of the mean
 * gradient taken over all parameters of the model).
 * pex_sum_squares: acc[0] = (accumulate ? acc[0] : 0) + sum_i x[i]^2 in fp64, summed in a fixed order; call it on the
 *   S_id of every layer (accumulate = 0 for the first) to get ||sum_b g_b||^2.  x: fp32 device array of n elements,
 *   16-byte aligned; acc: one double in device memory; workspace: pex_sum_squares_workspace_bytes(n) bytes.
 * pex_adam_update_clipped: pex_adam_update with grad_scale multiplied by kappa and sq_scale by kappa^2, where
 *   kappa = min(1, max_norm / (|grad_scale| * sqrt(*sum_sq))) is formed on the device from the accumulated sum (no host
 *   synchronisation).  sum_sq: one double in device memory; max_norm > 0.
 */
size_t pex_sum_squares_workspace_bytes(int64_t n);
pex_status pex_sum_squares(const float *x, int64_t n, double *acc, int32_t accumulate, void *workspace,
                           size_t workspace_bytes, pex_stream_t stream);
pex_status pex_adam_update_clipped(float *theta, float *m, float *v, const float *S_id, const float *S_sq, int64_t n,
                                   pex_adam_variant variant, const pex_adam_params *p /* host */, const double *sum_sq,
                                   float max_norm, pex_stream_t stream);

/*
 * pex_moment_track -- on-line measurement of mu^2 and sigma^2 (Sec. 3.2.2, Eq. (musq_sigsq_est)), in place over n
 * parameters.  Two EMAs with the optimizer's beta2 follow nu_adam and nu_micro:
 *   mu_t = grad_scale*S_id ;  ema_adam  <- beta2*ema_adam  + (1-beta2)*mu_t^2
 *                             ema_micro <- beta2*ema_micro + (1-beta2)*sq_scale*S_sq
 *   a = ema_adam*k, q = ema_micro*k, k = debias ? 1/(1-beta2^step) : 1
 *   mu^2-hat = (a - q/B)/(1 - 1/B),  sigma^2-hat = (q - a)/(1 - 1/B)
 *   sums[0] = sum over the n parameters of mu^2-hat, sums[1] = sum of sigma^2-hat  (fp64, device memory)
 * The figures of Sec. 3.2.2 plot sums[0]/n, sums[1]/n and sums[0]/(sums[1]/B) (Adam) or sums[0]/sums[1] (MicroAdam),
 * with the sums of all layers added up by the caller.  ema_adam, ema_micro (read and written), S_id, S_sq: fp32 device
 * arrays of n elements, 16-byte aligned; sums: 2 doubles, 8-byte aligned; the workspace holds one pair of partial
 * sums per workgroup, added in a fixed order (the result does not depend on scheduling).  B >= 2, step >= 1.
 */
typedef struct {
    float beta2, grad_scale, sq_scale;
    int32_t B, debias;
    int64_t step;
} pex_moment_params;
size_t pex_moment_track_workspace_bytes(int64_t n);
pex_status pex_moment_track(float *ema_adam, float *ema_micro, const float *S_id, const float *S_sq, int64_t n,
                            const pex_moment_params *p /* host */, double *sums, void *workspace,
                            size_t workspace_bytes, pex_stream_t stream);

/*
 * pex_embed_stat -- per-example gradient statistics of an embedding table E[V, d].  A lookup is a dense layer on
 * one-hot inputs (Sec. 2.3 with X one-hot): row v of the per-example gradient M_b is the sum of G[b,t,:] over the
 * positions t of example b with ids[b,t] == v, and S = sum_b phi(M_b) with phi as in pex_stat (sgn(0) = 0).
 *   ids   [B, T] token ids, int32 (ids_bytes = 4) or int64 (ids_bytes = 8), device memory, aligned to their size;
 *         positions whose id is outside [0, V) (padding) contribute nothing
 *   G     [B, T, d] cotangents of the looked-up vectors, dt = fp32 or bf16, row-major, 16-byte aligned
 *   want  PEX_WANT_* bits; S_id, S_sq, S_sign: fp32 [V, d] each, 16-byte aligned, NULL where not wanted; every row
 *         is overwritten (rows of tokens that do not occur with zeros)
 * The workspace holds the positions sorted by token (about 20 bytes per position plus 4 per vocabulary row) and, for
 * the runs of frequent tokens, two partial rows of each statistic per 256 positions (about 0.1 * d bytes per position);
 * no per-example gradient is stored.  Results do not depend on scheduling: positions are sorted stably and
 * sums run in a fixed order.  Bound by HBM bandwidth.  B*T < 2^31, V < 2^31 - 1.
 */
size_t pex_embed_stat_workspace_bytes(int64_t B, int64_t T, int64_t V, int64_t d);
pex_status pex_embed_stat(const void *ids, int32_t ids_bytes, const void *G, int64_t B, int64_t T, int64_t V, int64_t d,
                          pex_dtype dt, uint32_t want, float *S_id, float *S_sq, float *S_sign, void *workspace,
                          size_t workspace_bytes, pex_stream_t stream);

/*
 * pex_mfma_probe -- measurement aid, not part of the method: one launch that issues nothing but bf16 MFMAs
 * (v_mfma_f32_16x16x32_bf16, fp32 accumulation) in the register shape of the 256 x 256 tile contraction kernel, on
 * `workgroups` workgroups of 8 waves (use the number of compute units).  Its rate is the ceiling the matrix pipes of
 * the chip sustain at the clock they settle at under load; the contraction kernels are reported against it beside the
 * datasheet peak.  The values of the operands set the switching activity and with it the clock, so the caller supplies
 * them (for a like-for-like figure: the same distribution as the contraction's inputs).
 *   operands  device, pex_mfma_probe_operand_bytes() bytes of bf16 values, 16-byte aligned
 *   sink      device, pex_mfma_probe_sink_floats(workgroups) floats; receives one sum per lane (keeps the work alive)
 *   returns the FLOP the launch performs in *flop (host), 2*16*16*32 per MFMA
 */
size_t pex_mfma_probe_operand_bytes(void);
size_t pex_mfma_probe_sink_floats(int32_t workgroups);
pex_status pex_mfma_probe(const void *operands, int32_t workgroups, int32_t iters, float *sink, double *flop /* host */,
                          pex_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* PEX_H */
