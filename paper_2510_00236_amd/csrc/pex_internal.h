// pex_internal.h -- declarations shared by the translation units of libpex (host side only).
// Nothing here is visible through the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pex.h"

namespace pex {

// Which statistic a contraction kernel produces.  PHI_* match pex_phi; TOKEN_SQ is the per-token
// square (operands squared on the load path, one plain contraction over K = B*T).
// MODE_NORMS (per-example squared norms, no S) and MODE_WEIGHTED (sum_b w_b M_b) are per-example passes too.
// MODE_POWER is phi(m) = |m|^alpha.
enum Mode : int { MODE_IDENTITY = 0, MODE_SQUARE = 1, MODE_SIGN = 2, MODE_TOKEN_SQ = 3, MODE_NORMS = 4, MODE_WEIGHTED = 5, MODE_POWER = 6 };

// How one call is carried out.  Chosen on the host from the shape alone, so the workspace query and
// the launch always agree.
struct StatPlan {
    int kernel;        // 0 = generic SIMT kernel (odd shapes), 1 = bf16 MFMA kernel, 2 = fp32 MFMA kernel
    int nsplit;        // number of groups the batch (or, for plain contractions, B*T) is split into
    int64_t per_split; // examples (or rows of B*T) per group
    size_t presq_bytes; // per-token square through pre-squared copies of X and G: their size (256-byte multiple), else 0
    int64_t wide_cols; // bf16, one statistic on two register tiles: columns [0, wide_cols) of S run on 256 x 192 blocks as
                       // wide_nsplit groups of wide_per_split examples; nsplit / per_split then describe the remaining columns only
    int wide_nsplit;
    int64_t wide_per_split;
    size_t wide_ws_bytes; // partial sums of the wide part (first in the workspace after the squared copies), 0 if unsplit
    bool mem_fold;     // bf16, one statistic that would need two register tiles: 256 x 256 blocks, phi(M_b) added to the output
                       // in memory at the end of every example (nsplit / per_split describe the whole layer, wide_cols = 0)
    bool sign_bytes;   // MODE_SIGN on bf16 layers, split batch: the partial counts are bytes (per tile layout), not fp32
    bool gram;         // MODE_NORMS on bf16 layers: through the T x T Gram matrices instead of the contraction
    bool gram_wide;    // ... on 256 x 256 blocks whose X X^T part waits in the workspace (after the partials, 256-byte aligned)
    size_t ws_bytes;   // presq_bytes + wide_ws_bytes + (nsplit > 1 ? nsplit * din * (dout - wide_cols) * 4 : 0)
};

// allow_wide = false keeps the plan on one block shape (the launches that produce several statistics at once need it)
StatPlan plan_stat(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, Mode mode, bool allow_wide = true);

// Launchers.  `out` is S when plan.nsplit == 1, else the workspace holding [nsplit][din][dout] partials.
// MODE_WEIGHTED reads one weight per example from `weight`; MODE_NORMS writes no S but one partial of ||M_b||^2 per
// tile (generic kernel) into norm_partial[tile][B].
hipError_t launch_stat_generic(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                               pex_dtype dt, Mode mode, const StatPlan& plan, float* out, hipStream_t stream,
                               const float* weight = nullptr, float* norm_partial = nullptr, float alpha = 0.f);
// bf16 launchers take S and the partial-sum buffer both: which one a block writes depends on the plan
hipError_t launch_power_bf16(const void* X, const void* G, float alpha, int64_t B, int64_t T, int64_t din, int64_t dout,
                             const StatPlan& plan, float* S, float* partials, hipStream_t stream);
int64_t generic_norm_partials(int64_t din, int64_t dout);
int64_t bf16_norm_partials(int64_t din, int64_t dout);
hipError_t launch_norms_bf16(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, const StatPlan& plan,
                             float* norm_partial, hipStream_t stream);
hipError_t launch_weighted_bf16(const void* X, const void* G, const float* w, int64_t B, int64_t T, int64_t din, int64_t dout,
                                const StatPlan& plan, float* S, float* partials, hipStream_t stream);
// Per-example squared norms through the Gram matrices X_b X_b^T and G_b G_b^T (bf16): one partial per 128 x 128 block of
// their upper triangle and example, partial[block][B]
int64_t gram_norm_partials(int64_t T);
bool gram_supports(int64_t B, int64_t T, int64_t din, int64_t dout);
hipError_t launch_gram_norms(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, float* partial,
                             hipStream_t stream);
// The same on 256 x 256 blocks: one partial per block of the upper triangle and example, and 256 KiB of workspace per
// workgroup where the block of X_b X_b^T waits while G_b G_b^T is formed
int64_t gram_wide_partials(int64_t T);
size_t gram_wide_park_bytes(int64_t B, int64_t T);
hipError_t launch_gram_wide(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, float* partial, void* park,
                            hipStream_t stream);
// N[b] = sum_{p < nparts} partial[p][b], p ascending
hipError_t launch_reduce_norms(const float* partial, int64_t nparts, int64_t B, float* N, hipStream_t stream);
// N_tok[r] = |x_r|^2 |g_r|^2 for every row r of the flattened [B*T] axis
hipError_t launch_token_norms(const void* X, const void* G, int64_t rows, int64_t din, int64_t dout, pex_dtype dt, float* N_tok,
                              hipStream_t stream);
hipError_t launch_stat_bf16(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                            Mode mode, const StatPlan& plan, float* S, float* partials, hipStream_t stream);
// Two per-example statistics from one contraction; exactly one of the three outputs is NULL.  Uses the block
// shape of phi = square, so plan_stat(..., MODE_SQUARE) is its plan.
hipError_t launch_stat_bf16_pair(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                 const StatPlan& plan, float* out_id, float* out_sq, float* out_sg, hipStream_t stream);
// All three from one contraction, while a group of examples is small enough for byte-wide sign counters.
bool bf16_triple_supported(const StatPlan& plan);
hipError_t launch_stat_bf16_triple(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                   const StatPlan& plan, float* out_id, float* out_sq, float* out_sg, hipStream_t stream);
bool bf16_supports(int64_t B, int64_t T, int64_t din, int64_t dout);
bool f32_mfma_supports(int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode);
void f32_tile_shape(int* bm, int* bn);
hipError_t launch_stat_f32(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode,
                           const StatPlan& plan, float* out, hipStream_t stream, const float* weight, float alpha);
// out[i] = bf16(in[i]^2) (square in fp32, round to nearest even) for n bf16 values, n a multiple of 8
hipError_t launch_square_bf16(const void* in, void* out, int64_t n, hipStream_t stream);
void bf16_tile_shape(Mode mode, int64_t B, int* bm, int* bn);
void bf16_wide_tile_shape(int* bm, int* bn);
// byte-wide partial sign counts of a split batch (bf16, at most 127 examples per group): size of one group's partials,
// and their sum into S
bool sign_byte_partials_possible(int64_t B, int64_t per_split);
size_t sign_byte_partial_bytes(int64_t din, int64_t dout);
hipError_t launch_reduce_sign_bytes(const void* partial, int nsplit, int64_t din, int64_t dout, float* S, hipStream_t stream);

// Vector parameters (offsets, elementwise scales): the length axis of each example is cut into nrange ranges of
// rows_per_range tokens; the workspace holds [B][nrange][d] fp32 partial sums.
struct VecPlan {
    int nrange;
    int rows_per_range;
    size_t ws_bytes;
};
VecPlan plan_vec_stat(int64_t B, int64_t T, int64_t d, pex_dtype dt);
// s = sum_b phi(v_b), v_b[j] = sum_t A[b,t,j] * (C ? C[b,t,j] : 1); outputs that are NULL are not wanted
hipError_t launch_vec_stat(const void* A, const void* C, int64_t B, int64_t T, int64_t d, pex_dtype dt, const VecPlan& plan,
                           float* partial, float* s_id, float* s_sq, float* s_sign, hipStream_t stream);

// S[e] = sum_{s < nsplit} partial[s][e], s ascending (fixed order => deterministic).
hipError_t launch_reduce_partials(const float* partial, int nsplit, int64_t n, float* S, hipStream_t stream);
// the same for a range of columns: S[i * lds + j] = sum_s partial[s][i][j], i < rows, j < cols (cols a multiple of 4)
hipError_t launch_reduce_partials_cols(const float* partial, int nsplit, int64_t rows, int64_t cols, float* S, int64_t lds,
                                       hipStream_t stream);

hipError_t launch_adam_update(float* theta, float* m, float* v, const float* S_id, const float* S_sq, int64_t n,
                              pex_adam_variant variant, const pex_adam_params& p, hipStream_t stream,
                              const double* clip_sumsq = nullptr, float max_norm = 0.f);
// w[b] = min(1, max_norm / sqrt(sum_l N[l][b])) for N [nlayers][B]
hipError_t launch_clip_weights(const float* N, int64_t B, int nlayers, float max_norm, float* w, hipStream_t stream);
size_t sum_squares_workspace(int64_t n);
hipError_t launch_sum_squares(const float* x, int64_t n, double* acc, int accumulate, double* partial, hipStream_t stream);
hipError_t launch_sign_update(float* theta, float* m, const float* S, int64_t n, pex_sign_variant variant, float lr, float beta,
                              float weight_decay, int32_t B, int32_t debias, int64_t step, hipStream_t stream);

size_t moment_track_workspace(int64_t n);
hipError_t launch_moment_track(float* ema_adam, float* ema_micro, const float* S_id, const float* S_sq, int64_t n,
                               const pex_moment_params& p, double* sums, double* partial, hipStream_t stream);

size_t embed_workspace(int64_t B, int64_t T, int64_t V, int64_t d);
hipError_t launch_embed_stat(const void* ids, int ids_bytes, const void* G, int64_t B, int64_t T, int64_t V, int64_t d,
                             pex_dtype dt, uint32_t want, float* S_id, float* S_sq, float* S_sign, void* workspace,
                             hipStream_t stream);

size_t probe_operand_bytes();
size_t probe_sink_floats(int workgroups);
double probe_flop(int workgroups, int iters);
hipError_t launch_mfma_probe(const void* operands, int workgroups, int iters, float* sink, hipStream_t stream);

}  // namespace pex
