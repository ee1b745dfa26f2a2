// pex_update.hip -- elementwise optimizer updates that consume the statistics (Algorithm 1, App. E, with
// the estimators of Eq. (musq_sigsq_est); the three placements of sign of Sec. 3.1: MicroSignSGD, SignSGD, SignEMA).  One pass, in place, bound by HBM
// bandwidth: Adam family 20 B read + 12 B written per parameter (16 + 12 for plain Adam, which never
// touches S_sq), MicroSignSGD 12 B read + 8 B written.  16-byte accesses, grid-stride, scalar tail.
#include "pex_internal.h"

namespace pex {
namespace {

struct AdamConsts {
    float beta1, one_m_beta1, beta2, one_m_beta2;
    float inv_bc1, inv_bc2;   // 1/(1-beta1^t), 1/(1-beta2^t)
    float eps, eps_root, lr, wd, gs, qs;
    float c_est, inv_B;       // 1/(1-1/B), 1/B
};

template <int VARIANT>
__device__ __forceinline__ void adam_one(float& th, float& m, float& v, float sid, float ssq, const AdamConsts& k)
{
    const float mu_t = k.gs * sid;
    const float nu_adam = mu_t * mu_t;
    float nu_t;
    if (VARIANT == PEX_ADAM) nu_t = nu_adam;
    else {
        const float nu_micro = k.qs * ssq;
        if (VARIANT == PEX_MICROADAM) nu_t = nu_micro;
        else if (VARIANT == PEX_MICROADAM_VAR) nu_t = k.c_est * (nu_micro - nu_adam);
        else nu_t = k.c_est * (nu_adam - nu_micro * k.inv_B);
    }
    m = fmaf(k.beta1, m, k.one_m_beta1 * mu_t);
    v = fmaf(k.beta2, v, k.one_m_beta2 * nu_t);
    const float mh = m * k.inv_bc1;
    float vh = v * k.inv_bc2;
    if (VARIANT == PEX_MICROADAM_VAR || VARIANT == PEX_MICROADAM_MSQ) vh = fmaxf(0.f, vh);
    const float u = mh / (sqrtf(vh + k.eps_root) + k.eps);
    th = th - k.lr * u - k.wd * th;
}

// clip_sumsq != nullptr: gradient clipping by the global norm (Sec. 3.2.3, App. C).  *clip_sumsq is the sum of S_id^2
// over all parameters of the model (device memory, written by sum_squares_kernel); every per-example gradient is
// multiplied by kappa = min(1, max_norm / (|grad_scale| * sqrt(*clip_sumsq))), i.e. the mean gradient by kappa and
// the per-example second moment by kappa^2.
template <int VARIANT>
__global__ __launch_bounds__(256) void adam_update_kernel(float* __restrict__ theta, float* __restrict__ m,
                                                          float* __restrict__ v, const float* __restrict__ S_id,
                                                          const float* __restrict__ S_sq, int64_t n, AdamConsts k,
                                                          const double* __restrict__ clip_sumsq, float max_norm)
{
    if (clip_sumsq) {
        const double norm = fabs((double)k.gs) * sqrt(*clip_sumsq);
        const float kappa = norm > (double)max_norm ? (float)((double)max_norm / norm) : 1.0f;
        k.gs *= kappa;
        k.qs *= kappa * kappa;
    }
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float4* th4 = reinterpret_cast<float4*>(theta);
    float4* m4 = reinterpret_cast<float4*>(m);
    float4* v4 = reinterpret_cast<float4*>(v);
    const float4* a4 = reinterpret_cast<const float4*>(S_id);
    const float4* q4 = reinterpret_cast<const float4*>(S_sq);
    for (int64_t e = gid; e < n4; e += stride) {
        float4 t = th4[e], mm = m4[e], vv = v4[e];
        const float4 a = a4[e];
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VARIANT != PEX_ADAM) q = q4[e];
        adam_one<VARIANT>(t.x, mm.x, vv.x, a.x, q.x, k);
        adam_one<VARIANT>(t.y, mm.y, vv.y, a.y, q.y, k);
        adam_one<VARIANT>(t.z, mm.z, vv.z, a.z, q.z, k);
        adam_one<VARIANT>(t.w, mm.w, vv.w, a.w, q.w, k);
        th4[e] = t; m4[e] = mm; v4[e] = vv;
    }
    for (int64_t e = n4 * 4 + gid; e < n; e += stride) {
        float t = theta[e], mm = m[e], vv = v[e];
        adam_one<VARIANT>(t, mm, vv, S_id[e], VARIANT != PEX_ADAM ? S_sq[e] : 0.f, k);
        theta[e] = t; m[e] = mm; v[e] = vv;
    }
}

// VARIANT: PEX_MICROSIGNSGD  m <- EMA(S/B), S = sum of per-example signs, step along m
//          PEX_SIGNSGD       m <- EMA(sign(S)), S = sum of gradients,     step along m
//          PEX_SIGNEMA       m <- EMA(S/B), S = sum of gradients,          step along sign(m)
template <int VARIANT>
__global__ __launch_bounds__(256) void signsgd_update_kernel(float* __restrict__ theta, float* __restrict__ m,
                                                             const float* __restrict__ S_sign, int64_t n, float lr,
                                                             float beta, float one_m_beta_over_B, float wd, float debias_mul)
{
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float4* th4 = reinterpret_cast<float4*>(theta);
    float4* m4 = reinterpret_cast<float4*>(m);
    const float4* s4 = reinterpret_cast<const float4*>(S_sign);
    auto sgn = [](float x) { return (float)((x > 0.f) - (x < 0.f)); };
    auto one = [&](float& t, float& mm, float s) {
        // for PEX_SIGNSGD the factor holds 1 - beta (the sign of S/B is the sign of S)
        mm = fmaf(beta, mm, one_m_beta_over_B * (VARIANT == PEX_SIGNSGD ? sgn(s) : s));
        const float dir = VARIANT == PEX_SIGNEMA ? sgn(mm) : mm * debias_mul;
        t = t - lr * dir - wd * t;
    };
    for (int64_t e = gid; e < n4; e += stride) {
        float4 t = th4[e], mm = m4[e];
        const float4 s = s4[e];
        one(t.x, mm.x, s.x); one(t.y, mm.y, s.y); one(t.z, mm.z, s.z); one(t.w, mm.w, s.w);
        th4[e] = t; m4[e] = mm;
    }
    for (int64_t e = n4 * 4 + gid; e < n; e += stride) {
        float t = theta[e], mm = m[e];
        one(t, mm, S_sign[e]);
        theta[e] = t; m[e] = mm;
    }
}

// On-line measurement of mu^2 and sigma^2 (Sec. 3.2.2): two EMAs with the optimizer's beta2 track nu_adam and nu_micro;
// the unbiased estimators of Eq. (musq_sigsq_est) are formed from the (bias-corrected) EMAs and summed over the
// parameters.  The EMAs are fp32 like the optimizer state; the estimators (differences of nearly equal numbers when
// one moment dominates) and their sums are formed in fp64.  Each workgroup writes one pair of partial sums; the
// second kernel adds the pairs in a fixed order, so the result does not depend on scheduling.
struct MomentConsts {
    float beta2, one_m_beta2, gs, qs;
    double corr, c_est, inv_B;   // 1/(1-beta2^t) or 1, 1/(1-1/B), 1/B
};

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ __launch_bounds__(256) void moment_track_kernel(float* __restrict__ ema_adam, float* __restrict__ ema_micro,
                                                           const float* __restrict__ S_id, const float* __restrict__ S_sq,
                                                           int64_t n, MomentConsts k, double* __restrict__ partial)
{
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float4* a4 = reinterpret_cast<float4*>(ema_adam);
    float4* q4 = reinterpret_cast<float4*>(ema_micro);
    const float4* i4 = reinterpret_cast<const float4*>(S_id);
    const float4* s4 = reinterpret_cast<const float4*>(S_sq);
    double sum_mu2 = 0.0, sum_sigma2 = 0.0;
    auto one = [&](float& a, float& q, float sid, float ssq) {
        const float mu_t = k.gs * sid;
        a = fmaf(k.beta2, a, k.one_m_beta2 * (mu_t * mu_t));
        q = fmaf(k.beta2, q, k.one_m_beta2 * (k.qs * ssq));
        const double ah = (double)a * k.corr, qh = (double)q * k.corr;
        sum_mu2 += k.c_est * (ah - qh * k.inv_B);
        sum_sigma2 += k.c_est * (qh - ah);
    };
    for (int64_t e = gid; e < n4; e += stride) {
        float4 a = a4[e], q = q4[e];
        const float4 si = i4[e], ss = s4[e];
        one(a.x, q.x, si.x, ss.x); one(a.y, q.y, si.y, ss.y); one(a.z, q.z, si.z, ss.z); one(a.w, q.w, si.w, ss.w);
        a4[e] = a; q4[e] = q;
    }
    for (int64_t e = n4 * 4 + gid; e < n; e += stride) {
        float a = ema_adam[e], q = ema_micro[e];
        one(a, q, S_id[e], S_sq[e]);
        ema_adam[e] = a; ema_micro[e] = q;
    }
    __shared__ double red[4][2];
    sum_mu2 = wave_sum(sum_mu2);
    sum_sigma2 = wave_sum(sum_sigma2);
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6][0] = sum_mu2; red[threadIdx.x >> 6][1] = sum_sigma2; }
    __syncthreads();
    if (threadIdx.x < 2) partial[(int64_t)blockIdx.x * 2 + threadIdx.x] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ __launch_bounds__(1024) void moment_finalize_kernel(const double* __restrict__ partial, int nparts, double* __restrict__ sums)
{
    // thread t adds partials t, t + 1024, ... (eight loads in flight), then the usual fixed-order tree
    double s0 = 0.0, s1 = 0.0;
    int i = threadIdx.x;
    for (; i + 7 * 1024 < nparts; i += 8 * 1024) {
        double a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { a[u] = partial[2 * (i + u * 1024)]; b[u] = partial[2 * (i + u * 1024) + 1]; }
#pragma unroll
        for (int u = 0; u < 8; ++u) { s0 += a[u]; s1 += b[u]; }
    }
    for (; i < nparts; i += 1024) { s0 += partial[2 * i]; s1 += partial[2 * i + 1]; }
    __shared__ double red[16][2];
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6][0] = s0; red[threadIdx.x >> 6][1] = s1; }
    __syncthreads();
    if (threadIdx.x < 2) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w][threadIdx.x];
        sums[threadIdx.x] = t;
    }
}

// acc[0] (+)= sum of x^2, squares and sums in fp64, fixed order (per thread, wave butterfly, workgroup, then one
// workgroup over the partials): the global gradient norm the clipping needs, reproducible bit for bit.
__global__ __launch_bounds__(256) void sum_squares_kernel(const float* __restrict__ x, int64_t n, double* __restrict__ partial)
{
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    double s = 0.0;
    for (int64_t e = gid; e < n4; e += stride) {
        const float4 a = x4[e];
        s += ((double)a.x * a.x + (double)a.y * a.y) + ((double)a.z * a.z + (double)a.w * a.w);
    }
    for (int64_t e = n4 * 4 + gid; e < n; e += stride) s += (double)x[e] * x[e];
    __shared__ double red[4];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(1024) void sum_squares_finalize_kernel(const double* __restrict__ partial, int nparts, int accumulate,
                                                                    double* __restrict__ acc)
{
    double s = 0.0;
    for (int i = threadIdx.x; i < nparts; i += 1024) s += partial[i];
    __shared__ double red[16];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w];
        acc[0] = accumulate ? acc[0] + t : t;
    }
}

inline unsigned update_grid(int64_t n)
{
    int64_t blocks = (n / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    const int64_t cap = 256 * 32;   // 256 CUs x 32 workgroups: enough loads in flight, short tail (measured best of 8 / 16 / 32)
    return (unsigned)(blocks > cap ? cap : blocks);
}

}  // namespace

hipError_t launch_adam_update(float* theta, float* m, float* v, const float* S_id, const float* S_sq, int64_t n,
                              pex_adam_variant variant, const pex_adam_params& p, hipStream_t stream, const double* clip_sumsq,
                              float max_norm)
{
    AdamConsts k;
    k.beta1 = p.beta1; k.one_m_beta1 = 1.f - p.beta1;
    k.beta2 = p.beta2; k.one_m_beta2 = 1.f - p.beta2;
    k.inv_bc1 = (float)(1.0 / (1.0 - pow((double)p.beta1, (double)p.step)));
    k.inv_bc2 = (float)(1.0 / (1.0 - pow((double)p.beta2, (double)p.step)));
    k.eps = p.eps; k.eps_root = p.eps_root; k.lr = p.lr; k.wd = p.weight_decay;
    k.gs = p.grad_scale; k.qs = p.sq_scale;
    k.inv_B = 1.f / (float)p.B;
    k.c_est = p.B > 1 ? (float)(1.0 / (1.0 - 1.0 / (double)p.B)) : 0.f;
    const dim3 grid(update_grid(n)), block(256);
    switch (variant) {
    case PEX_ADAM: adam_update_kernel<PEX_ADAM><<<grid, block, 0, stream>>>(theta, m, v, S_id, S_sq, n, k, clip_sumsq, max_norm); break;
    case PEX_MICROADAM: adam_update_kernel<PEX_MICROADAM><<<grid, block, 0, stream>>>(theta, m, v, S_id, S_sq, n, k, clip_sumsq, max_norm); break;
    case PEX_MICROADAM_VAR: adam_update_kernel<PEX_MICROADAM_VAR><<<grid, block, 0, stream>>>(theta, m, v, S_id, S_sq, n, k, clip_sumsq, max_norm); break;
    case PEX_MICROADAM_MSQ: adam_update_kernel<PEX_MICROADAM_MSQ><<<grid, block, 0, stream>>>(theta, m, v, S_id, S_sq, n, k, clip_sumsq, max_norm); break;
    }
    return hipGetLastError();
}

namespace {

// w[b] = min(1, max_norm / sqrt(sum over the layers of N[l][b])), the layers added in ascending order; an example
// whose squared norm is zero (or whose norm does not exceed max_norm) keeps w = 1
__global__ __launch_bounds__(256) void clip_weights_kernel(const float* __restrict__ N, int64_t B, int nlayers, float max_norm,
                                                           float* __restrict__ w)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    double total = 0.0;
    for (int l = 0; l < nlayers; ++l) total += (double)N[(int64_t)l * B + b];
    const double norm = sqrt(total);
    w[b] = norm > (double)max_norm ? (float)((double)max_norm / norm) : 1.0f;
}

}  // namespace

hipError_t launch_clip_weights(const float* N, int64_t B, int nlayers, float max_norm, float* w, hipStream_t stream)
{
    clip_weights_kernel<<<dim3((unsigned)((B + 255) / 256)), dim3(256), 0, stream>>>(N, B, nlayers, max_norm, w);
    return hipGetLastError();
}

size_t sum_squares_workspace(int64_t n) { return (size_t)update_grid(n) * sizeof(double); }

hipError_t launch_sum_squares(const float* x, int64_t n, double* acc, int accumulate, double* partial, hipStream_t stream)
{
    const unsigned grid = update_grid(n);
    sum_squares_kernel<<<dim3(grid), dim3(256), 0, stream>>>(x, n, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    sum_squares_finalize_kernel<<<dim3(1), dim3(1024), 0, stream>>>(partial, (int)grid, accumulate, acc);
    return hipGetLastError();
}

size_t moment_track_workspace(int64_t n) { return (size_t)update_grid(n) * 2 * sizeof(double); }

hipError_t launch_moment_track(float* ema_adam, float* ema_micro, const float* S_id, const float* S_sq, int64_t n,
                               const pex_moment_params& p, double* sums, double* partial, hipStream_t stream)
{
    MomentConsts k;
    k.beta2 = p.beta2; k.one_m_beta2 = 1.f - p.beta2;
    k.gs = p.grad_scale; k.qs = p.sq_scale;
    k.corr = p.debias ? 1.0 / (1.0 - pow((double)p.beta2, (double)p.step)) : 1.0;
    k.inv_B = 1.0 / (double)p.B;
    k.c_est = 1.0 / (1.0 - k.inv_B);
    const unsigned grid = update_grid(n);
    moment_track_kernel<<<dim3(grid), dim3(256), 0, stream>>>(ema_adam, ema_micro, S_id, S_sq, n, k, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    moment_finalize_kernel<<<dim3(1), dim3(1024), 0, stream>>>(partial, (int)grid, sums);
    return hipGetLastError();
}

hipError_t launch_sign_update(float* theta, float* m, const float* S, int64_t n, pex_sign_variant variant, float lr, float beta,
                              float weight_decay, int32_t B, int32_t debias, int64_t step, hipStream_t stream)
{
    const float debias_mul = debias ? (float)(1.0 / (1.0 - pow((double)beta, (double)step))) : 1.f;
    const float w = (1.f - beta) / (float)B;
    const dim3 grid(update_grid(n)), block(256);
    switch (variant) {
    case PEX_MICROSIGNSGD: signsgd_update_kernel<PEX_MICROSIGNSGD><<<grid, block, 0, stream>>>(theta, m, S, n, lr, beta, w, weight_decay, debias_mul); break;
    case PEX_SIGNSGD: signsgd_update_kernel<PEX_SIGNSGD><<<grid, block, 0, stream>>>(theta, m, S, n, lr, beta, 1.f - beta, weight_decay, debias_mul); break;
    case PEX_SIGNEMA: signsgd_update_kernel<PEX_SIGNEMA><<<grid, block, 0, stream>>>(theta, m, S, n, lr, beta, w, weight_decay, 1.f); break;
    }
    return hipGetLastError();
}

}  // namespace pex
