// pex_vec_stat.hip -- per-example statistics of vector parameters (offsets, elementwise scales).
//
// An offset added on the batch and the length axis is a contraction of the cotangents with a vector of ones
// (App. B, "Affine operations"): its per-example gradient is v_b[j] = sum_t A[b,t,j]; an elementwise scale
// applied to an activation C has v_b[j] = sum_t A[b,t,j] * C[b,t,j].  The statistic is s = sum_b phi(v_b), phi as
// for weight matrices (Sec. 2.3).  Every input byte is read once and the arithmetic is one FMA per element, so
// the bound is HBM bandwidth: B*T*d*sizeof(element) bytes per operand.
//
// Two kernels, both deterministic (fixed summation order, no atomics):
//   vec_partial_kernel   block = 64 column lanes x 4 row lanes; a lane owns VEC consecutive columns (16 bytes) and
//                        every 4th row of one range of tokens of one example; the four row lanes are summed
//                        through LDS and the block writes partial[b][range][columns] in fp32;
//   vec_finalize_kernel  per column: v_b = sum over ranges (ascending), then the requested phi, then sum over b
//                        (examples dealt to four lanes, combined in lane order).
// The partial sums are B * ranges * d floats: the per-example gradients of a *vector* parameter, which is the one
// place where holding them is cheap (B*d, not B*din*dout).
#include "pex_internal.h"

namespace pex {
namespace {

constexpr int CW = 64, RW = 4;   // column lanes and row lanes of a block

template <typename TIn> struct VecOf;
template <> struct VecOf<uint16_t> { static constexpr int N = 8; };   // 8 bf16 = 16 bytes
template <> struct VecOf<float> { static constexpr int N = 4; };      // 4 fp32 = 16 bytes

__device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float widen(float f) { return f; }

template <typename TIn, int VEC>
__device__ __forceinline__ void load_vec(const TIn* p, float (&v)[VEC])
{
    if constexpr (VEC == 1) v[0] = widen(p[0]);
    else {
        typedef __attribute__((ext_vector_type(4))) unsigned int u4;
        const u4 raw = __builtin_nontemporal_load((const u4*)p);
        if constexpr (sizeof(TIn) == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[2 * e] = __uint_as_float(raw[e] << 16);
                v[2 * e + 1] = __uint_as_float(raw[e] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(raw[e]);
        }
    }
}

// partial[(b * nrange + range) * d + j] = sum over the tokens of the range of A[b,t,j] * (HAS_C ? C[b,t,j] : 1)
template <typename TIn, int VEC, bool HAS_C>
__global__ __launch_bounds__(CW * RW) void vec_partial_kernel(const TIn* __restrict__ A, const TIn* __restrict__ C, int T, int64_t d,
                                                              int nrange, int rows_per_range, float* __restrict__ partial)
{
    __shared__ float red[RW][CW][VEC];
    const int cl = threadIdx.x % CW, rl = threadIdx.x / CW;
    const int64_t j = ((int64_t)blockIdx.x * CW + cl) * VEC;
    const int b = blockIdx.y / nrange, range = blockIdx.y % nrange;
    const int t0 = range * rows_per_range;
    const int t1 = (t0 + rows_per_range < T) ? t0 + rows_per_range : T;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    if (j < d) {
        const TIn* a = A + ((int64_t)b * T) * d + j;
        const TIn* c = HAS_C ? C + ((int64_t)b * T) * d + j : nullptr;
        int t = t0 + rl;
        // four rows in flight per lane
        for (; t + 3 * RW < t1; t += 4 * RW) {
            float x[4][VEC], y[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                load_vec<TIn, VEC>(a + (int64_t)(t + u * RW) * d, x[u]);
                if (HAS_C) load_vec<TIn, VEC>(c + (int64_t)(t + u * RW) * d, y[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = HAS_C ? fmaf(x[u][e], y[u][e], acc[e]) : acc[e] + x[u][e];
        }
        for (; t < t1; t += RW) {
            float x0[VEC], y0[VEC];
            load_vec<TIn, VEC>(a + (int64_t)t * d, x0);
            if (HAS_C) load_vec<TIn, VEC>(c + (int64_t)t * d, y0);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = HAS_C ? fmaf(x0[e], y0[e], acc[e]) : acc[e] + x0[e];
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[rl][cl][e] = acc[e];
    __syncthreads();
    if (rl == 0 && j < d) {
        float* dst = partial + ((int64_t)b * nrange + range) * d + j;
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[e] = ((red[0][cl][e] + red[1][cl][e]) + red[2][cl][e]) + red[3][cl][e];
    }
}

// per column: v_b = sum over ranges (ascending); the examples are dealt to four lanes (b mod 4), each sums its
// phi(v_b) in ascending b, and the four lanes are combined in lane order
__global__ __launch_bounds__(CW * RW) void vec_finalize_kernel(const float* __restrict__ partial, int B, int nrange, int64_t d,
                                                               float* __restrict__ s_id, float* __restrict__ s_sq,
                                                               float* __restrict__ s_sign)
{
    __shared__ float red[3][RW][CW];
    const int cl = threadIdx.x % CW, bl = threadIdx.x / CW;
    const int64_t j = (int64_t)blockIdx.x * CW + cl;
    float a_id = 0.f, a_sq = 0.f, a_sg = 0.f;
    if (j < d) {
        for (int b = bl; b < B; b += RW) {
            const float* p = partial + (int64_t)b * nrange * d + j;
            float v = 0.f;
            int r = 0;
            for (; r + 8 <= nrange; r += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = p[(int64_t)(r + u) * d];
#pragma unroll
                for (int u = 0; u < 8; ++u) v += x[u];
            }
            for (; r < nrange; ++r) v += p[(int64_t)r * d];
            a_id += v;
            a_sq = fmaf(v, v, a_sq);
            a_sg += (float)((v > 0.f) - (v < 0.f));
        }
    }
    red[0][bl][cl] = a_id;
    red[1][bl][cl] = a_sq;
    red[2][bl][cl] = a_sg;
    __syncthreads();
    if (bl == 0 && j < d) {
        if (s_id) s_id[j] = ((red[0][0][cl] + red[0][1][cl]) + red[0][2][cl]) + red[0][3][cl];
        if (s_sq) s_sq[j] = ((red[1][0][cl] + red[1][1][cl]) + red[1][2][cl]) + red[1][3][cl];
        if (s_sign) s_sign[j] = ((red[2][0][cl] + red[2][1][cl]) + red[2][2][cl]) + red[2][3][cl];
    }
}

template <typename TIn>
hipError_t launch_typed(const TIn* A, const TIn* C, int64_t B, int64_t T, int64_t d, const VecPlan& plan, float* partial,
                        hipStream_t stream)
{
    constexpr int V = VecOf<TIn>::N;
    const bool wide = (d % V == 0) && ((((uintptr_t)A | (uintptr_t)C) & 15u) == 0);
    const int vec = wide ? V : 1;
    const dim3 grid((unsigned)((d + (int64_t)CW * vec - 1) / ((int64_t)CW * vec)), (unsigned)(B * plan.nrange));
    const dim3 block(CW * RW);
#define PEX_VEC_LAUNCH(VEC, HAS_C) \
    vec_partial_kernel<TIn, VEC, HAS_C><<<grid, block, 0, stream>>>(A, C, (int)T, d, plan.nrange, plan.rows_per_range, partial)
    if (wide) {
        if (C) PEX_VEC_LAUNCH(V, true);
        else PEX_VEC_LAUNCH(V, false);
    } else {
        if (C) PEX_VEC_LAUNCH(1, true);
        else PEX_VEC_LAUNCH(1, false);
    }
#undef PEX_VEC_LAUNCH
    return hipGetLastError();
}

}  // namespace

VecPlan plan_vec_stat(int64_t B, int64_t T, int64_t d, pex_dtype dt)
{
    // as many blocks as are resident at once (eight per compute unit) and no more, so that there is no second,
    // mostly empty round of blocks; ranges of at least 32 tokens
    VecPlan p{};
    const int vec = dt == PEX_BF16 ? 8 : 4;
    const int64_t chunks = (d + CW * vec - 1) / (CW * vec);
    int64_t nrange = 2048 / (chunks * B);
    const int64_t max_range = (T + 31) / 32;
    if (nrange > max_range) nrange = max_range;
    if (nrange < 1) nrange = 1;
    int64_t rows = (T + nrange - 1) / nrange;
    rows = (rows + RW - 1) / RW * RW;
    nrange = (T + rows - 1) / rows;
    p.nrange = (int)nrange;
    p.rows_per_range = (int)rows;
    p.ws_bytes = (size_t)B * (size_t)nrange * (size_t)d * sizeof(float);
    return p;
}

hipError_t launch_vec_stat(const void* A, const void* C, int64_t B, int64_t T, int64_t d, pex_dtype dt, const VecPlan& plan,
                           float* partial, float* s_id, float* s_sq, float* s_sign, hipStream_t stream)
{
    hipError_t e = dt == PEX_F32 ? launch_typed((const float*)A, (const float*)C, B, T, d, plan, partial, stream)
                                 : launch_typed((const uint16_t*)A, (const uint16_t*)C, B, T, d, plan, partial, stream);
    if (e != hipSuccess) return e;
    vec_finalize_kernel<<<dim3((unsigned)((d + CW - 1) / CW)), dim3(CW * RW), 0, stream>>>(partial, (int)B, plan.nrange, d, s_id, s_sq, s_sign);
    return hipGetLastError();
}

}  // namespace pex
