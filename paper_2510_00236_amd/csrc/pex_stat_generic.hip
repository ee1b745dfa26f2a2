// pex_stat_generic.hip -- shape-agnostic SIMT kernel for S = sum_b phi(X_b^T G_b) and the per-token
// square.  Handles any B, T, din, dout >= 1 and both storage types with true fp32 products; it is the
// path for fp32 inputs and for bf16 shapes the MFMA kernel does not take.  Latency/ALU bound by design:
// the tuned path lives in pex_stat_bf16.hip.
//
// One workgroup (16 x 16 lanes) owns a 64 x 64 tile of S for one group of examples.  For each example it
// walks the sequence in slabs of 16 tokens staged through LDS, keeps the running tile of M_b in registers
// (4 x 4 per lane), applies phi at the end of the sequence and adds into a second register tile
// (Sec. 2.3: reduce over the length first, then phi, then over the batch).
#include "pex_internal.h"

namespace pex {
namespace {

constexpr int TM = 64, TN = 64, TK = 16, NTHREADS = 256;

__device__ __forceinline__ float load_as_float(const float* p) { return *p; }
__device__ __forceinline__ float load_as_float(const uint16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }

// end of an example: acc2 += phi(M_b) (weighted identity for MODE_WEIGHTED), norm += ||M_b||^2 of this lane's part
template <int MODE>
__device__ __forceinline__ void fold(float (&acc2)[4][4], float (&acc)[4][4], float w, float& norm)
{
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float m = acc[a][c];
            if (MODE == MODE_SQUARE) acc2[a][c] = fmaf(m, m, acc2[a][c]);
            else if (MODE == MODE_SIGN) acc2[a][c] += (float)((m > 0.f) - (m < 0.f));
            else if (MODE == MODE_WEIGHTED) acc2[a][c] = fmaf(w, m, acc2[a][c]);
            else if (MODE == MODE_POWER) acc2[a][c] += __builtin_amdgcn_exp2f(w * __builtin_amdgcn_logf(__builtin_fabsf(m)));
            else if (MODE == MODE_NORMS) norm = fmaf(m, m, norm);
            acc[a][c] = 0.f;
        }
}

// Rows of the flattened [B*T] axis processed by this workgroup: [row_begin, row_end); for the
// per-example modes the range is a whole number of examples and `T` marks the example boundaries.
template <typename TIn, int MODE>
__global__ __launch_bounds__(NTHREADS) void stat_generic_kernel(const TIn* __restrict__ X, const TIn* __restrict__ G,
                                                                int64_t rows_total, int64_t T, int din, int dout,
                                                                int64_t rows_per_split, float* __restrict__ out,
                                                                const float* __restrict__ weight,
                                                                float* __restrict__ norm_partial, int examples_total, float alpha)
{
    __shared__ float sX[TK][TM + 4];
    __shared__ float sG[TK][TN + 4];
    __shared__ float sN[NTHREADS];

    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
    const int64_t row_begin = (int64_t)blockIdx.z * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;

    constexpr bool PER_EXAMPLE = (MODE == MODE_SQUARE || MODE == MODE_SIGN || MODE == MODE_NORMS || MODE == MODE_WEIGHTED || MODE == MODE_POWER);
    float acc[4][4], acc2[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = acc2[a][c] = 0.f;

    const int lr = tid / 16;        // slab row this lane stages
    const int lc = (tid % 16) * 4;  // first of the 4 columns this lane stages

    // segment = one example for the per-example modes, the whole range otherwise
    const int64_t seg_len = PER_EXAMPLE ? T : (row_end - row_begin);
    for (int64_t seg = row_begin; seg < row_end; seg += seg_len) {
        for (int64_t r0 = 0; r0 < seg_len; r0 += TK) {
            const int64_t r = seg + r0 + lr;
            const bool row_ok = (r0 + lr) < seg_len;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = i0 + lc + e, j = j0 + lc + e;
                float xv = (row_ok && i < din) ? load_as_float(X + r * din + i) : 0.f;
                float gv = (row_ok && j < dout) ? load_as_float(G + r * dout + j) : 0.f;
                if (MODE == MODE_TOKEN_SQ) { xv *= xv; gv *= gv; }
                sX[lr][lc + e] = xv;
                sG[lr][lc + e] = gv;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < TK; ++k) {
                float xa[4], gb[4];
#pragma unroll
                for (int a = 0; a < 4; ++a) xa[a] = sX[k][ty * 4 + a];
#pragma unroll
                for (int c = 0; c < 4; ++c) gb[c] = sG[k][tx * 4 + c];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(xa[a], gb[c], acc[a][c]);
            }
            __syncthreads();
        }
        if (PER_EXAMPLE) {
            const int example = (int)(seg / T);
            float norm = 0.f;
            fold<MODE>(acc2, acc, MODE == MODE_WEIGHTED ? weight[example] : (MODE == MODE_POWER ? alpha : 1.0f), norm);
            if (MODE == MODE_NORMS) {
                // this tile's part of ||M_b||^2: fixed-order tree over the 256 lanes
                sN[tid] = norm;
                __syncthreads();
                for (int h = NTHREADS / 2; h >= 1; h >>= 1) {
                    if (tid < h) sN[tid] += sN[tid + h];
                    __syncthreads();
                }
                if (tid == 0) norm_partial[((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * examples_total + example] = sN[0];
            }
        }
    }
    if (MODE == MODE_NORMS) return;

    float* dst = out + (int64_t)blockIdx.z * din * dout;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int i = i0 + ty * 4 + a;
        if (i >= din) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = j0 + tx * 4 + c;
            if (j < dout) dst[(int64_t)i * dout + j] = PER_EXAMPLE ? acc2[a][c] : acc[a][c];
        }
    }
}

template <typename TIn>
hipError_t launch_typed(const TIn* X, const TIn* G, int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode,
                        const StatPlan& plan, float* out, hipStream_t stream, const float* weight, float* norm_partial, float alpha)
{
    const dim3 grid((unsigned)((dout + TN - 1) / TN), (unsigned)((din + TM - 1) / TM), (unsigned)plan.nsplit);
    const dim3 block(NTHREADS);
    const int64_t rows_total = B * T;
    const bool per_example = (mode == MODE_SQUARE || mode == MODE_SIGN || mode == MODE_NORMS || mode == MODE_WEIGHTED || mode == MODE_POWER);
    const int64_t rows_per_split = per_example ? plan.per_split * T : plan.per_split;
    switch (mode) {
    case MODE_IDENTITY:
        stat_generic_kernel<TIn, MODE_IDENTITY><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_SQUARE:
        stat_generic_kernel<TIn, MODE_SQUARE><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_SIGN:
        stat_generic_kernel<TIn, MODE_SIGN><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_NORMS:
        stat_generic_kernel<TIn, MODE_NORMS><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_WEIGHTED:
        stat_generic_kernel<TIn, MODE_WEIGHTED><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_POWER:
        stat_generic_kernel<TIn, MODE_POWER><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    case MODE_TOKEN_SQ:
        stat_generic_kernel<TIn, MODE_TOKEN_SQ><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out, weight, norm_partial, (int)B, alpha);
        break;
    }
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int nsplit, int64_t n,
                                                              float* __restrict__ S)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) {
        float s = partial[e];
        for (int k = 1; k < nsplit; ++k) s += partial[(int64_t)k * n + e];
        S[e] = s;
    }
}

// the same sum for a range of columns of S: partial rows are `cols` long, S rows `ld`; four columns per lane
__global__ __launch_bounds__(256) void reduce_partials_cols_kernel(const float4* __restrict__ partial, int nsplit, int64_t rows, int64_t cols4,
                                                                   float* __restrict__ S, int64_t ld)
{
    const int64_t n4 = rows * cols4, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n4; e += stride) {
        float4 s = partial[e];
        for (int k = 1; k < nsplit; ++k) {
            const float4 p = partial[(int64_t)k * n4 + e];
            s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
        }
        const int64_t i = e / cols4, j4 = e - i * cols4;
        *(float4*)(S + i * ld + j4 * 4) = s;
    }
}

}  // namespace

hipError_t launch_stat_generic(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                               pex_dtype dt, Mode mode, const StatPlan& plan, float* out, hipStream_t stream,
                               const float* weight, float* norm_partial, float alpha)
{
    if (dt == PEX_F32)
        return launch_typed((const float*)X, (const float*)G, B, T, din, dout, mode, plan, out, stream, weight, norm_partial, alpha);
    return launch_typed((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, mode, plan, out, stream, weight, norm_partial, alpha);
}

int64_t generic_norm_partials(int64_t din, int64_t dout) { return ((din + TM - 1) / TM) * ((dout + TN - 1) / TN); }

namespace {

// one block per example: lanes sum a strided subset in ascending order, then a fixed-order tree
__global__ __launch_bounds__(256) void reduce_norms_kernel(const float* __restrict__ partial, int64_t nparts, int64_t B,
                                                           float* __restrict__ N)
{
    __shared__ float red[256];
    const int64_t b = blockIdx.x;
    float s = 0.f;
    for (int64_t p = threadIdx.x; p < nparts; p += 256) s += partial[p * B + b];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) N[b] = red[0];
}

// sum of squares of n values starting at p, this lane's share: 16-byte loads when WIDE, scalar otherwise
template <typename TIn, bool WIDE>
__device__ __forceinline__ float lane_sumsq(const TIn* p, int64_t n, int lane)
{
    float s = 0.f;
    if constexpr (WIDE) {
        typedef __attribute__((ext_vector_type(4))) unsigned int u4;
        constexpr int PER = 16 / (int)sizeof(TIn);
        for (int64_t i = (int64_t)lane * PER; i < n; i += 64 * PER) {
            const u4 raw = __builtin_nontemporal_load((const u4*)(p + i));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (sizeof(TIn) == 2) {
                    const float lo = __uint_as_float(raw[e] << 16), hi = __uint_as_float(raw[e] & 0xffff0000u);
                    s = fmaf(lo, lo, s);
                    s = fmaf(hi, hi, s);
                } else {
                    const float v = __uint_as_float(raw[e]);
                    s = fmaf(v, v, s);
                }
            }
        }
    } else {
        for (int64_t i = lane; i < n; i += 64) { const float v = load_as_float(p + i); s = fmaf(v, v, s); }
    }
    return s;
}

// one wave per row: |x_r|^2 * |g_r|^2, lanes stride over the features, butterfly sum
template <typename TIn, bool WIDE>
__global__ __launch_bounds__(256) void token_norms_kernel(const TIn* __restrict__ X, const TIn* __restrict__ G, int64_t rows,
                                                          int64_t din, int64_t dout, float* __restrict__ N_tok)
{
    const int lane = threadIdx.x % 64;
    const int64_t r = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (r >= rows) return;
    float sx = lane_sumsq<TIn, WIDE>(X + r * din, din, lane);
    float sg = lane_sumsq<TIn, WIDE>(G + r * dout, dout, lane);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { sx += __shfl_xor(sx, off); sg += __shfl_xor(sg, off); }
    if (lane == 0) N_tok[r] = sx * sg;
}

}  // namespace

hipError_t launch_reduce_norms(const float* partial, int64_t nparts, int64_t B, float* N, hipStream_t stream)
{
    reduce_norms_kernel<<<dim3((unsigned)B), dim3(256), 0, stream>>>(partial, nparts, B, N);
    return hipGetLastError();
}

hipError_t launch_token_norms(const void* X, const void* G, int64_t rows, int64_t din, int64_t dout, pex_dtype dt, float* N_tok,
                              hipStream_t stream)
{
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    const int per = dt == PEX_F32 ? 4 : 8;
    const bool wide = din % per == 0 && dout % per == 0 && ((((uintptr_t)X | (uintptr_t)G) & 15u) == 0);
    if (dt == PEX_F32) {
        if (wide) token_norms_kernel<float, true><<<grid, block, 0, stream>>>((const float*)X, (const float*)G, rows, din, dout, N_tok);
        else token_norms_kernel<float, false><<<grid, block, 0, stream>>>((const float*)X, (const float*)G, rows, din, dout, N_tok);
    } else {
        if (wide) token_norms_kernel<uint16_t, true><<<grid, block, 0, stream>>>((const uint16_t*)X, (const uint16_t*)G, rows, din, dout, N_tok);
        else token_norms_kernel<uint16_t, false><<<grid, block, 0, stream>>>((const uint16_t*)X, (const uint16_t*)G, rows, din, dout, N_tok);
    }
    return hipGetLastError();
}

hipError_t launch_reduce_partials_cols(const float* partial, int nsplit, int64_t rows, int64_t cols, float* S, int64_t ld,
                                       hipStream_t stream)
{
    if (cols % 4 != 0 || ld % 4 != 0) return hipErrorInvalidValue;
    int64_t blocks = (rows * (cols / 4) + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    reduce_partials_cols_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const float4*)partial, nsplit, rows, cols / 4, S, ld);
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const float* partial, int nsplit, int64_t n, float* S, hipStream_t stream)
{
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    reduce_partials_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(partial, nsplit, n, S);
    return hipGetLastError();
}

}  // namespace pex
