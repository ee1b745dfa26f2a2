// pex_stat_generic.hip -- shape-agnostic SIMT kernel for S = sum_b phi(X_b^T G_b) and the per-token
// square.  Handles any B, T, din, dout >= 1 and both storage types with true fp32 products; it is the
// path for fp32 inputs and for bf16 shapes the MFMA kernel does not take.  Latency/ALU bound by design:
// the tuned path lives in pex_stat_mfma.hip.
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

template <int MODE>
__device__ __forceinline__ void fold(float (&acc2)[4][4], float (&acc)[4][4])
{
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float m = acc[a][c];
            if (MODE == MODE_SQUARE) acc2[a][c] = fmaf(m, m, acc2[a][c]);
            else if (MODE == MODE_SIGN) acc2[a][c] += (float)((m > 0.f) - (m < 0.f));
            acc[a][c] = 0.f;
        }
}

// Rows of the flattened [B*T] axis processed by this workgroup: [row_begin, row_end); for the
// per-example modes the range is a whole number of examples and `T` marks the example boundaries.
template <typename TIn, int MODE>
__global__ __launch_bounds__(NTHREADS) void stat_generic_kernel(const TIn* __restrict__ X, const TIn* __restrict__ G,
                                                                int64_t rows_total, int64_t T, int din, int dout,
                                                                int64_t rows_per_split, float* __restrict__ out)
{
    __shared__ float sX[TK][TM + 4];
    __shared__ float sG[TK][TN + 4];

    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
    const int64_t row_begin = (int64_t)blockIdx.z * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;

    constexpr bool PER_EXAMPLE = (MODE == MODE_SQUARE || MODE == MODE_SIGN);
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
        if (PER_EXAMPLE) fold<MODE>(acc2, acc);
    }

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
                        const StatPlan& plan, float* out, hipStream_t stream)
{
    const dim3 grid((unsigned)((dout + TN - 1) / TN), (unsigned)((din + TM - 1) / TM), (unsigned)plan.nsplit);
    const dim3 block(NTHREADS);
    const int64_t rows_total = B * T;
    const bool per_example = (mode == MODE_SQUARE || mode == MODE_SIGN);
    const int64_t rows_per_split = per_example ? plan.per_split * T : plan.per_split;
    switch (mode) {
    case MODE_IDENTITY:
        stat_generic_kernel<TIn, MODE_IDENTITY><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out);
        break;
    case MODE_SQUARE:
        stat_generic_kernel<TIn, MODE_SQUARE><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out);
        break;
    case MODE_SIGN:
        stat_generic_kernel<TIn, MODE_SIGN><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out);
        break;
    case MODE_TOKEN_SQ:
        stat_generic_kernel<TIn, MODE_TOKEN_SQ><<<grid, block, 0, stream>>>(X, G, rows_total, T, (int)din, (int)dout, rows_per_split, out);
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

}  // namespace

hipError_t launch_stat_generic(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                               pex_dtype dt, Mode mode, const StatPlan& plan, float* out, hipStream_t stream)
{
    if (dt == PEX_F32)
        return launch_typed((const float*)X, (const float*)G, B, T, din, dout, mode, plan, out, stream);
    return launch_typed((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, mode, plan, out, stream);
}

hipError_t launch_reduce_partials(const float* partial, int nsplit, int64_t n, float* S, hipStream_t stream)
{
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    reduce_partials_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(partial, nsplit, n, S);
    return hipGetLastError();
}

}  // namespace pex
