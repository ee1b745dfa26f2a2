// pex_stat_f32.hip -- fp32 MFMA kernel for S = sum_b phi(X_b^T G_b) and the per-token square, fp32 inputs (gfx950).
//
// Same mathematics as the bf16 kernel (Sec. 2.3): M_b = X_b^T G_b accumulates in registers, phi is applied to the
// finished per-example tile, the per-example gradient never leaves the register file.  fp32 inputs keep true fp32
// products (the 1e-4 tolerance of fp32 inputs forbids rounding them to bf16): v_mfma_f32_32x32x2_f32, 157 TFLOP/s at
// the datasheet clock -- the same as the vector FMA rate with packed operations, which this library is built without,
// so the matrix pipe is the only way past ~79 TFLOP/s.
//
// The fp32 pipe is 16 times slower than the bf16 one per byte of operand, so this kernel is bound by its MFMAs and
// needs none of the bf16 kernel's machinery: a workgroup of 4 waves owns a 128 x 128 tile (64 x 64 per wave, 2 x 2
// accumulators), slabs of 16 (or 8) tokens go global -> registers -> LDS through two buffers (the loads of slab s+1 are in
// flight while slab s is multiplied), one barrier per slab.  The t-major layout is what the MFMA wants as it is: the
// operand of 32x32x2 is one float per lane, row (lane % 32) of token (lane / 32), i.e. a plain ds_read_b32 of 32
// consecutive floats of one token and 32 of the next; LDS rows are padded by 32 floats so that the two tokens sit in
// different halves of the banks.  Three workgroups share a compute unit (at most 40 KB of LDS each), which is where
// the overlap of loads, LDS reads and MFMAs comes from.
#include "pex_internal.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(16))) float float16_t;

constexpr int F_BM = 128, F_BN = 128, F_LD = 128 + 32, F_THREADS = 256;

__device__ __forceinline__ float sign_of(float m) { return (float)((m > 0.f) - (m < 0.f)); }

// F_BK = tokens per slab.  Three workgroups per compute unit (three waves per SIMD) is where loads, LDS reads and
// MFMAs overlap best (measured against two and four), which caps a wave at 168 registers: two 64-register tiles plus
// the staging registers of a 16-token slab fit, except with the extra temporaries of sign and the powers, which take
// slabs of 8.
template <int MODE, int F_BK>
__global__ __launch_bounds__(F_THREADS) __attribute__((amdgpu_waves_per_eu(3, 3))) void stat_f32_kernel(const float* __restrict__ X, const float* __restrict__ G, int64_t rows_total,
                                                            int seg_len, int din, int dout, int64_t rows_per_split,
                                                            float* __restrict__ out, const float* __restrict__ weight, float alpha)
{
    constexpr bool PER_EXAMPLE = !(MODE == MODE_IDENTITY || MODE == MODE_TOKEN_SQ);
    constexpr int F_LOADS = F_BK * F_BM / 4 / F_THREADS;   // float4 loads per thread, operand and slab
    __shared__ __attribute__((aligned(16))) float Xs[2][F_BK][F_LD];
    __shared__ __attribute__((aligned(16))) float Gs[2][F_BK][F_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * F_BM, j0 = blockIdx.x * F_BN;
    const int64_t row_begin = (int64_t)blockIdx.z * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;
    const int slen = PER_EXAMPLE ? seg_len : (int)(row_end - row_begin);   // segment: one example, or the whole range
    const int nseg = PER_EXAMPLE ? (int)((row_end - row_begin) / seg_len) : (row_end > row_begin ? 1 : 0);
    const int nst = (slen + F_BK - 1) / F_BK;
    const int total = nseg * nst;

    float16_t acc[2][2], acc2[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[a][c][r] = 0.f; acc2[a][c][r] = 0.f; }

    // loader: float4 number q = tid + 256*u of a slab is row q / 32, columns 4*(q % 32) ..
    float4 xr[F_LOADS], gr[F_LOADS];
    auto gload = [&](int s) {
        const int seg = s / nst, st = s - seg * nst;
        const int64_t row0 = row_begin + (int64_t)seg * slen + (int64_t)st * F_BK;
        const int valid = (slen - st * F_BK) < F_BK ? (slen - st * F_BK) : F_BK;
#pragma unroll
        for (int u = 0; u < F_LOADS; ++u) {
            const int q = tid + F_THREADS * u, r = q >> 5, c = (q & 31) * 4;
            xr[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            gr[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < valid) {
                if (i0 + c < din) xr[u] = *(const float4*)(X + (row0 + r) * din + i0 + c);   // din % 4 == 0: whole or nothing
                if (j0 + c < dout) gr[u] = *(const float4*)(G + (row0 + r) * dout + j0 + c);
            }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int u = 0; u < F_LOADS; ++u) {
            const int q = tid + F_THREADS * u, r = q >> 5, c = (q & 31) * 4;
            float4 x = xr[u], g = gr[u];
            if (MODE == MODE_TOKEN_SQ) {   // exact fp32 squares
                x = make_float4(x.x * x.x, x.y * x.y, x.z * x.z, x.w * x.w);
                g = make_float4(g.x * g.x, g.y * g.y, g.z * g.z, g.w * g.w);
            }
            *(float4*)&Xs[buf][r][c] = x;
            *(float4*)&Gs[buf][r][c] = g;
        }
    };
    auto multiply = [&](int buf) {
        const int kk = lane >> 5, col = lane & 31;
#pragma unroll
        for (int ks = 0; ks < F_BK / 2; ++ks) {
            float a[2], b[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) a[m] = Xs[buf][2 * ks + kk][wm * 64 + m * 32 + col];
#pragma unroll
            for (int n = 0; n < 2; ++n) b[n] = Gs[buf][2 * ks + kk][wn * 64 + n * 32 + col];
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 2; ++n) acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m], b[n], acc[m][n], 0, 0, 0);
        }
    };
    int example = (int)(row_begin / (seg_len > 0 ? seg_len : 1));
    auto fold = [&]() {
        float w = 1.f;
        if (MODE == MODE_WEIGHTED) w = weight[example];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float m = acc[a][c][r];
                    if (MODE == MODE_SQUARE) acc2[a][c][r] = fmaf(m, m, acc2[a][c][r]);
                    if (MODE == MODE_SIGN) acc2[a][c][r] += sign_of(m);
                    if (MODE == MODE_WEIGHTED) acc2[a][c][r] = fmaf(w, m, acc2[a][c][r]);
                    if (MODE == MODE_POWER) acc2[a][c][r] += __builtin_amdgcn_exp2f(alpha * __builtin_amdgcn_logf(__builtin_fabsf(m)));
                    acc[a][c][r] = 0.f;
                }
        ++example;
    };

    if (total > 0) {
        gload(0);
        sstore(0);
        __syncthreads();
        int st_in_seg = 0;
        for (int s = 0; s < total; ++s) {
            if (s + 1 < total) gload(s + 1);     // in flight during the MFMAs of slab s
            multiply(s & 1);
            if (s + 1 < total) sstore((s + 1) & 1);
            __syncthreads();
            if (PER_EXAMPLE && ++st_in_seg == nst) { st_in_seg = 0; fold(); }
        }
    }

    // epilogue: lane holds column (lane % 32), rows 8*(r/4) + 4*(lane/32) + r%4 of each 32 x 32 tile
    float* dst = out + (int64_t)blockIdx.z * din * dout;
    const int jn = lane & 31, ib = 4 * (lane >> 5);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int j = j0 + wn * 64 + c * 32 + jn;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wm * 64 + a * 32 + 8 * (r / 4) + ib + (r % 4);
                if (i < din && j < dout) dst[(int64_t)i * dout + j] = PER_EXAMPLE ? acc2[a][c][r] : acc[a][c][r];
            }
        }
}

}  // namespace

void f32_tile_shape(int* bm, int* bn)
{
    *bm = F_BM;
    *bn = F_BN;
}

bool f32_mfma_supports(int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode)
{
    // rows of 16-byte multiples, at least a quarter of a tile, and every mode but the norms (which write no S)
    if (mode == MODE_NORMS) return false;
    return din % 4 == 0 && dout % 4 == 0 && din >= 32 && dout >= 32 && B * T >= 16;
}

hipError_t launch_stat_f32(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode,
                           const StatPlan& plan, float* out, hipStream_t stream, const float* weight, float alpha)
{
    const dim3 grid((unsigned)((dout + F_BN - 1) / F_BN), (unsigned)((din + F_BM - 1) / F_BM), (unsigned)plan.nsplit);
    const dim3 block(F_THREADS);
    const int64_t rows_total = B * T;
    const bool per_example = !(mode == MODE_IDENTITY || mode == MODE_TOKEN_SQ);
    const int64_t rows_per_split = per_example ? plan.per_split * T : plan.per_split;
    const float* x = (const float*)X;
    const float* g = (const float*)G;
#define PEX_F32_LAUNCH(M) stat_f32_kernel<M, (M == MODE_SIGN || M == MODE_POWER) ? 8 : 16><<<grid, block, 0, stream>>>(x, g, rows_total, (int)T, (int)din, (int)dout, rows_per_split, out, weight, alpha)
    switch (mode) {
    case MODE_IDENTITY: PEX_F32_LAUNCH(MODE_IDENTITY); break;
    case MODE_SQUARE: PEX_F32_LAUNCH(MODE_SQUARE); break;
    case MODE_SIGN: PEX_F32_LAUNCH(MODE_SIGN); break;
    case MODE_TOKEN_SQ: PEX_F32_LAUNCH(MODE_TOKEN_SQ); break;
    case MODE_WEIGHTED: PEX_F32_LAUNCH(MODE_WEIGHTED); break;
    case MODE_POWER: PEX_F32_LAUNCH(MODE_POWER); break;
    default: return hipErrorInvalidValue;
    }
#undef PEX_F32_LAUNCH
    return hipGetLastError();
}

}  // namespace pex
