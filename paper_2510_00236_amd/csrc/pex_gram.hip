// pex_gram.hip -- per-example squared gradient norms through the T x T Gram matrices (gfx950, bf16 inputs).
//
// Sec. 2.3 remarks that the squared norm of a per-example gradient of a dense sequence layer needs no gradient at
// all ("ghost" norm):
//     N_b = || X_b^T G_b ||_F^2 = sum_{t,t'} (X_b X_b^T)[t,t'] * (G_b G_b^T)[t,t'],
// 2 T^2 (din + dout) FLOP per example against 2 T din dout for the contraction itself -- cheaper when
// T < din*dout/(din+dout), and, what matters more on layers with few tiles, with no partial sums of S to exchange:
// a workgroup produces one number.
//
// One workgroup (4 waves) owns a 64 x 64 block (ti, tj), ti <= tj, of the two Gram matrices of one example; each
// wave a 32 x 32 quarter as 2 x 2 accumulators of v_mfma_f32_16x16x32_bf16, once for X X^T and once for G G^T.  The
// contraction runs over the features, which are contiguous in memory: an operand fragment is 16 rows x 32 features
// with 16 bytes per lane, read from LDS with plain ds_read_b128 (rows padded to 144 bytes: the 16 lanes of a read
// fall in 16 different groups of four banks).  Steps of 64 features go global -> registers -> LDS through two
// buffers, the loads of step s+1 in flight while step s is multiplied, one barrier per step; the steps over din and
// over dout form one pipeline.  At the end the block contributes sum(A o B), twice if it is off the diagonal
// (both matrices are symmetric), added over the workgroup in a fixed order.  Rows beyond T and features beyond the
// row are loaded as zeros.
#include "pex_internal.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int uint4_t;

constexpr int GB = 64;                 // block edge, tokens
constexpr int GK = 64;                 // features per step (128 halves the barriers but the LDS it takes costs more: measured)
constexpr int GLD = GK * 2 + 16;       // LDS row pitch, bytes
constexpr int G_THREADS = 256;
constexpr int G_CHUNKS = GB * GK * 2 / 16 / G_THREADS;   // 16-byte chunks per thread, panel and step (2)

__global__ __launch_bounds__(G_THREADS) void gram_norms_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ G, int T,
                                                                int din, int dout, int nb, float* __restrict__ partial, int B)
{
    __shared__ __attribute__((aligned(16))) unsigned char Ls[2][2][GB][GLD];     // [buffer][panel: rows of ti, rows of tj]
    __shared__ float red[G_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave >> 1, wj = wave & 1;
    const int b = blockIdx.y;
    // pair number -> (ti, tj) with ti <= tj, rows of the upper triangle one after the other
    int ti = 0, rem = blockIdx.x;
    while (rem >= nb - ti) { rem -= nb - ti; ++ti; }
    const int tj = ti + rem;

    const int nx = (din + GK - 1) / GK, ng = (dout + GK - 1) / GK, nsteps = nx + ng;
    const uint16_t* xb = X + (int64_t)b * T * din;
    const uint16_t* gb = G + (int64_t)b * T * dout;

    // loader: chunk q = tid + 256*u of a panel is row q / (GK/8), features 8*(q % (GK/8)) .. +7 of the step
    uint4_t stage[2][G_CHUNKS];
    auto fetch = [&](int s) {
        const bool in_x = s < nx;
        const uint16_t* src = in_x ? xb : gb;
        const int d = in_x ? din : dout, k0 = (in_x ? s : s - nx) * GK;
#pragma unroll
        for (int pn = 0; pn < 2; ++pn)
#pragma unroll
            for (int u = 0; u < G_CHUNKS; ++u) {
                const int q = tid + G_THREADS * u, row = q / (GK / 8), f = k0 + 8 * (q % (GK / 8));
                const int t = (pn == 0 ? ti : tj) * GB + row;
                stage[pn][u] = (t < T && f < d) ? *(const uint4_t*)(src + (int64_t)t * d + f) : uint4_t{0u, 0u, 0u, 0u};
            }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int pn = 0; pn < 2; ++pn)
#pragma unroll
            for (int u = 0; u < G_CHUNKS; ++u) {
                const int q = tid + G_THREADS * u;
                *(uint4_t*)&Ls[buf][pn][q / (GK / 8)][16 * (q % (GK / 8))] = stage[pn][u];
            }
    };

    float4_t accx[2][2], accg[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            accx[a][c] = float4_t{0.f, 0.f, 0.f, 0.f};
            accg[a][c] = float4_t{0.f, 0.f, 0.f, 0.f};
        }
    const int li = lane & 15, blk = lane >> 4;
    auto multiply = [&](int buf, float4_t (&acc)[2][2]) {
#pragma unroll
        for (int ks = 0; ks < GK / 32; ++ks) {
            bf16x8_t fi[2], fj[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fi[a] = *(const bf16x8_t*)&Ls[buf][0][32 * wi + 16 * a + li][(ks * 32 + 8 * blk) * 2];
#pragma unroll
            for (int c = 0; c < 2; ++c) fj[c] = *(const bf16x8_t*)&Ls[buf][1][32 * wj + 16 * c + li][(ks * 32 + 8 * blk) * 2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c) acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fi[a], fj[c], acc[a][c], 0, 0, 0);
        }
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        if (s + 1 < nsteps) fetch(s + 1);
        if (s < nx) multiply(s & 1, accx);
        else multiply(s & 1, accg);
        if (s + 1 < nsteps) stash((s + 1) & 1);
        __syncthreads();
    }

    // this block's share of sum_{t,t'} (X X^T) o (G G^T)
    float sum = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum = fmaf(accx[a][c][r], accg[a][c][r], sum);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        const float total = ((red[0] + red[1]) + red[2]) + red[3];
        partial[(int64_t)blockIdx.x * B + b] = ti == tj ? total : 2.0f * total;
    }
}

}  // namespace

int64_t gram_norm_partials(int64_t T)
{
    const int64_t nb = (T + GB - 1) / GB;
    return nb * (nb + 1) / 2;
}

bool gram_supports(int64_t B, int64_t T, int64_t din, int64_t dout)
{
    // 16-byte chunks of a row; the examples sit in the second grid dimension
    return din % 8 == 0 && dout % 8 == 0 && B <= 65535 && gram_norm_partials(T) < ((int64_t)1 << 31);
}

hipError_t launch_gram_norms(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, float* partial,
                             hipStream_t stream)
{
    const int nb = (int)((T + GB - 1) / GB);
    const dim3 grid((unsigned)gram_norm_partials(T), (unsigned)B), block(G_THREADS);
    gram_norms_kernel<<<grid, block, 0, stream>>>((const uint16_t*)X, (const uint16_t*)G, (int)T, (int)din, (int)dout, nb, partial, (int)B);
    return hipGetLastError();
}

}  // namespace pex
