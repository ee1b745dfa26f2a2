// pex_gram.hip -- per-example squared gradient norms through the T x T Gram matrices (gfx950, bf16 inputs).
//
// Sec. 2.3 remarks that the squared norm of a per-example gradient of a dense sequence layer needs no gradient at
// all ("ghost" norm):
//     N_b = || X_b^T G_b ||_F^2 = sum_{t,t'} (X_b X_b^T)[t,t'] * (G_b G_b^T)[t,t'],
// 2 T^2 (din + dout) FLOP per example against 2 T din dout for the contraction itself -- cheaper when
// T < din*dout/(din+dout), and, what matters more on layers with few tiles, with no partial sums of S to exchange:
// a workgroup produces one number.
//
// One workgroup (4 waves, one per SIMD) owns a 128 x 128 block (ti, tj), ti <= tj, of the two Gram matrices of one
// example; each wave a 64 x 64 quarter as 4 x 4 accumulators of v_mfma_f32_16x16x32_bf16, once for X X^T and once
// for G G^T (128 registers).  The contraction runs over the features, which are contiguous in memory: an operand
// fragment is 16 rows x 32 features with 16 bytes per lane, a plain ds_read_b128.  Steps of 64 features (the rows of
// block row ti and of block row tj: two panels of 128 rows x 128 bytes) arrive by direct-to-LDS loads in a ring of four
// buffers, three steps ahead of the MFMAs, one barrier per step; the steps over din and over dout form one pipeline.
// A wave's load covers 8 rows x 128 bytes; the 16-byte chunks of a row are stored at position chunk ^ (row mod 8), so
// that the 8 lanes a fragment read serves per cycle (8 rows, one chunk) fall into 8 different groups of four banks.
// Rows beyond T lie outside the buffer descriptor and arrive as zeros; features beyond the row are masked per lane
// in the last step.  A block on the diagonal loads its panel once.  At the end the block contributes sum(A o B), twice
// if it is off the diagonal (both matrices are symmetric), added over the workgroup in a fixed order.
#include <mutex>

#include "pex_internal.h"
#include "pex_lds_dma.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef bf16x8_t __attribute__((address_space(3)))* lds_frag;

constexpr int GB = 128;                       // block edge, tokens
constexpr int GK = 64;                        // features per step
constexpr int ROW = GK * 2;                   // bytes of a panel row in LDS
constexpr int PANEL = GB * ROW;               // 16 KiB
constexpr int STAGE = 2 * PANEL;              // both panels of a step
constexpr int NS = 4;                         // ring
constexpr int G_THREADS = 256, G_WAVES = 4;
constexpr int LPP = PANEL / 1024 / G_WAVES;   // loads per wave, panel and step (4)
constexpr int GRAM_LDS = NS * STAGE;          // 128 KiB

// DIAG: ti == tj, one panel per step.
template <bool DIAG>
__device__ __forceinline__ float gram_block(const uint16_t* __restrict__ xb, const uint16_t* __restrict__ gb, int T, int din, int dout,
                                            int ti, int tj, unsigned char* lds)
{
    constexpr int LPS = DIAG ? LPP : 2 * LPP;             // loads per wave and step
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wj = wave & 1;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void)lds;

    const int nx = (din + GK - 1) / GK, ng = (dout + GK - 1) / GK, nsteps = nx + ng;

    // loader: load q = wave*LPP + n of a panel covers its rows 8q .. 8q+7; lane L fills slot L%8 of row 8q + L/8 with
    // the row's chunk (L%8) ^ (L/8).  Offsets are relative to the example's first element and the step's first feature.
    const int lrow = lane >> 3, lchunk = (lane & 7) ^ lrow;
    uint32_t off_x[2][LPP], off_g[2][LPP];
#pragma unroll
    for (int pn = 0; pn < 2; ++pn)
#pragma unroll
        for (int n = 0; n < LPP; ++n) {
            const int64_t row = (int64_t)(pn == 0 ? ti : tj) * GB + (wave * LPP + n) * 8 + lrow;
            // rows at or beyond T must fall outside the descriptor whatever 32-bit arithmetic does: clamp them there
            const int64_t r = row < T ? row : T;
            off_x[pn][n] = (uint32_t)((r * din + lchunk * 8) * 2);
            off_g[pn][n] = (uint32_t)((r * dout + lchunk * 8) * 2);
        }
    // The loads of one step: prepare_step() fixes the descriptor and the ring buffer, issue_load(k) sends load k of LPS.
    int iss = 0;                                           // next step to load
    int4_t rs;
    bool cut = false, in_x = true;
    uint32_t buf_addr = 0;
    auto prepare_step = [&]() {
        const bool past = iss >= nsteps;
        in_x = iss < nx;
        const int d = in_x ? din : dout, k0 = (in_x ? iss : iss - nx) * GK;
        const uint16_t* src = (in_x ? xb : gb) + k0;
        // the descriptor ends with row T-1; its base moves with the step, so a lane's offset does not
        rs = make_rsrc(src, past ? 0u : (uint32_t)(((int64_t)T * d - k0) * 2));
        cut = lchunk * 8 >= d - k0;                        // this lane's chunk lies beyond the end of the row
        buf_addr = lds_base + (uint32_t)((iss % NS) * STAGE);
        ++iss;
    };
    auto issue_load = [&](int k) {
        const int pn = k / LPP, n = k % LPP;
        const uint32_t off = in_x ? off_x[pn][n] : off_g[pn][n];
        dma_load_16(buf_addr + (uint32_t)(pn * PANEL + (wave * LPP + n) * 1024), cut ? 0x80000000u : off, rs);
    };

    float4_t accx[4][4], accg[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            accx[a][c] = float4_t{0.f, 0.f, 0.f, 0.f};
            accg[a][c] = float4_t{0.f, 0.f, 0.f, 0.f};
        }
    // fragment (16 rows x 32 features): lane (blk, li) = (lane/16, lane%16) reads row li, chunk 4*ks + blk, which sits
    // at position chunk ^ (row mod 8)
    const int li = lane & 15, blk = lane >> 4;
    int a_addr[2], b_addr[2];                              // per 32-feature half of the step; fragment row adds 16 rows
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int pos = ((4 * ks + blk) ^ (li & 7)) * 16;
        a_addr[ks] = (wi * 64 + li) * ROW + pos;
        b_addr[ks] = (DIAG ? 0 : PANEL) + (wj * 64 + li) * ROW + pos;
    }
    // One step: all 16 fragment reads first, then the 32 MFMAs with the loads of step s+NS-1 spread between them (one
    // wave per SIMD: whatever is issued between two MFMAs costs MFMA time, but less than in front of the reads, where the
    // wave would wait for the LDS afterwards anyway).  The fences pin that order.
    auto step = [&](int s, float4_t (&acc)[4][4]) {
        wait_vmcnt<(NS - 2) * LPS>();                      // this wave's part of step s has landed
        wait_lds_and_barrier();                            // everyone's has, and everyone is done reading step s-1
        const unsigned char* buf = lds + (s % NS) * STAGE;
        bf16x8_t fi[2][4], fj[2][4];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int a = 0; a < 4; ++a) fi[ks][a] = *(lds_frag)(buf + a_addr[ks] + a * 16 * ROW);
#pragma unroll
            for (int c = 0; c < 4; ++c) fj[ks][c] = *(lds_frag)(buf + b_addr[ks] + c * 16 * ROW);
        }
        prepare_step();                                    // step s+NS-1, into the buffer step s-1 was read from
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fi[ks][a], fj[ks][c], acc[a][c], 0, 0, 0);
                    const int i = (ks * 4 + a) * 4 + c;    // every (32 / LPS)-th MFMA is followed by a load
                    if ((i + 1) % (32 / LPS) == 0) {
                        __builtin_amdgcn_sched_barrier(0);
                        issue_load(i / (32 / LPS));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
        prepare_step();
#pragma unroll
        for (int k = 0; k < LPS; ++k) issue_load(k);
    }
    // one loop per matrix, so that each set of accumulators stays where it is while the other is worked on
    for (int s = 0; s < nx; ++s) step(s, accx);
    for (int s = nx; s < nsteps; ++s) step(s, accg);
    wait_vmcnt<0>();                                       // the (empty) loads issued past the end

    // this wave's share of sum_{t,t'} (X X^T) o (G G^T) over the block
    float sum = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum = fmaf(accx[a][c][r], accg[a][c][r], sum);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    return sum;
}

// (register budget of two waves per SIMD: with all 512 registers of a lone wave the compiler spreads the accumulators over both
// halves of the file and moves them around inside the loop)
__global__ __launch_bounds__(G_THREADS, 2) void gram_norms_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ G, int T,
                                                                   int din, int dout, int nb, float* __restrict__ partial, int B)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    __shared__ float red[G_WAVES];
    const int b = blockIdx.y;
    // pair number -> (ti, tj) with ti <= tj, rows of the upper triangle one after the other
    int ti = 0, rem = blockIdx.x;
    while (rem >= nb - ti) { rem -= nb - ti; ++ti; }
    const int tj = ti + rem;
    const uint16_t* xb = X + (int64_t)b * T * din;
    const uint16_t* gb = G + (int64_t)b * T * dout;
    const float sum = ti == tj ? gram_block<true>(xb, gb, T, din, dout, ti, tj, lds) : gram_block<false>(xb, gb, T, din, dout, ti, tj, lds);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
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
    // 16-byte chunks of a row; the examples sit in the second grid dimension; byte offsets inside an example are 32 bits
    const int64_t lim = (int64_t)1 << 31;
    return din % 8 == 0 && dout % 8 == 0 && B <= 65535 && gram_norm_partials(T) < lim && (T + 1) * din * 2 < lim && (T + 1) * dout * 2 < lim;
}

hipError_t launch_gram_norms(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, float* partial,
                             hipStream_t stream)
{
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] {
        attr_err = hipFuncSetAttribute((const void*)gram_norms_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, GRAM_LDS);
    });
    if (attr_err != hipSuccess) return attr_err;
    const int nb = (int)((T + GB - 1) / GB);
    const dim3 grid((unsigned)gram_norm_partials(T), (unsigned)B), block(G_THREADS);
    gram_norms_kernel<<<grid, block, GRAM_LDS, stream>>>((const uint16_t*)X, (const uint16_t*)G, (int)T, (int)din, (int)dout, nb, partial,
                                                         (int)B);
    return hipGetLastError();
}

}  // namespace pex
