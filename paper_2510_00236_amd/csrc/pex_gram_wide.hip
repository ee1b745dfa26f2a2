// pex_gram_wide.hip -- per-example squared gradient norms through the Gram matrices on 256 x 256 blocks (gfx950, bf16).
//
// Same quantity and the same pipeline as pex_gram.hip (N_b = sum_{t,t'} (X_b X_b^T)[t,t'] (G_b G_b^T)[t,t'], Sec. 2.3),
// on blocks of four times the area: a block of 256 x 256 draws half the bytes per FLOP from L2 that a 128 x 128 block
// does, which is what bounds that kernel.  Eight waves, 128 x 64 per wave = 8 x 4 accumulators of
// v_mfma_f32_16x16x32_bf16 = 128 registers -- for ONE matrix.  Both Gram blocks must be complete before their product,
// so the block of X_b X_b^T waits in memory: after the steps over din every wave parks its accumulators in the
// workspace (256 KiB per workgroup, lane-contiguous 16-byte stores), runs the steps over dout into the same registers
// and reads the parked block back for sum(A o B).  The parked bytes are a few per cent of what the panels bring in.
//
// Steps of 32 features (rows of 64 bytes; two panels of 256 rows = 32 KiB, one on the diagonal) in a ring of four
// buffers, three steps ahead.  A wave's load covers 16 rows x 64 bytes; chunk c of row r is stored at position
// c ^ ((r / 4) mod 4), so that the 8 lanes a fragment read serves per cycle (8 rows, one chunk) fall into 8 different
// groups of four banks.  Blocks (I, J), I <= J, of the upper triangle; a diagonal block is computed whole (both
// triangles of it), an off-diagonal one counts twice.  Rows beyond T lie outside the buffer descriptor and arrive as zeros.
#include <mutex>

#include "pex_internal.h"
#include "pex_lds_dma.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef bf16x8_t __attribute__((address_space(3)))* lds_frag;

constexpr int SB = 256;                       // block edge, tokens
constexpr int SK = 32;                        // features per step
constexpr int ROW = SK * 2;                   // bytes of a panel row in LDS
constexpr int PANEL = SB * ROW;               // 16 KiB
constexpr int STAGE = 2 * PANEL;
constexpr int NS = 4;
constexpr int W_THREADS = 512, W_WAVES = 8;
constexpr int LPP = PANEL / 1024 / W_WAVES;   // loads per wave, panel and step (2)
constexpr int WIDE_LDS = NS * STAGE;          // 128 KiB
constexpr int FM = 8, FN = 4;                 // 16 x 16 accumulators per wave: 128 x 64
constexpr int PARK_FLOATS = W_THREADS * FM * FN * 4;   // per workgroup: 65536 floats

template <bool DIAG>
__device__ __forceinline__ float gram_wide_block(const uint16_t* __restrict__ xb, const uint16_t* __restrict__ gb, int T, int din, int dout,
                                                 int bi, int bj, unsigned char* lds, float4_t* __restrict__ park)
{
    constexpr int LPS = DIAG ? LPP : 2 * LPP;             // loads per wave and step
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void)lds;
    const int nx = (din + SK - 1) / SK, ng = (dout + SK - 1) / SK, nsteps = nx + ng;

    // loader: load q = wave*LPP + n of a panel covers its rows 16q .. 16q+15; lane L fills slot L%4 of row 16q + L/4
    // with the row's chunk (L%4) ^ ((L/16) mod 4).  Offsets are relative to the example's first element and the step's
    // first feature.
    const int lrow = lane >> 2, lchunk = (lane & 3) ^ (lane >> 4);
    uint32_t off_x[2][LPP], off_g[2][LPP];
#pragma unroll
    for (int pn = 0; pn < 2; ++pn)
#pragma unroll
        for (int n = 0; n < LPP; ++n) {
            const int64_t row = (int64_t)(pn == 0 ? bi : bj) * SB + (wave * LPP + n) * 16 + lrow;
            const int64_t r = row < T ? row : T;          // rows at or beyond T: outside the descriptor for certain
            off_x[pn][n] = (uint32_t)((r * din + lchunk * 8) * 2);
            off_g[pn][n] = (uint32_t)((r * dout + lchunk * 8) * 2);
        }
    int iss = 0;
    int4_t rs;
    bool cut = false, in_x = true;
    uint32_t buf_addr = 0;
    auto prepare_step = [&]() {
        const bool past = iss >= nsteps;
        in_x = iss < nx;
        const int d = in_x ? din : dout, k0 = (in_x ? iss : iss - nx) * SK;
        const uint16_t* src = (in_x ? xb : gb) + k0;
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

    float4_t acc[FM][FN];
    auto clear = [&]() {
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int c = 0; c < FN; ++c) acc[a][c] = float4_t{0.f, 0.f, 0.f, 0.f};
    };
    clear();
    // fragment (16 rows x 32 features): lane (blk, li) = (lane/16, lane%16) reads row li, chunk blk, which sits at
    // position blk ^ ((row / 4) mod 4); the fragments of a wave are 16 rows = 1 KiB apart
    const int li = lane & 15, blk = lane >> 4;
    const int pos = (blk ^ ((li >> 2) & 3)) * 16;
    const int a_addr = (wm * 128 + li) * ROW + pos;
    const int b_addr = (DIAG ? 0 : PANEL) + (wn * 64 + li) * ROW + pos;

    // One step: eight fragment reads first, then the 32 MFMAs with the other four reads and the loads of step s+NS-1
    // spread between them.
    auto step = [&](int s) {
        wait_vmcnt<(NS - 2) * LPS>();                      // this wave's part of step s has landed
        wait_lds_and_barrier();                            // everyone's has, and everyone is done reading step s-1
        const unsigned char* buf = lds + (s % NS) * STAGE;
        bf16x8_t fi[FM], fj[FN];
#pragma unroll
        for (int c = 0; c < FN; ++c) fj[c] = *(lds_frag)(buf + b_addr + c * 16 * ROW);
#pragma unroll
        for (int a = 0; a < FM / 2; ++a) fi[a] = *(lds_frag)(buf + a_addr + a * 16 * ROW);
        prepare_step();                                    // step s+NS-1, into the buffer step s-1 was read from
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int c = 0; c < FN; ++c) {
                acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fi[a], fj[c], acc[a][c], 0, 0, 0);
                const int i = a * FN + c;
                // the second half of the row fragments is read behind the first MFMAs, one fragment after every other MFMA
                if (i % 2 == 1 && i / 2 < FM / 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    fi[FM / 2 + i / 2] = *(lds_frag)(buf + a_addr + (FM / 2 + i / 2) * 16 * ROW);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if ((i + 1) % (32 / LPS) == 0) {           // every (32 / LPS)-th MFMA is followed by a load
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
    for (int s = 0; s < nx; ++s) step(s);
    // X_b X_b^T of this block is complete: it waits in memory while the same registers take G_b G_b^T.  (These stores
    // count in vmcnt like the loads, so the next few waits are longer than they need be; they are never too short,
    // because loads return in order among themselves.)
    float4_t* mine = park + (int64_t)wave * (FM * FN * 64) + lane;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) mine[(a * FN + c) * 64] = acc[a][c];
    clear();
    for (int s = nx; s < nsteps; ++s) step(s);
    wait_vmcnt<0>();                                       // the (empty) loads issued past the end, and the parked block

    float sum = 0.f;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            const float4_t ax = mine[(a * FN + c) * 64];
#pragma unroll
            for (int r = 0; r < 4; ++r) sum = fmaf(ax[r], acc[a][c][r], sum);
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    return sum;
}

__global__ __launch_bounds__(W_THREADS, 1) void gram_wide_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ G, int T,
                                                                  int din, int dout, int nb, float* __restrict__ partial,
                                                                  float4_t* __restrict__ park, int B)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    __shared__ float red[W_WAVES];
    const int b = blockIdx.y;
    int bi = 0, rem = blockIdx.x;                          // pair number -> (bi, bj), bi <= bj
    while (rem >= nb - bi) { rem -= nb - bi; ++bi; }
    const int bj = bi + rem;
    const uint16_t* xb = X + (int64_t)b * T * din;
    const uint16_t* gb = G + (int64_t)b * T * dout;
    float4_t* my_park = park + ((int64_t)b * gridDim.x + blockIdx.x) * (PARK_FLOATS / 4);
    const float sum = bi == bj ? gram_wide_block<true>(xb, gb, T, din, dout, bi, bj, lds, my_park)
                               : gram_wide_block<false>(xb, gb, T, din, dout, bi, bj, lds, my_park);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = red[0];
#pragma unroll
        for (int w = 1; w < W_WAVES; ++w) total += red[w];
        partial[(int64_t)blockIdx.x * B + b] = bi == bj ? total : 2.0f * total;
    }
}

}  // namespace

int64_t gram_wide_partials(int64_t T)
{
    const int64_t nb = (T + SB - 1) / SB;
    return nb * (nb + 1) / 2;
}

// bytes of the parked blocks: one per workgroup
size_t gram_wide_park_bytes(int64_t B, int64_t T) { return (size_t)B * (size_t)gram_wide_partials(T) * PARK_FLOATS * sizeof(float); }

hipError_t launch_gram_wide(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, float* partial, void* park,
                            hipStream_t stream)
{
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] {
        attr_err = hipFuncSetAttribute((const void*)gram_wide_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, WIDE_LDS);
    });
    if (attr_err != hipSuccess) return attr_err;
    const int nb = (int)((T + SB - 1) / SB);
    const dim3 grid((unsigned)gram_wide_partials(T), (unsigned)B), block(W_THREADS);
    gram_wide_kernel<<<grid, block, WIDE_LDS, stream>>>((const uint16_t*)X, (const uint16_t*)G, (int)T, (int)din, (int)dout, nb, partial,
                                                        (float4_t*)park, (int)B);
    return hipGetLastError();
}

}  // namespace pex
