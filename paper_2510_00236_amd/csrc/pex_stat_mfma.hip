// pex_stat_mfma.hip -- bf16 MFMA kernel for S = sum_b phi(X_b^T G_b) and the per-token square on gfx950.
//
// The per-example gradient M_b = X_b^T G_b (Sec. 2.3) is a "TN" contraction: both operands are stored with
// the contracted index t as the slow one.  One workgroup of 4 waves owns a BM x BN tile of S for a group of
// examples; a wave owns a WM x WN sub-tile as (WM/32) x (WN/32) MFMA 32x32x16 accumulators.  For each
// example the sequence is walked in slabs of BK tokens:
//     HBM --16-byte coalesced loads--> VGPRs --ds_write_b128--> LDS slab [BK][BM+pad] / [BK][BN+pad]
//     LDS --ds_read_b64_tr_b16 (transposing read: 4 consecutive t for one i)--> MFMA operands
// At the end of an example phi is applied to the fp32 accumulators in registers and added into a second
// register tile; the accumulators restart from zero.  No per-example gradient leaves the register file.
// The slab pipeline runs across example boundaries: while slab s is multiplied, slab s+1 sits in VGPRs on
// its way to the other LDS buffer.
//
// Rows of a slab beyond the end of the example and columns beyond din/dout are zero-filled, which adds
// exact zeros to the sums, so any T and any din, dout that are multiples of 8 (16-byte rows) are taken.
#include "pex_internal.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(8))) short short8_t;
typedef __attribute__((ext_vector_type(16))) float float16_t;

constexpr int NTHREADS = 256;
constexpr int PAD = 32;   // bf16 elements of padding per LDS row: row stride = 64 bytes mod 256, so the four
                          // rows a transposing read touches per 16 lanes fall in four different bank groups

template <int BM_, int BN_, int WM_, int WN_, int BK_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_;
    static constexpr int FM = WM / 32, FN = WN / 32;          // MFMA tiles per wave
    static constexpr int WAVES_N = BN / WN;
    static constexpr int SX = (BM + PAD) * 2, SG = (BN + PAD) * 2;   // LDS row strides in bytes
    static constexpr int STAGE_BYTES = BK * (SX + SG);
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int CX = BM / 8, CG = BN / 8;            // 16-byte chunks per slab row
    static constexpr int NX = BK * CX / NTHREADS, NG = BK * CG / NTHREADS;   // chunks per lane per slab
    static_assert((BM / WM) * (BN / WN) == 4, "four waves per workgroup");
    static_assert(BK * CX % NTHREADS == 0 && BK * CG % NTHREADS == 0, "slab must divide over the lanes");
    static_assert(BK % 16 == 0, "slab depth is a multiple of the MFMA depth");
};

__device__ __forceinline__ uint32_t square_pair_rne(uint32_t packed)
{
    // two bf16 values -> squares in fp32 -> two bf16 (round to nearest even)
    const float lo = __uint_as_float(packed << 16), hi = __uint_as_float(packed & 0xffff0000u);
    const __bf16 l2 = (__bf16)(lo * lo), h2 = (__bf16)(hi * hi);
    return (uint32_t)__builtin_bit_cast(uint16_t, l2) | ((uint32_t)__builtin_bit_cast(uint16_t, h2) << 16);
}

__device__ __forceinline__ uint4 square_chunk(uint4 v)
{
    return make_uint4(square_pair_rne(v.x), square_pair_rne(v.y), square_pair_rne(v.z), square_pair_rne(v.w));
}

template <int MODE>
__device__ __forceinline__ void fold(float16_t& acc2, float16_t& acc)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float m = acc[r];
        if (MODE == MODE_SQUARE) acc2[r] = fmaf(m, m, acc2[r]);
        else acc2[r] += (float)((m > 0.f) - (m < 0.f));
        acc[r] = 0.f;
    }
}

// Workgroup id -> (split, tile_m, tile_n).  Hardware hands consecutive workgroup ids to the 8 XCDs in turn;
// the first step undoes that so that each XCD owns a contiguous range of the tile order, the second walks
// tiles in groups of 4 tile rows so that the ~32 workgroups resident on one XCD form a compact patch and
// share their X and G panels through that XCD's L2.
__device__ __forceinline__ void map_workgroup(int tiles_m, int tiles_n, int& split, int& tm, int& tn)
{
    const int n = gridDim.x, id = blockIdx.x;
    const int xcd = id % 8, local = id / 8;
    const int base = n / 8, rem = n % 8;
    const int nid = xcd * base + (xcd < rem ? xcd : rem) + local;
    const int tiles = tiles_m * tiles_n;
    split = nid / tiles;
    const int q = nid - split * tiles;
    constexpr int GROUP_M = 4;
    const int per_group = GROUP_M * tiles_n;
    const int group = q / per_group;
    const int first_m = group * GROUP_M;
    const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int r = q - group * per_group;
    tm = first_m + r % gm;
    tn = r / gm;
}

template <typename TL, int MODE>
__global__ __launch_bounds__(NTHREADS, 1) void stat_mfma_kernel(const uint16_t* __restrict__ X,
                                                                 const uint16_t* __restrict__ G, int64_t rows_total,
                                                                 int seg_len, int din, int dout,
                                                                 int64_t rows_per_split, int tiles_m, int tiles_n,
                                                                 float* __restrict__ out)
{
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK, FM = TL::FM, FN = TL::FN;
    constexpr int SX = TL::SX, SG = TL::SG, NX = TL::NX, NG = TL::NG, CX = TL::CX, CG = TL::CG;
    constexpr bool PER_EXAMPLE = (MODE == MODE_SQUARE || MODE == MODE_SIGN);
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    int split, tm, tn;
    map_workgroup(tiles_m, tiles_n, split, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;
    const int64_t row_begin = (int64_t)split * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;
    // segment = one example (phi applied at its end) or the whole row range (plain contraction)
    const int slen = PER_EXAMPLE ? seg_len : (int)(row_end - row_begin);
    const int nseg = PER_EXAMPLE ? (int)((row_end - row_begin) / seg_len) : 1;
    const int nst = (slen + BK - 1) / BK;          // slabs per segment
    const int total = nseg * nst;

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / TL::WAVES_N, wn = wave % TL::WAVES_N;

    // ---- loader geometry: chunk c = tid + n*256 -> (row, col) of the slab
    uint4 rx[NX], rg[NG];
    auto gload = [&](int g) {
        const int seg = g / nst, off = (g - seg * nst) * BK;
        const int64_t rbase = row_begin + (int64_t)seg * slen + off;
        const int valid = (slen - off) < BK ? (slen - off) : BK;
#pragma unroll
        for (int n = 0; n < NX; ++n) {
            const int c = tid + n * NTHREADS, row = c / CX, col = (c % CX) * 8;
            const bool ok = row < valid && (i0 + col) < din;
            rx[n] = ok ? *reinterpret_cast<const uint4*>(X + (rbase + row) * din + i0 + col) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int n = 0; n < NG; ++n) {
            const int c = tid + n * NTHREADS, row = c / CG, col = (c % CG) * 8;
            const bool ok = row < valid && (j0 + col) < dout;
            rg[n] = ok ? *reinterpret_cast<const uint4*>(G + (rbase + row) * dout + j0 + col) : make_uint4(0, 0, 0, 0);
        }
    };
    auto lstore = [&](int buf) {
        unsigned char* bx = lds + buf * TL::STAGE_BYTES;
        unsigned char* bg = bx + BK * SX;
#pragma unroll
        for (int n = 0; n < NX; ++n) {
            const int c = tid + n * NTHREADS, row = c / CX, col = (c % CX);
            uint4 v = rx[n];
            if (MODE == MODE_TOKEN_SQ) v = square_chunk(v);
            *reinterpret_cast<uint4*>(bx + row * SX + col * 16) = v;
        }
#pragma unroll
        for (int n = 0; n < NG; ++n) {
            const int c = tid + n * NTHREADS, row = c / CG, col = (c % CG);
            uint4 v = rg[n];
            if (MODE == MODE_TOKEN_SQ) v = square_chunk(v);
            *reinterpret_cast<uint4*>(bg + row * SG + col * 16) = v;
        }
    };

    // ---- fragment geometry for the transposing LDS read.  Within a block of 16 lanes, lane i supplies the
    // address of slab row (i/4), columns 4*(i%4)..+3 and receives column i, rows 0..3.  Blocks 0,1 cover 32
    // columns for k-group 0 (slab rows 0..7 of the 16-deep step), blocks 2,3 the same columns for k-group 1.
    const int blk = lane / 16, li = lane % 16;
    const int frow = 8 * (blk / 2) + li / 4;                 // + 4*h + 16*kstep
    const int fcol = 16 * (blk % 2) + 4 * (li % 4);          // + 32*f + wave offset
    const int a_off = frow * SX + (wm * TL::WM + fcol) * 2;
    const int b_off = frow * SG + (wn * TL::WN + fcol) * 2;
    typedef short4_t __attribute__((address_space(3)))* lds_v4;

    float16_t acc[FM][FN], acc2[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[a][c][r] = 0.f; acc2[a][c][r] = 0.f; }

    if (total > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
        if (total > 1) gload(1);
    }
    int st_in_seg = 0;
    for (int g = 0; g < total; ++g) {
        const int buf = g & 1;
        const unsigned char* bx = lds + buf * TL::STAGE_BYTES;
        const unsigned char* bg = bx + BK * SX;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[FM], bfr[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a) {
                const unsigned char* p = bx + a_off + ks * 16 * SX + a * 64;
                const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
                const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * SX));
                const short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                af[a] = __builtin_bit_cast(bf16x8_t, v);
            }
#pragma unroll
            for (int c = 0; c < FN; ++c) {
                const unsigned char* p = bg + b_off + ks * 16 * SG + c * 64;
                const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
                const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * SG));
                const short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bfr[c] = __builtin_bit_cast(bf16x8_t, v);
            }
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int c = 0; c < FN; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[c], acc[a][c], 0, 0, 0);
        }
        if (PER_EXAMPLE) {
            if (++st_in_seg == nst) {
                st_in_seg = 0;
#pragma unroll
                for (int a = 0; a < FM; ++a)
#pragma unroll
                    for (int c = 0; c < FN; ++c) fold<MODE>(acc2[a][c], acc[a][c]);
            }
        }
        if (g + 1 < total) {
            lstore(buf ^ 1);          // the other buffer was last read one iteration ago, before the barrier below
            __syncthreads();
            if (g + 2 < total) gload(g + 2);
        }
    }

    // ---- epilogue: lane holds column (lane%32), rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 tile
    float* dst = out + (int64_t)split * din * dout;
    const int jn = lane % 32, ib = 4 * (lane / 32);
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            const int j = j0 + wn * TL::WN + c * 32 + jn;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wm * TL::WM + a * 32 + 8 * (r / 4) + ib + (r % 4);
                if (i < din && j < dout) dst[(int64_t)i * dout + j] = PER_EXAMPLE ? acc2[a][c][r] : acc[a][c][r];
            }
        }
}

using Tile0 = Tile<256, 128, 128, 64, 32>;

template <typename TL, int MODE>
hipError_t launch_one(const uint16_t* X, const uint16_t* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                      const StatPlan& plan, float* out, hipStream_t stream)
{
    constexpr bool PER_EXAMPLE = (MODE == MODE_SQUARE || MODE == MODE_SIGN);
    const int tiles_m = (int)((din + TL::BM - 1) / TL::BM), tiles_n = (int)((dout + TL::BN - 1) / TL::BN);
    const int64_t rows_per_split = PER_EXAMPLE ? plan.per_split * T : plan.per_split;
    auto kern = stat_mfma_kernel<TL, MODE>;
    static bool attr_set = false;     // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n * plan.nsplit)), block(NTHREADS);
    kern<<<grid, block, TL::LDS_BYTES, stream>>>(X, G, B * T, (int)T, (int)din, (int)dout, rows_per_split, tiles_m,
                                                 tiles_n, out);
    return hipGetLastError();
}

template <typename TL>
hipError_t launch_mode(const uint16_t* X, const uint16_t* G, int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode,
                       const StatPlan& plan, float* out, hipStream_t stream)
{
    switch (mode) {
    case MODE_IDENTITY: return launch_one<TL, MODE_IDENTITY>(X, G, B, T, din, dout, plan, out, stream);
    case MODE_SQUARE: return launch_one<TL, MODE_SQUARE>(X, G, B, T, din, dout, plan, out, stream);
    case MODE_SIGN: return launch_one<TL, MODE_SIGN>(X, G, B, T, din, dout, plan, out, stream);
    case MODE_TOKEN_SQ: return launch_one<TL, MODE_TOKEN_SQ>(X, G, B, T, din, dout, plan, out, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

void mfma_tile_shape(int variant, Mode, int* bm, int* bn)
{
    (void)variant;
    *bm = Tile0::BM;
    *bn = Tile0::BN;
}

bool mfma_bf16_supports(int64_t B, int64_t T, int64_t din, int64_t dout, Mode, int)
{
    // 16-byte rows; 32-bit tile arithmetic; tiny problems are latency-bound and stay on the SIMT kernel
    if (din % 8 != 0 || dout % 8 != 0) return false;
    if (din < 32 || dout < 32) return false;
    if (B * T < 16) return false;
    const int64_t tiles = ((din + Tile0::BM - 1) / Tile0::BM) * ((dout + Tile0::BN - 1) / Tile0::BN);
    return tiles * 16 < ((int64_t)1 << 31);
}

hipError_t launch_stat_mfma_bf16(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                 Mode mode, const StatPlan& plan, float* out, hipStream_t stream)
{
    return launch_mode<Tile0>((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, mode, plan, out, stream);
}

}  // namespace pex
