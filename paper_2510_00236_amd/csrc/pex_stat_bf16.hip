// pex_stat_bf16.hip -- bf16 MFMA kernel for S = sum_b phi(X_b^T G_b) and for the per-token square (gfx950).
//
// Mathematics (Sec. 2.3, dense layers in sequence models): contract over the sequence, M_b = X_b^T G_b, apply phi
// to the complete per-example tile while it is still in registers, sum over the batch.  The per-example gradient
// never leaves the register file.  The per-token square (X o X)^T (G o G) is one plain contraction over all
// B*T rows whose operands are squared on the way.
//
// Data path
//   * One workgroup = 8 waves (two per SIMD) owns a BM x BN tile of S; a wave owns WM x WN of it as FM x FN
//     accumulators of v_mfma_f32_16x16x32_bf16.  (Same FLOP per cycle as the 32x32x16 form and the same LDS reads per
//     FLOP, but half the accumulator traffic; on this power-limited chip an MFMA-only loop sustains 2.02 PFLOP/s
//     with it against 1.80 with 32x32x16 on Gaussian operands, and the contraction gained 7 %.)  phi = identity, sign
//     and the per-token square use 256 x 256 tiles (128 x 64 per wave); phi = square needs a second fp32 register tile for the running sum and uses 256 x 128 (64 x 64 per
//     wave); sign counts are integers of magnitude <= B and are kept as packed fp16 pairs while B <= 2048, which
//     is what lets sign use the large tile.
//   * Slabs of BK tokens go HBM -> LDS with buffer_load_dwordx4 ... lds: no VGPR staging, no LDS write
//     instructions.  Out-of-range lanes of a buffer load write zeros, which gives the zero fill of ragged slab
//     rows (num_records of a per-slab descriptor) and of ragged tile columns (a poisoned lane offset) for free.
//     (The per-token square is the exception: its operands have to be squared on the way, so its slabs go through
//     registers -- same descriptors, same offsets, same places in the ring.)
//   * Each such instruction writes 1 KiB contiguous, so slab rows cannot be padded; instead the 16-byte chunks of
//     slab row r are stored at chunk index c ^ 4*(r mod 4).  The transposing read ds_read_b64_tr_b16 of a 16-lane
//     group touches 4 consecutive rows x 32 bytes; the swizzle puts those in 4 different 64-byte bank groups.  The
//     lane group served in the same cycle reads the same columns 8 rows further down, i.e. the same banks: a two-way
//     conflict per read (SQ_LDS_BANK_CONFLICT = 2 x reads) that costs 1.4 % of the cycles.  Moving those rows by 32
//     bytes (chunk index ^ 2 on bit 3 of the row) removes the conflicts but makes lanes fetch the halves of a
//     64-byte segment out of order, which doubled the L2 misses and cost 4.5 % of the time; shifting every group of 8
//     rows by 32 bytes at the destination of the loads instead removes them too and changes no timing (the reads
//     have slack in their phase).  Neither is done.
//   * NS slabs form a ring in LDS.
//
// Schedule: two groups of four waves (one wave of each group per SIMD) run half a slab apart, so that whenever
// one wave of a SIMD sits at a barrier, waits for LDS data or folds phi, the other one is in the middle of its
// MFMAs.  A wave alternates between
//   read phase     : most operand fragments of slab g come from LDS into registers (all of G, the first of X),
//                    then this wave's global->LDS loads of a later slab are issued;
//   multiply phase : all MFMAs of slab g at raised priority, the reads of the remaining X fragments (which the
//                    last MFMAs use) slotted in between the first of them,
// and every phase ends at a workgroup barrier where the groups swap roles:
//   phase 2g   : group 0 reads slab g       | group 1 multiplies slab g-1
//   phase 2g+1 : group 0 multiplies slab g  | group 1 reads slab g
// Measured facts behind this shape (MI355X): a wave gets one LDS instruction through per ~16 cycles whatever its
// width, and the transposing read is 8 bytes per lane, so the 2*(FM+FN) = 24 reads of a 32-token slab cost three
// quarters of the issue time of its 32 MFMAs: with the global->LDS loads on top, all reads of a slab in one phase
// would make that phase longer than the multiply phase it hides behind.  The memory pipeline takes one 1 KiB direct-to-LDS load per ~40-60 cycles per compute unit
// when the whole chip is loading; a wave that stalls on that in its read phase delays nothing, in the multiply
// phase it would starve the MFMA pipe.  Priority is raised only while a wave issues MFMAs: a wave that waits at
// a barrier with raised priority slows the other wave of its SIMD.
// Buffer life: slab g is read during phases 2g .. 2g+2.  In its read phase of slab h, group 1 (phase 2h+1)
// refills the buffer of slab h-1 with slab h+NS-1; group 0 (phase 2h, when group 1 may still read slab h-1)
// refills the buffer of slab h-2 with slab h+NS-2, i.e. its loads run one slab behind.  Every wave makes sure its
// part of slab g+1 has landed before the barrier that ends phase 2g+1.  Steady state is branch-free: loads past
// the end of the range carry an empty descriptor and write zeros into a buffer nobody reads.
//
// Plain contractions (phi = identity, the pre-squared per-token square, split partial sums) over long ranges run on a
// second kernel, stat_bf16_quad_kernel: four waves, one per SIMD, each with a 128 x 128 register tile (256 accumulator
// registers, which only a wave that has its SIMD's register file to itself can hold).  A wave then reads 16 fragments
// per 64 MFMAs instead of 12 per 32: a third less LDS traffic per FLOP.  With realistic operand values the chip is
// bound by power, not by issue slots (all-zero inputs run 30 % faster on either kernel), and the lower energy per FLOP
// is worth 5-8 % although nothing hides a wave's own LDS, load and scalar instructions: with one wave per SIMD every
// instruction that is not an MFMA costs about four cycles of MFMA time (measured: 1024 + 4 x 60 cycles per slab), so
// that kernel is written to issue as few of them as possible (see there).
#include <cstdlib>
#include <mutex>
#include <type_traits>
#include <utility>

#include "pex_internal.h"
#include "pex_lds_dma.h"

namespace pex {
namespace {

// What one launch produces (bit set).  A launch with only OUT_ID or only OUT_TOKEN is a plain contraction over
// all rows (the accumulators are the result); every other set applies phi per example: the accumulators hold
// M_b and are folded into one register tile per requested statistic at the end of each example.
// OUT_SIGN_PK keeps the sign counts as packed fp16 pairs (exact up to 2048 examples), OUT_SIGN_F32 as fp32,
// OUT_SIGN_U8 as four biased byte counters per register: each example adds sign+1 in {0,1,2}, so a byte never
// borrows from its neighbour and holds up to 127 examples; the count is byte - examples.  A quarter of the
// registers of an fp32 tile, which is what lets identity, square and sign share one contraction.
// OUT_NORM writes ||M_b||_F^2 of every example (one partial per tile and wave, summed by a second kernel);
// OUT_IDW is the identity statistic with one weight per example, sum_b w_b M_b (what clipping needs).
// OUT_POW is phi(m) = |m|^alpha through the hardware log2 / exp2 (relative error of a term about 1e-6 * alpha * |log2 m|).
// OUT_MEM (with exactly one of OUT_SQ, OUT_IDW, OUT_POW): that statistic has no register tile; at the end of an example
// phi(M_b) is added to the output in memory (the first example of the range stores).  Every entry belongs to one lane
// of one workgroup, which adds its examples in ascending order: the result is the same sequential fp32 sum as in
// registers, and as reproducible.
constexpr int OUT_ID = 1, OUT_SQ = 2, OUT_SIGN_PK = 4, OUT_SIGN_F32 = 8, OUT_TOKEN = 16, OUT_SIGN_U8 = 32, OUT_NORM = 64,
              OUT_IDW = 128, OUT_POW = 256, OUT_MEM = 512;
constexpr int MAX_U8_EXAMPLES = 127;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int uint4_t;
typedef __attribute__((ext_vector_type(2))) _Float16 half2_t;
typedef short4_t __attribute__((address_space(3)))* lds_v4;
typedef uint4_t __attribute__((address_space(3)))* lds_u4;

// One dword per lane to (descriptor base + voff + soff): plain store, or fp32 add performed by the L2 (no value
// returned).  Lanes whose offset is outside the descriptor's range do nothing.  Both count in vmcnt like the loads.
// The sum of the offsets is formed inside the statement (the range check does not see the instruction's own scalar
// offset), so that the compiler cannot keep one precomputed address per accumulator register alive across the main loop.
__device__ __forceinline__ void mem_store_f32(float v, uint32_t voff, uint32_t soff, int4_t rsrc)
{
    uint32_t at;
    asm volatile("v_add_u32 %0, %2, %3\n\tbuffer_store_dword %1, %0, %4, 0 offen" : "=&v"(at) : "v"(v), "v"(voff), "s"(soff), "s"(rsrc) : "memory");
}
__device__ __forceinline__ void mem_add_f32(float v, uint32_t voff, uint32_t soff, int4_t rsrc)
{
    uint32_t at;
    asm volatile("v_add_u32 %0, %2, %3\n\tbuffer_atomic_add_f32 %1, %0, %4, 0 offen" : "=&v"(at) : "v"(v), "v"(voff), "s"(soff), "s"(rsrc) : "memory");
}

// two bf16 values -> squares in fp32 -> two bf16 (round to nearest even, one packed conversion); zero stays zero
__device__ __forceinline__ uint32_t square_pair_rne(uint32_t packed)
{
    typedef __attribute__((ext_vector_type(2))) float float2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const float lo = __uint_as_float(packed << 16), hi = __uint_as_float(packed & 0xffff0000u);
    const float2_t sq = {lo * lo, hi * hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(sq, bf16x2_t));
}

// sign(m) in {-1, 0, +1} as a float without compares: scaling by 2^200 sends every non-zero value (denormals
// included) beyond +-1 and keeps +-0 at 0, the median with -1 and +1 clamps it.
__device__ __forceinline__ float sign_as_float(float m)
{
    return __builtin_amdgcn_fmed3f(__builtin_ldexpf(m, 200), -1.0f, 1.0f);
}

// |m|^alpha = 2^(alpha * log2 |m|), alpha > 0; zero stays zero (log2 0 = -inf, 2^-inf = 0)
__device__ __forceinline__ float abs_power(float m, float alpha)
{
    return __builtin_amdgcn_exp2f(alpha * __builtin_amdgcn_logf(__builtin_fabsf(m)));
}

// End of an example, one finished 16x16 tile of M_b (four registers per lane): every requested statistic takes its
// phi(M_b), M_b restarts from 0.  Sign counts of a tile as 2 fp16 pairs per lane: integers up to 2048 are exact in
// fp16, so the count of at most 2048 examples is exact, at half the registers of an fp32 tile; or as one register of
// four biased byte counters.
template <int OUTS>
__device__ __forceinline__ void fold_tile(float4_t& acc, float4_t& acc_id, float4_t& acc_sq, float4_t& acc_sg, half2_t (&cnt)[2],
                                          uint32_t& cnt8, float weight, float& norm)
{
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float m = acc[r];
        if (OUTS & OUT_ID) acc_id[r] += m;
        if (OUTS & OUT_IDW) acc_id[r] = fmaf(weight, m, acc_id[r]);
        if (OUTS & OUT_NORM) norm = fmaf(m, m, norm);
        if (OUTS & OUT_SQ) acc_sq[r] = fmaf(m, m, acc_sq[r]);
        if (OUTS & OUT_POW) acc_sq[r] += abs_power(m, weight);        // the exponent travels in the weight slot
        if (OUTS & OUT_SIGN_F32) acc_sg[r] += sign_as_float(m);
    }
    if (OUTS & OUT_SIGN_PK) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
            cnt[r] += __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(sign_as_float(acc[2 * r]), sign_as_float(acc[2 * r + 1])));
    }
    if (OUTS & OUT_SIGN_U8) {
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) w = __builtin_amdgcn_cvt_pk_u8_f32(sign_as_float(acc[k]) + 1.0f, k, w);
        cnt8 += w;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = 0.f;
}

// Workgroup id -> (split, tile_m, tile_n): undo the round-robin assignment of consecutive ids to the 8 XCDs,
// then walk tiles in groups of GROUP_M tile rows so the workgroups resident on one XCD form a compact patch
// that shares X and G panels in that XCD's L2.
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

// Tile geometry.  RC_ = fragments of a slab's last k-step that are read in the multiply phase (the rest of the
// slab's fragments are read in the read phase).  LEAD_ = 0: the multiply phase walks the wave's sub-tile row by row
// (X fragment outer, G fragments inner), the late fragments are the last X fragments and late read i follows MFMA i.
// LEAD_ > 0: column by column (G fragment outer), the late fragments are the last G fragments, each read LEAD_
// MFMAs before the first MFMA that uses it -- for sub-tiles with more fragment columns than rows, where more
// fragments can be late.
template <int BM_, int BN_, int WM_, int WN_, int BK_, int NS_, int RC_, int LEAD_ = 0>
struct Bf16Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_, NS = NS_;
    static constexpr int FM = WM / 16, FN = WN / 16, KS = BK / 32;
    static constexpr int FPK = FM + FN;                                // fragments per k-step
    static constexpr int RC = RC_ < FPK ? RC_ : FPK;
    static constexpr int LEAD = LEAD_;
    static constexpr bool N_OUTER = LEAD_ > 0;
    // which late fragment (0 .. RC-1) is read after MFMA i of a slab, -1: none
    static constexpr int late_read_after(int i)
    {
        if (!N_OUTER) return i < RC ? i : -1;
        for (int k = 0; k < RC; ++k) {
            const int use = (KS - 1) * FM * FN + (FN - RC + k) * FM;      // first MFMA that needs late fragment k
            int at = use - LEAD;
            if (at < k) at = k;
            if (at == i) return k;
        }
        return -1;
    }
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN, NWAVES = WAVES_M * WAVES_N, NT = NWAVES * 64;
    static constexpr int XROW = BM * 2, GROW = BN * 2;                 // bytes per slab row
    static constexpr int X_BYTES = BK * XROW, G_BYTES = BK * GROW, STAGE = X_BYTES + G_BYTES;
    static constexpr int LDS_BYTES = NS * STAGE;
    // Loads per wave per slab.  The G part of a slab need not divide evenly over eight waves (a 192-column tile has
    // 12 KiB per slab): the waves of group 1 take NGI1 loads each, those of group 0 the rest (NGI0 >= NGI1 each).
    static constexpr int NXI = X_BYTES / 1024 / NWAVES, G_LOADS = G_BYTES / 1024;
    static constexpr int NGI1 = G_LOADS / NWAVES, NGI0 = (G_LOADS - 4 * NGI1) / 4;
    static constexpr int LPS0 = NXI + NGI0, LPS1 = NXI + NGI1;         // per wave of group 0 / group 1
    static constexpr int RX = 1024 / XROW;                             // slab rows covered by one load of X
    static constexpr int XCH = XROW / 16, GCH = GROW / 16;             // 16-byte chunks per slab row
    static_assert(NWAVES == 8, "eight waves per workgroup: two groups of four");
    static_assert(X_BYTES % (1024 * NWAVES) == 0 && G_BYTES % 4096 == 0 && 4 * (NGI0 + NGI1) == G_LOADS, "slab must divide over the waves");
    static_assert(BK % 32 == 0 && XROW <= 1024 && GROW <= 1024, "tile limits");
    static_assert((XROW & (XROW - 1)) == 0 && ((GROW & (GROW - 1)) == 0 || GROW % 256 == 128), "row pitches the swizzles cover");
    static_assert(NS >= 3, "the ring holds the slab being read, the one landing and at least one more");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS ring too large");
    static_assert(RC <= KS * FM * FN && RC < (N_OUTER ? FN : FM), "the multiply phase has a slot for every late read");
    static_assert(!N_OUTER || FM >= 2, "late reads are issued in order, each before its first use");
};

// Where the 16-byte chunk c of slab row r sits inside the row in LDS (chunk position), and the inverse.  The
// transposing read of a 16-lane group touches 4 consecutive rows x 32 bytes, which must fall into different 64-byte
// bank groups.  Rows whose pitch is a multiple of 256 bytes all start at bank 0: position = c ^ 4*(r mod 4).  A pitch
// of 128 mod 256 bytes (192-column tiles: 384 bytes) already alternates between the two halves of the banks from row
// to row, so rows 2 and 3 of every four are rotated by 64 bytes: position = (c + 4*((r/2) mod 2)) mod chunks-per-row.
template <int ROW_BYTES>
__device__ __forceinline__ int chunk_position(int c, int r)
{
    if constexpr ((ROW_BYTES & (ROW_BYTES - 1)) == 0) return c ^ (4 * (r & 3));
    else return (c + 4 * ((r >> 1) & 1)) % (ROW_BYTES / 16);
}
template <int ROW_BYTES>
__device__ __forceinline__ int chunk_at_position(int pos, int r)
{
    if constexpr ((ROW_BYTES & (ROW_BYTES - 1)) == 0) return pos ^ (4 * (r & 3));
    else return (pos + ROW_BYTES / 16 - 4 * ((r >> 1) & 1)) % (ROW_BYTES / 16);
}

template <typename TL, int OUTS>
__global__ __launch_bounds__(TL::NT, 1) void stat_bf16_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ G,
                                                              int64_t rows_total, int seg_len, int din, int dout, int ldg, int ldo,
                                                              int64_t rows_per_split, int tiles_m, int tiles_n,
                                                              float* __restrict__ out_id, float* __restrict__ out_sq,
                                                              float* __restrict__ out_sg, const float* __restrict__ weight,
                                                              float* __restrict__ norm_partial, int examples_total, float alpha,
                                                              int byte_partials)
{
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK, NS = TL::NS, FM = TL::FM, FN = TL::FN, KS = TL::KS;
    constexpr int XROW = TL::XROW, GROW = TL::GROW, NXI = TL::NXI, NGI0 = TL::NGI0, NGI1 = TL::NGI1, RX = TL::RX;
    constexpr int LPS0 = TL::LPS0, LPS1 = TL::LPS1, FPK = TL::FPK, RC = TL::RC;
    constexpr bool TOKEN = (OUTS == OUT_TOKEN);
    static_assert(!TOKEN || NGI0 == NGI1, "the register staging assumes every wave loads the same share");
    constexpr int NGI = NGI0, LPS = LPS0;      // the per-token square only: both groups alike
    constexpr bool PER_EXAMPLE = !(OUTS == OUT_ID || OUTS == OUT_TOKEN);
    constexpr bool HAS_W = (OUTS & OUT_IDW) != 0, HAS_NORM = (OUTS & OUT_NORM) != 0;
    constexpr bool HAS_POW = (OUTS & OUT_POW) != 0;
    constexpr bool TO_MEM = (OUTS & OUT_MEM) != 0;
    constexpr bool HAS_ID = !TO_MEM && ((PER_EXAMPLE && (OUTS & OUT_ID)) || HAS_W);
    constexpr bool HAS_SQ = !TO_MEM && ((OUTS & OUT_SQ) != 0 || HAS_POW);
    constexpr bool HAS_PK = (OUTS & OUT_SIGN_PK) != 0, HAS_SF = (OUTS & OUT_SIGN_F32) != 0, HAS_U8 = (OUTS & OUT_SIGN_U8) != 0;
    static_assert(HAS_PK + HAS_SF + HAS_U8 <= 1 && (OUTS & 1023) == OUTS && OUTS != 0, "one representation of the sign counts");
    static_assert(!TO_MEM || OUTS == (OUT_MEM | OUT_SQ) || OUTS == (OUT_MEM | OUT_IDW) || OUTS == (OUT_MEM | OUT_POW),
                  "memory accumulation carries one statistic");
    static_assert(!(HAS_W && (OUTS & OUT_ID)), "identity is either weighted or not");
    static_assert(!(HAS_POW && ((OUTS & OUT_SQ) || HAS_W)), "the power statistic uses the square's register tile and the weight slot");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    int split, tm, tn;
    map_workgroup(tiles_m, tiles_n, split, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;
    const int64_t row_begin = (int64_t)split * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;
    const int slen = PER_EXAMPLE ? seg_len : (int)(row_end - row_begin);   // segment: one example, or the whole range
    const int nseg = PER_EXAMPLE ? (int)((row_end - row_begin) / seg_len) : 1;
    const int nst = (slen + BK - 1) / BK;
    const int total = nseg * nst;

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int group = wave / 4;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void)lds;
    const int wm = wave / TL::WAVES_N, wn = wave % TL::WAVES_N;

    // ---- loader geometry.  Load q of a slab (q = wave*NXI + n) fills LDS bytes [q*1024, q*1024+1024) of the X
    // part: slab rows q*RX .. q*RX+RX-1.  Lane L fills 16-byte slot (L mod XROW/16) of row q*RX + L/(XROW/16)
    // with global chunk c = slot ^ 4*(row mod 4).
    // G: load q of a slab fills the 64 chunks from q*64 on of the G part, chunk k = row k / GCH, position k % GCH;
    // group 0 takes loads 0 .. 4*NGI0-1, group 1 the rest.  `ldg` is the row pitch of G in elements, `dout` the
    // width of the column range this launch covers (G points at its first column).
    uint32_t xoff[NXI], goff[NGI0];
#pragma unroll
    for (int n = 0; n < NXI; ++n) {
        const int q = wave * NXI + n, r = q * RX + lane / TL::XCH, slot = lane % TL::XCH;
        const int c = chunk_at_position<XROW>(slot, r);
        xoff[n] = (i0 + c * 8 < din) ? (uint32_t)(r * din + c * 8) * 2u : 0x80000000u;
    }
    const int gq0 = group == 0 ? wave * NGI0 : 4 * NGI0 + (wave - 4) * NGI1;     // this wave's first load of G
#pragma unroll
    for (int n = 0; n < NGI0; ++n) {
        const int k = (gq0 + n) * 64 + lane, r = k / TL::GCH, slot = k % TL::GCH;
        const int c = chunk_at_position<GROW>(slot, r);
        goff[n] = (j0 + c * 8 < dout) ? (uint32_t)(r * ldg + c * 8) * 2u : 0x80000000u;
    }
    const int din_avail = din - i0, dout_avail = dout - j0;   // columns of this tile that exist

    // The next slab to load, kept incrementally: its number, its offset inside the example, its first row and
    // its ring buffer.  Descriptor: base at the tile's first column of slab row 0; num_records ends with the last
    // valid row, so rows past the end of the example (and everything once the range is exhausted) read as zero.
    int iss_slab = 0, iss_off = 0, iss_buf = 0;
    const uint16_t* xnext = X + row_begin * din + i0;
    const uint16_t* gnext = G + row_begin * ldg + j0;
    auto issue_slab = [&](auto GROUPC) {
        constexpr int MY_NGI = decltype(GROUPC)::value == 0 ? NGI0 : NGI1;
        int valid = 0;
        if (iss_slab < total) valid = (slen - iss_off) < BK ? (slen - iss_off) : BK;
        const uint32_t bx = lds_base + (uint32_t)(iss_buf * TL::STAGE);
        const uint32_t bg = bx + TL::X_BYTES;
        const uint32_t nrx = valid > 0 ? (uint32_t)(((valid - 1) * din + din_avail) * 2) : 0u;
        const uint32_t nrg = valid > 0 ? (uint32_t)(((valid - 1) * ldg + dout_avail) * 2) : 0u;
        const int4_t rx = make_rsrc(xnext, nrx);
        const int4_t rg = make_rsrc(gnext, nrg);
#pragma unroll
        for (int n = 0; n < NXI; ++n) dma_load_16(bx + (uint32_t)((wave * NXI + n) * 1024), xoff[n], rx);
#pragma unroll
        for (int n = 0; n < MY_NGI; ++n) dma_load_16(bg + (uint32_t)((gq0 + n) * 1024), goff[n], rg);
        xnext += (int64_t)valid * din;
        gnext += (int64_t)valid * ldg;
        iss_off += valid;
        if (iss_off >= slen) iss_off = 0;
        ++iss_slab;
        iss_buf = (iss_buf + 1 == NS) ? 0 : iss_buf + 1;
    };
    // Per-token square: no direct-to-LDS loads.  A wave's share of a slab (the same 16-byte chunks, the same places
    // in the ring) goes global -> registers, is squared there -- in fp32, rounded to bf16 (nearest even); the zero fill
    // stays zero -- and is written to LDS once.  Squaring it in place in LDS (a read and a write of every byte on top of the
    // load's own write) cost 60 % over the plain contraction; this way the LDS sees one write per byte, as it does
    // from a direct load.  Two register sets: slab s uses set s mod 2, its loads are issued two slabs before it is
    // written to the ring, which happens one slab before its first reader; the compiler tracks these loads itself.
    // (load_slab repeats the slab bookkeeping of issue_slab on purpose: sharing it through a helper changed the code
    // generated for every other flavour -- about 50 more instructions per kernel, phi = square 4 % slower.)
    [[maybe_unused]] uint4_t stage[2][TOKEN ? LPS : 1];
    auto load_slab = [&](auto SETC) {
        constexpr int S = decltype(SETC)::value;
        int valid = 0;
        if (iss_slab < total) valid = (slen - iss_off) < BK ? (slen - iss_off) : BK;
        const int nrx = valid > 0 ? ((valid - 1) * din + din_avail) * 2 : 0;
        const int nrg = valid > 0 ? ((valid - 1) * ldg + dout_avail) * 2 : 0;
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)xnext, 0, nrx, 0x00020000);
        const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc((void*)gnext, 0, nrg, 0x00020000);
#pragma unroll
        for (int n = 0; n < NXI; ++n) stage[S][n] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xoff[n], 0, 0);
#pragma unroll
        for (int n = 0; n < NGI; ++n) stage[S][NXI + n] = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)goff[n], 0, 0);
        xnext += (int64_t)valid * din;
        gnext += (int64_t)valid * ldg;
        iss_off += valid;
        if (iss_off >= slen) iss_off = 0;
        ++iss_slab;
    };
    auto square_store = [&](auto SETC, int buf) {
        constexpr int S = decltype(SETC)::value;
        unsigned char* bx = lds + buf * TL::STAGE;
        unsigned char* bg = bx + TL::X_BYTES;
#pragma unroll
        for (int n = 0; n < (TOKEN ? LPS : 1); ++n)
#pragma unroll
            for (int e = 0; e < 4; ++e) stage[S][n][e] = square_pair_rne(stage[S][n][e]);
#pragma unroll
        for (int n = 0; n < NXI; ++n) *(lds_u4)(bx + (wave * NXI + n) * 1024 + lane * 16) = stage[S][n];
#pragma unroll
        for (int n = 0; n < NGI; ++n) *(lds_u4)(bg + (wave * NGI + n) * 1024 + lane * 16) = stage[S][NXI + n];
    };

    // ---- fragment geometry.  An operand fragment of v_mfma_f32_16x16x32_bf16 is 16 columns of the slab x 32 tokens:
    // lane (blk, li) = (lane / 16, lane % 16) holds column li, tokens 8*blk .. 8*blk+7.  ds_read_b64_tr_b16 works on
    // 16-lane groups: lane li supplies the address of 4 columns (4*(li%4) ..) of slab row (li/4) of a 4-row block
    // and receives column li of those 4 rows; two reads (rows 8*blk + 0..3 and + 4..7) make a lane's 8 tokens.
    // Row r = 32*ks + 8*blk + 4*h + li/4, so r mod 4 = li/4: the swizzle term of this lane's rows.
    const int blk = lane / 16, li = lane % 16;
    const int frow = 8 * blk + li / 4;
    const int sw = 4 * (li / 4);
    const int low = (li % 4) * 8;                                   // bytes inside the fragment's two 16-byte chunks
    int a_addr[FM], b_addr[FN];
#pragma unroll
    for (int a = 0; a < FM; ++a) a_addr[a] = frow * XROW + ((((wm * TL::WM + a * 16) / 8) ^ sw) * 16) + low;
#pragma unroll
    for (int c = 0; c < FN; ++c) b_addr[c] = frow * GROW + chunk_position<GROW>((wn * TL::WN + c * 16) / 8, frow) * 16 + low;

    // register tiles: the running contraction, and one per requested per-example statistic
    float4_t acc[FM][FN];
    float4_t acc_id[HAS_ID ? FM : 1][HAS_ID ? FN : 1], acc_sq[HAS_SQ ? FM : 1][HAS_SQ ? FN : 1];
    float4_t acc_sg[HAS_SF ? FM : 1][HAS_SF ? FN : 1];
    half2_t cnt[HAS_PK ? FM : 1][HAS_PK ? FN : 1][2];
    uint32_t cnt8[HAS_U8 ? FM : 1][HAS_U8 ? FN : 1];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                acc[a][c][r] = 0.f;
                if (HAS_ID) acc_id[a][c][r] = 0.f;
                if (HAS_SQ) acc_sq[a][c][r] = 0.f;
                if (HAS_SF) acc_sg[a][c][r] = 0.f;
                if (HAS_PK) cnt[a][c][r / 2] = half2_t{(_Float16)0, (_Float16)0};
            }
            if (HAS_U8) cnt8[a][c] = 0u;
        }

    // Memory accumulation: descriptor over this tile's part of the output (base at its first entry, ending with its
    // last valid one: rows beyond the layer fall outside), one byte offset per lane and fragment column (columns
    // beyond the layer get an offset outside every range).
    [[maybe_unused]] uint32_t mem_off[FN];
    [[maybe_unused]] int4_t mem_rsrc;
    if constexpr (TO_MEM) {
        float* base = (HAS_W ? out_id : out_sq) + (int64_t)split * din * ldo + (int64_t)i0 * ldo + j0;
        const int rows_valid = din_avail < BM ? din_avail : BM, cols_valid = dout_avail < BN ? dout_avail : BN;
        mem_rsrc = make_rsrc(base, (uint32_t)(((rows_valid - 1) * ldo + cols_valid) * 4));
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            const int j = wn * TL::WN + c * 16 + li;
            mem_off[c] = j < dout_avail ? (uint32_t)(((wm * TL::WM + 4 * blk) * ldo + j) * 4) : 0x80000000u;
        }
    }

    // Fragments of one slab.  Fragment number f of a k-step: first the G fragments, then the X fragments, so the
    // ones read late (in the multiply phase) are the X fragments the last MFMAs use.
    bf16x8_t fa[KS][FM], fb[KS][FN];
    const unsigned char* rd_bx = lds;                  // buffer of the slab being read
    int rd_buf = 0;
    auto read_frag = [&](int ks, int f) {
        // the operand read last is the one of the outer loop of the multiply phase
        const bool is_g = TL::N_OUTER ? f >= FM : f < FN;
        const int k = TL::N_OUTER ? (is_g ? f - FM : f) : (is_g ? f : f - FN);
        if (is_g) {
            const unsigned char* p = rd_bx + TL::X_BYTES + b_addr[k] + ks * 32 * GROW;
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * GROW));
            fb[ks][k] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            const unsigned char* p = rd_bx + a_addr[k] + ks * 32 * XROW;
            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * XROW));
            fa[ks][k] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    auto read_phase = [&](auto GROUPC) {
        rd_bx = lds + rd_buf * TL::STAGE;
        rd_buf = (rd_buf + 1 == NS) ? 0 : rd_buf + 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int f = 0; f < FPK; ++f)
                if (ks < KS - 1 || f < FPK - RC) read_frag(ks, f);
        issue_slab(GROUPC);   // after the reads: a wave that stalls on the memory pipeline here has its reads in flight
    };
    // per-token square: after the reads of slab g, this wave's part of slab g+1 is squared and written to the ring (a
    // phase or more ahead of its first reader), and the registers it leaves take the loads of slab g+3
    auto read_phase_staged = [&](auto SETC) {
        rd_bx = lds + rd_buf * TL::STAGE;
        rd_buf = (rd_buf + 1 == NS) ? 0 : rd_buf + 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int f = 0; f < FPK; ++f)
                if (ks < KS - 1 || f < FPK - RC) read_frag(ks, f);
        square_store(SETC, rd_buf);
        load_slab(SETC);
    };
    // Multiply phase: MFMA number i is followed by fragment read i of the last k-step (while i < RC).  The
    // scheduling fences pin this order; the compiler adds the LDS waits the MFMAs need.  The G fragment index runs
    // back and forth ("snake"), so consecutive MFMAs share an operand register wherever they can: measured +2 % on an
    // MFMA-only loop (less switching on the operand reads, and the chip's clock is set by power).
    auto multiply_phase = [&]() {
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int o = 0; o < (TL::N_OUTER ? FN : FM); ++o)
#pragma unroll
                for (int ii = 0; ii < (TL::N_OUTER ? FM : FN); ++ii) {
                    const int in = (o & 1) ? (TL::N_OUTER ? FM : FN) - 1 - ii : ii;       // the inner index runs back and forth
                    const int a = TL::N_OUTER ? in : o, c = TL::N_OUTER ? o : in;
                    const int i = (ks * (TL::N_OUTER ? FN : FM) + o) * (TL::N_OUTER ? FM : FN) + ii;
                    acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ks][a], fb[ks][c], acc[a][c], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    const int late = TL::late_read_after(i);
                    if (late >= 0) {
                        read_frag(KS - 1, FPK - RC + late);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
        __builtin_amdgcn_s_setprio(0);
    };
    // end of an example: fold every tile; the example's number is needed for its weight and its norm
    int example = (int)(row_begin / (seg_len > 0 ? seg_len : 1));
    [[maybe_unused]] const int first_example = example;
    auto fold_all = [&]() {
        float w = 1.0f, norm = 0.f;
        if constexpr (HAS_W) w = weight[example];
        if constexpr (HAS_POW) w = alpha;
        if constexpr (TO_MEM) {
            // phi(M_b) leaves for memory, row by row of the wave's sub-tile; the waits on vmcnt that follow count these
            // operations too, which only makes them wait longer (loads return in order among themselves)
            auto emit = [&](auto FIRST) {
#pragma unroll
                for (int a = 0; a < FM; ++a)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t row_off = (uint32_t)((a * 16 + r) * ldo * 4);
#pragma unroll
                        for (int c = 0; c < FN; ++c) {
                            const float m = acc[a][c][r];
                            const float v = HAS_W ? w * m : (HAS_POW ? abs_power(m, w) : m * m);
                            if constexpr (decltype(FIRST)::value) mem_store_f32(v, mem_off[c], row_off, mem_rsrc);
                            else mem_add_f32(v, mem_off[c], row_off, mem_rsrc);
                            acc[a][c][r] = 0.f;
                        }
                    }
            };
            if (example == first_example) emit(std::true_type{});
            else emit(std::false_type{});
            ++example;
            return;
        }
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int c = 0; c < FN; ++c)
                if constexpr (PER_EXAMPLE)
                    fold_tile<OUTS>(acc[a][c], acc_id[HAS_ID ? a : 0][HAS_ID ? c : 0], acc_sq[HAS_SQ ? a : 0][HAS_SQ ? c : 0],
                                    acc_sg[HAS_SF ? a : 0][HAS_SF ? c : 0], cnt[HAS_PK ? a : 0][HAS_PK ? c : 0],
                                    cnt8[HAS_U8 ? a : 0][HAS_U8 ? c : 0], w, norm);
        if constexpr (HAS_NORM) {
            // this wave's part of ||M_b||^2 for this tile: lanes summed in a fixed butterfly order
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) norm += __shfl_xor(norm, off);
            if (lane == 0) norm_partial[((int64_t)(tm * tiles_n + tn) * TL::NWAVES + wave) * examples_total + example] = norm;
        }
        ++example;
    };

    constexpr int AHEAD0 = NS - 2, AHEAD1 = NS - 1;   // slabs a group has issued before its first phase
    // loads that may still be in flight when this wave's part of slab g+1 must have landed (end of phase 2g+1)
    constexpr int INFLIGHT0 = (NS - 3) * LPS0;         // group 0, after its multiply phase of slab g
    constexpr int INFLIGHT1 = (NS - 2) * LPS1;         // group 1, after its read phase of slab g
    constexpr std::integral_constant<int, 0> G0{};
    constexpr std::integral_constant<int, 1> G1{};
    if constexpr (TOKEN) {
        constexpr std::integral_constant<int, 0> S0{};
        constexpr std::integral_constant<int, 1> S1{};
        if (total > 0) {
            load_slab(S0);
            load_slab(S1);
            square_store(S0, 0);
            load_slab(S0);                        // slab 2
            wait_lds_and_barrier();               // slab 0 is visible to every wave
            // iteration g writes slab g+1 from set (g+1) mod 2: two iterations per trip, so that the set is fixed in the code
            auto iteration = [&](auto SETC) {
                read_phase_staged(SETC);
                __builtin_amdgcn_sched_barrier(0);
                wait_lds_and_barrier();
                multiply_phase();
                __builtin_amdgcn_sched_barrier(0);
                plain_barrier();
            };
            if (group == 1) plain_barrier();      // start one phase late
            int g = 0;
            for (; g + 1 < total; g += 2) {
                iteration(S1);
                iteration(S0);
            }
            if (g < total) iteration(S1);
            if (group == 0) plain_barrier();      // the other group's last multiply phase
        }
    } else
    if (total > 0) {
        if (group == 0) {
#pragma unroll
            for (int s = 0; s < AHEAD0; ++s) issue_slab(G0);
            wait_vmcnt<(AHEAD0 - 1) * LPS0>();
        } else {
#pragma unroll
            for (int s = 0; s < AHEAD1; ++s) issue_slab(G1);
            wait_vmcnt<(AHEAD1 - 1) * LPS1>();
        }
        wait_lds_and_barrier();               // slab 0 is visible to every wave
        int st_in_seg = 0;
        if (group == 0) {
            for (int g = 0; g < total; ++g) {
                read_phase(G0);
                __builtin_amdgcn_sched_barrier(0);
                wait_lds_and_barrier();       // ends phase 2g
                multiply_phase();
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt<INFLIGHT0>();   // this wave's part of slab g+1 has landed
                plain_barrier();              // ends phase 2g+1
                if (PER_EXAMPLE && ++st_in_seg == nst) { st_in_seg = 0; fold_all(); }
            }
            plain_barrier();                  // the other group's last multiply phase
        } else {
            plain_barrier();                  // start one phase late
            for (int g = 0; g < total; ++g) {
                read_phase(G1);
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt<INFLIGHT1>();   // this wave's part of slab g+1 has landed
                wait_lds_and_barrier();       // ends phase 2g+1
                multiply_phase();
                __builtin_amdgcn_sched_barrier(0);
                plain_barrier();              // ends phase 2g+2
                if (PER_EXAMPLE && ++st_in_seg == nst) { st_in_seg = 0; fold_all(); }
            }
        }
    }
    wait_vmcnt<0>();   // drain the (empty) loads issued past the end before the LDS is released

    // ---- epilogue: lane holds column (lane%16), rows 4*(lane/16) + r of each 16x16 tile
    // Packed sign counts of a split batch leave as bytes: one dword per lane and 16 x 16 tile holding the lane's four
    // counts (rows ib .. ib+3 of column jn; at most 127 examples per group), laid out [split][tile][wave][tile of the
    // wave][lane] -- a quarter of the bytes of fp32 partial sums, in dense 256-byte stores.
    if constexpr (HAS_PK) {
        if (byte_partials) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(out_sg) +
                            ((((int64_t)split * tiles_m + tm) * tiles_n + tn) * TL::NWAVES + wave) * (int64_t)(FM * FN * 64) + lane;
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int c = 0; c < FN; ++c) {
                    uint32_t w = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) w |= ((uint32_t)(int)cnt[a][c][r / 2][r % 2] & 0xffu) << (8 * r);
                    dst[(a * FN + c) * 64] = w;
                }
            return;
        }
    }
    // outputs have their own row pitch: S itself (pointing at the first column of the range, pitch of the whole
    // layer) or partials [split][din][ldo]
    const int64_t split_off = (int64_t)split * din * ldo;
    const int jn = lane % 16, ib = 4 * (lane / 16);
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            const int j = j0 + wn * TL::WN + c * 16 + jn;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = i0 + wm * TL::WM + a * 16 + ib + r;
                if (i < din && j < dout) {
                    const int64_t e = split_off + (int64_t)i * ldo + j;
                    if constexpr (!PER_EXAMPLE) out_id[e] = acc[a][c][r];
                    if constexpr (HAS_ID) out_id[e] = acc_id[a][c][r];
                    if constexpr (HAS_SQ) out_sq[e] = acc_sq[a][c][r];
                    if constexpr (HAS_SF) out_sg[e] = acc_sg[a][c][r];
                    if constexpr (HAS_PK) out_sg[e] = (float)cnt[a][c][r / 2][r % 2];
                    if constexpr (HAS_U8) out_sg[e] = (float)((int)((cnt8[a][c] >> (8 * r)) & 0xffu) - nseg);
                }
            }
        }
}

// out = bf16(in^2), 8 values per lane per step
__global__ __launch_bounds__(256) void square_bf16_kernel(const uint4_t* __restrict__ in, uint4_t* __restrict__ out, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        uint4_t v = __builtin_nontemporal_load(in + i);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = square_pair_rne(v[e]);
        out[i] = v;
    }
}

// plain contractions and packed sign counts: 256 x 256 block, 128 x 64 per wave, slabs of 32 tokens, ring of 4;
// the per-token square stages its slabs through registers (no loads in flight into the ring) and takes a ring of 3;
// two fp32 register tiles (phi = square, sign counts beyond 2048 examples): 256 x 128 block, 64 x 64 per wave, or --
// for a single statistic -- 256 x 192 (64 x 96 per wave, 96 + 96 accumulators): 22 % fewer bytes from L2 into LDS and
// 17 % fewer fragment reads per FLOP.
using TileWide = Bf16Tile<256, 256, 128, 64, 32, 4, 5>;
using TileToken = Bf16Tile<256, 256, 128, 64, 32, 3, 5>;
using TilePhi = Bf16Tile<256, 128, 64, 64, 32, 4, 3>;
// (ring of 5 slabs = 140 KB; five of its ten fragments -- G fragments, its sub-tile being walked column by column -- are
// read in the multiply phase, each 7 MFMAs ahead of its first use: measured best of rings of 4 and 5, 1 to 5 late
// fragments and leads of 5 to 10, a spread of 3 %)
using TilePhi192 = Bf16Tile<256, 192, 64, 96, 32, 5, 5, 7>;

// A launch may cover only the columns [col0, col0 + ncols) of the layer, so that launches of different block shapes
// can sit side by side: G keeps the row pitch of the whole layer; the outputs point at their first element and
// have the row pitch `ldo` (the layer's when they are S itself, the range's when they are partial sums).
struct ColumnRange {
    int64_t col0 = 0, ncols = -1, ldo = -1;      // ncols < 0: the whole layer
};

template <typename TL, int OUTS>
hipError_t launch_one(const uint16_t* X, const uint16_t* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                      const StatPlan& plan, float* out_id, float* out_sq, float* out_sg, hipStream_t stream,
                      const float* weight = nullptr, float* norm_partial = nullptr, float alpha = 0.f,
                      ColumnRange range = ColumnRange{}, bool byte_partials = false)
{
    constexpr bool PER_EXAMPLE = !(OUTS == OUT_ID || OUTS == OUT_TOKEN);
    const int64_t ldg = dout;
    int64_t ldo = dout;
    if (range.ncols >= 0) {
        G += range.col0;
        dout = range.ncols;
        ldo = range.ldo;
    }
    const int tiles_m = (int)((din + TL::BM - 1) / TL::BM), tiles_n = (int)((dout + TL::BN - 1) / TL::BN);
    const int64_t rows_per_split = PER_EXAMPLE ? plan.per_split * T : plan.per_split;
    auto kern = stat_bf16_kernel<TL, OUTS>;
    // once per kernel and process, also when several host threads launch at the same time
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] { attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES); });
    if (attr_err != hipSuccess) return attr_err;
    const dim3 grid((unsigned)(tiles_m * tiles_n * plan.nsplit)), block(TL::NT);
    kern<<<grid, block, TL::LDS_BYTES, stream>>>(X, G, B * T, (int)T, (int)din, (int)dout, (int)ldg, (int)ldo, rows_per_split, tiles_m,
                                                 tiles_n, out_id, out_sq, out_sg, weight, norm_partial, (int)B, alpha, byte_partials ? 1 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Four waves, one per SIMD, 128 x 128 per wave: the kernel of plain contractions over long ranges.
//
// Same tile, slabs, swizzle, fragment reads and zero-filling descriptors as above; what differs is the schedule.
// There is no second wave on a SIMD to hide anything behind, so a wave interleaves everything itself: iteration g
// issues the 64 MFMAs of slab g from one set of fragment registers and, between them, the 32 fragment reads of slab
// g+1 into the other set and its 8 loads of slab g+NS-1, whose ring buffer held slab g-1 (every wave's MFMAs of slab
// g-1 came before the barrier that ended iteration g-1, and they had waited for that slab's fragments).  One
// barrier per slab: before it a wave makes sure its part of slab g+2 has landed.
// Every instruction between two MFMAs costs MFMA time here, so there are as few as can be:
//   * the loop is unrolled over a whole period of (fragment set, ring buffer), which turns every LDS address into
//     lane base + immediate;
//   * the four loads of an operand share one write of M0 (the LDS base): load n adds n KiB through its instruction
//     offset, which moves the LDS address and the global address alike, so lane offsets are lowered by n KiB -- and,
//     to keep them non-negative, raised by 3 KiB against a descriptor base 3 KiB lower (nothing below the true base
//     is touched: every effective offset is >= 3 KiB, and a range of 3 KiB or less reads as empty);
//   * the descriptors are kept in scalar registers and only moved on: a slab is full, the last one, or past the end.
constexpr int QUAD_NS = 5;
struct QuadTile {
    static constexpr int BM = 256, BN = 256, WM = 128, WN = 128, BK = 32, NS = QUAD_NS;
    static constexpr int FM = WM / 16, FN = WN / 16, NWAVES = 4, NT = NWAVES * 64;
    static constexpr int XROW = BM * 2, GROW = BN * 2, X_BYTES = BK * XROW, G_BYTES = BK * GROW, STAGE = X_BYTES + G_BYTES;
    static constexpr int LDS_BYTES = NS * STAGE;
    static constexpr int NXI = X_BYTES / 1024 / NWAVES, NGI = G_BYTES / 1024 / NWAVES, LPS = NXI + NGI;
    static constexpr int RX = 1024 / XROW, RG = 1024 / GROW;
    static constexpr int PERIOD = (NS % 2 == 0) ? NS : 2 * NS;     // iterations after which fragment set and buffers repeat
    static constexpr int BIAS = (NXI > NGI ? NXI : NGI) * 1024 - 1024;
    // after which MFMA of an iteration things are issued: fragment half k after MFMA 2k+1, load n after MFMA 4+7n
    static constexpr int READ_FIRST = 1, READ_STEP = 2, LOAD_FIRST = 4, LOAD_STEP = 7, ADVANCE_AT = 60;
    static_assert(LDS_BYTES <= 160 * 1024 && NS >= 4, "ring");
    static_assert(NXI * 1024 <= 4096 && NGI * 1024 <= 4096, "instruction offsets are 12 bits");
    static_assert(READ_FIRST + READ_STEP * (2 * (FM + FN) - 1) < FM * FN, "every fragment read has its MFMA");
    static_assert(LOAD_FIRST >= 3 && LOAD_FIRST + LOAD_STEP * (LPS - 1) < ADVANCE_AT && ADVANCE_AT < FM * FN,
                  "loads sit between the descriptor update and the move to the next slab");
};

// LDS base of a group of direct-to-LDS loads.  M0 must stay as it is until the group's last load: no instruction the
// compiler generates for this kernel writes it.  A load may not follow the write directly; WAIT adds the wait state
// where no other instruction sits between.
template <int OFF, bool WAIT>
__device__ __forceinline__ void dma_set_base(uint32_t sbase)
{
    if constexpr (WAIT) asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0" : : "s"(sbase), "n"(OFF) : "memory", "m0", "scc");
    else asm volatile("s_add_u32 m0, %0, %1" : : "s"(sbase), "n"(OFF) : "memory", "m0", "scc");
}
// one load of the group: 1 KiB to LDS (base in M0) + IOFF + lane*16, from descriptor base + voff + IOFF
template <int IOFF>
__device__ __forceinline__ void dma_load_16_off(uint32_t voff, int4_t rsrc)
{
    asm volatile("buffer_load_dwordx4 %0, %1, 0 offen offset:%2 lds" : : "v"(voff), "s"(rsrc), "n"(IOFF) : "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// which fragment half (G fragments first, two halves each) is read after MFMA i of an iteration, which load is issued; -1: none
constexpr int quad_read_slot(int i)
{
    const int k = (i - QuadTile::READ_FIRST) / QuadTile::READ_STEP;
    return (i >= QuadTile::READ_FIRST && (i - QuadTile::READ_FIRST) % QuadTile::READ_STEP == 0 && k < 2 * (QuadTile::FM + QuadTile::FN)) ? k : -1;
}
constexpr int quad_load_slot(int i)
{
    const int n = (i - QuadTile::LOAD_FIRST) / QuadTile::LOAD_STEP;
    return (i >= QuadTile::LOAD_FIRST && (i - QuadTile::LOAD_FIRST) % QuadTile::LOAD_STEP == 0 && n < QuadTile::LPS) ? n : -1;
}

__global__ __launch_bounds__(QuadTile::NT, 1) void stat_bf16_quad_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ G,
                                                                         int64_t rows_total, int din, int dout, int64_t rows_per_split,
                                                                         int tiles_m, int tiles_n, float* __restrict__ out)
{
    using TL = QuadTile;
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK, NS = TL::NS, FM = TL::FM, FN = TL::FN;
    constexpr int XROW = TL::XROW, GROW = TL::GROW, NXI = TL::NXI, NGI = TL::NGI, RX = TL::RX, RG = TL::RG, LPS = TL::LPS;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    int split, tm, tn;
    map_workgroup(tiles_m, tiles_n, split, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;
    const int64_t row_begin = (int64_t)split * rows_per_split;
    int64_t row_end = row_begin + rows_per_split;
    if (row_end > rows_total) row_end = rows_total;
    const int slen = (int)(row_end - row_begin);
    const int total = (slen + BK - 1) / BK;
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void)lds;
    const int wm = wave / 2, wn = wave % 2;

    // ---- loader geometry: as in the eight-wave kernel (load q = wave*NXI + n fills slab rows q*RX ..), with the
    // group bias and the instruction offset of load n taken out of the lane offset
    uint32_t xoff[NXI], goff[NGI];
#pragma unroll
    for (int n = 0; n < NXI; ++n) {
        const int q = wave * NXI + n, r = q * RX + lane / (XROW / 16), slot = lane % (XROW / 16);
        const int c = slot ^ (4 * (r & 3));
        xoff[n] = ((i0 + c * 8 < din) ? (uint32_t)(r * din + c * 8) * 2u : 0x80000000u) + (uint32_t)(TL::BIAS - n * 1024);
    }
#pragma unroll
    for (int n = 0; n < NGI; ++n) {
        const int q = wave * NGI + n, r = q * RG + lane / (GROW / 16), slot = lane % (GROW / 16);
        const int c = slot ^ (4 * (r & 3));
        goff[n] = ((j0 + c * 8 < dout) ? (uint32_t)(r * dout + c * 8) * 2u : 0x80000000u) + (uint32_t)(TL::BIAS - n * 1024);
    }
    const uint32_t wave_x = lds_base + (uint32_t)(wave * NXI * 1024);                  // this wave's part of a buffer
    const uint32_t wave_g = lds_base + (uint32_t)(TL::X_BYTES + wave * NGI * 1024);

    // ---- descriptors of the next slab to issue.  Base: the tile's first column of the slab's first row (minus the
    // bias); range: up to the tile's last column of the slab's last valid row, i.e. rows * row bytes minus the bytes
    // left of the tile (plus the bias).  A slab is full (BK rows), the last one of the range, or past the end (no
    // rows: the range is at most the bias, so every lane reads zero).
    const int xrow_bytes = din * 2, grow_bytes = dout * 2, xcut = i0 * 2 - TL::BIAS, gcut = j0 * 2 - TL::BIAS;
    const int last_rows = slen - (total - 1) * BK;
    const int xfull = BK * xrow_bytes, gfull = BK * grow_bytes, xlast = last_rows * xrow_bytes, glast = last_rows * grow_bytes;
    uint64_t xptr = (uint64_t)(X + row_begin * din + i0) - TL::BIAS, gptr = (uint64_t)(G + row_begin * dout + j0) - TL::BIAS;
    int left = total, xadv = 0, gadv = 0;          // slabs not yet issued; bytes the bases move after this one
    int4_t rx, rg;
    auto slab_rows = [&]() {
        xadv = left > 1 ? xfull : (left == 1 ? xlast : 0);
        gadv = left > 1 ? gfull : (left == 1 ? glast : 0);
    };
    auto slab_range = [&]() {
        const int nx = xadv - xcut, ng = gadv - gcut;
        // word 1: address bits 32..47 only, so that stride and swizzle stay 0 whatever the upper address bits are
        rx = int4_t{(int)(uint32_t)xptr, (int)((uint32_t)(xptr >> 32) & 0xffffu), nx > 0 ? nx : 0, 0x00020000};
        rg = int4_t{(int)(uint32_t)gptr, (int)((uint32_t)(gptr >> 32) & 0xffffu), ng > 0 ? ng : 0, 0x00020000};
    };
    auto slab_advance = [&]() {
        xptr += (uint32_t)xadv;
        gptr += (uint32_t)gadv;
        --left;
    };
    auto set_group = [&](auto BUFC, auto GROUPC, auto WAITC) {
        constexpr int BUF = decltype(BUFC)::value;
        constexpr bool WAIT = decltype(WAITC)::value;
        if constexpr (decltype(GROUPC)::value == 0) dma_set_base<BUF * TL::STAGE, WAIT>(wave_x);
        else dma_set_base<BUF * TL::STAGE, WAIT>(wave_g);
    };
    auto issue_one = [&](auto NC) {
        constexpr int n = decltype(NC)::value;
        if constexpr (n < NXI) dma_load_16_off<n * 1024>(xoff[n], rx);
        else dma_load_16_off<(n - NXI) * 1024>(goff[n - NXI], rg);
    };

    // ---- fragment geometry: as in the eight-wave kernel
    const int blk = lane / 16, li = lane % 16;
    const int frow = 8 * blk + li / 4;
    const int sw = 4 * (li / 4);
    const int low = (li % 4) * 8;
    int a_addr[FM], b_addr[FN];
#pragma unroll
    for (int a = 0; a < FM; ++a) a_addr[a] = frow * XROW + ((((wm * TL::WM + a * 16) / 8) ^ sw) * 16) + low;
#pragma unroll
    for (int c = 0; c < FN; ++c) b_addr[c] = frow * GROW + ((((wn * TL::WN + c * 16) / 8) ^ sw) * 16) + low;

    float4_t acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[a][c][r] = 0.f;

    // two sets of fragments, each fragment as the two transposing reads that make it
    short4_t fa[2][FM][2], fb[2][FN][2];
    // half h (tokens 8*blk + 4*h .. + 3) of fragment f (G fragments first) of the slab in buffer BUF
    auto read_half = [&](auto SETC, auto BUFC, int f, int h) {
        constexpr int SET = decltype(SETC)::value, BUF = decltype(BUFC)::value;
        const unsigned char* base = lds + BUF * TL::STAGE;
        if (f < FN) fb[SET][f][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(base + TL::X_BYTES + b_addr[f] + h * 4 * GROW));
        else fa[SET][f - FN][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(base + a_addr[f - FN] + h * 4 * XROW));
    };
    auto whole = [&](const short4_t (&h)[2]) { return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7)); };

    // Iteration g: fragment set CUR holds slab g; buffer RB holds slab g+1; buffer WB is free for slab g+NS-1.
    auto iteration = [&](auto CURC, auto RBC, auto WBC) {
        constexpr int CUR = decltype(CURC)::value;
        static_for<FM * FN>([&](auto IC) {
            constexpr int i = decltype(IC)::value, a = i / FN, cc = i % FN, c = (a & 1) ? FN - 1 - cc : cc;
            acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(whole(fa[CUR][a]), whole(fb[CUR][c]), acc[a][c], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (i == 0) { slab_rows(); __builtin_amdgcn_sched_barrier(0); }
            if constexpr (i == 1) { slab_range(); __builtin_amdgcn_sched_barrier(0); }
            if constexpr (i == TL::ADVANCE_AT) { slab_advance(); __builtin_amdgcn_sched_barrier(0); }
            constexpr int k = quad_read_slot(i);
            if constexpr (k >= 0) {
                read_half(std::integral_constant<int, 1 - CUR>{}, RBC, k / 2, k % 2);
                __builtin_amdgcn_sched_barrier(0);
            }
            constexpr int nb = quad_load_slot(i + 1);      // a group's LDS base is set one MFMA ahead of its first load
            if constexpr (nb == 0 || nb == NXI) {
                set_group(WBC, std::integral_constant<int, nb == 0 ? 0 : 1>{}, std::false_type{});
                __builtin_amdgcn_sched_barrier(0);
            }
            constexpr int n = quad_load_slot(i);
            if constexpr (n >= 0) {
                issue_one(std::integral_constant<int, n>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        wait_vmcnt<(NS - 3) * LPS>();     // this wave's part of slab g+2 has landed (slabs g+3 .. g+NS-1 may be in flight)
        plain_barrier();
    };

    if (total > 0) {
        static_for<NS - 1>([&](auto SC) {      // slabs 0 .. NS-2 into buffers 0 .. NS-2
            slab_rows();
            slab_range();
            set_group(SC, std::integral_constant<int, 0>{}, std::true_type{});
            static_for<NXI>([&](auto NC) { issue_one(NC); });
            set_group(SC, std::integral_constant<int, 1>{}, std::true_type{});
            static_for<NGI>([&](auto NC) { issue_one(std::integral_constant<int, NXI + decltype(NC)::value>{}); });
            slab_advance();
        });
        wait_vmcnt<(NS - 2) * LPS>();
        plain_barrier();                        // slab 0 is visible to every wave
#pragma unroll
        for (int f = 0; f < FM + FN; ++f) {
            read_half(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, f, 0);
            read_half(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, f, 1);
        }
        wait_vmcnt<(NS - 3) * LPS>();
        plain_barrier();                        // so is slab 1
        // iteration g0 + k: set k mod 2, reads buffer (k+1) mod NS, refills buffer (k-1) mod NS
        for (int g0 = 0; g0 < total; g0 += TL::PERIOD) {
            static_for<TL::PERIOD>([&](auto KC) {
                constexpr int k = decltype(KC)::value;
                if (g0 + k < total)
                    iteration(std::integral_constant<int, k & 1>{}, std::integral_constant<int, (k + 1) % NS>{},
                              std::integral_constant<int, (k + NS - 1) % NS>{});
            });
        }
    }
    wait_vmcnt<0>();   // drain the (empty) loads issued past the end before the LDS is released

    // ---- epilogue: lane holds column (lane%16), rows 4*(lane/16) + r of each 16x16 tile
    const int64_t split_off = (int64_t)split * din * dout;
    const int jn = lane % 16, ib = 4 * (lane / 16);
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            const int j = j0 + wn * TL::WN + c * 16 + jn;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = i0 + wm * TL::WM + a * 16 + ib + r;
                if (i < din && j < dout) out[split_off + (int64_t)i * dout + j] = acc[a][c][r];
            }
        }
}

// Ranges shorter than this many rows per workgroup stay on the eight-wave kernel, whose start-up is shorter.
constexpr int64_t QUAD_MIN_ROWS = 1024;

hipError_t launch_quad(const uint16_t* X, const uint16_t* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                       const StatPlan& plan, float* out, hipStream_t stream)
{
    using TL = QuadTile;
    const int tiles_m = (int)((din + TL::BM - 1) / TL::BM), tiles_n = (int)((dout + TL::BN - 1) / TL::BN);
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [] { attr_err = hipFuncSetAttribute((const void*)stat_bf16_quad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES); });
    if (attr_err != hipSuccess) return attr_err;
    const dim3 grid((unsigned)(tiles_m * tiles_n * plan.nsplit)), block(TL::NT);
    stat_bf16_quad_kernel<<<grid, block, TL::LDS_BYTES, stream>>>(X, G, B * T, (int)din, (int)dout, plan.per_split, tiles_m, tiles_n, out);
    return hipGetLastError();
}

// sign counts are packed (and the tile is 256 x 256) while a group of examples cannot exceed 2048
bool sign_is_packed(int64_t B) { return B <= 2048; }

// S = sum over the groups of the byte-wide partial sign counts the 256 x 256 kernel leaves (see its epilogue): one
// thread per dword, groups added in ascending order (integers: any order gives the same sum)
__global__ __launch_bounds__(256) void reduce_sign_bytes_kernel(const uint32_t* __restrict__ partial, int nsplit, int tiles_m, int tiles_n,
                                                                int din, int dout, float* __restrict__ S)
{
    using TL = TileWide;
    constexpr int PER_WAVE = TL::FM * TL::FN * 64, PER_TILE = PER_WAVE * TL::NWAVES;
    const int64_t total = (int64_t)tiles_m * tiles_n * PER_TILE;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int sum[4] = {0, 0, 0, 0};
    for (int s = 0; s < nsplit; ++s) {
        const uint32_t w = partial[(int64_t)s * total + idx];
#pragma unroll
        for (int r = 0; r < 4; ++r) sum[r] += (int)(signed char)((w >> (8 * r)) & 0xffu);
    }
    const int lane = (int)(idx % 64), f = (int)((idx / 64) % (TL::FM * TL::FN)), wave = (int)((idx / PER_WAVE) % TL::NWAVES);
    const int tile = (int)(idx / PER_TILE), tm = tile / tiles_n, tn = tile % tiles_n;
    const int a = f / TL::FN, c = f % TL::FN, wm = wave / TL::WAVES_N, wn = wave % TL::WAVES_N;
    const int j = tn * TL::BN + wn * TL::WN + c * 16 + lane % 16;
    const int i = tm * TL::BM + wm * TL::WM + a * 16 + 4 * (lane / 16);
    if (j < dout) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (i + r < din) S[(int64_t)(i + r) * dout + j] = (float)sum[r];
    }
}

}  // namespace

// Packed sign counts of a split batch can leave the kernel as bytes when no group exceeds 127 examples.
bool sign_byte_partials_possible(int64_t B, int64_t per_split) { return sign_is_packed(B) && per_split <= MAX_U8_EXAMPLES; }
size_t sign_byte_partial_bytes(int64_t din, int64_t dout)
{
    return (size_t)((din + TileWide::BM - 1) / TileWide::BM) * (size_t)((dout + TileWide::BN - 1) / TileWide::BN) * (size_t)(TileWide::BM * TileWide::BN);
}
hipError_t launch_reduce_sign_bytes(const void* partial, int nsplit, int64_t din, int64_t dout, float* S, hipStream_t stream)
{
    const int tiles_m = (int)((din + TileWide::BM - 1) / TileWide::BM), tiles_n = (int)((dout + TileWide::BN - 1) / TileWide::BN);
    const int64_t total = (int64_t)tiles_m * tiles_n * (TileWide::BM * TileWide::BN / 4);
    reduce_sign_bytes_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>((const uint32_t*)partial, nsplit, tiles_m, tiles_n,
                                                                                             (int)din, (int)dout, S);
    return hipGetLastError();
}

void bf16_tile_shape(Mode mode, int64_t B, int* bm, int* bn)
{
    if (mode == MODE_IDENTITY || mode == MODE_TOKEN_SQ || mode == MODE_NORMS || (mode == MODE_SIGN && sign_is_packed(B))) { *bm = TileWide::BM; *bn = TileWide::BN; }
    else { *bm = TilePhi::BM; *bn = TilePhi::BN; }
}

bool bf16_supports(int64_t B, int64_t T, int64_t din, int64_t dout)
{
    // 16-byte chunks of a row; tiny problems are latency-bound and stay on the SIMT kernel
    if (din % 8 != 0 || dout % 8 != 0 || din < 32 || dout < 32 || B * T < 16) return false;
    // per-slab descriptors and lane offsets are 32-bit byte counts: one slab of rows must stay below 2 GiB
    const int64_t bk = 32;
    if (bk * din * 2 + 4096 >= ((int64_t)1 << 31) || bk * dout * 2 + 4096 >= ((int64_t)1 << 31)) return false;
    return true;
}

hipError_t launch_square_bf16(const void* in, void* out, int64_t n, hipStream_t stream)
{
    const int64_t n16 = n / 8;
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    square_bf16_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>((const uint4_t*)in, (uint4_t*)out, n16);
    return hipGetLastError();
}

namespace {

// One statistic that needs two fp32 register tiles (phi = square, |.|^alpha, weighted sums) -- or, where the plan says
// so, one register tile on 256 x 256 blocks and additions to the output in memory.  The first
// plan.wide_cols columns of S run on 256 x 192 blocks as plan.wide_nsplit groups of examples, the remaining columns
// on 256 x 128 blocks as plan.nsplit groups; each part writes straight into S when it is one group, else into partial
// sums of its own row pitch (the wide part's first in the buffer).
template <int OUTS>
hipError_t launch_two_tile(const uint16_t* x, const uint16_t* g, int64_t B, int64_t T, int64_t din, int64_t dout, const StatPlan& plan,
                           float* S, float* partials, hipStream_t stream, const float* weight, float alpha)
{
    constexpr bool TO_ID = (OUTS & OUT_IDW) != 0;       // which output slot of the kernel the statistic leaves through
    auto go = [&](auto tile, const StatPlan& p, float* out, ColumnRange range) {
        using TL = decltype(tile);
        return launch_one<TL, OUTS>(x, g, B, T, din, dout, p, TO_ID ? out : nullptr, TO_ID ? nullptr : out, nullptr, stream, weight, nullptr,
                                    alpha, range);
    };
    if (plan.mem_fold) {
        float* out = plan.nsplit > 1 ? partials : S;
        return launch_one<TileWide, OUTS | OUT_MEM>(x, g, B, T, din, dout, plan, TO_ID ? out : nullptr, TO_ID ? nullptr : out, nullptr, stream,
                                                    weight, nullptr, alpha);
    }
    if (plan.wide_cols == 0) return go(TilePhi{}, plan, plan.nsplit > 1 ? partials : S, ColumnRange{});
    StatPlan wide = plan;
    wide.nsplit = plan.wide_nsplit;
    wide.per_split = plan.wide_per_split;
    hipError_t e = go(TilePhi192{}, wide, wide.nsplit > 1 ? partials : S, ColumnRange{0, plan.wide_cols, wide.nsplit > 1 ? plan.wide_cols : dout});
    const int64_t rest = dout - plan.wide_cols;
    float* rest_partials = (float*)((char*)partials + plan.wide_ws_bytes);
    if (e == hipSuccess && rest > 0)
        e = go(TilePhi{}, plan, plan.nsplit > 1 ? rest_partials : S + plan.wide_cols, ColumnRange{plan.wide_cols, rest, plan.nsplit > 1 ? rest : dout});
    return e;
}

}  // namespace

void bf16_wide_tile_shape(int* bm, int* bn) { *bm = TilePhi192::BM; *bn = TilePhi192::BN; }

hipError_t launch_stat_bf16(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, Mode mode,
                            const StatPlan& plan, float* S, float* partials, hipStream_t stream)
{
    const uint16_t* x = (const uint16_t*)X;
    const uint16_t* g = (const uint16_t*)G;
    float* out = plan.nsplit > 1 ? partials : S;
    switch (mode) {
    case MODE_IDENTITY:
        if (plan.per_split >= QUAD_MIN_ROWS) return launch_quad(x, g, B, T, din, dout, plan, out, stream);
        return launch_one<TileWide, OUT_ID>(x, g, B, T, din, dout, plan, out, nullptr, nullptr, stream);
    case MODE_TOKEN_SQ: return launch_one<TileToken, OUT_TOKEN>(x, g, B, T, din, dout, plan, out, nullptr, nullptr, stream);
    case MODE_SQUARE:
        return launch_two_tile<OUT_SQ>(x, g, B, T, din, dout, plan, S, partials, stream, nullptr, 0.f);
    case MODE_SIGN:
        if (sign_is_packed(B))
            return launch_one<TileWide, OUT_SIGN_PK>(x, g, B, T, din, dout, plan, nullptr, nullptr, out, stream, nullptr, nullptr, 0.f,
                                                     ColumnRange{}, plan.sign_bytes);
        return launch_one<TilePhi, OUT_SIGN_F32>(x, g, B, T, din, dout, plan, nullptr, nullptr, out, stream);
    default: return hipErrorInvalidValue;
    }
}

// N partial sums of ||M_b||_F^2: [tiles][8 waves][B]; tiles of the 256 x 256 block shape
int64_t bf16_norm_partials(int64_t din, int64_t dout)
{
    return ((din + TileWide::BM - 1) / TileWide::BM) * ((dout + TileWide::BN - 1) / TileWide::BN) * TileWide::NWAVES;
}

// per-example squared norms: a per-example contraction on the large tile whose only output is the norm partials
hipError_t launch_norms_bf16(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, const StatPlan& plan,
                             float* norm_partial, hipStream_t stream)
{
    return launch_one<TileWide, OUT_NORM>((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, plan, nullptr, nullptr, nullptr, stream,
                                          nullptr, norm_partial);
}

// S = sum_b w_b M_b (two register tiles: block shape of phi = square)
hipError_t launch_weighted_bf16(const void* X, const void* G, const float* w, int64_t B, int64_t T, int64_t din, int64_t dout,
                                const StatPlan& plan, float* S, float* partials, hipStream_t stream)
{
    return launch_two_tile<OUT_IDW>((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, plan, S, partials, stream, w, 0.f);
}

// S = sum_b |M_b|^alpha
hipError_t launch_power_bf16(const void* X, const void* G, float alpha, int64_t B, int64_t T, int64_t din, int64_t dout,
                             const StatPlan& plan, float* S, float* partials, hipStream_t stream)
{
    return launch_two_tile<OUT_POW>((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, plan, S, partials, stream, nullptr, alpha);
}

// Identity, square and sign from one contraction: possible while a group of examples fits the byte counters.
bool bf16_triple_supported(const StatPlan& plan) { return plan.per_split <= MAX_U8_EXAMPLES; }

hipError_t launch_stat_bf16_triple(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                   const StatPlan& plan, float* out_id, float* out_sq, float* out_sg, hipStream_t stream)
{
    if (!bf16_triple_supported(plan) || !out_id || !out_sq || !out_sg) return hipErrorInvalidValue;
    return launch_one<TilePhi, OUT_ID | OUT_SQ | OUT_SIGN_U8>((const uint16_t*)X, (const uint16_t*)G, B, T, din, dout, plan, out_id,
                                                              out_sq, out_sg, stream);
}

// Two statistics from one contraction (always on the two-register-tile block shape).  A NULL output is not wanted.
hipError_t launch_stat_bf16_pair(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                 const StatPlan& plan, float* out_id, float* out_sq, float* out_sg, hipStream_t stream)
{
    const uint16_t* x = (const uint16_t*)X;
    const uint16_t* g = (const uint16_t*)G;
    const bool pk = sign_is_packed(B);
    if (out_id && out_sq && !out_sg) return launch_one<TilePhi, OUT_ID | OUT_SQ>(x, g, B, T, din, dout, plan, out_id, out_sq, nullptr, stream);
    if (out_id && !out_sq && out_sg) {
        if (pk) return launch_one<TilePhi, OUT_ID | OUT_SIGN_PK>(x, g, B, T, din, dout, plan, out_id, nullptr, out_sg, stream);
        return launch_one<TilePhi, OUT_ID | OUT_SIGN_F32>(x, g, B, T, din, dout, plan, out_id, nullptr, out_sg, stream);
    }
    if (!out_id && out_sq && out_sg) {
        if (pk) return launch_one<TilePhi, OUT_SQ | OUT_SIGN_PK>(x, g, B, T, din, dout, plan, nullptr, out_sq, out_sg, stream);
        return launch_one<TilePhi, OUT_SQ | OUT_SIGN_F32>(x, g, B, T, din, dout, plan, nullptr, out_sq, out_sg, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace pex
