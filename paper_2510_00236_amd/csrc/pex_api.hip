// pex_api.hip -- the C ABI of libpex: host-side validation, planning and kernel dispatch.
// Every entry point validates first and launches nothing on error.
#include <atomic>
#include <cstdlib>
#include <mutex>

#include "pex_internal.h"

// Scratch of pex_stat_noalloc: device memory that belongs to the library, one copy per GPU, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels and copies take the address that
// call returns for the current device.
static __device__ __align__(256) unsigned char scratch[PEX_NOALLOC_SCRATCH_BYTES];

namespace pex {

// The address of `scratch` on the current device, looked up once per device.
static hipError_t scratch_address(void** out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void* ptr[MAX_DEVICES] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

// Planner options.  Their first values come from the environment, read once per process; afterwards only
// pex_set_option changes them.  Atomics, so a host thread that plans while another one sets an option reads a
// whole value; a plan made under one value and launched under another is caught as PEX_ERR_WORKSPACE.
constexpr int NUM_OPTIONS = 5;
struct Options {
    std::atomic<int> v[NUM_OPTIONS];
};

static bool known_option(int opt) { return opt >= 0 && opt < NUM_OPTIONS; }

static int clamp_option(int opt, int value)
{
    if (opt == PEX_OPT_MAX_SPLIT) return value < 1 ? 1 : (value > 32 ? 32 : value);
    if (opt == PEX_OPT_GRAM_NORMS) return value < 0 ? 0 : (value > 3 ? 3 : value);   // 2, 3: forced, on small / large blocks
    return value < 0 ? 0 : (value > 2 ? 2 : value);      // every other option: 0 = off, 1 = cost model, 2 = forced
}

static Options& options()
{
    static Options o;
    static std::once_flag once;
    std::call_once(once, [] {
        const char* names[NUM_OPTIONS] = {"PEX_MAX_SPLIT", "PEX_TOKEN_PRESQUARE", "PEX_WIDE_BLOCKS", "PEX_GRAM_NORMS", "PEX_MEMORY_FOLD"};
        const int dflt[NUM_OPTIONS] = {32, 1, 1, 1, 1};
        for (int k = 0; k < NUM_OPTIONS; ++k) {
            const char* e = getenv(names[k]);
            o.v[k].store(clamp_option(k, (e && *e) ? atoi(e) : dflt[k]));
        }
    });
    return o;
}

static int option(int opt) { return options().v[opt].load(); }

// The bf16 kernels run one workgroup per compute unit, so a launch of `tiles` blocks with the batch in `ns` groups takes
//   rounds(ns) * ceil(units / ns)  unit-times,  rounds = ceil(tiles * ns / 256),
// its workgroups write ns copies of the output (s_bytes each) and the fixed-order reduction reads them back and writes
// the sum, all at ~4 TB/s.
// fold_bytes > 0: every workgroup adds that many bytes to the output in memory after each of its units but the first
// (which stores); the workgroups of a round do so at the same time, and what they move -- read and written back
// across the fabric -- goes at ~5.5 TB/s while they wait (measured: 22 - 29 us for the 67 MB of a 1B-scale layer).
// Returns the cheapest cost over ns <= max_split and the split that reaches it.
static double cheapest_split(int64_t tiles, int64_t units, double t_unit, double s_bytes, int max_split, int64_t* nsplit, int64_t* per,
                             double fold_bytes = 0.0)
{
    double best = 0.0;
    const int64_t lim = units < max_split ? units : max_split;
    for (int64_t ns = 1; ns <= lim; ++ns) {
        const int64_t pu = (units + ns - 1) / ns;
        const int64_t ns_eff = (units + pu - 1) / pu;
        const int64_t rounds = (tiles * ns_eff + 255) / 256;
        double cost = (double)rounds * (double)pu * t_unit;
        if (fold_bytes > 0.0) {
            const int64_t at_once = tiles * ns_eff < 256 ? tiles * ns_eff : 256;
            cost += (double)rounds * (double)(pu - 1) * (2.0 * (double)at_once * fold_bytes / 5.5e12 + 2.0e-6);
        }
        if (ns_eff > 1) cost += (2 * ns_eff + 1) * s_bytes / 4.0e12 + 3.0e-6;
        if (ns == 1 || cost < best) { best = cost; *nsplit = ns_eff; *per = pu; }
    }
    return best;
}

// Sustained rate of one compute unit on the bf16 blocks, FLOP/s (measured on Gaussian operands, 1B-scale layers):
// the larger the block, the fewer bytes go from L2 into LDS and from LDS into registers per FLOP.
// chip-wide rates of the two routes to the per-example norms, FLOP/s (measured)
constexpr double GRAM_RATE = 6.0e14, GRAM_STEP = 0.45e-6, GRAM_WIDE_STEP_FULL = 0.9e-6, GRAM_WIDE_STEP = 0.75e-6, DIRECT_NORM_RATE = 1.3e15;

static double bf16_block_rate(int bm, int bn)
{
    const int area = bm * bn;
    return area >= 256 * 256 ? 5.5e12 : (area >= 256 * 192 ? 4.8e12 : 4.3e12);
}

StatPlan plan_stat(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, Mode mode, bool allow_wide)
{
    StatPlan p{};
    const bool per_example = (mode == MODE_SQUARE || mode == MODE_SIGN || mode == MODE_NORMS || mode == MODE_WEIGHTED || mode == MODE_POWER);
    p.kernel = (dt == PEX_BF16 && bf16_supports(B, T, din, dout)) ? 1 : 0;
    if (dt == PEX_F32 && f32_mfma_supports(B, T, din, dout, mode)) p.kernel = 2;

    // The unit the batch axis is split in: whole examples when phi is applied per example (the sum over
    // the sequence must be complete before phi), slabs of 64 rows of the flattened [B*T] axis otherwise.
    int64_t tiles, target, units;
    int bm = 64, bn = 64;
    if (p.kernel == 1) {
        bf16_tile_shape(mode, B, &bm, &bn);
        target = 256;    // one workgroup per compute unit
    } else if (p.kernel == 2) {
        f32_tile_shape(&bm, &bn);
        target = 768;    // three workgroups of four waves per compute unit, so that loads and MFMAs overlap
    } else {
        target = 1024;   // four small workgroups per compute unit
    }
    tiles = ((din + bm - 1) / bm) * ((dout + bn - 1) / bn);
    const int64_t slab = 64;
    units = per_example ? B : (B * T + slab - 1) / slab;
    const int max_split = option(PEX_OPT_MAX_SPLIT);
    int64_t nsplit = 1, per = units;
    int64_t wide_cols = 0, wide_nsplit = 1, wide_per = units;
    bool sign_bytes = false, mem_fold = false;
    if (p.kernel != 1) {
        nsplit = (target + tiles - 1) / tiles;
        if (nsplit > max_split) nsplit = max_split;
        if (nsplit > units) nsplit = units;
        if (nsplit < 1) nsplit = 1;
        per = (units + nsplit - 1) / nsplit;
    } else {
        // A unit-time is one example (or 64 rows) on one block.
        const double rows_per_unit = per_example ? (double)T : (double)slab;
        const double t_unit = 2.0 * rows_per_unit * bm * bn / bf16_block_rate(bm, bn);
        // (the per-example norms exchange no partial sums of S, only one number per workgroup and example)
        double best = cheapest_split(tiles, units, t_unit, mode == MODE_NORMS ? 0.0 : (double)din * (double)dout * 4.0, max_split, &nsplit, &per);
        // Packed sign counts can be exchanged as bytes while a group holds at most 127 examples: a quarter of the
        // traffic, so more groups pay.  Planned with that cost; kept if the groups it gives are small enough.
        if (mode == MODE_SIGN && bm == 256 && bn == 256) {
            int64_t ns_b = 1, per_b = units;
            const double cost_b = cheapest_split(tiles, units, t_unit, (double)sign_byte_partial_bytes(din, dout), max_split, &ns_b, &per_b);
            if (ns_b > 1 && sign_byte_partials_possible(B, per_b) && cost_b <= best) {
                best = cost_b;
                nsplit = ns_b;
                per = per_b;
                sign_bytes = true;
            }
        }
        // One statistic on two register tiles may put its first columns on the wider block (256 x 192) and only the
        // remaining columns on the 256 x 128 block, each part with a split of the batch of its own.  Candidates: every
        // number of wide block columns up to 64, beyond that the largest number that fits k rounds of 256 workgroups,
        // and all columns wide.
        const int wide_opt = option(PEX_OPT_WIDE_BLOCKS);
        if (allow_wide && wide_opt != 0 && (mode == MODE_SQUARE || mode == MODE_WEIGHTED || mode == MODE_POWER) && bm == 256 && bn == 128) {
            int wm, wn;
            bf16_wide_tile_shape(&wm, &wn);
            const int64_t tiles_m = (din + wm - 1) / wm, max_wide = dout / wn;
            const double t_wide = 2.0 * (double)T * wm * wn / bf16_block_rate(wm, wn);
            auto consider = [&](int64_t na, bool forced) {
                const int64_t rest = dout - na * wn;
                int64_t ns_w = 1, per_w = units, ns_r = 1, per_r = units;
                double cost = cheapest_split(tiles_m * na, units, t_wide, (double)din * (double)(na * wn) * 4.0, max_split, &ns_w, &per_w);
                if (rest > 0)
                    cost += 5.0e-6 + cheapest_split(tiles_m * ((rest + bn - 1) / bn), units, t_unit, (double)din * (double)rest * 4.0, max_split,
                                                    &ns_r, &per_r);
                if (forced || cost < best) {
                    best = cost;
                    wide_cols = na * wn;
                    wide_nsplit = (units + per_w - 1) / per_w;
                    wide_per = per_w;
                    nsplit = ns_r;
                    per = per_r;
                }
            };
            for (int64_t na = 1; na <= max_wide && na <= 64; ++na) consider(na, false);
            for (int64_t k = 1; k <= 64 && max_wide > 64; ++k) {
                const int64_t na = (256 * k) / tiles_m;
                if (na > 64 && na < max_wide) consider(na, false);
            }
            if (max_wide > 64) consider(max_wide, false);
            if (wide_opt == 2 && max_wide >= 1) consider(max_wide, true);      // forced: as many wide block columns as fit
        }
        // ... or keep no second register tile at all: 256 x 256 blocks (eight waves: 5.2e12 FLOP/s per compute unit) that
        // add phi(M_b) to the output in memory at the end of every example
        const int fold_opt = option(PEX_OPT_MEMORY_FOLD);
        if (allow_wide && fold_opt != 0 && (mode == MODE_SQUARE || mode == MODE_WEIGHTED || mode == MODE_POWER) && bm == 256 && bn == 128 &&
            dout < ((int64_t)1 << 20)) {      // 32-bit byte offsets inside a tile of the output
            int fm, fn;
            bf16_tile_shape(MODE_IDENTITY, B, &fm, &fn);
            const int64_t tiles_f = ((din + fm - 1) / fm) * ((dout + fn - 1) / fn);
            int64_t ns_f = 1, per_f = units;
            const double cost = cheapest_split(tiles_f, units, 2.0 * (double)T * fm * fn / 5.2e12, (double)din * (double)dout * 4.0, max_split,
                                               &ns_f, &per_f, (double)fm * fn * 4.0);
            if (fold_opt == 2 || cost < best) {
                best = cost;
                mem_fold = true;
                wide_cols = 0;
                wide_nsplit = 1;
                nsplit = ns_f;
                per = per_f;
            }
        }
    }
    nsplit = (units + per - 1) / per;      // no empty group
    p.nsplit = (int)nsplit;
    p.per_split = per_example ? per : per * slab;
    // Per-token square on the MFMA kernel: squaring the operands inside the kernel (global -> registers -> LDS instead
    // of direct-to-LDS loads, plus the arithmetic) costs about +50 % time; squaring them once into bf16 copies costs one
    // pass over X and G at HBM speed (~5.5 TB/s, 4 bytes moved per element).  The copies win when din*dout/(din+dout)
    // is large.
    p.presq_bytes = 0;
    const int presquare = option(PEX_OPT_TOKEN_PRESQUARE);
    if (mode == MODE_TOKEN_SQ && p.kernel == 1 && presquare != 0) {
        const double elems = (double)B * (double)T * (double)(din + dout);
        const double t_pre = 4.0 * elems / 5.5e12 + 6.0e-6;
        const double t_fused_extra = 0.5 * 2.0 * (double)B * (double)T * (double)din * (double)dout / 1.3e15;
        if (t_pre < t_fused_extra || presquare == 2)
            p.presq_bytes = (((size_t)B * (size_t)T * (size_t)(din + dout) * 2) + 255) & ~(size_t)255;
    }
    p.sign_bytes = sign_bytes && nsplit > 1;
    p.mem_fold = mem_fold;
    p.wide_cols = wide_cols;
    p.wide_nsplit = (int)wide_nsplit;
    p.wide_per_split = wide_per;
    p.wide_ws_bytes = (wide_cols > 0 && wide_nsplit > 1) ? (size_t)wide_nsplit * (size_t)din * (size_t)wide_cols * sizeof(float) : 0;
    p.ws_bytes = p.presq_bytes + p.wide_ws_bytes +
                 ((nsplit > 1 && dout > wide_cols) ? (size_t)nsplit * (size_t)din * (size_t)(dout - wide_cols) * sizeof(float) : 0);
    if (p.sign_bytes) p.ws_bytes = (size_t)nsplit * sign_byte_partial_bytes(din, dout);
    if (mode == MODE_NORMS) {   // no S at all: one partial of ||M_b||^2 per tile (and wave) and example
        p.ws_bytes = (size_t)(p.kernel == 1 ? bf16_norm_partials(din, dout) : generic_norm_partials(din, dout)) * (size_t)B * sizeof(float);
        // Through the Gram matrices instead: 2 T^2 (din + dout) FLOP per example (a little over half of it with the
        // symmetry, in 128 x 128 blocks) against 2 T din dout, on a kernel of lower rate but with one workgroup per block
        // and example -- no batch split, however few tiles the layer has.
        const int gram_opt = option(PEX_OPT_GRAM_NORMS);
        if (dt == PEX_BF16 && gram_opt != 0 && gram_supports(B, T, din, dout)) {
            // Gram kernel: 6.0e14 FLOP/s on a full chip (its 128 x 128 blocks draw twice the bytes per FLOP from L2 that
            // the 256 x 256 blocks of the contraction do), and never faster than its serial loop over the features, one
            // 64-feature step per ~0.45 us (measured with fewer workgroups than compute units).  Contraction: the plan's
            // rounds, plus ~20 us of start-up, epilogue and reduction on small layers.
            const double steps = (double)((din + 63) / 64 + (dout + 63) / 64);
            double t_gram = 2.0 * (double)B * (double)gram_norm_partials(T) * 128.0 * 128.0 * (double)(din + dout) / GRAM_RATE;
            if (t_gram < steps * GRAM_STEP) t_gram = steps * GRAM_STEP;
            t_gram += 6.0e-6;
            double t_direct = 2.0 * (double)B * (double)T * (double)din * (double)dout / DIRECT_NORM_RATE;
            if (p.kernel == 1) {
                const double t_unit = 2.0 * (double)T * bm * bn / bf16_block_rate(bm, bn);
                const double t_rounds = (double)((tiles * p.nsplit + 255) / 256) * (double)((B + p.nsplit - 1) / p.nsplit) * t_unit;
                if (t_rounds > t_direct) t_direct = t_rounds;
            }
            t_direct += 20.0e-6;
            // On 256 x 256 blocks: half the bytes per FLOP; one workgroup per block and example in rounds of 256, each a
            // serial loop of 32-feature steps (measured: ~0.9 us per step on a full chip, ~0.75 us below that), and the
            // parked blocks written and read once (~4 TB/s); while they stay below a quarter of a GiB.
            const size_t park = gram_wide_park_bytes(B, T);
            const double steps_w = (double)((din + 31) / 32 + (dout + 31) / 32);
            const int64_t wgs = B * gram_wide_partials(T);
            double t_wide = (double)((wgs + 255) / 256) * steps_w * (wgs > 256 ? GRAM_WIDE_STEP_FULL : GRAM_WIDE_STEP);
            t_wide += 2.0 * (double)park / 4.0e12 + 8.0e-6;
            const bool wide_ok = park <= ((size_t)256 << 20);
            if (gram_opt == 3 ? wide_ok : (gram_opt == 1 && wide_ok && t_wide < t_gram && t_wide < t_direct)) {
                p.gram = p.gram_wide = true;
                p.ws_bytes = (((size_t)gram_wide_partials(T) * (size_t)B * sizeof(float) + 255) & ~(size_t)255) + park;
            } else if (gram_opt == 2 || gram_opt == 3 || t_gram < t_direct) {
                p.gram = true;
                p.ws_bytes = (size_t)gram_norm_partials(T) * (size_t)B * sizeof(float);
            }
        }
    }
    return p;
}

static pex_status check_stat_args(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout,
                                  pex_dtype dt, const float* S)
{
    if (!X || !G || !S) return PEX_ERR_NULL;
    if (dt != PEX_F32 && dt != PEX_BF16) return PEX_ERR_DTYPE;
    if (B < 1 || T < 1 || din < 1 || dout < 1) return PEX_ERR_SHAPE;
    const int64_t lim = (int64_t)1 << 31;
    if (din >= lim || dout >= lim || B >= lim || T >= lim || B * T >= lim) return PEX_ERR_SHAPE;
    if (((uintptr_t)X | (uintptr_t)G | (uintptr_t)S) & 15u) return PEX_ERR_ALIGN;
    // The fp32 and the SIMT kernels put the tiles of din (128 and 64 rows) in the second grid dimension.
    const StatPlan plan = plan_stat(B, T, din, dout, dt, MODE_IDENTITY);
    if (plan.kernel != 1 && din > 65535 * (int64_t)(plan.kernel == 2 ? 128 : 64)) return PEX_ERR_SHAPE;
    return PEX_OK;
}

static pex_status run_stat(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                           Mode mode, float* S, void* workspace, size_t workspace_bytes, hipStream_t stream,
                           const float* weight = nullptr, float alpha = 0.f)
{
    const StatPlan plan = plan_stat(B, T, din, dout, dt, mode);
    float* out = S;
    if (plan.ws_bytes > 0) {
        if (!workspace || workspace_bytes < plan.ws_bytes) return PEX_ERR_WORKSPACE;
        if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    }
    float* partials = (float*)((char*)workspace + plan.presq_bytes);
    if (plan.nsplit > 1) out = partials;
    hipError_t e;
    if (plan.presq_bytes > 0) {
        // squared copies of X and G at the front of the workspace, then the plain contraction on them
        uint16_t* x2 = (uint16_t*)workspace;
        uint16_t* g2 = x2 + B * T * din;
        e = launch_square_bf16(X, x2, B * T * din, stream);
        if (e == hipSuccess) e = launch_square_bf16(G, g2, B * T * dout, stream);
        if (e == hipSuccess) e = launch_stat_bf16(x2, g2, B, T, din, dout, MODE_IDENTITY, plan, S, partials, stream);
    } else if (plan.kernel == 2) {
        e = launch_stat_f32(X, G, B, T, din, dout, mode, plan, out, stream, weight, alpha);
    } else if (mode == MODE_POWER) {
        e = plan.kernel == 1 ? launch_power_bf16(X, G, alpha, B, T, din, dout, plan, S, partials, stream)
                             : launch_stat_generic(X, G, B, T, din, dout, dt, mode, plan, out, stream, nullptr, nullptr, alpha);
    } else if (mode == MODE_WEIGHTED) {
        e = plan.kernel == 1 ? launch_weighted_bf16(X, G, weight, B, T, din, dout, plan, S, partials, stream)
                             : launch_stat_generic(X, G, B, T, din, dout, dt, mode, plan, out, stream, weight, nullptr);
    } else if (plan.kernel == 1) e = launch_stat_bf16(X, G, B, T, din, dout, mode, plan, S, partials, stream);
    else e = launch_stat_generic(X, G, B, T, din, dout, dt, mode, plan, out, stream);
    if (e != hipSuccess) return PEX_ERR_HIP;
    if (plan.wide_cols > 0) {
        // the wide part's partial sums come first in the workspace, then those of the columns beyond it
        if (plan.wide_nsplit > 1) {
            e = launch_reduce_partials_cols(partials, plan.wide_nsplit, din, plan.wide_cols, S, dout, stream);
            if (e != hipSuccess) return PEX_ERR_HIP;
        }
        if (plan.nsplit > 1 && dout > plan.wide_cols) {
            const float* rest_partials = (const float*)((const char*)partials + plan.wide_ws_bytes);
            e = launch_reduce_partials_cols(rest_partials, plan.nsplit, din, dout - plan.wide_cols, S + plan.wide_cols, dout, stream);
            if (e != hipSuccess) return PEX_ERR_HIP;
        }
    } else if (plan.nsplit > 1) {
        e = plan.sign_bytes ? launch_reduce_sign_bytes(partials, plan.nsplit, din, dout, S, stream)
                            : launch_reduce_partials(partials, plan.nsplit, din * dout, S, stream);
        if (e != hipSuccess) return PEX_ERR_HIP;
    }
    return PEX_OK;
}

// How pex_stat_multi is carried out: `pair` = two or three of the statistics from one MFMA contraction (bf16
// layers), the rest one at a time.
struct MultiPlan {
    bool pair;            // a fused launch is used
    uint32_t pair_want;   // for which statistics
    uint32_t single_want; // served by separate pex_stat passes
    StatPlan pair_plan;
    size_t ws_bytes;
};

static MultiPlan plan_multi(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, uint32_t want)
{
    MultiPlan m{};
    const int n = __builtin_popcount(want);
    const StatPlan sq = plan_stat(B, T, din, dout, dt, MODE_SQUARE, false);
    m.pair = (n >= 2 && sq.kernel == 1);
    if (m.pair) {
        // three wanted: all from one contraction while the sign counts fit bytes; otherwise identity and square
        // share a contraction and sign keeps its own (packed counts, large tile)
        m.pair_want = (n == 3 && !bf16_triple_supported(sq)) ? (PEX_WANT_IDENTITY | PEX_WANT_SQUARE) : want;
        m.single_want = want & ~m.pair_want;
        m.pair_plan = sq;
        m.pair_plan.ws_bytes = sq.nsplit > 1 ? __builtin_popcount(m.pair_want) * sq.ws_bytes : 0;
        m.ws_bytes = m.pair_plan.ws_bytes;
    } else {
        m.single_want = want;
    }
    for (int phi = 0; phi < 3; ++phi)
        if (m.single_want & (1u << phi)) {
            const size_t w = plan_stat(B, T, din, dout, dt, (Mode)phi).ws_bytes;
            if (w > m.ws_bytes) m.ws_bytes = w;     // passes run one after the other on the stream and reuse it
        }
    return m;
}

}  // namespace pex

using namespace pex;

extern "C" {

const char* pex_status_string(pex_status s)
{
    switch (s) {
    case PEX_OK: return "PEX_OK";
    case PEX_ERR_NULL: return "PEX_ERR_NULL: a required pointer is NULL";
    case PEX_ERR_SHAPE: return "PEX_ERR_SHAPE: a dimension is out of range";
    case PEX_ERR_DTYPE: return "PEX_ERR_DTYPE: unknown storage type";
    case PEX_ERR_PHI: return "PEX_ERR_PHI: unknown phi or optimizer variant";
    case PEX_ERR_ALIGN: return "PEX_ERR_ALIGN: a pointer is not 16-byte aligned";
    case PEX_ERR_WORKSPACE: return "PEX_ERR_WORKSPACE: workspace missing or too small";
    case PEX_ERR_HIP: return "PEX_ERR_HIP: the HIP runtime reported an error";
    case PEX_ERR_TOO_LARGE: return "PEX_ERR_TOO_LARGE: the call needs more scratch than the library's static buffer holds";
    }
    return "PEX: unknown status";
}

int pex_version(void) { return 200; }

pex_status pex_set_option(pex_option opt, int32_t value)
{
    if (!known_option(opt)) return PEX_ERR_PHI;
    if (value != clamp_option(opt, value)) return PEX_ERR_SHAPE;
    options().v[opt].store(value);
    return PEX_OK;
}

int32_t pex_get_option(pex_option opt)
{
    if (!known_option(opt)) return -1;
    return option(opt);
}

size_t pex_stat_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, pex_phi phi)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    if (phi != PEX_PHI_IDENTITY && phi != PEX_PHI_SQUARE && phi != PEX_PHI_SIGN) return 0;
    return plan_stat(B, T, din, dout, dt, (Mode)phi).ws_bytes;
}

pex_status pex_stat(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                    pex_phi phi, float* S, void* workspace, size_t workspace_bytes, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, S);
    if (st != PEX_OK) return st;
    if (phi != PEX_PHI_IDENTITY && phi != PEX_PHI_SQUARE && phi != PEX_PHI_SIGN) return PEX_ERR_PHI;
    return run_stat(X, G, B, T, din, dout, dt, (Mode)phi, S, workspace, workspace_bytes, (hipStream_t)stream);
}

pex_status pex_stat_noalloc(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                            pex_phi phi, float* S, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, S);
    if (st != PEX_OK) return st;
    if (phi != PEX_PHI_IDENTITY && phi != PEX_PHI_SQUARE && phi != PEX_PHI_SIGN) return PEX_ERR_PHI;
    const size_t need = plan_stat(B, T, din, dout, dt, (Mode)phi).ws_bytes;
    if (need > (size_t)PEX_NOALLOC_SCRATCH_BYTES) return PEX_ERR_TOO_LARGE;
    void* ws = nullptr;
    if (need > 0 && scratch_address(&ws) != hipSuccess) return PEX_ERR_HIP;
    // Every partial sum the reduction reads is written by the contraction of the same call, so nothing in the
    // scratch has to start at zero.
    return run_stat(X, G, B, T, din, dout, dt, (Mode)phi, S, ws, need, (hipStream_t)stream);
}

size_t pex_stat_multi_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt, uint32_t want)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    if (want == 0 || (want & ~7u)) return 0;
    return plan_multi(B, T, din, dout, dt, want).ws_bytes;
}

pex_status pex_stat_multi(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                          uint32_t want, float* S_id, float* S_sq, float* S_sign, void* workspace,
                          size_t workspace_bytes, pex_stream_t stream)
{
    if (want == 0 || (want & ~7u)) return PEX_ERR_PHI;
    float* outs[3] = {(want & PEX_WANT_IDENTITY) ? S_id : nullptr, (want & PEX_WANT_SQUARE) ? S_sq : nullptr,
                      (want & PEX_WANT_SIGN) ? S_sign : nullptr};
    for (int phi = 0; phi < 3; ++phi) {
        if (!(want & (1u << phi))) continue;
        const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, outs[phi]);
        if (st != PEX_OK) return st;
    }
    const MultiPlan m = plan_multi(B, T, din, dout, dt, want);
    if (m.ws_bytes > 0) {
        if (!workspace || workspace_bytes < m.ws_bytes) return PEX_ERR_WORKSPACE;
        if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    }
    hipStream_t hs = (hipStream_t)stream;
    if (m.pair) {
        const StatPlan& p = m.pair_plan;
        const int64_t n = din * dout;
        float* po[3] = {nullptr, nullptr, nullptr};
        int k = 0;
        for (int phi = 0; phi < 3; ++phi)
            if (m.pair_want & (1u << phi)) po[phi] = p.nsplit > 1 ? (float*)workspace + (int64_t)(k++) * p.nsplit * n : outs[phi];
        const hipError_t e = (__builtin_popcount(m.pair_want) == 3)
                                 ? launch_stat_bf16_triple(X, G, B, T, din, dout, p, po[0], po[1], po[2], hs)
                                 : launch_stat_bf16_pair(X, G, B, T, din, dout, p, po[0], po[1], po[2], hs);
        if (e != hipSuccess) return PEX_ERR_HIP;
        if (p.nsplit > 1)
            for (int phi = 0; phi < 3; ++phi)
                if (po[phi] && launch_reduce_partials(po[phi], p.nsplit, n, outs[phi], hs) != hipSuccess) return PEX_ERR_HIP;
    }
    for (int phi = 0; phi < 3; ++phi) {
        if (!(m.single_want & (1u << phi))) continue;
        const pex_status st = run_stat(X, G, B, T, din, dout, dt, (Mode)phi, outs[phi], workspace, workspace_bytes, hs);
        if (st != PEX_OK) return st;
    }
    return PEX_OK;
}

size_t pex_vec_stat_workspace_bytes(int64_t B, int64_t T, int64_t d, pex_dtype dt)
{
    if (B < 1 || T < 1 || d < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    return plan_vec_stat(B, T, d, dt).ws_bytes;
}

pex_status pex_vec_stat(const void* A, const void* C, int64_t B, int64_t T, int64_t d, pex_dtype dt, uint32_t want,
                        float* s_id, float* s_sq, float* s_sign, void* workspace, size_t workspace_bytes,
                        pex_stream_t stream)
{
    if (!A) return PEX_ERR_NULL;
    if (want == 0 || (want & ~7u)) return PEX_ERR_PHI;
    float* outs[3] = {(want & PEX_WANT_IDENTITY) ? s_id : nullptr, (want & PEX_WANT_SQUARE) ? s_sq : nullptr,
                      (want & PEX_WANT_SIGN) ? s_sign : nullptr};
    for (int phi = 0; phi < 3; ++phi)
        if ((want & (1u << phi)) && !outs[phi]) return PEX_ERR_NULL;
    if (dt != PEX_F32 && dt != PEX_BF16) return PEX_ERR_DTYPE;
    const int64_t lim = (int64_t)1 << 31;
    if (B < 1 || T < 1 || d < 1 || B >= lim || T >= lim || d >= lim || B * T >= lim) return PEX_ERR_SHAPE;
    const uintptr_t esz = dt == PEX_BF16 ? 2 : 4;
    if (((uintptr_t)A | (uintptr_t)C) & (esz - 1)) return PEX_ERR_ALIGN;
    if (((uintptr_t)outs[0] | (uintptr_t)outs[1] | (uintptr_t)outs[2]) & 3u) return PEX_ERR_ALIGN;
    const VecPlan plan = plan_vec_stat(B, T, d, dt);
    if (B * plan.nrange >= 65536) return PEX_ERR_SHAPE;      // grid limit of the second launch dimension
    if (!workspace || workspace_bytes < plan.ws_bytes) return PEX_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    return launch_vec_stat(A, C, B, T, d, dt, plan, (float*)workspace, outs[0], outs[1], outs[2], (hipStream_t)stream) ==
                   hipSuccess
               ? PEX_OK
               : PEX_ERR_HIP;
}

size_t pex_example_norms_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    return plan_stat(B, T, din, dout, dt, MODE_NORMS).ws_bytes;
}

pex_status pex_example_norms(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                             float* N, void* workspace, size_t workspace_bytes, pex_stream_t stream)
{
    pex_status st = check_stat_args(X, G, B, T, din, dout, dt, (const float*)0x10);
    if (st != PEX_OK) return st;
    if (!N) return PEX_ERR_NULL;
    if ((uintptr_t)N & 3u) return PEX_ERR_ALIGN;
    const StatPlan plan = plan_stat(B, T, din, dout, dt, MODE_NORMS);
    if (!workspace || workspace_bytes < plan.ws_bytes) return PEX_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    hipStream_t hs = (hipStream_t)stream;
    float* partial = (float*)workspace;
    hipError_t e;
    int64_t nparts;
    if (plan.gram_wide) {
        nparts = gram_wide_partials(T);
        void* park = (char*)workspace + (((size_t)nparts * (size_t)B * sizeof(float) + 255) & ~(size_t)255);
        e = launch_gram_wide(X, G, B, T, din, dout, partial, park, hs);
    } else if (plan.gram) {
        nparts = gram_norm_partials(T);
        e = launch_gram_norms(X, G, B, T, din, dout, partial, hs);
    } else if (plan.kernel == 1) {
        nparts = bf16_norm_partials(din, dout);
        e = launch_norms_bf16(X, G, B, T, din, dout, plan, partial, hs);
    } else {
        nparts = generic_norm_partials(din, dout);
        e = launch_stat_generic(X, G, B, T, din, dout, dt, MODE_NORMS, plan, nullptr, hs, nullptr, partial);
    }
    if (e != hipSuccess) return PEX_ERR_HIP;
    return launch_reduce_norms(partial, nparts, B, N, hs) == hipSuccess ? PEX_OK : PEX_ERR_HIP;
}

size_t pex_weighted_sum_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    return plan_stat(B, T, din, dout, dt, MODE_WEIGHTED).ws_bytes;
}

pex_status pex_weighted_sum(const void* X, const void* G, const float* w, int64_t B, int64_t T, int64_t din, int64_t dout,
                            pex_dtype dt, float* S, void* workspace, size_t workspace_bytes, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, S);
    if (st != PEX_OK) return st;
    if (!w) return PEX_ERR_NULL;
    if ((uintptr_t)w & 3u) return PEX_ERR_ALIGN;
    return run_stat(X, G, B, T, din, dout, dt, MODE_WEIGHTED, S, workspace, workspace_bytes, (hipStream_t)stream, w);
}

pex_status pex_clip_weights(const float* N, int64_t B, int32_t nlayers, float max_norm, float* w, pex_stream_t stream)
{
    if (!N || !w) return PEX_ERR_NULL;
    if (B < 1 || nlayers < 1 || B >= ((int64_t)1 << 31) || !(max_norm > 0.f)) return PEX_ERR_SHAPE;
    if (((uintptr_t)N | (uintptr_t)w) & 3u) return PEX_ERR_ALIGN;
    return launch_clip_weights(N, B, nlayers, max_norm, w, (hipStream_t)stream) == hipSuccess ? PEX_OK : PEX_ERR_HIP;
}

size_t pex_stat_power_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    return plan_stat(B, T, din, dout, dt, MODE_POWER).ws_bytes;
}

pex_status pex_stat_power(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                          float alpha, float* S, void* workspace, size_t workspace_bytes, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, S);
    if (st != PEX_OK) return st;
    if (!(alpha > 0.f) || !(alpha <= 64.f)) return PEX_ERR_PHI;
    return run_stat(X, G, B, T, din, dout, dt, MODE_POWER, S, workspace, workspace_bytes, (hipStream_t)stream, nullptr, alpha);
}

pex_status pex_token_norms(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                           float* N_tok, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, (const float*)0x10);
    if (st != PEX_OK) return st;
    if (!N_tok) return PEX_ERR_NULL;
    if ((uintptr_t)N_tok & 3u) return PEX_ERR_ALIGN;
    return launch_token_norms(X, G, B * T, din, dout, dt, N_tok, (hipStream_t)stream) == hipSuccess ? PEX_OK : PEX_ERR_HIP;
}

size_t pex_token_sq_workspace_bytes(int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt)
{
    if (B < 1 || T < 1 || din < 1 || dout < 1) return 0;
    if (dt != PEX_F32 && dt != PEX_BF16) return 0;
    return plan_stat(B, T, din, dout, dt, MODE_TOKEN_SQ).ws_bytes;
}

pex_status pex_token_sq(const void* X, const void* G, int64_t B, int64_t T, int64_t din, int64_t dout, pex_dtype dt,
                        float* S_tok, void* workspace, size_t workspace_bytes, pex_stream_t stream)
{
    const pex_status st = check_stat_args(X, G, B, T, din, dout, dt, S_tok);
    if (st != PEX_OK) return st;
    return run_stat(X, G, B, T, din, dout, dt, MODE_TOKEN_SQ, S_tok, workspace, workspace_bytes, (hipStream_t)stream);
}

pex_status pex_adam_update(float* theta, float* m, float* v, const float* S_id, const float* S_sq, int64_t n,
                           pex_adam_variant variant, const pex_adam_params* p, pex_stream_t stream)
{
    if (!theta || !m || !v || !S_id || !p) return PEX_ERR_NULL;
    if (variant != PEX_ADAM && variant != PEX_MICROADAM && variant != PEX_MICROADAM_VAR && variant != PEX_MICROADAM_MSQ)
        return PEX_ERR_PHI;
    if (variant != PEX_ADAM && !S_sq) return PEX_ERR_NULL;
    if (n < 1 || p->step < 1 || p->B < 1) return PEX_ERR_SHAPE;
    if ((variant == PEX_MICROADAM_VAR || variant == PEX_MICROADAM_MSQ) && p->B < 2) return PEX_ERR_SHAPE;
    if (((uintptr_t)theta | (uintptr_t)m | (uintptr_t)v | (uintptr_t)S_id | (uintptr_t)S_sq) & 15u) return PEX_ERR_ALIGN;
    return launch_adam_update(theta, m, v, S_id, S_sq, n, variant, *p, (hipStream_t)stream) == hipSuccess ? PEX_OK
                                                                                                           : PEX_ERR_HIP;
}

size_t pex_embed_stat_workspace_bytes(int64_t B, int64_t T, int64_t V, int64_t d)
{
    const int64_t lim = (int64_t)1 << 31;
    if (B < 1 || T < 1 || V < 1 || d < 1 || B >= lim || T >= lim || B * T >= lim || V >= lim - 1) return 0;
    return embed_workspace(B, T, V, d);
}

pex_status pex_embed_stat(const void* ids, int32_t ids_bytes, const void* G, int64_t B, int64_t T, int64_t V, int64_t d,
                          pex_dtype dt, uint32_t want, float* S_id, float* S_sq, float* S_sign, void* workspace,
                          size_t workspace_bytes, pex_stream_t stream)
{
    if (want == 0 || (want & ~7u)) return PEX_ERR_PHI;
    if (!ids || !G) return PEX_ERR_NULL;
    if ((want & PEX_WANT_IDENTITY) && !S_id) return PEX_ERR_NULL;
    if ((want & PEX_WANT_SQUARE) && !S_sq) return PEX_ERR_NULL;
    if ((want & PEX_WANT_SIGN) && !S_sign) return PEX_ERR_NULL;
    if (dt != PEX_F32 && dt != PEX_BF16) return PEX_ERR_DTYPE;
    if (ids_bytes != 4 && ids_bytes != 8) return PEX_ERR_DTYPE;
    const int64_t lim = (int64_t)1 << 31;
    if (B < 1 || T < 1 || V < 1 || d < 1 || B >= lim || T >= lim || B * T >= lim || V >= lim - 1 || d >= lim) return PEX_ERR_SHAPE;
    uintptr_t al = (uintptr_t)G;
    if (want & PEX_WANT_IDENTITY) al |= (uintptr_t)S_id;
    if (want & PEX_WANT_SQUARE) al |= (uintptr_t)S_sq;
    if (want & PEX_WANT_SIGN) al |= (uintptr_t)S_sign;
    if ((al & 15u) || ((uintptr_t)ids & (uintptr_t)(ids_bytes - 1))) return PEX_ERR_ALIGN;
    if (!workspace || workspace_bytes < embed_workspace(B, T, V, d)) return PEX_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    return launch_embed_stat(ids, ids_bytes, G, B, T, V, d, dt, want, S_id, S_sq, S_sign, workspace, (hipStream_t)stream) == hipSuccess
               ? PEX_OK
               : PEX_ERR_HIP;
}

size_t pex_sum_squares_workspace_bytes(int64_t n) { return n < 1 ? 0 : sum_squares_workspace(n); }

pex_status pex_sum_squares(const float* x, int64_t n, double* acc, int32_t accumulate, void* workspace, size_t workspace_bytes,
                           pex_stream_t stream)
{
    if (!x || !acc) return PEX_ERR_NULL;
    if (n < 1) return PEX_ERR_SHAPE;
    if (((uintptr_t)x & 15u) || ((uintptr_t)acc & 7u)) return PEX_ERR_ALIGN;
    if (!workspace || workspace_bytes < sum_squares_workspace(n)) return PEX_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    return launch_sum_squares(x, n, acc, accumulate, (double*)workspace, (hipStream_t)stream) == hipSuccess ? PEX_OK : PEX_ERR_HIP;
}

pex_status pex_adam_update_clipped(float* theta, float* m, float* v, const float* S_id, const float* S_sq, int64_t n,
                                   pex_adam_variant variant, const pex_adam_params* p, const double* sum_sq, float max_norm,
                                   pex_stream_t stream)
{
    if (!theta || !m || !v || !S_id || !p || !sum_sq) return PEX_ERR_NULL;
    if (variant != PEX_ADAM && variant != PEX_MICROADAM && variant != PEX_MICROADAM_VAR && variant != PEX_MICROADAM_MSQ)
        return PEX_ERR_PHI;
    if (variant != PEX_ADAM && !S_sq) return PEX_ERR_NULL;
    if (n < 1 || p->step < 1 || p->B < 1 || !(max_norm > 0.f)) return PEX_ERR_SHAPE;
    if ((variant == PEX_MICROADAM_VAR || variant == PEX_MICROADAM_MSQ) && p->B < 2) return PEX_ERR_SHAPE;
    if (((uintptr_t)theta | (uintptr_t)m | (uintptr_t)v | (uintptr_t)S_id | (uintptr_t)S_sq) & 15u) return PEX_ERR_ALIGN;
    if ((uintptr_t)sum_sq & 7u) return PEX_ERR_ALIGN;
    return launch_adam_update(theta, m, v, S_id, S_sq, n, variant, *p, (hipStream_t)stream, sum_sq, max_norm) == hipSuccess
               ? PEX_OK
               : PEX_ERR_HIP;
}

size_t pex_mfma_probe_operand_bytes(void) { return probe_operand_bytes(); }
size_t pex_mfma_probe_sink_floats(int32_t workgroups) { return workgroups < 1 ? 0 : probe_sink_floats(workgroups); }

pex_status pex_mfma_probe(const void* operands, int32_t workgroups, int32_t iters, float* sink, double* flop, pex_stream_t stream)
{
    if (!operands || !sink) return PEX_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24)) return PEX_ERR_SHAPE;
    if (((uintptr_t)operands | (uintptr_t)sink) & 15u) return PEX_ERR_ALIGN;
    if (flop) *flop = probe_flop(workgroups, iters);
    return launch_mfma_probe(operands, workgroups, iters, sink, (hipStream_t)stream) == hipSuccess ? PEX_OK : PEX_ERR_HIP;
}

size_t pex_moment_track_workspace_bytes(int64_t n) { return n < 1 ? 0 : moment_track_workspace(n); }

pex_status pex_moment_track(float* ema_adam, float* ema_micro, const float* S_id, const float* S_sq, int64_t n,
                            const pex_moment_params* p, double* sums, void* workspace, size_t workspace_bytes,
                            pex_stream_t stream)
{
    if (!ema_adam || !ema_micro || !S_id || !S_sq || !p || !sums) return PEX_ERR_NULL;
    if (n < 1 || p->step < 1 || p->B < 2) return PEX_ERR_SHAPE;
    if (((uintptr_t)ema_adam | (uintptr_t)ema_micro | (uintptr_t)S_id | (uintptr_t)S_sq) & 15u) return PEX_ERR_ALIGN;
    if ((uintptr_t)sums & 7u) return PEX_ERR_ALIGN;
    if (!workspace || workspace_bytes < moment_track_workspace(n)) return PEX_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15u) return PEX_ERR_ALIGN;
    return launch_moment_track(ema_adam, ema_micro, S_id, S_sq, n, *p, sums, (double*)workspace, (hipStream_t)stream) == hipSuccess
               ? PEX_OK
               : PEX_ERR_HIP;
}

pex_status pex_sign_update(float* theta, float* m, const float* S, int64_t n, pex_sign_variant variant, float lr, float beta,
                           float weight_decay, int32_t B, int32_t debias, int64_t step, pex_stream_t stream)
{
    if (!theta || !m || !S) return PEX_ERR_NULL;
    if (variant != PEX_MICROSIGNSGD && variant != PEX_SIGNSGD && variant != PEX_SIGNEMA) return PEX_ERR_PHI;
    if (n < 1 || B < 1 || step < 1) return PEX_ERR_SHAPE;
    if (((uintptr_t)theta | (uintptr_t)m | (uintptr_t)S) & 15u) return PEX_ERR_ALIGN;
    return launch_sign_update(theta, m, S, n, variant, lr, beta, weight_decay, B, debias, step, (hipStream_t)stream) == hipSuccess
               ? PEX_OK
               : PEX_ERR_HIP;
}

pex_status pex_signsgd_update(float* theta, float* m, const float* S_sign, int64_t n, float lr, float beta,
                              float weight_decay, int32_t B, int32_t debias, int64_t step, pex_stream_t stream)
{
    return pex_sign_update(theta, m, S_sign, n, PEX_MICROSIGNSGD, lr, beta, weight_decay, B, debias, step, stream);
}

}  // extern "C"
