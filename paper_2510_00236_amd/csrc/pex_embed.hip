// pex_embed.hip -- per-example gradient statistics of an embedding table.
//
// A lookup h[b,t,:] = E[ids[b,t],:] is a dense layer applied to one-hot inputs (Sec. 2.3 with X one-hot), so the
// per-example gradient M_b = onehot(ids_b)^T G_b has, in row v, the sum of the cotangents of the positions of example
// b that hold token v; S = sum_b phi(M_b).  Nothing is contracted: the work is a gather of the rows of G grouped by
// (token, example), so the bound is HBM bandwidth -- G read once, every row of S written once (rows of tokens that do
// not occur are written as zeros), plus the ids.
//
// Everything is deterministic (no floating-point atomics):
//   1. a stable least-significant-digit radix sort (8 bits per pass, a counting and a placing launch per pass) of
//      the B*T positions by token id; positions enter in the order p = b*T + t, so inside a token's run
//      they stay ordered by example and then by t; ids outside [0, V) (padding) get the key V and are never consumed;
//   2. row_start[v] = first sorted index whose key is >= v;
//   3. each wave owns 16 consecutive sorted positions and every vocabulary row whose run starts among them: cotangent
//      rows are loaded 16 at a time and added per example, phi is applied whenever the example changes, and the result
//      is added to the row's sums.  Rows with many positions are done by all waves of the workgroup, each on a
//      contiguous run of whole examples, and combined in wave order; rows without positions are zero-filled by
//      further workgroups of the same launch.
#include <type_traits>

#include "pex_internal.h"

namespace pex {
namespace {

constexpr int SORT_MAX_BLOCKS = 64;   // workgroups of the sort; a workgroup's tile is a multiple of 2048 keys

template <typename TId>
__device__ __forceinline__ int load_key(const TId* __restrict__ ids, int p, int V)
{
    const int64_t v = (int64_t)ids[p];
    return (v >= 0 && v < (int64_t)V) ? (int)v : V;
}

// Stable least-significant-digit radix sort, 8 bits per pass.  hist[block * 256 + digit] counts the keys of that
// block's tile *of the pass's input* with that digit (the tiles of a later pass hold other keys than those of the
// first, so every pass counts its own input; the counting is in LDS, where many equal keys cost little).
// A tile is a multiple of 2048 keys: 8 rounds of 256 at a time, their loads issued together.
constexpr int SORT_BATCH = 8;

template <typename TId, bool FIRST>
__global__ __launch_bounds__(256) void sort_hist_kernel(const TId* __restrict__ ids, const int* __restrict__ keys_in, int N, int V,
                                                        int shift, int tile, int* __restrict__ hist)
{
    __shared__ int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * tile + threadIdx.x;
    for (int r0 = 0; r0 < tile; r0 += 256 * SORT_BATCH) {
        int key[SORT_BATCH];
#pragma unroll
        for (int j = 0; j < SORT_BATCH; ++j) {
            const int64_t p = base + r0 + j * 256;
            key[j] = p < N ? (FIRST ? load_key(ids, (int)p, V) : keys_in[p]) : -1;
        }
#pragma unroll
        for (int j = 0; j < SORT_BATCH; ++j)
            if (key[j] >= 0) atomicAdd(&h[(key[j] >> shift) & 255], 1);
    }
    __syncthreads();
    hist[(int64_t)blockIdx.x * 256 + threadIdx.x] = h[threadIdx.x];
}

// One pass.  A key goes to (keys with a smaller digit) + (keys with the same digit in earlier tiles) + (its rank among
// the keys of its tile with the same digit, in tile order): the first two from the counters (every workgroup adds
// them up for itself: at most 64 tiles), the rank from 8 ballots per key.  FIRST reads the keys from the ids and uses
// the position itself as the value.
template <typename TId, bool FIRST>
__global__ __launch_bounds__(256) void sort_scatter_kernel(const TId* __restrict__ ids, const int* __restrict__ keys_in,
                                                           const int* __restrict__ vals_in, int* __restrict__ keys_out,
                                                           int* __restrict__ vals_out, int N, int V, int shift, int tile, int nblocks,
                                                           const int* __restrict__ hist)
{
    __shared__ int base[256];
    __shared__ int wcnt[4][256];
    __shared__ int wtot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    {
        int before = 0, total = 0;   // this digit: in earlier tiles, in all tiles
#pragma unroll 8
        for (int b = 0; b < nblocks; ++b) {
            const int c = hist[b * 256 + tid];
            before += b < (int)blockIdx.x ? c : 0;
            total += c;
        }
        int incl = total;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        int smaller = incl - total;   // keys with a smaller digit
        for (int w = 0; w < wave; ++w) smaller += wtot[w];
        base[tid] = smaller + before;
    }
#pragma unroll
    for (int w = 0; w < 4; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    for (int r0 = 0; r0 < tile; r0 += 256 * SORT_BATCH) {
        int keyb[SORT_BATCH], valb[SORT_BATCH];
#pragma unroll
        for (int j = 0; j < SORT_BATCH; ++j) {
            const int64_t idx = (int64_t)blockIdx.x * tile + r0 + j * 256 + tid;
            keyb[j] = -1;
            valb[j] = 0;
            if (idx < N) {
                keyb[j] = FIRST ? load_key(ids, (int)idx, V) : keys_in[idx];
                valb[j] = FIRST ? (int)idx : vals_in[idx];
                if (keyb[j] < 0) keyb[j] = V;   // keys are in [0, V]
            }
        }
#pragma unroll
        for (int j = 0; j < SORT_BATCH; ++j) {
            const bool active = keyb[j] >= 0;
            const int key = keyb[j], val = valb[j];
            const int dg = (key >> shift) & 255;
            // lanes of this wave that are active and hold the same digit
            unsigned long long same = __ballot(active);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (dg >> bit) & 1;
                const unsigned long long bb = __ballot(one);
                same &= one ? bb : ~bb;
            }
            const int rank = __popcll(same & ((1ull << lane) - 1ull));
            if (active && rank == 0) wcnt[wave][dg] = __popcll(same);
            __syncthreads();
            if (active) {
                int dest = base[dg] + rank;
                for (int w = 0; w < wave; ++w) dest += wcnt[w][dg];
                if (dest >= 0 && dest < N) {   // always true when the counts are those of this very input
                    keys_out[dest] = key;
                    vals_out[dest] = val;
                }
            }
            __syncthreads();
            base[tid] += (wcnt[0][tid] + wcnt[1][tid]) + (wcnt[2][tid] + wcnt[3][tid]);
#pragma unroll
            for (int w = 0; w < 4; ++w) wcnt[w][tid] = 0;
            __syncthreads();
        }
    }
}

// row_start[v] = first index k of the sorted keys with key[k] >= v, for v = 0 .. V (N if there is none).  Thread k
// writes the entries between its left neighbour's key and its own, so every entry is written exactly once.
__global__ __launch_bounds__(256) void row_start_kernel(const int* __restrict__ keys, int N, int V, int* __restrict__ row_start)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k > N) return;
    int prev = k == 0 ? -1 : keys[k - 1];
    int cur = k == N ? V : keys[k];
    prev = prev < -1 ? -1 : (prev > V ? V : prev);   // keys are in [0, V]; the clamps keep the writes inside the array regardless
    cur = cur > V ? V : cur;
    for (int v = prev + 1; v <= cur; ++v) row_start[v] = (int)k;
}

__device__ __forceinline__ float widen_el(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float widen_el(float f) { return f; }

// What a lane loads from a cotangent row: CH elements (4 fp32 = 16 bytes, 4 bf16 = 8 bytes, or one element), kept as
// loaded until it is added: widening bf16 early would double the registers a lane holds in flight.  Four columns per
// lane make the fp32 stores of a wave dense (16 bytes per lane, 1 KiB per instruction); eight bf16 columns per lane
// would leave every store instruction writing half of each 32 bytes.
template <typename TIn, int CH>
struct Chunk {
    typedef __attribute__((ext_vector_type(4))) unsigned int u4;
    typedef __attribute__((ext_vector_type(2))) unsigned int u2;
    typedef typename std::conditional<CH == 1, TIn, typename std::conditional<sizeof(TIn) == 2, u2, u4>::type>::type Raw;
    static_assert(CH == 1 || CH == 4, "one element or four");
    static __device__ __forceinline__ Raw zero()
    {
        if constexpr (CH == 1) return (TIn)0;
        else if constexpr (sizeof(TIn) == 2) return u2{0u, 0u};
        else return u4{0u, 0u, 0u, 0u};
    }
    static __device__ __forceinline__ Raw load(const TIn* p)
    {
        if constexpr (CH == 1) return p[0];
        else return *(const Raw*)p;
    }
    static __device__ __forceinline__ void add_to(float (&acc)[CH], const Raw& raw)
    {
        if constexpr (CH == 1) acc[0] += widen_el(raw);
        else if constexpr (sizeof(TIn) == 2) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                acc[2 * e] += __uint_as_float(raw[e] << 16);
                acc[2 * e + 1] += __uint_as_float(raw[e] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += __uint_as_float(raw[e]);
        }
    }
};

template <int CH>
__device__ __forceinline__ void store_chunk(float* p, const float (&v)[CH])
{
    if constexpr (CH == 1) p[0] = v[0];
    else {
#pragma unroll
        for (int e = 0; e < CH; e += 4) *(float4*)(p + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
    }
}

constexpr int EMB_WAVES = 16;    // waves of a workgroup
constexpr int EMB_ZROWS = 8;     // vocabulary rows a zero-fill wave looks at
constexpr int EMB_U = 16;        // sorted positions a wave owns = cotangent rows a lane keeps in flight
constexpr int EMB_ALONE = 64;    // a vocabulary row with at most this many positions is done by one wave

template <int CH>
struct RowSums {
    float id[CH], sq[CH], sg[CH];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int e = 0; e < CH; ++e) id[e] = sq[e] = sg[e] = 0.f;
    }
};

// first index in [lo, hi) whose position is >= limit (positions ascend inside a row's run); the whole wave calls it
// with the same arguments and looks at 64 positions per step -- an example rarely holds more of one token than that
__device__ __forceinline__ int first_at_least(const int* __restrict__ pos, int lo, int hi, int limit)
{
    const int lane = threadIdx.x & 63;
    while (lo < hi) {
        const int k = lo + lane;
        const bool hit = k >= hi || pos[k] >= limit;
        const unsigned long long m = __ballot(hit);
        if (m) {
            const int r = lo + (int)__builtin_ctzll(m);
            return r < hi ? r : hi;
        }
        lo += 64;
    }
    return hi;
}

// Accumulates the cotangent rows of one vocabulary row, example by example: acc holds the running sum of the current
// example, phi(acc) goes to the row's sums when the example changes.
template <typename TIn, int CH, int WANT>
struct RowAccumulator {
    RowSums<CH> sums;
    float acc[CH];
    int limit;     // first position of the next example
    bool open;     // acc holds something
    int T;
    __device__ __forceinline__ void start(int T_)
    {
        T = T_;
        sums.clear();
#pragma unroll
        for (int e = 0; e < CH; ++e) acc[e] = 0.f;
        limit = 0;
        open = false;
    }
    __device__ __forceinline__ void fold()
    {
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            if (WANT & 1) sums.id[e] += acc[e];
            if (WANT & 2) sums.sq[e] = fmaf(acc[e], acc[e], sums.sq[e]);
            if (WANT & 4) sums.sg[e] += (float)((acc[e] > 0.f) - (acc[e] < 0.f));
            acc[e] = 0.f;
        }
    }
    // p is uniform over the wave
    __device__ __forceinline__ void add(int p, const typename Chunk<TIn, CH>::Raw& raw)
    {
        if (p >= limit) {
            if (open) fold();
            open = true;
            limit = (p / T + 1) * T;
        }
        Chunk<TIn, CH>::add_to(acc, raw);
    }
    __device__ __forceinline__ void finish()
    {
        if (open) fold();
        open = false;
        limit = 0;
    }
};

// WANT: bit 0 identity, bit 1 square, bit 2 sign.
// grid.x = chunk workgroups, then zero-fill workgroups; grid.y = blocks of 64 * CH columns.
//   chunk workgroup: wave i owns the sorted positions [c0, c0 + EMB_U) and with them every vocabulary row whose run
//     starts there (a run may continue past the chunk).  It loads EMB_U cotangent rows at a time whatever rows and
//     examples they belong to, then adds them in order.  Runs longer than EMB_ALONE are only noted; after a barrier
//     the whole workgroup does each of them, every wave on a contiguous run of whole examples, combined in wave order.
//   zero-fill workgroup: wave i looks at EMB_ZROWS vocabulary rows and writes zeros to those without positions.
template <typename TIn, int CH, int WANT>
__global__ __launch_bounds__(EMB_WAVES * 64) void embed_rows_kernel(const TIn* __restrict__ G, const int* __restrict__ row_start,
                                                                    const int* __restrict__ keys, const int* __restrict__ pos,
                                                                    int N, int V, int T, int64_t d, int chunk_groups,
                                                                    float* __restrict__ partial, float* __restrict__ S_id,
                                                                    float* __restrict__ S_sq, float* __restrict__ S_sg)
{
    typedef Chunk<TIn, CH> Ck;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t col = ((int64_t)blockIdx.y * 64 + lane) * CH;
    const bool col_ok = col < d;
    auto store_row = [&](int v, const RowSums<CH>& sums) {
        if (!col_ok) return;
        const int64_t o = (int64_t)v * d + col;
        if (WANT & 1) store_chunk<CH>(S_id + o, sums.id);
        if (WANT & 2) store_chunk<CH>(S_sq + o, sums.sq);
        if (WANT & 4) store_chunk<CH>(S_sg + o, sums.sg);
    };

    if ((int)blockIdx.x >= chunk_groups) {
        // whole rows, all column blocks by the same wave: an empty row is one contiguous run of d floats, and empty
        // rows are often neighbours
        if (blockIdx.y != 0) return;
        const int v = (((int)blockIdx.x - chunk_groups) * EMB_WAVES + wave) * EMB_ZROWS + lane;
        const bool empty = lane < EMB_ZROWS && v < V && row_start[v] == row_start[v + 1];
        unsigned long long todo = __ballot(empty);
        RowSums<CH> zeros;
        zeros.clear();
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int64_t o = (int64_t)(v - lane + l) * d;
            for (int64_t c = (int64_t)lane * CH; c < d; c += 64 * CH) {
                if (WANT & 1) store_chunk<CH>(S_id + o + c, zeros.id);
                if (WANT & 2) store_chunk<CH>(S_sq + o + c, zeros.sq);
                if (WANT & 4) store_chunk<CH>(S_sg + o + c, zeros.sg);
            }
        }
        return;
    }

    __shared__ int heavy_row[EMB_WAVES];   // the long run that starts among wave i's positions, or -1
    __shared__ float comb[3][64 * CH];
    if (lane == 0) heavy_row[wave] = -1;

    RowAccumulator<TIn, CH, WANT> ra;
    ra.start(T);
    {
        const int64_t c0l = ((int64_t)blockIdx.x * EMB_WAVES + wave) * EMB_U;
        const int c0 = c0l < N ? (int)c0l : N;
        const int c1 = c0 + EMB_U < N ? c0 + EMB_U : N;
        int k0 = c0;
        int cur_v = -1;      // the row being accumulated
        int open_end = 0;    // where its run ends
        while (k0 < (c1 > open_end ? c1 : open_end)) {
            // lane u < EMB_U looks up position k0 + u: its token, the extent of the token's run, whether the run is ours
            const int k = k0 + lane;
            const bool valid = lane < EMB_U && k < N;
            int key = V, p = -1, rs = 0, re = 0;
            if (valid) { key = keys[k]; p = pos[k]; }
            key = key < 0 ? V : (key > V ? V : key);
            if (valid && key < V) { rs = row_start[key]; re = row_start[key + 1]; }
            re = re > N ? N : re;
            const bool ours = valid && key < V && rs >= c0 && rs < c1;
            const bool is_heavy = re - rs > EMB_ALONE;
            if (ours && is_heavy && k == rs) heavy_row[wave] = key;   // at most one such run can start among EMB_U positions
            const int p_ld = (ours && !is_heavy && p >= 0 && p < N) ? p : -1;
            int pu[EMB_U], ku[EMB_U], eu[EMB_U];
            typename Ck::Raw data[EMB_U];
#pragma unroll
            for (int u = 0; u < EMB_U; ++u) {
                pu[u] = __builtin_amdgcn_readlane(p_ld, u);
                ku[u] = __builtin_amdgcn_readlane(key, u);
                eu[u] = __builtin_amdgcn_readlane(re, u);
            }
#pragma unroll
            for (int u = 0; u < EMB_U; ++u) data[u] = (pu[u] >= 0 && col_ok) ? Ck::load(G + (int64_t)pu[u] * d + col) : Ck::zero();
#pragma unroll
            for (int u = 0; u < EMB_U; ++u) {
                if (pu[u] < 0) continue;
                if (ku[u] != cur_v) {
                    if (cur_v >= 0) { ra.finish(); store_row(cur_v, ra.sums); ra.sums.clear(); }
                    cur_v = ku[u];
                    open_end = eu[u];
                }
                ra.add(pu[u], data[u]);
            }
            // the last position of the batch decides where the next batch starts: inside a run that is loaded the next
            // batch follows on; a run that is not (another wave's, or a long one) is skipped to its end
            const int last_ld = pu[EMB_U - 1], last_end = eu[EMB_U - 1];
            const int next = k0 + EMB_U;
            k0 = (last_ld >= 0 || last_end < next) ? next : last_end;
        }
        if (cur_v >= 0) { ra.finish(); store_row(cur_v, ra.sums); }
    }
    __syncthreads();
    // Long runs: this workgroup does, of every long run that overlaps its EMB_WAVES * EMB_U positions [sc0, sc1), the
    // examples that start there -- candidate -1 is the run that continues from the positions before sc0, candidate i the
    // run that starts among wave i's positions.  A run that lies inside [sc0, sc1) is finished here; of any other the
    // sums go to `partial` (slot 0: continues from before, slot 1: starts here and goes on) for embed_combine_kernel.
    const int64_t sc0l = (int64_t)blockIdx.x * (EMB_WAVES * EMB_U);
    const int sc0 = sc0l < N ? (int)sc0l : N;
    const int sc1 = sc0 + EMB_WAVES * EMB_U < N ? sc0 + EMB_WAVES * EMB_U : N;
    for (int c = -1; c < EMB_WAVES; ++c) {
        int hv = -1;
        if (c >= 0) hv = heavy_row[c];
        else if (sc0 > 0 && sc0 < N) {
            const int key = keys[sc0];
            if (key >= 0 && key < V && row_start[key] < sc0 && row_start[key + 1] - row_start[key] > EMB_ALONE) hv = key;
        }
        if (hv < 0 || hv >= V) continue;   // the same for every wave of the workgroup
        int hs = row_start[hv], he = row_start[hv + 1];
        hs = hs < 0 ? 0 : (hs > N ? N : hs);
        he = he < hs ? hs : (he > N ? N : he);
        // first position at or after k (hs < k < he) that begins an example
        auto example_start = [&](int k) {
            const int limit = (pos[k - 1] / T + 1) * T;
            return first_at_least(pos, k, he, limit);
        };
        const bool from_before = hs < sc0, goes_on = he > sc1;
        const int plo = from_before ? example_start(sc0) : hs;
        const int phi = goes_on ? example_start(sc1) : he;
        // wave i takes the examples that start in [bound(i), bound(i + 1)): an even split of the positions, moved
        // forward to the next change of example
        auto bound = [&](int i) {
            if (i <= 0 || phi <= plo) return plo;
            if (i >= EMB_WAVES) return phi;
            const int k = plo + (int)(((int64_t)(phi - plo) * i) / EMB_WAVES);
            if (k <= plo) return plo;
            const int b2 = example_start(k);
            return b2 < phi ? b2 : phi;
        };
        const int lo = bound(wave), hi = bound(wave + 1);
        ra.start(T);
        for (int k0 = lo; k0 < hi; k0 += EMB_U) {
            int pp[EMB_U];
            typename Ck::Raw data[EMB_U];
#pragma unroll
            for (int u = 0; u < EMB_U; ++u) {
                pp[u] = (k0 + u < hi) ? pos[k0 + u] : -1;
                if (pp[u] >= N) pp[u] = -1;   // positions are in [0, N)
            }
#pragma unroll
            for (int u = 0; u < EMB_U; ++u) data[u] = (pp[u] >= 0 && col_ok) ? Ck::load(G + (int64_t)pp[u] * d + col) : Ck::zero();
#pragma unroll
            for (int u = 0; u < EMB_U; ++u)
                if (pp[u] >= 0) ra.add(pp[u], data[u]);
        }
        ra.finish();
        for (int i = 0; i < EMB_WAVES; ++i) {
            if (wave == i) {
#pragma unroll
                for (int e2 = 0; e2 < CH; ++e2) {
                    const int o = lane * CH + e2;
                    if (i == 0) { comb[0][o] = ra.sums.id[e2]; comb[1][o] = ra.sums.sq[e2]; comb[2][o] = ra.sums.sg[e2]; }
                    else { comb[0][o] += ra.sums.id[e2]; comb[1][o] += ra.sums.sq[e2]; comb[2][o] += ra.sums.sg[e2]; }
                }
            }
            __syncthreads();
        }
        if (wave == 0) {
#pragma unroll
            for (int e2 = 0; e2 < CH; ++e2) {
                const int o = lane * CH + e2;
                ra.sums.id[e2] = comb[0][o]; ra.sums.sq[e2] = comb[1][o]; ra.sums.sg[e2] = comb[2][o];
            }
            if (!from_before && !goes_on) store_row(hv, ra.sums);
            else if (col_ok) {
                float* pr = partial + (((int64_t)blockIdx.x * 2 + (from_before ? 0 : 1)) * 3) * d + col;
                if (WANT & 1) store_chunk<CH>(pr, ra.sums.id);
                if (WANT & 2) store_chunk<CH>(pr + d, ra.sums.sq);
                if (WANT & 4) store_chunk<CH>(pr + 2 * d, ra.sums.sg);
            }
        }
        __syncthreads();
    }
}

// Finishes the long runs that span several workgroups of embed_rows_kernel: the workgroup-sized slice s in which such a
// run starts adds up the partial sums of the slices the run covers, in slice order, and stores the row.
// grid = (slices, column blocks), one wave each.
template <int CH, int WANT>
__global__ __launch_bounds__(64) void embed_combine_kernel(const int* __restrict__ row_start, const int* __restrict__ keys, int N, int V,
                                                           int64_t d, const float* __restrict__ partial, float* __restrict__ S_id,
                                                           float* __restrict__ S_sq, float* __restrict__ S_sg)
{
    constexpr int SLICE = EMB_WAVES * EMB_U;
    const int64_t sc0 = (int64_t)blockIdx.x * SLICE, sc1 = sc0 + SLICE;
    if (sc1 >= N) return;   // nothing goes on past the last slice
    const int key = keys[sc1 - 1];
    if (key < 0 || key >= V) return;
    const int rs = row_start[key], re = row_start[key + 1];
    if (!(rs >= sc0 && re > sc1 && re <= N && re - rs > EMB_ALONE)) return;
    const int64_t col = ((int64_t)blockIdx.y * 64 + threadIdx.x) * CH;
    if (col >= d) return;
    float sum[3][CH];
    auto take = [&](int64_t slice, int slot, bool first) {
        const float* pr = partial + ((slice * 2 + slot) * 3) * d + col;
#pragma unroll
        for (int o = 0; o < 3; ++o) {
            if (!(WANT & (1 << o))) continue;
#pragma unroll
            for (int e = 0; e < CH; ++e) sum[o][e] = first ? pr[o * d + e] : sum[o][e] + pr[o * d + e];
        }
    };
    take(blockIdx.x, 1, true);
    for (int64_t sl = (int64_t)blockIdx.x + 1; sl * SLICE < re; ++sl) take(sl, 0, false);
    const int64_t o = (int64_t)key * d + col;
    if (WANT & 1) store_chunk<CH>(S_id + o, sum[0]);
    if (WANT & 2) store_chunk<CH>(S_sq + o, sum[1]);
    if (WANT & 4) store_chunk<CH>(S_sg + o, sum[2]);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct EmbedLayout {
    int passes, tile, nblocks;
    size_t hist, keys_a, vals_a, keys_b, vals_b, row_start, partial, total;   // byte offsets into the workspace
};

EmbedLayout embed_layout(int64_t N, int64_t V, int64_t d)
{
    EmbedLayout L;
    int bits = 0;
    while (((int64_t)1 << bits) <= V) ++bits;   // the largest key is V
    L.passes = (bits + 7) / 8;
    if (L.passes < 1) L.passes = 1;
    int64_t tile = (N + SORT_MAX_BLOCKS - 1) / SORT_MAX_BLOCKS;
    tile = (tile + 2047) / 2048 * 2048;
    L.tile = (int)tile;
    L.nblocks = (int)((N + tile - 1) / tile);
    size_t o = 0;
    L.hist = o; o += align256((size_t)256 * L.nblocks * sizeof(int));
    L.keys_a = o; o += align256((size_t)N * sizeof(int));
    L.vals_a = o; o += align256((size_t)N * sizeof(int));
    L.keys_b = o; o += align256((size_t)N * sizeof(int));
    L.vals_b = o; o += align256((size_t)N * sizeof(int));
    L.row_start = o; o += align256((size_t)(V + 2) * sizeof(int));
    // two partial sums of three statistics per slice of EMB_WAVES * EMB_U positions, for runs that cross slices
    const int64_t slices = (N + EMB_WAVES * EMB_U - 1) / (EMB_WAVES * EMB_U);
    L.partial = o; o += align256((size_t)slices * 2 * 3 * d * sizeof(float));
    L.total = o;
    return L;
}

template <typename TId>
hipError_t sort_positions(const TId* ids, int N, int V, const EmbedLayout& L, char* ws, const int** keys, const int** vals,
                          hipStream_t stream)
{
    int* hist = (int*)(ws + L.hist);
    int* ka = (int*)(ws + L.keys_a);
    int* va = (int*)(ws + L.vals_a);
    int* kb = (int*)(ws + L.keys_b);
    int* vb = (int*)(ws + L.vals_b);
    const dim3 grid(L.nblocks), block(256);
    const int* kin = nullptr;
    const int* vin = nullptr;
    int* kout = ka;
    int* vout = va;
    for (int ps = 0; ps < L.passes; ++ps) {
        if (ps == 0) {
            sort_hist_kernel<TId, true><<<grid, block, 0, stream>>>(ids, nullptr, N, V, 0, L.tile, hist);
            sort_scatter_kernel<TId, true><<<grid, block, 0, stream>>>(ids, nullptr, nullptr, kout, vout, N, V, 0, L.tile, L.nblocks, hist);
        } else {
            sort_hist_kernel<TId, false><<<grid, block, 0, stream>>>(ids, kin, N, V, 8 * ps, L.tile, hist);
            sort_scatter_kernel<TId, false><<<grid, block, 0, stream>>>(ids, kin, vin, kout, vout, N, V, 8 * ps, L.tile, L.nblocks, hist);
        }
        kin = kout; vin = vout;
        kout = (kout == ka) ? kb : ka;
        vout = (vout == va) ? vb : va;
    }
    *keys = kin;
    *vals = vin;
    return hipGetLastError();
}

template <typename TIn, int CH, int WANT>
hipError_t launch_rows(const TIn* G, const int* row_start, const int* keys, const int* pos, int N, int V, int T, int64_t d,
                       float* partial, float* S_id, float* S_sq, float* S_sg, hipStream_t stream)
{
    const int64_t per_group = (int64_t)EMB_WAVES * EMB_U;
    const int chunk_groups = (int)((N + per_group - 1) / per_group);
    const int zero_groups = (int)(((int64_t)V + EMB_WAVES * EMB_ZROWS - 1) / (EMB_WAVES * EMB_ZROWS));
    const unsigned colblocks = (unsigned)((d + 64 * CH - 1) / (64 * CH));
    embed_rows_kernel<TIn, CH, WANT><<<dim3((unsigned)(chunk_groups + zero_groups), colblocks), dim3(EMB_WAVES * 64), 0, stream>>>(
        G, row_start, keys, pos, N, V, T, d, chunk_groups, partial, S_id, S_sq, S_sg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    embed_combine_kernel<CH, WANT><<<dim3((unsigned)chunk_groups, colblocks), dim3(64), 0, stream>>>(row_start, keys, N, V, d, partial,
                                                                                                   S_id, S_sq, S_sg);
    return hipGetLastError();
}

template <typename TIn, int CH>
hipError_t launch_rows_want(uint32_t want, const TIn* G, const int* rs, const int* keys, const int* pos, int N, int V, int T, int64_t d, float* pr, float* a,
                            float* q, float* g, hipStream_t st)
{
    switch (want) {
    case 1: return launch_rows<TIn, CH, 1>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    case 2: return launch_rows<TIn, CH, 2>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    case 3: return launch_rows<TIn, CH, 3>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    case 4: return launch_rows<TIn, CH, 4>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    case 5: return launch_rows<TIn, CH, 5>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    case 6: return launch_rows<TIn, CH, 6>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    default: return launch_rows<TIn, CH, 7>(G, rs, keys, pos, N, V, T, d, pr, a, q, g, st);
    }
}

}  // namespace

size_t embed_workspace(int64_t B, int64_t T, int64_t V, int64_t d) { return embed_layout(B * T, V, d).total; }

hipError_t launch_embed_stat(const void* ids, int ids_bytes, const void* G, int64_t B, int64_t T, int64_t V, int64_t d,
                             pex_dtype dt, uint32_t want, float* S_id, float* S_sq, float* S_sign, void* workspace,
                             hipStream_t stream)
{
    const int N = (int)(B * T);
    const EmbedLayout L = embed_layout(N, V, d);
    char* ws = (char*)workspace;
    const int* keys = nullptr;
    const int* pos = nullptr;
    hipError_t e = ids_bytes == 8 ? sort_positions<int64_t>((const int64_t*)ids, N, (int)V, L, ws, &keys, &pos, stream)
                                  : sort_positions<int32_t>((const int32_t*)ids, N, (int)V, L, ws, &keys, &pos, stream);
    if (e != hipSuccess) return e;
    int* row_start = (int*)(ws + L.row_start);
    float* partial = (float*)(ws + L.partial);
    row_start_kernel<<<dim3((unsigned)(((int64_t)N + 1 + 255) / 256)), dim3(256), 0, stream>>>(keys, N, (int)V, row_start);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dt == PEX_BF16) {
        if (d % 4 == 0) return launch_rows_want<uint16_t, 4>(want, (const uint16_t*)G, row_start, keys, pos, N, (int)V, (int)T, d, partial, S_id, S_sq, S_sign, stream);
        return launch_rows_want<uint16_t, 1>(want, (const uint16_t*)G, row_start, keys, pos, N, (int)V, (int)T, d, partial, S_id, S_sq, S_sign, stream);
    }
    if (d % 4 == 0) return launch_rows_want<float, 4>(want, (const float*)G, row_start, keys, pos, N, (int)V, (int)T, d, partial, S_id, S_sq, S_sign, stream);
    return launch_rows_want<float, 1>(want, (const float*)G, row_start, keys, pos, N, (int)V, (int)T, d, partial, S_id, S_sq, S_sign, stream);
}

}  // namespace pex
