// pex_embed.hip -- per-example gradient statistics of an embedding table.
//
// A lookup h[b,t,:] = E[ids[b,t],:] is a dense layer applied to one-hot inputs (Sec. 2.3 with X one-hot), so the
// per-example gradient M_b = onehot(ids_b)^T G_b has, in row v, the sum of the cotangents of the positions of example
// b that hold token v; S = sum_b phi(M_b).  Nothing is contracted: the work is a gather of the rows of G grouped by
// (token, example), so the bound is HBM bandwidth -- G read once, every row of S written once (rows of tokens that do
// not occur are written as zeros), plus the ids.
//
// Everything is deterministic (no floating-point atomics):
//   1. a stable least-significant-digit radix sort (8 bits per pass) of the B*T positions by token id; positions
//      enter in the order p = b*T + t, so inside a token's run they stay ordered by example and then by t;
//      ids outside [0, V) (padding) get the key V and are never consumed;
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

constexpr int SORT_TILE = 2048;   // keys per workgroup of the sort: 256 threads x 8 rounds

template <typename TId>
__device__ __forceinline__ int load_key(const TId* __restrict__ ids, int p, int V)
{
    const int64_t v = (int64_t)ids[p];
    return (v >= 0 && v < (int64_t)V) ? (int)v : V;
}

// hist[digit * nblocks + block] = number of keys of this block's tile of the pass's input whose digit (bits shift ..
// shift+7) has that value.  The tiles of a later pass hold other keys than those of the first, so every pass counts
// its own input.
template <typename TId, bool FIRST>
__global__ __launch_bounds__(256) void sort_hist_kernel(const TId* __restrict__ ids, const int* __restrict__ keys_in, int N, int V,
                                                        int shift, int nblocks, int* __restrict__ hist)
{
    __shared__ int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_TILE / 256; ++r) {
        const int64_t p = base + r * 256 + threadIdx.x;
        if (p < N) {
            const int key = FIRST ? load_key(ids, (int)p, V) : keys_in[p];
            atomicAdd(&h[(key >> shift) & 255], 1);
        }
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// exclusive prefix sum, in place, of the `entries` counters (digit-major, block-minor: the order in which a stable
// sort lays the keys out); one workgroup walks the array in tiles of 4096 counters, four per thread
__global__ __launch_bounds__(1024) void sort_scan_kernel(int* __restrict__ h, int64_t entries)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __shared__ int wsum[2][16];
    int carry = 0;
    int par = 0;
    int nxt[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) nxt[e] = ((int64_t)threadIdx.x * 4 + e < entries) ? h[(int64_t)threadIdx.x * 4 + e] : 0;
    for (int64_t t0 = 0; t0 < entries; t0 += 4096, par ^= 1) {
        const int64_t i0 = t0 + (int64_t)threadIdx.x * 4;
        int v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = nxt[e];
            nxt[e] = (i0 + 4096 + e < entries) ? h[i0 + 4096 + e] : 0;   // the next tile's counters, in flight during this tile
        }
        const int s = (v[0] + v[1]) + (v[2] + v[3]);
        int incl = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wsum[par][wave] = incl;
        __syncthreads();   // the other half of wsum is still being read by slower waves of the previous tile
        int run = carry + incl - s, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int t = wsum[par][w];
            if (w < wave) run += t;
            total += t;
        }
        carry += total;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (i0 + e < entries) h[i0 + e] = run;
            run += v[e];
        }
    }
}

// One pass: key/value pairs go to offs[digit][block] + (rank of the pair among the pairs of its tile with the same
// digit, in tile order).  FIRST reads the keys from the ids and uses the position itself as the value.
template <typename TId, bool FIRST>
__global__ __launch_bounds__(256) void sort_scatter_kernel(const TId* __restrict__ ids, const int* __restrict__ keys_in,
                                                           const int* __restrict__ vals_in, int* __restrict__ keys_out,
                                                           int* __restrict__ vals_out, int N, int V, int shift, int nblocks,
                                                           const int* __restrict__ offs)
{
    __shared__ int base[256];
    __shared__ int wcnt[4][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    base[tid] = offs[(int64_t)tid * nblocks + blockIdx.x];
#pragma unroll
    for (int w = 0; w < 4; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    for (int r = 0; r < SORT_TILE / 256; ++r) {
        const int64_t idx = (int64_t)blockIdx.x * SORT_TILE + r * 256 + tid;
        const bool active = idx < N;
        int key = 0, val = 0;
        if (active) {
            key = FIRST ? load_key(ids, (int)idx, V) : keys_in[idx];
            val = FIRST ? (int)idx : vals_in[idx];
        }
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

// first index in [lo, hi) whose position is >= limit (positions ascend inside a row's run)
__device__ __forceinline__ int first_at_least(const int* __restrict__ pos, int lo, int hi, int limit)
{
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (pos[mid] < limit) lo = mid + 1;
        else hi = mid;
    }
    return lo;
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
                                                                    float* __restrict__ S_id, float* __restrict__ S_sq,
                                                                    float* __restrict__ S_sg)
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

    __shared__ int n_heavy;
    __shared__ int heavy_row[EMB_WAVES];
    __shared__ float comb[3][64 * CH];
    if (threadIdx.x == 0) n_heavy = 0;
    __syncthreads();

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
            if (ours && is_heavy && k == rs) {
                const int slot = atomicAdd(&n_heavy, 1);   // at most one such run can start among EMB_U positions
                if (slot < EMB_WAVES) heavy_row[slot] = key;
            }
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
    const int nh = n_heavy < EMB_WAVES ? n_heavy : EMB_WAVES;
    for (int h = 0; h < nh; ++h) {
        const int hv = heavy_row[h];
        int hs = row_start[hv], he = row_start[hv + 1];
        hs = hs < 0 ? 0 : (hs > N ? N : hs);
        he = he < hs ? hs : (he > N ? N : he);
        // wave i takes the run of whole examples that starts at bound(i): an even split of the positions, moved
        // forward to the next change of example
        auto bound = [&](int i) {
            if (i <= 0) return hs;
            if (i >= EMB_WAVES) return he;
            const int k = hs + (int)(((int64_t)(he - hs) * i) / EMB_WAVES);
            if (k <= hs) return hs;
            const int limit = (pos[k - 1] / T + 1) * T;
            return first_at_least(pos, k, he, limit);
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
            store_row(hv, ra.sums);
        }
        __syncthreads();
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct EmbedLayout {
    int passes, nblocks;
    size_t hist, keys_a, vals_a, keys_b, vals_b, row_start, total;   // byte offsets into the workspace
};

EmbedLayout embed_layout(int64_t N, int64_t V)
{
    EmbedLayout L;
    int bits = 0;
    while (((int64_t)1 << bits) <= V) ++bits;   // the largest key is V
    L.passes = (bits + 7) / 8;
    if (L.passes < 1) L.passes = 1;
    L.nblocks = (int)((N + SORT_TILE - 1) / SORT_TILE);
    size_t o = 0;
    L.hist = o; o += align256((size_t)256 * L.nblocks * sizeof(int));
    L.keys_a = o; o += align256((size_t)N * sizeof(int));
    L.vals_a = o; o += align256((size_t)N * sizeof(int));
    L.keys_b = o; o += align256((size_t)N * sizeof(int));
    L.vals_b = o; o += align256((size_t)N * sizeof(int));
    L.row_start = o; o += align256((size_t)(V + 2) * sizeof(int));
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
    const int64_t entries = (int64_t)256 * L.nblocks;
    const dim3 grid(L.nblocks), block(256);
    const int* kin = nullptr;
    const int* vin = nullptr;
    int* kout = ka;
    int* vout = va;
    for (int ps = 0; ps < L.passes; ++ps) {
        if (ps == 0) sort_hist_kernel<TId, true><<<grid, block, 0, stream>>>(ids, nullptr, N, V, 0, L.nblocks, hist);
        else sort_hist_kernel<TId, false><<<grid, block, 0, stream>>>(ids, kin, N, V, 8 * ps, L.nblocks, hist);
        sort_scan_kernel<<<dim3(1), dim3(1024), 0, stream>>>(hist, entries);
        if (ps == 0) sort_scatter_kernel<TId, true><<<grid, block, 0, stream>>>(ids, nullptr, nullptr, kout, vout, N, V, 0, L.nblocks, hist);
        else sort_scatter_kernel<TId, false><<<grid, block, 0, stream>>>(ids, kin, vin, kout, vout, N, V, 8 * ps, L.nblocks, hist);
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
                       float* S_id, float* S_sq, float* S_sg, hipStream_t stream)
{
    const int64_t per_group = (int64_t)EMB_WAVES * EMB_U;
    const int chunk_groups = (int)((N + per_group - 1) / per_group);
    const int zero_groups = (int)(((int64_t)V + EMB_WAVES * EMB_ZROWS - 1) / (EMB_WAVES * EMB_ZROWS));
    const dim3 grid((unsigned)(chunk_groups + zero_groups), (unsigned)((d + 64 * CH - 1) / (64 * CH)));
    embed_rows_kernel<TIn, CH, WANT><<<grid, dim3(EMB_WAVES * 64), 0, stream>>>(G, row_start, keys, pos, N, V, T, d, chunk_groups,
                                                                                  S_id, S_sq, S_sg);
    return hipGetLastError();
}

template <typename TIn, int CH>
hipError_t launch_rows_want(uint32_t want, const TIn* G, const int* rs, const int* keys, const int* pos, int N, int V, int T, int64_t d, float* a,
                            float* q, float* g, hipStream_t st)
{
    switch (want) {
    case 1: return launch_rows<TIn, CH, 1>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    case 2: return launch_rows<TIn, CH, 2>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    case 3: return launch_rows<TIn, CH, 3>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    case 4: return launch_rows<TIn, CH, 4>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    case 5: return launch_rows<TIn, CH, 5>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    case 6: return launch_rows<TIn, CH, 6>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    default: return launch_rows<TIn, CH, 7>(G, rs, keys, pos, N, V, T, d, a, q, g, st);
    }
}

}  // namespace

size_t embed_workspace(int64_t B, int64_t T, int64_t V) { return embed_layout(B * T, V).total; }

hipError_t launch_embed_stat(const void* ids, int ids_bytes, const void* G, int64_t B, int64_t T, int64_t V, int64_t d,
                             pex_dtype dt, uint32_t want, float* S_id, float* S_sq, float* S_sign, void* workspace,
                             hipStream_t stream)
{
    const int N = (int)(B * T);
    const EmbedLayout L = embed_layout(N, V);
    char* ws = (char*)workspace;
    const int* keys = nullptr;
    const int* pos = nullptr;
    hipError_t e = ids_bytes == 8 ? sort_positions<int64_t>((const int64_t*)ids, N, (int)V, L, ws, &keys, &pos, stream)
                                  : sort_positions<int32_t>((const int32_t*)ids, N, (int)V, L, ws, &keys, &pos, stream);
    if (e != hipSuccess) return e;
    int* row_start = (int*)(ws + L.row_start);
    row_start_kernel<<<dim3((unsigned)(((int64_t)N + 1 + 255) / 256)), dim3(256), 0, stream>>>(keys, N, (int)V, row_start);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dt == PEX_BF16) {
        if (d % 4 == 0) return launch_rows_want<uint16_t, 4>(want, (const uint16_t*)G, row_start, keys, pos, N, (int)V, (int)T, d, S_id, S_sq, S_sign, stream);
        return launch_rows_want<uint16_t, 1>(want, (const uint16_t*)G, row_start, keys, pos, N, (int)V, (int)T, d, S_id, S_sq, S_sign, stream);
    }
    if (d % 4 == 0) return launch_rows_want<float, 4>(want, (const float*)G, row_start, keys, pos, N, (int)V, (int)T, d, S_id, S_sq, S_sign, stream);
    return launch_rows_want<float, 1>(want, (const float*)G, row_start, keys, pos, N, (int)V, (int)T, d, S_id, S_sq, S_sign, stream);
}

}  // namespace pex
