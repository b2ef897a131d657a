// Sorting a batch of new conformity scores into ascending keys (first half of "Online Calibration": the
// scores of newly pre-sampled outputs join the calibration multiset, which this library keeps sorted).
//
// Two regimes:
//   * up to kSmallSortMax scores (cache-resident, latency-bound): every workgroup sorts one run of kSortChunk keys
//     in registers + LDS (block_sort_kernel), then ONE pass places every key at its final position
//     (multiway_place_kernel: own index in its run + its counts in all other runs, searched in windows of the
//     other runs staged in LDS).  A run is sorted by ONE compute unit, whose instruction issue bounds it; shorter
//     runs sort faster but make the placement pass (one window per other run) slower: 8192 measured best.
//   * larger batches (bandwidth-bound): least-significant-digit radix sort, four passes of 8 bits.  A pass is
//     three launches: per-tile digit histograms, a scan per digit over the tiles, and a stable scatter (ranks
//     inside a tile by wavefront-wide digit matching, keys reordered through LDS so that each digit's keys of a
//     tile leave as one contiguous run).  No inter-workgroup waiting anywhere.
#include "common.h"
#include "keys.h"

namespace atts {
namespace {

// ------------------------------------------------------------------------------------------------------------
// small batches: block sort + multi-way placement
// ------------------------------------------------------------------------------------------------------------
constexpr int kSortChunk = 8192;             // keys per block-sort workgroup (one sorted run)
constexpr int kSortVT = 8;                   // keys per thread
constexpr int kSortThreads = kSortChunk / kSortVT;
constexpr int kMaxPlaceRuns = 8;
constexpr int kSmallSortMax = kMaxPlaceRuns * kSortChunk;   // 65,536: at most 8 runs are placed in one pass
constexpr int kPlaceThreads = 1024;          // keys per placement workgroup
constexpr int kWindowCap = 16384;            // LDS keys that hold the other runs' windows of one placement workgroup

__device__ __forceinline__ void cswap(uint32_t& x, uint32_t& y) {
    const uint32_t lo = min(x, y), hi = max(x, y);
    x = lo;
    y = hi;
}

// Each workgroup turns kSortChunk scores into one ascending run of keys: 8 keys per thread sorted in registers
// (odd-even transposition network), then log2(threads) rounds of pairwise merges of sorted runs through two LDS
// buffers, one barrier per round.  In a round every thread produces 8 consecutive outputs of its pair of runs: merge
// path gives the first input of each run, the next 8 keys of both runs are loaded at once (one LDS latency instead
// of eight dependent ones) and the 8 smallest of the 16 are taken by a bitonic network in registers.
// The last run is padded with kPadKey up to a multiple of 16 keys.
__global__ __launch_bounds__(kSortThreads) void block_sort_kernel(const float* __restrict__ scores, int64_t n,
                                                                  uint32_t* __restrict__ runs) {
    constexpr int VT = kSortVT;
    static_assert(VT == 8, "register networks below take 8 keys");
    __shared__ uint32_t buf[2][kSortChunk];
    const int64_t base = (int64_t)blockIdx.x * kSortChunk;
    const int tid = threadIdx.x;
    uint32_t k[VT];
#pragma unroll
    for (int e = 0; e < VT; ++e) {                                 // coalesced: key e of the thread is element e * threads + tid
        const int64_t i = base + e * kSortThreads + tid;
        k[e] = i < n ? score_to_key(scores[i]) : kPadKey;
    }
#pragma unroll
    for (int round = 0; round < VT; ++round) {
#pragma unroll
        for (int e = round & 1; e + 1 < VT; e += 2) cswap(k[e], k[e + 1]);
    }
#pragma unroll
    for (int e = 0; e < VT; ++e) buf[0][tid * VT + e] = k[e];
    int cur = 0;
    for (int width = VT; width < kSortChunk; width *= 2) {
        __syncthreads();
        const uint32_t* src = buf[cur];
        uint32_t* dst = buf[cur ^ 1];
        const int o = tid * VT;
        const int pair = o & ~(2 * width - 1);
        const uint32_t* a = src + pair;
        const uint32_t* b = a + width;
        const int ia = merge_path<int>(a, width, b, width, o - pair);
        const int ib = o - pair - ia;
        uint32_t x[VT], y[VT];
#pragma unroll
        for (int e = 0; e < VT; ++e) {
            x[e] = ia + e < width ? a[ia + e] : kPadKey;
            y[VT - 1 - e] = ib + e < width ? b[ib + e] : kPadKey;  // second run reversed: (x, y) is a bitonic sequence
        }
#pragma unroll
        for (int e = 0; e < VT; ++e) k[e] = min(x[e], y[e]);       // the 8 smallest of the 16, as a bitonic sequence
#pragma unroll
        for (int stride = VT / 2; stride > 0; stride >>= 1)
#pragma unroll
            for (int e = 0; e < VT; ++e)
                if ((e & stride) == 0) cswap(k[e], k[e + stride]);
#pragma unroll
        for (int e = 0; e < VT; ++e) dst[o + e] = k[e];
        cur ^= 1;
    }
    __syncthreads();
    const int64_t n16 = (n + 15) & ~(int64_t)15;
    for (int i = tid; i < kSortChunk; i += kSortThreads)
        if (base + i < n16) runs[base + i] = buf[cur][i];
}

// #{keys of the ascending array a[0, len) that are < y}, found by the 64 lanes of a wavefront together: each round
// the lanes probe 64 evenly spaced keys of the remaining range and a ballot narrows it (three dependent rounds for
// 8192 keys instead of thirteen).  All lanes return the count.
__device__ __forceinline__ int wave_count_below(const uint32_t* __restrict__ a, int len, uint32_t y) {
    const int lane = threadIdx.x & 63;
    int lo = 0, hi = len;                       // the count lies in [lo, hi]: a[lo - 1] < y (or lo == 0), a[hi] >= y (or hi == len)
    while (hi > lo) {
        const int span = hi - lo;
        const int step = (span + 63) >> 6;      // probes at lo + step - 1, lo + 2 step - 1, ...
        const int at = lo + (lane + 1) * step - 1;
        const bool below = at < hi && a[at] < y;
        const int c = __popcll(__ballot(below));             // the probes below y form a prefix
        const int new_lo = c > 0 ? lo + c * step : lo;
        const int new_hi = min(hi, lo + (c + 1) * step - 1); // the first probe not below y (if any) bounds the count
        lo = min(new_lo, hi);
        hi = max(new_hi, lo);
    }
    return lo;
}

// Final position of every key of <= 8 sorted runs of kSortChunk keys (the last one shorter).  Stable: among equal
// keys, those of earlier runs come first.
//   position = index in the own run + sum over the other runs q of #{keys of run q that go before x},
//   "before" = "<= x" for an earlier run, "< x" for a later one = "< x + bias" (x < 2^32 - 1).
// A workgroup places 1024 consecutive keys of one run.  Their counts in another run lie between the counts of
// the first and of the last of them (each found by one wavefront): that window of the other run (about 1024 keys
// when the runs are alike) is copied to LDS with coalesced loads and every key finds its count there by binary
// search.  Windows that do not fit the LDS budget together (very unlike runs) are searched in global memory instead.
__global__ __launch_bounds__(kPlaceThreads) void multiway_place_kernel(const uint32_t* __restrict__ runs, int64_t n,
                                                                       uint32_t* __restrict__ out) {
    __shared__ uint32_t win[kWindowCap];
    __shared__ int w_lo[kMaxPlaceRuns], w_hi[kMaxPlaceRuns], w_off[kMaxPlaceRuns + 1];
    const int n_runs = (int)((n + kSortChunk - 1) / kSortChunk);
    const int64_t e0 = (int64_t)blockIdx.x * kPlaceThreads;
    const int cnt = (int)min((int64_t)kPlaceThreads, n - e0);           // >= 1
    const int my_run = (int)(e0 / kSortChunk);                          // kPlaceThreads divides kSortChunk
    const int tid = threadIdx.x, wave = tid >> 6;
    auto run_len = [&](int q) { return (int)min((int64_t)kSortChunk, n - (int64_t)q * kSortChunk); };
    // wavefront w: one end of the window of run w / 2
    if (wave < 2 * n_runs) {
        const int q = wave >> 1;
        const uint32_t x_end = runs[e0 + ((wave & 1) ? cnt - 1 : 0)];
        const int c = q == my_run ? 0 : wave_count_below(runs + (int64_t)q * kSortChunk, run_len(q), x_end + (q < my_run ? 1u : 0u));
        if ((tid & 63) == 0) ((wave & 1) ? w_hi : w_lo)[q] = c;
    }
    __syncthreads();
    if (tid == 0) {
        int total = 0;
        for (int q = 0; q < n_runs; ++q) {
            w_off[q] = total;
            total += w_hi[q] - w_lo[q];                                  // 0 for the own run
        }
        w_off[n_runs] = total;
    }
    __syncthreads();
    const bool staged = w_off[n_runs] <= kWindowCap;                     // block-uniform
    if (staged) {
        for (int q = 0; q < n_runs; ++q) {
            const uint32_t* src = runs + (int64_t)q * kSortChunk + w_lo[q];
            const int len = w_hi[q] - w_lo[q];
            for (int i = tid; i < len; i += kPlaceThreads) win[w_off[q] + i] = src[i];
        }
    }
    __syncthreads();
    if (tid >= cnt) return;
    const uint32_t x = runs[e0 + tid];
    int pos = (int)((e0 + tid) % kSortChunk);
    // all windows together, their binary searches in lock step (the probes of one step are independent loads)
    constexpr int G = kMaxPlaceRuns;
    const uint32_t* a[G];
    int lo[G], len[G], longest = 0;
    uint32_t y[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int q = min(j, n_runs - 1);
        a[j] = staged ? win + w_off[q] : runs + (int64_t)q * kSortChunk + w_lo[q];
        len[j] = j < n_runs ? w_hi[q] - w_lo[q] : 0;                      // block-uniform
        y[j] = x + (q < my_run ? 1u : 0u);
        lo[j] = 0;
        longest = max(longest, len[j]);
        pos += j < n_runs ? w_lo[q] : 0;
    }
    // invariant per window: the count (first index with a[idx] >= y) lies in [lo, lo + len]
    while (longest > 0) {                                                // block-uniform trip count
#pragma unroll
        for (int j = 0; j < G; ++j) {
            if (len[j] > 0) {
                const int half = len[j] >> 1;
                const bool below = a[j][lo[j] + half] < y[j];
                lo[j] = below ? lo[j] + half + 1 : lo[j];
                len[j] = below ? len[j] - half - 1 : half;
            }
        }
        longest >>= 1;
    }
#pragma unroll
    for (int j = 0; j < G; ++j) pos += lo[j];
    out[pos] = x;
}

// ------------------------------------------------------------------------------------------------------------
// large batches: LSD radix sort, 8 bits per pass
// ------------------------------------------------------------------------------------------------------------
constexpr int kRadixThreads = 256;
constexpr int kRadixItems = 16;                              // keys per thread
constexpr int kRadixTile = kRadixThreads * kRadixItems;      // 4096 keys per workgroup
constexpr int kRadixBins = 256;

// exclusive prefix of v over the 256 threads of the workgroup (thread order) and the total; red: 4 words of LDS
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* red, uint32_t& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    __syncthreads();
    if (lane == 63) red[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kRadixThreads / 64; ++w) {
        const uint32_t r = red[w];
        before += w < wave ? r : 0u;
        all += r;
    }
    total = all;
    return before + incl - v;
}

// key of element idx of the pass input: the first pass reads the scores themselves
template <bool FIRST>
__device__ __forceinline__ uint32_t load_key(const void* __restrict__ in, int64_t idx) {
    if constexpr (FIRST) return score_to_key(reinterpret_cast<const float*>(in)[idx]);
    else return reinterpret_cast<const uint32_t*>(in)[idx];
}

// counts[d n_tiles + tile] = number of keys of the tile whose digit (key >> shift) & 255 is d
template <bool FIRST>
__global__ __launch_bounds__(kRadixThreads) void radix_hist_kernel(const void* __restrict__ in, int64_t n, int shift,
                                                                   int n_tiles, uint32_t* __restrict__ counts) {
    __shared__ uint32_t h[kRadixBins];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kRadixTile;
#pragma unroll 8
    for (int i = 0; i < kRadixItems; ++i) {
        const int64_t idx = base + i * kRadixThreads + threadIdx.x;
        if (idx < n) atomicAdd(&h[(load_key<FIRST>(in, idx) >> shift) & 255u], 1u);
    }
    __syncthreads();
    counts[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = h[threadIdx.x];
}

// One workgroup per digit d: counts[d][*] becomes its exclusive prefix over the tiles, digit_tot[d] the digit's total.
__global__ __launch_bounds__(kRadixThreads) void radix_scan_kernel(uint32_t* __restrict__ counts, int n_tiles,
                                                                   uint32_t* __restrict__ digit_tot) {
    __shared__ uint32_t red[4];
    uint32_t* p = counts + (int64_t)blockIdx.x * n_tiles;
    uint32_t carry = 0;
    for (int t0 = 0; t0 < n_tiles; t0 += kRadixThreads) {
        const int t = t0 + threadIdx.x;
        const uint32_t v = t < n_tiles ? p[t] : 0u;
        uint32_t total;
        const uint32_t ex = block_excl_scan(v, red, total);
        if (t < n_tiles) p[t] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) digit_tot[blockIdx.x] = carry;
}

// Stable scatter of one tile.  Order inside the tile: wavefront w owns a quarter of the tile (consecutive keys) and walks
// it in rounds of 64 consecutive keys.  In a round, the lanes that hold the same digit find each other with
// 8 ballots; a key's rank among its digit's keys of the wavefront = the digit's count so far (an LDS counter per
// wavefront and digit, read by all lanes of the group, advanced by its lowest lane) + the group's lanes below it.
// Prefixes over the wavefronts and digits then give every key its place in the tile's digit-sorted order; the
// keys go to that place in LDS and leave in tile order, so each digit's keys are written as one contiguous run.
template <bool FIRST>
__global__ __launch_bounds__(kRadixThreads) void radix_scatter_kernel(const void* __restrict__ in, int64_t n, int shift,
                                                                      int n_tiles, const uint32_t* __restrict__ tile_ofs,
                                                                      const uint32_t* __restrict__ digit_tot,
                                                                      uint32_t* __restrict__ out) {
    constexpr int kWaves = kRadixThreads / 64;
    __shared__ uint32_t wcnt[kWaves][kRadixBins];
    __shared__ uint32_t lkeys[kRadixTile];
    __shared__ uint32_t gdelta[kRadixBins];     // global position of a key = gdelta[digit] + its place in the tile (mod 2^32)
    __shared__ uint32_t lstart[kRadixBins];     // first place of the digit in the tile's digit-sorted order
    __shared__ uint32_t red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = (int64_t)blockIdx.x * kRadixTile + (int64_t)wave * (64 * kRadixItems);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) wcnt[w][tid] = 0;
    uint32_t key[kRadixItems];
#pragma unroll
    for (int i = 0; i < kRadixItems; ++i) {
        const int64_t idx = base + i * 64 + lane;
        key[i] = idx < n ? load_key<FIRST>(in, idx) : kPadKey;
    }
    __syncthreads();
    volatile uint32_t* mine = wcnt[wave];
    const uint64_t below_me = ((uint64_t)1 << lane) - 1;
    uint32_t rank[kRadixItems];
#pragma unroll
    for (int i = 0; i < kRadixItems; ++i) {
        const bool valid = base + i * 64 + lane < n;
        const uint32_t d = (key[i] >> shift) & 255u;
        const uint64_t live = __ballot(valid);
        uint32_t g_lo = (uint32_t)live, g_hi = (uint32_t)(live >> 32);     // lanes whose digit equals this lane's
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint32_t mb = 0u - ((d >> b) & 1u);                       // all ones if the bit is set
            const uint64_t vote = __ballot(mb != 0u);
            g_lo &= ~((uint32_t)vote ^ mb);
            g_hi &= ~((uint32_t)(vote >> 32) ^ mb);
        }
        const uint32_t so_far = mine[d];
        const uint32_t lower = (uint32_t)(__popc(g_lo & (uint32_t)below_me) + __popc(g_hi & (uint32_t)(below_me >> 32)));
        rank[i] = so_far + lower;
        __builtin_amdgcn_wave_barrier();                      // every lane has read the counter before its group's leader advances it
        if (valid && lower == 0) mine[d] = so_far + (uint32_t)(__popc(g_lo) + __popc(g_hi));
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // thread d: prefixes of digit d over the wavefronts, the digit's count in the tile, its global offset
    uint32_t cnt = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t c = wcnt[w][tid];
        wcnt[w][tid] = cnt;
        cnt += c;
    }
    uint32_t tile_total, all;
    const uint32_t first = block_excl_scan(cnt, red, tile_total);
    const uint32_t digit_base = block_excl_scan(digit_tot[tid], red, all);
    lstart[tid] = first;
    gdelta[tid] = digit_base + tile_ofs[(int64_t)tid * n_tiles + blockIdx.x] - first;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kRadixItems; ++i) {
        if (base + i * 64 + lane < n) {
            const uint32_t d = (key[i] >> shift) & 255u;
            lkeys[lstart[d] + wcnt[wave][d] + rank[i]] = key[i];
        }
    }
    __syncthreads();
    for (uint32_t j = tid; j < tile_total; j += kRadixThreads) {
        const uint32_t k = lkeys[j];
        out[gdelta[(k >> shift) & 255u] + j] = k;
    }
}

template <bool FIRST>
int32_t radix_pass(const void* in, int64_t n, int shift, int n_tiles, uint32_t* counts, uint32_t* out, hipStream_t stream) {
    uint32_t* digit_tot = counts + (int64_t)kRadixBins * n_tiles;
    hipLaunchKernelGGL(radix_hist_kernel<FIRST>, dim3((unsigned)n_tiles), dim3(kRadixThreads), 0, stream, in, n, shift, n_tiles, counts);
    ATTS_LAUNCH_CHECK("radix_hist_kernel");
    hipLaunchKernelGGL(radix_scan_kernel, dim3(kRadixBins), dim3(kRadixThreads), 0, stream, counts, n_tiles, digit_tot);
    ATTS_LAUNCH_CHECK("radix_scan_kernel");
    hipLaunchKernelGGL(radix_scatter_kernel<FIRST>, dim3((unsigned)n_tiles), dim3(kRadixThreads), 0, stream, in, n, shift, n_tiles,
                       counts, digit_tot, out);
    ATTS_LAUNCH_CHECK("radix_scatter_kernel");
    return ATTS_OK;
}

}  // namespace

// radix sort: a digit histogram per tile + the digit totals (the small-batch path needs no scratch)
int64_t sort_scratch_words(int64_t n) { return (int64_t)kRadixBins * ceil_div(n > 0 ? n : 1, kRadixTile) + kRadixBins; }

int32_t launch_sort_scores(const float* scores, int64_t n, uint32_t* a, uint32_t* b, uint32_t* scratch, const uint32_t** sorted,
                           hipStream_t stream) {
    if (n <= kSmallSortMax) {
        const int64_t n_runs = ceil_div(n, kSortChunk);
        hipLaunchKernelGGL(block_sort_kernel, dim3((unsigned)n_runs), dim3(kSortThreads), 0, stream, scores, n, a);
        ATTS_LAUNCH_CHECK("block_sort_kernel");
        *sorted = a;
        if (n_runs > 1) {
            hipLaunchKernelGGL(multiway_place_kernel, dim3((unsigned)ceil_div(n, kPlaceThreads)), dim3(kPlaceThreads), 0, stream, a, n, b);
            ATTS_LAUNCH_CHECK("multiway_place_kernel");
            *sorted = b;
        }
        return ATTS_OK;
    }
    const int n_tiles = (int)ceil_div(n, kRadixTile);
    int32_t rc = radix_pass<true>(scores, n, 0, n_tiles, scratch, a, stream);
    if (rc == ATTS_OK) rc = radix_pass<false>(a, n, 8, n_tiles, scratch, b, stream);
    if (rc == ATTS_OK) rc = radix_pass<false>(b, n, 16, n_tiles, scratch, a, stream);
    if (rc == ATTS_OK) rc = radix_pass<false>(a, n, 24, n_tiles, scratch, b, stream);
    *sorted = b;
    return rc;
}

}  // namespace atts
