// Online conformal calibration and ordinal classification (integer work, bit-exact).
//
// The calibration multiset is kept on the device as an ascending array of 32-bit keys; a key is
// an order-preserving image of the fp32 score (-0 folded onto +0, every NaN onto key 0, below
// -inf), so all comparisons are unsigned-integer comparisons that reproduce the IEEE ones.
//
//   append (Online Calibration):  keys of the new scores are sorted (bitonic block sort in LDS,
//       then either a one-pass multi-way placement or pairwise merge passes) and merged with the
//       resident array by a merge-path kernel into the other half of a ping-pong buffer.
//   classify (Eq. "p-value", Eq. "prediction_set"):  one binary search per test score gives
//       ranks = #{cal >= s}; the class is an integer comparison of ranks + 1 with
//       r_l = floor(alpha_l (N + 1)); the quantile thresholds of Eq. "quantile" are read straight
//       from the sorted array.
#include "common.h"

#include <math.h>
#include <new>

struct atts_calib {
    uint32_t* keys[2];   // ping-pong sorted arrays, capacity each
    uint32_t* runs;      // sorted runs of the batch being appended
    uint32_t* batch;     // fully sorted batch
    int64_t capacity;
    int64_t n;
    int cur;
};

namespace atts {
namespace {

constexpr int kSortChunk = 8192;    // keys per block-sort workgroup
constexpr int kSortThreads = 1024;
constexpr int kMergeSeg = 2048;     // outputs per merge workgroup
constexpr int kMergeThreads = 256;
constexpr int kMergePer = kMergeSeg / kMergeThreads;
constexpr int kMaxMultiwayRuns = 16;
constexpr uint32_t kPadKey = 0xFFFFFFFFu;   // above the key of +inf (0xFF800000)

// Integer-only, so that sub-normal scores keep their order whatever the float mode is.
__device__ __forceinline__ bool score_is_nan(float f) { return (__float_as_uint(f) & 0x7FFFFFFFu) > 0x7F800000u; }
__device__ __forceinline__ uint32_t score_to_key(float f) {
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0u;   // NaN
    if ((b & 0x7FFFFFFFu) == 0u) b = 0u;              // -0 -> +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_score(uint32_t k) {
    if (k == 0u) return __uint_as_float(0x7FC00000u);
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// first index in [0, n) with a[idx] >= x  (n if none)
__device__ __forceinline__ int64_t lower_bound(const uint32_t* __restrict__ a, int64_t n, uint32_t x) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}
// first index with a[idx] > x
__device__ __forceinline__ int64_t upper_bound(const uint32_t* __restrict__ a, int64_t n, uint32_t x) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (a[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---- merge path ------------------------------------------------------------------------------------
// Number of elements taken from a[] among the first `diag` outputs of the stable merge (a first on ties).
template <typename Index>
__device__ __forceinline__ Index merge_path(const uint32_t* a, Index na, const uint32_t* b, Index nb, Index diag) {
    Index lo = diag > nb ? diag - nb : 0, hi = diag < na ? diag : na;
    while (lo < hi) {
        Index mid = (lo + hi) >> 1;
        if (a[mid] <= b[diag - 1 - mid]) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---- block sort: each workgroup turns kSortChunk scores into one ascending run of keys ----------
// 8 keys per thread: sorted in registers (odd-even transposition network), then log2(1024) rounds of pairwise
// merges of sorted runs through two LDS buffers (each thread finds its 8 outputs by merge path and merges them
// sequentially), one barrier per round.
__device__ __forceinline__ void cswap(uint32_t& x, uint32_t& y) {
    const uint32_t lo = min(x, y), hi = max(x, y);
    x = lo;
    y = hi;
}

__global__ __launch_bounds__(kSortThreads) void block_sort_kernel(const float* __restrict__ scores, int64_t n,
                                                                  uint32_t* __restrict__ runs) {
    constexpr int VT = kSortChunk / kSortThreads;   // 8
    static_assert(VT == 8, "register network below sorts 8 keys");
    __shared__ uint32_t buf[2][kSortChunk];
    const int64_t base = (int64_t)blockIdx.x * kSortChunk;
    const int tid = threadIdx.x;
    for (int i = tid; i < kSortChunk; i += kSortThreads) buf[0][i] = base + i < n ? score_to_key(scores[base + i]) : kPadKey;
    __syncthreads();
    uint32_t k[VT];
#pragma unroll
    for (int e = 0; e < VT; ++e) k[e] = buf[0][tid * VT + e];
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
        int ia = merge_path<int>(a, width, b, width, o - pair);
        int ib = o - pair - ia;
        uint32_t ka = ia < width ? a[ia] : kPadKey, kb = ib < width ? b[ib] : kPadKey;
#pragma unroll
        for (int e = 0; e < VT; ++e) {
            const bool take_a = ib >= width || (ia < width && ka <= kb);
            k[e] = take_a ? ka : kb;
            if (take_a) {
                ++ia;
                ka = ia < width ? a[ia] : kPadKey;
            } else {
                ++ib;
                kb = ib < width ? b[ib] : kPadKey;
            }
        }
#pragma unroll
        for (int e = 0; e < VT; ++e) dst[o + e] = k[e];
        cur ^= 1;
    }
    __syncthreads();
    for (int i = tid; i < kSortChunk; i += kSortThreads)
        if (base + i < n) runs[base + i] = buf[cur][i];
}

// ---- multi-way placement: final position of every element of <= kMaxMultiwayRuns sorted runs -----
// Stable: among equal keys, elements of earlier runs come first.
__global__ __launch_bounds__(256) void multiway_place_kernel(const uint32_t* __restrict__ runs, int64_t n,
                                                             uint32_t* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const uint32_t x = runs[e];
    const int my_run = (int)(e / kSortChunk);
    const int n_runs = (int)((n + kSortChunk - 1) / kSortChunk);
    int64_t pos = e % kSortChunk;
    for (int q = 0; q < n_runs; ++q) {
        if (q == my_run) continue;
        const int64_t off = (int64_t)q * kSortChunk;
        const int64_t len = min((int64_t)kSortChunk, n - off);
        pos += q < my_run ? upper_bound(runs + off, len, x) : lower_bound(runs + off, len, x);
    }
    out[pos] = x;
}

// ---- merging two sorted arrays --------------------------------------------------------------------
struct MergeJob {
    const uint32_t* a;   // pair y: a + 2 y run, length min(run, n - 2 y run)   (pairwise mode: run > 0)
    int64_t na;
    const uint32_t* b;   // pair y: a + (2 y + 1) run
    int64_t nb;
    uint32_t* out;       // pair y: out + 2 y run
    int64_t run;         // 0: single job (a, na, b, nb, out) as given
    int64_t n;           // pairwise mode: total elements
};

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(MergeJob job) {
    const uint32_t* a = job.a;
    const uint32_t* b = job.b;
    uint32_t* out = job.out;
    int64_t na = job.na, nb = job.nb;
    if (job.run > 0) {
        const int64_t off = 2 * (int64_t)blockIdx.y * job.run;
        if (off >= job.n) return;
        a = job.a + off;
        na = min(job.run, job.n - off);
        b = a + na;
        nb = max((int64_t)0, min(job.run, job.n - off - job.run));
        out = job.out + off;
    }
    const int64_t total = na + nb;
    const int64_t o0 = (int64_t)blockIdx.x * kMergeSeg;
    if (o0 >= total) return;
    const int64_t o1 = min(o0 + kMergeSeg, total);

    __shared__ int64_t split[2];
    __shared__ uint32_t buf[kMergeSeg];
    // Merge-path split of both segment ends at once: threads 0..127 search the diagonal o0, threads 128..255 the
    // diagonal o1.  Each round probes 128 evenly spaced candidates of the current range in parallel (one load
    // latency per round instead of one per halving step); "a[i] <= b[diag - 1 - i]" is true below the split.
    {
        __shared__ int64_t s_lo[2], s_hi[2];
        __shared__ int s_cnt[2];
        const int h = threadIdx.x >> 7, t = threadIdx.x & 127;
        const int64_t diag = h ? o1 : o0;
        if (t == 0) {
            s_lo[h] = diag > nb ? diag - nb : 0;
            s_hi[h] = diag < na ? diag : na;
        }
        __syncthreads();
        while (s_lo[0] != s_hi[0] || s_lo[1] != s_hi[1]) {      // block-uniform
            const int64_t lo = s_lo[h], hi = s_hi[h], range = hi - lo;
            if (t == 0) s_cnt[h] = 0;
            __syncthreads();
            const int64_t step = (range + 127) / 128;
            const int64_t i = lo + t * step;
            const bool pred = range > 0 && i < hi && a[i] <= b[diag - 1 - i];
            const int c_wave = __popcll(__ballot(pred));
            if ((threadIdx.x & 63) == 0 && c_wave) atomicAdd(&s_cnt[h], c_wave);
            __syncthreads();
            if (t == 0 && range > 0) {
                const int64_t c = s_cnt[h], n_probe = (range + step - 1) / step;
                s_lo[h] = c > 0 ? lo + (c - 1) * step + 1 : lo;
                s_hi[h] = c == 0 ? lo : (c < n_probe ? lo + c * step : hi);
            }
            __syncthreads();
        }
        if (t == 0) split[h] = s_lo[h];
    }
    __syncthreads();
    const int64_t i0 = split[0], i1 = split[1];
    const int64_t j0 = o0 - i0, j1 = o1 - i1;
    const int la = (int)(i1 - i0), lb = (int)(j1 - j0);
    for (int i = threadIdx.x; i < la; i += kMergeThreads) buf[i] = a[i0 + i];
    for (int i = threadIdx.x; i < lb; i += kMergeThreads) buf[la + i] = b[j0 + i];
    __syncthreads();

    const int len = la + lb;
    const int d0 = min((int)threadIdx.x * kMergePer, len);
    const int d1 = min(d0 + kMergePer, len);
    int ia = merge_path<int>(buf, la, buf + la, lb, d0);
    int ib = d0 - ia;
    for (int d = d0; d < d1; ++d) {
        bool take_a = ib >= lb || (ia < la && buf[ia] <= buf[la + ib]);
        out[o0 + d] = take_a ? buf[ia++] : buf[la + ib++];
    }
}

// ---- classification ----------------------------------------------------------------------------------
struct ClassifyLevels {
    int64_t r[ATTS_MAX_ALPHAS];   // reject ranks floor(alpha_l (N + 1))
    int32_t n_alpha;
};

constexpr int kTopEntries = 1024;   // LDS index: every (n / 1024 rounded up to a power of two)-th key

__global__ __launch_bounds__(256) void classify_kernel(const uint32_t* __restrict__ keys, int64_t n,
                                                       const float* __restrict__ test, int64_t m, ClassifyLevels lv,
                                                       int top_shift, int32_t* __restrict__ ranks,
                                                       float* __restrict__ pvalues, uint8_t* __restrict__ classes,
                                                       float* __restrict__ thresholds) {
    // top[i] = keys[i << top_shift]: the first ~10 steps of every binary search run in LDS, the rest touch a
    // window of at most 2^top_shift keys.
    __shared__ uint32_t top[kTopEntries];
    const int n_top = (int)((n + ((int64_t)1 << top_shift) - 1) >> top_shift);
    for (int i = threadIdx.x; i < n_top; i += 256) top[i] = keys[(int64_t)i << top_shift];
    __syncthreads();
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && thresholds && (int)threadIdx.x < lv.n_alpha) {
        const int64_t kth = n + 1 - lv.r[threadIdx.x];     // 1-indexed order statistic
        thresholds[threadIdx.x] = kth > n ? INFINITY : (kth < 1 ? -INFINITY : key_to_score(keys[kth - 1]));
    }
    if (i >= m) return;
    const float s = test[i];
    int64_t c = 0;
    if (!score_is_nan(s)) {
        const uint32_t x = score_to_key(s);
        int lo = 0, hi = n_top;                            // t = number of index entries < x
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (top[mid] < x) lo = mid + 1; else hi = mid;
        }
        int64_t lb = 0;
        if (lo > 0) {                                      // keys[(lo - 1) << shift] < x <= keys[lo << shift]
            const int64_t w0 = ((int64_t)(lo - 1) << top_shift) + 1;
            const int64_t w1 = min(n, (int64_t)lo << top_shift);
            lb = w0 + lower_bound(keys + w0, w1 - w0, x);
        }
        c = n - lb;
    }
    ranks[i] = (int32_t)c;
    if (pvalues) pvalues[i] = (float)((double)(c + 1) / (double)(n + 1));
    int cls = 0;
    for (int l = 0; l < lv.n_alpha; ++l) cls += (c + 1 <= lv.r[l]) ? 1 : 0;
    classes[i] = (uint8_t)cls;
}

__global__ void export_kernel(const uint32_t* __restrict__ keys, int64_t n, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = key_to_score(keys[i]);
}

}  // namespace
}  // namespace atts

using namespace atts;

extern "C" {

int32_t atts_calib_create(int64_t capacity, atts_calib** out) {
    if (!out) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_create: out is NULL");
    *out = nullptr;
    if (capacity < 1 || capacity > ((int64_t)1 << 30))
        return fail(ATTS_ERR_INVALID_ARG, "atts_calib_create: capacity %lld outside [1, 2^30]", (long long)capacity);
    atts_calib* c = new (std::nothrow) atts_calib();
    if (!c) return fail(ATTS_ERR_HIP, "atts_calib_create: out of host memory");
    c->capacity = capacity;
    c->n = 0;
    c->cur = 0;
    // sorted runs are padded to whole chunks only in LDS, never in memory
    uint32_t** bufs[4] = {&c->keys[0], &c->keys[1], &c->runs, &c->batch};
    for (int i = 0; i < 4; ++i) *bufs[i] = nullptr;
    for (int i = 0; i < 4; ++i) {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(bufs[i]), (size_t)capacity * sizeof(uint32_t));
        if (e != hipSuccess) {
            for (int j = 0; j < 4; ++j)
                if (*bufs[j]) (void)hipFree(*bufs[j]);
            delete c;
            return fail(ATTS_ERR_HIP, "atts_calib_create: hipMalloc of %lld keys failed: %s", (long long)capacity,
                        hipGetErrorString(e));
        }
    }
    *out = c;
    return ATTS_OK;
}

int32_t atts_calib_destroy(atts_calib* c) {
    if (!c) return ATTS_OK;
    (void)hipFree(c->keys[0]);
    (void)hipFree(c->keys[1]);
    (void)hipFree(c->runs);
    (void)hipFree(c->batch);
    delete c;
    return ATTS_OK;
}

int32_t atts_calib_size(const atts_calib* c, int64_t* out_n) {
    if (!c || !out_n) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_size: NULL argument");
    *out_n = c->n;
    return ATTS_OK;
}

int32_t atts_calib_reset(atts_calib* c) {
    if (!c) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_reset: NULL handle");
    c->n = 0;
    return ATTS_OK;
}

int32_t atts_calibrate_online(atts_calib* c, const float* new_scores, int64_t n_new, void* hip_stream) {
    if (!c) return fail(ATTS_ERR_INVALID_ARG, "atts_calibrate_online: NULL handle");
    if (n_new < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_calibrate_online: n_new = %lld < 0", (long long)n_new);
    if (n_new == 0) return ATTS_OK;
    if (!new_scores) return fail(ATTS_ERR_INVALID_ARG, "atts_calibrate_online: new_scores is NULL");
    if (c->n + n_new > c->capacity)
        return fail(ATTS_ERR_CAPACITY, "atts_calibrate_online: %lld + %lld scores exceed the capacity %lld", (long long)c->n,
                    (long long)n_new, (long long)c->capacity);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // 1. keys of the new scores, sorted in runs of kSortChunk
    const int64_t n_runs = ceil_div(n_new, kSortChunk);
    hipLaunchKernelGGL(block_sort_kernel, dim3((unsigned)n_runs), dim3(kSortThreads), 0, stream, new_scores, n_new, c->runs);
    ATTS_LAUNCH_CHECK("block_sort_kernel");

    // 2. one sorted batch
    const uint32_t* sorted = c->runs;
    if (n_runs > 1 && n_runs <= kMaxMultiwayRuns) {
        hipLaunchKernelGGL(multiway_place_kernel, dim3((unsigned)ceil_div(n_new, 256)), dim3(256), 0, stream, c->runs, n_new,
                           c->batch);
        ATTS_LAUNCH_CHECK("multiway_place_kernel");
        sorted = c->batch;
    } else if (n_runs > 1) {
        uint32_t* src = c->runs;
        uint32_t* dst = c->batch;
        for (int64_t run = kSortChunk; run < n_new; run *= 2) {
            MergeJob job{src, 0, nullptr, 0, dst, run, n_new};
            dim3 grid((unsigned)ceil_div(2 * run, kMergeSeg), (unsigned)ceil_div(n_new, 2 * run));
            hipLaunchKernelGGL(merge_kernel, grid, dim3(kMergeThreads), 0, stream, job);
            ATTS_LAUNCH_CHECK("merge_kernel (pairwise)");
            uint32_t* t = src;
            src = dst;
            dst = t;
        }
        sorted = src;
    }

    // 3. merge with the resident array into the other half of the ping-pong buffer
    MergeJob job{c->keys[c->cur], c->n, sorted, n_new, c->keys[c->cur ^ 1], 0, 0};
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)ceil_div(c->n + n_new, kMergeSeg)), dim3(kMergeThreads), 0, stream, job);
    ATTS_LAUNCH_CHECK("merge_kernel");
    c->cur ^= 1;
    c->n += n_new;
    return ATTS_OK;
}

int32_t atts_classify_ordinal(const atts_calib* c, const float* test_scores, int64_t M, const double* alphas, int32_t n_alpha,
                              int32_t* ranks, float* pvalues, uint8_t* classes, float* thresholds, void* hip_stream) {
    if (!c) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: NULL handle");
    if (M < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: M = %lld < 0", (long long)M);
    if (!alphas || n_alpha < 1 || n_alpha > ATTS_MAX_ALPHAS)
        return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: need 1..%d alpha levels", ATTS_MAX_ALPHAS);
    for (int l = 0; l < n_alpha; ++l) {
        if (!(alphas[l] > 0.0 && alphas[l] < 1.0))
            return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: alpha[%d] = %g is not inside (0, 1)", l, alphas[l]);
        if (l > 0 && alphas[l] < alphas[l - 1])
            return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: alpha levels must be non-decreasing");
    }
    if (c->n < 1) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: the calibration set is empty");
    if (M > 0 && (!test_scores || !ranks || !classes))
        return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: test_scores, ranks and classes must not be NULL");
    if (M > ((int64_t)1 << 31) * 255) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: M too large");
    ClassifyLevels lv;
    lv.n_alpha = n_alpha;
    for (int l = 0; l < ATTS_MAX_ALPHAS; ++l) lv.r[l] = 0;
    for (int l = 0; l < n_alpha; ++l) lv.r[l] = (int64_t)floor(alphas[l] * (double)(c->n + 1));
    if (M == 0 && !thresholds) return ATTS_OK;
    const unsigned blocks = (unsigned)(M > 0 ? ceil_div(M, 256) : 1);
    int top_shift = 0;
    while (((c->n + ((int64_t)1 << top_shift) - 1) >> top_shift) > kTopEntries) ++top_shift;
    hipLaunchKernelGGL(classify_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), c->keys[c->cur],
                       c->n, test_scores, M, lv, top_shift, ranks, pvalues, classes, thresholds);
    ATTS_LAUNCH_CHECK("classify_kernel");
    return ATTS_OK;
}

int32_t atts_calib_export(const atts_calib* c, float* out, void* hip_stream) {
    if (!c) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_export: NULL handle");
    if (c->n == 0) return ATTS_OK;
    if (!out) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_export: out is NULL");
    hipLaunchKernelGGL(export_kernel, dim3((unsigned)ceil_div(c->n, 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       c->keys[c->cur], c->n, out);
    ATTS_LAUNCH_CHECK("export_kernel");
    return ATTS_OK;
}

}  // extern "C"
