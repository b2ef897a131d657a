// Online conformal calibration and ordinal classification (integer work, bit-exact).
//
// The calibration multiset is kept on the device as an ascending array of 32-bit keys; a key is
// an order-preserving image of the fp32 score (-0 folded onto +0, every NaN onto key 0, below
// -inf), so all comparisons are unsigned-integer comparisons that reproduce the IEEE ones.
//
//   append (Online Calibration):  keys of the new scores are sorted (sort.hip: block sort + one-pass
//       multi-way placement for small batches, radix sort for large ones) and
//       merged with the resident array by a merge-path kernel into the other half of a ping-pong
//       buffer.  The same pass writes four sampled copies of its output (every 32nd, 1024th, 32768th,
//       2^20-th key), the levels of a static 32-ary search index: a node is one 128-byte line, the unit the L2
//       fills from memory.
//   classify (Eq. "p-value", Eq. "prediction_set"):  ranks = #{cal >= s} by one search per test
//       score: the coarsest index level sits in LDS, every further level costs one aligned 128-byte
//       line.  The class is an integer comparison of ranks + 1 with r_l = floor(alpha_l (N + 1));
//       the quantile thresholds of Eq. "quantile" are read straight from the sorted array.
//   conditional coverage (Proposition 2):  no state; one wavefront ranks the candidates of one input against
//       that input's own calibration scores.
#include "common.h"
#include "keys.h"

#include <math.h>
#include <new>

constexpr int kIndexLevels = 4;
constexpr int kFanBits = 5;                 // 32 keys per index node (one 128-byte line)
constexpr int kFan = 1 << kFanBits;

struct atts_calib {
    uint32_t* keys[2];                  // ping-pong sorted arrays, capacity each
    uint32_t* index[2][kIndexLevels];   // index[side][k][j] = keys[side][j * 32^(k+1)]
    uint32_t* runs;                     // the batch being appended: two buffers the sort alternates between
    uint32_t* batch;
    uint32_t* sort_scratch;             // digit histograms of the radix sort
    int32_t* splits;                    // merge-path splits of one streaming merge launch
    int64_t splits_len;
    int64_t capacity;
    int64_t n;
    int cur;
};

namespace atts {
namespace {

constexpr int kMergeThreads = 256;
constexpr int kMergeSegSmall = 2048;   // outputs per merge workgroup: cache-resident sizes (more workgroups)
constexpr int kMergeSegLarge = 4096;   // ... and streaming sizes (split search amortised over more keys; 8 workgroups per CU)
constexpr int64_t kMergeLargeFrom = (int64_t)1 << 22;

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

// ---- merging two sorted arrays --------------------------------------------------------------------
struct MergeJob {
    const uint32_t* a;   // resident keys (first on ties)
    int64_t na;
    const uint32_t* b;   // the sorted batch
    int64_t nb;
    uint32_t* out;
    uint32_t* index[kIndexLevels];   // EMIT only: index[k][j] = out[j * 32^(k+1)]
};

// LDS position of element i: one pad word per 32, so that the accesses "thread t, element t * PER + e" fall
// into distinct banks
__device__ __forceinline__ int lds_pad(int i) { return i + (i >> 5); }

// For a streaming merge launch of `segs` workgroups: splits[x] = elements taken from a[] among the first
// min(x seg, total) outputs.  One thread per entry: the searches run in parallel here instead of serially in front of
// every workgroup's loads.
__global__ __launch_bounds__(256) void merge_split_kernel(MergeJob job, int seg, int segs, int32_t* __restrict__ splits) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x > segs) return;
    const int64_t diag = min(x * (int64_t)seg, job.na + job.nb);
    splits[x] = (int32_t)merge_path<int64_t>(job.a, job.na, job.b, job.nb, diag);
}

// Each workgroup produces SEG consecutive outputs (out + segment start is 16-byte aligned).  PRESPLIT: the segment's
// merge-path splits come from merge_split_kernel.
template <int SEG, bool EMIT, bool PRESPLIT>
__global__ __launch_bounds__(kMergeThreads) void merge_kernel(MergeJob job, const int32_t* __restrict__ splits) {
    constexpr int PER = SEG / kMergeThreads;
    const uint32_t* __restrict__ a = job.a;
    const uint32_t* __restrict__ b = job.b;
    uint32_t* __restrict__ out = job.out;
    const int64_t na = job.na, nb = job.nb;
    const int64_t total = na + nb;
    const int64_t o0 = (int64_t)blockIdx.x * SEG;
    if (o0 >= total) return;
    const int64_t o1 = min(o0 + SEG, total);

    __shared__ int64_t split[2];
    __shared__ uint32_t buf[SEG + SEG / 32];
    if constexpr (PRESPLIT) {
        if (threadIdx.x < 2) split[threadIdx.x] = splits[blockIdx.x + threadIdx.x];
    } else
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
    const int len = la + lb;
    uint32_t k[PER];
    // all PER loads of a thread are issued before the first is consumed
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int i = (int)threadIdx.x + e * kMergeThreads;
        k[e] = kPadKey;
        if (i < la) k[e] = a[i0 + i];
        else if (i < len) k[e] = b[j0 + (i - la)];
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) buf[lds_pad((int)threadIdx.x + e * kMergeThreads)] = k[e];
    __syncthreads();

    // every thread merges PER consecutive outputs into registers
    const int d0 = min((int)threadIdx.x * PER, len);
    int ia, ib;
    {
        int lo = d0 > lb ? d0 - lb : 0, hi = d0 < la ? d0 : la;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (buf[lds_pad(mid)] <= buf[lds_pad(la + d0 - 1 - mid)]) lo = mid + 1; else hi = mid;
        }
        ia = lo;
        ib = d0 - lo;
    }
    uint32_t ka = ia < la ? buf[lds_pad(ia)] : kPadKey, kb = ib < lb ? buf[lds_pad(la + ib)] : kPadKey;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const bool take_a = ib >= lb || (ia < la && ka <= kb);
        k[e] = take_a ? ka : kb;
        if (take_a) {
            ++ia;
            ka = ia < la ? buf[lds_pad(ia)] : kPadKey;
        } else {
            ++ib;
            kb = ib < lb ? buf[lds_pad(la + ib)] : kPadKey;
        }
    }
    __syncthreads();
    // through LDS again, so that the segment leaves in whole 16-byte pieces per lane
#pragma unroll
    for (int e = 0; e < PER; ++e) buf[lds_pad((int)threadIdx.x * PER + e)] = k[e];
    __syncthreads();
    uint32_t* o = out + o0;
    for (int i = (int)threadIdx.x * 4; i < len; i += kMergeThreads * 4) {
        if (i + 4 <= len) {
            uint4 v;
            v.x = buf[lds_pad(i)];
            v.y = buf[lds_pad(i + 1)];
            v.z = buf[lds_pad(i + 2)];
            v.w = buf[lds_pad(i + 3)];
            *reinterpret_cast<uint4*>(o + i) = v;
        } else {
            for (int r = i; r < len; ++r) o[r] = buf[lds_pad(r)];
        }
    }
    if constexpr (EMIT) {
#pragma unroll
        for (int lvl = 0; lvl < kIndexLevels; ++lvl) {
            const int shift = kFanBits * (lvl + 1);
            if (((int64_t)1 << shift) <= SEG) {
                for (int t = threadIdx.x; (t << shift) < len; t += kMergeThreads)
                    job.index[lvl][(o0 >> shift) + t] = buf[lds_pad(t << shift)];
            } else if (threadIdx.x == 0 && (o0 & (((int64_t)1 << shift) - 1)) == 0) {
                job.index[lvl][o0 >> shift] = buf[lds_pad(0)];
            }
        }
    }
}

// ---- classification ----------------------------------------------------------------------------------
struct ClassifyLevels {
    int64_t r[ATTS_MAX_ALPHAS];   // reject ranks floor(alpha_l (N + 1))
    int32_t n_alpha;
};

constexpr int kTopEntries = 8192;   // LDS copy of the coarsest level (or of every 2^top_shift-th entry of it): 32 KB

struct SearchIndex {
    const uint32_t* lvl[kIndexLevels + 1];   // lvl[0] = the sorted keys, lvl[k][j] = keys[j * 32^k]
    int64_t len[kIndexLevels + 1];
    int32_t top_level;                       // the level staged in LDS
    int32_t top_shift;
    int32_t per_thread;                      // test scores per thread
};

// One level of the index for the four test keys of a quad of lanes (lane l of the quad owns key x_l and the count
// t_l of entries of the next coarser level below it).  Result for each lane: the same count for level L, whose
// candidates are the 32 entries of one aligned 128-byte line (the whole line the L2 fetches is used).  The quad takes
// its four keys in turn: in round r all four lanes work on lane r's key, each loading and comparing a quarter
// (32 bytes) of its line, so that one load instruction of the wavefront touches 16 lines instead of 64 (the vector
// cache looks up one line per cycle: a lane-per-line load costs four times the tag look-ups).  Values move inside the
// quad by DPP, not through LDS.  Every lane of the quad must be active; a lane without work passes t = 0 (nothing is
// loaded for it).
template <int CTRL>
__device__ __forceinline__ int quad_perm(int v) { return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true); }

__device__ __forceinline__ int quad_descend(const uint32_t* __restrict__ L, int64_t len, int t, uint32_t x) {
    const int q = threadIdx.x & 3;
    int out = 0;
    auto round = [&](int xr_, int tr, int r) {
        const uint32_t xr = (uint32_t)xr_;
        int c = 0;
        const int base = (tr - 1) << kFanBits;
        if (tr > 0) {
            const uint4 v0 = *reinterpret_cast<const uint4*>(L + base + 8 * q);
            const uint4 v1 = *reinterpret_cast<const uint4*>(L + base + 8 * q + 4);
            const int valid = (int)min((int64_t)kFan, len - base) - 8 * q;     // entries of this quarter that exist
            c = ((valid > 0 && v0.x < xr) ? 1 : 0) + ((valid > 1 && v0.y < xr) ? 1 : 0) + ((valid > 2 && v0.z < xr) ? 1 : 0) +
                ((valid > 3 && v0.w < xr) ? 1 : 0) + ((valid > 4 && v1.x < xr) ? 1 : 0) + ((valid > 5 && v1.y < xr) ? 1 : 0) +
                ((valid > 6 && v1.z < xr) ? 1 : 0) + ((valid > 7 && v1.w < xr) ? 1 : 0);
        }
        c += quad_perm<0xB1>(c);      // lanes (1, 0, 3, 2)
        c += quad_perm<0x4E>(c);      // lanes (2, 3, 0, 1)
        if (q == r) out = tr > 0 ? base + c : 0;
    };
    round(quad_perm<0x00>((int)x), quad_perm<0x00>(t), 0);
    round(quad_perm<0x55>((int)x), quad_perm<0x55>(t), 1);
    round(quad_perm<0xAA>((int)x), quad_perm<0xAA>(t), 2);
    round(quad_perm<0xFF>((int)x), quad_perm<0xFF>(t), 3);
    return out;
}

__global__ __launch_bounds__(256) void classify_kernel(SearchIndex ix, const float* __restrict__ test, int64_t m,
                                                       ClassifyLevels lv, int32_t* __restrict__ ranks,
                                                       float* __restrict__ pvalues, uint8_t* __restrict__ classes,
                                                       float* __restrict__ thresholds) {
    __shared__ uint32_t top[kTopEntries];
    const uint32_t* __restrict__ T = ix.lvl[ix.top_level];
    const int64_t top_len = ix.len[ix.top_level], n = ix.len[0];
    const int s = ix.top_shift;
    const int n_top = (int)((top_len + ((int64_t)1 << s) - 1) >> s);
    for (int i = threadIdx.x; i < n_top; i += 256) top[i] = T[(int64_t)i << s];
    __syncthreads();
    if (blockIdx.x == 0 && thresholds && (int)threadIdx.x < lv.n_alpha) {
        const int64_t kth = n + 1 - lv.r[threadIdx.x];     // 1-indexed order statistic
        thresholds[threadIdx.x] = kth > n ? INFINITY : (kth < 1 ? -INFINITY : key_to_score(ix.lvl[0][kth - 1]));
    }
    for (int j = 0; j < ix.per_thread; ++j) {
        const int64_t i0 = ((int64_t)blockIdx.x * ix.per_thread + j) * 256;      // block-uniform: whole quads stay in the loop
        if (i0 >= m) break;
        const int64_t i = i0 + threadIdx.x;
        const float sc = i < m ? test[i] : __uint_as_float(0x7FC00000u);
        const bool searching = !score_is_nan(sc);
        const uint32_t x = score_to_key(sc);
        int t = 0;                                             // number of entries of the current level below x
        if (searching) {
            int lo = 0, hi = n_top;                            // number of staged entries < x
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (top[mid] < x) lo = mid + 1; else hi = mid;
            }
            t = lo;
            if (s > 0 && lo > 0) {
                const int64_t w0 = ((int64_t)(lo - 1) << s) + 1;
                const int64_t w1 = min(top_len, (int64_t)lo << s);
                t = (int)(w0 + lower_bound(T + w0, w1 - w0, x));
            }
        }
#pragma unroll
        for (int l = kIndexLevels - 1; l >= 0; --l)
            if (l < ix.top_level) t = quad_descend(ix.lvl[l], ix.len[l], t, x);      // a NaN or absent score carries t = 0 down
        if (i >= m) continue;
        const int64_t c = searching ? n - t : 0;
        ranks[i] = (int32_t)c;
        if (pvalues) pvalues[i] = (float)((double)(c + 1) / (double)(n + 1));
        int cls = 0;
        for (int l = 0; l < lv.n_alpha; ++l) cls += (c + 1 <= lv.r[l]) ? 1 : 0;
        classes[i] = (uint8_t)cls;
    }
}

// ---- classes only: the decision rule in its quantile form (Eq. "quantile") ------------------------------------
// ranks + 1 <= r_l  <=>  fewer than r_l calibration scores are >= s  <=>  s > the (N + 1 - r_l)-th smallest one.
// With the thresholds read from the sorted array once, a class costs n_alpha integer compares and no search:
// a pure streaming pass.  r_l = 0 never rejects, r_l > N always does; a NaN test score (rank 0) is rejected by
// every level with r_l >= 1.
__global__ __launch_bounds__(256) void classify_threshold_kernel(const uint32_t* __restrict__ keys, int64_t n,
                                                                 const float* __restrict__ test, int64_t m, ClassifyLevels lv,
                                                                 uint8_t* __restrict__ classes, float* __restrict__ thresholds) {
    __shared__ uint32_t q_key[ATTS_MAX_ALPHAS];
    if ((int)threadIdx.x < lv.n_alpha) {
        const int64_t kth = n + 1 - lv.r[threadIdx.x];        // 1-indexed order statistic
        const uint32_t qk = (kth >= 1 && kth <= n) ? keys[kth - 1] : 0u;
        q_key[threadIdx.x] = qk;
        if (blockIdx.x == 0 && thresholds)
            thresholds[threadIdx.x] = kth > n ? INFINITY : (kth < 1 ? -INFINITY : key_to_score(qk));
    }
    __syncthreads();
    auto classify_one = [&](float s) {
        const bool nan = score_is_nan(s);
        const uint32_t x = score_to_key(s);
        int cls = 0;
        for (int l = 0; l < lv.n_alpha; ++l) {
            const int64_t r = lv.r[l];
            const bool rej = r > n ? true : (r < 1 ? false : (nan ? true : x > q_key[l]));
            cls += rej ? 1 : 0;
        }
        return (uint32_t)cls;
    };
    // four scores per thread and step: one 16-byte load, one 4-byte store (both arrays are 16- / 4-byte aligned at
    // index 0 whenever the caller's pointers are; a misaligned pair or the tail goes one by one)
    const int64_t stride = (int64_t)gridDim.x * 256;
    const bool vec = ((reinterpret_cast<uintptr_t>(test) & 15) | (reinterpret_cast<uintptr_t>(classes) & 3)) == 0;
    const int64_t m4 = vec ? m / 4 : 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < m4; i += stride) {
        const float4 s4 = reinterpret_cast<const float4*>(test)[i];
        const uint32_t packed = classify_one(s4.x) | (classify_one(s4.y) << 8) | (classify_one(s4.z) << 16) | (classify_one(s4.w) << 24);
        reinterpret_cast<uint32_t*>(classes)[i] = packed;
    }
    for (int64_t i = m4 * 4 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < m; i += stride) classes[i] = (uint8_t)classify_one(test[i]);
}

// ---- conditional coverage: one wavefront per input, its own calibration scores as the set ------------------
struct ConditionalLevels {
    double alpha[ATTS_MAX_ALPHAS];
    int32_t n_alpha;
};

__global__ __launch_bounds__(256) void conditional_kernel(const float* __restrict__ cal, const int64_t* __restrict__ cal_off,
                                                          const float* __restrict__ test, const int64_t* __restrict__ test_off,
                                                          int64_t n_inputs, ConditionalLevels lv, int32_t* __restrict__ ranks,
                                                          float* __restrict__ pvalues, uint8_t* __restrict__ classes) {
    const int lane = threadIdx.x & 63;
    const int64_t x = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (x >= n_inputs) return;                                   // whole wavefronts leave together
    const int64_t c0 = cal_off[x], t0 = test_off[x];
    const int64_t m = max((int64_t)0, cal_off[x + 1] - c0), k = max((int64_t)0, test_off[x + 1] - t0);
    int64_t r[ATTS_MAX_ALPHAS];
#pragma unroll
    for (int l = 0; l < ATTS_MAX_ALPHAS; ++l) r[l] = l < lv.n_alpha ? (int64_t)floor(lv.alpha[l] * (double)(m + 1)) : 0;
    // 64 candidates at a time, one per lane; the calibration scores pass by in blocks of 64 held one per lane and
    // broadcast lane by lane
    for (int64_t tb = 0; tb < k; tb += 64) {
        const bool has = tb + lane < k;
        const float s = has ? test[t0 + tb + lane] : 0.f;
        const uint32_t xk = score_to_key(s);
        int64_t c = 0;
        for (int64_t cb = 0; cb < m; cb += 64) {
            const int nb = (int)min((int64_t)64, m - cb);        // wave-uniform
            const uint32_t mine = lane < nb ? score_to_key(cal[c0 + cb + lane]) : 0u;   // key 0 (NaN) never counts
            int cnt = 0;
#pragma unroll
            for (int j = 0; j < 64; ++j) {                        // lane j's key through a scalar register
                const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)mine, j);
                cnt += (j < nb && kj >= xk) ? 1 : 0;
            }
            c += cnt;
        }
        if (!has) continue;
        if (score_is_nan(s)) c = 0;
        const int64_t t = t0 + tb + lane;
        ranks[t] = (int32_t)c;
        if (pvalues) pvalues[t] = (float)((double)(c + 1) / (double)(m + 1));
        int cls = 0;
#pragma unroll
        for (int l = 0; l < ATTS_MAX_ALPHAS; ++l) cls += (l < lv.n_alpha && c + 1 <= r[l]) ? 1 : 0;
        classes[t] = (uint8_t)cls;
    }
}

__global__ void export_kernel(const uint32_t* __restrict__ keys, int64_t n, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = key_to_score(keys[i]);
}

// keys and the four index levels of an array that is already in key order
struct ImportJob {
    uint32_t* keys;
    uint32_t* index[kIndexLevels];
};
__global__ void import_kernel(const float* __restrict__ scores, int64_t n, ImportJob job) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t k = score_to_key(scores[i]);
    job.keys[i] = k;
#pragma unroll
    for (int lvl = 0; lvl < kIndexLevels; ++lvl) {
        const int shift = kFanBits * (lvl + 1);
        if ((i & (((int64_t)1 << shift) - 1)) == 0) job.index[lvl][i >> shift] = k;
    }
}

// One merge launch producing `total` outputs.
template <bool EMIT>
int32_t launch_merge(atts_calib* c, const MergeJob& job, int64_t total, bool streaming, hipStream_t stream) {
    if (streaming) {
        const int64_t segs = ceil_div(total, kMergeSegLarge);
        if (segs + 1 <= c->splits_len) {
            hipLaunchKernelGGL(merge_split_kernel, dim3((unsigned)ceil_div(segs + 1, 256)), dim3(256), 0, stream, job,
                               kMergeSegLarge, (int)segs, c->splits);
            ATTS_LAUNCH_CHECK("merge_split_kernel");
            hipLaunchKernelGGL((merge_kernel<kMergeSegLarge, EMIT, true>), dim3((unsigned)segs), dim3(kMergeThreads), 0, stream, job, c->splits);
        } else {
            hipLaunchKernelGGL((merge_kernel<kMergeSegLarge, EMIT, false>), dim3((unsigned)segs), dim3(kMergeThreads), 0, stream, job, nullptr);
        }
    } else {
        hipLaunchKernelGGL((merge_kernel<kMergeSegSmall, EMIT, false>), dim3((unsigned)ceil_div(total, kMergeSegSmall)), dim3(kMergeThreads), 0,
                           stream, job, nullptr);
    }
    ATTS_LAUNCH_CHECK("merge_kernel");
    return ATTS_OK;
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
    // Every array is rounded up to whole 128-byte lines plus one: the index search reads whole lines (entries
    // past the fill are masked, not avoided).  Sorted runs are padded to whole chunks only in LDS.
    uint32_t** bufs[5 + 2 * kIndexLevels] = {&c->keys[0], &c->keys[1], &c->runs, &c->batch, &c->sort_scratch};
    int64_t sizes[5 + 2 * kIndexLevels];
    for (int i = 0; i < 4; ++i) sizes[i] = capacity;
    sizes[4] = sort_scratch_words(capacity);
    for (int side = 0; side < 2; ++side)
        for (int k = 0; k < kIndexLevels; ++k) {
            bufs[5 + side * kIndexLevels + k] = &c->index[side][k];
            sizes[5 + side * kIndexLevels + k] = ceil_div(capacity, (int64_t)1 << (kFanBits * (k + 1)));
        }
    constexpr int n_bufs = 5 + 2 * kIndexLevels;
    for (int i = 0; i < n_bufs; ++i) *bufs[i] = nullptr;
    for (int i = 0; i < n_bufs; ++i) {
        const size_t bytes = ((size_t)ceil_div(sizes[i], kFan) * kFan + kFan) * sizeof(uint32_t);
        hipError_t e = hipMalloc(reinterpret_cast<void**>(bufs[i]), bytes);
        if (e != hipSuccess) {
            for (int j = 0; j < n_bufs; ++j)
                if (*bufs[j]) (void)hipFree(*bufs[j]);
            delete c;
            return fail(ATTS_ERR_HIP, "atts_calib_create: hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        }
    }
    c->splits_len = capacity / kMergeSegLarge + 64;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->splits), (size_t)c->splits_len * sizeof(int32_t));
    if (e != hipSuccess) {
        for (int j = 0; j < n_bufs; ++j) (void)hipFree(*bufs[j]);
        delete c;
        return fail(ATTS_ERR_HIP, "atts_calib_create: hipMalloc of the split table failed: %s", hipGetErrorString(e));
    }
    *out = c;
    return ATTS_OK;
}

int32_t atts_calib_destroy(atts_calib* c) {
    if (!c) return ATTS_OK;
    (void)hipFree(c->splits);
    (void)hipFree(c->keys[0]);
    (void)hipFree(c->keys[1]);
    for (int side = 0; side < 2; ++side)
        for (int k = 0; k < kIndexLevels; ++k) (void)hipFree(c->index[side][k]);
    (void)hipFree(c->runs);
    (void)hipFree(c->batch);
    (void)hipFree(c->sort_scratch);
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

    // 1. ascending keys of the new scores
    const uint32_t* sorted = nullptr;
    {
        StageTimer t_(ATTS_STAGE_CALIB_SORT, stream);
        int32_t rc = launch_sort_scores(new_scores, n_new, c->runs, c->batch, c->sort_scratch, &sorted, stream);
        if (rc != ATTS_OK) return rc;
    }

    // 2. merge with the resident array into the other half of the ping-pong buffer (+ its search index)
    const int to = c->cur ^ 1;
    MergeJob job{c->keys[c->cur], c->n, sorted, n_new, c->keys[to], {}};
    for (int k = 0; k < kIndexLevels; ++k) job.index[k] = c->index[to][k];
    const int64_t total = c->n + n_new;
    StageTimer t_(ATTS_STAGE_CALIB_MERGE, stream);
    int32_t rc = launch_merge<true>(c, job, total, total >= kMergeLargeFrom, stream);
    if (rc != ATTS_OK) return rc;
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
    if (M > 0 && (!test_scores || !classes))
        return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: test_scores and classes must not be NULL");
    if (!ranks && pvalues) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: pvalues without ranks");
    if (M > ((int64_t)1 << 31) * 255) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_ordinal: M too large");
    ClassifyLevels lv;
    lv.n_alpha = n_alpha;
    for (int l = 0; l < ATTS_MAX_ALPHAS; ++l) lv.r[l] = 0;
    for (int l = 0; l < n_alpha; ++l) lv.r[l] = (int64_t)floor(alphas[l] * (double)(c->n + 1));
    if (M == 0 && !thresholds) return ATTS_OK;
    if (!ranks) {
        // decisions only: compare with the thresholds, no search
        const int64_t want = M > 0 ? ceil_div(M, (int64_t)256 * 16) : 1;
        const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 4096 ? 4096 : want));
        StageTimer t_(ATTS_STAGE_CLASSIFY, static_cast<hipStream_t>(hip_stream));
        hipLaunchKernelGGL(classify_threshold_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                           c->keys[c->cur], c->n, test_scores, M, lv, classes, thresholds);
        ATTS_LAUNCH_CHECK("classify_threshold_kernel");
        return ATTS_OK;
    }
    SearchIndex ix;
    ix.lvl[0] = c->keys[c->cur];
    ix.len[0] = c->n;
    for (int k = 1; k <= kIndexLevels; ++k) {
        ix.lvl[k] = c->index[c->cur][k - 1];
        ix.len[k] = ceil_div(c->n, (int64_t)1 << (kFanBits * k));
    }
    ix.top_level = 0;
    while (ix.top_level < kIndexLevels && ix.len[ix.top_level] > kTopEntries) ++ix.top_level;
    ix.top_shift = 0;
    while (ceil_div(ix.len[ix.top_level], (int64_t)1 << ix.top_shift) > kTopEntries) ++ix.top_shift;
    // enough workgroups to fill the chip, few enough that staging the top level stays a small part of the work
    int64_t per = M / ((int64_t)256 * 2048);
    ix.per_thread = (int32_t)(per < 1 ? 1 : (per > 16 ? 16 : per));
    const unsigned blocks = (unsigned)(M > 0 ? ceil_div(M, (int64_t)256 * ix.per_thread) : 1);
    StageTimer t_(ATTS_STAGE_CLASSIFY, static_cast<hipStream_t>(hip_stream));
    hipLaunchKernelGGL(classify_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), ix, test_scores, M,
                       lv, ranks, pvalues, classes, thresholds);
    ATTS_LAUNCH_CHECK("classify_kernel");
    return ATTS_OK;
}

int32_t atts_classify_conditional(const float* cal_scores, const int64_t* cal_offsets, const float* test_scores,
                                  const int64_t* test_offsets, int64_t n_inputs, const double* alphas, int32_t n_alpha,
                                  int32_t* ranks, float* pvalues, uint8_t* classes, void* hip_stream) {
    if (n_inputs < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: n_inputs = %lld < 0", (long long)n_inputs);
    if (!alphas || n_alpha < 1 || n_alpha > ATTS_MAX_ALPHAS)
        return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: need 1..%d alpha levels", ATTS_MAX_ALPHAS);
    ConditionalLevels lv;
    lv.n_alpha = n_alpha;
    for (int l = 0; l < ATTS_MAX_ALPHAS; ++l) lv.alpha[l] = 0.0;
    for (int l = 0; l < n_alpha; ++l) {
        if (!(alphas[l] > 0.0 && alphas[l] < 1.0))
            return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: alpha[%d] = %g is not inside (0, 1)", l, alphas[l]);
        if (l > 0 && alphas[l] < alphas[l - 1])
            return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: alpha levels must be non-decreasing");
        lv.alpha[l] = alphas[l];
    }
    if (n_inputs == 0) return ATTS_OK;
    if (!cal_offsets || !test_offsets) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: offsets must not be NULL");
    // score and output arrays may be NULL only if every range is empty, which the host cannot see: require them
    if (!cal_scores || !test_scores || !ranks || !classes)
        return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: cal_scores, test_scores, ranks and classes must not be NULL");
    if (n_inputs > ((int64_t)1 << 31) * 2) return fail(ATTS_ERR_INVALID_ARG, "atts_classify_conditional: too many inputs");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    StageTimer t_(ATTS_STAGE_CLASSIFY, stream);
    hipLaunchKernelGGL(conditional_kernel, dim3((unsigned)ceil_div(n_inputs, 4)), dim3(256), 0, stream, cal_scores, cal_offsets,
                       test_scores, test_offsets, n_inputs, lv, ranks, pvalues, classes);
    ATTS_LAUNCH_CHECK("conditional_kernel");
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

int32_t atts_calib_import(atts_calib* c, const float* scores, int64_t n, void* hip_stream) {
    if (!c) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_import: NULL handle");
    if (n < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_import: n = %lld < 0", (long long)n);
    if (n > c->capacity)
        return fail(ATTS_ERR_CAPACITY, "atts_calib_import: %lld scores exceed the capacity %lld", (long long)n, (long long)c->capacity);
    if (n > 0 && !scores) return fail(ATTS_ERR_INVALID_ARG, "atts_calib_import: scores is NULL");
    if (n > 0) {
        ImportJob job{c->keys[c->cur], {}};
        for (int k = 0; k < kIndexLevels; ++k) job.index[k] = c->index[c->cur][k];
        hipLaunchKernelGGL(import_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), scores, n, job);
        ATTS_LAUNCH_CHECK("import_kernel");
    }
    c->n = n;
    return ATTS_OK;
}

}  // extern "C"
