// The classic, synchronous conformal pipeline (Sec. "Preliminary", "Classic Setup"): the comparator of the
// asynchronous design.  Three steps, each needing data the asynchronous rule never waits for:
//   normalise   Eq. "softmax": the score of candidate k of an input is its share exp(-l_k) / sum_j exp(-l_j) of the
//               likelihood of ALL m candidates of that input, so no candidate can be scored before the m-th arrives;
//   threshold   Eq. "quantile": tau = an order statistic of ALL normalised calibration scores: a global sort;
//   sets        Eq. "pred_set": C(X_i) = {k : s_i^k >= tau}.
// The time of these launches, plus the wait for the slowest candidate in front of them, is the synchronisation term
// T_s of the asynchronous arithmetic intensity (Sec. "Q1").
#include "common.h"
#include "keys.h"

#include <math.h>

namespace atts {
namespace {

// One wavefront per input: minimum of the m losses, sum of exp(min - l), then the shares.  fp32 throughout
// (the unnormalised scores are fp32); the sum is taken in a fixed order (lane-strided partial sums, then a butterfly).
__global__ __launch_bounds__(256) void classic_normalize_kernel(const float* __restrict__ nll, int64_t n, int32_t m,
                                                                float* __restrict__ s) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;                                         // whole wavefronts leave together
    const float* __restrict__ row = nll + i * m;
    float* __restrict__ out = s + i * m;
    float lo = INFINITY;
    for (int k = lane; k < m; k += 64) lo = fminf(lo, row[k]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lo = fminf(lo, __shfl_xor(lo, o));
    float sum = 0.f;
    for (int k = lane; k < m; k += 64) sum += expf(lo - row[k]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    for (int k = lane; k < m; k += 64) out[k] = expf(lo - row[k]) / sum;
}

// tau = score of the kth smallest key (1-indexed); +inf above the range, -inf below
__global__ void classic_pick_kernel(const uint32_t* __restrict__ sorted, int64_t n, int64_t kth, float* __restrict__ tau) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *tau = kth > n ? INFINITY : (kth < 1 ? -INFINITY : key_to_score(sorted[kth - 1]));
}

// member[i] = s[i] >= tau (IEEE: a NaN on either side is not a member)
__global__ __launch_bounds__(256) void classic_sets_kernel(const float* __restrict__ s, int64_t count, const float* __restrict__ tau,
                                                           uint8_t* __restrict__ member) {
    const float t = *tau;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) member[i] = s[i] >= t ? 1 : 0;
}

// workspace: two key buffers of n rounded up to 16, plus 16, words each, then the sort's scratch
int64_t key_buffer_words(int64_t n) { return ceil_div(n, 16) * 16 + 16; }

}  // namespace
}  // namespace atts

using namespace atts;

extern "C" {

int32_t atts_classic_workspace_bytes(int64_t n_scores, size_t* out_bytes) {
    if (!out_bytes) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_workspace_bytes: out_bytes is NULL");
    if (n_scores < 1 || n_scores > ((int64_t)1 << 30))
        return fail(ATTS_ERR_INVALID_ARG, "atts_classic_workspace_bytes: n_scores = %lld outside [1, 2^30]", (long long)n_scores);
    *out_bytes = align_up((size_t)(2 * key_buffer_words(n_scores) + sort_scratch_words(n_scores)) * sizeof(uint32_t), 256);
    return ATTS_OK;
}

int32_t atts_classic_normalize(const float* nll, int64_t n_inputs, int32_t m, float* scores, void* hip_stream) {
    if (n_inputs < 0 || m < 1) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_normalize: need n_inputs >= 0 and m >= 1");
    if (n_inputs == 0) return ATTS_OK;
    if (!nll || !scores) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_normalize: NULL argument");
    if (n_inputs > ((int64_t)1 << 31) * 2) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_normalize: too many inputs");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(classic_normalize_kernel, dim3((unsigned)ceil_div(n_inputs, 4)), dim3(256), 0, stream, nll, n_inputs, m, scores);
    ATTS_LAUNCH_CHECK("classic_normalize_kernel");
    return ATTS_OK;
}

int32_t atts_classic_threshold(const float* cal_scores, int64_t n_scores, double alpha, float* tau, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
    if (!cal_scores || !tau) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_threshold: NULL argument");
    if (!(alpha > 0.0 && alpha < 1.0)) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_threshold: alpha = %g is not inside (0, 1)", alpha);
    size_t need = 0;
    int32_t rc = atts_classic_workspace_bytes(n_scores, &need);
    if (rc != ATTS_OK) return rc;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need)
        return fail(ATTS_ERR_WORKSPACE, "atts_classic_threshold: workspace missing, misaligned or smaller than %zu bytes", need);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t* a = static_cast<uint32_t*>(workspace);
    uint32_t* b = a + key_buffer_words(n_scores);
    uint32_t* scratch = b + key_buffer_words(n_scores);
    const uint32_t* sorted = nullptr;
    rc = launch_sort_scores(cal_scores, n_scores, a, b, scratch, &sorted, stream);
    if (rc != ATTS_OK) return rc;
    const int64_t kth = n_scores + 1 - (int64_t)floor(alpha * (double)(n_scores + 1));
    hipLaunchKernelGGL(classic_pick_kernel, dim3(1), dim3(64), 0, stream, sorted, n_scores, kth, tau);
    ATTS_LAUNCH_CHECK("classic_pick_kernel");
    return ATTS_OK;
}

int32_t atts_classic_prediction_sets(const float* scores, int64_t count, const float* tau, uint8_t* member, void* hip_stream) {
    if (count < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_prediction_sets: count = %lld < 0", (long long)count);
    if (count == 0) return ATTS_OK;
    if (!scores || !tau || !member) return fail(ATTS_ERR_INVALID_ARG, "atts_classic_prediction_sets: NULL argument");
    const int64_t want = ceil_div(count, (int64_t)256 * 4);
    hipLaunchKernelGGL(classic_sets_kernel, dim3((unsigned)(want > 4096 ? 4096 : want)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), scores, count, tau, member);
    ATTS_LAUNCH_CHECK("classic_sets_kernel");
    return ATTS_OK;
}

}  // extern "C"
