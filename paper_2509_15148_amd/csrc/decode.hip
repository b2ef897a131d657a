// Kernels of the target-model continuation ("Target Model Sampling"): one new token per continued candidate and step.
//
// The candidates continue different drafts of the same prompt, so their keys / values form the same token tree as
// in scoring: a shared prefix and one branch per candidate.  During a continuation call the keys (after RoPE) and
// values of the whole tree live per layer in a row-major cache
//     rows [0, P): prefix        rows P + j Tc + t: token t of branch j  (Tc = draft length + tokens to generate)
// and a decode step sends one row per branch through the model.
#include "common.h"

namespace atts {
namespace {

// rows [P, P + K T) of the scoring layout (branch j at P + j T) -> the cache layout (branch j at P + j Tc);
// `cols` consecutive elements per row, source pitch src_ld, destination pitch dst_ld.
template <typename T>
__global__ __launch_bounds__(256) void tree_rows_to_cache_kernel(const T* __restrict__ src, int64_t src_ld, T* __restrict__ dst,
                                                                 int64_t dst_ld, int P, int Tn, int Tc, int rows, int cols) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)rows * cols) return;
    const int r = (int)(i / cols), c = (int)(i % cols);           // r counts draft rows
    const int64_t dst_row = P + (int64_t)(r / Tn) * Tc + r % Tn;
    dst[dst_row * dst_ld + c] = src[(int64_t)(P + r) * src_ld + c];
}

// dst[r][c] = src[c][r]: the transposed value cache of a prefix handle -> value rows
template <typename T>
__global__ __launch_bounds__(256) void transpose_to_rows_kernel(const T* __restrict__ src, int64_t src_ld, T* __restrict__ dst,
                                                                int64_t dst_ld, int rows, int cols) {
    __shared__ T tile[64][65];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) tile[i][tx] = src[(int64_t)c * src_ld + r];
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        if (c < cols && r < rows) dst[(int64_t)r * dst_ld + c] = tile[tx][i];
    }
}

// h[j] = embedding of ids[j * stride]  (an id outside the vocabulary is read as 0 and sets the flag)
template <typename T>
__global__ __launch_bounds__(256) void embed_rows_kernel(const T* __restrict__ emb, int vocab, int d, const int32_t* __restrict__ ids,
                                                         int64_t stride, float* __restrict__ h, int32_t* __restrict__ err_flag) {
    const int j = blockIdx.x;
    int id = ids[(int64_t)j * stride];
    if (id < 0 || id >= vocab) {
        if (threadIdx.x == 0) *err_flag = 1;
        id = 0;
    }
    const T* src = emb + (int64_t)id * d;
    for (int c = threadIdx.x; c < d; c += 256) h[(int64_t)j * d + c] = to_f32<T>(src[c]);
}

// One decode row per branch: acc [Kr, (nq + 2 nkv) hd] fp32 (cleared on return) -> q (rotated) to q_out [Kr, nq hd]; k (rotated) and v
// to row `P + j Tc + t_new` of the layer's key / value cache.  cs: the (cos, sin) row of the new position.
template <typename T>
__global__ __launch_bounds__(256) void decode_qkv_finish_kernel(float* __restrict__ acc, const float2* __restrict__ cs, int Kr,
                                                                int nq, int nkv, int hd, int P, int Tc, int t_new,
                                                                T* __restrict__ q_out, T* __restrict__ k_cache,
                                                                T* __restrict__ v_cache) {
    const int half = hd >> 1, heads = nq + 2 * nkv;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)Kr * heads * half) return;
    const int i = (int)(idx % half);
    const int head = (int)((idx / half) % heads);
    const int j = (int)(idx / ((int64_t)half * heads));
    float* a = acc + (int64_t)j * heads * hd + head * hd + i;
    const float x1 = a[0], x2 = a[half];
    a[0] = 0.f;                                  // left clear for a K-split projection that adds into it
    a[half] = 0.f;
    const int64_t crow = P + (int64_t)j * Tc + t_new;
    if (head < nq + nkv) {
        const float2 c_s = cs[i];
        const float y1 = x1 * c_s.x - x2 * c_s.y, y2 = x2 * c_s.x + x1 * c_s.y;
        T* p = head < nq ? q_out + (int64_t)j * nq * hd + head * hd + i : k_cache + crow * nkv * hd + (head - nq) * hd + i;
        p[0] = from_f32<T>(y1);
        p[half] = from_f32<T>(y2);
    } else {
        T* p = v_cache + crow * nkv * hd + (head - nq - nkv) * hd + i;
        p[0] = from_f32<T>(x1);
        p[half] = from_f32<T>(x2);
    }
}

// One workgroup (kDecodeWaves wavefronts) per (branch, head): the new row of branch j attends to the prefix rows and
// to rows 0 .. t_new of its own branch.  Scores: one key per thread and pass (16-byte loads along the key row);
// output: every wavefront accumulates its share of the keys (lane = a pair of dims, 128 / 256 contiguous bytes per
// key), the partial sums are added in a fixed order.
constexpr int kDecodeWaves = 16, kDecodeThreads = 64 * kDecodeWaves;

template <typename T>
__global__ __launch_bounds__(kDecodeThreads) void attn_decode_kernel(const T* __restrict__ q, const T* __restrict__ k_cache,
                                                                     const T* __restrict__ v_cache, T* __restrict__ out, int P,
                                                                     int Tc, int t_new, int nq, int nkv, int hd, float scale) {
    extern __shared__ float sm[];           // [hd] query | [n] scores | [2 waves] reductions | [waves][hd] partial outputs
    const int n = P + t_new + 1;
    float* sq = sm;
    float* sp = sm + hd;
    float* red = sp + n;
    float* so = red + 2 * kDecodeWaves;
    const int j = blockIdx.x, head = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kvh = head / (nq / nkv);
    const int64_t ld = (int64_t)nkv * hd;
    const T* qp = q + (int64_t)j * nq * hd + head * hd;
    for (int c = tid; c < hd; c += kDecodeThreads) sq[c] = to_f32<T>(qp[c]) * scale;
    __syncthreads();
    const int64_t branch0 = P + (int64_t)j * Tc;
    auto key_row = [&](int i) { return i < P ? (int64_t)i : branch0 + (i - P); };
    constexpr int kVec = 16 / (int)sizeof(T);          // elements per 16-byte load (key rows are 16-byte aligned)
    float mx = -INFINITY;
    for (int i = tid; i < n; i += kDecodeThreads) {
        const T* k = k_cache + key_row(i) * ld + kvh * hd;
        float s = 0.f;
        if (hd % kVec == 0) {
            for (int c = 0; c < hd; c += kVec) {
                const uint4 raw = *reinterpret_cast<const uint4*>(k + c);
                const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
                for (int u = 0; u < kVec; ++u) s += sq[c + u] * to_f32<T>(e[u]);
            }
        } else {
            for (int c = 0; c < hd; ++c) s += sq[c] * to_f32<T>(k[c]);
        }
        sp[i] = s;
        mx = fmaxf(mx, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = red[0];
#pragma unroll
    for (int w = 1; w < kDecodeWaves; ++w) mx = fmaxf(mx, red[w]);
    float sum = 0.f;
    for (int i = tid; i < n; i += kDecodeThreads) {
        const float p = __expf(sp[i] - mx);
        sp[i] = p;
        sum += p;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red[kDecodeWaves + wave] = sum;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kDecodeWaves; ++w) tot += red[kDecodeWaves + w];
    const float inv = 1.f / tot;
    // output: wavefront w takes keys w, w + kDecodeWaves, ...; lane takes dims 2 c2, 2 c2 + 1 (hd is even)
    for (int c2 = lane; c2 < hd / 2; c2 += 64) {
        float a0 = 0.f, a1 = 0.f;
        const T* vbase = v_cache + kvh * hd + 2 * c2;
#pragma unroll 4
        for (int i = wave; i < n; i += kDecodeWaves) {
            const T* v = vbase + key_row(i) * ld;
            const float p = sp[i];
            a0 += p * to_f32<T>(v[0]);
            a1 += p * to_f32<T>(v[1]);
        }
        so[wave * hd + 2 * c2] = a0;
        so[wave * hd + 2 * c2 + 1] = a1;
    }
    __syncthreads();
    for (int c = tid; c < hd; c += kDecodeThreads) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) o += so[w * hd + c];
        out[(int64_t)j * nq * hd + head * hd + c] = from_f32<T>(o * inv);
    }
}

// ids[j * stride] = first index of the largest logit of row j
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ logits, int64_t ld, int V, int32_t* __restrict__ ids,
                                                          int64_t stride) {
    __shared__ float s_val[256];
    __shared__ int s_idx[256];
    const int j = blockIdx.x;
    const float* z = logits + (int64_t)j * ld;
    float best = -INFINITY;
    int at = 0x7fffffff;
    auto consider = [&](float v, int c) {               // NaN never wins; the first maximum is kept
        if (v > best || (v == best && c < at)) {
            best = v;
            at = c;
        }
    };
    const bool vec = (reinterpret_cast<uintptr_t>(z) & 15) == 0;
    const int v4 = vec ? V / 4 : 0;
#pragma unroll 4
    for (int c4 = threadIdx.x; c4 < v4; c4 += 256) {
        const float4 x = reinterpret_cast<const float4*>(z)[c4];
        consider(x.x, 4 * c4);
        consider(x.y, 4 * c4 + 1);
        consider(x.z, 4 * c4 + 2);
        consider(x.w, 4 * c4 + 3);
    }
    for (int c = 4 * v4 + threadIdx.x; c < V; c += 256) consider(z[c], c);
    s_val[threadIdx.x] = best;
    s_idx[threadIdx.x] = at;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const float v = s_val[threadIdx.x + o];
            const int c = s_idx[threadIdx.x + o];
            if (v > s_val[threadIdx.x] || (v == s_val[threadIdx.x] && c < s_idx[threadIdx.x])) {
                s_val[threadIdx.x] = v;
                s_idx[threadIdx.x] = c;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) ids[(int64_t)j * stride] = s_idx[0] == 0x7fffffff ? 0 : s_idx[0];
}

// ids[j * stride] = inverse-CDF sample of softmax(logits[j] * inv_temp) with the uniform u = uniforms[j * stride]:
// the first index v (vocabulary order) whose cumulative weight reaches u times the total.  Every thread owns a
// contiguous chunk of the row; chunk sums are scanned in index order by one thread, then the owner of the chunk the
// target falls into walks it.  Sums in fp32, fixed order.
constexpr int kSampleThreads = 1024;

__global__ __launch_bounds__(kSampleThreads) void sample_rows_kernel(const float* __restrict__ logits, int64_t ld, int V,
                                                                     float inv_temp, const float* __restrict__ uniforms,
                                                                     int32_t* __restrict__ ids, int64_t stride) {
    __shared__ float red[kSampleThreads / 64];
    __shared__ float chunk_sum[kSampleThreads];
    __shared__ float s_target, s_before;
    __shared__ int s_chunk;
    const int j = blockIdx.x, tid = threadIdx.x;
    const float* z = logits + (int64_t)j * ld;
    const int per = (V + kSampleThreads - 1) / kSampleThreads;
    const int c0 = min(tid * per, V), c1 = min(c0 + per, V);
    float mx = -INFINITY;
    for (int c = c0; c < c1; ++c) mx = fmaxf(mx, z[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = red[0];
#pragma unroll
    for (int w = 1; w < kSampleThreads / 64; ++w) mx = fmaxf(mx, red[w]);
    float sum = 0.f;
    for (int c = c0; c < c1; ++c) sum += __expf((z[c] - mx) * inv_temp);
    chunk_sum[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        float total = 0.f;
        for (int t = 0; t < kSampleThreads; ++t) total += chunk_sum[t];
        const float target = uniforms[(int64_t)j * stride] * total;
        float before = 0.f;
        int chunk = kSampleThreads - 1;
        for (int t = 0; t < kSampleThreads; ++t) {
            if (before + chunk_sum[t] >= target && chunk_sum[t] > 0.f) {
                chunk = t;
                break;
            }
            before += chunk_sum[t];
        }
        s_target = target;
        s_before = before;
        s_chunk = chunk;
    }
    __syncthreads();
    if (tid == s_chunk) {
        float run = s_before;
        int pick = -1, last_mass = -1;
        for (int c = c0; c < c1; ++c) {
            const float e = __expf((z[c] - mx) * inv_temp);
            run += e;
            if (e > 0.f) last_mass = c;
            if (run >= s_target) {
                pick = c;
                break;
            }
        }
        if (pick < 0) pick = last_mass >= 0 ? last_mass : (c1 > c0 ? c1 - 1 : V - 1);   // rounding left the target just past the chunk
        ids[(int64_t)j * stride] = pick;
    }
}

// xs[j] = rmsnorm(h[rows[j]]) with rows[j] = first + j * step
template <typename T>
__global__ __launch_bounds__(256) void norm_strided_rows_kernel(const float* __restrict__ h, const float* __restrict__ gain, float eps,
                                                                int d, int64_t first, int64_t step, T* __restrict__ xs) {
    __shared__ float red[4];
    const int j = blockIdx.x;
    const float* x = h + (first + (int64_t)j * step) * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) ss += x[c] * x[c];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float rs = rsqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) xs[(int64_t)j * d + c] = from_f32<T>(x[c] * rs * gain[c]);
}

}  // namespace

#define DISPATCH_T(dtype, ...)                       \
    if ((dtype) == ATTS_DTYPE_F32) {                 \
        typedef float T;                             \
        __VA_ARGS__                                  \
    } else {                                         \
        typedef bf16 T;                              \
        __VA_ARGS__                                  \
    }

int32_t launch_tree_rows_to_cache(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int32_t P, int32_t Tn,
                                  int32_t Tc, int32_t rows, int32_t cols, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return ATTS_OK;
    DISPATCH_T(dtype, hipLaunchKernelGGL(tree_rows_to_cache_kernel<T>, dim3((unsigned)ceil_div((int64_t)rows * cols, 256)), dim3(256), 0,
                                         stream, (const T*)src, src_ld, (T*)dst, dst_ld, P, Tn, Tc, rows, cols);)
    ATTS_LAUNCH_CHECK("tree_rows_to_cache_kernel");
    return ATTS_OK;
}

int32_t launch_transpose_to_rows(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int32_t rows,
                                 int32_t cols, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return ATTS_OK;
    dim3 grid((unsigned)ceil_div(rows, 64), (unsigned)ceil_div(cols, 64));
    DISPATCH_T(dtype, hipLaunchKernelGGL(transpose_to_rows_kernel<T>, grid, dim3(256), 0, stream, (const T*)src, src_ld, (T*)dst,
                                         dst_ld, rows, cols);)
    ATTS_LAUNCH_CHECK("transpose_to_rows_kernel");
    return ATTS_OK;
}

int32_t launch_embed_rows(int32_t dtype, const void* tok_embed, int32_t vocab, int32_t d, const int32_t* ids, int64_t stride,
                          int32_t rows, float* h, int32_t* err_flag, hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(embed_rows_kernel<T>, dim3(rows), dim3(256), 0, stream, (const T*)tok_embed, vocab, d, ids,
                                         stride, h, err_flag);)
    ATTS_LAUNCH_CHECK("embed_rows_kernel");
    return ATTS_OK;
}

int32_t launch_decode_qkv_finish(int32_t dtype, float* acc, const float2* cs, int32_t Kr, int32_t nq, int32_t nkv, int32_t hd,
                                 int32_t P, int32_t Tc, int32_t t_new, void* q_out, void* k_cache, void* v_cache,
                                 hipStream_t stream) {
    const int64_t total = (int64_t)Kr * (nq + 2 * nkv) * (hd / 2);
    DISPATCH_T(dtype, hipLaunchKernelGGL(decode_qkv_finish_kernel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, acc,
                                         cs, Kr, nq, nkv, hd, P, Tc, t_new, (T*)q_out, (T*)k_cache, (T*)v_cache);)
    ATTS_LAUNCH_CHECK("decode_qkv_finish_kernel");
    return ATTS_OK;
}

int32_t launch_attn_decode(int32_t dtype, const void* q, const void* k_cache, const void* v_cache, void* out, int32_t Kr, int32_t P,
                           int32_t Tc, int32_t t_new, int32_t nq, int32_t nkv, int32_t hd, hipStream_t stream) {
    const size_t lds = (size_t)((1 + kDecodeWaves) * hd + P + t_new + 1 + 2 * kDecodeWaves) * sizeof(float);
    if (lds > 60 * 1024) return fail(ATTS_ERR_SHAPE, "continuation: context of %d keys is too long", P + t_new + 1);
    const float scale = 1.f / sqrtf((float)hd);
    dim3 grid(Kr, nq);
    DISPATCH_T(dtype, hipLaunchKernelGGL(attn_decode_kernel<T>, grid, dim3(kDecodeThreads), lds, stream, (const T*)q, (const T*)k_cache,
                                         (const T*)v_cache, (T*)out, P, Tc, t_new, nq, nkv, hd, scale);)
    ATTS_LAUNCH_CHECK("attn_decode_kernel");
    return ATTS_OK;
}

int32_t launch_argmax_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, int32_t* ids, int64_t stride,
                           hipStream_t stream) {
    hipLaunchKernelGGL(argmax_rows_kernel, dim3(rows), dim3(256), 0, stream, logits, ld, V, ids, stride);
    ATTS_LAUNCH_CHECK("argmax_rows_kernel");
    return ATTS_OK;
}

int32_t launch_sample_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, float inv_temp, const float* uniforms,
                           int32_t* ids, int64_t stride, hipStream_t stream) {
    hipLaunchKernelGGL(sample_rows_kernel, dim3(rows), dim3(kSampleThreads), 0, stream, logits, ld, V, inv_temp, uniforms, ids, stride);
    ATTS_LAUNCH_CHECK("sample_rows_kernel");
    return ATTS_OK;
}

int32_t launch_norm_strided_rows(int32_t dtype, const float* h, const float* gain, float eps, int32_t d, int64_t first, int64_t step,
                                 int32_t rows, void* xs, hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(norm_strided_rows_kernel<T>, dim3(rows), dim3(256), 0, stream, h, gain, eps, d, first, step,
                                         (T*)xs);)
    ATTS_LAUNCH_CHECK("norm_strided_rows_kernel");
    return ATTS_OK;
}

}  // namespace atts
