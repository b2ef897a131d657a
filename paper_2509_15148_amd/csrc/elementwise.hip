// Memory-bound stages of the scoring path: embedding gather, RMSNorm, rotary embedding +
// V transpose, scoring-row gather + final norm, score reduction.
// All are HBM-bound and tiny next to the GEMMs; they are written for coalesced 16-byte
// accesses and fixed reduction orders (no float atomics, so results are run-to-run stable).
#include "common.h"

namespace atts {
namespace {

// ---- wave / block reductions -------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum over a block of kBlock threads (kBlock multiple of 64, <= 1024); result valid in all threads.
template <int kBlock>
__device__ __forceinline__ float block_sum(float v, float* red /* [kBlock / 64] */) {
    v = wave_sum(v);
    if constexpr (kBlock == 64) return v;
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kBlock / 64; ++i) t += red[i];
    return t;
}

// Row of the token tree -> (is it a draft row, which draft, which position in the draft)
__device__ __forceinline__ int tree_position(int r, int P, int T) { return r < P ? r : P + (r - P) % T; }

// ---- S0: embedding gather ------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ emb, int vocab, int d,
                                                    const int32_t* __restrict__ prefix_ids,
                                                    const int32_t* __restrict__ draft_ids,
                                                    const int32_t* __restrict__ draft_lens, int P, int Tn, int row0,
                                                    float* __restrict__ h, int32_t* __restrict__ err_flag) {
    const int r = row0 + blockIdx.x;
    int id;
    bool padding = false;
    if (r < P) {
        id = prefix_ids[r];
    } else {
        int k = (r - P) / Tn, t = (r - P) % Tn;
        id = draft_ids[(int64_t)k * Tn + t];
        padding = draft_lens && t >= draft_lens[k];
    }
    if (id < 0 || id >= vocab) {
        if (!padding && threadIdx.x == 0) *err_flag = 1;
        id = 0;
    }
    const T* src = emb + (int64_t)id * d;
    float* dst = h + (int64_t)r * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = to_f32<T>(src[c]);
}

// ---- S1: RMSNorm over rows of the fp32 residual stream ---------------------------------------
// One row per workgroup, 16-byte loads; up to 4 float4 per thread (d <= 4096) stay in registers between the
// sum-of-squares pass and the scaling pass, longer rows are read again (from L2).  d % 4 == 0.
template <typename T>
__device__ __forceinline__ void store4(T* dst, float4 v);
template <>
__device__ __forceinline__ void store4<float>(float* dst, float4 v) { *reinterpret_cast<float4*>(dst) = v; }
template <>
__device__ __forceinline__ void store4<bf16>(bf16* dst, float4 v) {
    bf16x4 o;
    o[0] = (bf16)v.x; o[1] = (bf16)v.y; o[2] = (bf16)v.z; o[3] = (bf16)v.w;
    *reinterpret_cast<bf16x4*>(dst) = o;
}

template <typename T>
__device__ __forceinline__ void rmsnorm_row(const float* __restrict__ x, const float* __restrict__ gain, float eps, int d,
                                            T* __restrict__ o, float* red) {
    constexpr int kKeep = 4;
    const int n4 = d >> 2;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    float4 keep[kKeep];
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        const int c = threadIdx.x + 256 * q;
        keep[q] = c < n4 ? x4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        ss += keep[q].x * keep[q].x + keep[q].y * keep[q].y + keep[q].z * keep[q].z + keep[q].w * keep[q].w;
    }
    for (int c = threadIdx.x + 256 * kKeep; c < n4; c += 256) {
        const float4 v = x4[c];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = block_sum<256>(ss, red);
    const float inv = rsqrtf(ss / (float)d + eps);
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        const int c = threadIdx.x + 256 * q;
        if (c < n4) {
            const float4 g = g4[c];
            store4<T>(o + 4 * c, make_float4(keep[q].x * inv * g.x, keep[q].y * inv * g.y, keep[q].z * inv * g.z,
                                             keep[q].w * inv * g.w));
        }
    }
    for (int c = threadIdx.x + 256 * kKeep; c < n4; c += 256) {
        const float4 v = x4[c], g = g4[c];
        store4<T>(o + 4 * c, make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h, const float* __restrict__ gain,
                                                      float eps, int d, T* __restrict__ out) {
    __shared__ float red[4];
    rmsnorm_row<T>(h + (int64_t)blockIdx.x * d, gain, eps, d, out + (int64_t)blockIdx.x * d, red);
}

// ---- residual update from K-slice partial sums, fused with the next RMSNorm ------------------------------
// One row per workgroup: h[r] += part[0][r] + part[1][r] + ... (slice order, so the sum does not depend on which
// workgroup of the projection finished first), then, with a gain vector, out[r] = rmsnorm(h[r]).  Up to 4 float4 per
// thread stay in registers between the passes; longer rows are read back (each thread re-reads what it wrote itself).
template <typename T>
__global__ __launch_bounds__(256) void resid_norm_kernel(float* __restrict__ h, const float* __restrict__ part, int n_slices,
                                                         int64_t pitch, const float* __restrict__ gain, float eps, int d,
                                                         T* __restrict__ out) {
    __shared__ float red[4];
    constexpr int kKeep = 4;
    const int n4 = d >> 2;
    float4* x4 = reinterpret_cast<float4*>(h + (int64_t)blockIdx.x * d);
    const float4* p4 = reinterpret_cast<const float4*>(part + (int64_t)blockIdx.x * d);
    const int64_t pitch4 = pitch >> 2;
    // the slices are requested four at a time for all of the thread's chunks (16 independent loads in flight: with few
    // rows this kernel is a handful of workgroups whose time is the latency of their loads), then added in slice order;
    // a slice past the last one contributes +0
    float4 keep[kKeep];
    constexpr int kBatch = 4;
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        const int c = threadIdx.x + 256 * q;
        keep[q] = c < n4 ? x4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int s0 = 0; s0 < n_slices; s0 += kBatch) {
        float4 t[kBatch][kKeep];
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
#pragma unroll
            for (int q = 0; q < kKeep; ++q) {
                const int c = threadIdx.x + 256 * q;
                t[u][q] = (s0 + u < n_slices && c < n4) ? p4[(s0 + u) * pitch4 + c] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
#pragma unroll
            for (int q = 0; q < kKeep; ++q) {
                keep[q].x += t[u][q].x; keep[q].y += t[u][q].y; keep[q].z += t[u][q].z; keep[q].w += t[u][q].w;
            }
    }
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        const int c = threadIdx.x + 256 * q;
        if (c < n4) x4[c] = keep[q];
        ss += keep[q].x * keep[q].x + keep[q].y * keep[q].y + keep[q].z * keep[q].z + keep[q].w * keep[q].w;
    }
    for (int c = threadIdx.x + 256 * kKeep; c < n4; c += 256) {
        float4 v = x4[c];
        for (int s0 = 0; s0 < n_slices; s0 += kBatch) {
            float4 t[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) t[u] = s0 + u < n_slices ? p4[(s0 + u) * pitch4 + c] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) { v.x += t[u].x; v.y += t[u].y; v.z += t[u].z; v.w += t[u].w; }
        }
        x4[c] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    if (!gain) return;                                          // block-uniform
    ss = block_sum<256>(ss, red);
    const float inv = rsqrtf(ss / (float)d + eps);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    T* o = out + (int64_t)blockIdx.x * d;
#pragma unroll
    for (int q = 0; q < kKeep; ++q) {
        const int c = threadIdx.x + 256 * q;
        if (c < n4) {
            const float4 g = g4[c];
            store4<T>(o + 4 * c, make_float4(keep[q].x * inv * g.x, keep[q].y * inv * g.y, keep[q].z * inv * g.z,
                                             keep[q].w * inv * g.w));
        }
    }
    for (int c = threadIdx.x + 256 * kKeep; c < n4; c += 256) {
        const float4 v = x4[c], g = g4[c];
        store4<T>(o + 4 * c, make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w));
    }
}

// ---- rotary table per row: (cos, sin)(pos(r) * theta^(-2 i / hd)) in fp64, rounded once ----------
__global__ void rope_table_kernel(float2* __restrict__ cs, int row0, int R, int P, int Tn, int half,
                                  double log_theta_over_half) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // up to 2^24 rows x 128 pairs
    if (idx >= (int64_t)(R - row0) * half) return;
    const int r = row0 + (int)(idx / half), i = (int)(idx % half);
    double ang = (double)tree_position(r, P, Tn) * exp(-(double)i * log_theta_over_half);
    double s, c;
    sincos(ang, &s, &c);
    cs[(int64_t)r * half + i] = make_float2((float)c, (float)s);
}

// ---- S2 epilogue (unfused): rotate q and k in place -------------------------------------------
// One thread per (row, head, pair).  Heads 0 .. nq + nkv - 1 of the qkv row are rotated.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ qkv, const float2* __restrict__ cs, int R,
                                                   int n_rot_heads, int hd, int64_t ld) {
    const int half = hd >> 1;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)R * n_rot_heads * half;
    if (idx >= total) return;
    int i = (int)(idx % half);
    int head = (int)((idx / half) % n_rot_heads);
    int r = (int)(idx / ((int64_t)half * n_rot_heads));
    float2 c_s = cs[(int64_t)r * half + i];
    T* p = qkv + (int64_t)r * ld + head * hd + i;
    float x1 = to_f32<T>(p[0]), x2 = to_f32<T>(p[half]);
    p[0] = from_f32<T>(x1 * c_s.x - x2 * c_s.y);
    p[half] = from_f32<T>(x2 * c_s.x + x1 * c_s.y);
}

// ---- V transpose: vt[kvh][c][r] = qkv[r][v_off + kvh hd + c] ------------------------------------
// 64 x 64 tiles through LDS so both the read and the write are coalesced.  Columns r in [R, ldv)
// are written as zero: the attention kernel loads whole 64-key tiles and multiplies the masked
// probabilities (exact zeros) with whatever it finds there.
template <typename T>
__global__ __launch_bounds__(256) void transpose_v_kernel(const T* __restrict__ qkv, int row0, int R, int64_t ld, int v_off,
                                                          int hd, T* __restrict__ vt, int64_t ldv) {
    __shared__ T tile[64][65];
    const int r0 = row0 / 64 * 64 + blockIdx.x * 64, c0 = blockIdx.y * 64, kvh = blockIdx.z;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        int r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < R && c < hd) ? qkv[(int64_t)r * ld + v_off + kvh * hd + c] : from_f32<T>(0.f);
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        int c = c0 + i, r = r0 + tx;
        if (c < hd && r >= row0 && r < ldv) vt[((int64_t)kvh * hd + c) * ldv + r] = tile[tx][i];
    }
}

// dst[r][c] = src[r][c] for a rows x cols block of two pitched arrays (prefix cache <-> workspace)
template <typename T>
__global__ __launch_bounds__(256) void copy2d_kernel(const T* __restrict__ src, int64_t src_ld, T* __restrict__ dst,
                                                     int64_t dst_ld, int64_t rows, int64_t cols) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * cols) return;
    const int64_t r = i / cols, c = i % cols;
    dst[r * dst_ld + c] = src[r * src_ld + c];
}

// Finish of a K-split QKV projection: acc [n_slices][rows, (nq + 2 nkv) hd] holds the fp32 partial sums of the K slices,
// added here in slice order.  One thread per (row, head, rotation pair i < hd / 2): q and k heads are rotated
// (rotate-half RoPE, table row cs[r]) and stored to the qkv row, v heads are stored to the transposed copy
// vt [nkv hd, ldv] at column r.
template <typename T>
__global__ __launch_bounds__(256) void qkv_finish_kernel(const float* __restrict__ acc, int n_slices, int64_t pitch,
                                                         const float2* __restrict__ cs, int rows, int nq, int nkv, int hd,
                                                         T* __restrict__ qkv, T* __restrict__ vt, int64_t ldv) {
    const int half = hd >> 1, heads = nq + 2 * nkv;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)rows * heads * half) return;
    const int i = (int)(idx % half);
    const int head = (int)((idx / half) % heads);
    const int r = (int)(idx / ((int64_t)half * heads));
    const int64_t ld = (int64_t)heads * hd;
    const float* a = acc + (int64_t)r * ld + head * hd + i;
    float x1 = 0.f, x2 = 0.f;
    for (int s0 = 0; s0 < n_slices; s0 += 4) {          // four slices' loads in flight, added in slice order
        float t1[4], t2[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            t1[u] = s0 + u < n_slices ? a[(s0 + u) * pitch] : 0.f;
            t2[u] = s0 + u < n_slices ? a[(s0 + u) * pitch + half] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            x1 += t1[u];
            x2 += t2[u];
        }
    }
    if (head < nq + nkv) {
        const float2 c_s = cs[(int64_t)r * half + i];
        T* p = qkv + (int64_t)r * ld + head * hd + i;
        p[0] = from_f32<T>(x1 * c_s.x - x2 * c_s.y);
        p[half] = from_f32<T>(x2 * c_s.x + x1 * c_s.y);
    } else {
        T* p = vt + ((int64_t)(head - nq - nkv) * hd + i) * ldv + r;
        p[0] = from_f32<T>(x1);
        p[(int64_t)half * ldv] = from_f32<T>(x2);
    }
}

// Zero columns [R, ldv) of every row of V^T (for a producer that writes only the R real columns).
template <typename T>
__global__ __launch_bounds__(256) void zero_vt_tail_kernel(T* __restrict__ vt, int64_t rows, int R, int64_t ldv) {
    const int tail = (int)(ldv - R);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * tail) return;
    vt[(i / tail) * ldv + R + (i % tail)] = from_f32<T>(0.f);
}

// ---- S6: gather the scoring rows, final RMSNorm, targets -----------------------------------------
// Scoring row b = k T + t reads the hidden state that predicts y^k_t: the last prefix row for
// t = 0, else the row of y^k_{t-1}.
template <typename T>
__global__ __launch_bounds__(256) void gather_norm_kernel(const float* __restrict__ h, const float* __restrict__ gain,
                                                          float eps, int d, const int32_t* __restrict__ draft_ids,
                                                          const int32_t* __restrict__ draft_lens, int vocab, int P,
                                                          int Tn, T* __restrict__ xs, int32_t* __restrict__ targets,
                                                          uint8_t* __restrict__ valid) {
    __shared__ float red[4];
    const int b = blockIdx.x;
    const int k = b / Tn, t = b % Tn;
    const int src_row = t == 0 ? P - 1 : P + k * Tn + t - 1;
    rmsnorm_row<T>(h + (int64_t)src_row * d, gain, eps, d, xs + (int64_t)b * d, red);
    if (threadIdx.x == 0) {
        int id = draft_ids[b];
        bool ok = !(draft_lens && t >= draft_lens[k]);
        if (id < 0 || id >= vocab) id = 0;   // flagged by the embedding kernel already
        targets[b] = id;
        valid[b] = ok ? 1 : 0;
    }
}

// ---- S8: conformity score per draft, fixed-order tree sum ------------------------------------------
__global__ __launch_bounds__(256) void score_reduce_kernel(const float* __restrict__ lp,
                                                           const int32_t* __restrict__ draft_lens, int Tn, int mode,
                                                           float* __restrict__ token_logprobs,
                                                           float* __restrict__ scores) {
    __shared__ float red[4];
    const int k = blockIdx.x;
    const int len = draft_lens ? min(max(draft_lens[k], 0), Tn) : Tn;
    float s = 0.f;
    for (int t = threadIdx.x; t < Tn; t += 256) {
        float v = t < len ? lp[(int64_t)k * Tn + t] : 0.f;
        if (token_logprobs) token_logprobs[(int64_t)k * Tn + t] = v;
        s += v;
    }
    s = block_sum<256>(s, red);
    if (threadIdx.x == 0) scores[k] = mode == ATTS_SCORE_MEAN_NLL ? -s / (float)max(len, 1) : -s;
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

int32_t launch_embed(int32_t dtype, const void* tok_embed, int32_t vocab, int32_t d, const int32_t* prefix_ids,
                     const int32_t* draft_ids, const int32_t* draft_lens, ScoreShape s, int32_t row0, float* h,
                     int32_t* err_flag, hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(embed_kernel<T>, dim3(s.R() - row0), dim3(256), 0, stream, (const T*)tok_embed, vocab, d,
                                         prefix_ids, draft_ids, draft_lens, s.P, s.T, row0, h, err_flag);)
    ATTS_LAUNCH_CHECK("embed_kernel");
    return ATTS_OK;
}

int32_t launch_rmsnorm(int32_t dtype, const float* h, const float* gain, float eps, int32_t rows, int32_t d, void* out,
                       hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(rmsnorm_kernel<T>, dim3(rows), dim3(256), 0, stream, h, gain, eps, d, (T*)out);)
    ATTS_LAUNCH_CHECK("rmsnorm_kernel");
    return ATTS_OK;
}

int32_t launch_rope_table(float2* cs, ScoreShape s, int32_t row0, int32_t hd, float theta, hipStream_t stream) {
    const int half = hd / 2;
    const int64_t total = (int64_t)(s.R() - row0) * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, cs, row0, s.R(), s.P, s.T, half,
                       log((double)theta) / (double)half);
    ATTS_LAUNCH_CHECK("rope_table_kernel");
    return ATTS_OK;
}

int32_t launch_transpose_v(int32_t dtype, const void* qkv, int32_t row0, int32_t R, int32_t nq, int32_t nkv, int32_t hd,
                           void* vt, int64_t ldv, hipStream_t stream) {
    const int64_t ld = (int64_t)(nq + 2 * nkv) * hd;
    dim3 grid((unsigned)ceil_div(ldv - row0 / 64 * 64, 64), (unsigned)ceil_div(hd, 64), nkv);
    DISPATCH_T(dtype, hipLaunchKernelGGL(transpose_v_kernel<T>, grid, dim3(256), 0, stream, (const T*)qkv, row0, R, ld,
                                         (nq + nkv) * hd, hd, (T*)vt, ldv);)
    ATTS_LAUNCH_CHECK("transpose_v_kernel");
    return ATTS_OK;
}

int32_t launch_zero_vt_tail(int32_t dtype, void* vt, int64_t rows, int32_t R, int64_t ldv, hipStream_t stream) {
    const int tail = (int)(ldv - R);
    if (tail <= 0 || rows <= 0) return ATTS_OK;
    const int64_t total = rows * tail;
    DISPATCH_T(dtype, hipLaunchKernelGGL(zero_vt_tail_kernel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                                         (T*)vt, rows, R, ldv);)
    ATTS_LAUNCH_CHECK("zero_vt_tail_kernel");
    return ATTS_OK;
}

int32_t launch_rope_split(int32_t dtype, void* qkv, const float2* cs, ScoreShape s, int32_t row0, int32_t nq, int32_t nkv,
                          int32_t hd, void* vt, int64_t ldv, hipStream_t stream) {
    const int64_t ld = (int64_t)(nq + 2 * nkv) * hd;
    const int rows = s.R() - row0;
    const int64_t total = (int64_t)rows * (nq + nkv) * (hd / 2);
    DISPATCH_T(dtype, hipLaunchKernelGGL(rope_kernel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                                         (T*)qkv + (int64_t)row0 * ld, cs + (int64_t)row0 * (hd / 2), rows, nq + nkv, hd, ld);)
    ATTS_LAUNCH_CHECK("rope_kernel");
    if (vt) return launch_transpose_v(dtype, qkv, row0, s.R(), nq, nkv, hd, vt, ldv, stream);
    return ATTS_OK;
}

int32_t launch_qkv_finish(int32_t dtype, const float* acc, int32_t n_slices, int64_t slice_pitch, const float2* cs, int32_t rows,
                          int32_t nq, int32_t nkv, int32_t hd, void* qkv, void* vt, int64_t ldv, hipStream_t stream) {
    const int64_t total = (int64_t)rows * (nq + 2 * nkv) * (hd / 2);
    DISPATCH_T(dtype, hipLaunchKernelGGL(qkv_finish_kernel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, acc,
                                         n_slices, slice_pitch, cs, rows, nq, nkv, hd, (T*)qkv, (T*)vt, ldv);)
    ATTS_LAUNCH_CHECK("qkv_finish_kernel");
    return ATTS_OK;
}

int32_t launch_resid_norm(int32_t dtype, float* h, const float* partials, int32_t n_slices, int64_t slice_pitch, const float* gain,
                          float eps, int32_t rows, int32_t d, void* xn, hipStream_t stream) {
    if (rows <= 0) return ATTS_OK;
    if (d % 4 || slice_pitch % 4) return fail(ATTS_ERR_SHAPE, "residual update: row length and slice pitch must be multiples of 4");
    DISPATCH_T(dtype, hipLaunchKernelGGL(resid_norm_kernel<T>, dim3(rows), dim3(256), 0, stream, h, partials, n_slices, slice_pitch,
                                         gain, eps, d, (T*)xn);)
    ATTS_LAUNCH_CHECK("resid_norm_kernel");
    return ATTS_OK;
}

int32_t launch_copy2d(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int64_t rows, int64_t cols,
                      hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return ATTS_OK;
    DISPATCH_T(dtype, hipLaunchKernelGGL(copy2d_kernel<T>, dim3((unsigned)ceil_div(rows * cols, 256)), dim3(256), 0, stream,
                                         (const T*)src, src_ld, (T*)dst, dst_ld, rows, cols);)
    ATTS_LAUNCH_CHECK("copy2d_kernel");
    return ATTS_OK;
}

int32_t launch_gather_norm(int32_t dtype, const float* h, const float* gain, float eps, int32_t d,
                           const int32_t* draft_ids, const int32_t* draft_lens, int32_t vocab, ScoreShape s, void* xs,
                           int32_t* targets, uint8_t* valid, hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(gather_norm_kernel<T>, dim3(s.B()), dim3(256), 0, stream, h, gain, eps, d,
                                         draft_ids, draft_lens, vocab, s.P, s.T, (T*)xs, targets, valid);)
    ATTS_LAUNCH_CHECK("gather_norm_kernel");
    return ATTS_OK;
}

int32_t launch_score_reduce(const float* lp, const int32_t* draft_lens, int32_t K, int32_t T, int32_t mode,
                            float* token_logprobs, float* scores, hipStream_t stream) {
    hipLaunchKernelGGL(score_reduce_kernel, dim3(K), dim3(256), 0, stream, lp, draft_lens, T, mode, token_logprobs, scores);
    ATTS_LAUNCH_CHECK("score_reduce_kernel");
    return ATTS_OK;
}

}  // namespace atts
