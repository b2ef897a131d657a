// Kernels of the target-model continuation ("Target Model Sampling"): one new token per continued candidate and step.
//
// The candidates continue different drafts of the same prompt, so their keys / values form the same token tree as
// in scoring: a shared prefix and one branch per candidate.  During a continuation call the keys (after RoPE) and
// values of the whole tree live per layer in a row-major cache
//     rows [0, P): prefix        rows P + j Tc + t: token t of branch j  (Tc = draft length + tokens to generate)
// and a decode step sends one row per branch through the model.
#include "common.h"

#include <type_traits>

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

// One decode row per branch: acc [n_slices][Kr, (nq + 2 nkv) hd] fp32 partial sums (added in slice order) -> q (rotated) to
// q_out [Kr, nq hd]; k (rotated) and v to row `P + j Tc + pos.at(j)` of the layer's key / value cache.  cs: (cos, sin)
// rows indexed by absolute position.
template <typename T>
__global__ __launch_bounds__(256) void decode_qkv_finish_kernel(const float* __restrict__ acc, int n_slices, int64_t pitch,
                                                                const float2* __restrict__ cs, int Kr, int nq, int nkv, int hd,
                                                                int P, int Tc, BranchPos pos, T* __restrict__ q_out,
                                                                T* __restrict__ k_cache, T* __restrict__ v_cache) {
    const int half = hd >> 1, heads = nq + 2 * nkv;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)Kr * heads * half) return;
    const int i = (int)(idx % half);
    const int head = (int)((idx / half) % heads);
    const int j = (int)(idx / ((int64_t)half * heads));
    const float* a = acc + (int64_t)j * heads * hd + head * hd + i;
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
    const int t_new = pos.at(j);
    const int64_t crow = P + (int64_t)j * Tc + t_new;
    if (head < nq + nkv) {
        const float2 c_s = cs[(int64_t)(P + t_new) * half + i];
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
// to rows 0 .. pos.at(j) of its own branch.  Scores: one key per thread and pass (16-byte loads along the key row);
// output: every wavefront accumulates its share of the keys (lane = a pair of dims, 128 / 256 contiguous bytes per
// key), the partial sums are added in a fixed order.
constexpr int kDecodeWaves = 16, kDecodeThreads = 64 * kDecodeWaves;

template <typename T>
__global__ __launch_bounds__(kDecodeThreads) void attn_decode_kernel(const T* __restrict__ q, const T* __restrict__ k_cache,
                                                                     const T* __restrict__ v_cache, T* __restrict__ out, int P,
                                                                     int Tc, BranchPos pos, int nq, int nkv, int hd, float scale) {
    extern __shared__ float sm[];           // [hd] query | [n] scores | [2 waves] reductions | [waves][hd] partial outputs
    const int n = P + pos.at(blockIdx.x) + 1;
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

// Dot product of two 16-byte pieces (8 bf16 or 4 fp32 elements).
template <typename T> __device__ __forceinline__ float dot_piece(const uint4& a, const uint4& b);
template <> __device__ __forceinline__ float dot_piece<float>(const uint4& a, const uint4& b) {
    const float* x = reinterpret_cast<const float*>(&a);
    const float* y = reinterpret_cast<const float*>(&b);
    return x[0] * y[0] + x[1] * y[1] + x[2] * y[2] + x[3] * y[3];
}
template <> __device__ __forceinline__ float dot_piece<bf16>(const uint4& a, const uint4& b) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2* x = reinterpret_cast<const bf16x2*>(&a);
    const bf16x2* y = reinterpret_cast<const bf16x2*>(&b);
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) s = __builtin_amdgcn_fdot2_f32_bf16(x[u], y[u], s, false);   // fp32 accumulation
    return s;
}

// Sum of s over aligned groups of `lanes` (a power of two <= 64) neighbouring lanes, in every lane of the group.  Inside a
// row of 16 lanes the exchanges are DPP permutations (pairs, quads, mirrored half rows, mirrored rows: any pairing of
// disjoint partial sums will do); beyond that, LDS-crossbar shuffles.
__device__ __forceinline__ float group_sum(float s, int lanes) {
    auto dpp = [](float v, auto ctrl) __attribute__((always_inline)) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    if (lanes > 1) s += dpp(s, std::integral_constant<int, 0xB1>{});     // quad_perm [1, 0, 3, 2]
    if (lanes > 2) s += dpp(s, std::integral_constant<int, 0x4E>{});     // quad_perm [2, 3, 0, 1]
    if (lanes > 4) s += dpp(s, std::integral_constant<int, 0x141>{});    // row_half_mirror
    if (lanes > 8) s += dpp(s, std::integral_constant<int, 0x140>{});    // row_mirror
    for (int o = 16; o < lanes; o <<= 1) s += __shfl_xor(s, o);
    return s;
}

// The same attention step when a key / value row of one head is a power-of-two number of 16-byte pieces (every bf16
// model with head_dim 128): lanes_per_key lanes cover one row, so a wavefront reads g = 64 / lanes_per_key whole rows
// per instruction; lane (sub = lane / lanes_per_key, piece = lane % lanes_per_key) of wavefront w takes the keys
// (w g + sub) + kDecodeWaves g m, in batches of kDecodeBatch.  One CU serves a whole (branch, head), so the step is
// bound by memory round trips and by instruction issue, not by bytes:
//   * two key batches and two value batches are requested before anything is waited for: a context of up to
//     2 kDecodeBatch kDecodeWaves g keys costs one round trip (longer ones: one more per further batch);
//   * every wavefront runs its own softmax over its keys (running maximum m, sum l and unnormalised output, all in
//     registers: a lane's probabilities multiply the value rows the same lane loaded), and the wavefronts are
//     merged once at the end with the weights exp(m_w - max m): one barrier, no per-key LDS, no limit on the context;
//   * the query piece stays in registers in the model dtype (bf16: packed dot products, v_dot2_f32_bf16), the
//     1 / sqrt(head_dim) factor is applied to the finished score, and the group sums use DPP.
constexpr int kDecodeBatch = 7;

template <typename T>
__global__ __launch_bounds__(kDecodeThreads) void attn_decode_pieces_kernel(const T* __restrict__ q, const T* __restrict__ k_cache,
                                                                            const T* __restrict__ v_cache, T* __restrict__ out,
                                                                            int P, int Tc, BranchPos pos, int nq, int nkv, int hd,
                                                                            float scale) {
    extern __shared__ float sm[];           // [waves] running maxima | [waves] sums | [waves][hd] unnormalised outputs
    constexpr int kVec = 16 / (int)sizeof(T);
    const int n = P + pos.at(blockIdx.x) + 1;
    float* red = sm;
    float* so = sm + 2 * kDecodeWaves;
    const int j = blockIdx.x, head = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = head / (nq / nkv);
    const int64_t ld = (int64_t)nkv * hd;
    const int lanes_per_key = hd / kVec, g = 64 / lanes_per_key, sub = lane / lanes_per_key, piece = lane % lanes_per_key;
    const int stride = kDecodeWaves * g, span = kDecodeBatch * stride;
    const int first = wave * g;                         // wave-uniform; the lane's keys are first + sub + stride m
    // cache row of key i: i (prefix) or P + j Tc + (i - P) (own branch) = i + (i >= P ? j Tc : 0)
    const int64_t own = (int64_t)j * Tc * ld;
    const int64_t lane_off = (int64_t)kvh * hd + piece * kVec + (int64_t)sub * ld;
    auto load_rows = [&](const T* base, int i0, uint4 (&raw)[kDecodeBatch]) __attribute__((always_inline)) {
        const T* p0 = base + lane_off + (int64_t)i0 * ld;
#pragma unroll
        for (int b = 0; b < kDecodeBatch; ++b) {
            const int i = i0 + sub + b * stride;
            const T* p = p0 + (int64_t)b * stride * ld + (i >= P ? own : 0);
            raw[b] = i < n ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
        }
    };
    uint4 k0[kDecodeBatch], k1[kDecodeBatch], v0[kDecodeBatch], v1[kDecodeBatch];
    load_rows(k_cache, first, k0);
    load_rows(k_cache, first + span, k1);
    load_rows(v_cache, first, v0);
    load_rows(v_cache, first + span, v1);
    const uint4 qv = *reinterpret_cast<const uint4*>(q + (int64_t)j * nq * hd + head * hd + piece * kVec);

    // scores of a batch (-inf past the end) and their maximum; every lane of the wavefront takes part
    auto score = [&](int i0, const uint4 (&raw)[kDecodeBatch], float (&sc)[kDecodeBatch]) __attribute__((always_inline)) {
        float bm = -INFINITY;
#pragma unroll
        for (int b = 0; b < kDecodeBatch; ++b) {
            const float s = group_sum(dot_piece<T>(qv, raw[b]), lanes_per_key) * scale;
            sc[b] = i0 + sub + b * stride < n ? s : -INFINITY;
            bm = fmaxf(bm, sc[b]);
        }
        return bm;
    };
    auto wave_max = [&](float v) __attribute__((always_inline)) {      // the lanes of a key hold equal values: only the groups differ
        for (int o = lanes_per_key; o < 64; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
        return v;
    };
    float m = -INFINITY, l = 0.f;                       // running maximum (wave-uniform), sum over this lane's keys
    float acc[kVec];
#pragma unroll
    for (int u = 0; u < kVec; ++u) acc[u] = 0.f;
    auto rescale = [&](float m_new) __attribute__((always_inline)) {   // m_new finite
        const float corr = __expf(m - m_new);           // m = -inf: 0 (nothing accumulated yet)
        l *= corr;
#pragma unroll
        for (int u = 0; u < kVec; ++u) acc[u] *= corr;
        m = m_new;
    };
    auto accumulate = [&](const float (&sc)[kDecodeBatch], const uint4 (&raw)[kDecodeBatch]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < kDecodeBatch; ++b) {
            const float p = __expf(sc[b] - m);          // -inf score: 0
            l += p;
            const T* e = reinterpret_cast<const T*>(&raw[b]);
#pragma unroll
            for (int u = 0; u < kVec; ++u) acc[u] += p * to_f32<T>(e[u]);
        }
    };
    {
        float s0[kDecodeBatch], s1[kDecodeBatch];
        const float bm = wave_max(fmaxf(score(first, k0, s0), score(first + span, k1, s1)));
        if (bm > -INFINITY) {                           // wave-uniform: the wavefront has at least one key
            rescale(bm);
            accumulate(s0, v0);
            accumulate(s1, v1);
        }
    }
    for (int i0 = first + 2 * span; i0 < n; i0 += span) {              // long contexts: one batch at a time
        float s0[kDecodeBatch];
        load_rows(k_cache, i0, k0);
        load_rows(v_cache, i0, v0);
        const float bm = wave_max(score(i0, k0, s0));
        if (bm > -INFINITY) {
            if (bm > m) rescale(bm);
            accumulate(s0, v0);
        }
    }
    // the piece lanes of a key all added its probability to their l: the sum over the groups counts every key once
    for (int o = lanes_per_key; o < 64; o <<= 1) l += __shfl_xor(l, o);
#pragma unroll
    for (int u = 0; u < kVec; ++u) {
        for (int o = lanes_per_key; o < 64; o <<= 1) acc[u] += __shfl_xor(acc[u], o);
        if (sub == 0) so[wave * hd + piece * kVec + u] = acc[u];
    }
    if (lane == 0) {
        red[wave] = m;
        red[kDecodeWaves + wave] = l;
    }
    __syncthreads();
    for (int c = tid; c < hd; c += kDecodeThreads) {
        float top = red[0];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) top = fmaxf(top, red[w]);           // finite: wavefront 0 holds key 0
        float tot = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float wgt = __expf(red[w] - top);                                // a wavefront without keys: 0
            tot += wgt * red[kDecodeWaves + w];
            o += wgt * so[w * hd + c];
        }
        out[(int64_t)j * nq * hd + head * hd + c] = from_f32<T>(o / tot);
    }
}

// ids[j * stride] = first index of the largest logit of row j, in two launches: kArgmaxChunks workgroups per row each
// reduce a slice of the vocabulary to (value, index), then one wavefront per row reduces those.  (One workgroup per
// row cannot pull a row of 150k logits through a single CU fast enough.)
constexpr int kArgmaxChunks = 32;
struct ArgmaxPart {
    float v;
    int32_t at;
};
__device__ __forceinline__ void argmax_take(float& best, int& at, float v, int c) {   // NaN never wins; the first maximum is kept
    if (v > best || (v == best && c < at)) {
        best = v;
        at = c;
    }
}

__global__ __launch_bounds__(256) void argmax_partial_kernel(const float* __restrict__ logits, int64_t ld, int V,
                                                             ArgmaxPart* __restrict__ part) {
    __shared__ float s_val[256];
    __shared__ int s_idx[256];
    const int j = blockIdx.x, chunk = blockIdx.y;
    const float* z = logits + (int64_t)j * ld;
    const int per = (int)((V + kArgmaxChunks * 4 - 1) / (kArgmaxChunks * 4)) * 4;      // columns per chunk, a multiple of 4
    const int c0 = min(chunk * per, V), c1 = min(c0 + per, V);
    float best = -INFINITY;
    int at = 0x7fffffff;
    const bool vec = (reinterpret_cast<uintptr_t>(z) & 15) == 0;
    const int q0 = c0 / 4, q1 = vec ? c1 / 4 : q0;                                     // whole float4 groups of the chunk
#pragma unroll 4
    for (int c4 = q0 + threadIdx.x; c4 < q1; c4 += 256) {
        const float4 x = reinterpret_cast<const float4*>(z)[c4];
        argmax_take(best, at, x.x, 4 * c4);
        argmax_take(best, at, x.y, 4 * c4 + 1);
        argmax_take(best, at, x.z, 4 * c4 + 2);
        argmax_take(best, at, x.w, 4 * c4 + 3);
    }
    for (int c = 4 * q1 + threadIdx.x; c < c1; c += 256) argmax_take(best, at, z[c], c);
    s_val[threadIdx.x] = best;
    s_idx[threadIdx.x] = at;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) argmax_take(s_val[threadIdx.x], s_idx[threadIdx.x], s_val[threadIdx.x + o], s_idx[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) part[j * kArgmaxChunks + chunk] = ArgmaxPart{s_val[0], s_idx[0]};
}

__global__ __launch_bounds__(64) void argmax_final_kernel(const ArgmaxPart* __restrict__ part, int32_t* __restrict__ ids, int64_t stride,
                                                          int eos_id, bool has_prev) {
    const int j = blockIdx.x, lane = threadIdx.x;
    if (eos_id >= 0 && has_prev && ids[(int64_t)j * stride - 1] == eos_id) {      // the branch has ended: it stays ended
        if (lane == 0) ids[(int64_t)j * stride] = eos_id;
        return;
    }
    static_assert(kArgmaxChunks <= 64, "one wavefront reduces the partial results");
    float best = -INFINITY;
    int at = 0x7fffffff;
    if (lane < kArgmaxChunks) {
        const ArgmaxPart p = part[j * kArgmaxChunks + lane];
        argmax_take(best, at, p.v, p.at);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) argmax_take(best, at, __shfl_xor(best, o), __shfl_xor(at, o));
    if (lane == 0) ids[(int64_t)j * stride] = at == 0x7fffffff ? 0 : at;
}

// ids[j * stride] = inverse-CDF sample of softmax(logits[j] * inv_temp) with the uniform u = uniforms[j * stride]:
// the first index v (vocabulary order) whose cumulative weight reaches u times the total.  Two launches, like the
// arg max: kArgmaxChunks workgroups per row reduce a contiguous slice of the vocabulary to (slice maximum m_c,
// S_c = sum exp((z - m_c) inv_temp)); then one workgroup per row puts the slices on the row maximum, finds the slice
// the target falls into by adding the slice weights in index order, gives each thread a contiguous piece of that
// slice, finds the piece the same way and walks it.  Sums in fp32, fixed order.
struct SamplePart {
    float m, s;
};
constexpr int kSampleThreads = 256;

__device__ __forceinline__ int sample_slice_len(int V) { return (int)((V + kArgmaxChunks * 4 - 1) / (kArgmaxChunks * 4)) * 4; }

__global__ __launch_bounds__(256) void sample_partial_kernel(const float* __restrict__ logits, int64_t ld, int V, float inv_temp,
                                                             SamplePart* __restrict__ part) {
    __shared__ float red[4];
    const int j = blockIdx.x, chunk = blockIdx.y, tid = threadIdx.x;
    const float* z = logits + (int64_t)j * ld;
    const int per = sample_slice_len(V);
    const int c0 = min(chunk * per, V), c1 = min(c0 + per, V);
    float mx = -INFINITY;
    for (int c = c0 + tid; c < c1; c += 256) mx = fmaxf(mx, z[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.f;
    for (int c = c0 + tid; c < c1; c += 256) sum += __expf((z[c] - mx) * inv_temp);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if ((tid & 63) == 0) red[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) part[j * kArgmaxChunks + chunk] = SamplePart{mx, red[0] + red[1] + red[2] + red[3]};   // empty slice: (-inf, 0)
}

__global__ __launch_bounds__(kSampleThreads) void sample_final_kernel(const float* __restrict__ logits, int64_t ld, int V, float inv_temp,
                                                                      const SamplePart* __restrict__ part,
                                                                      const float* __restrict__ uniforms, int32_t* __restrict__ ids,
                                                                      int64_t stride, int eos_id, bool has_prev) {
    __shared__ float piece_sum[kSampleThreads], group_sum[kSampleThreads / 16];
    __shared__ float s_top, s_target, s_before;
    __shared__ int s_chunk, s_piece;
    const int j = blockIdx.x, tid = threadIdx.x;
    if (eos_id >= 0 && has_prev && ids[(int64_t)j * stride - 1] == eos_id) {      // the branch has ended: it stays ended
        if (tid == 0) ids[(int64_t)j * stride] = eos_id;
        return;
    }
    const float* z = logits + (int64_t)j * ld;
    if (tid == 0) {
        const SamplePart* p = part + j * kArgmaxChunks;
        float top = -INFINITY;
        for (int c = 0; c < kArgmaxChunks; ++c) top = fmaxf(top, p[c].m);
        float w[kArgmaxChunks], total = 0.f;
        for (int c = 0; c < kArgmaxChunks; ++c) {
            w[c] = p[c].s > 0.f ? p[c].s * __expf((p[c].m - top) * inv_temp) : 0.f;
            total += w[c];
        }
        const float target = uniforms[(int64_t)j * stride] * total;
        float before = 0.f;
        int chunk = -1, last_mass = 0;
        for (int c = 0; c < kArgmaxChunks; ++c) {
            if (w[c] > 0.f) {
                last_mass = c;
                if (before + w[c] >= target) {
                    chunk = c;
                    break;
                }
            }
            before += w[c];
        }
        if (chunk < 0) {                                 // rounding left the target just past the end: the last slice with mass
            chunk = last_mass;
            before = 0.f;
            for (int c = 0; c < chunk; ++c) before += w[c];
        }
        s_top = top;
        s_target = target;
        s_before = before;
        s_chunk = chunk;
    }
    __syncthreads();
    // the slice, cut into one contiguous piece per thread
    const int per = sample_slice_len(V);
    const int c0 = min(s_chunk * per, V), c1 = min(c0 + per, V);
    const int piece = (c1 - c0 + kSampleThreads - 1) / kSampleThreads;
    const int q0 = min(c0 + tid * piece, c1), q1 = min(q0 + piece, c1);
    const float top = s_top;
    float sum = 0.f;
    for (int c = q0; c < q1; ++c) sum += __expf((z[c] - top) * inv_temp);
    piece_sum[tid] = sum;
    __syncthreads();
    // pieces are added in index order in two levels (16 groups of 16, then the groups): 48 dependent steps, not 256
    constexpr int kGroup = 16, kGroups = kSampleThreads / kGroup;
    if (tid < kGroups) {
        float gs = 0.f;
        for (int t = 0; t < kGroup; ++t) gs += piece_sum[tid * kGroup + t];
        group_sum[tid] = gs;
    }
    __syncthreads();
    if (tid == 0) {
        // first unit (group, then piece) with mass whose running total reaches the target; else the last one with mass
        auto locate = [&](const float* w, int n, float& before) {
            const float start = before;
            int pick = -1, last_mass = 0;
            for (int t = 0; t < n; ++t) {
                if (w[t] > 0.f) {
                    last_mass = t;
                    if (before + w[t] >= s_target) {
                        pick = t;
                        break;
                    }
                }
                before += w[t];
            }
            if (pick < 0) {
                pick = last_mass;
                before = start;
                for (int t = 0; t < pick; ++t) before += w[t];
            }
            return pick;
        };
        float before = s_before;
        const int grp = locate(group_sum, kGroups, before);
        const int pick = grp * kGroup + locate(piece_sum + grp * kGroup, kGroup, before);
        s_piece = pick;
        s_before = before;
    }
    __syncthreads();
    if (tid == s_piece) {
        float run = s_before;
        int pick = -1, last_mass = -1;
        for (int c = q0; c < q1; ++c) {
            const float e = __expf((z[c] - top) * inv_temp);
            run += e;
            if (e > 0.f) last_mass = c;
            if (run >= s_target) {
                pick = c;
                break;
            }
        }
        if (pick < 0) pick = last_mass >= 0 ? last_mass : (q1 > q0 ? q1 - 1 : V - 1);   // rounding left the target just past the piece
        ids[(int64_t)j * stride] = pick;
    }
}

// xs[j] = rmsnorm(h[rows[j]]) with rows[j] = first + j * step + pos.at(j)
template <typename T>
__global__ __launch_bounds__(256) void norm_strided_rows_kernel(const float* __restrict__ h, const float* __restrict__ gain, float eps,
                                                                int d, int64_t first, int64_t step, BranchPos pos, T* __restrict__ xs) {
    __shared__ float red[4];
    const int j = blockIdx.x;
    const float* x = h + (first + (int64_t)j * step + pos.at(j)) * d;
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

int32_t launch_decode_qkv_finish(int32_t dtype, const float* acc, int32_t n_slices, int64_t slice_pitch, const float2* cs, int32_t Kr,
                                 int32_t nq, int32_t nkv, int32_t hd, int32_t P, int32_t Tc, BranchPos pos, void* q_out,
                                 void* k_cache, void* v_cache, hipStream_t stream) {
    const int64_t total = (int64_t)Kr * (nq + 2 * nkv) * (hd / 2);
    DISPATCH_T(dtype, hipLaunchKernelGGL(decode_qkv_finish_kernel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, acc,
                                         n_slices, slice_pitch, cs, Kr, nq, nkv, hd, P, Tc, pos, (T*)q_out, (T*)k_cache, (T*)v_cache);)
    ATTS_LAUNCH_CHECK("decode_qkv_finish_kernel");
    return ATTS_OK;
}

// head rows that are a power-of-two number of 16-byte pieces take the kernel without a context limit; the general one
// holds one score per key in LDS
static bool decode_by_pieces(int32_t dtype, int32_t hd) {
    const int lanes_per_key = hd * (int)dtype_size(dtype) / 16;
    return (hd * dtype_size(dtype)) % 16 == 0 && lanes_per_key <= 64 && (lanes_per_key & (lanes_per_key - 1)) == 0;
}
static size_t decode_general_lds(int32_t hd, int64_t n_max) { return (size_t)((1 + kDecodeWaves) * hd + n_max + 2 * kDecodeWaves) * sizeof(float); }

int32_t decode_context_check(const char* fn, int32_t dtype, int32_t hd, int64_t n_max) {
    if (decode_by_pieces(dtype, hd) || decode_general_lds(hd, n_max) <= 60 * 1024) return ATTS_OK;
    return fail(ATTS_ERR_SHAPE, "%s: a context of %lld keys is too long for the decoding attention of this dtype / head_dim", fn,
                (long long)n_max);
}

int32_t launch_attn_decode(int32_t dtype, const void* q, const void* k_cache, const void* v_cache, void* out, int32_t Kr, int32_t P,
                           int32_t Tc, BranchPos pos, int32_t nq, int32_t nkv, int32_t hd, hipStream_t stream) {
    const float scale = 1.f / sqrtf((float)hd);
    dim3 grid(Kr, nq);
    if (decode_by_pieces(dtype, hd)) {
        const size_t lds = (size_t)(kDecodeWaves * hd + 2 * kDecodeWaves) * sizeof(float);
        DISPATCH_T(dtype, hipLaunchKernelGGL(attn_decode_pieces_kernel<T>, grid, dim3(kDecodeThreads), lds, stream, (const T*)q,
                                             (const T*)k_cache, (const T*)v_cache, (T*)out, P, Tc, pos, nq, nkv, hd, scale);)
        ATTS_LAUNCH_CHECK("attn_decode_pieces_kernel");
        return ATTS_OK;
    }
    const int n_max = P + pos.T + pos.done + 1;        // the longest branch
    const size_t lds = decode_general_lds(hd, n_max);
    if (lds > 60 * 1024) return fail(ATTS_ERR_SHAPE, "continuation: context of %d keys is too long", n_max);
    DISPATCH_T(dtype, hipLaunchKernelGGL(attn_decode_kernel<T>, grid, dim3(kDecodeThreads), lds, stream, (const T*)q, (const T*)k_cache,
                                         (const T*)v_cache, (T*)out, P, Tc, pos, nq, nkv, hd, scale);)
    ATTS_LAUNCH_CHECK("attn_decode_kernel");
    return ATTS_OK;
}

size_t argmax_scratch_bytes(int32_t rows) { return (size_t)rows * kArgmaxChunks * sizeof(ArgmaxPart); }

int32_t launch_argmax_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, void* scratch, int32_t* ids, int64_t stride,
                           int32_t eos_id, bool has_prev, hipStream_t stream) {
    ArgmaxPart* part = static_cast<ArgmaxPart*>(scratch);
    hipLaunchKernelGGL(argmax_partial_kernel, dim3(rows, kArgmaxChunks), dim3(256), 0, stream, logits, ld, V, part);
    ATTS_LAUNCH_CHECK("argmax_partial_kernel");
    hipLaunchKernelGGL(argmax_final_kernel, dim3(rows), dim3(64), 0, stream, part, ids, stride, eos_id, has_prev);
    ATTS_LAUNCH_CHECK("argmax_final_kernel");
    return ATTS_OK;
}

int32_t launch_sample_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, float inv_temp, const float* uniforms,
                           void* scratch, int32_t* ids, int64_t stride, int32_t eos_id, bool has_prev, hipStream_t stream) {
    static_assert(sizeof(SamplePart) == sizeof(ArgmaxPart), "both selections use the same per-slice scratch");
    SamplePart* part = static_cast<SamplePart*>(scratch);
    hipLaunchKernelGGL(sample_partial_kernel, dim3(rows, kArgmaxChunks), dim3(256), 0, stream, logits, ld, V, inv_temp, part);
    ATTS_LAUNCH_CHECK("sample_partial_kernel");
    hipLaunchKernelGGL(sample_final_kernel, dim3(rows), dim3(kSampleThreads), 0, stream, logits, ld, V, inv_temp, part, uniforms, ids,
                       stride, eos_id, has_prev);
    ATTS_LAUNCH_CHECK("sample_final_kernel");
    return ATTS_OK;
}

int32_t launch_norm_strided_rows(int32_t dtype, const float* h, const float* gain, float eps, int32_t d, int64_t first, int64_t step,
                                 BranchPos pos, int32_t rows, void* xs, hipStream_t stream) {
    DISPATCH_T(dtype, hipLaunchKernelGGL(norm_strided_rows_kernel<T>, dim3(rows), dim3(256), 0, stream, h, gain, eps, d, first, step,
                                         pos, (T*)xs);)
    ATTS_LAUNCH_CHECK("norm_strided_rows_kernel");
    return ATTS_OK;
}

}  // namespace atts
