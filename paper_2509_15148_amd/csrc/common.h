// Shared host/device helpers for the ATTS HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "atts.h"

namespace atts {

typedef __bf16 bf16;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// Records the calling thread's error text and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define ATTS_HIP_TRY(expr)                                                                   \
    do {                                                                                     \
        hipError_t e__ = (expr);                                                             \
        if (e__ != hipSuccess)                                                               \
            return ::atts::fail(ATTS_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

// After a kernel launch: report a launch-configuration error without synchronising.
#define ATTS_LAUNCH_CHECK(name)                                                              \
    do {                                                                                     \
        hipError_t e__ = hipGetLastError();                                                  \
        if (e__ != hipSuccess)                                                               \
            return ::atts::fail(ATTS_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(e__)); \
    } while (0)

// Brackets the launches issued during its lifetime with an event pair on `stream`, while atts_profile_enable is on.
class StageTimer {
public:
    StageTimer(int32_t stage, hipStream_t stream);
    ~StageTimer();
    StageTimer(const StageTimer&) = delete;
    StageTimer& operator=(const StageTimer&) = delete;
private:
    hipStream_t st_;
    int32_t stage_;
    hipEvent_t start_{}, stop_{};
    bool live_ = false;
};

// Raises the dynamic LDS limit of a kernel, once per device (the attribute belongs to the device's copy of the code).
template <auto kKernel>
inline int32_t allow_dynamic_lds(size_t bytes) {
    static std::mutex mutex;
    static bool done[64] = {};
    int dev = 0;
    ATTS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(ATTS_ERR_HIP, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(mutex);
    if (!done[dev]) {
        ATTS_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kKernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
        done[dev] = true;
    }
    return ATTS_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t dtype_size(int32_t dtype) { return dtype == ATTS_DTYPE_F32 ? 4 : 2; }

// ---- device-side conversions ------------------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE

// ---- direct global -> LDS loads and explicit waits (device code) -------------------------------
#define ATTS_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define ATTS_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void block_barrier() {
    // bare s_barrier (no fence): ordering against our own LDS traffic is done with the explicit
    // waits around it; the asm statements keep the compiler from moving memory operations across.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ---- launch wrappers (each enqueues on `stream`, returns ATTS_OK / ATTS_ERR_HIP) ----------

// Epilogues of the NT GEMM  acc[M, N] = A[M, Kd] . W[N, Kd]^T
enum GemmEpilogue : int32_t {
    EPI_STORE_ACT = 0,   // out (T) [M, ldc]      = acc
    EPI_STORE_F32 = 1,   // out (float) [M, ldc]  = acc
    EPI_RESID_F32 = 2,   // out (float) [M, ldc] += acc            (residual stream update)
    EPI_SWIGLU = 3,      // W = [gate rows (F) ; up rows (F)], N = F: out (T) [M, ldc] = silu(gate) * up
    EPI_LMHEAD = 4,      // per-row online-softmax partials over this tile's columns + target logit
    EPI_QKV_ROPE = 5,    // QKV projection: q/k heads rotated (rotate-half RoPE) and stored to out (T) [M, ldc];
                         // v heads stored transposed to vt [n_kv, 128, ldv].  head_dim 128, aligned bf16 shapes only.
    EPI_LMHEAD_T = 7,    // EPI_LMHEAD with the operands exchanged (rows of the product = vocabulary entries, columns = scoring
                         // rows): launch_gemm takes it by itself for EPI_LMHEAD calls whose shape allows it
    EPI_PARTIAL_F32 = 6, // out (float) [n_slices][M, ldc]: the K range is cut into n_slices = gemm_partial_slices(...)
                         // slices whose partial sums are stored one after the other (pitch M ldc floats); the consumer
                         // adds them in slice order.  For projections with few rows and a narrow output, whose tiles
                         // alone would leave most of the chip idle while the weights stream by.  No atomics: the
                         // result does not depend on the order in which the workgroups finish.
};

struct GemmArgs {
    const void* a;       // [M, Kd] row-major, leading dimension lda (elements)
    const void* w;       // [N, Kd] row-major, leading dimension ldw  (EPI_SWIGLU: [2N, Kd])
    void* out;           // see GemmEpilogue
    int32_t M, N, Kd;
    int64_t lda, ldw, ldc;
    bool a_rows_padded;  // rows M .. next multiple of 768 of `a` are readable (any values; their results are dropped)
    // EPI_LMHEAD only:
    const int32_t* targets;  // [M] target column per row
    float2* partials;        // [M, n_part] (running max, sum of exp) per column slab
    float* target_logit;     // [M]
    int32_t n_part;          // number of column slabs = lmhead_num_partials(...) of this call
    // EPI_QKV_ROPE only:
    const float2* rope;      // [M, 64] (cos, sin) per row and rotation pair
    void* vt;                // [n_kv, 128, ldv] transposed V
    int64_t ldv;
    int32_t n_rot_heads;     // n_q + n_kv: heads (of 128 columns) that are rotated; the rest are V heads
    // EPI_PARTIAL_F32 only:
    int32_t n_slices;        // must equal gemm_partial_slices(dtype, M, N, Kd, a_rows_padded)
};

// Column slabs (partials per row) the LM-head epilogue of this call writes; lmhead_max_partials bounds it for any
// dtype / Kd / padding (workspace sizing).
int32_t lmhead_num_partials(int32_t dtype, int32_t M, int32_t N, int32_t Kd, bool a_rows_padded);
int32_t lmhead_max_partials(int32_t N);
int32_t launch_gemm(int32_t dtype, GemmEpilogue epi, const GemmArgs& g, hipStream_t stream);
// The kernel for at most 16 rows of A (skinny.hip): launch_gemm hands it the calls it serves.
bool gemm_skinny_ok(int32_t dtype, GemmEpilogue epi, const GemmArgs& g);
int32_t launch_gemm_skinny(GemmEpilogue epi, const GemmArgs& g, hipStream_t stream);
// true if the EPI_QKV_ROPE epilogue can serve this QKV projection (else: EPI_STORE_ACT + launch_rope_split)
bool qkv_rope_fusable(int32_t dtype, int32_t M, int32_t N, int32_t Kd, int32_t head_dim, bool a_rows_padded);
// vt [rows, ldv]: zero columns [R, ldv) of every row (the attention kernel reads whole 64-key tiles of V^T).
int32_t launch_zero_vt_tail(int32_t dtype, void* vt, int64_t rows, int32_t R, int64_t ldv, hipStream_t stream);

// lp[b] = target_logit[b] - logsumexp over the n_part partials of row b; rows with valid[b] == 0
// (or b beyond) get 0.  valid may be NULL.
int32_t launch_lmhead_combine(const float2* partials, const float* target_logit, int32_t B, int32_t n_part,
                              const uint8_t* valid, float* lp, hipStream_t stream);

struct ScoreShape {
    int32_t P, K, T;        // prefix length, drafts, padded draft length
    int32_t R() const { return P + K * T; }
    int32_t B() const { return K * T; }
};

int32_t launch_embed(int32_t dtype, const void* tok_embed, int32_t vocab, int32_t d,
                     const int32_t* prefix_ids, const int32_t* draft_ids, const int32_t* draft_lens,
                     ScoreShape s, int32_t row0, float* h, int32_t* err_flag, hipStream_t stream);
int32_t launch_rmsnorm(int32_t dtype, const float* h, const float* gain, float eps, int32_t rows, int32_t d,
                       void* out, hipStream_t stream);
// Several launchers take row0: only rows [row0, R) of the token tree are produced (rows before it belong to a
// cached prefix); buffers are always indexed by absolute row.
// rope table per row of the token tree: cs[r][i] = (cos, sin)(pos(r) * theta^(-2 i / hd)), i < hd / 2
int32_t launch_rope_table(float2* cs, ScoreShape s, int32_t row0, int32_t hd, float theta, hipStream_t stream);
// In-place rotate-half RoPE on the q and k columns of qkv [R, (nq + 2 nkv) hd]; writes V transposed
// to vt [nkv, hd, ldv] (ldv >= R) when vt != NULL.
int32_t launch_rope_split(int32_t dtype, void* qkv, const float2* cs, ScoreShape s, int32_t row0, int32_t nq, int32_t nkv,
                          int32_t hd, void* vt, int64_t ldv, hipStream_t stream);
int32_t launch_transpose_v(int32_t dtype, const void* qkv, int32_t row0, int32_t R, int32_t nq, int32_t nkv, int32_t hd,
                           void* vt, int64_t ldv, hipStream_t stream);
// acc [n_slices][rows, (nq + 2 nkv) hd] fp32 (partial sums of a K-split QKV projection, added here in slice order) -> RoPE
// on the q / k heads (cs, qkv, vt already point at the first of the `rows` rows / columns), stored to qkv; v heads to
// vt [nkv hd, ldv]
int32_t launch_qkv_finish(int32_t dtype, const float* acc, int32_t n_slices, int64_t slice_pitch, const float2* cs, int32_t rows,
                          int32_t nq, int32_t nkv, int32_t hd, void* qkv, void* vt, int64_t ldv, hipStream_t stream);
// K slices an EPI_PARTIAL_F32 projection of this shape is cut into (1: cutting would not help, the caller takes the
// direct epilogue instead).  Depends on the shape only.
int32_t gemm_partial_slices(int32_t dtype, int32_t M, int32_t N, int32_t Kd, bool a_rows_padded);
int32_t skinny_partial_slices(int32_t N, int32_t Kd);     // the same for the kernel that serves at most 16 rows
// h[r] += sum over the slices (in slice order) of partials[s][r]  for `rows` rows of d floats (slice pitch in floats);
// gain != NULL: then xn[r] = rmsnorm(h[r]; gain) in the model dtype (residual update and the next norm in one pass)
int32_t launch_resid_norm(int32_t dtype, float* h, const float* partials, int32_t n_slices, int64_t slice_pitch, const float* gain,
                          float eps, int32_t rows, int32_t d, void* xn, hipStream_t stream);
// dst[r][c] = src[r][c], rows x cols elements of the model dtype, pitches in elements
int32_t launch_copy2d(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int64_t rows, int64_t cols,
                      hipStream_t stream);
// xs[b] = rmsnorm(h[row(b)]) for the B = K T scoring rows; targets[b] / valid[b] from the draft ids.
int32_t launch_gather_norm(int32_t dtype, const float* h, const float* gain, float eps, int32_t d,
                           const int32_t* draft_ids, const int32_t* draft_lens, int32_t vocab, ScoreShape s,
                           void* xs, int32_t* targets, uint8_t* valid, hipStream_t stream);
int32_t launch_score_reduce(const float* lp, const int32_t* draft_lens, int32_t K, int32_t T, int32_t mode,
                            float* token_logprobs, float* scores, hipStream_t stream);

// ---- continuation (decode.hip): key / value cache rows [0, P) prefix, P + j Tc + t = token t of branch j ----------
int32_t launch_tree_rows_to_cache(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int32_t P, int32_t Tn,
                                  int32_t Tc, int32_t rows, int32_t cols, hipStream_t stream);
int32_t launch_transpose_to_rows(int32_t dtype, const void* src, int64_t src_ld, void* dst, int64_t dst_ld, int32_t rows,
                                 int32_t cols, hipStream_t stream);
int32_t launch_embed_rows(int32_t dtype, const void* tok_embed, int32_t vocab, int32_t d, const int32_t* ids, int64_t stride,
                          int32_t rows, float* h, int32_t* err_flag, hipStream_t stream);
// Branch j of a continuation holds len_j = lens[j] draft tokens (read as clamped to [1, T]; T when lens is NULL) and `done`
// generated ones: at(j) = len_j + done is the position, inside the branch, of the row a decoding step appends.
struct BranchPos {
    const int32_t* lens;   // device [Kr] or NULL
    int32_t T, done;
    __device__ int at(int j) const { return (lens ? min(max(lens[j], 1), T) : T) + done; }
};
// cs: (cos, sin) rows indexed by absolute position (prefix length + position in the branch)
// acc [n_slices][Kr, (nq + 2 nkv) hd]: partial sums, added in slice order
int32_t launch_decode_qkv_finish(int32_t dtype, const float* acc, int32_t n_slices, int64_t slice_pitch, const float2* cs, int32_t Kr,
                                 int32_t nq, int32_t nkv, int32_t hd, int32_t P, int32_t Tc, BranchPos pos, void* q_out,
                                 void* k_cache, void* v_cache, hipStream_t stream);
int32_t launch_attn_decode(int32_t dtype, const void* q, const void* k_cache, const void* v_cache, void* out, int32_t Kr, int32_t P,
                           int32_t Tc, BranchPos pos, int32_t nq, int32_t nkv, int32_t hd, hipStream_t stream);
// eos_id >= 0 and has_prev: a row whose previous token (ids[j stride - 1]) is eos_id gets eos_id again
// scratch: argmax_scratch_bytes(rows) bytes (per-slice results of the first of the two launches; launch_sample_rows
// takes the same)
size_t argmax_scratch_bytes(int32_t rows);
int32_t launch_argmax_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, void* scratch, int32_t* ids, int64_t stride,
                           int32_t eos_id, bool has_prev, hipStream_t stream);
int32_t launch_sample_rows(const float* logits, int64_t ld, int32_t V, int32_t rows, float inv_temp, const float* uniforms,
                           void* scratch, int32_t* ids, int64_t stride, int32_t eos_id, bool has_prev, hipStream_t stream);
// xs[j] = rmsnorm(h[first + j step + pos.at(j)])
int32_t launch_norm_strided_rows(int32_t dtype, const float* h, const float* gain, float eps, int32_t d, int64_t first, int64_t step,
                                 BranchPos pos, int32_t rows, void* xs, hipStream_t stream);

// ---- sorting a batch of scores (sort.hip) -----------------------------------------------------------------------
// Ascending order-preserving keys of scores[0, n) (n >= 1).  a, b: two key buffers of at least n rounded up to 16, plus
// 16, words; scratch: sort_scratch_words(n) words.  *sorted is set to whichever of a / b ends up holding the result.
int64_t sort_scratch_words(int64_t n);
int32_t launch_sort_scores(const float* scores, int64_t n, uint32_t* a, uint32_t* b, uint32_t* scratch, const uint32_t** sorted,
                           hipStream_t stream);

bool attention_uses_vt(int32_t dtype, int32_t hd);
// ATTS_OK if launch_attention / launch_attn_decode can serve the context, else ATTS_ERR_SHAPE (host only: callers ask before
// they enqueue anything).  P + T = prefix + longest draft; n_max = keys of the longest branch of a continuation.
int32_t attention_context_check(const char* fn, int32_t dtype, int32_t hd, int32_t P, int32_t T);
int32_t decode_context_check(const char* fn, int32_t dtype, int32_t hd, int64_t n_max);
// queries are the rows [row0, R); keys / values of all rows [0, R) must be present
int32_t launch_attention(int32_t dtype, const void* qkv, const void* vt, int64_t ldv, void* out, ScoreShape s, int32_t row0,
                         int32_t nq, int32_t nkv, int32_t hd, hipStream_t stream);

}  // namespace atts
