// NT GEMM for at most 16 rows of A (bf16):  acc[M, N] = A[M, Kd] . W[N, Kd]^T,  M <= 16.
//
// One decoding step of the target model ("Target Model Sampling": the rejected candidates are continued by the
// target model, one token per step) multiplies a handful of activation rows with every weight matrix once: the
// cost is reading the weights from HBM, so the kernel is organised around keeping many weight bytes in flight
// rather than around the matrix cores.
//
//   * A work item is (group of 32 output columns, slice of the K range) and belongs to ONE wavefront: no LDS, no
//     barrier.  Consecutive wavefronts take neighbouring column groups of the same K slice, so their (identical)
//     A fragments come from the vector L1.
//   * v_mfma_f32_16x16x32_bf16: lane (r = l % 16, q = l / 16) supplies A[r][32 s + 8 q .. + 8] and, for each of
//     the two 16-column blocks, W[col r][same k]; a wave-wide load of W therefore reads 64 contiguous bytes of
//     16 weight rows.  Rows of A beyond M repeat row M - 1 and are dropped by the epilogue.
//   * Weights go global -> registers with kSkinnyUnroll k-steps per buffer and two buffers (ping-pong), so
//     up to 2 x 3 x kSkinnyUnroll 16-byte loads per lane are outstanding while the other buffer feeds the MFMAs.
//     Deeper buffers did not stream faster; what counts is that every CU has about four such wavefronts.
//   * EPI_PARTIAL_F32 cuts the K range into slices (the output is narrow, so column groups alone would leave
//     the chip idle); every slice stores its partial sums in its own copy of the output, and the consumer adds the
//     copies in slice order (no atomics: bit-reproducible).
//     EPI_STORE_F32 and EPI_SWIGLU (gate block + up block of the same 16 features per wavefront) take the
//     whole K range in one wavefront.
#include "common.h"

namespace atts {
namespace {

constexpr int kSkinnyRows = 16;
constexpr int kSkinnyWaves = 4;      // wavefronts (independent work items) per workgroup
constexpr int kSkinnyUnroll = 2;     // k-steps per register buffer
constexpr int kStepElems = 32;       // K elements per MFMA
constexpr int kSkinnyWavesTarget = 1024;   // wavefronts a K-split launch aims for

struct SkinnyDims {
    int32_t M, N, n_w_rows;
    int64_t lda, ldw, ldc;
    int32_t n_groups, k_slices, n_steps, steps_per_slice;
    int64_t slice_pitch;
};

struct SkinnyFrags {
    bf16x8 a[kSkinnyUnroll], w0[kSkinnyUnroll], w1[kSkinnyUnroll];
};

template <int EPI>
__global__ __launch_bounds__(64 * kSkinnyWaves) void gemm_skinny_kernel(const bf16* __restrict__ gA, const bf16* __restrict__ gW,
                                                                        void* __restrict__ g_out, SkinnyDims d) {
    const int lane = threadIdx.x & 63;
    // The wavefront index is made a scalar: every branch on the K range below must be a scalar branch, because the
    // matrix instructions do not honour the lane mask that a (seemingly) divergent branch would be turned into.
    const int item = blockIdx.x * kSkinnyWaves + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (item >= d.n_groups * d.k_slices) return;     // whole wavefronts leave; nothing below synchronises
    const int grp = item % d.n_groups, slice = item / d.n_groups;
    const int r = lane & 15, q = lane >> 4;
    const int ks0 = slice * d.steps_per_slice;
    const int ks1 = min(ks0 + d.steps_per_slice, d.n_steps);

    // weight rows of the two column blocks (clamped: the epilogue drops columns beyond N)
    int c0, c1;
    if constexpr (EPI == EPI_SWIGLU) {
        c0 = min(grp * 16 + r, d.N - 1);          // gate row of feature grp 16 + r
        c1 = d.N + c0;                            // its up row
    } else {
        c0 = min(grp * 32 + r, d.n_w_rows - 1);
        c1 = min(grp * 32 + 16 + r, d.n_w_rows - 1);
    }
    const bf16* ap = gA + (int64_t)min(r, d.M - 1) * d.lda + q * 8;
    const bf16* w0p = gW + (int64_t)c0 * d.ldw + q * 8;
    const bf16* w1p = gW + (int64_t)c1 * d.ldw + q * 8;

    auto load = [&](SkinnyFrags& f, int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSkinnyUnroll; ++u) {
            const int64_t off = (int64_t)min(ks + u, ks1 - 1) * kStepElems;     // past the end: a repeat, not used
            f.w0[u] = *reinterpret_cast<const bf16x8*>(w0p + off);
            f.w1[u] = *reinterpret_cast<const bf16x8*>(w1p + off);
            f.a[u] = *reinterpret_cast<const bf16x8*>(ap + off);
        }
    };
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    auto mma = [&](const SkinnyFrags& f, int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSkinnyUnroll; ++u)
            if (ks + u < ks1) {                      // wave-uniform
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[u], f.w0[u], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[u], f.w1[u], acc1, 0, 0, 0);
            }
    };

    SkinnyFrags fa, fb;
    load(fa, ks0);
    for (int ks = ks0; ks < ks1; ks += 2 * kSkinnyUnroll) {
        // the loads are issued on every path (past the end they repeat the last k-step and hit the cache): the count
        // of outstanding loads is then known at compile time and the MFMAs wait only for their own buffer
        load(fb, ks + kSkinnyUnroll);
        mma(fa, ks);
        load(fa, ks + 2 * kSkinnyUnroll);
        mma(fb, ks + kSkinnyUnroll);                 // skips the k-steps past the end
    }

    // acc[v] is element (row 4 q + v, column r) of its 16 x 16 block
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int row = 4 * q + v;
        if (row >= d.M) continue;
        if constexpr (EPI == EPI_SWIGLU) {
            const int col = grp * 16 + r;
            if (col < d.N) {
                const float gate = acc0[v], up = acc1[v];
                const float y = gate * __builtin_amdgcn_rcpf(1.f + __expf(-gate)) * up;   // hardware reciprocal, as in the tiled kernels
                reinterpret_cast<bf16*>(g_out)[(int64_t)row * d.ldc + col] = from_f32<bf16>(y);
            }
        } else {
            float* out = reinterpret_cast<float*>(g_out) + (int64_t)slice * d.slice_pitch + (int64_t)row * d.ldc;   // pitch 0 unless partial
            const int col0 = grp * 32 + r, col1 = col0 + 16;
            if (col0 < d.N) out[col0] = acc0[v];
            if (col1 < d.N) out[col1] = acc1[v];
        }
    }
}

// K steps per slice of the partial-sum form: about four wavefronts per CU stream fastest (measured: fewer leave CUs
// idle, many more shorten every wavefront's run), each with at least two buffers of k-steps
int32_t skinny_steps_per_slice(int32_t N, int32_t Kd) {
    const int64_t n_groups = ceil_div(N, 32), n_steps = Kd / kStepElems;
    int64_t s = kSkinnyWavesTarget / n_groups;
    const int64_t max_s = n_steps / (2 * kSkinnyUnroll);
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    return (int32_t)align_up((size_t)ceil_div(n_steps, s), 2 * kSkinnyUnroll);
}

template <int EPI>
int32_t launch_skinny_epi(const GemmArgs& g, hipStream_t stream) {
    SkinnyDims d;
    d.M = g.M; d.N = g.N;
    d.n_w_rows = EPI == EPI_SWIGLU ? 2 * g.N : g.N;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc;
    d.n_groups = (int32_t)ceil_div(g.N, EPI == EPI_SWIGLU ? 16 : 32);
    d.n_steps = g.Kd / kStepElems;
    d.k_slices = 1;
    d.steps_per_slice = d.n_steps;
    d.slice_pitch = 0;
    if (EPI == EPI_PARTIAL_F32) {
        d.steps_per_slice = skinny_steps_per_slice(g.N, g.Kd);
        d.k_slices = (int32_t)ceil_div(d.n_steps, d.steps_per_slice);
        d.slice_pitch = (int64_t)g.M * g.ldc;
    }
    const int64_t items = (int64_t)d.n_groups * d.k_slices;
    hipLaunchKernelGGL(gemm_skinny_kernel<EPI>, dim3((unsigned)ceil_div(items, kSkinnyWaves)), dim3(64 * kSkinnyWaves), 0, stream,
                       reinterpret_cast<const bf16*>(g.a), reinterpret_cast<const bf16*>(g.w), g.out, d);
    ATTS_LAUNCH_CHECK("gemm_skinny_kernel");
    return ATTS_OK;
}

}  // namespace

bool gemm_skinny_ok(int32_t dtype, GemmEpilogue epi, const GemmArgs& g) {
    return dtype == ATTS_DTYPE_BF16 && (epi == EPI_STORE_F32 || epi == EPI_PARTIAL_F32 || epi == EPI_SWIGLU) && g.M >= 1 &&
           g.M <= kSkinnyRows && g.N >= 1 && g.Kd >= kStepElems && g.Kd % kStepElems == 0 && g.lda % 8 == 0 && g.ldw % 8 == 0 &&
           (int64_t)g.N * (epi == EPI_SWIGLU ? 2 : 1) < (1ll << 30);
}

int32_t skinny_partial_slices(int32_t N, int32_t Kd) {
    return (int32_t)ceil_div(Kd / kStepElems, skinny_steps_per_slice(N, Kd));
}

int32_t launch_gemm_skinny(GemmEpilogue epi, const GemmArgs& g, hipStream_t stream) {
    switch (epi) {
        case EPI_STORE_F32: return launch_skinny_epi<EPI_STORE_F32>(g, stream);
        case EPI_PARTIAL_F32: return launch_skinny_epi<EPI_PARTIAL_F32>(g, stream);
        case EPI_SWIGLU: return launch_skinny_epi<EPI_SWIGLU>(g, stream);
        default: break;
    }
    return fail(ATTS_ERR_INVALID_ARG, "gemm (few rows): epilogue %d is not served", (int)epi);
}

}  // namespace atts
