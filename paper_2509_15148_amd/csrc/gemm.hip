// NT GEMM on MFMA for gfx950:  acc[M, N] = A[M, Kd] . W[N, Kd]^T  with fused epilogues.
//
// Every linear map of the target model (QKV, attention output, SwiGLU feed-forward, LM head)
// goes through one of the kernels below; scoring the drafts is the compute-bound part of the
// method (Sec. "Q1"), so this is where the time goes.
//
//   gemm_bf16_wide_kernel   aligned bf16 shapes (every projection of the bf16 models): 8 wavefronts,
//                           384 x 256, 256 x 256 or 128 x 256 output tiles, operand slabs of 128 bytes
//                           per row DMA-ed global -> LDS in whole 128-byte lines, explicit waits.
//   gemm_nt_kernel          any shape, bf16 or fp32 (v_mfma_f32_32x32x2_f32): 4 wavefronts (2 x 2),
//                           tile BM x BN, 128-byte slabs through registers with bounds checks,
//                           double-buffered, one barrier per slab; LDS chunk index XOR (row >> 1) & 7.
// All share gemm_epilogue (store / fp32 residual add / SwiGLU / LM-head partials / QKV + RoPE) and the
// workgroup-id remap that hands each XCD (id mod 8) a compact block of tiles, so that its private L2
// re-uses A and W slabs.
#include "common.h"

#include <atomic>
#include <type_traits>

namespace atts {
namespace {

constexpr int kThreads = 256;
constexpr int kRowBytes = 128;  // bytes of K per LDS row per slab

template <typename T> struct Mma;

template <> struct Mma<bf16> {
    static constexpr int kSteps = 4;  // 16-wide k-steps per 64-element slab
    typedef bf16x8 Frag;
    // lane (row = l % 32, half = l / 32) holds k = 16 step + 8 half + [0, 8)
    static __device__ __forceinline__ Frag load(const char* row_ptr, int row, int step, int half) {
        int chunk = step * 2 + half;
        return *reinterpret_cast<const Frag*>(row_ptr + ((chunk ^ ((row >> 1) & 7)) << 4));
    }
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

template <> struct Mma<float> {
    static constexpr int kSteps = 8;  // one 16-byte chunk (4 floats) per step, two MFMAs
    typedef float2 Frag;
    // half h of the wave takes floats 2h, 2h+1 of the chunk: the k-order inside a chunk is
    // permuted identically for A and W, which leaves the dot product unchanged.
    static __device__ __forceinline__ Frag load(const char* row_ptr, int row, int step, int half) {
        return *reinterpret_cast<const Frag*>(row_ptr + ((step ^ ((row >> 1) & 7)) << 4) + half * 8);
    }
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, c, 0, 0, 0);
    }
};

struct TileCoord {
    int tm, tn;
};

// XCD-aware, grouped tile order.
// round > 0: the launch has `round` workgroups that walk the tiles in rounds (pid = workgroup + i round); the tiles of
// one round are then `round` consecutive positions of the order, dealt to the XCDs in blocks, so that at any time the
// whole chip works inside one group of tile rows and its A rows stay in the Infinity Cache whatever the size of A
// (with the XCDs spread over the whole order instead, eight groups are live at once: 250 MB of A rows at the 32B
// workload, which the streaming W rows then push out; measured there 1993 -> 1881 ms per step, nothing at 7B).
template <int kGroupM = 8>
__device__ __forceinline__ TileCoord tile_of_block(int pid, int nt_m, int nt_n, int round = 0) {
    int n = nt_m * nt_n;
    int base = 0;
    if (round > 0) {
        base = pid / round * round;
        pid -= base;
        n = min(round, n - base);
    }
    int n8 = n & ~7;
    int lid = base + (pid < n8 ? (pid & 7) * (n8 >> 3) + (pid >> 3) : pid);
    int per_group = kGroupM * nt_n;
    int g = lid / per_group;
    int first_m = g * kGroupM;
    int gsz = min(kGroupM, nt_m - first_m);
    int in_g = lid - g * per_group;
    TileCoord t;
    t.tm = first_m + in_g % gsz;
    t.tn = in_g / gsz;
    return t;
}


// Scalars of one GEMM launch (pointers are passed as direct kernel arguments so that the compiler
// knows they are global addresses).
struct GemmDims {
    int32_t M, N, Kd;
    int64_t lda, ldw, ldc;
    int32_t n_part, nt_m, nt_n;
    int32_t round;          // workgroups of a tile-walking launch (0: one workgroup per tile)
    int64_t ldv;            // EPI_QKV_ROPE: row pitch of the transposed V
    int32_t n_rot_heads;    // EPI_QKV_ROPE: heads (128 columns each) that get rotated; later heads are V
    int32_t k_slices;       // EPI_PARTIAL_F32: the K range is split over this many workgroups per tile, slice s stores
    int64_t slice_pitch;    // its partial sums at out + s slice_pitch (floats); 1 for every other epilogue
};


// Epilogue shared by both kernels.  acc[i][j][v] is element (row, col) of the tile with
//   row = wm WM + 32 i + 8 (v / 4) + 4 half + (v % 4),   col = wn WN + 32 j + l32   (WM = 32 MI, WN = 32 NI).
// Start of a tile's accumulators: zero, or (EPI_RESID_F32) the old values of the output tile, so that the residual update
// out += A W^T is the accumulation itself and the epilogue is a plain store.  The old values are then requested while the
// first slabs are still on their way, instead of at the end of the tile, where every workgroup of a one-round launch
// would wait for them at once (7B step: O and down projections 1.9 ms faster than with a load / add / store epilogue);
// no atomics, one writer per element.
template <int MI, int NI, int EPI, bool kWide = false>
__device__ __forceinline__ void start_accumulators(f32x16 (&acc)[MI][NI], int m0, int n0, int wm, int wn, int l32, int half,
                                                   const void* __restrict__ g_out, const GemmDims& g) {
    constexpr int WM = 32 * MI, WN = 32 * NI;
    if constexpr (kWide && EPI == EPI_RESID_F32) {
        // aligned kernel: whole tiles in the column direction; addresses as wave-uniform base + lane offset, rows of a
        // last, partial tile row clamped to the last existing one (only when the wave-uniform test says there are any)
        const int rows_left = g.M - (m0 + wm * WM);
        const char* const wave_base = reinterpret_cast<const char*>(g_out) + ((int64_t)(m0 + wm * WM) * g.ldc + n0 + wn * WN) * 4;
        const uint32_t lane_off = (uint32_t)((4 * half * g.ldc + l32) * 4);
        auto rows = [&](auto checked) __attribute__((always_inline)) {
            constexpr bool kChecked = decltype(checked)::value;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = 32 * i + 8 * (v >> 2) + (v & 3);
                    const char* p = wave_base + (int64_t)r * g.ldc * 4 + lane_off;
                    if (kChecked) {     // this lane's row, clamped to the last row of the output (what it starts from is never stored)
                        const int row = min(m0 + wm * WM + r + 4 * half, g.M - 1);
                        p = reinterpret_cast<const char*>(g_out) + ((int64_t)row * g.ldc + n0 + wn * WN + l32) * 4;
                    }
#pragma unroll
                    for (int j = 0; j < NI; ++j) acc[i][j][v] = *reinterpret_cast<const float*>(p + 32 * j * 4);
                }
        };
        if (rows_left >= WM) rows(std::false_type{}); else rows(std::true_type{});
        return;
    }
    const int row_base = m0 + wm * WM + 4 * half, col_base = n0 + wn * WN + l32;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[i][j][v] = 0.f;
                if (EPI == EPI_RESID_F32) {
                    // rows and columns past the end are clamped, not skipped (no branches: the loads go out back to
                    // back); what they start from is never stored
                    const int row = min(row_base + 32 * i + 8 * (v >> 2) + (v & 3), g.M - 1);
                    const int col = min(col_base + 32 * j, g.N - 1);
                    acc[i][j][v] = reinterpret_cast<const float*>(g_out)[(int64_t)row * g.ldc + col];
                }
            }
}

// kWide: called by the aligned kernel, whose tiles are whole in the column direction.  The plain stores and the SwiGLU
// then go without per-element checks (one wave-uniform test tells whether the tile is whole in the row direction too) and
// address each element as a wave-uniform base (scalar arithmetic) plus one 32-bit lane offset: the checked form costs
// about 25 instructions and a branch or two per element, which at 96 - 192 elements per lane and tile was a tenth of the
// gate/up tile's time with the matrix pipe idle.
template <typename T, int MI, int NI, int EPI, bool kWide = false>
__device__ __forceinline__ void gemm_epilogue_impl(f32x16 (&acc)[MI][NI], int m0, int n0, int wm, int wn, int l32, int half,
                                                   int tn, void* __restrict__ g_out, const int32_t* __restrict__ g_targets,
                                                   float2* __restrict__ g_partials, float* __restrict__ g_target_logit,
                                                   const float2* __restrict__ g_rope, void* __restrict__ g_vt,
                                                   const GemmDims& g) {
    constexpr int WM = 32 * MI, WN = 32 * NI;
    const int row_base = m0 + wm * WM + 4 * half;

    constexpr bool kPlain = EPI == EPI_STORE_ACT || EPI == EPI_STORE_F32 || EPI == EPI_RESID_F32 || EPI == EPI_PARTIAL_F32;
    if constexpr (kWide && (kPlain || EPI == EPI_SWIGLU)) {
        constexpr int kOutCols = EPI == EPI_SWIGLU ? WN / 2 : WN;      // output columns of this wave
        constexpr int kJ = EPI == EPI_SWIGLU ? NI / 2 : NI;
        constexpr int ES = (EPI == EPI_STORE_ACT || EPI == EPI_SWIGLU) ? (int)sizeof(T) : 4;
        const int rows_left = g.M - (m0 + wm * WM);                     // wave-uniform; >= WM: every row of the wave exists
        char* const wave_base = reinterpret_cast<char*>(g_out) + ((int64_t)(m0 + wm * WM) * g.ldc + n0 + wn * kOutCols) * ES;
        const uint32_t lane_off = (uint32_t)((4 * half * g.ldc + l32) * ES);
        auto value = [&](int i, int j, int v) __attribute__((always_inline)) {
            if constexpr (EPI == EPI_SWIGLU) {
                // blocks j < NI/2 hold gate, j + NI/2 the matching up columns; silu(gate) up with the hardware reciprocal
                // (1 ulp) instead of an IEEE division and its ten-instruction expansion
                const float gate = acc[i][j][v], up = acc[i][j + NI / 2][v];
                return gate * __builtin_amdgcn_rcpf(1.f + __expf(-gate)) * up;
            } else {
                return acc[i][j][v];
            }
        };
        auto rows = [&](auto checked) __attribute__((always_inline)) {
            constexpr bool kChecked = decltype(checked)::value;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = 32 * i + 8 * (v >> 2) + (v & 3);     // + 4 half: in lane_off
                    if (kChecked && r + 4 * half >= rows_left) continue;
                    char* const p = wave_base + (int64_t)r * g.ldc * ES + lane_off;
#pragma unroll
                    for (int j = 0; j < kJ; ++j) {
                        const float y = value(i, j, v);
                        if (ES == (int)sizeof(T) && ES != 4) *reinterpret_cast<T*>(p + 32 * j * ES) = from_f32<T>(y);
                        else *reinterpret_cast<float*>(p + 32 * j * ES) = y;
                    }
                }
        };
        if (rows_left >= WM) rows(std::false_type{}); else rows(std::true_type{});
    } else if constexpr (kPlain) {
        const int col_base = n0 + wn * WN + l32;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
                if (row >= g.M) continue;
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    int col = col_base + 32 * j;
                    if (col >= g.N) continue;
                    int64_t idx = (int64_t)row * g.ldc + col;
                    if (EPI == EPI_STORE_ACT) reinterpret_cast<T*>(g_out)[idx] = from_f32<T>(acc[i][j][v]);
                    // (EPI_PARTIAL_F32: slice base in g_out; EPI_RESID_F32: the accumulators started from the old values)
                    if (EPI == EPI_STORE_F32 || EPI == EPI_PARTIAL_F32 || EPI == EPI_RESID_F32) reinterpret_cast<float*>(g_out)[idx] = acc[i][j][v];
                }
            }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // blocks j < NI/2 hold gate, j + NI/2 the matching up columns
        const int col_base = n0 + wn * (WN / 2) + l32;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
                if (row >= g.M) continue;
#pragma unroll
                for (int j = 0; j < NI / 2; ++j) {
                    int col = col_base + 32 * j;
                    if (col >= g.N) continue;
                    float gate = acc[i][j][v], up = acc[i][j + NI / 2][v];
                    // silu(gate) up with the hardware reciprocal (1 ulp) instead of an IEEE division, whose ten-instruction
                    // expansion per element made this epilogue cost about as much again as its exponentials
                    float y = gate * __builtin_amdgcn_rcpf(1.f + __expf(-gate)) * up;
                    reinterpret_cast<T*>(g_out)[(int64_t)row * g.ldc + col] = from_f32<T>(y);
                }
            }
    } else if constexpr (EPI == EPI_QKV_ROPE) {
        // The wave's 128 columns are exactly one head (head_dim 128): blocks j = 0, 1 hold dims 0..63 and blocks
        // j + 2 the partner dims 64..127 of the rotate-half pairing, in the same lane.
        static_assert(NI == 4 && sizeof(T) == 2, "QKV epilogue needs 128-column bf16 wave tiles");
        const int col0 = n0 + wn * WN;
        const int head = col0 / 128;                                  // wave-uniform
        // Addresses as a wave-uniform base plus one lane offset, and one wave-uniform test for "every row of the wave
        // exists" instead of a test per element (as in the plain stores above).
        const int wrow0 = m0 + wm * WM;                               // first row of the wave
        const int rows_left = g.M - wrow0;
        if (head < g.n_rot_heads) {
            char* const obase = reinterpret_cast<char*>(g_out) + ((int64_t)wrow0 * g.ldc + col0) * sizeof(T);
            const char* const cbase = reinterpret_cast<const char*>(g_rope + (int64_t)wrow0 * 64);
            const uint32_t o_lane = (uint32_t)((4 * half * g.ldc + l32) * sizeof(T));
            const uint32_t c_lane = (uint32_t)((4 * half * 64 + l32) * sizeof(float2));
            // The (cos, sin) pairs of eight rows are requested together and only then used: the compiler keeps every load
            // behind the stores in front of it, so one row at a time means one exposed L2 round trip per row.
            auto rows = [&](auto checked) __attribute__((always_inline)) {
                constexpr bool kChecked = decltype(checked)::value;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int a2 = 0; a2 < 2; ++a2) {
                        float2 cs[8][2];
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int r = 32 * i + 8 * (2 * a2 + (q >> 2)) + (q & 3);
                            const int rc = kChecked ? min(r, max(rows_left - 1 - 4 * half, 0)) : r;     // a row that exists
                            const float2* crow = reinterpret_cast<const float2*>(cbase + (int64_t)rc * 64 * sizeof(float2) + c_lane);
                            cs[q][0] = crow[0];
                            cs[q][1] = crow[32];
                        }
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int v = 4 * (2 * a2 + (q >> 2)) + (q & 3);
                            const int r = 32 * i + 8 * (v >> 2) + (v & 3);
                            if (kChecked && r + 4 * half >= rows_left) continue;
                            T* orow = reinterpret_cast<T*>(obase + (int64_t)r * g.ldc * sizeof(T) + o_lane);
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const float x1 = acc[i][j][v], x2 = acc[i][j + 2][v];
                                orow[32 * j] = from_f32<T>(x1 * cs[q][j].x - x2 * cs[q][j].y);
                                orow[32 * j + 64] = from_f32<T>(x2 * cs[q][j].x + x1 * cs[q][j].y);
                            }
                        }
                    }
            };
            if (rows_left >= WM) rows(std::false_type{}); else rows(std::true_type{});
        } else {
            // V head: lane holds 4 consecutive rows (v % 4) of one head dim -> one 8-byte store into V^T
            typedef T T4 __attribute__((ext_vector_type(4)));
            char* const vbase = reinterpret_cast<char*>(g_vt) + ((int64_t)(head - g.n_rot_heads) * 128 * g.ldv + wrow0) * sizeof(T);
            const uint32_t v_lane = (uint32_t)(((int64_t)l32 * g.ldv + 4 * half) * sizeof(T));
            auto rows = [&](auto checked) __attribute__((always_inline)) {
                constexpr bool kChecked = decltype(checked)::value;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const int r0 = 32 * i + 8 * a + 4 * half;     // first of the lane's 4 consecutive rows, relative to the wave
                        if (kChecked && r0 >= rows_left) continue;
#pragma unroll
                        for (int j = 0; j < NI; ++j) {
                            T4 o4;
#pragma unroll
                            for (int b = 0; b < 4; ++b) o4[b] = from_f32<T>(acc[i][j][4 * a + b]);
                            T* dst = reinterpret_cast<T*>(vbase + ((int64_t)(32 * j) * g.ldv + 32 * i + 8 * a) * sizeof(T) + v_lane);
                            if (!kChecked || r0 + 4 <= rows_left) {
                                *reinterpret_cast<T4*>(dst) = o4;
                            } else {
#pragma unroll
                                for (int b = 0; b < 4; ++b)
                                    if (r0 + b < rows_left) dst[b] = o4[b];
                            }
                        }
                    }
            };
            if (rows_left >= WM) rows(std::false_type{}); else rows(std::true_type{});
        }
    } else if constexpr (EPI == EPI_LMHEAD) {
        // One (max, sum exp) partial per row for this wave's WN columns, plus the target logit.
        const int col0 = n0 + wn * WN;            // first column of this wave's slab
        const int part = tn * 2 + wn;
        bool col_ok[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) col_ok[j] = col0 + 32 * j + l32 < g.N;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
                bool row_ok = row < g.M;          // uniform over the 32 lanes that share `half`
                int tcol = row_ok ? g_targets[row] - col0 : -1;
                float mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    float z = acc[i][j][v];
                    if (col_ok[j]) mx = fmaxf(mx, z);
                    if (tcol == 32 * j + l32) g_target_logit[row] = z;
                }
#pragma unroll
                for (int o = 1; o < 32; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
                float sum = 0.f;
                if (mx > -INFINITY) {
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        if (col_ok[j]) sum += __expf(acc[i][j][v] - mx);
                }
#pragma unroll
                for (int o = 1; o < 32; o <<= 1) sum += __shfl_xor(sum, o);
                if (row_ok && l32 == 0) g_partials[(int64_t)row * g.n_part + part] = make_float2(mx, sum);
            }
    } else if constexpr (EPI == EPI_LMHEAD_T) {
        // Operands exchanged: the rows of this product are vocabulary entries (g.M of them), its columns the scoring rows.
        // A lane holds, for each of its NI scoring rows, the logits of the 16 MI vocabulary entries of its wave's row
        // block: maximum and sum of exponentials are taken inside the lane (no cross-lane reduction per scoring row, where
        // the other orientation needs ten), the two lane halves are merged with one exchange, and the wave's partial goes to
        // slot (tile row, wave row).  The target logit is stored by the lane that holds the target's vocabulary entry.
        const int part = (m0 / (4 * WM)) * 4 + wm;
        const int vrow0 = m0 + wm * WM + 4 * half;     // every vocabulary row of the tile exists (whole tiles, checked on the host)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn * WN + 32 * j + l32;              // scoring row; < g.N (whole tiles too)
            float mx = acc[0][j][0];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int v = (i == 0 ? 1 : 0); v < 16; ++v) mx = fmaxf(mx, acc[i][j][v]);
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) sum += __expf(acc[i][j][v] - mx);
            // The target's vocabulary entry relative to this lane's first one: the lane holds entries 32 i + 8 a + b
            // (b < 4).  Only about one wave in twelve holds any of its 128 scoring rows' targets, so the selection of the
            // accumulator entry sits behind a branch that is mostly not taken.
            const int trel = g_targets[col] - vrow0;
            if (trel >= 0 && trel < WM && (trel & 4) == 0) {
                const int ti = trel >> 5, tv = ((trel >> 3) & 3) * 4 + (trel & 3);
                float z = 0.f;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) z = (ti == i && tv == v) ? acc[i][j][v] : z;
                g_target_logit[col] = z;
            }
            // merge with the other half of the lane pair (l, l ^ 32): same scoring row, the rows in between
            const float mx_o = __shfl_xor(mx, 32), sum_o = __shfl_xor(sum, 32);
            const float m = fmaxf(mx, mx_o);
            float tot = 0.f;
            if (m > -INFINITY) tot = sum * __expf(mx - m) + sum_o * __expf(mx_o - m);   // a half with no entry: 0 * exp(-inf) = 0
            if (half == 0) g_partials[(int64_t)col * g.n_part + part] = make_float2(m, tot);
        }
    }
}

template <typename T, int MI, int NI, int EPI>
__device__ __forceinline__ void gemm_epilogue(f32x16 (&acc)[MI][NI], int m0, int n0, int wm, int wn, int l32, int half,
                                              int tn, void* __restrict__ g_out, const int32_t* __restrict__ g_targets,
                                              float2* __restrict__ g_partials, float* __restrict__ g_target_logit,
                                              const float2* __restrict__ g_rope, void* __restrict__ g_vt,
                                              const GemmDims& g) {
    gemm_epilogue_impl<T, MI, NI, EPI>(acc, m0, n0, wm, wn, l32, half, tn, g_out, g_targets, g_partials, g_target_logit, g_rope,
                                       g_vt, g);
}

template <typename T, int BM, int BN, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_nt_kernel(const char* __restrict__ gA, const char* __restrict__ gW,
                                                           void* __restrict__ g_out,
                                                           const int32_t* __restrict__ g_targets,
                                                           float2* __restrict__ g_partials,
                                                           float* __restrict__ g_target_logit,
                                                           const float2* __restrict__ g_rope, void* __restrict__ g_vt,
                                                           const GemmDims g) {
    constexpr int MI = BM / 64, NI = BN / 64;   // 32x32 blocks per wave along M / N
    constexpr int WM = BM / 2, WN = BN / 2;     // wave tile
    constexpr int kElemsPerChunk = 16 / (int)sizeof(T);
    constexpr int kSlabElems = kRowBytes / (int)sizeof(T);
    constexpr int A_CHUNKS = BM * 8 / kThreads, B_CHUNKS = BN * 8 / kThreads;
    constexpr int N_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;   // output columns per tile

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sA = smem;                           // [2][BM][128 B]
    char* sB = smem + 2 * BM * kRowBytes;      // [2][BN][128 B]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    const TileCoord tc = tile_of_block(blockIdx.x, g.nt_m, g.nt_n);
    const int m0 = tc.tm * BM;
    const int n0 = tc.tn * N_OUT;

    // Per-thread chunk coordinates: chunk c = tid + 256 i -> tile row (tid / 8) + 32 i, 16-byte
    // column tid % 8.  Row i of a thread differs from row 0 by a wave-uniform offset, so one base
    // pointer per operand is kept and the per-row offsets stay in scalar registers.
    const int crow = tid >> 3, ccol = tid & 7;
    const int64_t es = (int64_t)sizeof(T);
    const char* a_base = gA + ((int64_t)(m0 + crow) * g.lda + ccol * kElemsPerChunk) * es;
    const char* b_base = gW + ((int64_t)(n0 + crow) * g.ldw + ccol * kElemsPerChunk) * es;
    const int lds_off = crow * kRowBytes + ((ccol ^ ((crow >> 1) & 7)) << 4);  // + 32 i rows: swizzle term unchanged

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];

    auto load_slab = [&](int k0) __attribute__((always_inline)) {
        const bool k_ok = k0 + ccol * kElemsPerChunk < g.Kd;
        const int64_t koff = (int64_t)k0 * es;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const bool ok = k_ok && (m0 + crow + 32 * i < g.M);
            ra[i] = make_uint4(0, 0, 0, 0);
            if (ok) ra[i] = *reinterpret_cast<const uint4*>(a_base + koff + (int64_t)(32 * i) * g.lda * es);
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            // LDS row j = crow + 32 i of the W tile  <-  W row (n0 + crow) + row_off
            int64_t row_off;
            bool ok;
            if (EPI == EPI_SWIGLU) {
                // wave slab jw holds [gate | up] halves of WN / 2 features each
                constexpr int H = WN / 2;
                const int jw = (32 * i) / WN, jj = (32 * i) % WN;
                const int up = jj / H, feat_off = jw * H + jj % H;
                ok = n0 + crow + feat_off < g.N;
                row_off = (int64_t)up * g.N + feat_off;
            } else {
                ok = n0 + crow + 32 * i < g.N;
                row_off = 32 * i;
            }
            rb[i] = make_uint4(0, 0, 0, 0);
            if (ok && k_ok) rb[i] = *reinterpret_cast<const uint4*>(b_base + koff + row_off * g.ldw * es);
        }
    };
    auto store_slab = [&](int buf) __attribute__((always_inline)) {
        char* dA = sA + buf * BM * kRowBytes + lds_off;
        char* dB = sB + buf * BN * kRowBytes + lds_off;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<uint4*>(dA + i * 32 * kRowBytes) = ra[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<uint4*>(dB + i * 32 * kRowBytes) = rb[i];
    };

    f32x16 acc[MI][NI];
    start_accumulators<MI, NI, EPI>(acc, m0, n0, wm, wn, l32, half, g_out, g);

    const int nk = (g.Kd + kSlabElems - 1) / kSlabElems;
    load_slab(0);
    store_slab(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_slab((kt + 1) * kSlabElems);

        const char* pA = sA + buf * BM * kRowBytes + (wm * WM + l32) * kRowBytes;
        const char* pB = sB + buf * BN * kRowBytes + (wn * WN + l32) * kRowBytes;
#pragma unroll
        for (int s = 0; s < Mma<T>::kSteps; ++s) {
            typename Mma<T>::Frag fa[MI], fb[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[i] = Mma<T>::load(pA + i * 32 * kRowBytes, l32, s, half);
#pragma unroll
            for (int j = 0; j < NI; ++j) fb[j] = Mma<T>::load(pB + j * 32 * kRowBytes, l32, s, half);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) Mma<T>::mma(fa[i], fb[j], acc[i][j]);
        }

        if (kt + 1 < nk) store_slab(buf ^ 1);
        __syncthreads();
    }

    gemm_epilogue<T, MI, NI, EPI>(acc, m0, n0, wm, wn, l32, half, tc.tn, g_out, g_targets, g_partials, g_target_logit, g_rope, g_vt, g);
}

// ---------------------------------------------------------------------------------------------
// Wide-slab variant of the aligned kernel: 128 bytes of K per row and slab, so that every DMA instruction
// asks L2 for whole 128-byte lines (8 rows x 128 B instead of 16 rows x 64 B).  L2 -> LDS delivery, which bounds
// the 64-byte version, is ~1.4x faster that way; the price is LDS: 160 KB hold only 2.5 slabs of a 256 x 256 tile
// (a ring of five 32 KB units A0 W0 A1 W1 A2 ...: the A rows run two slabs ahead, the W rows one) or two slabs of
// a 384 x 256 tile.  A slab is four MFMA k-steps; the DMA of the following slabs is issued under the first two
// (under the first alone with two stages), one wait + barrier per slab at its end.
// ---------------------------------------------------------------------------------------------
template <int EPI, int kWavesM, int MI, int NI = 4 /* 32-column blocks per wave: 4 = 256-column tiles, 2 = 128-column tiles */>
__global__ __launch_bounds__(128 * kWavesM) void gemm_bf16_wide_kernel(const char* __restrict__ gA,
                                                                       const char* __restrict__ gW,
                                                                       void* __restrict__ g_out,
                                                                       const int32_t* __restrict__ g_targets,
                                                                       float2* __restrict__ g_partials,
                                                                       float* __restrict__ g_target_logit,
                                                                       const float2* __restrict__ g_rope,
                                                                       void* __restrict__ g_vt, const GemmDims g) {
    constexpr int WN = 32 * NI, BN = 2 * WN;
    constexpr int WM = 32 * MI, BM = kWavesM * WM;
    constexpr int kWaves = 2 * kWavesM;
    constexpr int N_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
    constexpr int BKB = 128, BK = BKB / 2, CHUNKS = BKB / 16;   // four MFMA k-steps per slab
    constexpr int ROWS_PER_DMA = 1024 / BKB;                     // 8
    constexpr int DMA_A = BM / ROWS_PER_DMA / kWaves, DMA_B = BN / ROWS_PER_DMA / kWaves;
    static_assert(DMA_A % 2 == 0 && DMA_B % 2 == 0, "the swizzle parity of a DMA instruction must not depend on the wave");
    constexpr bool kDeep = BM == 256;                            // five-unit ring, A two slabs ahead
    constexpr int kStages = BM == 128 ? 3 : 2;                   // whole-slab stages otherwise (160 KB of LDS)
    constexpr int UNIT_A = BM * BKB, UNIT_B = BN * BKB;
    static_assert(!kDeep || UNIT_A == UNIT_B, "ring units must have one size");

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    const int n_tiles = g.nt_m * g.nt_n;
    const int slice = g.k_slices > 1 ? (int)blockIdx.x / n_tiles : 0;
    const int nk_all = g.Kd / BK;
    const int k_first = (int)((int64_t)slice * nk_all / g.k_slices);
    const int nk = (int)((int64_t)(slice + 1) * nk_all / g.k_slices) - k_first;   // >= 3 (checked on the host)
    // Two-stage form without a K split: a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... and requests
    // the first slab of the next tile under the last slab of the current one, so that the DMA ring never runs dry at a
    // tile boundary and the epilogue's stores overlap that request.  (The host launches one workgroup per CU then;
    // with a grid of n_tiles workgroups the loop body runs once.)
    constexpr bool kTileLoop = !kDeep && kStages == 2;
    // Tile rows per group of the XCD-aware order.  The one-round calls of the 256-row tile do better with taller groups
    // (an XCD then touches fewer W columns, which come cold from HBM, at the price of more A rows, which the Infinity
    // Cache holds): O projection at 7B 3.79 -> 3.66 ms per step with 12 against 8, the other shapes within 0.5 %.
    constexpr int kGroup = kDeep ? 12 : 8;
    int tile = (int)blockIdx.x - slice * n_tiles;

    // LDS offsets of the operands of slab k
    auto a_slot = [&](int k) { return kDeep ? ((2 * k) % 5) * UNIT_A : (k % kStages) * (UNIT_A + UNIT_B); };
    auto b_slot = [&](int k) { return kDeep ? ((2 * k + 1) % 5) * UNIT_A : (k % kStages) * (UNIT_A + UNIT_B) + UNIT_A; };

    // ---- DMA addressing: instruction j of this wave fills LDS rows r0 = (wave DMA_x + j) 8 ... r0 + 7; lane i lands
    // at row r0 + i / 8, chunk slot i % 8 and fetches logical chunk slot ^ swz(row), swz(row) = (row >> 1) & 7.
    // r0 / 8 and j have the same parity, so two per-lane offsets per operand (even / odd j) serve every j.
    const int dq = lane / CHUNKS, dslot = lane % CHUNKS;
    uint32_t a_lane_off[2], b_lane_off[2];
    const char* a_base[DMA_A];
    const char* b_base[DMA_B];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int sw = (4 * p + (dq >> 1)) & 7;
        a_lane_off[p] = (uint32_t)dq * (uint32_t)(g.lda * 2) + (uint32_t)((dslot ^ sw) * 16) + (uint32_t)k_first * BKB;
        b_lane_off[p] = (uint32_t)dq * (uint32_t)(g.ldw * 2) + (uint32_t)((dslot ^ sw) * 16) + (uint32_t)k_first * BKB;
    }
    // DMA sources of a tile: the row pointers of this wave's instructions
    auto aim_dma = [&](int m0, int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < DMA_A; ++j) a_base[j] = gA + (int64_t)(m0 + (wave * DMA_A + j) * ROWS_PER_DMA) * g.lda * 2;
#pragma unroll
        for (int j = 0; j < DMA_B; ++j) {
            const int r0 = (wave * DMA_B + j) * ROWS_PER_DMA;
            int64_t wrow = r0;
            if (EPI == EPI_SWIGLU) {
                constexpr int H = WN / 2;                             // wave slab = [gate H | up H]
                const int jw = r0 / WN, jj = r0 % WN;
                wrow = (int64_t)(jj / H) * g.N + jw * H + jj % H;
            }
            b_base[j] = gW + (n0 + wrow) * g.ldw * 2;
        }
    };
    TileCoord tc = tile_of_block<kGroup>(tile, g.nt_m, g.nt_n, g.round);
    aim_dma(tc.tm * BM, tc.tn * N_OUT);
    auto issue_a = [&](int k) __attribute__((always_inline)) {
        char* dst = smem + a_slot(k);
#pragma unroll
        for (int j = 0; j < DMA_A; ++j)
            __builtin_amdgcn_global_load_lds(ATTS_GPTR(a_base[j] + a_lane_off[j & 1]),
                                             ATTS_LPTR(dst + (wave * DMA_A + j) * 1024), 16, 0, 0);
        a_lane_off[0] += BKB;
        a_lane_off[1] += BKB;
    };
    auto issue_b = [&](int k) __attribute__((always_inline)) {
        char* dst = smem + b_slot(k);
#pragma unroll
        for (int j = 0; j < DMA_B; ++j)
            __builtin_amdgcn_global_load_lds(ATTS_GPTR(b_base[j] + b_lane_off[j & 1]),
                                             ATTS_LPTR(dst + (wave * DMA_B + j) * 1024), 16, 0, 0);
        b_lane_off[0] += BKB;
        b_lane_off[1] += BKB;
    };

    // ---- fragments: rows wm WM + 32 i + l32 (A) / wn WN + 32 j + l32 (W); 32 i, WM, WN are multiples of 16, so the
    // swizzle term depends on l32 only
    const int frag_xor = (l32 >> 1) & 7;
    const int a_row_off = (wm * WM + l32) * BKB;
    const int b_row_off = (wn * WN + l32) * BKB;
    auto load_a = [&](int k, int s, bf16x8 (&fa)[MI]) __attribute__((always_inline)) {
        const char* pa = smem + a_slot(k) + a_row_off + (((2 * s + half) ^ frag_xor) << 4);
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(pa + i * 32 * BKB);
    };
    auto load_b1 = [&](int k, int s, int j) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8*>(smem + b_slot(k) + b_row_off + j * 32 * BKB + (((2 * s + half) ^ frag_xor) << 4));
    };

    f32x16 acc[MI][NI];

    // One k-step, column by column: the MI MFMAs of column j, then the W fragment of column j is replaced in place
    // by the one of the next k-step (it is free as soon as those MFMAs have issued, and not needed again before the
    // other columns are through).  Only the A fragments are double-buffered.
    bf16x8 fa[2][MI], fb[NI];
    auto kstep = [&](int k, int s, auto cur_, auto reload_) __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_)::value;
        constexpr bool reload = decltype(reload_)::value;   // fragments of k-step s + 1 of the same slab
        if (reload) load_a(k, s + 1, fa[cur ^ 1]);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
#pragma unroll
            for (int i = 0; i < MI; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[j], acc[i][j], 0, 0, 0);
            if (reload) fb[j] = load_b1(k, s + 1, j);
        }
    };
    // scheduling hint for one k-step with n_dma DMA issues: per column, MI MFMAs with one A read, the DMA issues and
    // the W reload placed among them
    auto kstep_hint = [&](auto reload_, auto n_dma_, auto sync_id) __attribute__((always_inline)) {
        constexpr int kId = decltype(sync_id)::value;
        constexpr bool reload = decltype(reload_)::value;
        constexpr int n_dma = decltype(n_dma_)::value;
        constexpr int per_col = (n_dma + NI - 1) / NI, a_per_col = (MI + NI - 1) / NI;
        if (MI < 3) return;   // measured: the 256-row tile does better with the compiler's own order
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, kId);                                           // MFMA
#pragma unroll
            for (int t = 0; t < a_per_col; ++t)
                if (reload && j * a_per_col + t < MI) __builtin_amdgcn_sched_group_barrier(0x100, 1, kId);  // DS read (A)
#pragma unroll
            for (int t = 0; t < per_col; ++t)
                if (j * per_col + t < n_dma) __builtin_amdgcn_sched_group_barrier(0x020, 1, kId);          // VMEM read (LDS DMA)
            __builtin_amdgcn_sched_group_barrier(0x008, MI - 1, kId);                                      // MFMA
            if (reload) __builtin_amdgcn_sched_group_barrier(0x100, 1, kId);                               // DS read (W)
        }
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using CDmaA = std::integral_constant<int, DMA_A>;
    using CDmaB = std::integral_constant<int, DMA_B>;
    using CDmaAB = std::integral_constant<int, DMA_A + DMA_B>;
    // Two whole-slab stages: the stage a slab is fetched into is free for one slab's time only, so all of the next slab is
    // requested under k-step 0 (measured against A rows under k-step 0 and W rows under k-step 1: 2 % faster; all of it
    // ahead of the first MFMA: slower again)
    constexpr bool kEarly = !kDeep && kStages == 2;
    using T_ = std::true_type;
    using F_ = std::false_type;

    // ---- prologue (the accumulators' start values are requested first, so that they are on their way with the first slabs)
    start_accumulators<MI, NI, EPI, true>(acc, tc.tm * BM, tc.tn * N_OUT, wm, wn, l32, half, g_out, g);
    constexpr int kLook = kStages - 1;                 // whole-slab stages: slab k + kLook is issued during slab k
    constexpr int kSteadyWait = kDeep ? DMA_A : (kStages - 2) * (DMA_A + DMA_B);   // loads that may stay in flight
    issue_a(0);
    issue_b(0);
    if (kDeep) {
        issue_a(1);
    } else {
#pragma unroll
        for (int q = 1; q < kLook; ++q) {              // nk >= kStages (checked on the host)
            issue_a(q);
            issue_b(q);
        }
    }
    // slab k.  first / second: the DMA halves issued under k-steps 0 and 1:
    //   deep ring:         W rows of slab k + 1 (into the unit slab k - 1 freed), then A rows of slab k + 2
    //   whole-slab stages: A rows, then W rows of slab k + kLook
    // steady: the loads issued under this slab may stay in flight across its end (else everything is awaited).
    // Two-stage form, last slab of a tile (has_next false, first and second true): the DMA issued under this slab is
    // slab 0 of the next tile, whose sources aim_dma has already been pointed at; it lands in the stage slab k - 1
    // occupied and is awaited at the top of the tile loop.
    auto slab = [&](int k, auto has_next, auto first, auto second, auto steady) __attribute__((always_inline)) {
        // k-step 0
        if (first) { if (kDeep) issue_b(k + 1); else issue_a(k + kLook); }
        if (kEarly && second) issue_b(k + kLook);
        kstep(k, 0, C0{}, T_{});
        if (kEarly && first && second) kstep_hint(T_{}, CDmaAB{}, std::integral_constant<int, 0>{});
        else if (first) { if (kDeep) kstep_hint(T_{}, CDmaB{}, std::integral_constant<int, 0>{}); else kstep_hint(T_{}, CDmaA{}, std::integral_constant<int, 0>{}); }
        else kstep_hint(T_{}, C0{}, std::integral_constant<int, 0>{});
        __builtin_amdgcn_sched_barrier(0);
        // k-step 1
        if (!kEarly && second) { if (kDeep) issue_a(k + 2); else issue_b(k + kLook); }
        kstep(k, 1, C1{}, T_{});
        if (!kEarly && second) { if (kDeep) kstep_hint(T_{}, CDmaA{}, std::integral_constant<int, 1>{}); else kstep_hint(T_{}, CDmaB{}, std::integral_constant<int, 1>{}); }
        else kstep_hint(T_{}, C0{}, std::integral_constant<int, 1>{});
        __builtin_amdgcn_sched_barrier(0);
        // k-step 2
        kstep(k, 2, C0{}, T_{});
        kstep_hint(T_{}, C0{}, std::integral_constant<int, 2>{});
        __builtin_amdgcn_sched_barrier(0);
        // k-step 3, then the slab boundary: slab k + 1 has landed for every wave, every wave is done with slab k
        kstep(k, 3, C1{}, F_{});
        if (has_next) {
            if (steady) wait_vmcnt<kSteadyWait>(); else wait_vmcnt<0>();
            block_barrier();
            load_a(k + 1, 0, fa[0]);
#pragma unroll
            for (int j = 0; j < NI; ++j) fb[j] = load_b1(k + 1, 0, j);
        }
    };
    struct Yes { constexpr operator bool() const { return true; } };
    struct No { constexpr operator bool() const { return false; } };
    void* out = g_out;
    if (EPI == EPI_PARTIAL_F32) out = reinterpret_cast<float*>(g_out) + (int64_t)slice * g.slice_pitch;

    // kb: slabs this workgroup has walked in earlier tiles (the ring positions go on across tiles)
    for (int kb = 0;; kb += nk) {
        const int m0 = tc.tm * BM, n0 = tc.tn * N_OUT, tn = tc.tn;
        // slab 0 of this tile has landed for every wave (and every wave is through with the tile before)
        if (kb == 0) wait_vmcnt<kSteadyWait>(); else wait_vmcnt<0>();
        block_barrier();
        load_a(kb, 0, fa[0]);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[j] = load_b1(kb, 0, j);
        bool more = false;
        int k = 0;
        if (kDeep) {
            for (; k + 2 < nk; ++k) slab(k, Yes{}, Yes{}, Yes{}, Yes{});
            slab(k, Yes{}, Yes{}, No{}, No{});    // k = nk - 2: only the W rows of the last slab are left to issue
            slab(k + 1, No{}, No{}, No{}, No{});
        } else {
            for (; k + kLook < nk; ++k) slab(kb + k, Yes{}, Yes{}, Yes{}, Yes{});
            for (; k + 1 < nk; ++k) slab(kb + k, Yes{}, No{}, No{}, No{});
            if (kTileLoop) {
                // The last slab always carries a slab's worth of DMA, so that there is one code path: slab 0 of the next
                // tile, or (no tile left) slab 0 of this tile once more, into the free stage, awaited before leaving.
                tile += (int)gridDim.x;
                more = g.k_slices == 1 && tile < n_tiles;
                if (more) tc = tile_of_block<kGroup>(tile, g.nt_m, g.nt_n, g.round);
                aim_dma(tc.tm * BM, tc.tn * N_OUT);
#pragma unroll
                for (int p = 0; p < 2; ++p) {          // every slab of the tile has been issued: back to its first slab
                    a_lane_off[p] -= (uint32_t)nk * BKB;
                    b_lane_off[p] -= (uint32_t)nk * BKB;
                }
                slab(kb + k, No{}, Yes{}, Yes{}, No{});
            } else {
                slab(kb + k, No{}, No{}, No{}, No{});
            }
        }

        // the lane coordinates are handed over as values of this iteration, so that the epilogue's address arithmetic is
        // not hoisted out of the tile loop (it would sit in registers all through the main loop)
        int l32_e = l32, half_e = half;
        if (kTileLoop) asm volatile("" : "+v"(l32_e), "+v"(half_e));
        gemm_epilogue_impl<bf16, MI, NI, EPI, true>(acc, m0, n0, wm, wn, l32_e, half_e, tn, out, g_targets, g_partials, g_target_logit,
                                              g_rope, g_vt, g);
        if (!(kTileLoop && more)) break;
        start_accumulators<MI, NI, EPI, true>(acc, tc.tm * BM, tc.tn * N_OUT, wm, wn, l32_e, half_e, g_out, g);
    }
    if (kTileLoop) wait_vmcnt<0>();   // no DMA may still be writing this workgroup's LDS when it is given up
}

#define ATTS_TRY_RC(expr)                 \
    do {                                  \
        int32_t rc__ = (expr);            \
        if (rc__ != ATTS_OK) return rc__; \
    } while (0)

constexpr int kWideBK = 64;           // K elements per slab of the aligned kernel
constexpr int kWavesM = 4;            // wavefronts along M (2 along N)
constexpr int kMinSlabs = 12;         // every K slice must fill the DMA ring

// Shapes the aligned bf16 kernel takes: whole tiles (or padded A rows), K a multiple of the slab.
bool fast_path_ok(int32_t dtype, int epi, const GemmArgs& g) {
    const int n_out = epi == EPI_SWIGLU ? 128 : 256;
    return dtype == ATTS_DTYPE_BF16 && (g.M % 256 == 0 || g.a_rows_padded) && g.N % n_out == 0 && g.Kd % kWideBK == 0 &&
           g.Kd >= kMinSlabs * kWideBK && g.lda * 2 * 17 < (1ll << 31) && g.ldw * 2 * 17 < (1ll << 31);
}

// Tile height of the aligned kernel: 384-row tiles move 1/6 fewer operand bytes per flop through L2 -> LDS than
// 256-row ones and are taken when they do not cost whole extra rounds of workgroups over the 256 CUs.
int fast_tile_rows(int epi, const GemmArgs& g) {
    const int n_out = epi == EPI_SWIGLU ? 128 : 256;
    if (g.M <= 128) return 128;                         // one half-height tile row: half the MFMA work per weight byte
    if (!(g.M % 384 == 0 || g.a_rows_padded) || g.M <= 256) return 256;
    const int64_t nt_n = g.N / n_out;
    const int64_t t256 = ceil_div(g.M, 256) * nt_n, t384 = ceil_div(g.M, 384) * nt_n;
    const int64_t cost256 = ceil_div(t256, 256) * 2, cost384 = ceil_div(t384, 256) * 3;   // rounds x tile height
    return cost384 * 9 <= cost256 * 10 ? 384 : 256;   // a 384-row tile runs ~10 % closer to the MFMA peak
}

// K slices per tile for the partial-sum epilogue: when the tiles alone leave most of the chip idle (few rows and a
// narrow output: the weight-streaming regime), the K range is cut so that about one workgroup per CU runs.
int fast_k_slices(int epi, int n_tiles, int nk) {
    if (epi != EPI_PARTIAL_F32 || n_tiles >= 128) return 1;
    int s = 256 / n_tiles;                                   // never more workgroups than CUs: no second round
    const int max_s = nk / 6;                                // every slice still walks several slabs
    if (s > max_s) s = max_s;
    return s < 1 ? 1 : s;
}

// Compute units of the current device (asked once per device).
int32_t device_cu_count(int* out) {
    static std::atomic<int> cached[64];
    int dev = 0;
    ATTS_HIP_TRY(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && cached[dev].load(std::memory_order_relaxed) > 0) {
        *out = cached[dev].load(std::memory_order_relaxed);
        return ATTS_OK;
    }
    int n = 0;
    ATTS_HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    if (n < 1) return fail(ATTS_ERR_HIP, "device %d reports %d compute units", dev, n);
    if (dev >= 0 && dev < 64) cached[dev].store(n, std::memory_order_relaxed);
    *out = n;
    return ATTS_OK;
}

template <int EPI, int MI, int NI = 4>
int32_t launch_wide_tile(const GemmArgs& g, hipStream_t stream) {
    constexpr int n_out = (EPI == EPI_SWIGLU) ? 32 * NI : 64 * NI;
    constexpr int BM = kWavesM * MI * 32;
    GemmDims d{};
    d.M = g.M; d.N = g.N; d.Kd = g.Kd;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc;
    d.n_part = g.n_part;
    d.ldv = g.ldv;
    d.n_rot_heads = g.n_rot_heads;
    d.nt_m = (int)ceil_div(g.M, BM);
    d.nt_n = g.N / n_out;
    d.k_slices = fast_k_slices(EPI, d.nt_m * d.nt_n, g.Kd / 64);
    d.slice_pitch = (int64_t)g.M * g.ldc;
    const size_t lds = 160 * 1024;
    ATTS_TRY_RC((allow_dynamic_lds<gemm_bf16_wide_kernel<EPI, kWavesM, MI, NI>>(lds)));
    // 384-row tiles without a K split: one workgroup per CU (a workgroup takes a CU's whole LDS), each walking
    // every n_cu-th tile with the next tile's first slab requested under the current tile's last
    int grid = d.nt_m * d.nt_n * d.k_slices;
    d.round = 0;
    if (MI == 3 && d.k_slices == 1) {
        int n_cu = 0;
        ATTS_TRY_RC(device_cu_count(&n_cu));
        n_cu &= ~7;                                   // the tile order deals workgroup ids to the 8 XCDs in turn
        if (n_cu >= 8 && grid > n_cu) grid = n_cu;
        d.round = grid;
    }
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<EPI, kWavesM, MI, NI>), dim3(grid), dim3(128 * kWavesM), lds, stream,
                       reinterpret_cast<const char*>(g.a), reinterpret_cast<const char*>(g.w), g.out, g.targets, g.partials,
                       g.target_logit, g.rope, g.vt, d);
    ATTS_LAUNCH_CHECK("gemm_bf16_wide_kernel");
    return ATTS_OK;
}

template <int EPI>
int32_t launch_fast(const GemmArgs& g, hipStream_t stream) {
    const int rows = fast_tile_rows(EPI, g);
    if (rows == 128) {
        // narrow outputs that split K: 128-column tiles double the tiles, so half as many K slices fill the chip
        if constexpr (EPI == EPI_PARTIAL_F32) return launch_wide_tile<EPI, 1, 2>(g, stream);
        return launch_wide_tile<EPI, 1>(g, stream);
    }
    if (rows == 384) {
        // A last round of tiles that would leave most CUs idle (32B-class O and down projections: 1820 tiles = 7.1 rounds
        // of 256) is avoided by giving the last tile rows to a second launch with 128-row tiles: 89 tile rows in 7 full
        // rounds, then 640 rows as 100 small tiles, each a third of the work.  Taken when the round count of the cost
        // model (rounds x tile height, small tiles priced 40 % dearer per row) drops by 4 % or more.
        constexpr bool kRowsShift = EPI != EPI_QKV_ROPE && EPI != EPI_PARTIAL_F32;   // outputs addressed by row alone
        constexpr int n_out = (EPI == EPI_SWIGLU) ? 128 : 256;
        const int64_t nt_n = g.N / n_out, nt_m = ceil_div(g.M, 384);
        int best_h = 0;
        if (kRowsShift && nt_m > 4) {
            const double single = (double)ceil_div(nt_m * nt_n, 256) * 3;
            double best = single * 0.96;
            for (int drop = 1; drop <= 3; ++drop) {
                const int64_t h = nt_m - drop, rem = g.M - h * 384;
                const double c = (double)ceil_div(h * nt_n, 256) * 3 + (double)ceil_div(ceil_div(rem, 128) * nt_n, 256) * 1.4 + 0.05;
                if (c < best) { best = c; best_h = (int)h; }
            }
        }
        if (best_h > 0) {
            GemmArgs head = g;
            head.M = best_h * 384;
            ATTS_TRY_RC((launch_wide_tile<EPI, 3>(head, stream)));
            GemmArgs tail = g;
            const int64_t r0 = head.M;
            constexpr int64_t out_bytes = (EPI == EPI_STORE_F32 || EPI == EPI_RESID_F32) ? 4 : 2;
            tail.M = g.M - head.M;
            tail.a = static_cast<const char*>(g.a) + r0 * g.lda * 2;
            if (g.out) tail.out = static_cast<char*>(g.out) + r0 * g.ldc * out_bytes;
            if (EPI == EPI_LMHEAD) {
                tail.targets = g.targets + r0;
                tail.partials = g.partials + r0 * g.n_part;
                tail.target_logit = g.target_logit + r0;
            }
            return launch_wide_tile<EPI, 1>(tail, stream);
        }
        return launch_wide_tile<EPI, 3>(g, stream);
    }
    return launch_wide_tile<EPI, 2>(g, stream);
}

template <typename T, int BM, int BN, int EPI>
int32_t launch_cfg(const GemmArgs& g, hipStream_t stream) {
    constexpr int n_out = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
    GemmDims d{};
    d.M = g.M; d.N = g.N; d.Kd = g.Kd;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc;
    d.n_part = g.n_part;
    d.ldv = g.ldv;
    d.n_rot_heads = g.n_rot_heads;
    d.k_slices = 1;
    d.slice_pitch = 0;
    d.nt_m = (int)ceil_div(g.M, BM);
    d.nt_n = (int)ceil_div(g.N, n_out);
    const size_t lds = 2 * (size_t)(BM + BN) * kRowBytes;
    ATTS_TRY_RC((allow_dynamic_lds<gemm_nt_kernel<T, BM, BN, EPI>>(lds)));
    hipLaunchKernelGGL((gemm_nt_kernel<T, BM, BN, EPI>), dim3(d.nt_m * d.nt_n), dim3(kThreads), lds, stream, reinterpret_cast<const char*>(g.a),
                       reinterpret_cast<const char*>(g.w), g.out, g.targets, g.partials, g.target_logit, g.rope, g.vt, d);
    ATTS_LAUNCH_CHECK("gemm_nt_kernel");
    return ATTS_OK;
}

// Tile choice of the general kernel: 256 x 256 when the problem fills the chip with such tiles, else 128 x 128.
bool use_big_tile(int32_t M, int32_t N) {
    return ceil_div(M, 256) * ceil_div(N, 256) >= 192;
}

// The aligned bf16 kernel serves every call it can (its DMA ring also streams weights well when the tiles are
// few); everything else goes to the general kernel.
template <typename T, int EPI>
int32_t launch_epi(const GemmArgs& g, hipStream_t stream) {
    if (sizeof(T) == 2 && fast_path_ok(ATTS_DTYPE_BF16, EPI, g)) return launch_fast<EPI>(g, stream);
    int32_t n_cols = (EPI == EPI_SWIGLU) ? 2 * g.N : g.N;
    if (use_big_tile(g.M, n_cols)) return launch_cfg<T, 256, 256, EPI>(g, stream);
    return launch_cfg<T, 128, 128, EPI>(g, stream);
}

template <typename T>
int32_t launch_t(GemmEpilogue epi, const GemmArgs& g, hipStream_t stream) {
    switch (epi) {
        case EPI_STORE_ACT: return launch_epi<T, EPI_STORE_ACT>(g, stream);
        case EPI_STORE_F32: return launch_epi<T, EPI_STORE_F32>(g, stream);
        case EPI_RESID_F32: return launch_epi<T, EPI_RESID_F32>(g, stream);
        case EPI_SWIGLU: return launch_epi<T, EPI_SWIGLU>(g, stream);
        case EPI_LMHEAD: return launch_epi<T, EPI_LMHEAD>(g, stream);
        case EPI_PARTIAL_F32: return launch_epi<T, EPI_PARTIAL_F32>(g, stream);
        case EPI_QKV_ROPE: break;   // fast path only, dispatched by launch_gemm
        case EPI_LMHEAD_T: break;   // taken by launch_gemm itself, never asked for
    }
    return fail(ATTS_ERR_INVALID_ARG, "unknown GEMM epilogue %d", (int)epi);
}

__global__ void lmhead_combine_kernel(const float2* __restrict__ partials, const float* __restrict__ target_logit,
                                      int B, int n_part, const uint8_t* __restrict__ valid, float* __restrict__ lp) {
    // one wavefront per row
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= B) return;
    if (valid && !valid[row]) {
        if (lane == 0) lp[row] = 0.f;
        return;
    }
    const float2* p = partials + (int64_t)row * n_part;
    float mx = -INFINITY;
    for (int i = lane; i < n_part; i += 64) mx = fmaxf(mx, p[i].x);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
    for (int i = lane; i < n_part; i += 64) {
        float2 q = p[i];
        if (q.y > 0.f) sum += q.y * __expf(q.x - mx);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) lp[row] = target_logit[row] - (mx + __logf(sum));
}

}  // namespace

// The LM head with the operands exchanged: the vocabulary tiles exactly by 384 rows and the scoring rows by 256 columns.
// No row of padding is computed (4096 scoring rows are 10.67 tiles of 384 in the other orientation), the tile count drops
// (7B: 6336 instead of 6534, 25 rounds instead of 26) and the epilogue reduces inside the lanes.
static bool lmhead_exchanged_ok(int32_t dtype, int32_t M, int32_t N, int32_t Kd, int64_t lda, int64_t ldw) {
    return dtype == ATTS_DTYPE_BF16 && N % 384 == 0 && M % 256 == 0 && Kd % kWideBK == 0 && Kd >= kMinSlabs * kWideBK &&
           lda * 2 * 17 < (1ll << 31) && ldw * 2 * 17 < (1ll << 31);
}

int32_t lmhead_num_partials(int32_t dtype, int32_t M, int32_t N, int32_t Kd, bool a_rows_padded) {
    if (lmhead_exchanged_ok(dtype, M, N, Kd, Kd, Kd)) return N / 384 * 4;
    GemmArgs g{};
    g.M = M; g.N = N; g.Kd = Kd; g.lda = Kd; g.ldw = Kd; g.a_rows_padded = a_rows_padded;
    const int bn = (fast_path_ok(dtype, EPI_LMHEAD, g) || use_big_tile(M, N)) ? 256 : 128;
    return (int32_t)ceil_div(N, bn) * 2;
}
int32_t lmhead_max_partials(int32_t N) { return (int32_t)ceil_div(N, 128) * 2; }

bool qkv_rope_fusable(int32_t dtype, int32_t M, int32_t N, int32_t Kd, int32_t head_dim, bool a_rows_padded) {
    GemmArgs g{};
    g.M = M; g.N = N; g.Kd = Kd; g.lda = Kd; g.ldw = Kd; g.a_rows_padded = a_rows_padded;
    return head_dim == 128 && fast_path_ok(dtype, EPI_QKV_ROPE, g);
}

int32_t gemm_partial_slices(int32_t dtype, int32_t M, int32_t N, int32_t Kd, bool a_rows_padded) {
    GemmArgs g{};
    g.M = M; g.N = N; g.Kd = Kd; g.lda = Kd; g.ldw = Kd; g.a_rows_padded = a_rows_padded;
    if (gemm_skinny_ok(dtype, EPI_PARTIAL_F32, g)) return skinny_partial_slices(N, Kd);
    if (!fast_path_ok(dtype, EPI_PARTIAL_F32, g)) return 1;
    const int bm = fast_tile_rows(EPI_PARTIAL_F32, g);
    const int64_t tiles = ceil_div(M, bm) * (N / (bm == 128 ? 128 : 256));
    return fast_k_slices(EPI_PARTIAL_F32, (int)tiles, Kd / 64);
}

int32_t launch_gemm(int32_t dtype, GemmEpilogue epi, const GemmArgs& g, hipStream_t stream) {
    const size_t es = dtype_size(dtype);
    if (g.M <= 0 || g.N <= 0 || g.Kd <= 0) return fail(ATTS_ERR_SHAPE, "gemm: empty shape %d x %d x %d", g.M, g.N, g.Kd);
    if ((g.Kd * es) % 16 || (g.lda * es) % 16 || (g.ldw * es) % 16)
        return fail(ATTS_ERR_SHAPE, "gemm: K (%d) and leading dimensions must be multiples of 16 bytes", g.Kd);
    if (((uintptr_t)g.a | (uintptr_t)g.w) & 15) return fail(ATTS_ERR_INVALID_ARG, "gemm: operands must be 16-byte aligned");
    if (epi == EPI_LMHEAD && g.n_part != lmhead_num_partials(dtype, g.M, g.N, g.Kd, g.a_rows_padded))
        return fail(ATTS_ERR_INVALID_ARG, "gemm: wrong partial count for the LM-head epilogue");
    if (epi == EPI_PARTIAL_F32 && g.n_slices != gemm_partial_slices(dtype, g.M, g.N, g.Kd, g.a_rows_padded))
        return fail(ATTS_ERR_INVALID_ARG, "gemm: wrong slice count for the partial-sum epilogue");
    if (epi == EPI_LMHEAD && lmhead_exchanged_ok(dtype, g.M, g.N, g.Kd, g.lda, g.ldw)) {
        if (!g.targets || !g.partials || !g.target_logit) return fail(ATTS_ERR_INVALID_ARG, "gemm: LM-head epilogue without its buffers");
        GemmArgs x = g;
        x.a = g.w; x.lda = g.ldw; x.M = g.N;
        x.w = g.a; x.ldw = g.lda; x.N = g.M;
        x.a_rows_padded = false;
        return launch_wide_tile<EPI_LMHEAD_T, 3>(x, stream);
    }
    if (epi == EPI_QKV_ROPE) {
        if (!qkv_rope_fusable(dtype, g.M, g.N, g.Kd, 128, g.a_rows_padded) || !g.rope || !g.vt || g.ldv < g.M || g.ldv % 4 ||
            g.n_rot_heads < 1 || g.n_rot_heads * 128 >= g.N)
            return fail(ATTS_ERR_SHAPE, "gemm: the fused QKV epilogue does not apply to this call");
        return launch_fast<EPI_QKV_ROPE>(g, stream);
    }
    // A decoding step (at most 16 rows) streams the weights once.  Narrow outputs (partial-sum epilogue) go to the
    // kernel that cuts K over single wavefronts; wide outputs (SwiGLU, logits) already give the aligned kernel
    // enough tiles, and it streams them as fast, so they only go there when it cannot serve the shape.
    if (gemm_skinny_ok(dtype, epi, g) && (epi == EPI_PARTIAL_F32 || !fast_path_ok(dtype, epi, g)))
        return launch_gemm_skinny(epi, g, stream);
    return dtype == ATTS_DTYPE_F32 ? launch_t<float>(epi, g, stream) : launch_t<bf16>(epi, g, stream);
}

int32_t launch_lmhead_combine(const float2* partials, const float* target_logit, int32_t B, int32_t n_part,
                              const uint8_t* valid, float* lp, hipStream_t stream) {
    const int rows_per_block = 4;
    hipLaunchKernelGGL(lmhead_combine_kernel, dim3((unsigned)ceil_div(B, rows_per_block)), dim3(64 * rows_per_block), 0,
                       stream, partials, target_logit, B, n_part, valid, lp);
    ATTS_LAUNCH_CHECK("lmhead_combine_kernel");
    return ATTS_OK;
}

}  // namespace atts
