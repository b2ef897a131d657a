// Shared-prefix (token-tree) attention.
//
// Rows of the call are laid out [prefix (P) | draft 0 (T) | ... | draft K-1 (T)].  All K drafts
// continue the same prompt, so the prefix keys/values exist once and every draft row attends
// to them ("shared-prefix mechanism", Introduction); a draft row additionally attends causally
// to the rows of its own draft.  With seg(r) = first row of r's draft (0 for a prefix row):
//     key j visible to query r   <=>   j <= r  and  (j < P  or  j >= seg(r)).
// This is exactly K independent causal sequences [prefix ; draft_k], evaluated without
// recomputing or re-storing the prefix.
//
// Two kernels:
//   * attn_mfma_kernel  bf16, head_dim 128: flash-style, 128 query rows of one head per
//     workgroup, key/value tiles of 64 rows staged in LDS and shared by the 4 wavefronts.
//     Works on transposed products so that no register transpose is needed:
//        S^T = K Q^T   (32 keys x 32 queries per MFMA block; a lane owns ONE query column,
//                       so the online-softmax statistics are per lane)
//        O^T = V^T P^T (P^T is fed straight from the S^T accumulator registers; V^T tiles
//                       come from a [n_kv, hd, rows] copy of V written after the QKV GEMM)
//   * attn_simple_kernel any dtype / head_dim: one wavefront per (row, head); used by the
//     fp32 model.
#include "common.h"

namespace atts {
namespace {

__device__ __forceinline__ int seg_start(int r, int P, int T) { return r < P ? 0 : P + (r - P) / T * T; }

// ------------------------------------------------------------------------------------------
// Simple kernel
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void attn_simple_kernel(const T* __restrict__ qkv, T* __restrict__ out, int row0, int P, int Tn,
                                                         int nq, int nkv, int hd, float scale) {
    extern __shared__ float sm[];           // [hd] query, then [n_keys] scores
    float* sq = sm;
    float* sp = sm + hd;
    const int r = row0 + blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
    const int kvh = head / (nq / nkv);
    const int64_t ld = (int64_t)(nq + 2 * nkv) * hd;
    const T* q = qkv + (int64_t)r * ld + head * hd;
    const T* kbase = qkv + (nq + kvh) * hd;
    const T* vbase = qkv + (nq + nkv + kvh) * hd;
    for (int c = lane; c < hd; c += 64) sq[c] = to_f32<T>(q[c]) * scale;
    __syncthreads();

    const int n1 = r < P ? r + 1 : P;                 // visible prefix keys
    const int s0 = seg_start(r, P, Tn);
    const int n2 = r < P ? 0 : r - s0 + 1;            // visible keys of the own draft
    const int n = n1 + n2;
    float mx = -INFINITY;
    for (int i = lane; i < n; i += 64) {
        const T* k = kbase + (int64_t)(i < n1 ? i : s0 + (i - n1)) * ld;
        float s = 0.f;
        for (int c = 0; c < hd; ++c) s += sq[c] * to_f32<T>(k[c]);
        sp[i] = s;
        mx = fmaxf(mx, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
    for (int i = lane; i < n; i += 64) {
        float p = __expf(sp[i] - mx);
        sp[i] = p;
        sum += p;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    __syncthreads();
    const float inv = 1.f / sum;
    for (int c = lane; c < hd; c += 64) {
        float acc = 0.f;
        for (int i = 0; i < n; ++i) acc += sp[i] * to_f32<T>(vbase[(int64_t)(i < n1 ? i : s0 + (i - n1)) * ld + c]);
        out[(int64_t)r * nq * hd + head * hd + c] = from_f32<T>(acc * inv);
    }
}

// ------------------------------------------------------------------------------------------
// MFMA kernel (bf16, hd = 128)
// ------------------------------------------------------------------------------------------
constexpr int kHd = 128;
constexpr int kKTile = 64;    // keys per LDS tile

// kWaves wavefronts of 32 query rows each share the key / value tiles of one head; kStages tiles of LDS form a ring.
// kPipe: the scores of tile t + 1 are issued to the matrix cores BEFORE the softmax of tile t, so that the exponentials
// (vector ALU) of one tile run while the matrix pipe works on the next one; needs the key tile t + 1 next to the value
// tile t in LDS, hence one more stage than the plain order for the same prefetch distance.
template <int kWaves, int kStages, bool kPipe>
__global__ __launch_bounds__(64 * kWaves, 512 / (64 * kWaves)) void attn_mfma_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ vt,
                                                           int64_t ldv, bf16* __restrict__ out, int row0, int R, int P, int Tn,
                                                           int nq, int nkv, float scale_log2e) {
    // Stages of [K tile: 64 keys x 256 B | V^T tile: 128 dims x 128 B], filled by direct global -> LDS loads.
    //   K rows are 256 B: 16-byte chunk index XOR (key & 15);  V^T rows are 128 B: chunk index XOR (dim >> 1) & 7.
    constexpr int kQTile = 32 * kWaves;                 // query rows per workgroup
    constexpr int kKBytes = kKTile * kHd * 2, kStage = 2 * kKBytes;
    constexpr int kDmaK = 16 / kWaves, kDmaV = 16 / kWaves;     // 1 KiB DMA instructions per wave and tile
    constexpr int kDmaTile = kDmaK + kDmaV;
    static_assert(kWaves == 4 || kWaves == 8, "DMA addressing below");
    static_assert(kStages >= (kPipe ? 3 : 2), "ring depth");
    extern __shared__ __attribute__((aligned(16))) char smem[];   // [kStages][kStage]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int head = blockIdx.y, kvh = head / (nq / nkv);
    const int r0 = row0 + blockIdx.x * kQTile;      // query tiles start at the first computed row
    const int r_last = min(r0 + kQTile, R) - 1;
    const int64_t ld = (int64_t)(nq + 2 * nkv) * kHd;

    // This lane's query row and its visibility window; the wave's row range decides which tiles it can skip.
    const int rw0 = r0 + wave * 32;                                  // first row of this wave
    const int rw1 = min(rw0 + 31, r_last);                           // last valid row (rw1 < rw0: the wave has no rows)
    const int r = rw0 + l32;
    const bool r_ok = r < R;
    const int ss = seg_start(r_ok ? r : r_last, P, Tn);
    const int ss_w0 = seg_start(min(rw0, r_last), P, Tn);            // draft start of the wave's first row
    const int ss_w1 = seg_start(max(rw1, rw0 <= r_last ? rw0 : r_last), P, Tn);   // ... and of its last row

    // Q fragments (B operand of S^T = K Q^T): lane holds Q[r][16 s + 8 g + (0..7)], s = 0..7.
    bf16x8 qf[8];
    {
        const bf16* qp = qkv + (int64_t)(r_ok ? r : 0) * ld + head * kHd + 8 * g;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (r_ok) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[s][e] = (bf16)0.f;
        }
    }

    // Tiles: the prefix range [0, min(P, r_last + 1)) and the range of the drafts this query
    // tile touches, both walked in 64-key tiles aligned to multiples of 64.
    const int pre_end = min(P, r_last + 1);
    const int n1 = (pre_end + kKTile - 1) / kKTile;
    const int s2 = max(n1 * kKTile, seg_start(r0, P, Tn) / kKTile * kKTile);
    const int n2 = r_last >= s2 ? (r_last - s2) / kKTile + 1 : 0;
    const int n_tiles = n1 + n2;
    auto tile_start = [&](int t) { return t < n1 ? t * kKTile : s2 + (t - n1) * kKTile; };

    // ---- DMA addressing (one wave-wide instruction moves 1 KiB = 4 K rows or 8 V^T rows).
    // K: instruction j of this wave fills tile rows (64 / kWaves) wave + 4 j + (lane >> 4); lane lands at chunk slot
    //    lane & 15 and fetches chunk slot ^ (row & 15).  Rows past the end are clamped to row R - 1 (their scores
    //    are masked).
    // V^T: instruction j fills dims (128 / kWaves) wave + 8 j + (lane >> 3); slot lane & 7 fetches chunk
    //    slot ^ ((dim >> 1) & 7).  Columns past R are zero in the V^T copy.
    const int kq = lane >> 4, kslot = lane & 15;
    const int vq = lane >> 3, vslot = lane & 7;
    const bf16* kg = qkv + (nq + kvh) * kHd;
    const bf16* vg = vt + ((int64_t)kvh * kHd + (128 / kWaves) * wave + vq) * ldv;
    auto issue_tile = [&](int t) __attribute__((always_inline)) {
        const int j0 = tile_start(t);
        char* stage = smem + (t % kStages) * kStage;
#pragma unroll
        for (int j = 0; j < kDmaK; ++j) {
            const int row = (64 / kWaves) * wave + 4 * j;             // wave-uniform part of the tile row
            const int key = min(j0 + row + kq, R - 1);
            const bf16* src = kg + (int64_t)key * ld + ((kslot ^ ((row + kq) & 15)) << 3);
            __builtin_amdgcn_global_load_lds(ATTS_GPTR(src), ATTS_LPTR(stage + row * 256), 16, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kDmaV; ++j) {
            const int dim = (128 / kWaves) * wave + 8 * j;
            const bf16* src = vg + (int64_t)(8 * j) * ldv + j0 + ((vslot ^ (((dim + vq) >> 1) & 7)) << 3);
            __builtin_amdgcn_global_load_lds(ATTS_GPTR(src), ATTS_LPTR(stage + kKBytes + dim * 128), 16, 0, 0);
        }
    };

    f32x16 acc_o[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[nb][v] = 0.f;
    float m_run = -1e30f;   // reference max (scaled, log2 domain), shared by the lane pair (l, l ^ 32)
    float l_run = 0.f;      // this lane's share of the running denominator

    // Wave-uniform visibility of tile t for the wave's rows rw0 .. rw1:
    //   nothing visible: the tile starts after the last row, or lies in drafts before the wave's first row's
    //   fully visible:   every key <= first row, and (a prefix tile or inside the draft of the last row)
    auto tile_none = [&](int t) {
        const int j0 = tile_start(t);
        return rw1 < rw0 || j0 > rw1 || (j0 >= P && j0 + kKTile <= ss_w0);
    };
    auto tile_full = [&](int t) {
        const int j0 = tile_start(t);
        return j0 + kKTile - 1 <= rw0 && (j0 + kKTile <= P || j0 >= ss_w1) && rw0 + 31 <= r_last;
    };

    // ---- S^T = K Q^T for the two 32-key blocks of tile t.  MFMA row i of a block is fed with key pi(i) of the block,
    // pi = exchange of bits 2 and 3: accumulator entry v of lane half g is then the score of key
    //     32 kb + 16 (v >> 3) + 8 g + (v & 7),
    // eight consecutive keys per lane and 16-key step: exactly the k order of a 16-byte V^T fragment, so the
    // probabilities feed the second product from registers and the value fragments are single 16-byte LDS reads.
    const int kperm = (l32 & 0x13) | ((l32 & 8) >> 1) | ((l32 & 4) << 1);
    auto score_tile = [&](int t, f32x16 (&acc_s)[2]) __attribute__((always_inline)) {
        const char* sK = smem + (t % kStages) * kStage;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_s[kb][v] = 0.f;
        // Fragments in groups of four (two 16-column slices of the head dimension x the two key blocks), double-buffered:
        // the reads of group q + 1 are issued behind the first MFMA of group q, whose wait has just drained the LDS
        // queue, and arrive under the other three.
        auto load_k = [&](int s_, int kb) __attribute__((always_inline)) {
            const int kr = kb * 32 + kperm;
            return *reinterpret_cast<const bf16x8*>(sK + kr * 256 + (((2 * s_ + g) ^ (kr & 15)) << 4));
        };
        bf16x8 kf[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) kf[0][i] = load_k(i >> 1, i & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc_s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[q & 1][0], qf[2 * q], acc_s[0], 0, 0, 0);
            if (q < 3) {
#pragma unroll
                for (int i = 0; i < 4; ++i) kf[(q + 1) & 1][i] = load_k(2 * (q + 1) + (i >> 1), i & 1);
            }
            acc_s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[q & 1][1], qf[2 * q], acc_s[1], 0, 0, 0);
            acc_s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[q & 1][2], qf[2 * q + 1], acc_s[0], 0, 0, 0);
            acc_s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[q & 1][3], qf[2 * q + 1], acc_s[1], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (q < 3) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- softmax of tile t (raw scores in acc_s) and O^T += V^T P^T.  The softmax works on
    // z = score * scale * log2(e): the scale is folded into the one fused multiply-add in front of exp2.
    auto softmax_pv = [&](int t, f32x16 (&acc_s)[2]) __attribute__((always_inline)) {
        const int j0 = tile_start(t);
        const char* sV = smem + (t % kStages) * kStage + kKBytes;
        if (!tile_full(t)) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int j = j0 + 32 * kb + 16 * (v >> 3) + 8 * g + (v & 7);
                    const bool vis = r_ok && j <= r && (j < P || j >= ss);
                    acc_s[kb][v] = vis ? acc_s[kb][v] : -INFINITY;
                }
        }
        float mx = fmaxf(acc_s[0][0], acc_s[1][0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, acc_s[0][v]), acc_s[1][v]);    // one three-operand maximum each
        {   // maximum over the lane pair (l, l ^ 32): the two 32-lane halves exchanged in registers (no LDS round trip
            // in the middle of the softmax): afterwards one result holds the lower half's values in every lane, the other
            // the upper half's
            const unsigned u = __builtin_bit_cast(unsigned, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
            mx = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1])) * scale_log2e;   // scale > 0: the order is kept
        }
        // Lazy rescaling: any reference value works in exp2(z - m) as long as it is the same for numerator and
        // denominator, so the running reference only moves when the new maximum exceeds it by more than 2^6
        // (p stays <= 64, far inside bf16 / fp32 range); the 64 accumulator multiplies are skipped otherwise.
        if (__builtin_amdgcn_ballot_w64(mx > m_run + 6.f) != 0) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc_o[nb][v] *= alpha;
        }
        // value fragments in groups of four (one 16-key slice x the four 32-dim blocks), double-buffered as the key
        // fragments; the first group is requested here, ahead of the exponentials, and has arrived when they are through
        auto load_v = [&](int s_, int nb) __attribute__((always_inline)) {
            const int n = nb * 32 + l32;
            return *reinterpret_cast<const bf16x8*>(sV + n * 128 + (((2 * s_ + g) ^ ((n >> 1) & 7)) << 4));
        };
        bf16x8 vf[2][4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) vf[0][nb] = load_v(0, nb);
        __builtin_amdgcn_sched_barrier(0);
        float psum = 0.f;
        bf16x8 pf[4];
        const float neg_m = -m_run;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(acc_s[kb][v], scale_log2e, neg_m));   // -inf -> 0
                psum += p;
                pf[kb * 2 + (v >> 3)][v & 7] = (bf16)p;
            }
        l_run += psum;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s_ = 0; s_ < 4; ++s_) {
            acc_o[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s_ & 1][0], pf[s_], acc_o[0], 0, 0, 0);
            if (s_ < 3) {
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) vf[(s_ + 1) & 1][nb] = load_v(s_ + 1, nb);
            }
#pragma unroll
            for (int nb = 1; nb < 4; ++nb) acc_o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s_ & 1][nb], pf[s_], acc_o[nb], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (s_ < 3) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // Ring of kStages tiles, tiles 0 .. kStages - 2 requested up front.
#pragma unroll
    for (int t = 0; t < kStages - 1; ++t)
        if (t < n_tiles) issue_tile(t);
    if constexpr (!kPipe) {
        // At the top of step t the tiles up to t + kStages - 2 have been requested, tile t must have landed (the
        // younger ones may stay in flight); after the barrier tile t + kStages - 1 goes into the stage of tile t - 1.
        for (int t = 0; t < n_tiles; ++t) {
            if (t + kStages - 2 < n_tiles) wait_vmcnt<(kStages - 2) * kDmaTile>(); else wait_vmcnt<0>();
            block_barrier();            // tile t is in LDS for every wave; every wave is done with tile t - 1
            if (t + kStages - 1 < n_tiles) issue_tile(t + kStages - 1);
            if (tile_none(t)) continue;
            f32x16 acc_s[2];
            score_tile(t, acc_s);
            softmax_pv(t, acc_s);
        }
    } else {
        // Step t: scores of tile t + 1, then softmax and value product of tile t.  At its top the tiles up to
        // t + kStages - 2 have been requested and tile t + 1 must have landed; after the barrier (every wave is done
        // with tile t - 1) tile t + kStages - 1 goes into that tile's stage.
        f32x16 acc_a[2], acc_b[2];
        if (n_tiles > 0) {
            if (kStages - 2 < n_tiles) wait_vmcnt<(kStages - 2) * kDmaTile>(); else wait_vmcnt<0>();
            block_barrier();
            if (!tile_none(0)) score_tile(0, acc_a);
        }
        auto step = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) __attribute__((always_inline)) {
            if (t + 1 < n_tiles) {
                if (t + kStages - 2 < n_tiles) wait_vmcnt<(kStages - 3) * kDmaTile>(); else wait_vmcnt<0>();
                block_barrier();
                if (t + kStages - 1 < n_tiles) issue_tile(t + kStages - 1);
                if (!tile_none(t + 1)) score_tile(t + 1, nxt);
            }
            if (!tile_none(t)) softmax_pv(t, cur);
        };
        for (int t = 0; t < n_tiles; t += 2) {
            step(t, acc_a, acc_b);
            if (t + 1 < n_tiles) step(t + 1, acc_b, acc_a);
        }
    }

    // ---- normalise and store: acc_o[nb][4 a + b] = O[r][32 nb + 8 a + 4 g + b]
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (r_ok) {
        const float inv = 1.f / l_tot;
        bf16* op = out + (int64_t)r * nq * kHd + head * kHd + 4 * g;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                bf16x4 o4;
#pragma unroll
                for (int b = 0; b < 4; ++b) o4[b] = (bf16)(acc_o[nb][4 * a + b] * inv);
                *reinterpret_cast<bf16x4*>(op + 32 * nb + 8 * a) = o4;
            }
    }
}

}  // namespace

bool attention_uses_vt(int32_t dtype, int32_t hd) { return dtype == ATTS_DTYPE_BF16 && hd == kHd; }

// the general kernel keeps one score per key of the longest context (prefix + one draft) in LDS
constexpr size_t kSimpleLdsMax = 60 * 1024;
static size_t simple_attention_lds(int32_t hd, int32_t P, int32_t T) { return ((size_t)hd + (size_t)P + (size_t)T) * sizeof(float); }

int32_t attention_context_check(const char* fn, int32_t dtype, int32_t hd, int32_t P, int32_t T) {
    if (attention_uses_vt(dtype, hd) || simple_attention_lds(hd, P, T) <= kSimpleLdsMax) return ATTS_OK;
    return fail(ATTS_ERR_SHAPE, "%s: a context of %lld keys (prefix + one draft) is too long for the attention kernel of this dtype / head_dim",
                fn, (long long)P + T);
}

int32_t launch_attention(int32_t dtype, const void* qkv, const void* vt, int64_t ldv, void* out, ScoreShape s, int32_t row0,
                         int32_t nq, int32_t nkv, int32_t hd, hipStream_t stream) {
    const int R = s.R();
    const float scale = 1.f / sqrtf((float)hd);
    if (attention_uses_vt(dtype, hd)) {
        if (!vt || ldv < (int64_t)align_up(R, kKTile) || ldv % 8)
            return fail(ATTS_ERR_WORKSPACE, "attention: transposed-V buffer missing or too narrow");
        // 256 query rows per workgroup (8 wavefronts, one workgroup per CU, four LDS stages, scores of the next tile issued
        // ahead of the softmax) once the call has enough rows to fill the chip that way; 128 rows (4 wavefronts, two
        // workgroups per CU) for smaller calls
        constexpr int kStage = 2 * kKTile * kHd * 2;
        const float sc2 = scale * 1.4426950408889634f;
        if ((int64_t)ceil_div(R - row0, 256) * nq >= 256) {
            constexpr size_t lds = 4 * kStage;
            int32_t rc = allow_dynamic_lds<attn_mfma_kernel<8, 4, true>>(lds);
            if (rc != ATTS_OK) return rc;
            hipLaunchKernelGGL((attn_mfma_kernel<8, 4, true>), dim3((unsigned)ceil_div(R - row0, 256), nq), dim3(512), lds, stream, (const bf16*)qkv,
                               (const bf16*)vt, ldv, (bf16*)out, row0, R, s.P, s.T, nq, nkv, sc2);
        } else {
            constexpr size_t lds = 2 * kStage;
            int32_t rc = allow_dynamic_lds<attn_mfma_kernel<4, 2, false>>(lds);
            if (rc != ATTS_OK) return rc;
            hipLaunchKernelGGL((attn_mfma_kernel<4, 2, false>), dim3((unsigned)ceil_div(R - row0, 128), nq), dim3(256), lds, stream, (const bf16*)qkv,
                               (const bf16*)vt, ldv, (bf16*)out, row0, R, s.P, s.T, nq, nkv, sc2);
        }
        ATTS_LAUNCH_CHECK("attn_mfma_kernel");
        return ATTS_OK;
    }
    const size_t lds = simple_attention_lds(hd, s.P, s.T);
    if (lds > kSimpleLdsMax) return fail(ATTS_ERR_SHAPE, "attention: context of %d keys is too long for this dtype/head_dim", s.P + s.T);
    dim3 grid(R - row0, nq);
    if (dtype == ATTS_DTYPE_F32)
        hipLaunchKernelGGL(attn_simple_kernel<float>, grid, dim3(64), lds, stream, (const float*)qkv, (float*)out, row0, s.P, s.T,
                           nq, nkv, hd, scale);
    else
        hipLaunchKernelGGL(attn_simple_kernel<bf16>, grid, dim3(64), lds, stream, (const bf16*)qkv, (bf16*)out, row0, s.P, s.T,
                           nq, nkv, hd, scale);
    ATTS_LAUNCH_CHECK("attn_simple_kernel");
    return ATTS_OK;
}

}  // namespace atts
