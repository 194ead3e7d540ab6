// decode_partial, vector-ALU form: per-chunk partial softmax statistics
// (m, l, o), a few (query token, head) rows of a GQA group at once.  This kernel
// serves fp32 K/V; bf16 runs on the matrix-core kernel in
// decode_partial_mfma.hip.  Tree Attention (arXiv 2408.04093)
// Algorithm 3 steps 1-2 with the chunks mapped to workgroups of one gfx950 GPU
// instead of devices; inside a chunk it is the running-max form of the
// Section 3 recurrence (n_i = n_{i-1} + v_i s_i, d_i = d_{i-1} + s_i) made safe
// by the max shift of Appendix F.
//
// Data movement (the whole cost: the kernel is HBM-bound)
//   * A K or V row is D fp32 = 256 or 512 bytes.  A lane owns EPL = 8 columns
//     of the head dimension: LPR = D/EPL lanes
//     share a row and fetch it with EPL/4 128-bit buffer loads, load j covering
//     bytes [16 LPR j, 16 LPR (j+1)) of the row, so every load instruction reads
//     RPW = 64/LPR contiguous pieces of 128-512 bytes.  Wider lanes mean fewer
//     lanes per row, and the cross-lane sums of the scores are what this kernel
//     spends its time on besides the fp64 products (EPL = 4 -> 8 at d = 128:
//     9.5 -> 5 vector instructions per key and head for the score; summed as a
//     reduce-scatter over the GT rows, see State: 16 -> 5 fp64 additions per key at GT = 4).
//   * Each lane belongs to one of RPW interleaved "row groups" of keys.
//     Each row group runs its own online softmax; they are merged at the end.
//   * Each wave keeps U K-loads and U V-loads of the NEXT step in flight
//     while it computes the current one (register double buffering), so with
//     8-16 resident waves a CU has tens of KB outstanding.
//   * GT <= 4 (query token, head-in-group) rows that share the KV head are
//     scored against the same registers.  Rows are numbered token-major (token *
//     g + head in group) and cut into slices of GT: with one query token and
//     g <= 4 every K/V byte is fetched once per group; wider groups and several
//     tokens (the causal energy of Appendix C.1 on the last Sq positions) take
//     Sq g / GT passes, each row with its own causal limit, launched so that the
//     slices of a chunk share it through L2.  (Eight rows per workgroup need 256
//     registers for q and the numerators alone and run at one wave per SIMD:
//     193 us for 8 rows against 2 x 72 us for two slices of 4.)
//
// Pass modes (the paper's Algorithm 3 against its Algorithms 1 and 2), as on the matrix-core kernel:
//   kFull (m, l, o) per chunk; kEnergy (m, l) only, K is the only stream; kGradient
//   o = sum_a exp(s_a - lse) v_a with the final lse given (no running max, no normaliser).
//
// Arithmetic
//   q.k and the running max in fp64 (full rate on gfx950) so that large
//   |score| does not cost precision; exponentials and sums in fp32.
//   Scores are kept in log2 units (score * scale * log2 e) so the exponential
//   is the bare v_exp_f32; the partial is converted to natural units on store.
#include "balanced_walk.hpp"
#include "chunking.hpp"
#include "ta_internal.hpp"
#include "wave_ops.hpp"

namespace ta {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// cache-policy bits of the K/V buffer loads.  2 = non-temporal: K/V are read once, and streaming them
// non-temporally measured 7.0 TB/s against 6.2 TB/s for default-policy loads on a read-only probe.
// 0 = default, when several row slices stream the same chunk at the same time (several query tokens,
// wide groups): what one workgroup fetched stays in its XCD's L2 for the others.
constexpr int kAuxStream = 2, kAuxShared = 0;
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

constexpr int kBytes = 4;   // fp32 K/V
using acc_t = double;       // score / running-max type
constexpr int kColumnsPerLane = 8;   // two 128-bit loads per row and lane

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes) {
    // raw buffer (stride 0): hardware returns 0 for any access past `bytes`
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// partial dot product of this lane's columns of a key row with q (q widened once to fp64)
template <int EPL>
__device__ __forceinline__ double lane_dot(const v4i (&k)[EPL / 4], const double (&q)[EPL]) {
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc = fma((double)__int_as_float(k[e >> 2][e & 3]), q[e], acc);
    return acc;
}

enum { kFull = 0, kEnergy = 1, kGradient = 2 };

template <int U, int EPL>
struct Tile {
    v4i k[U][EPL / 4];
    v4i v[U][EPL / 4];
};

// The scores of a key against the GT rows are summed across the lanes of a row as a reduce-scatter
// (scatter_sum in wave_ops.hpp): a lane ends with the score of ONE row, its "own" row, and keeps the
// running max and the normaliser of that row only; the exponential of a score is evaluated once per
// owner instead of by every lane, and the GT weights travel back to all lanes for the numerators.
// Per-row registers of a lane (q, o, weights) are indexed by slot: slot j holds row (j ^ own row).
template <int GT, int EPL>
struct State {
    acc_t m;            // running max of the lane's own row, log2 units
    float l;            // running normaliser of the lane's own row
    float o[GT][EPL];   // running numerators, [slot][this lane's columns]
};

__device__ __forceinline__ acc_t neg_inf() { return -__builtin_huge_val(); }

// One pipeline step: U keys per row group, GT rows.
//   row0: chunk-relative index of this lane's first key (u = 0); key u is
//   row0 + u*RPW.  MASKED steps treat keys >= lim_own as absent for the lane's own row (the end of
//   the chunk, or the row's causal limit inside it).
template <int D, int GT, int U, int EPL, bool MASKED, int MODE>
__device__ __forceinline__ void step(const Tile<U, EPL> &T, const double (&q)[GT][EPL], State<GT, EPL> &st, acc_t c,
                                     int row0, int lim_own) {
    constexpr int LPR = D / EPL, RPW = kWave / LPR;

    acc_t s2[U];   // score of key u against the lane's own row
#pragma unroll
    for (int u = 0; u < U; ++u) {
        acc_t x[GT];
#pragma unroll
        for (int j = 0; j < GT; ++j) x[j] = lane_dot<EPL>(T.k[u], q[j]);
        s2[u] = scatter_sum<LPR, GT>(x) * c;
        if constexpr (MASKED)
            if (row0 + u * RPW >= lim_own) s2[u] = neg_inf();
    }

    // Raise the running max only when some lane of the wave needs it; once the
    // stream is warm this is rare and the rescale of o is skipped.  (Gradient pass: the shift is the
    // given logsumexp and never moves.)
    if constexpr (MODE != kGradient) {
        acc_t mt = s2[0];
#pragma unroll
        for (int u = 1; u < U; ++u) mt = fmax(mt, s2[u]);
        const bool up = mt > st.m;
        if (__builtin_amdgcn_ballot_w64(up) != 0) {
            const float alpha = up ? exp2_hw((float)(st.m - mt)) : 1.0f;
            st.m = up ? mt : st.m;
            st.l *= alpha;
            if constexpr (MODE != kEnergy) {
                float al[GT];
                scatter_gather<LPR, GT>(alpha, al);
#pragma unroll
                for (int j = 0; j < GT; ++j)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) st.o[j][e] *= al[j];
            }
        }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        float p = exp2_hw((float)(s2[u] - st.m));
        if constexpr (MASKED)
            if (row0 + u * RPW >= lim_own) p = 0.f;
        st.l += p;
        if constexpr (MODE != kEnergy) {
            float vf[EPL], ph[GT];
#pragma unroll
            for (int e = 0; e < EPL; ++e) vf[e] = __int_as_float(T.v[u][e >> 2][e & 3]);
            scatter_gather<LPR, GT>(p, ph);
#pragma unroll
            for (int j = 0; j < GT; ++j)
#pragma unroll
                for (int e = 0; e < EPL; ++e) st.o[j][e] = fmaf(ph[j], vf[e], st.o[j][e]);
        }
    }
}

// LDS of a workgroup: the merge of its waves
template <int D, int GT>
struct MergeShared {
    float o[kWaves][GT][D];
    float l[kWaves][GT];
    acc_t m[kWaves][GT];
};

// The whole streaming computation for one range of keys of one (batch, kv head, row slice): called
// once per workgroup by the chunked kernel and once per piece by the balanced kernel.
template <int D, int GT, int MODE, bool BALANCED, int AUX>
__device__ __forceinline__ void process_range(const PartialArgs &a, const Range &cr, MergeShared<D, GT> &lds) {
    constexpr int EPL = kColumnsPerLane, NL = EPL / 4;   // columns and 128-bit loads per lane and row
    // keys per row group per pipeline step.  One with V in the stream (two: 288 registers at GT = 4, one
    // wave per SIMD, slower); two in the energy pass, whose tiles are half the bytes and whose lanes hold no
    // numerators (64k fp32 keys: 45.3 us against 48.5 with one and 49.6 with four)
    constexpr int U = MODE == kEnergy ? 2 : 1;
    constexpr int LPR = D / EPL, RPW = kWave / LPR;
    constexpr int ROWS_WAVE = U * RPW, ROWS_ITER = kWaves * ROWS_WAVE;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane % LPR, rg = lane / LPR;

    const int hk = cr.hk, b = cr.b;
    const int64_t lo = cr.lo;
    const int n = cr.n;

    // This workgroup's rows: (token, head in group) pairs cr.slice * GT + h of the kv head, numbered
    // token-major.  vrow: index of a row in the [B, Sq, Hq] arrays (q, lse) and, times P, in the partials.
    const int HqV = a.Sq * a.Hq;
    auto token_of = [&](int h) { return (cr.slice * GT + h) / a.g; };
    auto vrow = [&](int h) -> int64_t {
        return (int64_t)b * HqV + (int64_t)token_of(h) * a.Hq + hk * a.g + (cr.slice * GT + h) % a.g;
    };
    // index of a row's partial: [B, Sq*Hq, P] in a chunked launch, [piece, piece_rows] in a balanced one
    auto pidx_of = [&](int h) -> int64_t {
        if constexpr (BALANCED) return cr.slot * a.piece_rows + h;
        else return vrow(h) * a.P + cr.slot;
    };
    if (n <= 0) {   // empty chunk: the identity of the merge
        if constexpr (MODE != kEnergy) {
            for (int i = tid; i < GT * D; i += kThreads) a.part_o[pidx_of(i / D) * D + (i % D)] = 0.f;
        }
        if constexpr (MODE != kGradient) {
            if (tid < GT) {
                a.part_m[pidx_of(tid)] = -__builtin_huge_valf();
                a.part_l[pidx_of(tid)] = 0.f;
            }
        }
        return;
    }
    // keys of the chunk each row may see: token t attends keys < L - Sq + 1 + t (chunk-relative,
    // clamped to [0, n]); n for every row when there is one query token
    int lim[GT];
#pragma unroll
    for (int h = 0; h < GT; ++h) {
        const int64_t l = cr.L - a.Sq + 1 + token_of(h) - lo;
        lim[h] = (int)(l < 0 ? 0 : (l > n ? n : l));
    }

    // the row this lane ends up holding the scores of, and its limit
    const int own = scatter_own<LPR, GT>(sub);
    int lim_own = lim[0];
#pragma unroll
    for (int h = 1; h < GT; ++h) lim_own = own == h ? lim[h] : lim_own;

    // q: this lane's EPL columns of each row, kept in registers, slot j = row j ^ own.  Element
    // e = 4 j + r of a lane is column 4 (j LPR + sub) + r: load j of a row, this lane's 16 bytes of it.
    double q[GT][EPL];
#pragma unroll
    for (int h = 0; h < GT; ++h) {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const char *qp = (const char *)a.q + (vrow(h ^ own) * D + 4 * (j * LPR + sub)) * kBytes;
            const v4i raw = *reinterpret_cast<const v4i *>(qp);
#pragma unroll
            for (int r = 0; r < 4; ++r) q[h][4 * j + r] = (double)__int_as_float(raw[r]);
        }
    }

    const char *kb = (const char *)a.K + ((int64_t)b * a.k_sb + (int64_t)hk * a.k_sh) * kBytes +
                     lo * (int64_t)a.k_row_bytes;
    const char *vb = (const char *)a.V + ((int64_t)b * a.v_sb + (int64_t)hk * a.v_sh) * kBytes +
                     lo * (int64_t)a.v_row_bytes;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(kb, (uint32_t)(n - 1) * a.k_row_bytes + D * kBytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(vb, (uint32_t)(n - 1) * a.v_row_bytes + D * kBytes);

    const int n_iters = (n + ROWS_ITER - 1) / ROWS_ITER;
    const int n_full = lim[0] / ROWS_ITER;   // steps whose keys every row sees (rows are token-major: row 0 sees least)
    const int row_lane = w * ROWS_WAVE + rg;   // + it*ROWS_ITER + u*RPW

    uint32_t koff[U], voff[U];   // byte offsets of this lane's loads in iteration 0
#pragma unroll
    for (int u = 0; u < U; ++u) {
        koff[u] = (uint32_t)(row_lane + u * RPW) * a.k_row_bytes + sub * 16;
        voff[u] = (uint32_t)(row_lane + u * RPW) * a.v_row_bytes + sub * 16;
    }

    auto issue = [&](Tile<U, EPL> &T, int it) {
        if (it < n_full) {
            const uint32_t kinc = (uint32_t)it * ROWS_ITER * a.k_row_bytes;
            const uint32_t vinc = (uint32_t)it * ROWS_ITER * a.v_row_bytes;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int j = 0; j < NL; ++j)
                    T.k[u][j] = __builtin_amdgcn_raw_buffer_load_b128(krs, (int)(koff[u] + kinc + j * LPR * 16), 0, AUX);
            if constexpr (MODE != kEnergy) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < NL; ++j)
                        T.v[u][j] = __builtin_amdgcn_raw_buffer_load_b128(vrs, (int)(voff[u] + vinc + j * LPR * 16), 0, AUX);
            }
        } else {
            // ragged last step: rows past the chunk are redirected to its last
            // row (always in range) and masked out of the arithmetic
            uint32_t rc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int r = it * ROWS_ITER + row_lane + u * RPW;
                rc[u] = (uint32_t)(r < n ? r : n - 1);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int j = 0; j < NL; ++j)
                    T.k[u][j] = __builtin_amdgcn_raw_buffer_load_b128(krs, (int)(rc[u] * a.k_row_bytes + (j * LPR + sub) * 16), 0, AUX);
            if constexpr (MODE != kEnergy) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < NL; ++j)
                        T.v[u][j] = __builtin_amdgcn_raw_buffer_load_b128(vrs, (int)(rc[u] * a.v_row_bytes + (j * LPR + sub) * 16), 0, AUX);
            }
        }
    };

    State<GT, EPL> st;
    st.m = neg_inf();
    st.l = 0.f;
    if constexpr (MODE == kGradient) {
        // the shift is the given total logsumexp (natural log -> log2 units); a row with no key at
        // all (lse = -inf) gets +inf so that every exponential below is exactly 0
        const float given = a.lse_in[vrow(own)];
        st.m = given == -__builtin_huge_valf() ? __builtin_huge_val() : (acc_t)given * (acc_t)kLog2e;
    }
#pragma unroll
    for (int h = 0; h < GT; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) st.o[h][e] = 0.f;
    const acc_t c = (acc_t)a.c;

    auto compute = [&](const Tile<U, EPL> &T, int it) {
        const int row0 = it * ROWS_ITER + row_lane;
        if (it < n_full) step<D, GT, U, EPL, false, MODE>(T, q, st, c, row0, lim_own);
        else step<D, GT, U, EPL, true, MODE>(T, q, st, c, row0, lim_own);
    };

    // two register tiles, ping-pong: the loads of step it+1 are in flight
    // while step it is computed
    Tile<U, EPL> ta, tb;
    issue(ta, 0);
    for (int it = 0; it < n_iters; it += 2) {
        if (it + 1 < n_iters) issue(tb, it + 1);
        compute(ta, it);
        if (it + 1 >= n_iters) break;
        if (it + 2 < n_iters) issue(ta, it + 2);
        compute(tb, it + 1);
    }

    // ---- merge the RPW row groups of this wave (lanes LPR apart: they own the same row)
    {
        const acc_t mw = across_groups_max<LPR>(st.m);
        const float f = (st.m == mw) ? 1.0f : exp2_hw((float)(st.m - mw));
        st.m = mw;
        st.l = across_groups_sum<LPR>(st.l * f);
        if constexpr (MODE != kEnergy) {
            float fs[GT];
            scatter_gather<LPR, GT>(f, fs);
#pragma unroll
            for (int h = 0; h < GT; ++h)
#pragma unroll
                for (int e = 0; e < EPL; ++e) st.o[h][e] = across_groups_sum<LPR>(st.o[h][e] * fs[h]);
        }
    }

    // ---- merge the waves of the workgroup through LDS
    auto &lds_o = lds.o;
    auto &lds_l = lds.l;
    auto &lds_m = lds.m;
    if (rg == 0) {
        if constexpr (MODE != kEnergy) {
#pragma unroll
            for (int h = 0; h < GT; ++h)
#pragma unroll
                for (int e = 0; e < EPL; ++e) lds_o[w][h ^ own][4 * ((e >> 2) * LPR + sub) + (e & 3)] = st.o[h][e];
        }
        if (sub == own * (LPR / GT)) {   // the first of the lanes that own this row
            lds_m[w][own] = st.m;
            lds_l[w][own] = st.l;
        }
    }
    __syncthreads();

    const int col = tid % D;
    for (int h = tid / D; h < GT; h += kThreads / D) {
        acc_t ms = lds_m[0][h];
#pragma unroll
        for (int ww = 1; ww < kWaves; ++ww) ms = fmax(ms, lds_m[ww][h]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            const acc_t mw = lds_m[ww][h];
            const float f = (mw == ms) ? 1.0f : exp2_hw((float)(mw - ms));
            lt = fmaf(f, lds_l[ww][h], lt);
            if constexpr (MODE != kEnergy) ot = fmaf(f, lds_o[ww][h][col], ot);
        }
        // Natural-log units for the stored max.  The fp32 value written is not
        // exactly ms*ln2, so l and o are rescaled by the (tiny) residual to stay
        // consistent with the number a reader of part_m will see.
        const float m_nat = (float)(ms * (acc_t)kLn2);
        const acc_t resid = fma(-(acc_t)m_nat, (acc_t)kLog2e, ms);
        // a row that sees no key of the chunk (causal limit) keeps ms = -inf, l = o = 0: the identity
        const float fix = ms == neg_inf() ? 1.0f : exp2_hw((float)resid);
        const int64_t pidx = pidx_of(h);
        if constexpr (MODE == kGradient) {
            a.part_o[pidx * D + col] = ot;   // weights were final all along: the shift is not stored
        } else {
            if constexpr (MODE == kFull) a.part_o[pidx * D + col] = ot * fix;
            if (col == 0) {
                a.part_m[pidx] = m_nat;
                a.part_l[pidx] = lt * fix;
            }
        }
    }
}

// Chunked launch: one workgroup per (batch, kv head, row slice, chunk).
template <int D, int GT, int MODE, bool SHARED = false>
__global__ void __launch_bounds__(kThreads) decode_partial_kernel(const PartialArgs a) {
    __shared__ MergeShared<D, GT> lds;
    __shared__ int sh_rank[kMaxRankedChunks + 1];
    const ChunkRange cr = select_chunk<kThreads>(a, sh_rank);
    if (cr.surplus) return;
    const Range rg{cr.b, cr.hk, cr.slice, cr.lo, cr.n, cr.L, cr.chunk};
    process_range<D, GT, MODE, false, SHARED ? kAuxShared : kAuxStream>(a, rg, lds);
}

// Balanced launch for ragged batches: every workgroup walks its equal-cost share of all keys, piece
// by piece (balanced_walk.hpp).
template <int D, int GT, int MODE>
__global__ void __launch_bounds__(kThreads) decode_balanced_kernel(const PartialArgs a) {
    __shared__ MergeShared<D, GT> lds;
    __shared__ BalancedShared walk;
    balanced_walk<kThreads, kBytes * D>(a, walk, [&](const Range &rg) { process_range<D, GT, MODE, true, kAuxStream>(a, rg, lds); });
}

template <int D, int GT>
hipError_t launch_one(const PartialArgs &a, int mode, hipStream_t s) {
    const dim3 grid((uint32_t)launch_blocks(a));
    if (a.slices > 1) {   // several slices per (batch, kv head) stream the same K/V: share it through L2
        switch (mode) {
            case kEnergy: return launch_kernel(decode_partial_kernel<D, GT, kEnergy, true>, grid, dim3(kThreads), s, a);
            case kGradient: return launch_kernel(decode_partial_kernel<D, GT, kGradient, true>, grid, dim3(kThreads), s, a);
            default: return launch_kernel(decode_partial_kernel<D, GT, kFull, true>, grid, dim3(kThreads), s, a);
        }
    }
    switch (mode) {
        case kEnergy: return launch_kernel(decode_partial_kernel<D, GT, kEnergy>, grid, dim3(kThreads), s, a);
        case kGradient: return launch_kernel(decode_partial_kernel<D, GT, kGradient>, grid, dim3(kThreads), s, a);
        default: return launch_kernel(decode_partial_kernel<D, GT, kFull>, grid, dim3(kThreads), s, a);
    }
}

// resident workgroups per compute unit of one instantiation (register-bound)
template <int D, int GT>
int occupancy_one() {
    static const int cached = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_partial_kernel<D, GT, kFull>, kThreads, 0) !=
                hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = GT >= 4 ? 2 : GT >= 2 ? 3 : 4;   // what the gfx950 build gives
        }
        return n;
    }();
    return cached;
}

template <int D, int GT>
hipError_t launch_balanced_one(const PartialArgs &a, int mode, hipStream_t s) {
    const dim3 grid((uint32_t)a.W);
    switch (mode) {
        case kEnergy: return launch_kernel(decode_balanced_kernel<D, GT, kEnergy>, grid, dim3(kThreads), s, a);
        case kGradient: return launch_kernel(decode_balanced_kernel<D, GT, kGradient>, grid, dim3(kThreads), s, a);
        default: return launch_kernel(decode_balanced_kernel<D, GT, kFull>, grid, dim3(kThreads), s, a);
    }
}

template <int D, int GT>
int balanced_occupancy_one() {
    static const int cached = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_balanced_kernel<D, GT, kFull>, kThreads, 0) !=
                hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 1;
        }
        return n;
    }();
    return cached;
}

#define TA_DISPATCH(FN, ...)                                                                   \
    do {                                                                                       \
        if (d == 128) { switch (gt) { case 4: return FN<128, 4>(__VA_ARGS__);                  \
                                      case 2: return FN<128, 2>(__VA_ARGS__);                  \
                                      default: return FN<128, 1>(__VA_ARGS__); } }             \
        switch (gt) { case 4: return FN<64, 4>(__VA_ARGS__);                                   \
                      case 2: return FN<64, 2>(__VA_ARGS__);                                   \
                      default: return FN<64, 1>(__VA_ARGS__); }                                \
    } while (0)

}  // namespace

hipError_t launch_decode_partial(const PartialArgs &a, int dtype, int d, int mode, hipStream_t s) {
    if (dtype != TA_F32) return hipErrorInvalidValue;   // bf16 belongs to the matrix-core kernel
    const int gt = a.Sq * a.g / a.slices;   // (token, head) rows per workgroup
    TA_DISPATCH(launch_one, a, mode, s);
}

int decode_partial_occupancy(int dtype, int d, int gt) {
    (void)dtype;
    TA_DISPATCH(occupancy_one);
}

hipError_t launch_decode_balanced(const PartialArgs &a, int d, int mode, hipStream_t s) {
    const int gt = a.Sq * a.g / a.slices;
    TA_DISPATCH(launch_balanced_one, a, mode, s);
}

int decode_balanced_occupancy(int d, int gt) { TA_DISPATCH(balanced_occupancy_one); }

}  // namespace ta
