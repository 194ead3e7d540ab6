// decode_partial on the matrix cores: bf16 K/V, d = 128 or 64, up to 64
// (query token, head) pairs per KV head in one pass.  The layout notes below
// are written for d = 128; Geo<D> holds what changes at d = 64 (64-bit row
// loads, 2 k-steps, 4 PV tiles).  Same contract as the VALU kernel in
// decode_partial.hip (Tree Attention, arXiv 2408.04093, Algorithm 3 steps 1-2:
// per-chunk partial (m, l, o); Section 3 recurrence with the Appendix F max
// shift), different arithmetic engine.
//
// Why MFMA here although the kernel is HBM-bound: with all heads of a GQA
// group sharing one K/V stream, the VALU form needs ~74 vector instructions
// per KB streamed at g = 4 (dot2 + cross-lane reductions + per-head exp/FMA)
// and twice that at g = 8 -- it measured ~80 % VALU-busy at g = 4 and
// VALU-bound (3.9 TB/s) at g = 8.  QK^T and PV as 16x16x32 bf16 MFMAs with
// the heads padded to the 16-row tile cost the same for any g <= 16
// and leave ~10 vector instructions per KB.
//
// Per wave and step: a tile of 32 keys (8 KB of K, 8 KB of V).
//   K   global --(8 coalesced 128-bit nt loads: 16 lanes x 16 B = one row)-->
//       VGPR --> LDS, row pitch 272 B --> VGPR in MFMA A layout
//       (lane (kb = l/16, m = l%16) reads key m, bytes 16*(4t+kb) of step t;
//       the 16-byte pad makes these reads bank-conflict-free).  With four row
//       blocks the lanes load exactly those 16 bytes from global memory
//       instead and LDS stays out of the loop (see kDirectK).
//       S[key][head] = sum_t A_t(K) x B_t(Q^T): 2 key groups x 4 k-steps.
//   D layout of S: lane (r = l/16, h = l%16) holds keys 16G + 4r + i of head h,
//       i.e. each lane owns 8 keys of ONE head: exactly the A layout needed
//       for P in  O[head][col] += P[head][key] x V[key][col].
//   V   stays in the registers it was loaded into.  Lane (r, c = l%16) loaded
//       columns 8c..8c+7 of the 8 keys that lanes of row r own, so for each of
//       its 8 columns j the lane already holds the 8 keys of B_j[k][n = c];
//       a 16-bit interleave of register pairs puts them in B layout.  8 MFMAs
//       (one per j) cover all 128 columns: acc_j[i] = O[head 4r+i][col 8c+j].
//   P is split into bf16 hi + bf16 lo (two MFMAs per j) so that the
//       probabilities keep 16 significant bits; rounding P to one bf16 costs
//       1.6e-3 relative error in the output (measured; 2.5e-6 with hi + lo).
// The contraction order of keys inside a tile is a fixed permutation
// (kappa below) applied to P and V alike.
#include <type_traits>

#include "balanced_walk.hpp"
#include "chunking.hpp"
#include "mfma_tile.hpp"
#include "ta_internal.hpp"
#include "wave_ops.hpp"

namespace ta {
namespace {

// Waves per SIMD the register budget is sized for.  With a 256-register budget (2 waves) the
// compiler keeps MFMA results in vector registers; one and two row blocks fit it (165 and 242
// registers; the balanced kernel, which also walks the share table, only with one).
constexpr int waves_per_simd(int nrb, bool balanced) { return balanced ? (nrb == 1 ? 2 : 1) : (nrb <= 2 ? 2 : 1); }
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

// NRB is the number of 16-row blocks of (query token, head) pairs that share the
// K tile in LDS and the V registers: 16 * NRB rows ride on one pass over K/V.

// Per-wave row statistics handed through LDS when the waves of a workgroup are merged.
template <int NRB>
struct WaveStats {
    static constexpr int kRows = 16 * NRB;
    float m[kWaves][kRows];   // shift the wave's l and o are relative to (log2 units)
    float t[kWaves][kRows];   // true row maximum seen by the wave
    float l[kWaves][kRows];   // normaliser
};

// LDS of a workgroup: the waves' K staging areas while the chunk is streamed; afterwards the same
// memory carries the numerators that change owner in the merge (three quarters of them).
template <int D, int NRB>
constexpr int smem_bytes() {
    return kWaves * Geo<D>::kStage > 3 * 16 * NRB * D * 4 ? kWaves * Geo<D>::kStage : 3 * 16 * NRB * D * 4;
}

// The whole streaming computation for one range: called once per workgroup by the chunked kernel
// and once per piece by the balanced kernel.  smem / st are the workgroup's LDS areas.
template <int D, int MODE, int NRB, bool BALANCED, int AUX = kAuxStream>
__device__ __forceinline__ void process_range(const PartialArgs &a, const Range &rg, char *smem,
                                              WaveStats<NRB> &st) {
    using G_ = Geo<D>;
    using row_t = typename G_::row_t;
    constexpr int kCols = G_::kCols, kSteps = G_::kSteps, kPitch = G_::kPitch, kStage = G_::kStage;
    constexpr int kLaneBytes = G_::kLaneBytes;
    // How the K tile reaches MFMA A layout.  Staged (one to two row blocks): coalesced row loads,
    // then through the wave's LDS area.  Direct (four row blocks): every lane loads its A operand's
    // 16 bytes itself, 16 rows x 64 bytes per instruction.  The direct form keeps LDS out of the
    // loop (8 writes, 8 reads and their waits per step: 220 against 236 us per launch at 256 rows, 87
    // against 89-91 us at 64), but each cache line is requested twice; with one row block, where HBM
    // is the bound, it measured 0.6 us slower at 128k keys, so the staged form stays there.
    // (Not in the energy pass: without V in the stream the loads are what the step waits for, and at
    // 64 rows the staged form takes 44.6 against 52.5 us at 128k keys.)
    constexpr bool kDirectK = NRB == 4 && MODE != kEnergy;
    // With four row blocks a lane needs more than 256 registers, and the compiler then gives EVERY
    // MFMA its result in accumulation registers, which the vector ALU cannot address: each score
    // would cost a v_accvgpr_read (8 cycles per instruction, 32 per step).  The numerators belong
    // there, the scores do not: their MFMAs are written as inline assembly with vector-register
    // results (130 against 135 us per launch at 128 rows, 220.5 against 223.5 at 256).
    constexpr bool kScoresInVgprs = NRB == 4;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;     // row group / (column block or row within a row block)
    const int g = a.g;                          // heads of the group, all in this workgroup
    const int hk = rg.hk, b = rg.b;
    const int64_t lo = rg.lo;
    const int n = rg.n;

    // MFMA rows: the (token, head in group) pairs of this kv head, numbered token-major
    // (token * g + head in group); this workgroup owns rows [r0, r0 + nrows), which may start
    // and end inside a token
    const int r0 = rg.slice * a.rows;
    const int nrows = (a.Sq * g - r0) < a.rows ? (a.Sq * g - r0) : a.rows;   // <= 16 * NRB
    const int HqV = a.Sq * a.Hq;                // (token, head) pairs per sequence
    // virtual head of a row: token-major [Sq][Hq]
    auto vhead = [&](int row) { return ((r0 + row) / g) * a.Hq + hk * g + (r0 + row) % g; };
    // index of a row's partial: [B, Sq*Hq, P] in a chunked launch, [piece, piece_rows] in a balanced one
    auto pindex = [&](int row) -> int64_t {
        if constexpr (BALANCED) return rg.slot * a.piece_rows + row;
        else return ((int64_t)b * HqV + vhead(row)) * a.P + rg.slot;
    };

    const bool direct = !BALANCED && a.lse_out != nullptr;   // P == 1: write the final result, not a partial
    if (n <= 0 && direct) {   // no key at all: out = 0, lse = -inf by definition
        if constexpr (MODE == kFull) {
            for (int i = tid; i < nrows * D; i += kThreads) {
                const int64_t o = ((int64_t)b * HqV + vhead(i / D)) * D + (i % D);
                if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[o] = 0;
                else reinterpret_cast<float *>(a.out)[o] = 0.f;
            }
        }
        if (tid < nrows) a.lse_out[(int64_t)b * HqV + vhead(tid)] = -__builtin_huge_valf();
        return;
    }
    if (n <= 0) {   // empty chunk: the identity of the merge
        if constexpr (MODE != kEnergy) {
            for (int i = tid; i < nrows * D; i += kThreads)
                a.part_o[pindex(i / D) * D + (i % D)] = 0.f;
        }
        if constexpr (MODE != kGradient) {
            if (tid < nrows) {
                const int64_t pi = pindex(tid);
                a.part_m[pi] = -__builtin_huge_valf();
                a.part_l[pi] = 0.f;
            }
        }
        return;
    }

    // Per row block: the row this lane serves as "row lane" (row = 16 rb + c), its causal limit
    // (token t sees keys < L - Sq + 1 + t; chunk-relative, clamped to [0, n]) and its slice of
    // Q^T as MFMA B operand: lane (kb = r, row c) holds q[row][32t + 8r .. +8], zero for padding.
    // The q loads are only issued here; their data is first touched (finish_q) after the first K
    // and V tiles have been requested, so that the stream does not start one memory latency late.
    int my_row[NRB], nlim[NRB];
    v4i qraw[NRB][kSteps];
    bf16x8 qb[NRB][kSteps];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = 16 * rb + c;
        my_row[rb] = row < nrows ? row : 0;
        const int64_t lim = rg.L - a.Sq + 1 + (r0 + my_row[rb]) / g - lo;
        nlim[rb] = (int)(lim < 0 ? 0 : (lim > n ? n : lim));
        const char *qp = (const char *)a.q + (((int64_t)b * HqV + vhead(my_row[rb])) * D + 8 * r) * 2;
#pragma unroll
        for (int t = 0; t < kSteps; ++t) qraw[rb][t] = *reinterpret_cast<const v4i *>(qp + 64 * t);
    }
    auto finish_q = [&]() {
        __builtin_amdgcn_sched_barrier(0);   // nothing that waits for q may move above the K/V requests
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                v4i raw = qraw[rb][t];
                if (16 * rb + c >= nrows) raw = v4i{0, 0, 0, 0};
                // a negative scale is moved into q (flipping bf16 sign bits is exact), so that the
                // multiplier below is >= 0 and the row maximum can be taken on unscaled scores
                if (a.c < 0.0) raw ^= v4i{(int)0x80008000u, (int)0x80008000u, (int)0x80008000u, (int)0x80008000u};
                qb[rb][t] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    };
    int n_common;   // keys every row may use: steps below it need no masking
    {
        const int64_t limc = rg.L - a.Sq + 1 + r0 / g - lo;
        n_common = (int)(limc < 0 ? 0 : (limc > n ? n : limc));
    }

    const char *kb = (const char *)a.K + ((int64_t)b * a.k_sb + (int64_t)hk * a.k_sh) * 2 + lo * (int64_t)a.k_row_bytes;
    const char *vb = (const char *)a.V + ((int64_t)b * a.v_sb + (int64_t)hk * a.v_sh) * 2 + lo * (int64_t)a.v_row_bytes;
    const __amdgpu_buffer_rsrc_t krs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(kb), 0, (int)((uint32_t)(n - 1) * a.k_row_bytes + D * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(vb), 0, (int)((uint32_t)(n - 1) * a.v_row_bytes + D * 2), 0x00020000);

    constexpr int ROWS_ITER = kWaves * kTile;
    const int n_iters = (n + ROWS_ITER - 1) / ROWS_ITER;
    const int n_full = n_common / ROWS_ITER;   // steps in which every key is visible to every row

    int trow[8];                // tile row of slot e for this lane
#pragma unroll
    for (int e = 0; e < 8; ++e) trow[e] = kappa(r, e);
    char *stage = smem + w * kStage;

    // Loads of a full tile.  A lane's 8 rows are kappa(r, e) = 4r + (16 (e / 4) + e % 4): the lane part
    // goes into one vector offset, the slot part and the step into the scalar offset of each load, so
    // that a step costs no address arithmetic on the vector ALU.  No branch either: the steady-state
    // loop below has one fixed pattern of outstanding loads and every wait can be exact.
    const uint32_t klane = (uint32_t)(w * kTile + 4 * r) * a.k_row_bytes + c * kLaneBytes;
    const uint32_t vlane = (uint32_t)(w * kTile + 4 * r) * a.v_row_bytes + c * kLaneBytes;
    auto issue_k_full = [&](row_t (&kr)[8], int it) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            kr[e] = G_::template load<AUX>(krs, (int)klane, (int)((uint32_t)(it * ROWS_ITER + 16 * (e >> 2) + (e & 3)) * a.k_row_bytes));
    };
    auto issue_v_full = [&](row_t (&vr)[8], int it) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            vr[e] = G_::template load<AUX>(vrs, (int)vlane, (int)((uint32_t)(it * ROWS_ITER + 16 * (e >> 2) + (e & 3)) * a.v_row_bytes));
    };
    auto issue_k = [&](row_t (&kr)[8], int it) {
        if (it < n_full) {
            issue_k_full(kr, it);
        } else {   // ragged last steps: rows past the chunk are redirected to its last row
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int row = it * ROWS_ITER + w * kTile + trow[e];
                row = row < n ? row : n - 1;
                kr[e] = G_::template load<AUX>(krs, (int)((uint32_t)row * a.k_row_bytes + c * kLaneBytes));
            }
        }
    };
    auto issue_v = [&](row_t (&vr)[8], int it) {
        if (it < n_full) {
            issue_v_full(vr, it);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int row = it * ROWS_ITER + w * kTile + trow[e];
                row = row < n ? row : n - 1;
                vr[e] = G_::template load<AUX>(vrs, (int)((uint32_t)row * a.v_row_bytes + c * kLaneBytes));
            }
        }
    };

    // K straight into MFMA A layout: lane (kb = r, key m = c) of key group G and k-step t holds bytes
    // 16 (4t + r) .. + 16 of key 16 G + c: 16-byte loads, 16 rows x 64 bytes per instruction
    const uint32_t kdlane = (uint32_t)(w * kTile + c) * a.k_row_bytes + r * 16;
    auto issue_kd_full = [&](v4i (&ka)[2][kSteps], int it) {
#pragma unroll
        for (int G = 0; G < 2; ++G)
#pragma unroll
            for (int t = 0; t < kSteps; ++t)
                ka[G][t] = __builtin_amdgcn_raw_buffer_load_b128(krs, (int)kdlane, (int)((uint32_t)(it * ROWS_ITER + 16 * G) * a.k_row_bytes + 64 * t), AUX);
    };
    auto issue_kd = [&](v4i (&ka)[2][kSteps], int it) {
        if (it < n_full) {
            issue_kd_full(ka, it);
        } else {
#pragma unroll
            for (int G = 0; G < 2; ++G) {
                int row = it * ROWS_ITER + w * kTile + 16 * G + c;
                row = row < n ? row : n - 1;
#pragma unroll
                for (int t = 0; t < kSteps; ++t)
                    ka[G][t] = __builtin_amdgcn_raw_buffer_load_b128(krs, (int)((uint32_t)row * a.k_row_bytes + (4 * t + r) * 16), 0, AUX);
            }
        }
    };

    const float cs = fabsf((float)a.c);   // |scale| * log2(e); the sign sits in q
    float m_run[NRB];              // shift of this lane's row (log2 units): a past row maximum, at most kLazy
                                   // below the current one; same in all 4 row groups
    float m_top[NRB];              // largest unscaled score this LANE has seen in its row (the row's true
                                   // maximum is the maximum over its 4 lanes, taken once at the end)
    float thr[NRB];                // (m_run + kLazy) / |c|: the unscaled score beyond which the shift must move
    float l_run[NRB];              // this lane's share of the row's normaliser
    f32x4 acc[NRB][kCols];         // acc[rb][j][i] = O[row 16rb + 4r + i][col kCols c + j]
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        m_run[rb] = m_top[rb] = thr[rb] = -__builtin_huge_valf();
        l_run[rb] = 0.f;
        if constexpr (MODE == kGradient) {
            // the shift is the given total logsumexp (natural log -> log2 units); a row with no key
            // at all (lse = -inf) gets +inf so that every exp below is exactly 0
            const float given = a.lse_in[(int64_t)b * HqV + vhead(my_row[rb])];
            m_run[rb] = given == -__builtin_huge_valf() ? __builtin_huge_valf() : given * (float)kLog2e;
        }
#pragma unroll
        for (int j = 0; j < kCols; ++j) acc[rb][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // One pipeline step on the register tiles (kr, vr) holding step `it`, in two halves around the
    // only data-dependent decision, whether a running max must be raised:
    //   front: K tile into A layout, next K tile in flight, S = K Q^T, (masked) scores, lane maxima
    //   back:  exponentials, P, O += P V, next V tile in flight
    // TAIL is a compile-time flag (std::true_type / std::false_type).  Steady steps (TAIL false) are
    // full tiles followed by another full tile: no masking arithmetic, and the next tile's loads are
    // issued unconditionally.  Tail steps mask rows beyond each row's limit and issue the next tile
    // only if there is one.
    float sv[NRB][8];   // unscaled scores q.k of the current step, slot e = 4G + i (-inf where masked)
    float m8[NRB];      // largest of this lane's 8 unscaled scores of the current step

    // `ahead`: which later step the K registers are refilled with once they have been consumed (1, or 2
    // where two K tiles alternate).
    auto front = [&](auto tail_c, row_t (&kr)[8], v4i (&ka)[2][kSteps], int it, int ahead = 1) -> bool {
        constexpr bool masked = decltype(tail_c)::value;
        if constexpr (!kDirectK) {
            // ---- K tile: registers -> LDS (row-major, padded), next tile requested
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *reinterpret_cast<row_t *>(stage + trow[e] * kPitch + c * kLaneBytes) = kr[e];
            if constexpr (!masked) issue_k_full(kr, it + ahead);
            else if (it + ahead < n_iters) issue_k(kr, it + ahead);
        }

        // S = K Q^T.  The 2 key groups x NRB row blocks are independent accumulation chains; the
        // k-step loop is outermost so that consecutive MFMAs never depend on each other.
        v4i af[2][kSteps];
#pragma unroll
        for (int G = 0; G < 2; ++G)
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                if constexpr (kDirectK) af[G][t] = ka[G][t];
                else af[G][t] = *reinterpret_cast<const v4i *>(stage + (16 * G + c) * kPitch + (4 * t + r) * 16);
            }
        f32x4 s[NRB][2];
        if constexpr (!kScoresInVgprs) {
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) s[rb][0] = s[rb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < kSteps; ++t)
#pragma unroll
                for (int G = 0; G < 2; ++G)
#pragma unroll
                    for (int rb = 0; rb < NRB; ++rb)
                        s[rb][G] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[G][t]), qb[rb][t],
                                                                            s[rb][G], 0, 0, 0);
        } else {
            // Same MFMAs, two row blocks per statement, written out so that S lands in vector
            // registers (see kScoresInVgprs).  Four independent chains per statement, k-step
            // outermost; operands: %0-%3 = S[rb][G] of the two row blocks, then the A operands
            // af[G][t], then the two row blocks' q[t].  The compiler does not see inside: the
            // trailing s_nop covers the wait the vector ALU needs before it may read an MFMA
            // result (8 wait states for this instruction; every earlier result is older).
#pragma unroll
            for (int rb = 0; rb < NRB; rb += 2) {
                if constexpr (kSteps == 4) {
                    asm volatile(
                        "v_mfma_f32_16x16x32_bf16 %0, %4, %12, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %4, %16, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %8, %12, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %8, %16, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %0, %5, %13, %0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %5, %17, %2\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %9, %13, %1\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %9, %17, %3\n"
                        "v_mfma_f32_16x16x32_bf16 %0, %6, %14, %0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %6, %18, %2\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %10, %14, %1\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %10, %18, %3\n"
                        "v_mfma_f32_16x16x32_bf16 %0, %7, %15, %0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %7, %19, %2\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %11, %15, %1\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %11, %19, %3\n"
                        "s_nop 15\n"
                        : "=&v"(s[rb][0]), "=&v"(s[rb][1]), "=&v"(s[rb + 1][0]), "=&v"(s[rb + 1][1])
                        : "v"(af[0][0]), "v"(af[0][1]), "v"(af[0][2]), "v"(af[0][3]),
                          "v"(af[1][0]), "v"(af[1][1]), "v"(af[1][2]), "v"(af[1][3]),
                          "a"(qb[rb][0]), "a"(qb[rb][1]), "a"(qb[rb][2]), "a"(qb[rb][3]),
                          "a"(qb[rb + 1][0]), "a"(qb[rb + 1][1]), "a"(qb[rb + 1][2]), "a"(qb[rb + 1][3]));
                } else {
                    asm volatile(
                        "v_mfma_f32_16x16x32_bf16 %0, %4, %8, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %4, %10, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %6, %8, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %6, %10, 0\n"
                        "v_mfma_f32_16x16x32_bf16 %0, %5, %9, %0\n"
                        "v_mfma_f32_16x16x32_bf16 %2, %5, %11, %2\n"
                        "v_mfma_f32_16x16x32_bf16 %1, %7, %9, %1\n"
                        "v_mfma_f32_16x16x32_bf16 %3, %7, %11, %3\n"
                        "s_nop 15\n"
                        : "=&v"(s[rb][0]), "=&v"(s[rb][1]), "=&v"(s[rb + 1][0]), "=&v"(s[rb + 1][1])
                        : "v"(af[0][0]), "v"(af[0][1]), "v"(af[1][0]), "v"(af[1][1]),
                          "a"(qb[rb][0]), "a"(qb[rb][1]), "a"(qb[rb + 1][0]), "a"(qb[rb + 1][1]));
                }
            }
        }
        if constexpr (kDirectK) {   // the MFMAs above have read the tile: request the next one
            if constexpr (!masked) issue_kd_full(ka, it + ahead);
            else if (it + ahead < n_iters) issue_kd(ka, it + ahead);
        }

        // per row block this lane owns 8 keys of one row.  The steady state needs no row maximum,
        // only the knowledge that no score exceeds the shift by more than kLazy: a per-lane
        // comparison against the row's threshold, and no cross-lane work at all (raise() does that
        // on the rare step where some lane says yes).
        bool any_up = false;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                sv[rb][e] = s[rb][e >> 2][e & 3];
                if constexpr (masked)
                    if (it * ROWS_ITER + w * kTile + trow[e] >= nlim[rb]) sv[rb][e] = -__builtin_huge_valf();
            }
            if constexpr (MODE != kGradient) {
                float top = sv[rb][0];
#pragma unroll
                for (int e = 1; e < 8; ++e) top = fmaxf(top, sv[rb][e]);
                m8[rb] = top;
                m_top[rb] = fmaxf(m_top[rb], top);
                any_up |= top > thr[rb];   // also true on a row's first visible keys (thr = -inf)
            }
        }
        if constexpr (MODE != kGradient) return __builtin_amdgcn_ballot_w64(any_up) != 0;
        return false;
    };

    // move the shifts up to the current step's row maxima: after a row's first keys this only
    // happens when its scores jump by more than kLazy
    auto raise = [&]() {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            // row maximum of the step in log2 units (-inf stays -inf also when the scale is 0)
            const float mx = rows_max(m8[rb] == -__builtin_huge_valf() ? m8[rb] : m8[rb] * cs);
            const bool up = mx > m_run[rb] + kLazy;
            const float alpha = up ? exp2_hw(m_run[rb] - mx) : 1.0f;
            m_run[rb] = up ? mx : m_run[rb];
            thr[rb] = (m_run[rb] + kLazy) / cs;   // +inf when the scale is 0: the shift never moves again
            l_run[rb] *= alpha;
            if constexpr (MODE == kFull) {
                // acc[rb][.][i] belongs to row 4r+i of the block, whose alpha sits in lane (r, 4r+i)
                float ai[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) ai[i] = __shfl(alpha, (lane & 48) | (4 * r + i));
                if constexpr (waves_per_simd(NRB, BALANCED) == 2) {
                    // kernels sized for 256 registers keep everything in vector registers: scale in place
#pragma unroll
                    for (int j = 0; j < kCols; ++j)
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[rb][j][i] *= ai[i];
                } else {
                    // With more row blocks the accumulators live in accumulation registers, which only
                    // MFMAs and memory instructions can address.  They are stored to the wave's K
                    // staging area (free here: S has been computed), scaled there through temporaries,
                    // and loaded back, so that no vector-ALU instruction ever reads or defines an
                    // accumulator inside the loop; otherwise the register allocator keeps a
                    // vector-register copy of all of them and moves them back and forth on every
                    // step.  Each lane reads only what it wrote: no barrier needed.
                    f32x4 *bounce = reinterpret_cast<f32x4 *>(stage) + lane;
#pragma unroll
                    for (int j = 0; j < kCols; ++j) bounce[j * kWave] = acc[rb][j];
                    asm volatile("" ::: "memory");   // keeps loads from being forwarded from the stores
#pragma unroll
                    for (int j = 0; j < kCols; ++j) {
                        f32x4 t = bounce[j * kWave];
#pragma unroll
                        for (int i = 0; i < 4; ++i) t[i] *= ai[i];
                        bounce[j * kWave] = t;
                    }
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int j = 0; j < kCols; ++j) acc[rb][j] = bounce[j * kWave];
                    asm volatile("" ::: "memory");
                }
            }
        }
    };

    // Probabilities of one row block from its scores: p = 2^(s c - shift), the lane's share of the
    // normaliser, and (unless only the energy is wanted) P = hi + lo as MFMA A operand: lane
    // (r, row c), k = 8r + e.
    // (SHIFTED: sv already holds s c - shift, as the pipelined loop leaves it.)
    auto make_p = [&](auto tail_c, auto shifted_c, int rb, bf16x8 &hi, bf16x8 &lo) {
        constexpr bool masked = decltype(tail_c)::value, shifted = decltype(shifted_c)::value;
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = exp2_hw(shifted ? sv[rb][e] : fmaf(sv[rb][e], cs, -m_run[rb]));
            if constexpr (masked && !shifted)
                if (sv[rb][e] == -__builtin_huge_valf()) p[e] = 0.f;   // also when m_run is still -inf
            l_run[rb] += p[e];
        }
        if constexpr (MODE != kEnergy) {
            uint32_t ph[4], pl[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                ph[x] = pack_bf16_rne(p[2 * x], p[2 * x + 1]);
                // opaque to the optimiser, which otherwise converts p[2x] a second time to get the
                // low half on its own
                asm volatile("" : "+v"(ph[x]));
                const float h0 = __uint_as_float(ph[x] << 16), h1 = __uint_as_float(ph[x] & 0xffff0000u);
                pl[x] = pack_bf16_rne(p[2 * x] - h0, p[2 * x + 1] - h1);
            }
            hi = __builtin_bit_cast(bf16x8, v4i{(int)ph[0], (int)ph[1], (int)ph[2], (int)ph[3]});
            lo = __builtin_bit_cast(bf16x8, v4i{(int)pl[0], (int)pl[1], (int)pl[2], (int)pl[3]});
        }
    };
    // column j of the V tile in MFMA B layout: key pairs interleaved by one byte permute per
    // register, the low (j even) or high (j odd) halves of the two keys' registers
    auto v_operand = [&](row_t (&vr)[8], int j) {
        uint32_t bj[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const uint32_t v0 = (uint32_t)vr[2 * x][j >> 1], v1 = (uint32_t)vr[2 * x + 1][j >> 1];
            bj[x] = __builtin_amdgcn_perm(v1, v0, (j & 1) ? 0x07060302u : 0x05040100u);
        }
        return __builtin_bit_cast(bf16x8, v4i{(int)bj[0], (int)bj[1], (int)bj[2], (int)bj[3]});
    };

    auto back = [&](auto tail_c, auto shifted_c, row_t (&vr)[8], int it) {
        constexpr bool masked = decltype(tail_c)::value;
        bf16x8 pa_hi[NRB], pa_lo[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) make_p(tail_c, shifted_c, rb, pa_hi[rb], pa_lo[rb]);
        if constexpr (MODE != kEnergy) {
            // ---- PV: each of this lane's columns goes into B layout once for all row blocks
#pragma unroll
            for (int j = 0; j < kCols; ++j) {
                const bf16x8 vbj = v_operand(vr, j);
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    acc[rb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi[rb], vbj, acc[rb][j], 0, 0, 0);
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    acc[rb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo[rb], vbj, acc[rb][j], 0, 0, 0);
            }
            if constexpr (!masked) issue_v_full(vr, it + 1);
            else if (it + 1 < n_iters) issue_v(vr, it + 1);
        }
    };

    // ---- Four row blocks: the steady step as an explicit software pipeline.
    // At 64 rows per wave the SIMD's issue slots are the bound, a 16x16x32 MFMA keeps the matrix pipe
    // busy for 16 cycles, and independent vector instructions of the same wave can use part of
    // them -- but only if the program order offers some: the compiler's order is "all vector work,
    // then all MFMAs".  The step is therefore written as a sequence of SLOTS, one MFMA plus two to
    // four vector instructions each, pinned by scheduling barriers, and the loop is rotated so that
    // independent work exists: step `it` of the loop runs
    //     slots 0-31    S(it + 1) = K Q^T, all row blocks (into a second set of score registers)
    //                   under the V tile's interleave and the first row block's exponentials / P split
    //     slots 32-79   PV of row block rb under the exponentials / P split of row block rb + 1 and the
    //                   lane maxima of S(it + 1)
    //     slots 80-95   PV of the last row block under the multiply-adds that put S(it + 1) c - shift into
    //                   the score registers (inside this loop they hold the exponent, not the raw score)
    // and returns what maxima(it + 1) would: the caller raises shifts before the next step.  The
    // score MFMAs are single inline-assembly statements here (vector-register results, q from
    // accumulation registers); nothing reads a result sooner than 16 slots after its MFMA, far
    // beyond the 8 wait states the vector ALU needs.
    // (Not in the balanced kernel, which also keeps its walk over the share table in registers and
    // would spill.)
    constexpr bool kPipelined = NRB == 4 && MODE != kEnergy && !BALANCED;
    auto pipelined_step = [&](row_t (&vr)[8], v4i (&ka)[2][kSteps], int it) -> bool {
        constexpr int kQK = 2 * kSteps * NRB;   // score MFMAs of a step
        constexpr int kPV = 2 * kCols;          // PV MFMAs of one row block
        f32x4 sn[NRB][2];                       // S(it + 1)
        uint32_t hi[NRB][4], lo[NRB][4];        // P = hi + lo as MFMA A operands
        float pn[8], h0[4], h1[4];              // the row block whose P is being made
        bool any_up = false;
        // slice k = 0..15 of one row block's exponentials and P split: three vector instructions
        auto p_slice = [&](int rb, int k) {
            if (k < 8) {
                pn[k] = exp2_hw(sv[rb][k]);   // sv is s c - shift inside this loop
                l_run[rb] += pn[k];
            } else {
                const int x = (k - 8) >> 1;
                if (((k - 8) & 1) == 0) {
                    hi[rb][x] = pack_bf16_rne(pn[2 * x], pn[2 * x + 1]);
                    asm volatile("" : "+v"(hi[rb][x]));   // converted once (see make_p)
                    h0[x] = __uint_as_float(hi[rb][x] << 16);
                    h1[x] = __uint_as_float(hi[rb][x] & 0xffff0000u);
                } else {
                    lo[rb][x] = pack_bf16_rne(pn[2 * x] - h0[x], pn[2 * x + 1] - h1[x]);
                }
            }
        };
        // lane maximum of row block rb in S(it + 1), as maxima() takes it
        auto next_max = [&](int rb) {
            if constexpr (MODE != kGradient) {
                float top = sn[rb][0][0];
#pragma unroll
                for (int e = 1; e < 8; ++e) top = fmaxf(top, sn[rb][e >> 2][e & 3]);
                m8[rb] = top;
                m_top[rb] = fmaxf(m_top[rb], top);
                any_up |= top > thr[rb];
            }
        };
        auto operand = [&](const uint32_t (&x)[4]) {
            return __builtin_bit_cast(bf16x8, v4i{(int)x[0], (int)x[1], (int)x[2], (int)x[3]});
        };
        // the vector work of slots 0 .. kQK - 1: kCols interleaves, then the 16 slices of row block 0
        bf16x8 vb[kCols];
        auto first_items = [&](int item) {
            if (item < kCols) vb[item] = v_operand(vr, item);
            else p_slice(0, item - kCols);
        };
        constexpr int kFirstItems = kCols + 16;

        __builtin_amdgcn_sched_barrier(0);
        // ---- slots 0 .. kQK - 1: eight independent chains (row block, key group), k-step outermost
#pragma unroll
        for (int t = 0; t < kSteps; ++t)
#pragma unroll
            for (int G = 0; G < 2; ++G)
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) {
                    const int i = (t * 2 + G) * NRB + rb;
                    if (t == 0)
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=&v"(sn[rb][G]) : "v"(ka[G][t]), "a"(qb[rb][t]));
                    else
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(sn[rb][G]) : "v"(ka[G][t]), "a"(qb[rb][t]));
#pragma unroll
                    for (int item = i * kFirstItems / kQK; item < (i + 1) * kFirstItems / kQK; ++item) first_items(item);
                    __builtin_amdgcn_sched_barrier(0);
                }
        // both tiles have been consumed: request the next ones, K first (the order the loop is entered with)
        issue_kd_full(ka, it + 2);
        __builtin_amdgcn_sched_barrier(0);
        issue_v_full(vr, it + 1);
        __builtin_amdgcn_sched_barrier(0);
        // ---- PV of row block rb
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            const bf16x8 a_hi = operand(hi[rb]), a_lo = operand(lo[rb]);
#pragma unroll
            for (int i = 0; i < kPV; ++i) {
                const int j = i % kCols;
                acc[rb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(i < kCols ? a_hi : a_lo, vb[j], acc[rb][j], 0, 0, 0);
                if (rb + 1 < NRB) {
#pragma unroll
                    for (int k = i * 16 / kPV; k < (i + 1) * 16 / kPV; ++k) p_slice(rb + 1, k);
                    // lane maxima of S(it + 1): two row blocks under PV(1), two under PV(2)
                    if (rb >= 1 && (i == kPV / 4 || i == 3 * kPV / 4)) next_max(2 * (rb - 1) + (i > kPV / 2));
                } else {
                    // S(it + 1) becomes the current scores: row block i / (kPV / NRB), its share of the 8 values
                    constexpr int kPer = kPV / NRB;            // slots per row block: 4 or 2
                    const int mb = i / kPer, part = i % kPer;
#pragma unroll
                    for (int e = part * 8 / kPer; e < (part + 1) * 8 / kPer; ++e)
                        sv[mb][e] = fmaf(sn[mb][e >> 2][e & 3], cs, -m_run[mb]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (MODE != kGradient) return __builtin_amdgcn_ballot_w64(any_up) != 0;
        return false;
    };

    // One register tile of K and one of V per wave, refilled with the next step as soon as it has
    // been consumed.  (More tiles in flight do not help.  One row block: a second V tile requested a
    // whole step ahead measured no faster at 128k keys and 2.6 % slower at 1M, the stream is
    // DRAM-bound.  Four row blocks: two K and two V tiles in flight, 232 against 235 us per launch
    // at 256 rows.)  The steady-state loop is entered with exactly the pattern of outstanding loads
    // it leaves behind on every step (K tile, then V tile), so the compiler's wait counts are exact.
    row_t kr[8], vr[8];
    v4i ka[2][kSteps];
    int it = 0;
    if constexpr (MODE == kEnergy && D == 64) {
        // K is the only stream, a step is short (no PV) and at d = 64 a wave's tile is 4 KB: with one
        // tile in flight the launch is bound by latency (256k keys: 52.9 us against 42.9).  Two K tiles
        // alternate, each refilled with the step after next as soon as it has been consumed.  (At
        // d = 128, with 8 KB per tile, the second tile costs 1 us at 128k keys and 6 us at 1M.)
        row_t kr2[8];
        v4i ka2[2][kSteps];
        auto issue_any = [&](row_t (&r8)[8], v4i (&a8)[2][kSteps], int i) {
            if constexpr (kDirectK) issue_kd(a8, i); else issue_k(r8, i);
        };
        const int n_steady = n_full > 2 ? (n_full - 2) & ~1 : 0;   // pairs of full tiles whose refills are full tiles too
        issue_any(kr, ka, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (n_iters > 1) issue_any(kr2, ka2, 1);
        finish_q();
        for (; it < n_steady; it += 2) {
            if (front(std::false_type{}, kr, ka, it, 2)) raise();
            back(std::false_type{}, std::false_type{}, vr, it);
            if (front(std::false_type{}, kr2, ka2, it + 1, 2)) raise();
            back(std::false_type{}, std::false_type{}, vr, it + 1);
        }
        for (; it < n_iters; it += 2) {   // last full tiles, ragged tail, causal limits
            if (front(std::true_type{}, kr, ka, it, 2)) raise();
            back(std::true_type{}, std::false_type{}, vr, it);
            if (it + 1 < n_iters) {
                if (front(std::true_type{}, kr2, ka2, it + 1, 2)) raise();
                back(std::true_type{}, std::false_type{}, vr, it + 1);
            }
        }
    } else if constexpr (!kPipelined) {
        const int n_steady = n_full > 0 ? n_full - 1 : 0;   // full tiles whose successor is a full tile too
        if (n_steady > 0) {
            if constexpr (kDirectK) issue_kd_full(ka, 0); else issue_k_full(kr, 0);
            // the K loads must be the older ones, as on every later step: without the barrier the
            // scheduler is free to issue V first, and the wait counts of the whole loop follow the entry
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (MODE != kEnergy) issue_v_full(vr, 0);
            finish_q();
            for (; it < n_steady; ++it) {
                if (front(std::false_type{}, kr, ka, it)) raise();
                back(std::false_type{}, std::false_type{}, vr, it);
            }
        } else {
            if constexpr (kDirectK) issue_kd(ka, 0); else issue_k(kr, 0);
            if constexpr (MODE != kEnergy) issue_v(vr, 0);
            finish_q();
        }
        for (; it < n_iters; ++it) {   // last full tile, ragged tail, causal limits
            if (front(std::true_type{}, kr, ka, it)) raise();
            back(std::true_type{}, std::false_type{}, vr, it);
        }
    } else {
        // rotated: the scores and maxima of a step are made during the step before
        const int n_steady = n_full > 2 ? n_full - 2 : 0;   // full tiles whose two successors are full tiles too
        bool pending;                                        // must a shift move before back(it)?
        if (n_steady > 0) {
            issue_kd_full(ka, 0);
            finish_q();
            pending = front(std::false_type{}, kr, ka, 0);   // S(0); leaves the K tile of step 1 in flight
            __builtin_amdgcn_sched_barrier(0);
            issue_v_full(vr, 0);
            // Inside the loop the score registers hold s c - shift instead of s: the step writes them
            // with the multiply-add that the exponentials need anyway, in place of a move.  A shift that
            // moves afterwards (rare) takes the difference out again.
            if (pending) raise();
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
                for (int e = 0; e < 8; ++e) sv[rb][e] = fmaf(sv[rb][e], cs, -m_run[rb]);
            for (; it < n_steady; ++it) {
                pending = pipelined_step(vr, ka, it);
                if (pending) {
                    float m_old[NRB];
#pragma unroll
                    for (int rb = 0; rb < NRB; ++rb) m_old[rb] = m_run[rb];
                    raise();
#pragma unroll
                    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
                        for (int e = 0; e < 8; ++e) sv[rb][e] -= m_run[rb] - m_old[rb];
                }
            }
            // the first step after the loop finds its scores in that form, shifts already raised
            back(std::true_type{}, std::true_type{}, vr, it);
            if (it + 1 < n_iters) pending = front(std::true_type{}, kr, ka, it + 1);
            ++it;
        } else {
            issue_kd(ka, 0);
            issue_v(vr, 0);
            finish_q();
            pending = front(std::true_type{}, kr, ka, 0);
        }
        for (; it < n_iters; ++it) {   // last full tiles, ragged tail, causal limits
            if (pending) raise();
            back(std::true_type{}, std::false_type{}, vr, it);
            if (it + 1 < n_iters) pending = front(std::true_type{}, kr, ka, it + 1);
        }
    }

    // ---- merge the four waves (each holds every row over its own keys) through LDS as a
    // reduce-scatter.  The accumulators are cut into four units (row block rb, group ig of IW of the
    // lane's four rows 4r + i), unit u owned by wave u.  (A) every wave publishes its row statistics;
    // (B) every lane derives the weight of its wave in each of its rows (and the factor that moves
    // the row to the stored maximum), scales its accumulators in registers and writes the three
    // units it does not own to LDS as 128-bit lines; (C) the owner adds the three other waves'
    // lines to its own registers and stores the result: whole rows, a lane's kCols adjacent columns
    // at a time (16 lanes cover a row).  Two barriers, 3/4 of the numerators written and read once,
    // all of it 128-bit wide.
    constexpr int kUnitsPerBlock = kWaves / NRB;           // row groups per row block: 4, 2, 1
    constexpr int IW = 4 / kUnitsPerBlock;                  // rows of a lane per unit: 1, 2, 4
    constexpr int kVec = IW * kCols / 4;                    // IW rows x kCols columns = kVec 128-bit lines per lane and unit
    f32x4 *lds_x = reinterpret_cast<f32x4 *>(smem);         // [owner][slot 0..2][kVec][lane]
    const float ninf = -__builtin_huge_valf();
    __syncthreads();                                        // every wave has left its K staging area
    float lw[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        lw[rb] = rows_sum(l_run[rb]);                       // the normaliser is spread over the 4 row groups
        float m_true = rows_max(m_top[rb]);                 // so is the largest score; to log2 units
        m_true = m_true == ninf ? ninf : m_true * cs;       // (-inf stays -inf also when the scale is 0)
        if (r == 0) {
            st.m[w][16 * rb + c] = m_run[rb];
            st.t[w][16 * rb + c] = m_true;
            st.l[w][16 * rb + c] = lw[rb];
        }
    }
    __syncthreads();

    // (B) scalars of the rows, one thread per row; nothing below waits for them
    if constexpr (MODE != kGradient) {
        if (tid < nrows) {
            const int h = tid;
            float ms = st.m[0][h], mt = st.t[0][h];   // common shift of the merge, true maximum
#pragma unroll
            for (int ww = 1; ww < kWaves; ++ww) {
                ms = fmaxf(ms, st.m[ww][h]);
                mt = fmaxf(mt, st.t[ww][h]);
            }
            const int64_t vrow = (int64_t)b * HqV + vhead(h);
            const int64_t pidx = pindex(h);
            if (ms == ninf) {   // this row saw no key of the chunk (causal limit)
                if (direct) {
                    a.lse_out[vrow] = ms;
                } else {
                    a.part_m[pidx] = ms;
                    a.part_l[pidx] = 0.f;
                }
            } else {
                float lt = 0.f;
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) {
                    const float mw = st.m[ww][h];
                    lt = fmaf((mw == ms) ? 1.0f : exp2_hw(mw - ms), st.l[ww][h], lt);
                }
                if (direct) {   // single chunk: Algorithm 3 step 6 right here
                    a.lse_out[vrow] = fmaf(ms, (float)kLn2, logf(lt));
                } else {
                    // the stored m is the true maximum in natural-log units; l and o, so far relative
                    // to the shift ms, are moved to the value actually stored (this also absorbs its
                    // rounding)
                    const float m_nat = mt * (float)kLn2;
                    a.part_m[pidx] = m_nat;
                    a.part_l[pidx] = lt * exp2_hw(fmaf(-m_nat, (float)kLog2e, ms));
                }
            }
        }
    }

    if constexpr (MODE != kEnergy) {
        // (B) weight of this wave in row 16 rb + c (the row this lane serves as row lane), handed to the
        // lanes that hold the row's numerators (rows 4r + i of lane (r, .)) and applied in registers
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            float scale = 1.0f;   // gradient pass: weights were final all along, the waves' numerators simply add
            if constexpr (MODE != kGradient) {
                const int h = 16 * rb + c;
                float ms = st.m[0][h], mt = st.t[0][h], lt = 0.f;
#pragma unroll
                for (int ww = 1; ww < kWaves; ++ww) {
                    ms = fmaxf(ms, st.m[ww][h]);
                    mt = fmaxf(mt, st.t[ww][h]);
                }
                const float mine = m_run[rb];
                if (ms == ninf) {
                    scale = 0.f;             // the numerators are all 0 (and stay 0)
                } else if (direct) {
#pragma unroll
                    for (int ww = 0; ww < kWaves; ++ww) {
                        const float mw = st.m[ww][h];
                        lt = fmaf((mw == ms) ? 1.0f : exp2_hw(mw - ms), st.l[ww][h], lt);
                    }
                    scale = ((mine == ms) ? 1.0f : exp2_hw(mine - ms)) / lt;   // out = o / l
                } else {
                    const float m_nat = mt * (float)kLn2;
                    scale = ((mine == ms) ? 1.0f : exp2_hw(mine - ms)) * exp2_hw(fmaf(-m_nat, (float)kLog2e, ms));
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float si = MODE == kGradient ? 1.0f : __shfl(scale, (lane & 48) | (4 * r + i));
#pragma unroll
                for (int j = 0; j < kCols; ++j) acc[rb][j][i] *= si;
            }
        }
        // (B) the three units this wave does not own go to their owners
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int ig = 0; ig < kUnitsPerBlock; ++ig) {
                const int owner = rb * kUnitsPerBlock + ig;
                if (owner != w) {
                    const int slot = (w - owner - 1) & 3;   // 0..2
                    f32x4 *dst = lds_x + ((owner * 3 + slot) * kVec) * kWave + lane;
                    // IW rows x kCols columns of the lane, flattened (ii, j) -> lines of four floats
#pragma unroll
                    for (int v = 0; v < kVec; ++v) {
                        f32x4 x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int flat = 4 * v + e, ii = flat / kCols, j = flat % kCols;
                            x[e] = acc[rb][j][ig * IW + ii];
                        }
                        dst[v * kWave] = x;
                    }
                }
            }
        }
    }
    if constexpr (MODE != kEnergy) {
        __syncthreads();
        // (C) the owner sums and stores
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int ig = 0; ig < kUnitsPerBlock; ++ig) {
                const int owner = rb * kUnitsPerBlock + ig;
                if (owner == w) {
                    float o[IW][kCols];
#pragma unroll
                    for (int ii = 0; ii < IW; ++ii)
#pragma unroll
                        for (int j = 0; j < kCols; ++j) o[ii][j] = acc[rb][j][ig * IW + ii];
                    f32x4 x[3][kVec];
#pragma unroll
                    for (int slot = 0; slot < 3; ++slot)
#pragma unroll
                        for (int v = 0; v < kVec; ++v) x[slot][v] = lds_x[((owner * 3 + slot) * kVec + v) * kWave + lane];
#pragma unroll
                    for (int slot = 0; slot < 3; ++slot)
#pragma unroll
                        for (int v = 0; v < kVec; ++v)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int flat = 4 * v + e;
                                o[flat / kCols][flat % kCols] += x[slot][v][e];
                            }
#pragma unroll
                    for (int ii = 0; ii < IW; ++ii) {
                        const int h = 16 * rb + 4 * r + ig * IW + ii;
                        if (h < nrows) {
                            if (direct && MODE == kFull) {
                                const int64_t vrow = (int64_t)b * HqV + vhead(h);
                                if (a.out_dtype == TA_BF16) {
                                    unsigned short *dst = reinterpret_cast<unsigned short *>(a.out) + vrow * D + kCols * c;
#pragma unroll
                                    for (int j = 0; j < kCols; ++j) dst[j] = f32_to_bf16_rne(o[ii][j]);
                                } else {
                                    float *dst = reinterpret_cast<float *>(a.out) + vrow * D + kCols * c;
#pragma unroll
                                    for (int j = 0; j < kCols; ++j) dst[j] = o[ii][j];
                                }
                            } else {
                                float *dst = a.part_o + pindex(h) * D + kCols * c;
#pragma unroll
                                for (int j = 0; j < kCols; ++j) dst[j] = o[ii][j];
                            }
                        }
                    }
                }
            }
        }
    }
}

// Chunked launch: one workgroup per (batch, kv head, token slice, chunk).
// SHARED: the launch has several row slices per (batch, kv head), i.e. several workgroups stream
// the same chunk of K/V at the same time on the same XCD (see select_chunk): default-policy loads
// instead of non-temporal ones, so that what one of them fetched stays in that XCD's L2 for the
// others (64 query tokens at the llama shape: 256 us against 273 us per launch).
template <int D, int MODE, int NRB, bool SHARED = false>
__global__ void __launch_bounds__(kThreads, waves_per_simd(NRB, false)) decode_partial_mfma_kernel(const PartialArgs a) {
    __shared__ __attribute__((aligned(16))) char smem[smem_bytes<D, NRB>()];
    __shared__ WaveStats<NRB> st;
    __shared__ int sh_rank[kMaxRankedChunks + 1];
    const ChunkRange cr = select_chunk<kThreads>(a, sh_rank);
    if (cr.surplus) return;
    const Range rg{cr.b, cr.hk, cr.slice, cr.lo, cr.n, cr.L, cr.chunk};
    process_range<D, MODE, NRB, false, SHARED ? kAuxShared : kAuxStream>(a, rg, smem, st);
}

// Balanced launch for ragged batches: every workgroup walks its equal-cost share of all keys, piece
// by piece (balanced_walk.hpp).
template <int D, int MODE, int NRB>
__global__ void __launch_bounds__(kThreads, waves_per_simd(NRB, true)) decode_balanced_mfma_kernel(const PartialArgs a) {
    __shared__ __attribute__((aligned(16))) char smem[smem_bytes<D, NRB>()];
    __shared__ WaveStats<NRB> st;
    __shared__ BalancedShared walk;
    balanced_walk<kThreads, 2 * D>(a, walk, [&](const Range &rg) { process_range<D, MODE, NRB, true>(a, rg, smem, st); });
}

}  // namespace

template <int D, int NRB, bool SHARED = false>
hipError_t launch_mode(const PartialArgs &a, int mode, dim3 grid, hipStream_t s) {
    switch (mode) {
        case kEnergy: return launch_kernel(decode_partial_mfma_kernel<D, kEnergy, NRB, SHARED>, grid, dim3(kThreads), s, a);
        case kGradient: return launch_kernel(decode_partial_mfma_kernel<D, kGradient, NRB, SHARED>, grid, dim3(kThreads), s, a);
        default: return launch_kernel(decode_partial_mfma_kernel<D, kFull, NRB, SHARED>, grid, dim3(kThreads), s, a);
    }
}

template <int D>
hipError_t launch_rows(const PartialArgs &a, int mode, hipStream_t s) {
    const dim3 grid((uint32_t)launch_blocks(a));
    const int rows = a.rows;
    if (rows <= 16) return launch_mode<D, 1>(a, mode, grid, s);
    if (rows <= 32) return launch_mode<D, 2>(a, mode, grid, s);
    if (a.slices > 1) return launch_mode<D, 4, true>(a, mode, grid, s);   // slices exist only at 64 rows
    return launch_mode<D, 4>(a, mode, grid, s);
}

hipError_t launch_decode_partial_mfma(const PartialArgs &a, int d, int mode, hipStream_t s) {
    if (d == 128) return launch_rows<128>(a, mode, s);
    if (d == 64) return launch_rows<64>(a, mode, s);
    return hipErrorInvalidValue;
}

template <int D, int MODE>
hipError_t launch_balanced(const PartialArgs &a, hipStream_t s) {
    const dim3 grid((uint32_t)a.W);
    const int rows = a.rows;
    if (rows <= 16) return launch_kernel(decode_balanced_mfma_kernel<D, MODE, 1>, grid, dim3(kThreads), s, a);
    if (rows <= 32) return launch_kernel(decode_balanced_mfma_kernel<D, MODE, 2>, grid, dim3(kThreads), s, a);
    return launch_kernel(decode_balanced_mfma_kernel<D, MODE, 4>, grid, dim3(kThreads), s, a);
}

hipError_t launch_decode_balanced_mfma(const PartialArgs &a, int d, int mode, hipStream_t s) {
    if (d != 128 && d != 64) return hipErrorInvalidValue;
    switch (mode) {
        case kFull: return d == 128 ? launch_balanced<128, kFull>(a, s) : launch_balanced<64, kFull>(a, s);
        case kEnergy: return d == 128 ? launch_balanced<128, kEnergy>(a, s) : launch_balanced<64, kEnergy>(a, s);
        case kGradient: return d == 128 ? launch_balanced<128, kGradient>(a, s) : launch_balanced<64, kGradient>(a, s);
    }
    return hipErrorInvalidValue;
}


}  // namespace ta
