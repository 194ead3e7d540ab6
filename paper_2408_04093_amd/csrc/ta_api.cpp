// C ABI of the decode-attention library: argument checks, chunk-count
// heuristic and kernel launches.  All checks run on the host before any
// launch; no pointer argument is dereferenced on the host except ta_problem.
#include <cmath>
#include <cstdint>
#include <mutex>

#include "balanced_walk.hpp"
#include "ta_internal.hpp"

namespace {

using namespace ta;

inline int elem_bytes(int dt) { return dt == TA_BF16 ? 2 : 4; }
inline int tokens(const ta_problem *p) { return p->Sq > 1 ? p->Sq : 1; }
// Matrix-core kernel: the (token, head-in-group) pairs of one kv head are numbered token-major and
// cut into slices of up to 64 rows (4 blocks of 16 MFMA rows); a slice shares one pass over K/V
constexpr int kMaxRows = 64;
inline int64_t total_rows(const ta_problem *p) { return (int64_t)tokens(p) * (p->Hq / p->Hkv); }
inline int rows_per_slice(const ta_problem *p) {
    if (!use_mfma_path(p->qkv_dtype, p->d)) return heads_per_workgroup(p->qkv_dtype, p->d, (int)total_rows(p));
    return (int)(total_rows(p) < kMaxRows ? total_rows(p) : kMaxRows);
}
// independent workgroup groups per chunk index
inline int64_t launch_groups(const ta_problem *p) {
    const int g = p->Hq / p->Hkv;
    if (use_mfma_path(p->qkv_dtype, p->d)) {
        return (int64_t)p->B * p->Hkv * ((total_rows(p) + kMaxRows - 1) / kMaxRows);
    }
    // vector-ALU kernel: the (token, head-in-group) rows of a kv head, a few per workgroup
    (void)g;
    return (int64_t)p->B * p->Hkv * (total_rows(p) / heads_per_workgroup(p->qkv_dtype, p->d, (int)total_rows(p)));
}
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape / stride / dtype checks common to every entry point that takes a problem.
ta_status check_problem(const ta_problem *p) {
    if (!p) return TA_ERR_NULL;
    if (p->qkv_dtype != TA_BF16 && p->qkv_dtype != TA_F32) return TA_ERR_DTYPE;
    if (p->out_dtype != TA_BF16 && p->out_dtype != TA_F32) return TA_ERR_DTYPE;
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->N < 1) return TA_ERR_SHAPE;
    if (p->Hq % p->Hkv != 0) return TA_ERR_SHAPE;
    if (p->d != 64 && p->d != 128) return TA_ERR_UNSUPPORTED;
    if (!std::isfinite(p->scale)) return TA_ERR_SHAPE;
    const int eb = elem_bytes(p->qkv_dtype);
    const int64_t strides[6] = {p->k_stride_b, p->k_stride_h, p->k_stride_n,
                                p->v_stride_b, p->v_stride_h, p->v_stride_n};
    for (int64_t s : strides) {
        if (s < 0) return TA_ERR_SHAPE;
        if ((s * eb) % 16 != 0) return TA_ERR_ALIGN;
    }
    if (p->k_stride_n < p->d || p->v_stride_n < p->d) return TA_ERR_SHAPE;
    // Row offsets inside ONE CHUNK are 32-bit (a chunk's base address is 64-bit), so a row must be
    // shorter than 4 GiB here; that the chunks themselves span less is checked where they are chosen.
    if (p->k_stride_n * eb >= ((int64_t)1 << 31) || p->v_stride_n * eb >= ((int64_t)1 << 31)) return TA_ERR_UNSUPPORTED;
    if (p->N >= ((int64_t)1 << 40)) return TA_ERR_UNSUPPORTED;
    if (p->Sq < 0 || p->Sq > 4096) return TA_ERR_SHAPE;
    if ((int64_t)p->B * p->Hq * tokens(p) >= ((int64_t)1 << 28)) return TA_ERR_SHAPE;
    return TA_OK;
}

// Most keys a chunk (or a piece of the balanced launch) may hold: its rows must lie within 4 GiB
// of its first row, whatever the row stride.
inline int64_t max_chunk_keys(const ta_problem *p) {
    const int64_t eb = elem_bytes(p->qkv_dtype);
    const int64_t row = (p->k_stride_n > p->v_stride_n ? p->k_stride_n : p->v_stride_n) * eb;
    return (((int64_t)1 << 32) - 1 - (int64_t)p->d * eb) / row;
}

int device_compute_units() {
    static std::once_flag once;
    static int cus = 256;   // MI355X
    std::call_once(once, [] {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        (void)hipGetLastError();
    });
    return cus;
}

// Chunk count (host-only heuristic, tuned on MI355X measurements).
//
// Matrix-core kernel (bf16; figures for d = 128): with equal work per workgroup the best
// launch is ONE workgroup per compute unit, each streaming one long contiguous
// share (7.2 TB/s at 1M keys; two per CU or a ragged last round measured
// 4-8 % slower).  So P = CUs / groups, times a whole number of rounds only
// when a chunk would exceed kLongChunk keys.  With more (batch, kv head)
// groups than CUs two workgroups are resident per CU and long chunks win
// (B = 64, N = 8192: P = 1 308 us, P = 4 318 us plus a combine): P is the
// smallest count that fills the last round of workgroups, usually 1.  A
// ragged batch too large for the balanced launch (lengths live on the device
// and are unknown here) is cut into chunks of kRaggedChunk keys (4096
// measured best on the ragged config, in chunk-major launch order) for the
// hardware dispatcher to balance.
//
// VALU kernel (fp32): rounds of CUs x resident workgroups, chunks
// near 4096 keys.
int32_t suggest_chunks(const ta_problem *p, int cus) {
    constexpr int64_t kMinChunk = 256;
    const int g = p->Hq / p->Hkv;
    const int gt = heads_per_workgroup(p->qkv_dtype, p->d, use_mfma_path(p->qkv_dtype, p->d) ? g : (int)total_rows(p));
    const int64_t groups = launch_groups(p);
    int64_t P;
    if (use_mfma_path(p->qkv_dtype, p->d)) {
        // thresholds tuned at d = 128 in keys; what matters is bytes, so d = 64 doubles them
        const int64_t kd = 128 / p->d;
        const int64_t kLongChunk = 32768 * kd, kRaggedChunk = 4096 * kd, kShortestSplit = 2048 * kd;
        const int64_t per_round = cus / groups;
        if (p->valid_len) {
            P = (p->N + kRaggedChunk - 1) / kRaggedChunk;
        } else if (per_round >= 1) {
            int64_t rounds = (p->N + per_round * kLongChunk / 2) / (per_round * kLongChunk);
            if (rounds < 1) rounds = 1;
            P = per_round * rounds;
        } else {
            // more groups than compute units: as few chunks per sequence as fill the last round of
            // workgroups to 90 % (each doubling of P costs 1-2 %, an uneven last round 3-4 %), and
            // with one chunk per sequence the streaming kernel finishes the result itself
            const int64_t p_fit = p->N / kShortestSplit;   // never split below kShortestSplit keys
            const int64_t p_max = p_fit < 1 ? 1 : (p_fit > 8 ? 8 : p_fit);
            double best = 0.0;
            P = 1;
            for (int64_t cand = 1; cand <= p_max; ++cand) {
                const int64_t wgs = groups * cand;
                const double fill = (double)wgs / (double)(((wgs + cus - 1) / cus) * cus);
                if (fill >= 0.9) {
                    P = cand;
                    break;
                }
                if (fill > best) {
                    best = fill;
                    P = cand;
                }
            }
        }
    } else {
        constexpr int64_t kTargetChunk = 4096;
        const int64_t slots = (int64_t)cus * decode_partial_occupancy(p->qkv_dtype, p->d, gt);
        const int64_t per_round = slots / groups;
        if (per_round >= 1) {
            int64_t rounds = (p->N + per_round * kTargetChunk / 2) / (per_round * kTargetChunk);
            if (rounds < 1) rounds = 1;
            P = per_round * rounds;
        } else {
            P = (p->N + kTargetChunk - 1) / kTargetChunk;
        }
    }
    const int64_t p_hi = (p->N + kMinChunk - 1) / kMinChunk;
    if (P > p_hi) P = p_hi;
    if (P < 1) P = 1;
    // a head slice beyond 4 GiB: enough chunks that each stays within the reach of 32-bit row offsets
    const int64_t cap = max_chunk_keys(p);
    while ((p->N + P - 1) / P > cap) ++P;
    if (P > 65536) P = 65536;
    return (int32_t)P;
}

// Ragged batches on the matrix-core kernel run the balanced launch: every workgroup gets an equal
// share of all keys (see decode_balanced_mfma_kernel).
// It pays while there are at most a few (batch, kv head) groups per compute unit: with many short
// sequences one workgroup per sequence (several resident per CU, their start-up latencies
// overlapping) is faster than one workgroup walking through many pieces in turn.  Measured with
// lengths uniform on [N/4, N]: 1024 groups of N = 4096 keys 217 us balanced against 243 us in
// chunks, but 1024 groups of N = 1024 keys 66 us against 61 us; hence no balanced launch for
// more groups than CUs when a sequence cannot exceed 4096 keys (at d = 128).
inline bool use_balanced(const ta_problem *p) {
    if (p->valid_len == nullptr || p->B > kMaxBalancedB) return false;
    if (p->N > max_chunk_keys(p)) return false;   // a piece may be a whole sequence
    const int64_t groups = launch_groups(p), cus = device_compute_units();
    if (groups <= cus) return true;
    return groups <= 4 * cus && p->N * p->d * elem_bytes(p->qkv_dtype) >= (int64_t)4096 * 128 * 2;
}

struct BalancedPlan {
    int32_t W;           // workgroups
    int64_t pieces;      // upper bound on piece ids: W + number of segments
    int32_t rows;        // rows reserved per piece
    size_t off_m, off_l, off_cum, bytes;   // byte offsets in the workspace (part_o at 0)
};

BalancedPlan balanced_plan(const ta_problem *p, int cus) {
    BalancedPlan b{};
    const int64_t groups = launch_groups(p);
    // one workgroup per compute unit (matrix-core kernel), or as many as are resident (vector-ALU kernel)
    b.W = use_mfma_path(p->qkv_dtype, p->d) ? cus : cus * decode_balanced_occupancy(p->d, rows_per_slice(p));
    b.pieces = b.W + groups;
    b.rows = rows_per_slice(p);
    const size_t slots = (size_t)b.pieces * b.rows;
    b.off_m = slots * p->d * sizeof(float);
    b.off_l = b.off_m + slots * sizeof(float);
    b.off_cum = (b.off_l + slots * sizeof(float) + 7) & ~(size_t)7;
    b.bytes = (b.off_cum + ((size_t)p->B + 1) * sizeof(int64_t) + 255) & ~(size_t)255;
    return b;
}

size_t workspace_bytes(const ta_problem *p, int32_t P) {
    const size_t floats = (size_t)p->B * tokens(p) * p->Hq * (size_t)P * (size_t)(p->d + 2);
    size_t bytes = (floats * sizeof(float) + 255) & ~(size_t)255;
    if (use_balanced(p)) {
        const size_t need = balanced_plan(p, device_compute_units()).bytes;
        if (need > bytes) bytes = need;
    }
    return bytes;
}

// The launch descriptor fields that depend only on the problem and the input pointers.
PartialArgs base_args(const ta_problem *p, const void *q, const void *K, const void *V) {
    const int eb = elem_bytes(p->qkv_dtype);
    PartialArgs a{};
    a.q = q; a.K = K; a.V = V ? V : K;
    a.valid_len = p->valid_len;
    a.out_dtype = p->out_dtype;
    a.N = p->N;
    a.k_sb = p->k_stride_b; a.k_sh = p->k_stride_h;
    a.v_sb = p->v_stride_b; a.v_sh = p->v_stride_h;
    a.k_row_bytes = (uint32_t)(p->k_stride_n * eb);
    a.v_row_bytes = (uint32_t)(p->v_stride_n * eb);
    a.B = p->B; a.Hq = p->Hq; a.Hkv = p->Hkv; a.P = 1;
    a.g = p->Hq / p->Hkv;
    a.Sq = tokens(p);
    a.rows = rows_per_slice(p);
    a.slices = (int32_t)(launch_groups(p) / ((int64_t)p->B * p->Hkv));
    // several slices read the same K/V: aligned to the 8 XCDs so that they share an L2 (see select_chunk)
    a.bh_launch = a.slices > 1 ? (p->B * p->Hkv + 7) / 8 * 8 : p->B * p->Hkv;
    a.c = (double)p->scale * kLog2e;
    return a;
}

inline bool out_aligned(const void *out, int out_dtype) {
    return (reinterpret_cast<uintptr_t>(out) & (out_dtype == TA_BF16 ? 1u : 3u)) == 0;
}

// Validate and launch one pass over the chunks.  mode: 0 = (m,l,o); 1 = energy pass (K only; V and
// part_o unused); 2 = gradient pass given lse_in (part_m, part_l unused).
ta_status run_partial(const ta_problem *p, const void *q, const void *K, const void *V, int32_t P,
                      const int64_t *chunk_bounds, float *part_m, float *part_l, float *part_o,
                      const float *lse_in, int mode, void *stream,
                      void *direct_out = nullptr, float *direct_lse = nullptr) {
    const ta_status st = check_problem(p);
    if (st != TA_OK) return st;
    if (!q || !K || (mode != 1 && !V)) return TA_ERR_NULL;
    if (P < 1 || P > (1 << 20)) return TA_ERR_SHAPE;
    // every chunk within 4 GiB of its first row: equal chunks hold ceil(N / P) keys, a table may hold any
    if ((chunk_bounds ? p->N : (p->N + P - 1) / P) > max_chunk_keys(p)) return TA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(K) || (V && !aligned16(V))) return TA_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(part_m) | reinterpret_cast<uintptr_t>(part_l) |
         reinterpret_cast<uintptr_t>(part_o) | reinterpret_cast<uintptr_t>(lse_in)) & 3u)
        return TA_ERR_ALIGN;

    PartialArgs a = base_args(p, q, K, V);
    a.bounds = chunk_bounds;
    a.part_m = part_m; a.part_l = part_l; a.part_o = part_o;
    a.lse_in = lse_in;
    a.out = direct_out; a.lse_out = direct_lse;
    a.P = P;
    a.t = (p->N + P - 1) / P;
    if (launch_blocks(a) >= ((int64_t)1 << 31)) return TA_ERR_SHAPE;
    const hipError_t e = use_mfma_path(p->qkv_dtype, p->d)
                             ? launch_decode_partial_mfma(a, p->d, mode, static_cast<hipStream_t>(stream))
                             : launch_decode_partial(a, p->qkv_dtype, p->d, mode, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? TA_OK : TA_ERR_HIP;
}

// Ragged batch on the balanced launch: equal shares of all keys per workgroup, then the combine over
// each row's pieces.  mode 0 = (m,l,o) -> out and lse; mode 1 = energy pass (K only) -> lse;
// mode 2 = gradient pass given lse -> out (plain sum of the pieces' numerators).
// The caller has checked the problem, the pointers and the workspace size.
ta_status run_balanced(const ta_problem *p, const void *q, const void *K, const void *V, void *workspace,
                       int mode, void *out, float *lse, void *stream) {
    const BalancedPlan bp = balanced_plan(p, device_compute_units());
    char *base = static_cast<char *>(workspace);
    PartialArgs a = base_args(p, q, K, V);
    a.part_o = reinterpret_cast<float *>(base);
    a.part_m = reinterpret_cast<float *>(base + bp.off_m);
    a.part_l = reinterpret_cast<float *>(base + bp.off_l);
    a.cum = reinterpret_cast<int64_t *>(base + bp.off_cum);
    a.lse_in = mode == 2 ? lse : nullptr;
    a.W = bp.W;
    a.piece_rows = bp.rows;
    const hipError_t el = use_mfma_path(p->qkv_dtype, p->d)
                              ? launch_decode_balanced_mfma(a, p->d, mode, static_cast<hipStream_t>(stream))
                              : launch_decode_balanced(a, p->d, mode, static_cast<hipStream_t>(stream));
    if (el != hipSuccess) return TA_ERR_HIP;
    CombineArgs c{};
    c.part_m = a.part_m; c.part_l = a.part_l; c.part_o = a.part_o;
    c.out = out; c.lse = lse;
    c.B = p->B; c.Hq = tokens(p) * p->Hq; c.P = 0;
    c.out_dtype = p->out_dtype;
    c.cum = a.cum;
    const int row_bytes = p->d * elem_bytes(p->qkv_dtype);
    c.W = bp.W; c.min_share = balanced_min_share_keys(row_bytes); c.piece_cost = balanced_piece_cost_keys(row_bytes);
    c.piece_rows = bp.rows;
    c.heads = p->Hq; c.g = a.g; c.Hkv = p->Hkv; c.slices = a.slices; c.rows = a.rows;
    const hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = mode == 1 ? launch_energy_combine(c, s)
                         : mode == 2 ? launch_sum_partials(c, p->d, s) : launch_tree_combine(c, p->d, s);
    return e == hipSuccess ? TA_OK : TA_ERR_HIP;
}

}  // namespace

// ---- ta_decode for callers that cannot allocate: the workspace is a fixed array in device memory that
// the library's code object brings along.  In host code the array's name is only a handle for the
// runtime; the array's device address is looked up once per device (with that device current) and
// that pointer is what is handed to the kernels.
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

static ta_status scratch_of_current_device(void **ptr) {
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TA_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TA_ERR_HIP;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return TA_OK;
}

extern "C" {

const char *ta_status_string(ta_status s) {
    switch (s) {
        case TA_OK: return "ok";
        case TA_ERR_NULL: return "null pointer";
        case TA_ERR_SHAPE: return "bad shape or stride";
        case TA_ERR_DTYPE: return "bad dtype";
        case TA_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
        case TA_ERR_WORKSPACE: return "workspace too small";
        case TA_ERR_UNSUPPORTED: return "unsupported configuration";
        case TA_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

int32_t ta_suggest_chunks(const ta_problem *p) {
    if (check_problem(p) != TA_OK) return 0;
    return suggest_chunks(p, device_compute_units());
}

size_t ta_workspace_bytes(const ta_problem *p, int32_t P) {
    if (check_problem(p) != TA_OK || P < 1) return 0;
    return workspace_bytes(p, P);
}

ta_status ta_decode_partial(const ta_problem *p, const void *q, const void *K, const void *V,
                            int32_t P, const int64_t *chunk_bounds,
                            float *part_m, float *part_l, float *part_o, void *stream) {
    if (!part_m || !part_l || !part_o) return TA_ERR_NULL;
    return run_partial(p, q, K, V, P, chunk_bounds, part_m, part_l, part_o, nullptr, 0, stream);
}

ta_status ta_tree_combine(int32_t B, int32_t Hq, int32_t d, int32_t P,
                          const float *part_m, const float *part_l, const float *part_o,
                          void *out, int32_t out_dtype, float *lse, void *stream) {
    if (!part_m || !part_l || !part_o || !out || !lse) return TA_ERR_NULL;
    if (out_dtype != TA_BF16 && out_dtype != TA_F32) return TA_ERR_DTYPE;
    if (B < 1 || Hq < 1 || P < 1 || (int64_t)B * Hq >= ((int64_t)1 << 28)) return TA_ERR_SHAPE;
    if (d != 64 && d != 128) return TA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(part_o) & 3u) || (reinterpret_cast<uintptr_t>(part_m) & 3u) ||
        (reinterpret_cast<uintptr_t>(part_l) & 3u) || (reinterpret_cast<uintptr_t>(lse) & 3u) ||
        (reinterpret_cast<uintptr_t>(out) & (out_dtype == TA_BF16 ? 1u : 3u)))
        return TA_ERR_ALIGN;
    CombineArgs a{};
    a.part_m = part_m; a.part_l = part_l; a.part_o = part_o;
    a.out = out; a.lse = lse;
    a.B = B; a.Hq = Hq; a.P = P;
    a.out_dtype = out_dtype;
    return launch_tree_combine(a, d, static_cast<hipStream_t>(stream)) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

ta_status ta_decode(const ta_problem *p, const void *q, const void *K, const void *V,
                    void *workspace, size_t workspace_bytes_given,
                    void *out, float *lse, void *stream) {
    const ta_status st = check_problem(p);
    if (st != TA_OK) return st;
    if (!q || !K || !V || !workspace || !out || !lse) return TA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || (reinterpret_cast<uintptr_t>(lse) & 3u)) return TA_ERR_ALIGN;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !out_aligned(out, p->out_dtype)) return TA_ERR_ALIGN;
    const int32_t P = suggest_chunks(p, device_compute_units());
    if (workspace_bytes_given < workspace_bytes(p, P)) return TA_ERR_WORKSPACE;

    if (use_balanced(p)) return run_balanced(p, q, K, V, workspace, 0, out, lse, stream);
    if (P == 1 && use_mfma_path(p->qkv_dtype, p->d)) {
        // one chunk per sequence: the streaming kernel normalises and writes out / lse itself
        return run_partial(p, q, K, V, 1, nullptr, nullptr, nullptr, nullptr, nullptr, 0, stream, out, lse);
    }
    // workspace layout: part_o [B,Hq,P,d] | part_m [B,Hq,P] | part_l [B,Hq,P]
    const size_t bhp = (size_t)p->B * tokens(p) * p->Hq * (size_t)P;
    float *part_o = static_cast<float *>(workspace);
    float *part_m = part_o + bhp * p->d;
    float *part_l = part_m + bhp;
    ta_status s2 = ta_decode_partial(p, q, K, V, P, nullptr, part_m, part_l, part_o, stream);
    if (s2 != TA_OK) return s2;
    return ta_tree_combine(p->B, tokens(p) * p->Hq, p->d, P, part_m, part_l, part_o, out, p->out_dtype, lse,
                           stream);
}

ta_status ta_decode_noalloc(const ta_problem *p, const void *q, const void *K, const void *V,
                            void *out, float *lse, void *stream) {
    const ta_status st = check_problem(p);
    if (st != TA_OK) return st;
    if (!q || !K || !V || !out || !lse) return TA_ERR_NULL;
    // the size check comes before the array is touched: too large a problem is refused on any machine
    if (workspace_bytes(p, suggest_chunks(p, device_compute_units())) > kScratchBytes) return TA_ERR_WORKSPACE;
    void *ws = nullptr;
    const ta_status s1 = scratch_of_current_device(&ws);
    if (s1 != TA_OK) return s1;
    return ta_decode(p, q, K, V, ws, kScratchBytes, out, lse, stream);
}

ta_status ta_energy(const ta_problem *p, const void *q, const void *K,
                    void *workspace, size_t workspace_bytes_given, float *lse, void *stream) {
    const ta_status st = check_problem(p);
    if (st != TA_OK) return st;
    if (!q || !K || !workspace || !lse) return TA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || (reinterpret_cast<uintptr_t>(lse) & 3u)) return TA_ERR_ALIGN;
    if (!aligned16(q) || !aligned16(K)) return TA_ERR_ALIGN;
    const int32_t P = suggest_chunks(p, device_compute_units());
    if (workspace_bytes_given < workspace_bytes(p, P)) return TA_ERR_WORKSPACE;
    if (use_balanced(p)) return run_balanced(p, q, K, nullptr, workspace, 1, nullptr, lse, stream);
    if (P == 1 && use_mfma_path(p->qkv_dtype, p->d))   // the matrix-core kernel finishes a single chunk itself
        return run_partial(p, q, K, nullptr, 1, nullptr, nullptr, nullptr, nullptr, nullptr, 1, stream, nullptr, lse);
    const size_t bhp = (size_t)p->B * tokens(p) * p->Hq * (size_t)P;
    float *part_m = static_cast<float *>(workspace) + bhp * p->d;      // same slots as in ta_decode
    float *part_l = part_m + bhp;
    const ta_status s2 = run_partial(p, q, K, nullptr, P, nullptr, part_m, part_l, nullptr, nullptr, 1, stream);
    if (s2 != TA_OK) return s2;
    CombineArgs c{};
    c.part_m = part_m; c.part_l = part_l;
    c.lse = lse;
    c.B = p->B; c.Hq = tokens(p) * p->Hq; c.P = P;
    return launch_energy_combine(c, static_cast<hipStream_t>(stream)) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

ta_status ta_decode_two_pass(const ta_problem *p, const void *q, const void *K, const void *V,
                             void *workspace, size_t workspace_bytes_given,
                             void *out, float *lse, void *stream) {
    const ta_status st = check_problem(p);
    if (st != TA_OK) return st;
    if (!q || !K || !V || !workspace || !out || !lse) return TA_ERR_NULL;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !out_aligned(out, p->out_dtype)) return TA_ERR_ALIGN;
    const ta_status s1 = ta_energy(p, q, K, workspace, workspace_bytes_given, lse, stream);
    if (s1 != TA_OK) return s1;
    // a ragged batch takes equal-cost shares in both passes
    if (use_balanced(p)) return run_balanced(p, q, K, V, workspace, 2, out, lse, stream);
    const int32_t P = suggest_chunks(p, device_compute_units());
    float *part_o = static_cast<float *>(workspace);
    const ta_status s2 = run_partial(p, q, K, V, P, nullptr, nullptr, nullptr, part_o, lse, 2, stream);
    if (s2 != TA_OK) return s2;
    CombineArgs c{};
    c.part_o = part_o;
    c.out = out;
    c.B = p->B; c.Hq = tokens(p) * p->Hq; c.P = P;
    c.out_dtype = p->out_dtype;
    return launch_sum_partials(c, p->d, static_cast<hipStream_t>(stream)) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

}  // extern "C"
