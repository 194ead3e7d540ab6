// Host-side launch descriptors shared by the API layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tree_attn.h"

namespace ta {

constexpr double kLog2e = 1.4426950408889634074;
constexpr double kLn2 = 0.69314718055994530942;

// Everything one decode_partial launch needs, passed by value.
struct PartialArgs {
    const void *q, *K, *V;
    const int32_t *valid_len;   // device [B] or null
    const int64_t *bounds;      // device [P+1] or null
    float *part_m, *part_l, *part_o;
    const float *lse_in;        // gradient pass only: total logsumexp per (b, token, head)
    // P == 1 shortcut (matrix-core kernel): the single chunk IS the result, written here directly
    // (normalised out, natural-log lse) instead of a partial; null = write partials
    void *out;
    float *lse_out;
    int32_t out_dtype;
    // balanced launch (matrix-core kernel, ragged batches): W workgroups share all keys equally
    int32_t W;                  // workgroups = shares
    int32_t piece_rows;         // rows reserved per piece in the partial arrays (= rows)
    int64_t *cum;               // device [B+1]: prefix sums of the virtual lengths (keys + piece charge),
                                // written by workgroup 0 for the combine kernel
    int64_t N;
    int64_t t;                  // keys per chunk when bounds == null
    int64_t k_sb, k_sh, v_sb, v_sh;   // elements
    uint32_t k_row_bytes, v_row_bytes;
    int32_t B, Hq, Hkv, P;
    int32_t g;                  // Hq / Hkv
    int32_t slices;             // VALU kernel: g / heads-per-workgroup; MFMA kernel: row slices
    int32_t bh_launch;          // (batch, kv head) pairs per slice in the launch index: B * Hkv, rounded up to a
                                // multiple of 8 when there are several slices (the surplus workgroups exit at once)
    int32_t Sq;                 // query tokens per sequence (>= 1)
    int32_t rows;               // MFMA kernel: (token, head-in-group) rows per slice, <= 64.  Rows are numbered
                                // token-major (row = token * g + head in group) and cut into slices of `rows`
    double c;                   // scale * log2(e)
};

struct CombineArgs {
    const float *part_m, *part_l, *part_o;
    void *out;
    float *lse;
    int32_t B, Hq, P;           // Hq counts (token, head) rows per sequence
    int32_t out_dtype;
    // balanced launch: the partials of row (b, t, h) are the consecutive pieces of its segment
    const int64_t *cum;         // null = chunked layout [B,Hq,P]
    int32_t W, min_share, piece_cost, piece_rows;
    int32_t heads, g, Hkv, slices, rows; // real Hq, group size, kv heads, row slices, rows per slice
};
// Launch a kernel that takes one descriptor struct by value and return THIS launch's status (not
// the runtime's sticky last-error state, which an unrelated earlier call may have set).
template <typename Args>
inline hipError_t launch_kernel(void (*kernel)(Args), dim3 grid, dim3 block, hipStream_t s, const Args &a) {
    void *params[] = {const_cast<Args *>(&a)};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, params, 0, s);
}

// energy pass: lse from (m, l) partials only; gradient pass: out = plain sum of the partial numerators
hipError_t launch_energy_combine(const CombineArgs &a, hipStream_t s);
hipError_t launch_sum_partials(const CombineArgs &a, int d, hipStream_t s);

// bf16 runs on the matrix-core kernel (any group size up to 16 in one pass);
// fp32 on the VALU kernel.
inline bool use_mfma_path(int dtype, int d) { return dtype == TA_BF16 && (d == 128 || d == 64); }

// (token, head) rows of one kv head handled by one workgroup, given their number.
inline int heads_per_workgroup(int dtype, int d, int g) {
    if (use_mfma_path(dtype, d)) return g;
    for (int gt : {4, 2}) if (g % gt == 0) return gt;   // vector-ALU kernel: 4, 2 or 1
    return 1;
}

// workgroups of a chunked launch
inline int64_t launch_blocks(const PartialArgs &a) { return (int64_t)a.bh_launch * a.slices * a.P; }

// fp32 K/V on the vector ALU; mode as below
hipError_t launch_decode_partial(const PartialArgs &a, int dtype, int d, int mode, hipStream_t s);
// resident workgroups per compute unit of the decode_partial instantiation for (dtype, d, heads per workgroup)
int decode_partial_occupancy(int dtype, int d, int gt);
// bf16, d in {64, 128}.  mode: 0 = (m,l,o), 1 = energy pass (m,l; K only), 2 = gradient pass given lse (o only)
hipError_t launch_decode_partial_mfma(const PartialArgs &a, int d, int mode, hipStream_t s);
// mode: 0 = (m,l,o), 1 = energy pass, 2 = gradient pass
hipError_t launch_decode_balanced_mfma(const PartialArgs &a, int d, int mode, hipStream_t s);
// balanced launch of the vector-ALU kernel (fp32 K/V), same modes; resident workgroups per compute unit
hipError_t launch_decode_balanced(const PartialArgs &a, int d, int mode, hipStream_t s);
int decode_balanced_occupancy(int d, int gt);
hipError_t launch_tree_combine(const CombineArgs &a, int d, hipStream_t s);

}  // namespace ta
