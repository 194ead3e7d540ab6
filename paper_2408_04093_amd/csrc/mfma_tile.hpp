// Pieces shared by the matrix-core streaming kernels (decode_partial_mfma.hip: key tiles split
// across the waves of a workgroup; decode_rows_mfma.hip: row blocks split across the waves):
// vector types, head-dimension geometry, the key order inside a 32-key tile, pass modes and the
// description of one range of keys.  Device code only.
#pragma once
#include "ta_internal.hpp"
#include "wave_ops.hpp"

namespace ta {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kAuxStream = 2;   // cache-policy bits of a buffer load: non-temporal (K/V are read once)
constexpr int kAuxShared = 0;   // default policy: lines stay in the XCD's L2 for other workgroups
constexpr int kTile = 32;       // keys per MFMA tile: 2 groups of 16 keys for QK^T, one 32-deep PV step

// Head-dimension geometry.  A K or V row (2 D bytes) is always spread over 16 lanes, so a lane
// holds D / 16 consecutive columns of each of its keys: 128-bit loads at d = 128, 64-bit at d = 64.
template <int D>
struct Geo {
    static_assert(D == 128 || D == 64, "head dimension");
    static constexpr int kCols = D / 16;            // columns per lane = PV tiles of 16 columns
    static constexpr int kLaneBytes = 2 * kCols;    // bytes per lane per row
    static constexpr int kWords = kCols / 2;        // dwords per lane per row
    static constexpr int kSteps = D / 32;           // k-steps of the QK^T contraction
    static constexpr int kPitch = 2 * D + 16;       // LDS bytes per staged K row (16-byte pad: conflict-free A reads)
    static constexpr int kStage = kTile * kPitch;   // one 32-key tile of K in LDS
    typedef int row_t __attribute__((ext_vector_type(kWords)));   // one lane's share of one row
    // off: per-lane byte offset (a vector register); soff: wave-uniform byte offset (a scalar register)
    // AUX: cache-policy bits of the load
    template <int AUX>
    static __device__ __forceinline__ row_t load(__amdgpu_buffer_rsrc_t rs, int off, int soff = 0) {
        if constexpr (D == 128) return __builtin_amdgcn_raw_buffer_load_b128(rs, off, soff, AUX);
        else return __builtin_amdgcn_raw_buffer_load_b64(rs, off, soff, AUX);
    }
};

// tile row owned by (row group r, slot e): e = 4G + i  ->  16G + 4r + i
__device__ __forceinline__ int kappa(int r, int e) { return 16 * (e >> 2) + 4 * r + (e & 3); }

__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    bf16x2 p = {(__bf16)a, (__bf16)b};   // v_cvt_pk_bf16_f32, round to nearest even
    uint32_t u;
    __builtin_memcpy(&u, &p, 4);
    return u;
}

// MODE selects what one pass computes (the paper's Algorithm 3 against its
// Algorithms 1 and 2):
//   kFull      (m, l, o) per chunk: Algorithm 3 steps 1-2.
//   kEnergy    (m, l) only, K is the only stream: the energy / logsumexp pass of
//              Algorithm 1 (zeta = 0 never materialised).
//   kGradient  o = sum_a exp(s_a - lse) v_a with the final lse given: Algorithm 2
//              step 5; no running max, no normaliser, partials add up plainly.
enum { kFull = 0, kEnergy = 1, kGradient = 2 };

// The running shift of a row is raised only when a step's row maximum exceeds it by more than
// this many log2 units, so exponentials stay below 2^kLazy.  Raising on every new maximum is
// not rare: with R rows riding on a wave, step t brings a new maximum for some row with
// probability ~R/t, i.e. on most steps of a 4096-key chunk once 16 or more rows are live.
constexpr float kLazy = 8.0f;

}  // namespace ta
