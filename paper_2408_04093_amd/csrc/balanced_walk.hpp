// Balanced launch for ragged batches (lengths known only on the device), the part both streaming
// kernels share.  The keys of all (batch, kv head, row slice) segments are laid end to end and cut
// into W equal shares, one per workgroup, so every workgroup streams the same number of bytes
// whatever the mix of lengths; a share that crosses a segment boundary is processed as several
// pieces.  Piece ids (workgroup index + segment index) are unique and the pieces of one segment are
// consecutive, which is all the combine kernel needs.  Associativity (Tree Attention, arXiv
// 2408.04093, Section 5.1) makes the cut points free.
//
// Shares are equal in COST, not in keys: every non-empty segment is charged extra "virtual keys" at
// its start for the fixed cost of a piece (q load, pipeline ramp, epilogue: ~3 us, the time a CU
// streams ~64 KB of K), so a workgroup that gets a run of tiny sequences gets fewer of them.
// Without the charge a share made of ~100 tiny segments took 2x the time of the others.
// The integer arithmetic (shares -> pieces, segment -> piece ids) is balanced_index.hpp.
#pragma once
#include "balanced_index.hpp"
#include "chunking.hpp"
#include "ta_internal.hpp"

namespace ta {

constexpr int kMaxBalancedB = 2048;          // sequences whose prefix sums fit the LDS table
constexpr int kMinShareBytes = 512 * 256;    // never cut finer than this many bytes of K (512 keys of bf16 at d = 128)
constexpr int kPieceCostBytes = 256 * 256;   // bytes of K charged per non-empty segment (256 such keys)

// in keys, for K rows of row_bytes (= d x element size)
constexpr int balanced_min_share_keys(int row_bytes) { return kMinShareBytes / row_bytes; }
constexpr int balanced_piece_cost_keys(int row_bytes) { return kPieceCostBytes / row_bytes; }

#if defined(__HIPCC__)
// LDS a workgroup needs for the walk
struct BalancedShared {
    int64_t cum[kMaxBalancedB + 1];
    int64_t scan[16];
};

// Called by every thread of a workgroup of THREADS threads: builds the prefix table of the virtual
// lengths (workgroup 0 also leaves it in a.cum for the combine kernel) and calls
// process(const Range &) for every piece of this workgroup's share, in key order, with a
// barrier between two pieces (a piece's epilogue may still be reading LDS).
template <int THREADS, int ROW_BYTES, typename F>
__device__ __forceinline__ void balanced_walk(const PartialArgs &a, BalancedShared &sh, F &&process) {
    constexpr int kMinShare = balanced_min_share_keys(ROW_BYTES), kPieceCost = balanced_piece_cost_keys(ROW_BYTES);
    constexpr int kWaveLanes = 64;
    static_assert(THREADS / kWaveLanes <= 16, "scan table");
    const int tid = threadIdx.x;
    auto len_of = [&](int bb) -> int64_t {   // virtual length of one segment of sequence bb
        int64_t L = a.N;
        if (a.valid_len) {
            L = a.valid_len[bb];
            L = L < 0 ? 0 : (L > a.N ? a.N : L);
        }
        return balanced::virtual_len(L, kPieceCost);
    };
    // exclusive prefix sums of the virtual lengths: each thread takes a run of sequences, then a
    // THREADS-wide scan of the run totals
    const int per = (a.B + THREADS - 1) / THREADS;
    int64_t mine = 0;
    for (int i = 0; i < per; ++i) {
        const int bb = tid * per + i;
        if (bb < a.B) mine += len_of(bb);
    }
    // inclusive scan: inside each wave by shuffles, then the wave totals through LDS
    int64_t incl = mine;
    {
        const int lane = tid & (kWaveLanes - 1);
#pragma unroll
        for (int off = 1; off < kWaveLanes; off <<= 1) {
            const int64_t v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        if (lane == kWaveLanes - 1) sh.scan[tid >> 6] = incl;
        __syncthreads();
        int64_t base = 0;
        for (int ww = 0; ww < (tid >> 6); ++ww) base += sh.scan[ww];
        incl += base;
    }
    int64_t run = incl - mine;
    for (int i = 0; i < per; ++i) {
        const int bb = tid * per + i;
        if (bb < a.B) {
            sh.cum[bb] = run;
            run += len_of(bb);
        }
    }
    if (tid == THREADS - 1) sh.cum[a.B] = incl;
    __syncthreads();
    if (blockIdx.x == 0)   // the combine kernel reads the same table
        for (int i = tid; i <= a.B; i += THREADS) a.cum[i] = sh.cum[i];

    // this workgroup's share of all (virtual) keys, piece by piece
    const int64_t G = (int64_t)a.Hkv * a.slices;
    bool first = true;
    balanced::for_each_piece(sh.cum, a.B, G, a.W, kMinShare, kPieceCost, (int)blockIdx.x, [&](const balanced::Piece &pc) {
        const Range rg{pc.b, (int)(pc.j / a.slices), (int)(pc.j % a.slices), pc.k0, pc.n, pc.L, pc.id};
        if (!first) __syncthreads();
        first = false;
        process(rg);
    });
}
#endif

}  // namespace ta
