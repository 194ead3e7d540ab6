// Workgroup -> (batch, kv head, head slice, chunk) mapping and the key range of
// the chunk.  Tree Attention (arXiv 2408.04093) Algorithm 3 step 1 with the
// chunks handed to workgroups instead of devices.  Device code only.
//
// Launch order matters because the hardware dispatcher hands out workgroups
// in index order, workgroup i to XCD i mod 8: the index is chunk-major (all
// groups' chunk 0 first), so in a ragged batch the empty chunks of short
// sequences sit at the end and leave at once; inside one chunk index the row
// slices (matrix-core kernel, more than 64 rows per kv head) are the slow
// axis, so that with B * Hkv a multiple of 8 the workgroups that stream the
// same chunk of K/V for different row slices start together on the same XCD
// and share its L2 (two slices: 153 us against 179-195 us per launch; when
// B * Hkv is not a multiple of 8 the launch index is padded to one, the
// surplus workgroups exit at once); with an explicit table of unequal chunks (P <= 256) the chunks are
// visited largest first (longest-processing-time order), which keeps a big
// chunk from starting late and running alone at the end.
#pragma once
#include "ta_internal.hpp"

namespace ta {

struct ChunkRange {
    bool surplus;  // padding workgroup of the launch index: nothing to do
    int b, hk, slice, chunk;
    int64_t lo;   // first key of the chunk
    int64_t L;    // valid length of the sequence
    int n;        // number of keys (0 = empty)
};

// Where one range of keys of one (batch, kv head, row slice) goes: what a streaming kernel processes
// in one go, a whole chunk (chunked launch) or one piece of a share (balanced launch).
struct Range {
    int b, hk, slice;
    int64_t lo;     // first key
    int n;          // number of keys
    int64_t L;      // valid length of the sequence (causal limits among query tokens)
    int64_t slot;   // chunked launch: chunk index; balanced launch: piece id
};

constexpr int kMaxRankedChunks = 256;

__device__ __forceinline__ void clamp_bounds(const PartialArgs &a, int chunk, int64_t L, int64_t &lo, int64_t &hi) {
    lo = a.bounds[chunk];
    hi = a.bounds[chunk + 1];
    lo = lo < 0 ? 0 : (lo > L ? L : lo);
    hi = hi < lo ? lo : (hi > L ? L : hi);
}

// sh: at least kMaxRankedChunks + 1 ints of LDS.  Must be called by every
// thread of the workgroup (it may synchronise).
template <int THREADS>
__device__ __forceinline__ ChunkRange select_chunk(const PartialArgs &a, int *sh) {
    static_assert(THREADS >= kMaxRankedChunks, "one thread per ranked chunk");
    ChunkRange c;
    const uint32_t bh = (uint32_t)a.bh_launch;
    const uint32_t groups = bh * (uint32_t)a.slices;
    uint32_t id = blockIdx.x;
    const int rank = id / groups;
    id %= groups;
    c.slice = id / bh;  id %= bh;
    // padded index (several slices): rotated by the chunk rank, or a batch with fewer than 8
    // (batch, kv head) pairs would put all its work on the first XCDs
    if (a.slices > 1) id = (id + bh - (uint32_t)rank % bh) % bh;
    c.hk = id % (uint32_t)a.Hkv;
    c.b = id / (uint32_t)a.Hkv;
    c.surplus = c.b >= a.B;
    if (c.surplus) return c;   // the whole workgroup, before any barrier

    int64_t L = a.N;
    if (a.valid_len) {
        L = a.valid_len[c.b];
        L = L < 0 ? 0 : (L > a.N ? a.N : L);
    }
    int64_t lo, hi;
    c.chunk = rank;
    if (a.bounds) {
        if (a.P <= kMaxRankedChunks) {
            // chunk with the rank-th largest size (ties by index): O(P) per thread, P threads
            const int t = threadIdx.x;
            int my = 0;
            if (t < a.P) {
                clamp_bounds(a, t, L, lo, hi);
                my = (int)(hi - lo);
                sh[t] = my;
            }
            __syncthreads();
            if (t < a.P) {
                int r = 0;
                for (int j = 0; j < a.P; ++j) {
                    const int sj = sh[j];
                    r += (sj > my || (sj == my && j < t)) ? 1 : 0;
                }
                if (r == rank) sh[kMaxRankedChunks] = t;
            }
            __syncthreads();
            c.chunk = sh[kMaxRankedChunks];
        }
        clamp_bounds(a, c.chunk, L, lo, hi);
    } else {
        lo = (int64_t)c.chunk * a.t;
        lo = lo > L ? L : lo;
        hi = lo + a.t;
        hi = hi > L ? L : hi;
    }
    c.lo = lo;
    c.L = L;
    c.n = (int)(hi - lo);
    return c;
}

}  // namespace ta
