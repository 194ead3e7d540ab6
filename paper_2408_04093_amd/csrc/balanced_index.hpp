// Index arithmetic of the balanced launch for ragged batches, in ONE place: the streaming kernel
// (which cuts the keys of all segments into equal-cost shares and walks its share) and the combine
// kernel (which has to find the pieces a row was cut into) both use these functions, and the same
// header compiles for the host, where a property test checks that the two views agree.
//
// Vocabulary.  A SEGMENT is one (batch b, index j) pair, j < G counting (kv head, row slice) pairs
// of the sequence; all G segments of sequence b hold the same L_b keys.  Segments are laid end to
// end in the order (b, j).  A non-empty segment is preceded by `piece_cost` VIRTUAL keys that stand
// for the fixed cost of starting a piece, so its virtual length is L_b + piece_cost; an empty one
// has virtual length 0.  cum[b] = sum of the virtual lengths of sequences < b (one segment each),
// so segment (b, j) starts at virtual position cum[b] * G + j * (cum[b+1] - cum[b]).  The T =
// cum[B] * G virtual keys are cut into shares of S = max(ceil(T / W), min_share), share w =
// [w S, (w+1) S).  The intersection of a share with the keys of a segment is a PIECE; its id is
// w + b G + j: unique, and consecutive over the shares a segment spans (Section 5.1 of the Tree
// Attention paper, arXiv 2408.04093: associativity makes every cut point legal).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TA_HOST_DEVICE __host__ __device__
#else
#define TA_HOST_DEVICE
#endif

namespace ta {
namespace balanced {

TA_HOST_DEVICE inline int64_t virtual_len(int64_t L, int piece_cost) { return L > 0 ? L + piece_cost : 0; }

// share size in virtual keys; total = cum[B] * G
TA_HOST_DEVICE inline int64_t share_size(int64_t total, int W, int min_share) {
    const int64_t S = (total + W - 1) / W;
    return S < min_share ? min_share : S;
}

struct Piece {
    int b;          // sequence
    int64_t j;      // segment of the sequence: (kv head, row slice) pair
    int64_t k0;     // first key
    int n;          // number of keys, > 0
    int64_t L;      // keys of the sequence
    int64_t id;     // piece id: share + b G + j
};

// Calls f(piece) for every piece of share w, in key order.  cum: B + 1 prefix sums.
template <typename F>
TA_HOST_DEVICE inline void for_each_piece(const int64_t *cum, int B, int64_t G, int W, int min_share, int piece_cost,
                                          int w, F &&f) {
    const int64_t T = cum[B] * G;
    const int64_t S = share_size(T, W, min_share);
    const int64_t x0 = (int64_t)w * S;
    const int64_t x1 = x0 + S < T ? x0 + S : T;
    if (x0 >= T) return;
    int b = 0, hi_b = B;   // cum[b] * G <= x0 < cum[hi_b] * G
    while (hi_b - b > 1) {
        const int mid = (b + hi_b) >> 1;
        if (cum[mid] * G <= x0) b = mid; else hi_b = mid;
    }
    for (int64_t x = x0; x < x1;) {
        while (cum[b + 1] * G <= x) ++b;              // also skips empty sequences; b < B because x < T
        const int64_t Lv = cum[b + 1] - cum[b];       // virtual length of this sequence's segments
        const int64_t Lb = Lv - piece_cost;           // its keys
        const int64_t rel = x - cum[b] * G;
        const int64_t j = rel / Lv;                   // segment of this sequence
        const int64_t v0 = rel - j * Lv;              // virtual offset inside the segment
        const int64_t span = (Lv - v0) < (x1 - x) ? (Lv - v0) : (x1 - x);
        // the first piece_cost virtual keys of a segment are the charge, the rest are its keys
        const int64_t k0 = v0 > piece_cost ? v0 - piece_cost : 0;
        int64_t k1 = v0 + span - piece_cost;
        k1 = k1 > Lb ? Lb : k1;
        if (k1 > k0) f(Piece{b, j, k0, (int)(k1 - k0), Lb, (int64_t)w + (int64_t)b * G + j});
        x += span;
    }
}

struct SegmentPieces {
    int64_t id0;   // id of the first piece
    int count;     // number of pieces (0 for an empty segment); their ids are id0 .. id0 + count - 1
};

// The pieces segment (b, j) was cut into.
TA_HOST_DEVICE inline SegmentPieces pieces_of_segment(const int64_t *cum, int B, int64_t G, int W, int min_share,
                                                      int piece_cost, int b, int64_t j) {
    const int64_t Lv = cum[b + 1] - cum[b];
    if (Lv <= 0) return SegmentPieces{0, 0};
    const int64_t Lb = Lv - piece_cost;
    const int64_t S = share_size(cum[B] * G, W, min_share);
    const int64_t seg0 = cum[b] * G + j * Lv + piece_cost;   // virtual position of the first key
    const int64_t w0 = seg0 / S, w1 = (seg0 + Lb - 1) / S;
    return SegmentPieces{w0 + (int64_t)b * G + j, (int)(w1 - w0 + 1)};
}

}  // namespace balanced
}  // namespace ta
