// Host property test of the balanced-launch index arithmetic (balanced_index.hpp), built with
// g++ -fsanitize=address,undefined by tests/test_balanced_index.py.  For seeded random length tables it
// walks every share the way the streaming kernel does and checks, against the combine kernel's view:
//   * every piece has n > 0 keys and an id in [0, W + B * G), no id is used twice;
//   * the pieces of every non-empty segment are exactly the ids pieces_of_segment() reports, in order;
//   * their key ranges tile [0, L_b) with no gap and no overlap; empty segments have no piece.
// Exit status 0 = all cases hold; otherwise the first violation is printed.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <vector>

#include "../paper_2408_04093_amd/csrc/balanced_index.hpp"

using namespace ta::balanced;

struct Seen { int64_t k0; int n; };

static int check_case(const std::vector<int64_t> &len, int64_t G, int W, int min_share, int piece_cost, const char *what) {
    const int B = (int)len.size();
    std::vector<int64_t> cum(B + 1, 0);
    for (int b = 0; b < B; ++b) cum[b + 1] = cum[b] + virtual_len(len[b], piece_cost);
    const int64_t id_limit = (int64_t)W + (int64_t)B * G;
    std::map<int64_t, std::pair<int64_t, Seen>> by_id;          // id -> (segment index, keys)
    int64_t last_key_end = -1, last_seg = -1;
    for (int w = 0; w < W; ++w) {
        int64_t prev_seg = -1;
        bool bad = false;
        for_each_piece(cum.data(), B, G, W, min_share, piece_cost, w, [&](const Piece &p) {
            const int64_t seg = (int64_t)p.b * G + p.j;
            if (p.n <= 0 || p.k0 < 0 || p.k0 + p.n > len[p.b] || p.L != len[p.b] || p.j < 0 || p.j >= G) {
                printf("%s: share %d: bad piece b=%d j=%lld k0=%lld n=%d L=%lld\n", what, w, p.b, (long long)p.j, (long long)p.k0, p.n, (long long)p.L);
                bad = true;
            }
            if (p.id < 0 || p.id >= id_limit || by_id.count(p.id)) {
                printf("%s: share %d: id %lld out of range or used twice (limit %lld)\n", what, w, (long long)p.id, (long long)id_limit);
                bad = true;
            }
            if (seg < prev_seg) { printf("%s: share %d: segments out of order\n", what, w); bad = true; }
            // key order across shares: a segment continues where it stopped, a new one starts at 0
            if (seg == last_seg ? p.k0 != last_key_end : p.k0 != 0) {
                printf("%s: share %d: segment %lld starts at key %lld, expected %lld\n", what, w, (long long)seg, (long long)p.k0,
                       (long long)(seg == last_seg ? last_key_end : 0));
                bad = true;
            }
            if (seg != last_seg && last_seg >= 0 && last_key_end != len[last_seg / G]) {
                printf("%s: segment %lld ended at key %lld of %lld\n", what, (long long)last_seg, (long long)last_key_end, (long long)len[last_seg / G]);
                bad = true;
            }
            prev_seg = seg; last_seg = seg; last_key_end = p.k0 + p.n;
            by_id[p.id] = {seg, Seen{p.k0, p.n}};
        });
        if (bad) return 1;
    }
    if (last_seg >= 0 && last_key_end != len[last_seg / G]) { printf("%s: last segment incomplete\n", what); return 1; }
    // the combine kernel's view of every segment
    size_t counted = 0;
    for (int b = 0; b < B; ++b) {
        for (int64_t j = 0; j < G; ++j) {
            const SegmentPieces sp = pieces_of_segment(cum.data(), B, G, W, min_share, piece_cost, b, j);
            if (len[b] == 0) {
                if (sp.count != 0) { printf("%s: empty segment (%d,%lld) reports %d pieces\n", what, b, (long long)j, sp.count); return 1; }
                continue;
            }
            if (sp.count < 1) { printf("%s: segment (%d,%lld) reports no piece\n", what, b, (long long)j); return 1; }
            int64_t next_key = 0;
            for (int i = 0; i < sp.count; ++i) {
                auto it = by_id.find(sp.id0 + i);
                if (it == by_id.end() || it->second.first != (int64_t)b * G + j || it->second.second.k0 != next_key) {
                    printf("%s: segment (%d,%lld): piece %d (id %lld) missing, foreign or out of order\n", what, b, (long long)j, i, (long long)(sp.id0 + i));
                    return 1;
                }
                next_key += it->second.second.n;
            }
            if (next_key != len[b]) { printf("%s: segment (%d,%lld): pieces cover %lld of %lld keys\n", what, b, (long long)j, (long long)next_key, (long long)len[b]); return 1; }
            counted += sp.count;
        }
    }
    if (counted != by_id.size()) { printf("%s: %zu pieces written, %zu located\n", what, by_id.size(), counted); return 1; }
    return 0;
}

int main(int argc, char **argv) {
    const int cases = argc > 1 ? atoi(argv[1]) : 400;
    std::mt19937_64 rng(20240804);
    auto uni = [&](int64_t lo, int64_t hi) { return lo + (int64_t)(rng() % (uint64_t)(hi - lo + 1)); };
    int done = 0;
    // hand-picked shapes first: all empty, one key, exactly one share, a giant among dwarfs, many ones
    const std::vector<std::vector<int64_t>> fixed = {
        {0}, {0, 0, 0}, {1}, {1, 1, 1, 1}, {0, 1, 0}, {262144}, {262144, 1, 0, 3, 0, 0, 7}, {511, 512, 513}, {256, 256},
        std::vector<int64_t>(2048, 1), std::vector<int64_t>(2048, 0), std::vector<int64_t>(300, 4096)};
    for (const auto &len : fixed)
        for (int64_t G : {1, 2, 8, 24})
            for (int W : {1, 7, 256, 304}) {
                if (check_case(len, G, W, 512, 256, "fixed")) return 1;
                if (check_case(len, G, W, 1024, 512, "fixed d64")) return 1;
                ++done;
            }
    for (int c = 0; c < cases; ++c) {
        const int B = (int)uni(1, c % 10 == 0 ? 2048 : 64);
        const int64_t G = uni(1, 16);
        const int W = (int)uni(1, 320);
        const int kind = (int)uni(0, 4);
        std::vector<int64_t> len(B);
        for (int b = 0; b < B; ++b) {
            switch (kind) {
                case 0: len[b] = uni(0, 3); break;                                    // zeros and ones
                case 1: len[b] = uni(8192, 65536); break;                             // the ragged config
                case 2: len[b] = b == (int)(c % B) ? uni(100000, 1 << 20) : uni(0, 600); break;   // one giant
                case 3: len[b] = uni(0, 1) ? 0 : uni(1, 5000); break;                 // half empty
                default: len[b] = uni(0, 70000); break;
            }
        }
        const bool d64 = c & 1;
        char what[64];
        snprintf(what, sizeof what, "case %d (B=%d G=%lld W=%d kind %d)", c, B, (long long)G, W, kind);
        if (check_case(len, G, W, d64 ? 1024 : 512, d64 ? 512 : 256, what)) return 1;
        ++done;
    }
    printf("balanced index: %d cases hold\n", done);
    return 0;
}
