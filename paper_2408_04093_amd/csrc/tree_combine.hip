// tree_combine: merge P partials (m, l, o) per (batch, query head) into the
// attention output and its logsumexp.  Tree Attention (arXiv 2408.04093)
// Algorithm 3 steps 3-6 -- the arithmetic of the max all-reduce, the two sum
// all-reduces and the division -- done as one P-ary reduction per head
// (Appendix B allows any fan-in) instead of three collectives:
//     m* = max_j m_j;  w_j = exp(m_j - m*);  l* = sum w_j l_j;  o* = sum w_j o_j
//     out = o* / l*;   lse = m* + log l*
//
// The work is KB-to-MB sized and latency-bound, so the kernel is laid out for
// few dependent memory round trips and many workgroups: one workgroup per
// (b, h, 32-column slice); its 256 threads are 8 groups of 32 lanes, group r
// taking partials j = r, r+8, ... with up to 8 rows in flight per thread, the
// first batch fetched before anything else.  max and the sum of l are
// log-depth wavefront reductions finished in LDS; the weights w_j are staged
// in LDS once per 1024 partials.
#include <type_traits>

#include "balanced_index.hpp"
#include "ta_internal.hpp"
#include "wave_ops.hpp"

namespace ta {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSlice = 32;                   // columns per workgroup (one 128-byte line per row)
constexpr int kGroups = kThreads / kSlice;   // partial groups per workgroup
constexpr int kBatch = 8;                    // rows in flight per thread
constexpr int kTile = 1024;                  // weights staged in LDS at a time

__device__ __forceinline__ float block_reduce(float x, float *sh, bool is_max) {
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float y = __shfl_xor(x, off);
        x = is_max ? fmaxf(x, y) : x + y;
    }
    __syncthreads();            // sh may still be read from a previous call
    if (lane == 0) sh[w] = x;
    __syncthreads();
    float r = sh[0];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) r = is_max ? fmaxf(r, sh[ww]) : r + sh[ww];
    return r;
}

// Where the partials of row bh = (b, token, head) live: [B,Hq,P] (chunked launch) or the
// consecutive pieces of the row's segment, piece_rows apart (balanced launch).
struct RowPartials {
    int P;                 // number of partials
    int64_t sm, so;        // strides between consecutive partials, in floats
    const float *pm, *pl;  // first m and l
    const float *po;       // first numerator row (column 0)
};

// D = 0: only m and l are located (energy pass: there are no numerators)
template <int D>
__device__ __forceinline__ RowPartials locate_row(const CombineArgs &a, int64_t bh) {
    RowPartials rp;
    rp.P = a.P;
    rp.sm = 1;
    rp.so = D;
    rp.pm = a.part_m + bh * a.P;
    rp.pl = a.part_l + bh * a.P;
    rp.po = D ? a.part_o + bh * a.P * D : nullptr;
    if (a.cum) {
        const int b = (int)(bh / a.Hq), vrow = (int)(bh % a.Hq);
        const int t = vrow / a.heads, hq = vrow % a.heads;
        const int grow = t * a.g + hq % a.g;            // row number inside the kv head, token-major
        const int row = grow % a.rows;
        const int64_t G = (int64_t)a.Hkv * a.slices;
        const int64_t j = (int64_t)(hq / a.g) * a.slices + grow / a.rows;   // segment of the sequence
        const balanced::SegmentPieces sp =
            balanced::pieces_of_segment(a.cum, a.B, G, a.W, a.min_share, a.piece_cost, b, j);
        rp.P = sp.count;
        if (sp.count > 0) {
            rp.sm = a.piece_rows;
            rp.so = (int64_t)a.piece_rows * D;
            rp.pm = a.part_m + sp.id0 * a.piece_rows + row;
            rp.pl = a.part_l + sp.id0 * a.piece_rows + row;
            rp.po = D ? a.part_o + (sp.id0 * a.piece_rows + row) * D : nullptr;
        }
    }
    return rp;
}

template <int D>
__global__ void __launch_bounds__(kThreads) tree_combine_kernel(const CombineArgs a) {
    constexpr float kLog2eF = 1.4426950408889634074f;
    constexpr int kSlices = D / kSlice;

    const int tid = threadIdx.x;
    const int c = tid & (kSlice - 1);
    const int r = tid / kSlice;
    const int64_t bh = blockIdx.x / kSlices;
    const int col = (blockIdx.x % kSlices) * kSlice + c;
    const RowPartials rp = locate_row<D>(a, bh);
    const int P = rp.P;
    const int64_t sm = rp.sm, so = rp.so;
    const float *pm = rp.pm, *pl = rp.pl, *po = rp.po + col;

    __shared__ float sh_red[kWaves];
    __shared__ float sh_w[kTile];
    __shared__ float sh_o[kGroups][kSlice];

    // first batch of numerator rows: in flight while the max is being found
    float x0[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
        const int j = r + i * kGroups;
        x0[i] = j < P ? po[(int64_t)j * so] : 0.f;
    }

    // m* = max over partials that hold keys (l_j > 0)
    float mx = -__builtin_huge_valf();
    for (int j = tid; j < P; j += kThreads)
        if (pl[j * sm] > 0.f) mx = fmaxf(mx, pm[j * sm]);
    const float mstar = block_reduce(mx, sh_red, true);

    if (mstar == -__builtin_huge_valf()) {   // no key anywhere: out = 0, lse = -inf by definition
        if (tid < kSlice) {
            if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[bh * D + col] = 0;
            else reinterpret_cast<float *>(a.out)[bh * D + col] = 0.f;
        }
        if (tid == 0 && blockIdx.x % kSlices == 0) a.lse[bh] = -__builtin_huge_valf();
        return;
    }

    float acc = 0.f, lsum = 0.f;
    for (int t0 = 0; t0 < P; t0 += kTile) {
        const int tn = P - t0 < kTile ? P - t0 : kTile;
        if (t0) __syncthreads();
        for (int j = tid; j < tn; j += kThreads) {
            const float lj = pl[(t0 + j) * sm];
            const float wj = lj > 0.f ? exp2_hw((pm[(t0 + j) * sm] - mstar) * kLog2eF) : 0.f;
            sh_w[j] = wj;
            lsum = fmaf(wj, lj, lsum);
        }
        __syncthreads();
        for (int j0 = r; j0 < tn; j0 += kGroups * kBatch) {
            float x[kBatch];
            if (t0 == 0 && j0 == r) {
#pragma unroll
                for (int i = 0; i < kBatch; ++i) x[i] = x0[i];
            } else {
#pragma unroll
                for (int i = 0; i < kBatch; ++i) {
                    const int j = j0 + i * kGroups;
                    x[i] = j < tn ? po[(int64_t)(t0 + j) * so] : 0.f;
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int j = j0 + i * kGroups;
                if (j < tn) {   // a partial without keys may hold anything: never multiplied
                    const float wv = sh_w[j];
                    acc = fmaf(wv, wv != 0.f ? x[i] : 0.f, acc);
                }
            }
        }
    }
    const float lstar = block_reduce(lsum, sh_red, false);

    sh_o[r][c] = acc;
    __syncthreads();
    if (tid < kSlice) {
        float o = 0.f;
#pragma unroll
        for (int rr = 0; rr < kGroups; ++rr) o += sh_o[rr][tid];
        const float z = o / lstar;
        if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[bh * D + col] = f32_to_bf16_rne(z);
        else reinterpret_cast<float *>(a.out)[bh * D + col] = z;
    }
    if (tid == 0 && blockIdx.x % kSlices == 0) a.lse[bh] = mstar + logf(lstar);
}

// The same reduction with one wavefront per row, four rows per workgroup, for launches with
// many rows (large batches, many query tokens): there the kernel above is bound by the rate at
// which workgroups can be dispatched (one per row and 32-column slice: 69 us for 8192 rows).
// Lane j holds the weight of partial j of the current batch of 64; the numerators are then
// added partial by partial, each lane owning D / 64 adjacent columns, 16 loads in flight.
template <int D>
__global__ void __launch_bounds__(kThreads) tree_combine_rows_kernel(const CombineArgs a) {
    constexpr float kLog2eF = 1.4426950408889634074f;
    constexpr int kCols = D / kWave;   // columns per lane: 2 or 1
    constexpr int kUnroll = 16;
    typedef float colv __attribute__((ext_vector_type(kCols)));
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t bh = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (bh >= (int64_t)a.B * a.Hq) return;   // whole wavefront; the kernel has no workgroup barrier
    const RowPartials rp = locate_row<D>(a, bh);
    const int P = rp.P;

    float mx = -__builtin_huge_valf();
    for (int j = lane; j < P; j += kWave)
        if (rp.pl[j * rp.sm] > 0.f) mx = fmaxf(mx, rp.pm[j * rp.sm]);
    const float mstar = wave_max(mx);

    colv acc;
#pragma unroll
    for (int k = 0; k < kCols; ++k) acc[k] = 0.f;
    float lsum = 0.f;
    if (mstar != -__builtin_huge_valf()) {
        for (int j0 = 0; j0 < P; j0 += kWave) {
            const int j = j0 + lane;
            const float lj = j < P ? rp.pl[j * rp.sm] : 0.f;
            const float wj = lj > 0.f ? exp2_hw((rp.pm[j * rp.sm] - mstar) * kLog2eF) : 0.f;
            lsum = fmaf(wj, lj, lsum);
            const int nb = P - j0 < kWave ? P - j0 : kWave;
            // batches of 16 partials while that many are left, then batches of 4
            auto batch = [&](auto unroll_c, int jj0) {
                constexpr int U = decltype(unroll_c)::value;
                colv x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int jj = jj0 + u < nb ? jj0 + u : nb - 1;   // clamped: loads stay inside the row's partials
                    x[u] = *reinterpret_cast<const colv *>(rp.po + (int64_t)(j0 + jj) * rp.so + kCols * lane);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int jj = jj0 + u;
                    float wv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wj), jj & (kWave - 1)));
                    if (jj >= nb) wv = 0.f;
#pragma unroll
                    for (int k = 0; k < kCols; ++k)   // a partial without keys may hold anything: never multiplied
                        acc[k] = fmaf(wv, wv != 0.f ? x[u][k] : 0.f, acc[k]);
                }
            };
            int jj0 = 0;
            for (; jj0 + kUnroll <= nb; jj0 += kUnroll) batch(std::integral_constant<int, kUnroll>{}, jj0);
            for (; jj0 < nb; jj0 += 4) batch(std::integral_constant<int, 4>{}, jj0);
        }
    }
    float lstar = lsum;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lstar += __shfl_xor(lstar, off);

    // no key anywhere: out = 0, lse = -inf by definition
    const bool empty = mstar == -__builtin_huge_valf();
    colv z;
#pragma unroll
    for (int k = 0; k < kCols; ++k) z[k] = empty ? 0.f : acc[k] / lstar;
    if (a.out_dtype == TA_BF16) {
        unsigned short *o = reinterpret_cast<unsigned short *>(a.out) + bh * D + kCols * lane;
        if constexpr (kCols == 2)
            *reinterpret_cast<uint32_t *>(o) = (uint32_t)f32_to_bf16_rne(z[0]) | ((uint32_t)f32_to_bf16_rne(z[1]) << 16);
        else
            o[0] = f32_to_bf16_rne(z[0]);
    } else {
        *reinterpret_cast<colv *>(reinterpret_cast<float *>(a.out) + bh * D + kCols * lane) = z;
    }
    if (lane == 0) a.lse[bh] = empty ? mstar : mstar + logf(lstar);
}

// Energy pass: lse = m* + log(sum_j exp(m_j - m*) l_j) from the (m, l) partials alone
// (Algorithm 1 steps 4-6 as one reduction).  One wavefront per (b, h), four per workgroup.
__global__ void __launch_bounds__(kThreads) energy_combine_kernel(const CombineArgs a) {
    constexpr float kLog2eF = 1.4426950408889634074f;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t bh = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (bh >= (int64_t)a.B * a.Hq) return;   // whole wavefront; the kernel has no workgroup barrier
    const RowPartials rp = locate_row<0>(a, bh);
    float mx = -__builtin_huge_valf();
    for (int j = lane; j < rp.P; j += kWave)
        if (rp.pl[j * rp.sm] > 0.f) mx = fmaxf(mx, rp.pm[j * rp.sm]);
    mx = wave_max(mx);
    if (mx == -__builtin_huge_valf()) {
        if (lane == 0) a.lse[bh] = mx;
        return;
    }
    float ls = 0.f;
    for (int j = lane; j < rp.P; j += kWave) {
        const float lj = rp.pl[j * rp.sm];
        if (lj > 0.f) ls = fmaf(exp2_hw((rp.pm[j * rp.sm] - mx) * kLog2eF), lj, ls);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ls += __shfl_xor(ls, off);
    if (lane == 0) a.lse[bh] = mx + logf(ls);
}

// Gradient pass (Algorithm 2 step 6): out = Reduce(sum) of the per-chunk numerators, no weights.
// The numerators of a row are its P chunks or, after a balanced launch, the pieces of its segment.
template <int D>
__global__ void __launch_bounds__(kThreads) sum_partials_kernel(const CombineArgs a) {
    constexpr int kSlices = D / kSlice;
    const int tid = threadIdx.x;
    const int c = tid & (kSlice - 1);
    const int r = tid / kSlice;
    const int64_t bh = blockIdx.x / kSlices;
    const int col = (blockIdx.x % kSlices) * kSlice + c;
    const RowPartials rp = locate_row<D>(a, bh);
    const float *po = rp.po + col;
    __shared__ float sh_o[kGroups][kSlice];

    float acc = 0.f;
    for (int j0 = r; j0 < rp.P; j0 += kGroups * kBatch) {
        float x[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int j = j0 + i * kGroups;
            x[i] = j < rp.P ? po[(int64_t)j * rp.so] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) acc += x[i];
    }
    sh_o[r][c] = acc;
    __syncthreads();
    if (tid < kSlice) {
        float o = 0.f;
#pragma unroll
        for (int rr = 0; rr < kGroups; ++rr) o += sh_o[rr][tid];
        if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[bh * D + col] = f32_to_bf16_rne(o);
        else reinterpret_cast<float *>(a.out)[bh * D + col] = o;
    }
}

}  // namespace

// One wavefront per row pays from 512 rows on (4 us against 6 us; 4 against 17 at 2048 rows) as
// long as a row has at most ~100 partials; a row of 256 partials takes it 1.5x as long as the
// workgroup-per-slice kernel.  With the balanced layout the partials per row are not known here;
// they are few except for a sequence much longer than the rest of its batch.
constexpr int kRowKernelMinRows = 512;
constexpr int kRowKernelMaxP = 128;

hipError_t launch_tree_combine(const CombineArgs &a, int d, hipStream_t s) {
    const int64_t rows = (int64_t)a.B * a.Hq;
    // the row kernel moves two adjacent columns per lane at d = 128: needs 8-byte aligned rows
    const bool pairs_ok = d == 64 || (((reinterpret_cast<uintptr_t>(a.part_o) | reinterpret_cast<uintptr_t>(a.out)) &
                                       (a.out_dtype == TA_BF16 ? 3u : 7u)) == 0 &&
                                      (reinterpret_cast<uintptr_t>(a.part_o) & 7u) == 0);
    if (rows >= kRowKernelMinRows && pairs_ok && (a.cum != nullptr || a.P <= kRowKernelMaxP)) {
        const dim3 grid((uint32_t)((rows + kWaves - 1) / kWaves));
        if (d == 128) return launch_kernel(tree_combine_rows_kernel<128>, grid, dim3(kThreads), s, a);
        return launch_kernel(tree_combine_rows_kernel<64>, grid, dim3(kThreads), s, a);
    }
    const dim3 grid((uint32_t)(rows * (d / kSlice)));
    if (d == 128) return launch_kernel(tree_combine_kernel<128>, grid, dim3(kThreads), s, a);
    return launch_kernel(tree_combine_kernel<64>, grid, dim3(kThreads), s, a);
}

hipError_t launch_energy_combine(const CombineArgs &a, hipStream_t s) {
    const int64_t rows = (int64_t)a.B * a.Hq;
    return launch_kernel(energy_combine_kernel, dim3((uint32_t)((rows + kWaves - 1) / kWaves)), dim3(kThreads), s, a);
}

hipError_t launch_sum_partials(const CombineArgs &a, int d, hipStream_t s) {
    const dim3 grid((uint32_t)((int64_t)a.B * a.Hq * (d / kSlice)));
    if (d == 128) return launch_kernel(sum_partials_kernel<128>, grid, dim3(kThreads), s, a);
    return launch_kernel(sum_partials_kernel<64>, grid, dim3(kThreads), s, a);
}

}  // namespace ta
