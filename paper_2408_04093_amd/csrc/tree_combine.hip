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

template <int D>
__global__ void __launch_bounds__(kThreads) tree_combine_kernel(const CombineArgs a) {
    constexpr float kLog2eF = 1.4426950408889634074f;
    constexpr int kSlices = D / kSlice;

    const int tid = threadIdx.x;
    const int c = tid & (kSlice - 1);
    const int r = tid / kSlice;
    const int64_t bh = blockIdx.x / kSlices;
    const int col = (blockIdx.x % kSlices) * kSlice + c;
    // where this row's partials live: [B,Hq,P] (chunked launch) or the consecutive pieces of the
    // row's segment, piece_rows apart (balanced launch)
    int P = a.P;
    int64_t sm = 1, so = D;                      // strides between consecutive partials
    const float *pm = a.part_m + bh * P;
    const float *pl = a.part_l + bh * P;
    const float *po = a.part_o + bh * P * D + col;
    if (a.cum) {
        const int b = (int)(bh / a.Hq), vrow = (int)(bh % a.Hq);
        const int t = vrow / a.heads, hq = vrow % a.heads;
        const int grow = t * a.g + hq % a.g;            // row number inside the kv head, token-major
        const int row = grow % a.rows;
        const int64_t G = (int64_t)a.Hkv * a.slices;
        const int64_t j = (int64_t)(hq / a.g) * a.slices + grow / a.rows;
        // cum holds virtual lengths: keys + piece_cost per non-empty segment, the keys coming last
        const int64_t Lv = a.cum[b + 1] - a.cum[b];
        const int64_t Lb = Lv - a.piece_cost;
        int64_t S = (a.cum[a.B] * G + a.W - 1) / a.W;
        S = S < a.min_share ? a.min_share : S;
        P = 0;
        if (Lv > 0) {
            const int64_t seg0 = a.cum[b] * G + j * Lv + a.piece_cost;   // first key, virtual position
            const int64_t w0 = seg0 / S, w1 = (seg0 + Lb - 1) / S;
            const int64_t id0 = w0 + (int64_t)b * G + j;
            P = (int)(w1 - w0 + 1);
            sm = a.piece_rows;
            so = (int64_t)a.piece_rows * D;
            pm = a.part_m + id0 * a.piece_rows + row;
            pl = a.part_l + id0 * a.piece_rows + row;
            po = a.part_o + (id0 * a.piece_rows + row) * D + col;
        }
    }

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
                if (j < tn) acc = fmaf(sh_w[j], x[i], acc);
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

// Energy pass: lse = m* + log(sum_j exp(m_j - m*) l_j) from the (m, l) partials alone
// (Algorithm 1 steps 4-6 as one reduction).  One wavefront per (b, h).
__global__ void __launch_bounds__(kWave) energy_combine_kernel(const CombineArgs a) {
    constexpr float kLog2eF = 1.4426950408889634074f;
    const int lane = threadIdx.x;
    const int64_t bh = blockIdx.x;
    const float *pm = a.part_m + bh * a.P;
    const float *pl = a.part_l + bh * a.P;
    float mx = -__builtin_huge_valf();
    for (int j = lane; j < a.P; j += kWave)
        if (pl[j] > 0.f) mx = fmaxf(mx, pm[j]);
    mx = wave_max(mx);
    if (mx == -__builtin_huge_valf()) {
        if (lane == 0) a.lse[bh] = mx;
        return;
    }
    float ls = 0.f;
    for (int j = lane; j < a.P; j += kWave) {
        const float lj = pl[j];
        if (lj > 0.f) ls = fmaf(exp2_hw((pm[j] - mx) * kLog2eF), lj, ls);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ls += __shfl_xor(ls, off);
    if (lane == 0) a.lse[bh] = mx + logf(ls);
}

// Gradient pass (Algorithm 2 step 6): out = Reduce(sum) of the per-chunk numerators, no weights.
template <int D>
__global__ void __launch_bounds__(kThreads) sum_partials_kernel(const CombineArgs a) {
    constexpr int kSlices = D / kSlice;
    const int tid = threadIdx.x;
    const int c = tid & (kSlice - 1);
    const int r = tid / kSlice;
    const int64_t bh = blockIdx.x / kSlices;
    const int col = (blockIdx.x % kSlices) * kSlice + c;
    const float *po = a.part_o + bh * a.P * D + col;
    __shared__ float sh_o[kGroups][kSlice];

    float acc = 0.f;
    for (int j0 = r; j0 < a.P; j0 += kGroups * kBatch) {
        float x[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int j = j0 + i * kGroups;
            x[i] = j < a.P ? po[(int64_t)j * D] : 0.f;
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

hipError_t launch_tree_combine(const CombineArgs &a, int d, hipStream_t s) {
    const dim3 grid((uint32_t)((int64_t)a.B * a.Hq * (d / kSlice)));
    if (d == 128) hipLaunchKernelGGL((tree_combine_kernel<128>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((tree_combine_kernel<64>), grid, dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_energy_combine(const CombineArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(energy_combine_kernel, dim3((uint32_t)((int64_t)a.B * a.Hq)), dim3(kWave), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_sum_partials(const CombineArgs &a, int d, hipStream_t s) {
    const dim3 grid((uint32_t)((int64_t)a.B * a.Hq * (d / kSlice)));
    if (d == 128) hipLaunchKernelGGL((sum_partials_kernel<128>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((sum_partials_kernel<64>), grid, dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace ta
