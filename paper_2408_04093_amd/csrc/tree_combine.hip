// tree_combine: merge P partials (m, l, o) per (batch, query head) into the
// attention output and its logsumexp.  Tree Attention (arXiv 2408.04093)
// Algorithm 3 steps 3-6 -- the arithmetic of the max all-reduce, the two sum
// all-reduces and the division -- done as one P-ary reduction per head
// (Appendix B allows any fan-in) instead of three collectives:
//     m* = max_j m_j;  w_j = exp(m_j - m*);  l* = sum w_j l_j;  o* = sum w_j o_j
//     out = o* / l*;   lse = m* + log l*
//
// One workgroup of 4 waves per (b, h).  The max over j is a log-depth
// wavefront reduction; the weighted sums stream the P x d partial tile with
// coalesced row reads, each wave taking every 4th partial, several rows in
// flight; the 4 wave results meet in LDS.  The work is KB-to-MB sized and
// latency-bound.
#include "ta_internal.hpp"
#include "wave_ops.hpp"

namespace ta {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <int D>
__global__ void __launch_bounds__(kThreads) tree_combine_kernel(const CombineArgs a) {
    constexpr int CPL = D / kWave;   // columns per lane: 2 (d=128) or 1 (d=64)
    constexpr float kLog2eF = 1.4426950408889634074f;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t bh = blockIdx.x;
    const int P = a.P;
    const float *pm = a.part_m + bh * P;
    const float *pl = a.part_l + bh * P;
    const float *po = a.part_o + bh * P * D;

    __shared__ float red_m[kWaves];
    __shared__ float red_l[kWaves];
    __shared__ float red_o[kWaves][D];

    // m* = max over partials that hold keys (l_j > 0)
    float mx = -__builtin_huge_valf();
    for (int j = tid; j < P; j += kThreads) {
        const float mj = pm[j];
        if (pl[j] > 0.f) mx = fmaxf(mx, mj);
    }
    mx = wave_max(mx);
    if (lane == 0) red_m[w] = mx;
    __syncthreads();
    float mstar = red_m[0];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) mstar = fmaxf(mstar, red_m[ww]);

    if (mstar == -__builtin_huge_valf()) {   // no key anywhere: defined as out = 0, lse = -inf
        if (tid < D) {
            if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[bh * D + tid] = 0;
            else reinterpret_cast<float *>(a.out)[bh * D + tid] = 0.f;
        }
        if (tid == 0) a.lse[bh] = -__builtin_huge_valf();
        return;
    }

    // weighted sums; wave w takes partials j = w, w+4, ...; UN rows are
    // fetched before any is consumed so their latencies overlap
    constexpr int UN = 8;
    float acc[CPL] = {};
    float lsum = 0.f;
    for (int j0 = w; j0 < P; j0 += kWaves * UN) {
        float x[UN][CPL];
        float wj[UN], lj[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const int j = j0 + i * kWaves;
            const bool ok = j < P;
            const int jj = ok ? j : w;          // any valid row; its weight is 0
            lj[i] = pl[jj];                     // wave-uniform scalar loads
            const float mj = pm[jj];
            wj[i] = (ok && lj[i] > 0.f) ? exp2_hw((mj - mstar) * kLog2eF) : 0.f;
            const float *row = po + (int64_t)jj * D + lane * CPL;
            if constexpr (CPL == 2) {
                const float2 v = *reinterpret_cast<const float2 *>(row);
                x[i][0] = v.x;
                x[i][1] = v.y;
            } else {
                x[i][0] = row[0];
            }
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            lsum = fmaf(wj[i], lj[i], lsum);
#pragma unroll
            for (int e = 0; e < CPL; ++e) acc[e] = fmaf(wj[i], x[i][e], acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < CPL; ++e) red_o[w][lane * CPL + e] = acc[e];
    if (lane == 0) red_l[w] = lsum;
    __syncthreads();

    float lstar = 0.f;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) lstar += red_l[ww];
    if (tid < D) {
        float o = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) o += red_o[ww][tid];
        const float z = o / lstar;
        if (a.out_dtype == TA_BF16) reinterpret_cast<unsigned short *>(a.out)[bh * D + tid] = f32_to_bf16_rne(z);
        else reinterpret_cast<float *>(a.out)[bh * D + tid] = z;
    }
    if (tid == 0) a.lse[bh] = mstar + logf(lstar);
}

}  // namespace

hipError_t launch_tree_combine(const CombineArgs &a, int d, hipStream_t s) {
    const dim3 grid((uint32_t)((int64_t)a.B * a.Hq));
    if (d == 128) hipLaunchKernelGGL((tree_combine_kernel<128>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((tree_combine_kernel<64>), grid, dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace ta
