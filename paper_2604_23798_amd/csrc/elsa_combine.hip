// Cross-block combine (second pass of split-KV) and the device layout probe.
#include "elsa_common.hpp"

namespace elsa {

// out = W/S of part_0 (+) ... (+) part_{C-1}  (Prop. 1).  The chunks are taken eight at a time:
// the 8 x (m, S, W) loads of a group are independent and in flight together, the group's maximum
// joins the running one, the running (S, W) is re-anchored (Eq. 3) and every chunk of the group
// enters with weight e^{m_c - m} <= 1.  Up to eight chunks this is the plain two-pass form
// (maximum first, then the weighted sums).  One thread owns four value columns of one query row;
// the d/4 threads of a row recompute the weights, which is cheap next to the part_W traffic.
// HBM-bound: reads C*(d+2) floats and writes d values per row.
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(CombineParams p) {
    constexpr int QPR = D / 4;
    constexpr int G = 8;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long row = idx / QPR;
    const int c4 = (int)(idx % QPR);
    if (row >= p.rows) return;
    const long long bh = row / p.n;
    const int i = (int)(row % p.n);
    const int C = p.num_splits;
    const float unit = p.m_natural ? kLog2e : 1.f;
    const long long base = bh * C * (long long)p.n + i;     // + c*n per chunk

    float m = -INFINITY, S = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < C; c0 += G) {
        float mc[G], Sc[G];
        f32x4 wv[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            // a group that sticks out of the chunk list re-reads the last chunk with weight zero
            const long long pr = base + (long long)min(c0 + g, C - 1) * p.n;
            mc[g] = p.part_m[pr];
            Sc[g] = p.part_S[pr];
            wv[g] = Io<float>::load4(p.part_W, pr * D + 4 * c4);
            if (c0 + g >= C) mc[g] = -INFINITY;
        }
        float mnew = m;
#pragma unroll
        for (int g = 0; g < G; ++g) mnew = fmaxf(mnew, mc[g]);
        const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
        const float keep = exp2_fast((m - msafe) * unit);       // 0 for the first group (m = -inf)
        S *= keep;
        acc *= keep;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float wgt = exp2_fast((mc[g] - msafe) * unit);
            S += Sc[g] * wgt;
            acc += wv[g] * wgt;
        }
        m = mnew;
    }
    const float msafe = (m == -INFINITY) ? 0.f : m;
    const float f = S > 0.f ? 1.f / S : 0.f;
    acc *= f;
    if (p.lse && c4 == 0) p.lse[row] = lse_of(msafe * unit, S);
    if (p.f16_out) Io<_Float16>::store4(p.out, row * D + 4 * c4, acc);
    else Io<float>::store4(p.out, row * D + 4 * c4, acc);
}

int launch_combine(const CombineParams &p, int d, hipStream_t s) {
    const long long threads = p.rows * (d / 4);
    const long long blocks = (threads + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    if (d == 32) hipLaunchKernelGGL(combine_kernel<32>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else if (d == 64) hipLaunchKernelGGL(combine_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else if (d == 96) hipLaunchKernelGGL(combine_kernel<96>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else if (d == 128) hipLaunchKernelGGL(combine_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else if (d == 256) hipLaunchKernelGGL(combine_kernel<256>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

// Layout probe: one wave reports where v_mfma_f32_32x32x2_f32 puts rows and columns of
// its result and what v_permlane32_swap returns, so a test can check the operand maps
// the forward kernel is built on.  out: 5 * 16 * 64 floats.
//   [0] C[m][n] for A[m][k] = (k==0)*(m+1), B[k][n] = (k==0)          -> row index + 1
//   [1] C[m][n] for A[m][k] = (k==0),       B[k][n] = (k==0)*(n+1)    -> column index + 1
//   [2] C[m][n] for A[m][k] = (k==1),       B[k][n] = (k==1)          -> all ones iff k = lane/32
//   [3] register 0: half_max(lane), register 1: half_sum(lane)
//   [4] register 0: 2^(-lane/8) from the hardware exp2
__global__ __launch_bounds__(64) void probe_kernel(float *out) {
    const int l = threadIdx.x, j = l & 31, h = l >> 5;
    f32x16 z;
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    f32x16 r0 = __builtin_amdgcn_mfma_f32_32x32x2f32(h == 0 ? (float)(j + 1) : 0.f, h == 0 ? 1.f : 0.f, z, 0, 0, 0);
    f32x16 r1 = __builtin_amdgcn_mfma_f32_32x32x2f32(h == 0 ? 1.f : 0.f, h == 0 ? (float)(j + 1) : 0.f, z, 0, 0, 0);
    f32x16 r2 = __builtin_amdgcn_mfma_f32_32x32x2f32(h == 1 ? 1.f : 0.f, h == 1 ? 1.f : 0.f, z, 0, 0, 0);
    for (int i = 0; i < 16; ++i) {
        out[(0 * 16 + i) * 64 + l] = r0[i];
        out[(1 * 16 + i) * 64 + l] = r1[i];
        out[(2 * 16 + i) * 64 + l] = r2[i];
        out[(3 * 16 + i) * 64 + l] = 0.f;
        out[(4 * 16 + i) * 64 + l] = 0.f;
    }
    out[(3 * 16 + 0) * 64 + l] = half_max((float)l);
    out[(3 * 16 + 1) * 64 + l] = half_sum((float)l);
    out[(4 * 16 + 0) * 64 + l] = exp2_fast(-(float)l / 8.f);
}

int launch_probe(float *out, hipStream_t s) {
    hipLaunchKernelGGL(probe_kernel, dim3(1), dim3(64), 0, s, out);
    return (int)hipGetLastError();
}

}  // namespace elsa
