// Combine and its backward (EvoMoE Eq. moe_weighted_sum_problem; Algorithm 1's accumulation
// y_s += G_{s,id} * e_id(x_s)).  Pure HBM streaming: 16-byte vector accesses, f32 accumulation,
// fixed (ascending expert) summation order.
#include "kernels.h"

namespace evomoe {

template <typename TX>
__global__ __launch_bounds__(256) void combine_kernel(
    const TX* __restrict__ O, const float* __restrict__ pair_gate, const int32_t* __restrict__ tok_off,
    const int32_t* __restrict__ tok_rows, int T, int d, int64_t P_cap, TX* __restrict__ y)
{
    constexpr int KV = Elem<TX>::kVec;
    const int vpr = d / KV;
    const int64_t total = (int64_t)T * vpr;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int t = (int)(i / vpr), v = (int)(i % vpr);
        int64_t j0 = tok_off[t], j1 = tok_off[t + 1];
        if (j1 > P_cap) j1 = P_cap;
        float acc[KV];
#pragma unroll
        for (int q = 0; q < KV; ++q) acc[q] = 0.f;
        // four rows at a time: indices, then weights and vectors, are loaded together; added in ascending
        // expert order
        for (int64_t j = j0; j < j1; j += 4) {
            int r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = tok_rows[j + u < j1 ? j + u : j1 - 1];
            float g[4], val[4][KV];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                g[u] = pair_gate[r[u]];
                Elem<TX>::load_vec(O + (size_t)r[u] * d + v * KV, val[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j + u < j1) {
#pragma unroll
                    for (int q = 0; q < KV; ++q) acc[q] += g[u] * val[u][q];
                }
        }
        Elem<TX>::store_vec(y + (size_t)t * d + v * KV, acc);
    }
}

hipError_t launch_combine(const Ctx& c, const evomoe_shape& s, const void* O, const float* pair_gate,
                          const int32_t* tok_off, const int32_t* tok_rows, void* y) {
    const int kv = s.dtype == EVOMOE_BF16 ? 8 : 4;
    const int64_t total = (int64_t)s.T * (s.d / kv);
    const int64_t want = (total + 255) / 256, cap = (int64_t)c.num_cu * 16;
    const int blocks = (int)(want < cap ? want : cap);
    ProfScope ps(c, EVOMOE_K_COMBINE);
    if (s.dtype == EVOMOE_BF16)
        hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(blocks), dim3(256), 0, c.stream,
                           (const bf16_t*)O, pair_gate, tok_off, tok_rows, s.T, s.d, s.P_cap, (bf16_t*)y);
    else
        hipLaunchKernelGGL(combine_kernel<float>, dim3(blocks), dim3(256), 0, c.stream,
                           (const float*)O, pair_gate, tok_off, tok_rows, s.T, s.d, s.P_cap, (float*)y);
    return hipGetLastError();
}

// One wave per row r:  dO[r,:] = G_r * dy[s(r),:],  dG_r = <dy[s(r),:], O[r,:]>.
template <typename TX>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const TX* __restrict__ dy, const TX* __restrict__ O, const float* __restrict__ pair_gate,
    const int32_t* __restrict__ pair_token, const int32_t* __restrict__ expert_offsets, int E, int d,
    int64_t P_cap, TX* __restrict__ dO, float* __restrict__ dG)
{
    constexpr int KV = Elem<TX>::kVec;
    const int P = clamp_pairs(expert_offsets[E], P_cap);
    const int lane = threadIdx.x & 63;
    const int wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * 4;
    const int vpr = d / KV;
    for (int r = wave_global; r < P; r += nwaves) {
        const int s = pair_token[r];
        const float g = pair_gate[r];
        float dot = 0.f;
        for (int v = lane; v < vpr; v += 64) {
            float a[KV], o[KV], out[KV];
            Elem<TX>::load_vec(dy + (size_t)s * d + v * KV, a);
            Elem<TX>::load_vec(O + (size_t)r * d + v * KV, o);
#pragma unroll
            for (int q = 0; q < KV; ++q) {
                dot += a[q] * o[q];
                out[q] = g * a[q];
            }
            Elem<TX>::store_vec(dO + (size_t)r * d + v * KV, out);
        }
        dot = wave_sum(dot);
        if (lane == 0) dG[r] = dot;
    }
}

hipError_t launch_combine_bwd(const Ctx& c, const evomoe_shape& s, const void* dy, const void* O,
                              const float* pair_gate, const int32_t* pair_token,
                              const int32_t* expert_offsets, void* dO, float* dG_pairs) {
    const int64_t want = (s.P_cap + 3) / 4, cap = (int64_t)c.num_cu * 16;
    const int blocks = (int)(want < cap ? want : cap);
    ProfScope ps(c, EVOMOE_K_COMBINE_BWD);
    if (s.dtype == EVOMOE_BF16)
        hipLaunchKernelGGL(combine_bwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, c.stream,
                           (const bf16_t*)dy, (const bf16_t*)O, pair_gate, pair_token, expert_offsets,
                           s.E, s.d, s.P_cap, (bf16_t*)dO, dG_pairs);
    else
        hipLaunchKernelGGL(combine_bwd_kernel<float>, dim3(blocks), dim3(256), 0, c.stream,
                           (const float*)dy, (const float*)O, pair_gate, pair_token, expert_offsets,
                           s.E, s.d, s.P_cap, (float*)dO, dG_pairs);
    return hipGetLastError();
}

}  // namespace evomoe
