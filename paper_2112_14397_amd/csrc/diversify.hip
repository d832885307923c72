// Expert-diversify (EvoMoE Stage 1; Algorithm 1's loop  e_i <- diversify(e, i)): the N experts of a layer are
// spawned from the one shared expert by setting a random part of its weights to 0, a different part per expert.
// The paper fixes neither the masked fraction (an argument here) nor the random source; this build draws from a
// counter-based generator so that a CPU implementation can draw the same numbers: weight number j of tensor t
// (0 = W1, 1 = W2) of expert i uses output number (t << 62 | i << 48 | j) of the SplitMix64 sequence seeded with
// `seed` and is masked when the top 24 bits of that output are below floor(ratio * 2^24).  Biases are copied.
// One pass: every 16-byte vector of the shared matrix is read once and written E times.
#include "kernels.h"

namespace evomoe {

__device__ __forceinline__ uint64_t splitmix64_output(uint64_t seed, uint64_t n) {
    uint64_t z = seed + (n + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Both weight matrices have d*F elements; blockIdx.y = tensor (0 = W1, 1 = W2).
template <typename TX>
__global__ __launch_bounds__(256) void diversify_kernel(const TX* __restrict__ W1s, const TX* __restrict__ W2s,
                                                        int64_t n_weights, int E, uint64_t seed, uint32_t limit,
                                                        TX* __restrict__ W1, TX* __restrict__ W2)
{
    constexpr int KV = Elem<TX>::kVec;
    const int tensor = blockIdx.y;
    const TX* src = tensor ? W2s : W1s;
    TX* dst = tensor ? W2 : W1;
    const int64_t nvec = n_weights / KV;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * 256) {
        float w[KV];
        Elem<TX>::load_vec(src + v * KV, w);
        for (int e = 0; e < E; ++e) {
            const uint64_t base = ((uint64_t)tensor << 62) | ((uint64_t)e << 48) | (uint64_t)(v * KV);
            float o[KV];
#pragma unroll
            for (int q = 0; q < KV; ++q)
                o[q] = (uint32_t)(splitmix64_output(seed, base + q) >> 40) >= limit ? w[q] : 0.f;
            Elem<TX>::store_vec(dst + (int64_t)e * n_weights + v * KV, o);
        }
    }
}

// b[e, :] = b_shared for every expert (either bias may be absent)
__global__ __launch_bounds__(256) void diversify_bias_kernel(const float* __restrict__ b1s, const float* __restrict__ b2s,
                                                             int F, int d, int E, float* __restrict__ b1,
                                                             float* __restrict__ b2)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (b1s && b1 && i < E * F) b1[i] = b1s[i % F];
    if (b2s && b2 && i < E * d) b2[i] = b2s[i % d];
}

hipError_t launch_diversify(const Ctx& c, const evomoe_shape& s, const void* W1s, const float* b1s, const void* W2s,
                            const float* b2s, uint64_t seed, float mask_ratio, void* W1, float* b1, void* W2,
                            float* b2) {
    const int64_t n = (int64_t)s.d * s.F;
    const uint32_t limit = (uint32_t)floor((double)mask_ratio * 16777216.0);
    const int kv = s.dtype == EVOMOE_BF16 ? 8 : 4;
    const int64_t want = (n / kv + 255) / 256, cap = (int64_t)c.num_cu * 8;
    const dim3 grid((unsigned)(want < cap ? want : cap), 2);
    ProfScope ps(c, EVOMOE_K_DIVERSIFY);
    if (s.dtype == EVOMOE_BF16)
        hipLaunchKernelGGL(diversify_kernel<bf16_t>, grid, dim3(256), 0, c.stream, (const bf16_t*)W1s,
                           (const bf16_t*)W2s, n, s.E, seed, limit, (bf16_t*)W1, (bf16_t*)W2);
    else
        hipLaunchKernelGGL(diversify_kernel<float>, grid, dim3(256), 0, c.stream, (const float*)W1s,
                           (const float*)W2s, n, s.E, seed, limit, (float*)W1, (float*)W2);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if ((b1s && b1) || (b2s && b2)) {
        const int m = s.E * (s.F > s.d ? s.F : s.d);
        hipLaunchKernelGGL(diversify_bias_kernel, dim3((m + 255) / 256), dim3(256), 0, c.stream, b1s, b2s, s.F, s.d,
                           s.E, b1, b2);
        err = hipGetLastError();
    }
    return err;
}

}  // namespace evomoe
