// DTS gate, forward and backward (EvoMoE Stage 2: Eq. gumbel_softmax, Eq. adaptive_sparsity, Algorithm 2).
//
// Forward: logits on the matrix cores with float32-exact products (f32 MFMA for a float32 layer, three
// bf16 MFMAs against a hi/mid/lo split of W_g for a bf16 layer: a selection decided by g' > c must not
// move), + bias + Gumbel noise, temperature softmax,
// strict threshold with the arg-max fallback, bit mask, per-token k, and the per-expert histogram
// (integer atomics into counts[E] and, if asked for, into the per-256-token histograms the dispatch
// starts from; both are cleared by gate_prep_kernel right before).
#include <type_traits>

#include "kernels.h"

namespace evomoe {

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
// Common tail of the gate kernels.  In: per-wave partial logit tiles acc[rt][n] (MFMA 16x16 layout:
// element r of lane (q = lane/16, i16 = lane%16) is token row 4q+r, expert column 16n+i16).
// Adds the four waves' tiles in wave order (fixed order => reproducible bits), then 16/RT threads per
// token apply bias, noise, temperature softmax, the strict threshold and the arg-max fallback, write
// g', weights, mask and k, and add the block's per-expert counts to counts[E] and to the histogram row of the
// 256-token group the block lies in (integer atomics: the sums do not depend on their order).
template <int NE, int RT>
__device__ __forceinline__ void gate_finish(
    f32x4 (&acc)[RT][NE], const float* __restrict__ bg, const float* __restrict__ noise, float tau, float c,
    int T, int E, float* __restrict__ gprime, float* __restrict__ gate_w, uint64_t* __restrict__ mask_bits,
    int32_t* __restrict__ k_per_token, int32_t* __restrict__ counts, int32_t* __restrict__ block_hist)
{
    constexpr int TPB = 16 * RT;           // tokens per block (divides kDispatchTokens)
    constexpr int EP = 16 * NE;            // experts padded to MFMA tiles
    constexpr int LDZ = EP + 4;            // LDS row stride (bank-conflict-free tile writes)
    constexpr int TPT = 256 / TPB;         // threads per token in the softmax phase
    constexpr int EPT = EP / TPT;          // experts per thread there
    __shared__ float zsum[TPB * LDZ];
    __shared__ int cnt[64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, q = lane >> 4;
    const int t0 = blockIdx.x * TPB;

    if (tid < 64) cnt[tid] = 0;
    // add the four waves' partial tiles in wave order (fixed order => reproducible bits)
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int n = 0; n < NE; ++n)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int idx = (rt * 16 + 4 * q + r) * LDZ + n * 16 + i16;
                        const float v = acc[rt][n][r];
                        zsum[idx] = (w == 0) ? v : zsum[idx] + v;
                    }
        }
        __syncthreads();
    }

    // ---- softmax / threshold: TPT threads per token ----
    const int tl = tid / TPT, sub = tid % TPT;
    const int t = t0 + tl;
    const bool tok_ok = t < T;
    float a[EPT];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int e = sub + j * TPT;
        float z = -INFINITY;
        if (tok_ok && e < E) {
            z = zsum[tl * LDZ + e];
            if (bg) z += bg[e];
            if (noise) z += noise[(size_t)t * E + e];
            z = z / tau;
        }
        a[j] = z;
        m = fmaxf(m, z);
    }
#pragma unroll
    for (int o = TPT >> 1; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float ssum = 0.f;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int e = sub + j * TPT;
        a[j] = (tok_ok && e < E) ? expf(a[j] - m) : 0.f;
        ssum += a[j];
    }
#pragma unroll
    for (int o = TPT >> 1; o > 0; o >>= 1) ssum += __shfl_xor(ssum, o, 64);

    uint64_t bits = 0;
    float best = -1.f;
    int best_e = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int e = sub + j * TPT;
        const float g = a[j] / ssum;
        a[j] = g;
        if (tok_ok && e < E) {
            if (g > c) bits |= (1ull << e);
            if (g > best) { best = g; best_e = e; }   // ascending e: keeps the lowest index on ties
        }
    }
#pragma unroll
    for (int o = TPT >> 1; o > 0; o >>= 1) {
        bits |= __shfl_xor(bits, o, 64);
        const float ob = __shfl_xor(best, o, 64);
        const int oe = __shfl_xor(best_e, o, 64);
        if (ob > best || (ob == best && oe < best_e)) { best = ob; best_e = oe; }
    }
    if (best_e > 63) best_e = 0;                        // no comparable score at all (a row of NaNs): expert 0
    if (tok_ok && bits == 0) bits = 1ull << best_e;     // Algorithm 2: len(id_s) >= 1

    if (tok_ok) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int e = sub + j * TPT;
            if (e < E) {
                const bool sel = (bits >> e) & 1ull;
                gprime[(size_t)t * E + e] = a[j];
                if (gate_w) gate_w[(size_t)t * E + e] = sel ? a[j] : 0.f;
                if (sel) atomicAdd(&cnt[e], 1);
            }
        }
        if (sub == 0) {
            mask_bits[t] = bits;
            if (k_per_token) k_per_token[t] = __popcll(bits);
        }
    }
    __syncthreads();

    // ---- per-expert histogram ----
    if (tid < E && cnt[tid]) {
        atomicAdd(&counts[tid], cnt[tid]);
        if (block_hist) atomicAdd(&block_hist[(size_t)(t0 / kDispatchTokens) * E + tid], cnt[tid]);
    }
}

// float32 layer: logits with v_mfma_f32_16x16x4_f32 (exact float32 products).  Block = 4 waves; the
// block owns 16*RT consecutive tokens; each wave takes every 4th K-slab of all of them.
template <typename TX, int NE, int RT>
__global__ __launch_bounds__(256) void dts_gate_kernel(
    const TX* __restrict__ x, const float* __restrict__ Wg, const float* __restrict__ bg,
    const float* __restrict__ noise, float tau, float c, int T, int d, int E,
    float* __restrict__ gprime, float* __restrict__ gate_w, uint64_t* __restrict__ mask_bits,
    int32_t* __restrict__ k_per_token, int32_t* __restrict__ counts, int32_t* __restrict__ block_hist)
{
    constexpr int KV = Elem<TX>::kVec;     // k's per 16-byte load
    constexpr int KB = 4 * KV;             // k's per slab (4 lane groups x KV)
    constexpr int TPB = 16 * RT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, q = lane >> 4;
    const int t0 = blockIdx.x * TPB;

    f32x4 acc[RT][NE];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int n = 0; n < NE; ++n) acc[rt][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kb = wave * KB; kb < d; kb += 4 * KB) {
        const int k0 = kb + q * KV;            // this lane group's first k
        float a[RT][KV];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int t = t0 + rt * 16 + i16;
            if (t < T && k0 < d) {
                Elem<TX>::load_vec(x + (size_t)t * d + k0, a[rt]);
            } else {
#pragma unroll
                for (int j = 0; j < KV; ++j) a[rt][j] = 0.f;
            }
        }
#pragma unroll
        for (int j = 0; j < KV; ++j) {
            const int k = k0 + j;
#pragma unroll
            for (int n = 0; n < NE; ++n) {
                const int e = n * 16 + i16;
                const float b = (k < d && e < E) ? Wg[(size_t)k * E + e] : 0.f;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[rt][j], b, acc[rt][n], 0, 0, 0);
            }
        }
    }
    gate_finish<NE, RT>(acc, bg, noise, tau, c, T, E, gprime, gate_w, mask_bits, k_per_token, counts, block_hist);
}

// bf16 layer.  x is exact in bf16, so W_g is split into three bf16 terms (hi + mid + lo carry all 24
// mantissa bits of the float32 weight) and the logits come from three v_mfma_f32_16x16x32_bf16 per 32 k's:
// every product is exact in float32 and the sum is accumulated in float32 -- the same accuracy as float32
// FMAs, at matrix-core rate.  gate_prep_kernel makes the split copy right before, in the order the gate kernel's
// lanes consume it: [k-block of 32][term][16-expert tile n][lane = 16 q + i16][8 k's], i.e. the B fragment of
// one MFMA (expert 16 n + i16, k = 32 kb + 8 q .. +7) is 1 KB of consecutive memory, and the twelve fragments of
// a k-block (E = 64) are 12 KB in a row: full cache lines, spread evenly over the L2 channels (rows of a plain
// transposed copy are 2 d bytes apart, and every block of the grid asks for the same sixteen of them at the
// same time).  Zero beyond E and beyond d.  The kernel also clears the integer sums the gate adds to
// (planes == null, float32 layer: clears only).
__global__ __launch_bounds__(256) void gate_prep_kernel(const float* __restrict__ Wg, int d, int E, int NE,
                                                        uint16_t* __restrict__ planes, int32_t* __restrict__ counts,
                                                        int32_t* __restrict__ block_hist, int n_hist)
{
    const int i = blockIdx.x * 256 + threadIdx.x;          // over nkb * NE * 512 elements of one term, destination order
    if (i < E) counts[i] = 0;
    if (block_hist && i < n_hist) block_hist[i] = 0;
    const int nkb = (d + 31) / 32;
    if (!planes || i >= nkb * NE * 512) return;
    const int j = i & 7, lane = (i >> 3) & 63, n = (i >> 9) % NE, kb = (i >> 9) / NE;
    const int e = n * 16 + (lane & 15), k = kb * 32 + (lane >> 4) * 8 + j;
    const float w = (e < E && k < d) ? Wg[(size_t)k * E + e] : 0.f;
    const uint32_t hi = f32_to_bf16_bits(w);
    const float r1 = w - bf16_bits_to_f32(hi);
    const uint32_t mid = f32_to_bf16_bits(r1);
    const float r2 = r1 - bf16_bits_to_f32(mid);
    const uint32_t lo = f32_to_bf16_bits(r2);
    // element (kb, term, n, lane, j)
    const size_t base = ((size_t)kb * 3 * NE + n) * 512 + (size_t)lane * 8 + j;
    planes[base] = (uint16_t)hi;
    planes[base + (size_t)NE * 512] = (uint16_t)mid;
    planes[base + (size_t)2 * NE * 512] = (uint16_t)lo;
}

template <int NE, int RT>
__global__ __launch_bounds__(256) void dts_gate_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ planes, const float* __restrict__ bg,
    const float* __restrict__ noise, float tau, float c, int T, int d, int E,
    float* __restrict__ gprime, float* __restrict__ gate_w, uint64_t* __restrict__ mask_bits,
    int32_t* __restrict__ k_per_token, int32_t* __restrict__ counts, int32_t* __restrict__ block_hist)
{
    constexpr int TPB = 16 * RT, EP = 16 * NE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, q = lane >> 4;
    const int t0 = blockIdx.x * TPB;
    f32x4 acc[RT][NE];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int n = 0; n < NE; ++n) acc[rt][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bf16x8 zero8 = {};
    // k-blocks of 32, dealt round-robin to the four waves; lane group q holds k = 32*kb + 8q .. +7.
    // XU k-blocks per round: their x fragments are fetched together (one trip to memory per round), and the
    // W_g terms of the next k-block are fetched while the current one multiplies.
    constexpr int XU = RT * NE >= 8 ? 2 : (RT * NE >= 4 ? 4 : 8);
    auto load_planes = [&](int kb, bf16x8 (&b)[NE][3]) {
        const bool kok = kb * 32 < d;
        const bf16_t* wp = planes + ((size_t)(kok ? kb : 0) * 3 * NE) * 512 + lane * 8;
#pragma unroll
        for (int n = 0; n < NE; ++n)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                b[n][pl] = kok ? *reinterpret_cast<const bf16x8*>(wp + (pl * NE + n) * 512) : zero8;
    };
    for (int kb0 = wave; kb0 * 32 < d; kb0 += 4 * XU) {
        bf16x8 a[XU][RT];
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int k0 = (kb0 + 4 * u) * 32 + q * 8;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int t = t0 + rt * 16 + i16;
                a[u][rt] = (k0 < d && t < T) ? *reinterpret_cast<const bf16x8*>(x + (size_t)t * d + k0) : zero8;
            }
        }
        bf16x8 b[2][NE][3];
        load_planes(kb0, b[0]);
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            if (u + 1 < XU) load_planes(kb0 + 4 * (u + 1), b[(u + 1) & 1]);
#pragma unroll
            for (int n = 0; n < NE; ++n)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    acc[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][rt], b[u & 1][n][2], acc[rt][n], 0, 0, 0);
                    acc[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][rt], b[u & 1][n][1], acc[rt][n], 0, 0, 0);
                    acc[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][rt], b[u & 1][n][0], acc[rt][n], 0, 0, 0);
                }
        }
    }
    gate_finish<NE, RT>(acc, bg, noise, tau, c, T, E, gprime, gate_w, mask_bits, k_per_token, counts, block_hist);
}

static int pick_rt(const Ctx& c, const evomoe_shape& s) {
    // as many tokens per block as still leaves a block for every compute unit (the W_g terms are read once per
    // block, and fewer blocks leave fewer partial histograms to add up)
    for (int rt = 4; rt > 1; rt >>= 1)
        if ((s.T + 16 * rt - 1) / (16 * rt) >= c.num_cu) return rt;
    return 1;
}


template <typename TX, int NE, int RT>
static hipError_t gate_launch_t(const Ctx& c, const evomoe_shape& s, const void* x, const float* Wg,
                                const float* bg, const float* noise, float tau, float thr,
                                float* gprime, float* gate_w, uint64_t* mask_bits, int32_t* counts,
                                int32_t* k_per_token, int32_t* block_hist) {
    const int blocks = (s.T + 16 * RT - 1) / (16 * RT);
    const int n_hist = dispatch_blocks(s) * s.E;
    ProfScope ps(c, EVOMOE_K_GATE);
    if constexpr (std::is_same<TX, bf16_t>::value) {
        const int n_split = (s.d + 31) / 32 * NE * 512;
        const int n = n_split > n_hist ? n_split : n_hist;
        hipLaunchKernelGGL(gate_prep_kernel, dim3((n + 255) / 256), dim3(256), 0, c.stream, Wg, s.d, s.E, NE,
                           c.wg_planes, counts, block_hist, n_hist);
        hipLaunchKernelGGL((dts_gate_bf16_kernel<NE, RT>), dim3(blocks), dim3(256), 0, c.stream,
                           (const bf16_t*)x, (const bf16_t*)c.wg_planes, bg, noise, tau, thr, s.T, s.d, s.E,
                           gprime, gate_w, mask_bits, k_per_token, counts, block_hist);
    } else {
        const int n = n_hist > s.E ? n_hist : s.E;
        hipLaunchKernelGGL(gate_prep_kernel, dim3((n + 255) / 256), dim3(256), 0, c.stream, Wg, s.d, s.E, 0,
                           (uint16_t*)nullptr, counts, block_hist, n_hist);
        hipLaunchKernelGGL((dts_gate_kernel<TX, NE, RT>), dim3(blocks), dim3(256), 0, c.stream,
                           (const TX*)x, Wg, bg, noise, tau, thr, s.T, s.d, s.E, gprime, gate_w,
                           mask_bits, k_per_token, counts, block_hist);
    }
    return hipGetLastError();
}

template <typename TX, int NE>
static hipError_t gate_launch_rt(int rt, const Ctx& c, const evomoe_shape& s, const void* x,
                                 const float* Wg, const float* bg, const float* noise, float tau,
                                 float thr, float* gp, float* gw, uint64_t* mb, int32_t* cn, int32_t* kt, int32_t* bh) {
    switch (rt) {
        case 4: return gate_launch_t<TX, NE, 4>(c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
        case 2: return gate_launch_t<TX, NE, 2>(c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
        default: return gate_launch_t<TX, NE, 1>(c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
    }
}

template <typename TX>
static hipError_t gate_launch_ne(const Ctx& c, const evomoe_shape& s, const void* x, const float* Wg,
                                 const float* bg, const float* noise, float tau, float thr, float* gp,
                                 float* gw, uint64_t* mb, int32_t* cn, int32_t* kt, int32_t* bh) {
    const int rt = pick_rt(c, s);
    switch ((s.E + 15) / 16) {
        case 1: return gate_launch_rt<TX, 1>(rt, c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
        case 2: return gate_launch_rt<TX, 2>(rt, c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
        case 3: return gate_launch_rt<TX, 3>(rt, c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
        default: return gate_launch_rt<TX, 4>(rt, c, s, x, Wg, bg, noise, tau, thr, gp, gw, mb, cn, kt, bh);
    }
}

hipError_t launch_dts_gate(const Ctx& c, const evomoe_shape& s, const void* x, const float* Wg,
                           const float* bg, const float* noise, float tau, float threshold,
                           float* gprime, float* gate_w, uint64_t* mask_bits, int32_t* counts,
                           int32_t* k_per_token, int32_t* block_hist) {
    if (s.dtype == EVOMOE_BF16)
        return gate_launch_ne<bf16_t>(c, s, x, Wg, bg, noise, tau, threshold, gprime, gate_w,
                                      mask_bits, counts, k_per_token, block_hist);
    return gate_launch_ne<float>(c, s, x, Wg, bg, noise, tau, threshold, gprime, gate_w, mask_bits,
                                 counts, k_per_token, block_hist);
}

// ---------------------------------------------------------------------------------------------
// backward
// ---------------------------------------------------------------------------------------------
// dz_sj = (g'_sj / tau) * (dG_sj - sum_i dG_si g'_si).  EP lanes (a power of two >= E) work on one token, lane e
// on expert e: dG_se sits in row tok_rows[tok_off[s] + (number of selected experts below e)] (rows of a token
// are listed in ascending expert id); the inner product is a butterfly sum over the EP lanes (fixed order).
// coef (optional, [E]): a gradient with respect to g'_si that is the same for every token (the balance
// loss's), added to dG_si for every expert, selected or not, times coef_scale.
template <int EP>
__global__ __launch_bounds__(256) void gate_dz_kernel(
    const float* __restrict__ dG_pairs, const int32_t* __restrict__ tok_off,
    const int32_t* __restrict__ tok_rows, const float* __restrict__ gprime,
    const uint64_t* __restrict__ mask_bits, float tau, int T, int E, int64_t P_cap,
    const float* __restrict__ coef, float coef_scale, float* __restrict__ dz)
{
    constexpr int TPB = 256 / EP;
    const int e = threadIdx.x % EP, tl = threadIdx.x / EP;
    const int t = blockIdx.x * TPB + tl;
    const bool ok = t < T && e < E;
    float g = 0.f, dg = 0.f;
    if (ok) {
        const uint64_t bits = mask_bits[t];
        g = gprime[(size_t)t * E + e];
        if (coef) dg = coef_scale * coef[e];
        if ((bits >> e) & 1ull) {
            const int64_t slot = (int64_t)tok_off[t] + __popcll(bits & ((1ull << e) - 1ull));
            if (slot < P_cap) dg += dG_pairs[tok_rows[slot]];
        }
    }
    float inner = dg * g;
#pragma unroll
    for (int o = EP >> 1; o > 0; o >>= 1) inner += __shfl_xor(inner, o, 64);
    if (ok) dz[(size_t)t * E + e] = g / tau * (dg - inner);
}

// CPT consecutive elements of a row <-> floats, one vector access (CPT = 1, 2 or 4)
template <typename TX, int CPT> struct RowVec;
template <int CPT> struct RowVec<float, CPT> {
    __device__ static __forceinline__ void load(const float* p, float* o) {
        if (CPT == 4) { const f32x4 v = *reinterpret_cast<const f32x4*>(p); o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
        else if (CPT == 2) { const float2 v = *reinterpret_cast<const float2*>(p); o[0] = v.x; o[1] = v.y; }
        else o[0] = *p;
    }
    __device__ static __forceinline__ void store(float* p, const float* o) {
        if (CPT == 4) { const f32x4 v = {o[0], o[1], o[2], o[3]}; *reinterpret_cast<f32x4*>(p) = v; }
        else if (CPT == 2) { *reinterpret_cast<float2*>(p) = make_float2(o[0], o[1]); }
        else *p = o[0];
    }
};
// float32 layer.  One block = TC tokens x 256*CPT columns of x.  A thread owns CPT consecutive columns k: it keeps W_g[k,:]
// and a partial dWg[k,:] in registers and walks the chunk's tokens:
//   dx[s,k] += <dz[s,:], W_g[k,:]>,   dWg_part[k,:] += x[s,k] dz[s,:].
template <typename TX, int EP, int CPT>
__global__ __launch_bounds__(256) void gate_bwd_kernel(
    const float* __restrict__ dz, const TX* __restrict__ x, const float* __restrict__ Wg,
    int T, int d, int E, int TC, TX* __restrict__ dx, float* __restrict__ dWg_part,
    float* __restrict__ dbg_part)
{
    extern __shared__ float sdz[];          // [TC][EP], zero beyond E
    const int chunk = blockIdx.x;
    const int s0 = chunk * TC;
    const int ns = min(TC, T - s0);
    for (int i = threadIdx.x; i < ns * EP; i += 256) {
        const int s = i / EP, e = i % EP;
        sdz[i] = (e < E) ? dz[(size_t)(s0 + s) * E + e] : 0.f;
    }
    __syncthreads();
    if (blockIdx.y == 0 && threadIdx.x < E) {     // bias gradient partial: sum_s dz[s,e]
        float sb = 0.f;
        for (int s = 0; s < ns; ++s) sb += sdz[s * EP + threadIdx.x];
        dbg_part[(size_t)chunk * (d + 1) * E + threadIdx.x] = sb;
    }
    const int k = (blockIdx.y * 256 + threadIdx.x) * CPT;
    if (k >= d) return;
    float w[CPT][EP], g[CPT][EP];
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            w[c][e] = (e < E) ? Wg[(size_t)(k + c) * E + e] : 0.f;
            g[c][e] = 0.f;
        }
    // tokens in groups of UG: a group's loads of x and dx are issued together, one group ahead of the group
    // being multiplied (double buffer), so that their latency runs under the arithmetic
    constexpr int UG = CPT == 1 ? 8 : 4;
    float xv[2][UG][CPT], dxv[2][UG][CPT];
    auto load_group = [&](int sb, int buf) {
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            const int s = min(sb + u, ns - 1);
            const size_t off = (size_t)(s0 + s) * d + k;
            RowVec<TX, CPT>::load(x + off, xv[buf][u]);
            RowVec<TX, CPT>::load(dx + off, dxv[buf][u]);
        }
    };
    auto use_group = [&](int sb, int buf) {
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            const int s = sb + u;
            if (s < ns) {
                float acc[CPT];
#pragma unroll
                for (int c = 0; c < CPT; ++c) acc[c] = 0.f;
#pragma unroll
                for (int e4 = 0; e4 < EP; e4 += 4) {
                    const f32x4 z4 = *reinterpret_cast<const f32x4*>(&sdz[s * EP + e4]);
                    const float z[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int c = 0; c < CPT; ++c) {
                            acc[c] += z[q] * w[c][e4 + q];
                            g[c][e4 + q] += xv[buf][u][c] * z[q];
                        }
                }
#pragma unroll
                for (int c = 0; c < CPT; ++c) acc[c] += dxv[buf][u][c];
                RowVec<TX, CPT>::store(dx + (size_t)(s0 + s) * d + k, acc);
            }
        }
    };
    if (ns > 0) load_group(0, 0);
    for (int sb = 0; sb < ns; sb += 2 * UG) {
        if (sb + UG < ns) load_group(sb + UG, 1);
        use_group(sb, 0);
        if (sb + 2 * UG < ns) load_group(sb + 2 * UG, 0);
        if (sb + UG < ns) use_group(sb + UG, 1);
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < EP; ++e)
            if (e < E) dWg_part[((size_t)chunk * (d + 1) + k + c) * E + e] = g[c][e];
}

// ---- bf16 layer: both contractions of the gate backward on the matrix cores ------------------------------
//   dx[s,k]   += sum_e dz[s,e] W_g[k,e]      (M = tokens, N = columns of x, K = experts)
//   dWg[k,e]   = sum_s x[s,k] dz[s,e]        (M = columns of x, N = experts, K = tokens)
// with v_mfma_f32_32x32x16_bf16.  x is bf16 already; the float32 factors are split into bf16 terms so that the
// products stay (nearly) exact: dz = hi + mid + lo (all 24 mantissa bits; x dz is then exact, accumulated in
// float32), W_g = hi + lo, and dx takes the three leading products (relative error 2^-16, far below the bf16
// rounding of the stored dx).  Block = 4 waves = one run of tokens x 256 columns (64 per wave), walked in
// chunks of 32 tokens; the chunk's dz terms sit in LDS as [token][expert] and feed dx directly (expert-contiguous)
// and dWg through the transposing LDS read, as does the wave's x tile [token][column].
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kGbTok = 32;       // tokens per chunk
constexpr int kGbCols = 256;     // columns per block

struct GbPlan { int slices, tokens_per_block, nblk; };
GbPlan gate_bwd_mfma_plan(const evomoe_shape& s) {
    GbPlan p;
    p.slices = (s.d + kGbCols - 1) / kGbCols;
    int n = 512 / p.slices;                          // about two blocks per compute unit
    const int cap = s.T / s.E > 32 ? s.T / s.E : 32; // bounds the partial dWg tables by the size of x
    if (n > cap) n = cap;
    if (n > 256) n = 256;
    if (n < 1) n = 1;
    p.tokens_per_block = ((s.T + n - 1) / n + kGbTok - 1) / kGbTok * kGbTok;
    p.nblk = (s.T + p.tokens_per_block - 1) / p.tokens_per_block;
    return p;
}

__device__ __forceinline__ bf16x8 lds_read_tr(const unsigned char* q, int row_bytes) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q + 4 * row_bytes));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// KE = k-steps of 16 experts (dx), NE = tiles of 32 experts (dWg)
template <int KE, int NE>
__global__ __launch_bounds__(256, 2) void gate_bwd_mfma_kernel(
    const float* __restrict__ dz, const bf16_t* __restrict__ x, const float* __restrict__ Wg, int T, int d, int E,
    int tokens_per_block, bf16_t* __restrict__ dx, float* __restrict__ dWg_part, float* __restrict__ dbg_part)
{
    constexpr int EPL = 32 * NE;                     // experts per LDS row (zero beyond E)
    constexpr int DZN = kGbTok * EPL / 256;          // dz values per thread and chunk
    constexpr int PROW = EPL * 2, XROW = 128;        // LDS row bytes: dz terms, x tile
    constexpr int STG_LD = 64 + 4;
    __shared__ __align__(16) unsigned char planes[3][kGbTok * PROW];
    __shared__ __align__(16) unsigned char xt[4][kGbTok * XROW];
    __shared__ __align__(16) float stg[4][kGbTok * STG_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    const int blk = blockIdx.x, slice = blockIdx.y;
    const int c0 = slice * kGbCols + wave * 64;      // this wave's first column
    const int s_begin = blk * tokens_per_block, s_end = min(T, s_begin + tokens_per_block);
    const int nch = (s_end - s_begin + kGbTok - 1) / kGbTok;

    // W_g fragments of the dx product (B operand: k = expert, n = column), hi and lo terms, kept in registers
    bf16x8 whi[2][KE], wlo[2][KE];
#pragma unroll
    for (int jc = 0; jc < 2; ++jc) {
        const int col = min(c0 + jc * 32 + l32, d - 1);
#pragma unroll
        for (int ks = 0; ks < KE; ++ks)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int e = ks * 16 + kg * 8 + q;
                const float w = e < E ? Wg[(size_t)col * E + e] : 0.f;
                const bf16_t h = (bf16_t)w;
                whi[jc][ks][q] = h;
                wlo[jc][ks][q] = (bf16_t)(w - (float)h);
            }
    }
    f32x16 acc_w[2][NE];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NE; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_w[i][j][r] = 0.f;
    float sb = 0.f;                                  // bias gradient partial (slice 0, thread = expert)

    // global <-> thread mapping of a 32-token x 64-column wave tile: 8 lanes x 16 bytes per row, 8 rows per pass
    const int trow = lane >> 3, tcol = (lane & 7) * 8;
    const int gcol = min(c0 + tcol, d - 8);
    const bool col_ok = c0 + tcol < d;
    u32x4 xr[4], dxr[4];
    float dzr[DZN];
    auto load_x_dz = [&](int s0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int t = min(s0 + it * 8 + trow, T - 1);
            xr[it] = *reinterpret_cast<const u32x4*>(x + (size_t)t * d + gcol);
        }
#pragma unroll
        for (int u = 0; u < DZN; ++u) {
            const int i = tid + 256 * u, t = s0 + i / EPL, e = i % EPL;
            dzr[u] = (e < E && t < T) ? dz[(size_t)t * E + e] : 0.f;
        }
    };
    auto load_dx = [&](int s0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int t = min(s0 + it * 8 + trow, T - 1);
            dxr[it] = *reinterpret_cast<const u32x4*>(dx + (size_t)t * d + gcol);
        }
    };
    if (nch > 0) {
        load_x_dz(s_begin);
        load_dx(s_begin);
    }
    for (int ch = 0; ch < nch; ++ch) {
        const int s0 = s_begin + ch * kGbTok;
        __syncthreads();                             // the previous chunk's readers are done with the dz terms
#pragma unroll
        for (int u = 0; u < DZN; ++u) {
            const int i = tid + 256 * u;
            const float v = dzr[u];
            const bf16_t h = (bf16_t)v;
            const float r1 = v - (float)h;
            const bf16_t m = (bf16_t)r1;
            const bf16_t l = (bf16_t)(r1 - (float)m);
            reinterpret_cast<bf16_t*>(planes[0])[i] = h;
            reinterpret_cast<bf16_t*>(planes[1])[i] = m;
            reinterpret_cast<bf16_t*>(planes[2])[i] = l;
        }
#pragma unroll
        for (int it = 0; it < 4; ++it)
            *reinterpret_cast<u32x4*>(xt[wave] + (it * 8 + trow) * XROW + (lane & 7) * 16) = xr[it];
        if (ch + 1 < nch) load_x_dz(s0 + kGbTok);    // next chunk's loads run under this chunk's arithmetic
        __syncthreads();

        if (slice == 0 && tid < E) {
            for (int t = 0; t < kGbTok; ++t) {
                const int i = t * EPL + tid;
                sb += ((float)reinterpret_cast<const bf16_t*>(planes[0])[i] +
                       (float)reinterpret_cast<const bf16_t*>(planes[1])[i]) +
                      (float)reinterpret_cast<const bf16_t*>(planes[2])[i];
            }
        }
        // dWg partial: A = x^T (rows = columns of x, k = token), B = dz terms (k = token, n = expert)
#pragma unroll
        for (int ks = 0; ks < kGbTok / 16; ++ks) {
            bf16x8 xa[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                xa[i] = lds_read_tr(xt[wave] + (ks * 16 + kg * 8 + (s16 >> 2)) * XROW + (i * 2 + half) * 32 + (s16 & 3) * 8,
                                    XROW);
#pragma unroll
            for (int j = 0; j < NE; ++j)
#pragma unroll
                for (int pl = 2; pl >= 0; --pl) {
                    const bf16x8 zb = lds_read_tr(
                        planes[pl] + (ks * 16 + kg * 8 + (s16 >> 2)) * PROW + (j * 2 + half) * 32 + (s16 & 3) * 8, PROW);
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc_w[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[i], zb, acc_w[i][j], 0, 0, 0);
                }
        }
        // gate part of dx: A = dz terms (rows = tokens, k = expert), B = W_g terms
        f32x16 acc_x[2];
#pragma unroll
        for (int jc = 0; jc < 2; ++jc)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_x[jc][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KE; ++ks) {
            const int off = l32 * PROW + (ks * 16 + kg * 8) * 2;
            const bf16x8 zh = *reinterpret_cast<const bf16x8*>(planes[0] + off);
            const bf16x8 zm = *reinterpret_cast<const bf16x8*>(planes[1] + off);
#pragma unroll
            for (int jc = 0; jc < 2; ++jc) {
                acc_x[jc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zm, whi[jc][ks], acc_x[jc], 0, 0, 0);
                acc_x[jc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, wlo[jc][ks], acc_x[jc], 0, 0, 0);
                acc_x[jc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, whi[jc][ks], acc_x[jc], 0, 0, 0);
            }
        }
        // acc_x[jc][r] is (token 8*(r/4) + 4*kg + r%4, column jc*32 + l32): through LDS to row-major 16-byte pieces
#pragma unroll
        for (int jc = 0; jc < 2; ++jc)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                stg[wave][(8 * (r >> 2) + 4 * kg + (r & 3)) * STG_LD + jc * 32 + l32] = acc_x[jc][r];
        __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): this wave's LDS writes have landed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = it * 8 + trow;
            const f32x4 v0 = *reinterpret_cast<const f32x4*>(&stg[wave][row * STG_LD + tcol]);
            const f32x4 v1 = *reinterpret_cast<const f32x4*>(&stg[wave][row * STG_LD + tcol + 4]);
            const u32x4 o = dxr[it];
            u32x4 w;
            w.x = pack_bf16x2(v0.x + lo_bf16(o.x), v0.y + hi_bf16(o.x));
            w.y = pack_bf16x2(v0.z + lo_bf16(o.y), v0.w + hi_bf16(o.y));
            w.z = pack_bf16x2(v1.x + lo_bf16(o.z), v1.y + hi_bf16(o.z));
            w.w = pack_bf16x2(v1.z + lo_bf16(o.w), v1.w + hi_bf16(o.w));
            if (col_ok && s0 + row < s_end) *reinterpret_cast<u32x4*>(dx + (size_t)(s0 + row) * d + gcol) = w;
        }
        __builtin_amdgcn_wave_barrier();
        if (ch + 1 < nch) load_dx(s0 + kGbTok);
    }
    // acc_w[i][j][r] is (column c0 + i*32 + 8*(r/4) + 4*kg + r%4, expert j*32 + l32)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NE; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int col = c0 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3), e = j * 32 + l32;
                if (col < d && e < E) dWg_part[((size_t)blk * (d + 1) + col) * E + e] = acc_w[i][j][r];
            }
    if (slice == 0 && tid < E) dbg_part[(size_t)blk * (d + 1) * E + tid] = sb;
}

bool gate_bwd_use_mfma(const evomoe_shape& s) { return s.dtype == EVOMOE_BF16; }   // (d is a multiple of 8 there)

}  // namespace

// out[i] = sum over chunks of part[chunk][i], i < n0 + n1; the first n0 sums go to out0, the rest to out1 (or
// nowhere if out1 is null).  Four thread groups take a quarter of the chunks each (ascending, 16 independent loads
// in flight), then the four partial sums are added in group order.  Fixed order: reproducible.
__global__ __launch_bounds__(256) void sum_chunks_kernel(const float* __restrict__ part, int nchunk, size_t n0,
                                                         size_t n1, float* __restrict__ out0,
                                                         float* __restrict__ out1)
{
    __shared__ float red[4][64];
    const int o = threadIdx.x & 63, gq = threadIdx.x >> 6;
    const size_t n = n0 + n1;
    const size_t i = (size_t)blockIdx.x * 64 + o;
    const int per = (nchunk + 3) / 4;
    const int c_lo = gq * per, c_hi = min(nchunk, c_lo + per);
    float s = 0.f;
    if (i < n) {
        for (int c0 = c_lo; c0 < c_hi; c0 += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = (c0 + u < c_hi) ? part[(size_t)(c0 + u) * n + i] : 0.f;
#pragma unroll
            for (int u = 0; u < 16; ++u) s += v[u];
        }
    }
    red[gq][o] = s;
    __syncthreads();
    if (gq == 0 && i < n) {
        const float r = ((red[0][o] + red[1][o]) + red[2][o]) + red[3][o];
        if (i < n0) out0[i] = r;
        else if (out1) out1[i - n0] = r;
    }
}

static int gate_bwd_chunk_tokens(const evomoe_shape& s) {
    int tc = 32;
    while ((s.T + tc - 1) / tc > 256) tc *= 2;
    // LDS holds [TC][E rounded up to 16] floats; stay within 64 KB
    while ((size_t)tc * (((s.E + 15) / 16) * 16) * 4 > 60 * 1024 && tc > 16) tc /= 2;
    return tc;
}

size_t gate_bwd_workspace_bytes(const evomoe_shape& s) {
    const int tc = gate_bwd_chunk_tokens(s);
    size_t nchunk = (s.T + tc - 1) / tc;
    if (gate_bwd_use_mfma(s)) nchunk = gate_bwd_mfma_plan(s).nblk;
    return ((size_t)s.T * s.E + nchunk * ((size_t)s.d * s.E + s.E)) * sizeof(float);
}

template <typename TX>
static hipError_t gate_bwd_t(const Ctx& c, const evomoe_shape& s, const float* dz, const void* x,
                             const float* Wg, void* dx, float* dWg_part, float* dbg_part, int tc,
                             int nchunk) {
    const int ep = ((s.E + 15) / 16) * 16;
    const int cpt = ep == 16 ? 4 : ep == 32 ? 2 : 1;         // columns per thread (register budget: 2*CPT*EP)
    dim3 grid(nchunk, (s.d + 256 * cpt - 1) / (256 * cpt));
    const size_t lds = (size_t)tc * ep * sizeof(float);
#define EVOMOE_GB(EPV, CPTV)                                                                     \
    hipLaunchKernelGGL((gate_bwd_kernel<TX, EPV, CPTV>), grid, dim3(256), lds, c.stream, dz,     \
                       (const TX*)x, Wg, s.T, s.d, s.E, tc, (TX*)dx, dWg_part, dbg_part)
    if (ep == 16) EVOMOE_GB(16, 4);
    else if (ep == 32) EVOMOE_GB(32, 2);
    else if (ep == 48) EVOMOE_GB(48, 1);
    else EVOMOE_GB(64, 1);
#undef EVOMOE_GB
    return hipGetLastError();
}

hipError_t launch_dts_gate_bwd(const Ctx& c, const evomoe_shape& s, const float* dG_pairs,
                               const int32_t* tok_off, const int32_t* tok_rows, const float* gprime,
                               const uint64_t* mask_bits, float tau, const void* x, const float* Wg,
                               float* dWg, float* dbg, void* dx, void* workspace,
                               const float* dgprime_coef, float coef_scale) {
    const int tc = gate_bwd_chunk_tokens(s);
    const bool mfma = gate_bwd_use_mfma(s);
    const GbPlan plan = gate_bwd_mfma_plan(s);
    const int nchunk = mfma ? plan.nblk : (s.T + tc - 1) / tc;
    float* dz = (float*)workspace;
    float* dWg_part = dz + (size_t)s.T * s.E;
    float* dbg_part = dWg_part + (size_t)s.d * s.E;     // chunk c: [dWg partial: d x E][dbg partial: E], contiguous
    {
        ProfScope ps(c, EVOMOE_K_GATE_BWD_DZ);
#define EVOMOE_DZ(EPV)                                                                                   \
    hipLaunchKernelGGL(gate_dz_kernel<EPV>, dim3((s.T + 256 / EPV - 1) / (256 / EPV)), dim3(256), 0, c.stream,  \
                       dG_pairs, tok_off, tok_rows, gprime, mask_bits, tau, s.T, s.E, s.P_cap, dgprime_coef,     \
                       coef_scale, dz)
        if (s.E <= 4) EVOMOE_DZ(4);
        else if (s.E <= 8) EVOMOE_DZ(8);
        else if (s.E <= 16) EVOMOE_DZ(16);
        else if (s.E <= 32) EVOMOE_DZ(32);
        else EVOMOE_DZ(64);
#undef EVOMOE_DZ
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    {
        ProfScope ps(c, EVOMOE_K_GATE_BWD_MAIN);
        if (mfma) {
            const dim3 grid(plan.nblk, plan.slices);
#define EVOMOE_GBM(KEV, NEV)                                                                             \
    hipLaunchKernelGGL((gate_bwd_mfma_kernel<KEV, NEV>), grid, dim3(256), 0, c.stream, dz, (const bf16_t*)x, Wg, \
                       s.T, s.d, s.E, plan.tokens_per_block, (bf16_t*)dx, dWg_part, dbg_part)
            if (s.E <= 16) EVOMOE_GBM(1, 1);
            else if (s.E <= 32) EVOMOE_GBM(2, 1);
            else if (s.E <= 48) EVOMOE_GBM(3, 2);
            else EVOMOE_GBM(4, 2);
#undef EVOMOE_GBM
            err = hipGetLastError();
        } else {
            err = gate_bwd_t<float>(c, s, dz, x, Wg, dx, dWg_part, dbg_part, tc, nchunk);
        }
    }
    if (err != hipSuccess) return err;
    const size_t n0 = (size_t)s.d * s.E, n1 = (size_t)s.E;
    ProfScope ps(c, EVOMOE_K_GATE_BWD_REDUCE);
    hipLaunchKernelGGL(sum_chunks_kernel, dim3((n0 + n1 + 63) / 64), dim3(256), 0, c.stream, dWg_part, nchunk, n0,
                       n1, dWg, dbg);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Balance loss (Eq. balance_loss): L = alpha N sum_i (count_i / T^2) sum_s g'_si and dL/dg'_si.
// Pass 1: per-block column sums of g' (thread = (token lane, expert), fixed-order LDS reduction over the
// token lanes).  Pass 2 (one block): block partials summed in block order, then the E terms in expert order.
// ---------------------------------------------------------------------------------------------
constexpr int kBalanceTokensPerBlock = 128;
int balance_blocks(const evomoe_shape& s) { return (s.T + kBalanceTokensPerBlock - 1) / kBalanceTokensPerBlock; }

__global__ __launch_bounds__(256) void balance_colsum_kernel(const float* __restrict__ gprime, int T, int E,
                                                             float* __restrict__ partial)
{
    __shared__ float red[256];
    const int EP = E <= 4 ? 4 : E <= 8 ? 8 : E <= 16 ? 16 : E <= 32 ? 32 : 64;     // expert lanes (power of two)
    const int TL = 256 / EP;                                                        // token lanes
    const int e = threadIdx.x % EP, tl = threadIdx.x / EP;
    const int t0 = blockIdx.x * kBalanceTokensPerBlock;
    const int t1 = min(T, t0 + kBalanceTokensPerBlock);
    float acc = 0.f;
    if (e < E)
        for (int t = t0 + tl; t < t1; t += TL) acc += gprime[(size_t)t * E + e];
    red[threadIdx.x] = acc;
    __syncthreads();
    if (tl == 0 && e < E) {
        float sum = 0.f;
        for (int l = 0; l < TL; ++l) sum += red[l * EP + e];
        partial[(size_t)blockIdx.x * E + e] = sum;
    }
}

__global__ __launch_bounds__(64) void balance_final_kernel(const float* __restrict__ partial, int nblk, int T, int E,
                                                           const int32_t* __restrict__ counts, float alpha,
                                                           float* __restrict__ loss, float* __restrict__ coef)
{
    __shared__ float term[64];
    const int e = threadIdx.x;
    float colsum = 0.f, cf = 0.f;
    if (e < E) {
        // block order, eight loads in flight at a time (the order of the additions does not change)
        int b = 0;
        for (; b + 8 <= nblk; b += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(b + u) * E + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) colsum += v[u];
        }
        for (; b < nblk; ++b) colsum += partial[(size_t)b * E + e];
        cf = alpha * (float)E * ((float)counts[e] / ((float)T * (float)T));
        if (coef) coef[e] = cf;
    }
    term[e] = cf * colsum;
    __syncthreads();
    if (e == 0) {
        float L = 0.f;
        for (int i = 0; i < E; ++i) L += term[i];
        loss[0] = L;
    }
}

hipError_t launch_balance_loss(const Ctx& c, const evomoe_shape& s, const float* gprime, const int32_t* counts,
                               float alpha, float* loss, float* dgprime_coef) {
    const int nblk = balance_blocks(s);
    float* partial = reinterpret_cast<float*>(c.block_counts);
    ProfScope ps(c, EVOMOE_K_BALANCE_LOSS);
    hipLaunchKernelGGL(balance_colsum_kernel, dim3(nblk), dim3(256), 0, c.stream, gprime, s.T, s.E, partial);
    hipLaunchKernelGGL(balance_final_kernel, dim3(1), dim3(64), 0, c.stream, partial, nblk, s.T, s.E, counts, alpha,
                       loss, dgprime_coef);
    return hipGetLastError();
}

}  // namespace evomoe
