// Dispatch: variable-k permutation of the selected (token, expert) pairs (EvoMoE Algorithm 1: the
// per-token loop over id in id_s, regrouped by expert; no capacity limit, every selected pair is kept).
// A stable counting sort: rows are expert-major and token-ascending, computed with integer ballots and
// prefix sums only, so the indices are reproducible bit for bit.
#include "kernels.h"

namespace evomoe {

int dispatch_blocks(const evomoe_shape& s) { return (s.T + kDispatchTokens - 1) / kDispatchTokens; }

// Histogram table of the dispatch entry point that allocates nothing: device memory that exists from the moment
// the library is loaded, one copy per GPU.  Host code never passes this name to a kernel (on the host it is only
// a stand-in for the symbol); it asks the runtime once per device for the array's device address and uses that.
static __device__ __align__(256) int32_t scratch[kStaticHistEntries];
static int32_t* g_scratch_ptr[kMaxDevices];     // per device; null = not looked up yet

hipError_t static_hist_table(int device, int32_t** table) {
    *table = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;        // the lookup is made with that device current
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<int32_t*>(p);
    }
    *table = g_scratch_ptr[device];
    return hipSuccess;
}

// Pass 1: per-block (256 consecutive tokens) expert histogram from wave ballots.
__global__ __launch_bounds__(256) void dispatch_hist_kernel(
    const uint64_t* __restrict__ mask_bits, int T, int E, int32_t* __restrict__ block_counts)
{
    __shared__ int wc[4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x * kDispatchTokens + tid;
    const uint64_t valid = E >= 64 ? ~0ull : (1ull << E) - 1ull;      // bits of experts that do not exist are ignored
    const uint64_t bits = (t < T) ? (mask_bits[t] & valid) : 0ull;
    for (int e = 0; e < E; ++e) {
        const uint64_t bal = __ballot((bits >> e) & 1ull);
        if (lane == 0) wc[wave][e] = __popcll(bal);
    }
    __syncthreads();
    if (tid < E)
        block_counts[(size_t)blockIdx.x * E + tid] = wc[0][tid] + wc[1][tid] + wc[2][tid] + wc[3][tid];
}

// Pass 2: one thread per token.  Every block first derives, from the [nblk][E] histogram table, what it needs
// of the scan: the expert offsets (column totals, scanned over the experts) and, per expert, the number of
// selected tokens in the blocks before it -- integer sums, so the order of addition is free.  (The table is a
// few KB; reading it in every block is cheaper than a third launch for a serial scan.)  Then
// row of pair (t, e) = offset[e] + earlier blocks' tokens of e + selected tokens of e before t inside the
// block (wave ballots).  Writes pair_token / pair_gate at the row and the token's CSR; block 0 also writes
// the expert offsets, P and the capacity flag.
template <int EP>
__global__ __launch_bounds__(256) void dispatch_scatter_kernel(
    const uint64_t* __restrict__ mask_bits, const float* __restrict__ scores, int T, int E, int nblk,
    int64_t P_cap, const int32_t* __restrict__ block_counts, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ pair_token, float* __restrict__ pair_gate, int32_t* __restrict__ tok_off,
    int32_t* __restrict__ tok_rows, int64_t* __restrict__ num_pairs, int32_t* __restrict__ status)
{
    __shared__ uint64_t wbal[4][64]; // wave w's ballot of expert e
    __shared__ int wc[4][64];        // its population count
    __shared__ int wbase[4][64];     // first row of expert e's tokens that live in wave w of this block
    __shared__ int base[64];
    __shared__ int pre[64], tot[64], offs[65];
    __shared__ int wk[4];
    __shared__ int tok_base_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x * kDispatchTokens + tid;
    const uint64_t valid = E >= 64 ? ~0ull : (1ull << E) - 1ull;      // bits of experts that do not exist are ignored
    const uint64_t bits = (t < T) ? (mask_bits[t] & valid) : 0ull;
    const uint64_t lt = (1ull << lane) - 1ull;

    // ---- the block's share of the scan ----
    if (tid < 64) { pre[tid] = 0; tot[tid] = 0; }
    __syncthreads();
    {
        const int e = tid % EP, rl = tid / EP;
        int p = 0, a = 0;
        if (e < E)
            for (int b = rl; b < nblk; b += 256 / EP) {
                const int v = block_counts[(size_t)b * E + e];
                a += v;
                if (b < (int)blockIdx.x) p += v;
            }
        if (a) atomicAdd(&tot[e], a);
        if (p) atomicAdd(&pre[e], p);
    }
    // ballots of this wave's 64 tokens, expert by expert; lane e keeps expert e's
    uint64_t mybal = 0;
#pragma unroll
    for (int e = 0; e < EP; ++e) {
        const uint64_t bal = __ballot((bits >> e) & 1ull);
        if (lane == e) mybal = bal;
    }
    wbal[wave][lane] = mybal;
    wc[wave][lane] = __popcll(mybal);
    // exclusive scan of k over the block's tokens -> CSR offsets
    const int k = __popcll(bits);
    int incl = k;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wk[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int v = lane < E ? tot[lane] : 0, pv = lane < E ? pre[lane] : 0;
        int eincl = v, psum = pv;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int u = __shfl_up(eincl, o, 64);
            if (lane >= o) eincl += u;
            psum += __shfl_xor(psum, o, 64);
        }
        offs[lane + 1] = eincl;                      // offs[e + 1] = sum of the totals of experts 0..e
        if (lane == 0) { offs[0] = 0; tok_base_s = psum; }
        base[lane] = eincl - v + pv;
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if (tid <= E) expert_offsets[tid] = offs[tid];
        if (tid == 0) {
            const int64_t P = offs[E];
            *num_pairs = P;
            tok_off[T] = (int32_t)P;
            if (P > P_cap) atomicOr(status, 1);
        }
    }
    {   // thread (w, e): one table entry each
        int b = base[lane];
        for (int u = 0; u < wave; ++u) b += wc[u][lane];
        wbase[wave][lane] = b;
    }
    int64_t slot = tok_base_s + (incl - k);
    for (int w = 0; w < wave; ++w) slot += wk[w];
    if (t < T) tok_off[t] = (int32_t)slot;
    __syncthreads();

    // every token walks its own selected experts (k of them, not E), eight per round: the round's scores are
    // fetched together, then its pairs are written
    uint64_t rem = bits;
    while (rem) {
        constexpr int U = 8;
        int ee[U];
        bool on[U];
        float score[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            on[u] = rem != 0;
            ee[u] = on[u] ? __ffsll((unsigned long long)rem) - 1 : 0;
            rem &= rem - 1;                           // 0 stays 0
        }
#pragma unroll
        for (int u = 0; u < U; ++u) score[u] = on[u] ? scores[(size_t)t * E + ee[u]] : 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (on[u]) {
                const int r = wbase[wave][ee[u]] + __popcll(wbal[wave][ee[u]] & lt);
                if ((int64_t)r < P_cap) {
                    pair_token[r] = t;
                    pair_gate[r] = score[u];
                }
                if (slot < P_cap) tok_rows[slot] = (int64_t)r < P_cap ? r : (int32_t)(P_cap - 1);
                ++slot;
            }
    }
}

// Optional materialisation of the permuted input: x_perm[r,:] = x[pair_token[r],:], 16 bytes per thread.
__global__ __launch_bounds__(256) void gather_rows_kernel(
    const u32x4* __restrict__ x, const int32_t* __restrict__ pair_token,
    const int32_t* __restrict__ expert_offsets, int E, int64_t P_cap, int vec_per_row,
    u32x4* __restrict__ x_perm)
{
    const int P = clamp_pairs(expert_offsets[E], P_cap);
    const int64_t total = (int64_t)P * vec_per_row;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int r = (int)(i / vec_per_row), v = (int)(i % vec_per_row);
        x_perm[i] = x[(size_t)pair_token[r] * vec_per_row + v];
    }
}

hipError_t launch_gather_rows(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                              const int32_t* expert_offsets, void* x_perm) {
    const int esz = s.dtype == EVOMOE_BF16 ? 2 : 4;
    const int vec_per_row = s.d * esz / 16;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(c.num_cu * 8), dim3(256), 0, c.stream, (const u32x4*)x,
                       pair_token, expert_offsets, s.E, s.P_cap, vec_per_row, (u32x4*)x_perm);
    return hipGetLastError();
}

hipError_t launch_dispatch(const Ctx& c, const evomoe_shape& s, const uint64_t* mask_bits,
                           const float* scores, const int32_t* block_hist, int32_t* expert_offsets,
                           int32_t* pair_token, float* pair_gate, int32_t* tok_off, int32_t* tok_rows,
                           int64_t* num_pairs, const void* x, void* x_perm, int32_t* hist_scratch) {
    const int nblk = dispatch_blocks(s);
    const int32_t* table = block_hist;
    if (!table) {       // the per-block histograms did not come with the mask: count them here
        ProfScope ps(c, EVOMOE_K_DISPATCH_HIST);
        hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblk), dim3(256), 0, c.stream, mask_bits, s.T, s.E,
                           hist_scratch);
        table = hist_scratch;
    }
    {
        ProfScope ps(c, EVOMOE_K_DISPATCH_SCATTER);
#define EVOMOE_SCATTER(EPV)                                                                              \
    hipLaunchKernelGGL(dispatch_scatter_kernel<EPV>, dim3(nblk), dim3(256), 0, c.stream, mask_bits, scores, s.T, \
                       s.E, nblk, s.P_cap, table, expert_offsets, pair_token, pair_gate, tok_off, tok_rows,       \
                       num_pairs, c.status_dev)
        if (s.E <= 16) EVOMOE_SCATTER(16);
        else if (s.E <= 32) EVOMOE_SCATTER(32);
        else EVOMOE_SCATTER(64);
#undef EVOMOE_SCATTER
    }
    if (x_perm) return launch_gather_rows(c, s, x, pair_token, expert_offsets, x_perm);
    return hipGetLastError();
}

// dx[s,:] = sum of dXp over the token's rows, ascending expert, f32 accumulate.  One thread owns one
// 16-byte vector of one token's row.
template <typename TX>
__global__ __launch_bounds__(256) void dispatch_bwd_kernel(
    const TX* __restrict__ dXp, const int32_t* __restrict__ tok_off,
    const int32_t* __restrict__ tok_rows, int T, int d, int64_t P_cap, TX* __restrict__ dx)
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
        // four rows at a time: their indices, then their vectors, are loaded together (the loads of one row
        // depend on each other, those of different rows do not); added in ascending expert order
        for (int64_t j = j0; j < j1; j += 4) {
            int r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = tok_rows[j + u < j1 ? j + u : j1 - 1];
            float val[4][KV];
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<TX>::load_vec(dXp + (size_t)r[u] * d + v * KV, val[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j + u < j1) {
#pragma unroll
                    for (int q = 0; q < KV; ++q) acc[q] += val[u][q];
                }
        }
        Elem<TX>::store_vec(dx + (size_t)t * d + v * KV, acc);
    }
}

hipError_t launch_dispatch_bwd(const Ctx& c, const evomoe_shape& s, const void* dXp,
                               const int32_t* tok_off, const int32_t* tok_rows, void* dx) {
    const int kv = s.dtype == EVOMOE_BF16 ? 8 : 4;
    const int64_t total = (int64_t)s.T * (s.d / kv);
    const int blocks = (int)((total + 255) / 256 < (int64_t)c.num_cu * 16 ? (total + 255) / 256
                                                                           : (int64_t)c.num_cu * 16);
    ProfScope ps(c, EVOMOE_K_DISPATCH_BWD);
    if (s.dtype == EVOMOE_BF16)
        hipLaunchKernelGGL(dispatch_bwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, c.stream,
                           (const bf16_t*)dXp, tok_off, tok_rows, s.T, s.d, s.P_cap, (bf16_t*)dx);
    else
        hipLaunchKernelGGL(dispatch_bwd_kernel<float>, dim3(blocks), dim3(256), 0, c.stream,
                           (const float*)dXp, tok_off, tok_rows, s.T, s.d, s.P_cap, (float*)dx);
    return hipGetLastError();
}

}  // namespace evomoe
