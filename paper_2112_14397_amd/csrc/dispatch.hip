// Dispatch: variable-k permutation of the selected (token, expert) pairs (EvoMoE Algorithm 1: the
// per-token loop over id in id_s, regrouped by expert; no capacity limit, every selected pair is kept).
// A stable counting sort: rows are expert-major and token-ascending, computed with integer ballots and
// prefix sums only, so the indices are reproducible bit for bit.
#include "kernels.h"

namespace evomoe {

int dispatch_blocks(const evomoe_shape& s) { return (s.T + kDispatchTokens - 1) / kDispatchTokens; }

// Pass 1: per-block (256 consecutive tokens) expert histogram from wave ballots.
__global__ __launch_bounds__(256) void dispatch_hist_kernel(
    const uint64_t* __restrict__ mask_bits, int T, int E, int32_t* __restrict__ block_counts)
{
    __shared__ int wc[4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x * kDispatchTokens + tid;
    const uint64_t bits = (t < T) ? mask_bits[t] : 0ull;
    for (int e = 0; e < E; ++e) {
        const uint64_t bal = __ballot((bits >> e) & 1ull);
        if (lane == 0) wc[wave][e] = __popcll(bal);
    }
    __syncthreads();
    if (tid < E)
        block_counts[(size_t)blockIdx.x * E + tid] = wc[0][tid] + wc[1][tid] + wc[2][tid] + wc[3][tid];
}

// Pass 2 (one block): turns the [nblk][E] histogram table into  base[b][e] = first row of expert e's
// tokens that live in block b,  the expert offsets, the per-block start of the token CSR, P, and the
// capacity flag.  (A last-block-done ticket inside pass 1 would serialise one device-scope atomic per
// block on one address; a separate tiny launch is cheaper.)
__global__ __launch_bounds__(256) void dispatch_scan_kernel(
    int nblk, int T, int E, int64_t P_cap,
    int32_t* __restrict__ block_counts,   // [nblk][E] in: counts, out: bases
    int32_t* __restrict__ tok_base,       // [nblk]
    int32_t* __restrict__ expert_offsets, int32_t* __restrict__ tok_off,
    int64_t* __restrict__ num_pairs, int32_t* __restrict__ status)
{
    __shared__ int tot[65];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the table is walked in chunks staged through LDS
    constexpr int kChunkInts = 8192;
    __shared__ int tab[kChunkInts];
    const int rows_per_chunk = min(kChunkInts / E, 256);      // one thread per block row in the scan
    // pass A: column totals -> expert offsets
    int mysum = 0;                                   // thread e < E accumulates column e
    for (int b0 = 0; b0 < nblk; b0 += rows_per_chunk) {
        const int nr = min(rows_per_chunk, nblk - b0);
        for (int i = tid; i < nr * E; i += 256)
            tab[i] = block_counts[(size_t)b0 * E + i];
        __syncthreads();
        if (tid < E)
            for (int r = 0; r < nr; ++r) mysum += tab[r * E + tid];
        __syncthreads();
    }
    if (tid < E) tot[tid + 1] = mysum;
    if (tid == 0) tot[0] = 0;
    __syncthreads();
    if (tid == 0) {
        for (int e = 0; e < E; ++e) tot[e + 1] += tot[e];     // inclusive scan -> offsets
        const int64_t P = tot[E];
        *num_pairs = P;
        tok_off[T] = (int32_t)P;
        if (P > P_cap) atomicOr(status, 1);
    }
    __syncthreads();
    if (tid <= E) expert_offsets[tid] = tot[tid];
    // pass B: per-expert running base over blocks (thread e), and per-block CSR base (block scan)
    int run = (tid < E) ? tot[tid] : 0;
    int carry = 0;                                   // pairs owned by tokens of earlier chunks (uniform)
    __shared__ int wsum[4];
    for (int b0 = 0; b0 < nblk; b0 += rows_per_chunk) {
        const int nr = min(rows_per_chunk, nblk - b0);
        for (int i = tid; i < nr * E; i += 256)
            tab[i] = block_counts[(size_t)b0 * E + i];
        __syncthreads();
        // pairs of block b0+tid, then an exclusive scan over the chunk's blocks
        int mine = 0;
        if (tid < nr)
            for (int e = 0; e < E; ++e) mine += tab[tid * E + e];
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        int before = carry;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (tid < nr) tok_base[b0 + tid] = before + incl - mine;
        carry += wsum[0] + wsum[1] + wsum[2] + wsum[3];
        if (tid < E) {
            for (int r = 0; r < nr; ++r) {
                const int cur = tab[r * E + tid];
                tab[r * E + tid] = run;
                run += cur;
            }
        }
        __syncthreads();
        for (int i = tid; i < nr * E; i += 256) block_counts[(size_t)b0 * E + i] = tab[i];
        __syncthreads();
    }
}

// Pass 2: one thread per token.  Row of pair (t, e) = base[block][e] + (selected tokens of e before t
// inside the block), from wave ballots.  Writes pair_token / pair_gate at the row and the token's CSR.
__global__ __launch_bounds__(256) void dispatch_scatter_kernel(
    const uint64_t* __restrict__ mask_bits, const float* __restrict__ scores, int T, int E,
    int64_t P_cap, const int32_t* __restrict__ block_base, const int32_t* __restrict__ tok_base,
    int32_t* __restrict__ pair_token, float* __restrict__ pair_gate, int32_t* __restrict__ tok_off,
    int32_t* __restrict__ tok_rows)
{
    __shared__ int wc[4][64];
    __shared__ int base[64];
    __shared__ int wk[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x * kDispatchTokens + tid;
    const uint64_t bits = (t < T) ? mask_bits[t] : 0ull;
    const uint64_t lt = (1ull << lane) - 1ull;
    if (tid < E) base[tid] = block_base[(size_t)blockIdx.x * E + tid];
    for (int e = 0; e < E; ++e) {
        const uint64_t bal = __ballot((bits >> e) & 1ull);
        if (lane == 0) wc[wave][e] = __popcll(bal);
    }
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
    int64_t slot = tok_base[blockIdx.x] + (incl - k);
    for (int w = 0; w < wave; ++w) slot += wk[w];
    if (t < T) tok_off[t] = (int32_t)slot;

    for (int e = 0; e < E; ++e) {
        const uint64_t bal = __ballot((bits >> e) & 1ull);
        if ((bits >> e) & 1ull) {
            int r = base[e] + __popcll(bal & lt);
            for (int w = 0; w < wave; ++w) r += wc[w][e];
            if ((int64_t)r < P_cap) {
                pair_token[r] = t;
                pair_gate[r] = scores[(size_t)t * E + e];
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
                           const float* scores, int32_t* expert_offsets, int32_t* pair_token,
                           float* pair_gate, int32_t* tok_off, int32_t* tok_rows, int64_t* num_pairs,
                           const void* x, void* x_perm) {
    const int nblk = dispatch_blocks(s);
    int32_t* base = c.block_counts;
    int32_t* tok_base = c.block_counts + (size_t)nblk * s.E;
    {
        ProfScope ps(c, EVOMOE_K_DISPATCH_HIST);
        hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblk), dim3(256), 0, c.stream, mask_bits, s.T, s.E, base);
        hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(256), 0, c.stream, nblk, s.T, s.E, s.P_cap, base,
                           tok_base, expert_offsets, tok_off, num_pairs, c.status_dev);
    }
    {
        ProfScope ps(c, EVOMOE_K_DISPATCH_SCATTER);
        hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(nblk), dim3(256), 0, c.stream, mask_bits, scores,
                           s.T, s.E, s.P_cap, base, tok_base, pair_token, pair_gate, tok_off, tok_rows);
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
