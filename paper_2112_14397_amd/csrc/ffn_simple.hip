// Expert FFNs (EvoMoE Eq. ffn applied per expert over its ragged row range) -- the plain path.
//
// LDS-tiled float32-FMA grouped GEMMs, generic in the storage type.  This is the path of the float32
// layer (whose tolerance, 1e-5, needs full float32 products) and the fallback shape-wise; the bf16
// layer runs the MFMA kernels of ffn_mfma.hip instead.
#include "ffn_internal.h"

namespace evomoe {

namespace {

constexpr int BM = 64, BN = 64, BK = 16;

enum { EPI_HA = 0, EPI_BIAS = 1, EPI_ACTGRAD = 2, EPI_NONE = 3 };

// Row-grouped GEMM:  C[r, n] = sum_k A[arow(r), k] * B_g(k, n)  for r in expert g's row range,
// B_g(k, n) = Bmat[g*b_group_stride + k*sbk + n*sbn].
template <typename TX, int EPI>
__global__ __launch_bounds__(256) void ffn_rows_kernel(
    const TX* __restrict__ Amat, int lda, const int32_t* __restrict__ row_index,
    const int32_t* __restrict__ expert_offsets, int E, int64_t P_cap,
    const TX* __restrict__ Bmat, int64_t b_group_stride, int sbk, int sbn, int N, int K,
    const float* __restrict__ bias, const TX* __restrict__ Hin, TX* __restrict__ out1,
    TX* __restrict__ out2, int act)
{
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    __shared__ int offs[65];
    const int tid = threadIdx.x;
    if (tid <= E) offs[tid] = clamp_pairs(expert_offsets[tid], P_cap);
    __syncthreads();
    const int tx = tid & 15, ty = tid >> 4;      // 16 x 16 threads, 4 x 4 outputs each
    const int n0 = blockIdx.y * BN;

    for (int tile = blockIdx.x;; tile += gridDim.x) {
        // tile -> (expert, first row)
        int g = 0, row0 = 0, rows = 0, seen = 0;
        bool found = false;
        for (int e = 0; e < E; ++e) {
            const int ne = offs[e + 1] - offs[e];
            const int nt = (ne + BM - 1) / BM;
            if (tile < seen + nt) {
                g = e; row0 = offs[e] + (tile - seen) * BM; rows = min(BM, offs[e + 1] - row0);
                found = true;
                break;
            }
            seen += nt;
        }
        if (!found) break;          // uniform across the block

        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
        const TX* Bg = Bmat + (size_t)g * b_group_stride;

        for (int k0 = 0; k0 < K; k0 += BK) {
            // A tile: thread -> row tid/4, k (tid%4)*4 .. +3
            {
                const int r = tid >> 2, kk = (tid & 3) * 4;
                const bool ok = r < rows;
                size_t arow = 0;
                if (ok) arow = row_index ? (size_t)row_index[row0 + r] : (size_t)(row0 + r);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = k0 + kk + j;
                    As[kk + j][r] = (ok && k < K) ? Elem<TX>::load(Amat + arow * lda + k) : 0.f;
                }
            }
            // B tile
            if (sbk == 1) {         // k contiguous: thread -> n tid/4, k (tid%4)*4..+3
                const int n = tid >> 2, kk = (tid & 3) * 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = k0 + kk + j;
                    Bs[kk + j][n] = (n0 + n < N && k < K)
                                        ? Elem<TX>::load(Bg + (size_t)(n0 + n) * sbn + k) : 0.f;
                }
            } else {                // n contiguous: thread -> k tid/16, n (tid%16)*4..+3
                const int kk = tid >> 4, nn = (tid & 15) * 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = k0 + kk, n = n0 + nn + j;
                    Bs[kk][nn + j] = (n < N && k < K)
                                         ? Elem<TX>::load(Bg + (size_t)k * sbk + (size_t)n * sbn) : 0.f;
                }
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < BK; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
            }
            __syncthreads();
        }

#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = ty * 4 + i;
            if (r >= rows) continue;
            const size_t grow = (size_t)(row0 + r);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n >= N) continue;
                float v = acc[i][j];
                if (EPI == EPI_HA) {
                    if (bias) v += bias[(size_t)g * N + n];
                    Elem<TX>::store(out1 + grow * N + n, v);
                    Elem<TX>::store(out2 + grow * N + n, act_fwd(v, act));
                } else if (EPI == EPI_BIAS) {
                    if (bias) v += bias[(size_t)g * N + n];
                    Elem<TX>::store(out1 + grow * N + n, v);
                } else if (EPI == EPI_ACTGRAD) {
                    v *= act_grad(Elem<TX>::load(Hin + grow * N + n), act);
                    Elem<TX>::store(out1 + grow * N + n, v);
                } else {
                    Elem<TX>::store(out1 + grow * N + n, v);
                }
            }
        }
    }
}

// Weight gradient (contraction over the expert's rows):
//   C_g[m, n] = sum_{r in g} L[r, m] * R[rrow(r), n]     (+ C_g[m, n] if accumulate)
template <typename TX>
__global__ __launch_bounds__(256) void ffn_wgrad_kernel(
    const TX* __restrict__ L, int M, const TX* __restrict__ R, int N,
    const int32_t* __restrict__ row_index, const int32_t* __restrict__ expert_offsets, int E,
    int64_t P_cap, TX* __restrict__ C, int accumulate)
{
    __shared__ float Ls[BK][BM + 4];
    __shared__ float Rs[BK][BN + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int g = blockIdx.z, m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int r0 = clamp_pairs(expert_offsets[g], P_cap), r1 = clamp_pairs(expert_offsets[g + 1], P_cap);
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int rb = r0; rb < r1; rb += BK) {
        const int kk = tid >> 4, cc = (tid & 15) * 4;
        const int r = rb + kk;
        const bool ok = r < r1;
        size_t rr = 0;
        if (ok) rr = row_index ? (size_t)row_index[r] : (size_t)r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + cc + j, n = n0 + cc + j;
            Ls[kk][cc + j] = (ok && m < M) ? Elem<TX>::load(L + (size_t)r * M + m) : 0.f;
            Rs[kk][cc + j] = (ok && n < N) ? Elem<TX>::load(R + rr * N + n) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Ls[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Rs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            TX* p = C + ((size_t)g * M + m) * N + n;
            float v = acc[i][j];
            if (accumulate) v += Elem<TX>::load(p);
            Elem<TX>::store(p, v);
        }
    }
}

}  // namespace

// Bias gradient: db[g, n] = sum over the expert's rows of Mx[r, n]   (+ db if accumulate).
// Pass 1: block = 64 columns (8 lanes x 16 bytes) x 32 row lanes, one of kColsumSplit row ranges of one
// expert; f32 partial sums, tree-reduced over the row lanes in LDS, written to part[split][g][n].
// Pass 2 adds the splits in order.  No atomics: the result is reproducible bit for bit.

// A block streams whole row segments: CL column lanes x 16 bytes are contiguous in a row (up to 4 KB), RL = 256/CL
// row lanes take alternate rows, four rows of loads in flight per thread.
template <typename TX>
__global__ __launch_bounds__(256) void ffn_colsum_part_kernel(
    const TX* __restrict__ Mx, int N, int E, const int32_t* __restrict__ expert_offsets, int64_t P_cap,
    int CL, float* __restrict__ part)
{
    constexpr int KV = Elem<TX>::kVec;           // elements per 16-byte load
    extern __shared__ float red[];               // [RL][CL*KV]
    const int RL = 256 / CL;
    const int g = blockIdx.y, split = blockIdx.z;
    const int cl = threadIdx.x % CL, rl = threadIdx.x / CL;
    const int n = (blockIdx.x * CL + cl) * KV;
    const int r0 = clamp_pairs(expert_offsets[g], P_cap), r1 = clamp_pairs(expert_offsets[g + 1], P_cap);
    const int per = (r1 - r0 + kColsumSplit - 1) / kColsumSplit;
    const int rb = r0 + split * per, re = min(r1, rb + per);
    float acc[KV];
#pragma unroll
    for (int q = 0; q < KV; ++q) acc[q] = 0.f;
    if (n < N && rl < RL) {
        int r = rb + rl;
        for (; r + 3 * RL < re; r += 4 * RL) {
            float v[4][KV];
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<TX>::load_vec(Mx + (size_t)(r + u * RL) * N + n, v[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int q = 0; q < KV; ++q) acc[q] += v[u][q];
        }
        for (; r < re; r += RL) {
            float v[KV];
            Elem<TX>::load_vec(Mx + (size_t)r * N + n, v);
#pragma unroll
            for (int q = 0; q < KV; ++q) acc[q] += v[q];
        }
    }
    if (rl < RL) {
#pragma unroll
        for (int q = 0; q < KV; ++q) red[(size_t)rl * CL * KV + cl * KV + q] = acc[q];
    }
    __syncthreads();
    // row lanes added in order by the threads of lane 0
    if (rl == 0 && n < N) {
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            float sum = 0.f;
            for (int l = 0; l < RL; ++l) sum += red[(size_t)l * CL * KV + cl * KV + q];
            part[((size_t)split * E + g) * N + n + q] = sum;
        }
    }
}

__global__ __launch_bounds__(256) void ffn_colsum_final_kernel(const float* __restrict__ part, size_t n,
                                                               float* __restrict__ db, int accumulate)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float s = accumulate ? db[i] : 0.f;
    for (int k0 = 0; k0 < kColsumSplit; k0 += 8) {        // eight loads in flight, added in split order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(k0 + u) * n + i];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    db[i] = s;
}

size_t colsum_scratch_bytes(const evomoe_shape& s) {
    return (((size_t)kColsumSplit * s.E * (s.d > s.F ? s.d : s.F) * sizeof(float) + 255) & ~(size_t)255) +
           dh_colpart_bytes(s);
}

template <typename TX>
hipError_t launch_colsum_part(const Ctx& c, const evomoe_shape& s, const void* Mx, int N,
                              const int32_t* expert_offsets, float* scratch) {
    constexpr int KV = Elem<TX>::kVec;
    const int vecs = (N + KV - 1) / KV;                       // 16-byte vectors per row
    int CL = vecs >= 256 ? 256 : vecs;                        // column lanes (contiguous in a row)
    if (CL > 128) CL = 256;                                   // 129..255 vectors: two column blocks of 256 lanes
    const int RL = 256 / CL;
    hipLaunchKernelGGL(ffn_colsum_part_kernel<TX>, dim3((vecs + CL - 1) / CL, s.E, kColsumSplit), dim3(256),
                       (size_t)RL * CL * KV * sizeof(float), c.stream, (const TX*)Mx, N, s.E, expert_offsets,
                       s.P_cap, CL, scratch);
    return hipGetLastError();
}
template hipError_t launch_colsum_part<float>(const Ctx&, const evomoe_shape&, const void*, int, const int32_t*, float*);
template hipError_t launch_colsum_part<bf16_t>(const Ctx&, const evomoe_shape&, const void*, int, const int32_t*, float*);

template <typename TX>
hipError_t launch_colsum(const Ctx& c, const evomoe_shape& s, const void* Mx, int N,
                         const int32_t* expert_offsets, float* db, int accumulate, float* scratch) {
    hipError_t err = launch_colsum_part<TX>(c, s, Mx, N, expert_offsets, scratch);
    if (err != hipSuccess) return err;
    const size_t n = (size_t)s.E * N;
    hipLaunchKernelGGL(ffn_colsum_final_kernel, dim3((n + 255) / 256), dim3(256), 0, c.stream, scratch, n,
                       db, accumulate);
    return hipGetLastError();
}
template hipError_t launch_colsum<float>(const Ctx&, const evomoe_shape&, const void*, int, const int32_t*, float*, int, float*);
template hipError_t launch_colsum<bf16_t>(const Ctx&, const evomoe_shape&, const void*, int, const int32_t*, float*, int, float*);

static int row_tile_grid(const Ctx& c, const evomoe_shape& s) {
    const int64_t worst = (s.P_cap + BM - 1) / BM + s.E;
    const int64_t cap = (int64_t)c.num_cu * 8;
    return (int)(worst < cap ? worst : cap);
}

template <typename TX>
hipError_t simple_ffn_fwd(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                          const int32_t* expert_offsets, const void* W1, const float* b1,
                          const void* W2, const float* b2, void* H, void* A, void* O) {
    const int gx = row_tile_grid(c, s);
    // H = X W1^T + b1, A = act(H):  B_g(k, n) = W1[g][n][k]
    { ProfScope ps(c, EVOMOE_K_FFN_GEMM1);
    hipLaunchKernelGGL((ffn_rows_kernel<TX, EPI_HA>), dim3(gx, (s.F + BN - 1) / BN), dim3(256), 0, c.stream,
                       (const TX*)x, s.d, pair_token, expert_offsets, s.E, s.P_cap, (const TX*)W1,
                       (int64_t)s.F * s.d, 1, s.d, s.F, s.d, b1, (const TX*)nullptr, (TX*)H, (TX*)A, s.act); }
    if (!O) return hipGetLastError();     // O == nullptr: recomputation of H and A only
    // O = A W2^T + b2:  B_g(k, n) = W2[g][n][k]
    ProfScope ps(c, EVOMOE_K_FFN_GEMM2);
    hipLaunchKernelGGL((ffn_rows_kernel<TX, EPI_BIAS>), dim3(gx, (s.d + BN - 1) / BN), dim3(256), 0, c.stream,
                       (const TX*)A, s.F, (const int32_t*)nullptr, expert_offsets, s.E, s.P_cap,
                       (const TX*)W2, (int64_t)s.d * s.F, 1, s.F, s.d, s.F, b2, (const TX*)nullptr,
                       (TX*)O, (TX*)nullptr, s.act);
    return hipGetLastError();
}

template <typename TX>
hipError_t simple_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H,
                          const void* A, const void* x, const int32_t* pair_token,
                          const int32_t* expert_offsets, const void* W1, const void* W2, void* dW1,
                          float* db1, void* dW2, float* db2, void* dXp, int accumulate, void* dH) {
    const int gx = row_tile_grid(c, s);
    float* scratch = reinterpret_cast<float*>(static_cast<char*>(dH) + dh_bytes(s));
    // dH = (dO W2) * act'(H):  B_g(k, n) = W2[g][k][n]
    { ProfScope ps(c, EVOMOE_K_FFN_BWD_DH);
    hipLaunchKernelGGL((ffn_rows_kernel<TX, EPI_ACTGRAD>), dim3(gx, (s.F + BN - 1) / BN), dim3(256), 0,
                       c.stream, (const TX*)dO, s.d, (const int32_t*)nullptr, expert_offsets, s.E,
                       s.P_cap, (const TX*)W2, (int64_t)s.d * s.F, s.F, 1, s.F, s.d,
                       (const float*)nullptr, (const TX*)H, (TX*)dH, (TX*)nullptr, s.act); }
    // dXp = dH W1:  B_g(k, n) = W1[g][k][n]
    { ProfScope ps(c, EVOMOE_K_FFN_BWD_DX);
    hipLaunchKernelGGL((ffn_rows_kernel<TX, EPI_NONE>), dim3(gx, (s.d + BN - 1) / BN), dim3(256), 0,
                       c.stream, (const TX*)dH, s.F, (const int32_t*)nullptr, expert_offsets, s.E,
                       s.P_cap, (const TX*)W1, (int64_t)s.F * s.d, s.d, 1, s.d, s.F,
                       (const float*)nullptr, (const TX*)nullptr, (TX*)dXp, (TX*)nullptr, s.act); }
    if (dW2) { // dW2_g = dO_g^T A_g   [d, F]
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW2);
        hipLaunchKernelGGL(ffn_wgrad_kernel<TX>, dim3((s.F + BN - 1) / BN, (s.d + BM - 1) / BM, s.E),
                           dim3(256), 0, c.stream, (const TX*)dO, s.d, (const TX*)A, s.F,
                           (const int32_t*)nullptr, expert_offsets, s.E, s.P_cap, (TX*)dW2, accumulate);
    }
    if (dW1) { // dW1_g = dH_g^T X_g    [F, d]
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW1);
        hipLaunchKernelGGL(ffn_wgrad_kernel<TX>, dim3((s.d + BN - 1) / BN, (s.F + BM - 1) / BM, s.E),
                           dim3(256), 0, c.stream, (const TX*)dH, s.F, (const TX*)x, s.d, pair_token,
                           expert_offsets, s.E, s.P_cap, (TX*)dW1, accumulate);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    ProfScope ps(c, EVOMOE_K_FFN_BWD_DB);
    if (db2) err = launch_colsum<TX>(c, s, dO, s.d, expert_offsets, db2, accumulate, scratch);
    if (err != hipSuccess) return err;
    if (db1) err = launch_colsum<TX>(c, s, dH, s.F, expert_offsets, db1, accumulate, scratch);
    return err;
}

template hipError_t simple_ffn_fwd<float>(const Ctx&, const evomoe_shape&, const void*, const int32_t*, const int32_t*, const void*, const float*, const void*, const float*, void*, void*, void*);
template hipError_t simple_ffn_fwd<bf16_t>(const Ctx&, const evomoe_shape&, const void*, const int32_t*, const int32_t*, const void*, const float*, const void*, const float*, void*, void*, void*);
template hipError_t simple_ffn_bwd<float>(const Ctx&, const evomoe_shape&, const void*, const void*, const void*, const void*, const int32_t*, const int32_t*, const void*, const void*, void*, float*, void*, float*, void*, int, void*);
template hipError_t simple_ffn_bwd<bf16_t>(const Ctx&, const evomoe_shape&, const void*, const void*, const void*, const void*, const int32_t*, const int32_t*, const void*, const void*, void*, float*, void*, float*, void*, int, void*);

}  // namespace evomoe
