// Expert FFNs on the bf16 matrix cores (EvoMoE Eq. ffn per expert over its ragged row range, and its
// backward).  One grouped-GEMM kernel template, v_mfma_f32_32x32x16_bf16, f32 accumulation:
//
//   NT  C[r,n] = sum_k A[arow(r),k] * W_g[n,k]      forward GEMMs (A rows optionally gathered by token)
//   NN  C[r,n] = sum_k A[r,k]       * W_g[k,n]      dH = dO W2,  dXp = dH W1
//   TN  C_g[m,n] = sum_{r in g} L[r,m] * R[rrow(r),n]   weight gradients (contraction over the ragged rows)
//
// Block = 4 waves (2 x 2), block tile BM x BN, K slab 64, double-buffered LDS, operands fetched with
// 16-byte global loads.  Operands whose contraction index is contiguous in memory sit in LDS as
// [row][64 k] with an XOR swizzle of the 16-byte chunks and are read with ds_read_b128; operands whose
// contraction index is the row index sit as [k][cols] (padded rows) and are read with the transposing
// LDS load (ds_read_b64_tr_b16), so no operand is ever transposed in global memory.
// Epilogues (bias, activation, act'(H) product, accumulate) run in f32 on a row-major copy of the
// accumulators staged through LDS, and leave with 16-byte stores.
#include "ffn_internal.h"

namespace evomoe {

namespace {

constexpr int BK = 64;
enum { L_NT = 0, L_NN = 1, L_TN = 2 };
enum { E_HA = 0, E_BIAS = 1, E_ACTGRAD = 2, E_NONE = 3, E_WGRAD = 4 };

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

struct GemmArgs {
    const bf16_t* A;  int64_t lda;      // NT/NN: A rows [*,K];  TN: L [P,M] (lda = M)
    const bf16_t* B;  int64_t ldb;      // NT: W_g [N,K] (ldb = K);  NN: W_g [K,N] (ldb = N);  TN: R [*,N] (ldb = N)
    int64_t b_group_stride;             // NT/NN: elements between two experts' weight matrices
    const int32_t* a_rows;              // NT: gather of A rows (or null)
    const int32_t* b_rows;              // TN: gather of R rows (or null)
    const int32_t* expert_offsets;
    int E;
    int64_t P_cap;
    int M, N, K;                        // M: TN only.  K: NT/NN only (TN contracts over the expert's rows)
    const float* bias;                  // [E,N] or null
    const bf16_t* Hin;                  // E_ACTGRAD: pre-activations [P,N]
    bf16_t* out1;                       // C (H for E_HA)
    bf16_t* out2;                       // E_HA: A = act(H)
    int act, accumulate;
};

// ---- LDS geometry -------------------------------------------------------------------------------
// k-contiguous tile: [R][64] bf16, 128 B per row, 16-byte chunk c of row r stored at chunk c ^ (r & 7)
__device__ __forceinline__ int kc_off(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }
// k-strided tile: [64][C] bf16, row stride C*2 + 32 bytes
template <int C> __device__ __forceinline__ int ks_off(int k, int col) { return k * (C * 2 + 32) + col * 2; }
template <int R> constexpr int kc_bytes() { return R * 128; }
template <int C> constexpr int ks_bytes() { return 64 * (C * 2 + 32); }

template <int LAYOUT, int BM, int BN> struct Geo {
    static constexpr bool A_KC = (LAYOUT != L_TN);          // A operand k-contiguous?
    static constexpr bool B_KC = (LAYOUT == L_NT);
    static constexpr int A_BYTES = A_KC ? kc_bytes<BM>() : ks_bytes<BM>();
    static constexpr int B_BYTES = B_KC ? kc_bytes<BN>() : ks_bytes<BN>();
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int WM = BM / 2, WN = BN / 2;
    static constexpr int EPI_ROWS = 64;                      // rows of the wave tile staged per pass
    static constexpr int EPI_LD = WN + 4;                    // f32 row stride of the staging copy
    static constexpr int EPI_BYTES = 4 * EPI_ROWS * EPI_LD * 4;
    static constexpr int SMEM = (2 * STAGE > EPI_BYTES ? 2 * STAGE : EPI_BYTES);
};

__device__ __forceinline__ u32x4 ldg16(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

template <int LAYOUT, int EPI, int BM, int BN>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(GemmArgs p)
{
    using G = Geo<LAYOUT, BM, BN>;
    constexpr int WM = G::WM, WN = G::WN;
    constexpr int TM = WM / 32, TN_ = WN / 32;               // MFMA tiles per wave
    constexpr int A_LD = G::A_KC ? (BM * 8 / 256) : (64 * (BM / 8) / 256);   // 16-byte loads per thread per slab
    constexpr int B_LD = G::B_KC ? (BN * 8 / 256) : (64 * (BN / 8) / 256);

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int offs[65];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    if (tid <= p.E) offs[tid] = clamp_pairs(p.expert_offsets[tid], p.P_cap);
    __syncthreads();

    const int nct = (p.N + BN - 1) / BN;
    const int nmt = (LAYOUT == L_TN) ? (p.M + BM - 1) / BM : 1;

    for (int tile = blockIdx.x;; tile += gridDim.x) {
        // ---------------- tile -> (expert, origin, contraction range) ----------------
        int g = 0, row0 = 0, rows = 0, n0 = 0, m0 = 0, kbeg = 0, kend = 0;
        if (LAYOUT == L_TN) {
            if (tile >= p.E * nmt * nct) break;
            g = tile / (nmt * nct);
            const int rem = tile % (nmt * nct);
            m0 = (rem / nct) * BM;
            n0 = (rem % nct) * BN;
            kbeg = offs[g];
            kend = offs[g + 1];
        } else {
            const int rt = tile / nct;
            n0 = (tile % nct) * BN;
            int seen = 0;
            bool found = false;
            for (int e = 0; e < p.E; ++e) {
                const int ne = offs[e + 1] - offs[e];
                const int nt = (ne + BM - 1) / BM;
                if (rt < seen + nt) {
                    g = e;
                    row0 = offs[e] + (rt - seen) * BM;
                    rows = min(BM, offs[e + 1] - row0);
                    found = true;
                    break;
                }
                seen += nt;
            }
            if (!found) break;
            kbeg = 0;
            kend = p.K;
        }
        const int nslab = (kend - kbeg + BK - 1) / BK;

        // ---------------- per-thread global fetch plan ----------------
        // k-contiguous tile: thread -> chunk tid%8 of rows tid/8 + 32*i
        // k-strided tile  : thread -> chunk tid%(C/8) of k-rows tid/(C/8) + (256/(C/8))*i
        const bf16_t* a_ptr[A_LD];
        bool a_ok[A_LD];
        if (G::A_KC) {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int r = (tid >> 3) + 32 * i;
                a_ok[i] = r < rows;
                int64_t ar = 0;
                if (a_ok[i]) ar = p.a_rows ? (int64_t)p.a_rows[row0 + r] : (int64_t)(row0 + r);
                a_ptr[i] = p.A + ar * p.lda + (tid & 7) * 8;
            }
        }
        const bf16_t* Bg = (LAYOUT == L_TN) ? p.B : p.B + (int64_t)g * p.b_group_stride;

        u32x4 ra[A_LD], rb[B_LD];
        const u32x4 zero4 = {0u, 0u, 0u, 0u};

        auto fetch = [&](int slab) {
            const int k0 = kbeg + slab * BK;
            if (G::A_KC) {
#pragma unroll
                for (int i = 0; i < A_LD; ++i) {
                    const int k = k0 + (tid & 7) * 8;
                    ra[i] = (a_ok[i] && k < kend) ? ldg16(a_ptr[i] + k0) : zero4;
                }
            } else {      // TN: L[r, m0 + ...]
                constexpr int CPR = BM / 8, RPP = 256 / CPR;
#pragma unroll
                for (int i = 0; i < A_LD; ++i) {
                    const int r = k0 + tid / CPR + RPP * i;
                    const int m = m0 + (tid % CPR) * 8;
                    ra[i] = (r < kend && m < p.M) ? ldg16(p.A + (int64_t)r * p.lda + m) : zero4;
                }
            }
            if (G::B_KC) {  // NT: W_g[n0 + row, k]
#pragma unroll
                for (int i = 0; i < B_LD; ++i) {
                    const int n = n0 + (tid >> 3) + 32 * i;
                    const int k = k0 + (tid & 7) * 8;
                    rb[i] = (n < p.N && k < kend) ? ldg16(Bg + (int64_t)n * p.ldb + k) : zero4;
                }
            } else {
                constexpr int CPR = BN / 8, RPP = 256 / CPR;
#pragma unroll
                for (int i = 0; i < B_LD; ++i) {
                    const int r = k0 + tid / CPR + RPP * i;
                    const int n = n0 + (tid % CPR) * 8;
                    if (r < kend && n < p.N) {
                        int64_t br = r;
                        if (LAYOUT == L_TN && p.b_rows) br = p.b_rows[r];
                        rb[i] = ldg16(Bg + br * p.ldb + n);
                    } else {
                        rb[i] = zero4;
                    }
                }
            }
        };
        auto stash = [&](int buf) {
            unsigned char* sa = smem + buf * G::STAGE;
            unsigned char* sb = sa + G::A_BYTES;
            if (G::A_KC) {
#pragma unroll
                for (int i = 0; i < A_LD; ++i)
                    *reinterpret_cast<u32x4*>(sa + kc_off((tid >> 3) + 32 * i, tid & 7)) = ra[i];
            } else {
                constexpr int CPR = BM / 8, RPP = 256 / CPR;
#pragma unroll
                for (int i = 0; i < A_LD; ++i)
                    *reinterpret_cast<u32x4*>(sa + ks_off<BM>(tid / CPR + RPP * i, (tid % CPR) * 8)) = ra[i];
            }
            if (G::B_KC) {
#pragma unroll
                for (int i = 0; i < B_LD; ++i)
                    *reinterpret_cast<u32x4*>(sb + kc_off((tid >> 3) + 32 * i, tid & 7)) = rb[i];
            } else {
                constexpr int CPR = BN / 8, RPP = 256 / CPR;
#pragma unroll
                for (int i = 0; i < B_LD; ++i)
                    *reinterpret_cast<u32x4*>(sb + ks_off<BN>(tid / CPR + RPP * i, (tid % CPR) * 8)) = rb[i];
            }
        };

        f32x16 acc[TM][TN_];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN_; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        __syncthreads();          // previous tile's epilogue has left the LDS
        if (nslab > 0) {
            fetch(0);
            stash(0);
        }
        __syncthreads();

        for (int slab = 0; slab < nslab; ++slab) {
            const int buf = slab & 1;
            if (slab + 1 < nslab) fetch(slab + 1);
            const unsigned char* sa = smem + buf * G::STAGE;
            const unsigned char* sb = sa + G::A_BYTES;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8 fa[TM], fb[TN_];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if (G::A_KC) {
                        const int row = wm * WM + i * 32 + l32;
                        fa[i] = *reinterpret_cast<const bf16x8*>(sa + kc_off(row, ks * 2 + kg));
                    } else {
                        const int mb = wm * WM + i * 32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
                        const int kb = ks * 16 + kg * 8 + ((lane & 15) >> 2);
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4*)(sa + ks_off<BM>(kb, mb)));
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4*)(sa + ks_off<BM>(kb + 4, mb)));
                        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        fa[i] = __builtin_bit_cast(bf16x8, v);
                    }
                }
#pragma unroll
                for (int j = 0; j < TN_; ++j) {
                    if (G::B_KC) {
                        const int row = wn * WN + j * 32 + l32;
                        fb[j] = *reinterpret_cast<const bf16x8*>(sb + kc_off(row, ks * 2 + kg));
                    } else {
                        const int nb = wn * WN + j * 32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
                        const int kb = ks * 16 + kg * 8 + ((lane & 15) >> 2);
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4*)(sb + ks_off<BN>(kb, nb)));
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4*)(sb + ks_off<BN>(kb + 4, nb)));
                        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        fb[j] = __builtin_bit_cast(bf16x8, v);
                    }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN_; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            if (slab + 1 < nslab) stash(buf ^ 1);
            __syncthreads();
        }

        // ---------------- epilogue: stage f32 rows through LDS, finish row-major ----------------
        // acc[i][j][r] is C(row = i*32 + 8*(r/4) + 4*kg + r%4, col = j*32 + l32) of the wave tile.
        float* stg = reinterpret_cast<float*>(smem) + wave * (G::EPI_ROWS * G::EPI_LD);
        constexpr int CPW = WN / 8;                 // 8-column chunks per wave-tile row
        constexpr int RPI = 64 / CPW;               // rows finished per instruction
#pragma unroll
        for (int half = 0; half < WM / 64; ++half) {
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int i = half * 2 + ii;
#pragma unroll
                for (int j = 0; j < TN_; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = ii * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                        stg[row * G::EPI_LD + j * 32 + l32] = acc[i][j][r];
                    }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);     // this wave's LDS writes are done (lgkmcnt(0))
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < 64 / RPI; ++it) {
                const int lr = it * RPI + lane / CPW;            // row inside the 64-row pass
                const int lc = (lane % CPW) * 8;                 // first of 8 columns
                const int trow = wm * WM + half * 64 + lr;       // row inside the block tile
                const int col = n0 + wn * WN + lc;
                const f32x4 v0 = *reinterpret_cast<const f32x4*>(stg + lr * G::EPI_LD + lc);
                const f32x4 v1 = *reinterpret_cast<const f32x4*>(stg + lr * G::EPI_LD + lc + 4);
                float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                if (col >= p.N) continue;
                if (LAYOUT == L_TN) {
                    const int m = m0 + trow;
                    if (m >= p.M) continue;
                    bf16_t* dst = p.out1 + ((int64_t)g * p.M + m) * p.N + col;
                    if (p.accumulate) {
                        float old[8];
                        Elem<bf16_t>::load_vec(dst, old);
#pragma unroll
                        for (int q = 0; q < 8; ++q) v[q] += old[q];
                    }
                    Elem<bf16_t>::store_vec(dst, v);
                } else {
                    if (trow >= rows) continue;
                    const int64_t grow = (int64_t)(row0 + trow);
                    if (EPI == E_HA || EPI == E_BIAS) {
                        if (p.bias) {
                            const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + (int64_t)g * p.N + col);
                            const f32x4 b1 = *reinterpret_cast<const f32x4*>(p.bias + (int64_t)g * p.N + col + 4);
                            v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
                            v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
                        }
                    }
                    if (EPI == E_ACTGRAD) {
                        float h[8];
                        Elem<bf16_t>::load_vec(p.Hin + grow * p.N + col, h);
#pragma unroll
                        for (int q = 0; q < 8; ++q) v[q] *= act_grad(h[q], p.act);
                    }
                    Elem<bf16_t>::store_vec(p.out1 + grow * p.N + col, v);
                    if (EPI == E_HA) {
                        float a[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) a[q] = act_fwd(v[q], p.act);
                        Elem<bf16_t>::store_vec(p.out2 + grow * p.N + col, a);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

template <int LAYOUT, int EPI, int BM, int BN>
hipError_t launch_gemm(const Ctx& c, const GemmArgs& a, int64_t worst_tiles) {
    using G = Geo<LAYOUT, BM, BN>;
    auto kern = grouped_gemm_bf16<LAYOUT, EPI, BM, BN>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::SMEM);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int64_t cap = (int64_t)c.num_cu;
    const int grid = (int)(worst_tiles < cap ? worst_tiles : cap);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), G::SMEM, c.stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t mfma_ffn_fwd(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                        const int32_t* expert_offsets, const void* W1, const float* b1, const void* W2,
                        const float* b2, void* H, void* A, void* O) {
    constexpr int BM = 256, BN = 256;
    const int64_t row_tiles = (s.P_cap + BM - 1) / BM + s.E;
    GemmArgs a{};
    a.expert_offsets = expert_offsets; a.E = s.E; a.P_cap = s.P_cap; a.act = s.act;
    hipError_t err;
    {   // H = X W1^T + b1, A = act(H)
        ProfScope ps(c, EVOMOE_K_FFN_GEMM1);
        a.A = (const bf16_t*)x; a.lda = s.d; a.a_rows = pair_token;
        a.B = (const bf16_t*)W1; a.ldb = s.d; a.b_group_stride = (int64_t)s.F * s.d;
        a.N = s.F; a.K = s.d; a.bias = b1; a.out1 = (bf16_t*)H; a.out2 = (bf16_t*)A;
        err = launch_gemm<L_NT, E_HA, BM, BN>(c, a, row_tiles * ((s.F + BN - 1) / BN));
        if (err != hipSuccess) return err;
    }
    {   // O = A W2^T + b2
        ProfScope ps(c, EVOMOE_K_FFN_GEMM2);
        a.A = (const bf16_t*)A; a.lda = s.F; a.a_rows = nullptr;
        a.B = (const bf16_t*)W2; a.ldb = s.F; a.b_group_stride = (int64_t)s.d * s.F;
        a.N = s.d; a.K = s.F; a.bias = b2; a.out1 = (bf16_t*)O; a.out2 = nullptr;
        err = launch_gemm<L_NT, E_BIAS, BM, BN>(c, a, row_tiles * ((s.d + BN - 1) / BN));
    }
    return err;
}

hipError_t mfma_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H, const void* A,
                        const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                        const void* W1, const void* W2, void* dW1, float* db1, void* dW2, float* db2,
                        void* dXp, int accumulate, void* dH) {
    constexpr int BM = 256, BN = 256;
    const int64_t row_tiles = (s.P_cap + BM - 1) / BM + s.E;
    GemmArgs a{};
    a.expert_offsets = expert_offsets; a.E = s.E; a.P_cap = s.P_cap; a.act = s.act;
    hipError_t err;
    {   // dH = (dO W2) * act'(H)
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DH);
        a.A = (const bf16_t*)dO; a.lda = s.d; a.B = (const bf16_t*)W2; a.ldb = s.F;
        a.b_group_stride = (int64_t)s.d * s.F; a.N = s.F; a.K = s.d; a.Hin = (const bf16_t*)H;
        a.out1 = (bf16_t*)dH;
        err = launch_gemm<L_NN, E_ACTGRAD, BM, BN>(c, a, row_tiles * ((s.F + BN - 1) / BN));
        if (err != hipSuccess) return err;
    }
    {   // dXp = dH W1
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DX);
        a.A = (const bf16_t*)dH; a.lda = s.F; a.B = (const bf16_t*)W1; a.ldb = s.d;
        a.b_group_stride = (int64_t)s.F * s.d; a.N = s.d; a.K = s.F; a.Hin = nullptr;
        a.out1 = (bf16_t*)dXp;
        err = launch_gemm<L_NN, E_NONE, BM, BN>(c, a, row_tiles * ((s.d + BN - 1) / BN));
        if (err != hipSuccess) return err;
    }
    a.accumulate = accumulate;
    if (dW2) {   // dW2_g = dO_g^T A_g   [d,F]
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW2);
        a.A = (const bf16_t*)dO; a.lda = s.d; a.B = (const bf16_t*)A; a.ldb = s.F; a.b_rows = nullptr;
        a.M = s.d; a.N = s.F; a.out1 = (bf16_t*)dW2;
        err = launch_gemm<L_TN, E_WGRAD, BM, BN>(
            c, a, (int64_t)s.E * ((s.d + BM - 1) / BM) * ((s.F + BN - 1) / BN));
        if (err != hipSuccess) return err;
    }
    if (dW1) {   // dW1_g = dH_g^T X_g   [F,d]
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW1);
        a.A = (const bf16_t*)dH; a.lda = s.F; a.B = (const bf16_t*)x; a.ldb = s.d; a.b_rows = pair_token;
        a.M = s.F; a.N = s.d; a.out1 = (bf16_t*)dW1;
        err = launch_gemm<L_TN, E_WGRAD, BM, BN>(
            c, a, (int64_t)s.E * ((s.F + BM - 1) / BM) * ((s.d + BN - 1) / BN));
        if (err != hipSuccess) return err;
    }
    ProfScope ps(c, EVOMOE_K_FFN_BWD_DB);
    if (db2) err = launch_colsum<bf16_t>(c, s, dO, s.d, expert_offsets, db2, accumulate);
    if (err != hipSuccess) return err;
    if (db1) err = launch_colsum<bf16_t>(c, s, dH, s.F, expert_offsets, db1, accumulate);
    return err;
}

}  // namespace evomoe
