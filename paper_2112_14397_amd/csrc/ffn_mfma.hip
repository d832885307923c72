// Expert FFNs on the bf16 matrix cores (EvoMoE Eq. ffn per expert over its ragged row range, and its
// backward).  One grouped-GEMM kernel template, v_mfma_f32_32x32x16_bf16, f32 accumulation:
//
//   NT  C[r,n] = sum_k A[arow(r),k] * W_g[n,k]      forward GEMMs (A rows optionally gathered by token)
//   NN  C[r,n] = sum_k A[r,k]       * W_g[k,n]      dH = dO W2,  dXp = dH W1
//   TN  C_g[m,n] = sum_{r in g} L[r,m] * R[rrow(r),n]   weight gradients (contraction over the ragged rows)
//
// Block = 4 waves (2 x 2) or 8 waves (4 x 2), block tile BM x BN, K slabs of BK, NSTAGE LDS stages filled by direct
// global->LDS loads (no staging registers) that run NSTAGE-1 slabs ahead of the MFMAs.  Operands whose
// contraction index is contiguous in memory sit in LDS as [row][BK k] with an XOR swizzle of the 16-byte
// chunks and are read with ds_read_b128; operands whose contraction index is the row index sit as
// [k][cols] with a swizzle of 32-byte blocks and are read with the transposing LDS load
// (ds_read_b64_tr_b16), so no operand is ever transposed in global memory.  The persistent grid walks
// the tiles in an XCD-aware order.  Epilogues (bias, activation, act'(H) product, accumulate) run in f32
// on a row-major copy of the accumulators staged through LDS, and leave with 16-byte stores.
#include <type_traits>

#include "ffn_internal.h"

namespace evomoe {

namespace {

enum { L_NT = 0, L_NN = 1, L_TN = 2 };
enum { E_HA = 0, E_BIAS = 1, E_ACTGRAD = 2, E_NONE = 3, E_WGRAD = 4 };

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

struct GemmArgs {
    const bf16_t* A;  int64_t lda;      // NT/NN: A rows [*,K];  TN: L [P,M] (lda = M)
    const bf16_t* B;  int64_t ldb;      // NT: W_g [N,K] (ldb = K);  NN: W_g [K,N] (ldb = N);  TN: R [*,N] (ldb = N)
    int64_t b_group_stride;             // NT/NN: elements between two experts' weight matrices
    const int32_t* a_rows;              // NT: gather of A rows (or null)
    const int32_t* expert_offsets;
    int E;
    int64_t P_cap;
    int M, N, K;                        // M: TN only.  K: NT/NN only (TN contracts over the expert's rows)
    const float* bias;                  // [E,N] or null
    const bf16_t* Hin;                  // E_ACTGRAD: pre-activations [P,N]
    const float* row_scale;             // E_ACTGRAD: per-row factor applied in f32 before act' (or null)
    bf16_t* out1;                       // C (H for E_HA)
    bf16_t* out2;                       // E_HA: A = act(H)
    float* colpart;                     // E_ACTGRAD: per-tile column sums of C, [row tile][waves/2][N] (or null)
    int act, accumulate;
    int col_group;                      // NT/NN: column tiles per group of the tile order (1 .. all of them)
};

// ---- LDS geometry -------------------------------------------------------------------------------
// Operand tiles are written by direct global->LDS loads (64 lanes x 16 B land contiguously), so a stage
// is a dense array and bank conflicts are avoided by permuting 16-byte chunks on the global side:
// (the LDS has 64 banks of 4 B: a ds_read_b128 is served 16 lanes = 256 B at a time, a 64-bit read 32 lanes)
//  * k-contiguous tile [R][BK k] bf16: chunk c of row r sits at chunk c ^ key(r), key = (r >> 1) & 7
//    (BK = 64, 128-byte rows) or (r >> 2) & 3 (BK = 32, 64-byte rows): sixteen consecutive rows reading
//    the same k-chunk with ds_read_b128 cover all sixteen 16-byte slots of the 256-byte bank window;
//  * k-strided tile [BK k][C cols] bf16, 2C B per row: 32-byte block b of row k sits at block
//    b ^ 2(k & 3): the transposing read ds_read_b64_tr_b16 has 32 lanes take two adjacent blocks from
//    four consecutive k rows, which then land in eight different 32-byte slots.
template <int LAYOUT, int BM, int BN, int BK, int NSTAGE, int NW = 4> struct Geo {
    static constexpr bool A_KC = (LAYOUT != L_TN);          // A operand k-contiguous?
    static constexpr bool B_KC = (LAYOUT == L_NT);
    static constexpr int A_BYTES = BM * BK * 2;
    static constexpr int B_BYTES = BN * BK * 2;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int WM = BM / (NW / 2), WN = BN / 2;       // waves: (NW/2) x 2
    static constexpr int EPI_LD = WN + 4;                    // f32 row stride of the staging copy
    // rows of the wave tile staged per pass: as many as fit next to nothing else in the operand stages
    static constexpr int EPI_ROWS = (WM >= 64 && NW * 64 * EPI_LD * 4 <= NSTAGE * STAGE + 8192) ? 64 : 32;
    static constexpr int EPI_BYTES = NW * EPI_ROWS * EPI_LD * 4;
    static constexpr int MAIN = (NSTAGE * STAGE > EPI_BYTES ? NSTAGE * STAGE : EPI_BYTES);
    static constexpr int SMEM = MAIN;
};

// Phi(h), the standard normal CDF, as 0.5 + hc*Q(hc^2) with hc = h clamped to |h| <= 4.2: degree-8 minimax
// fit of Q, |error| < 1.2e-5 -- below the resolution of the bf16 values it is multiplied into -- and no
// transcendental.  gelu(h) = h*Phi(h);  gelu'(h) = Phi(h) + h*phi(h).
__device__ __forceinline__ float phi_cdf(float h, float& hc, float& u) {
    hc = __builtin_amdgcn_fmed3f(h, -4.2f, 4.2f);
    u = hc * hc;
    float q = 5.998071484e-11f;
    q = fmaf(q, u, -5.633320033e-09f);
    q = fmaf(q, u, 2.343674907e-07f);
    q = fmaf(q, u, -5.760770819e-06f);
    q = fmaf(q, u, 9.457441047e-05f);
    q = fmaf(q, u, -1.114148065e-03f);
    q = fmaf(q, u, 9.830130264e-03f);
    q = fmaf(q, u, -6.636036932e-02f);
    q = fmaf(q, u, 3.989074528e-01f);
    return fmaf(hc, q, 0.5f);
}
// Beyond the fitted range the values stay within 2.5e-4 of the true ones for any h: gelu(h) -> h for large h
// (Phi(4.2) = 1 - 1.3e-5) and -> max(h, -4.2) * 1.3e-5 for very negative h; gelu'(h) is evaluated at hc, where it
// has reached its limits 1 and 0 to 2.4e-4.
__device__ __forceinline__ float act_fwd_fast(float h, int act) {
    if (act == EVOMOE_RELU) return h > 0.f ? h : 0.f;
    float hc, u;
    const float Phi = phi_cdf(h, hc, u);
    return fmaxf(h, -4.2f) * Phi;
}
__device__ __forceinline__ float act_grad_fast(float h, int act) {
    if (act == EVOMOE_RELU) return h > 0.f ? 1.f : 0.f;
    float hc, u;
    const float Phi = phi_cdf(h, hc, u);
    const float dens = 0.39894228040143267794f * __builtin_amdgcn_exp2f(u * -0.72134752044448170368f);
    return fmaf(hc, dens, Phi);
}

// 16 bytes per lane, global -> LDS, no registers in between: lane l's data lands at lds + 16*l.
// Written as inline assembly on purpose: the compiler cannot tell which LDS stage a load fills, so with
// its own intrinsic it guards every later LDS read (and every barrier) with s_waitcnt vmcnt(0), which
// serialises the prefetch pipeline.  Here the kernel counts its loads itself (wait_vmcnt below).
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// Eight floats -> bf16, one 16-byte store with the streaming (non-temporal) hint: the outputs are far larger
// than the L2 and are not read again by this kernel, while the operand panels they would evict are.
__device__ __forceinline__ void store_out(bf16_t* p, const float* in) {
    u32x4 v = {pack_bf16x2(in[0], in[1]), pack_bf16x2(in[2], in[3]), pack_bf16x2(in[4], in[5]), pack_bf16x2(in[6], in[7])};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
// The global address is a wave-uniform base (an SGPR pair) plus a 32-bit unsigned byte offset per lane.
__device__ __forceinline__ void load_to_lds(const unsigned char* base, uint32_t voff, const unsigned char* lds_wave_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds_addr(lds_wave_base)) : "m0", "memory");
}
// Block barrier that orders LDS traffic only (global loads in flight stay in flight).
__device__ __forceinline__ void block_sync_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// s_waitcnt vmcnt(n) only (other counters left at their maxima)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int LAYOUT, int EPI, int BM, int BN, int BK, int NSTAGE, int WPE, int NW = 4>
__global__ __launch_bounds__(NW * 64, WPE) void grouped_gemm_bf16(GemmArgs q0, GemmArgs q1, int tiles0)
{
    // TN launches carry two independent problems (dW2 and dW1) in one grid, tiles [0, tiles0) and
    // [tiles0, ...), which evens out the last round of the persistent schedule; other layouts use q0 only.
    using G = Geo<LAYOUT, BM, BN, BK, NSTAGE, NW>;
    constexpr int WM = G::WM, WN = G::WN;
    constexpr int TM = WM / 32, TN_ = WN / 32;               // MFMA tiles per wave
    constexpr int KS = BK / 16;                              // k-steps per slab
    constexpr int A_LD = G::A_BYTES / (NW * 1024), B_LD = G::B_BYTES / (NW * 1024);   // 1 KB load instructions per wave per slab
    constexpr int KC_CH = BK / 8, KC_RPI = 64 / KC_CH;       // k-contiguous: 16 B chunks per row, rows per instruction
    constexpr int A_CPR = BM / 8, A_RPI = 64 / A_CPR;        // k-strided A: 16 B chunks per k-row, k-rows per instruction
    constexpr int B_CPR = BN / 8, B_RPI = 64 / B_CPR;
    constexpr int NMF = TM * TN_, NFR = TM + TN_, NLD = A_LD + B_LD;
    constexpr bool SPLIT_LD = NSTAGE >= 3;          // half of a slab's loads before the barrier, half after
    static_assert(BK == 32 || BK == 64, "slab");
    static_assert(NW == 4 || NW == 8, "waves");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && A_LD >= 1 && B_LD >= 1 && NSTAGE >= 2 && KS % 2 == 0, "tile");
    static_assert((NSTAGE - 2) * NLD + (NSTAGE - 1) * 2 <= 63, "vmcnt range");

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int offs[65];

    const int tid = threadIdx.x, lane_id = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: lives in an SGPR
    const int wm = wave >> 1, wn = wave & 1;
    __shared__ int tstart[65];      // NT/NN: number of row tiles before each expert (tstart[E] = all of them)
    if (tid <= q0.E) offs[tid] = clamp_pairs(q0.expert_offsets[tid], q0.P_cap);
    __syncthreads();
    if (LAYOUT != L_TN) {
        if (tid == 0) {
            int acc_t = 0;
            for (int e = 0; e < q0.E; ++e) {
                tstart[e] = acc_t;
                acc_t += (offs[e + 1] - offs[e] + BM - 1) / BM;
            }
            tstart[q0.E] = acc_t;
        }
        __syncthreads();
    }
    int cur_e = 0;                  // expert of the previous tile: row tiles only grow from tile to tile

    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.
    // TN: renumber the blocks so that one XCD works on a run of consecutive tiles per round (the tiles of one
    // expert share its row range).
    // NT/NN: the tile sequence runs expert by expert, inside an expert column group by column group (col_group
    // column tiles whose weight panels fit the L2 together), inside a group row tile by row tile.  When the column
    // tiles are split into groups, every XCD takes one contiguous eighth of that sequence and walks it round by
    // round: the weight panels of a group are fetched into that XCD's L2 once and stay there while the expert's row
    // panels stream past them.
    const bool xcd_split = (gridDim.x & 7) == 0;
    int vblock = blockIdx.x;
    if (xcd_split) vblock = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    int seq = 0, seq_end = 0, seq_step = 0;
    if (LAYOUT != L_TN) {
        const int nct = (q0.N + BN - 1) / BN;
        const int total = tstart[q0.E] * nct;
        if (xcd_split && q0.col_group < nct) {
            const int x = blockIdx.x & 7;
            seq = (int)((int64_t)total * x / 8) + (blockIdx.x >> 3);
            seq_end = (int)((int64_t)total * (x + 1) / 8);
            seq_step = gridDim.x >> 3;
        } else {            // one group holds every column tile: per round, a run of consecutive tiles per XCD
            seq = vblock;
            seq_end = total;
            seq_step = gridDim.x;
        }
    }

    for (int vtile = vblock;; vtile += gridDim.x, seq += seq_step) {
        // ---------------- tile -> (problem, expert, origin, contraction range) ----------------
        const bool second = (LAYOUT == L_TN) && vtile >= tiles0;
        const GemmArgs& p = second ? q1 : q0;
        const int tile = second ? vtile - tiles0 : vtile;
        const int nct = (p.N + BN - 1) / BN;
        const int nmt = (LAYOUT == L_TN) ? (p.M + BM - 1) / BM : 1;
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
            if (seq >= seq_end) break;
            while (seq >= tstart[cur_e + 1] * nct) ++cur_e;      // resumes where the previous tile's search ended
            g = cur_e;
            const int nrt = tstart[g + 1] - tstart[g];           // row tiles of this expert (>= 1 here)
            const int r = seq - tstart[g] * nct;                 // position inside the expert's nrt * nct tiles
            const int cgs = max(1, min(p.col_group, nct));       // column tiles per group
            const int cg = r / (nrt * cgs);
            const int r2 = r - cg * nrt * cgs;
            const int gc = min(cgs, nct - cg * cgs);             // column tiles of this group (the last may be short)
            const int rt_in = r2 / gc;
            n0 = (cg * cgs + (r2 - rt_in * gc)) * BN;
            row0 = offs[g] + rt_in * BM;
            rows = min(BM, offs[g + 1] - row0);
            kbeg = 0;
            kend = p.K;
        }
        // the tile's coordinates came through LDS: tell the compiler they are wave-uniform (SGPRs)
        g = __builtin_amdgcn_readfirstlane(g);
        row0 = __builtin_amdgcn_readfirstlane(row0);
        rows = __builtin_amdgcn_readfirstlane(rows);
        kbeg = __builtin_amdgcn_readfirstlane(kbeg);
        kend = __builtin_amdgcn_readfirstlane(kend);
        const int nslab = (kend - kbeg + BK - 1) / BK;
        const bool ragged = (kend - kbeg) % BK != 0;     // block-uniform: the last slab is partial
        const bf16_t* Bg = (LAYOUT == L_TN) ? p.B : p.B + (int64_t)g * p.b_group_stride;

        // Everything below that depends on the lane is recomputed for every tile from an opaque copy of the lane
        // number: the values then die with the main loop instead of occupying registers through the epilogue.
        int lane_t = lane_id;
        asm volatile("" : "+v"(lane_t));
        const int lane = lane_t;
        // LDS byte offsets of this lane's operand fragments inside one stage (k-step 0), per MFMA tile
        int fa_off[TM], fb_off[TN_];
        const int s16 = lane & 15, l32 = lane & 31, kg = lane >> 5;
    #pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (G::A_KC) {
                fa_off[i] = (wm * WM + i * 32 + l32) * (BK * 2);     // row base; the swizzled chunk is added per k-step
            } else {
                const int lb = (wm * WM + i * 32 + ((lane >> 4) & 1) * 16) >> 4;       // logical 32 B block
                fa_off[i] = (kg * 8 + (s16 >> 2)) * (BM * 2) + ((lb ^ (2 * (s16 >> 2))) << 5) + ((s16 & 3) << 3);
            }
        }
    #pragma unroll
        for (int j = 0; j < TN_; ++j) {
            if (G::B_KC) {
                fb_off[j] = (wn * WN + j * 32 + l32) * (BK * 2);
            } else {
                const int lb = (wn * WN + j * 32 + ((lane >> 4) & 1) * 16) >> 4;
                fb_off[j] = (kg * 8 + (s16 >> 2)) * (BN * 2) + ((lb ^ (2 * (s16 >> 2))) << 5) + ((s16 & 3) << 3);
            }
        }
        // swizzle key of this lane's fragment rows (tile rows start at multiples of 32)
        const int sw = (BK == 64) ? ((l32 >> 1) & 7) : ((l32 >> 2) & 3);

        // This lane's role in the 1 KB load instruction number (wave + NW*i) of a tile (NW waves):
        //   k-contiguous: row (wave+NW i)*KC_RPI + lane/KC_CH, physical chunk lane%KC_CH -> logical chunk ^ key(row)
        //   k-strided   : k-row (wave+NW i)*RPI + lane/CPR, physical chunk lane%CPR -> logical chunk via block ^ (k & 3)
        const int kc_row = lane / KC_CH;
        // key(row) of row (wave + NW i)*KC_RPI + kc_row does not depend on i
        const int kc_key = (BK == 64) ? ((4 * (wave & 1) + (kc_row >> 1)) & 7) : ((kc_row >> 2) & 3);
        const int kc_chunk = (lane % KC_CH) ^ kc_key;                           // logical 16 B chunk (8 k's)
        const int ksA_row = lane / A_CPR, ksB_row = lane / B_CPR;
        auto ks_col = [&](int pc, int krow) { return ((((pc >> 1) ^ (2 * (krow & 3))) << 1) | (pc & 1)) * 8; };

        // ---------------- global addresses: one scalar base per operand + 32-bit per-lane byte offsets ----
        // Rows / columns outside the tile are clamped onto valid ones (their products are never stored);
        // the tail of the contraction range is clamped too and then zeroed in LDS (A operand only).
        // k-contiguous operand: offset of (row, chunk) at k = 0, one register per load instruction.
        // k-strided operand   : offset = k-row * row bytes + column bytes; every load instruction of a lane
        //                       has the same column, its k-row is kr0 + a constant.
        const unsigned char* a_base;
        const unsigned char* b_base;
        uint32_t a_off[G::A_KC ? A_LD : 1], b_off[G::B_KC ? B_LD : 1];
        uint32_t a_col = 0, b_col = 0;                    // k-strided: column byte offset
        if (G::A_KC) {
            a_base = reinterpret_cast<const unsigned char*>(p.A) + (p.a_rows ? (int64_t)0 : (int64_t)row0 * p.lda * 2);
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int r = min((wave + NW * i) * KC_RPI + kc_row, rows - 1);
                const uint32_t ar = p.a_rows ? (uint32_t)p.a_rows[row0 + r] : (uint32_t)r;
                a_off[i] = (ar * (uint32_t)p.lda + kc_chunk * 8) * 2;
            }
        } else {
            a_base = reinterpret_cast<const unsigned char*>(p.A) + (int64_t)kbeg * p.lda * 2;
            a_col = 2 * min(m0 + ks_col(lane % A_CPR, wave * A_RPI + ksA_row), p.M - 8);
        }
        if (G::B_KC) {
            b_base = reinterpret_cast<const unsigned char*>(Bg);
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const int n = min(n0 + (wave + NW * i) * KC_RPI + kc_row, p.N - 1);
                b_off[i] = ((uint32_t)n * (uint32_t)p.ldb + kc_chunk * 8) * 2;
            }
        } else {
            b_base = reinterpret_cast<const unsigned char*>(Bg) + (int64_t)kbeg * p.ldb * 2;
            b_col = 2 * min(n0 + ks_col(lane % B_CPR, wave * B_RPI + ksB_row), p.N - 8);
        }
        const int klen = kend - kbeg;
        const int kc_lim = 2 * (kend - 8 - kc_chunk * 8);        // k-contiguous: last in-range chunk start (bytes)
        const uint32_t lda2 = (uint32_t)p.lda * 2, ldb2 = (uint32_t)p.ldb * 2;
        // issue load instruction `idx` (A: 0..A_LD-1, then B) of slab `slab` into its stage; addresses
        // are clamped into the contraction range (a no-op except in the last, partial slab)
        auto issue_one = [&](int idx, int slab) {
            unsigned char* sa = smem + (slab % NSTAGE) * G::STAGE + wave * 1024;
            unsigned char* sb = sa + G::A_BYTES;
            if (idx < A_LD) {
                const int i = idx;
                if (G::A_KC) {
                    load_to_lds(a_base, a_off[i] + (uint32_t)min(slab * (BK * 2), kc_lim), sa + i * (NW * 1024));
                } else {
                    const int kr = min(slab * BK + (wave + NW * i) * A_RPI + ksA_row, klen - 1);
                    load_to_lds(a_base, __umul24((uint32_t)kr, lda2) + a_col, sa + i * (NW * 1024));
                }
            } else {
                const int i = idx - A_LD;
                if (G::B_KC) {
                    load_to_lds(b_base, b_off[i] + (uint32_t)min(slab * (BK * 2), kc_lim), sb + i * (NW * 1024));
                } else {
                    const int kr = min(slab * BK + (wave + NW * i) * B_RPI + ksB_row, klen - 1);
                    load_to_lds(b_base, __umul24((uint32_t)kr, ldb2) + b_col, sb + i * (NW * 1024));
                }
            }
        };
        auto issue = [&](int slab) {
#pragma unroll
            for (int idx = 0; idx < NLD; ++idx) issue_one(idx, slab);
        };
        // zero the A operand beyond the end of the contraction range (last slab only)
        // (always the tile's last slab: its position comes from the tile, not from the loop counter, so that
        // no per-lane induction variable is carried through the main loop for this rare path)
        auto zero_tail = [&]() {
            const int slab = nslab - 1;
            unsigned char* sa = smem + (slab % NSTAGE) * G::STAGE + wave * 1024;
            const int k0 = kbeg + slab * BK;
            const u32x4 z = {0u, 0u, 0u, 0u};
            if (G::A_KC) {
                if (k0 + kc_chunk * 8 >= kend) {
#pragma unroll
                    for (int i = 0; i < A_LD; ++i) *reinterpret_cast<u32x4*>(sa + i * (NW * 1024) + lane * 16) = z;
                }
            } else {
#pragma unroll
                for (int i = 0; i < A_LD; ++i)
                    if (k0 + (wave + NW * i) * A_RPI + ksA_row >= kend)
                        *reinterpret_cast<u32x4*>(sa + i * (NW * 1024) + lane * 16) = z;
            }
        };
        // operand fragment number f (A tiles 0..TM-1, then B tiles) of k-step ks of slab `slab`
        auto read_frag = [&](int f, int slab, int ks, bf16x8* fa, bf16x8* fb) {
            const unsigned char* sa = smem + (slab % NSTAGE) * G::STAGE;
            const unsigned char* sb = sa + G::A_BYTES;
            if (f < TM) {
                const int i = f;
                if (G::A_KC) {
                    fa[i] = *reinterpret_cast<const bf16x8*>(sa + fa_off[i] + (((ks * 2 + kg) ^ sw) << 4));
                } else {
                    const unsigned char* q = sa + fa_off[i] + ks * 16 * (BM * 2);
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q + 4 * (BM * 2)));
                    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    fa[i] = __builtin_bit_cast(bf16x8, v);
                }
            } else {
                const int j = f - TM;
                if (G::B_KC) {
                    fb[j] = *reinterpret_cast<const bf16x8*>(sb + fb_off[j] + (((ks * 2 + kg) ^ sw) << 4));
                } else {
                    const unsigned char* q = sb + fb_off[j] + ks * 16 * (BN * 2);
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q + 4 * (BN * 2)));
                    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    fb[j] = __builtin_bit_cast(bf16x8, v);
                }
            }
        };

        f32x16 acc[TM][TN_];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN_; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // One k-step: NMF MFMAs on fragments (FA, FB), in 8 groups; after each of the first four groups a
        // share of the next k-step's fragment reads (into NA, NB; slab nslb, k-step nks) is issued, and
        // after every group, optionally, a share of a later slab's global->LDS loads.  The scheduling
        // fences pin this order.
#define KSTEP(FA, FB, READ_NEXT, NA, NB, nslb, nks, LD_LO, LD_HI, lslab)                          \
    _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                              \
        _Pragma("unroll") for (int x = NMF * q / 8; x < NMF * (q + 1) / 8; ++x)                  \
            acc[x / TN_][x % TN_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                     \
                FA[x / TN_], FB[x % TN_], acc[x / TN_][x % TN_], 0, 0, 0);                       \
        if (READ_NEXT && q < 4) {                                                                \
            _Pragma("unroll") for (int f = NFR * q / 4; f < NFR * (q + 1) / 4; ++f)              \
                read_frag(f, nslb, nks, NA, NB);                                                 \
        }                                                                                        \
        _Pragma("unroll") for (int x = (LD_LO) + ((LD_HI) - (LD_LO)) * q / 8;                    \
                               x < (LD_LO) + ((LD_HI) - (LD_LO)) * (q + 1) / 8; ++x)             \
            issue_one(x, lslab);                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                       \
    }

        // previous tile's epilogue has left the LDS; its global stores stay in flight under this tile's
        // first loads (a full barrier would drain them first)
        block_sync_lds();
        // Every load the compiler itself issued during the tile set-up (row indices, spill reloads) has to be
        // complete, and known to it as complete, before the pipeline starts: a wait that it places inside
        // the main loop for one of its own loads would also wait for the tile loads issued there.
        __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0)
        bf16x8 fa0[TM], fb0[TN_], fa1[TM], fb1[TN_];
        if (nslab > 0) {
            // prologue: put NSTAGE-1 slabs in flight, wait for the first
#pragma unroll
            for (int s = 0; s < NSTAGE - 1; ++s) {
                if (s < nslab) issue(s);
            }
            if (nslab >= NSTAGE - 1) wait_vmcnt<(NSTAGE - 2) * NLD>(); else wait_vmcnt<0>();
            block_sync_lds();
            if (nslab == 1 && ragged) {
                zero_tail();
                block_sync_lds();
            }
#pragma unroll
            for (int f = 0; f < NFR; ++f) read_frag(f, 0, 0, fa0, fb0);
        }

        // Slab s: k-steps 0..KS-1 on stage s % NSTAGE.  Fragments of the next k-step are read while the
        // current one multiplies; loads of slab s+NSTAGE-1 go out under k-step 0 into the stage that slab
        // s-1 has finished with; before the last k-step the block makes sure slab s+1 has landed.
        auto slab_body = [&](int slab, auto loads_c) {
            constexpr bool LOADS = decltype(loads_c)::value;
            // with three or more stages the second half of a slab's loads goes out after the barrier
            // (its stage was released one slab earlier), which keeps the load unit evenly busy
            constexpr int L0 = !LOADS ? 0 : (SPLIT_LD ? NLD / 2 : NLD), L1 = LOADS ? NLD : 0;
            KSTEP(fa0, fb0, true, fa1, fb1, slab, 1, 0, L0, slab + NSTAGE - 1);
            if (KS == 4) {
                KSTEP(fa1, fb1, true, fa0, fb0, slab, 2, 0, 0, 0);
                KSTEP(fa0, fb0, true, fa1, fb1, slab, 3, 0, 0, 0);
            }
            // everything issued after slab+1's loads may still be in flight
            if (LOADS) wait_vmcnt<(NSTAGE - 2) * NLD - (NLD - L0)>(); else wait_vmcnt<0>();
            block_sync_lds();
            if (slab + 2 == nslab && ragged) {
                zero_tail();
                block_sync_lds();
            }
            KSTEP(fa1, fb1, true, fa0, fb0, slab + 1, 0, L0, L1, slab + NSTAGE - 1);
        };
        int slab = 0;
        // two blocks per CU: the wave that is feeding the matrix pipe goes ahead of its neighbour's epilogue
        if (WPE > 1) __builtin_amdgcn_s_setprio(1);
        for (; slab + NSTAGE - 1 < nslab; ++slab) slab_body(slab, std::true_type{});
        for (; slab + 1 < nslab; ++slab) slab_body(slab, std::false_type{});
        if (nslab > 0) {           // last slab: nothing left to fetch or to read ahead
            KSTEP(fa0, fb0, true, fa1, fb1, slab, 1, 0, 0, 0);
            if (KS == 4) {
                KSTEP(fa1, fb1, true, fa0, fb0, slab, 2, 0, 0, 0);
                KSTEP(fa0, fb0, true, fa1, fb1, slab, 3, 0, 0, 0);
            }
            KSTEP(fa1, fb1, false, fa0, fb0, 0, 0, 0, 0, 0);
        }
#undef KSTEP
        if (WPE > 1) __builtin_amdgcn_s_setprio(0);
        block_sync_lds();         // every wave is done reading operands: LDS becomes the epilogue's staging area

        // ---------------- epilogue: stage f32 rows through LDS, finish row-major ----------------
        {
        // (a fresh opaque copy of the lane number again: the epilogue's lane constants are not carried through
        //  the main loop either)
        int lane_e = lane_id;
        asm volatile("" : "+v"(lane_e));
        const int lane = lane_e, l32 = lane_e & 31, kg = lane_e >> 5;
        // acc[i][j][r] is C(row = i*32 + 8*(r/4) + 4*kg + r%4, col = j*32 + l32) of the wave tile.
        constexpr int ER = G::EPI_ROWS;
        float* stg = reinterpret_cast<float*>(smem) + wave * (ER * G::EPI_LD);
        constexpr int CPW = WN / 8;                 // 8-column chunks per wave-tile row
        constexpr int RPI = 64 / CPW;               // rows finished per instruction
        constexpr int NIT = ER / RPI;               // store instructions per pass
        constexpr int EPI_UNROLL = NIT <= 8 ? NIT : 4;
        // this lane's 8 columns are the same in every pass and iteration; loads that feed the epilogue are
        // issued ahead of the loop that stores (a load after a store of unknown aliasing is not hoisted)
        const int lc = (lane % CPW) * 8;
        const int col = n0 + wn * WN + lc;
        const int col_c = min(col, p.N - 8);
        float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if ((EPI == E_HA || EPI == E_BIAS) && LAYOUT != L_TN) {
            if (p.bias) {
                const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + (int64_t)g * p.N + col_c);
                const f32x4 b1 = *reinterpret_cast<const f32x4*>(p.bias + (int64_t)g * p.N + col_c + 4);
                bias8[0] = b0.x; bias8[1] = b0.y; bias8[2] = b0.z; bias8[3] = b0.w;
                bias8[4] = b1.x; bias8[5] = b1.y; bias8[6] = b1.z; bias8[7] = b1.w;
            }
        }
        // E_ACTGRAD: column sums of the tile's valid rows (the bias gradient's share of this tile), f32
        float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int pass = 0; pass < WM / ER; ++pass) {
            u32x4 hraw[EPI == E_ACTGRAD ? NIT : 1];
            float rsc[EPI == E_ACTGRAD ? NIT : 1];
            if (EPI == E_ACTGRAD) {
#pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const int trow = min(wm * WM + pass * ER + it * RPI + lane / CPW, rows - 1);
                    hraw[it] = *reinterpret_cast<const u32x4*>(p.Hin + (int64_t)(row0 + trow) * p.N + col_c);
                    rsc[it] = p.row_scale ? p.row_scale[row0 + trow] : 1.f;
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int wrow = i * 32 + 8 * (r >> 2);           // + 4*kg + (r&3) < 8
                    if (wrow / ER != pass) continue;                  // compile-time after unrolling
#pragma unroll
                    for (int j = 0; j < TN_; ++j)
                        stg[(wrow % ER + 4 * kg + (r & 3)) * G::EPI_LD + j * 32 + l32] = acc[i][j][r];
                }
            // this wave's LDS writes are done -- and so are the loads issued above: waiting for them one by
            // one between the stores below would also wait for those stores (one counter covers both)
            if (pass == 0 || EPI == E_ACTGRAD) __builtin_amdgcn_s_waitcnt(0x0070);     // vmcnt(0) lgkmcnt(0)
            else __builtin_amdgcn_s_waitcnt(0xc07f);     // lgkmcnt(0) only: the first pass's stores stay in flight
            __builtin_amdgcn_wave_barrier();
#pragma unroll EPI_UNROLL
            for (int it = 0; it < NIT; ++it) {
                const int lr = it * RPI + lane / CPW;            // row inside the pass
                const int trow = wm * WM + pass * ER + lr;       // row inside the block tile
                const f32x4 v0 = *reinterpret_cast<const f32x4*>(stg + lr * G::EPI_LD + lc);
                const f32x4 v1 = *reinterpret_cast<const f32x4*>(stg + lr * G::EPI_LD + lc + 4);
                float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                // the arithmetic runs for every lane (out-of-tile lanes on clamped addresses); only the
                // stores are predicated, so no wait for a load ends up inside divergent control flow
                if (LAYOUT == L_TN) {
                    const int m = m0 + trow;
                    const bool ok = col < p.N && m < p.M;
                    bf16_t* dst = p.out1 + ((int64_t)g * p.M + min(m, p.M - 1)) * p.N + col_c;
                    if (p.accumulate) {
                        float old[8];
                        Elem<bf16_t>::load_vec(dst, old);
#pragma unroll
                        for (int q = 0; q < 8; ++q) v[q] += old[q];
                    }
                    if (ok) store_out(dst, v);
                } else {
                    const bool ok = col < p.N && trow < rows;
                    const int64_t grow = (int64_t)(row0 + min(trow, rows - 1));
                    if (EPI == E_HA || EPI == E_BIAS) {
#pragma unroll
                        for (int q = 0; q < 8; ++q) v[q] += bias8[q];
                    }
                    if (EPI == E_ACTGRAD) {
                        const u32x4 hw = hraw[it];
                        const float h[8] = {lo_bf16(hw.x), hi_bf16(hw.x), lo_bf16(hw.y), hi_bf16(hw.y),
                                            lo_bf16(hw.z), hi_bf16(hw.z), lo_bf16(hw.w), hi_bf16(hw.w)};
                        // one branch per eight values (not per value): the eight polynomial chains interleave
                        const float sc = rsc[it];
                        if (p.act == EVOMOE_RELU) {
#pragma unroll
                            for (int q = 0; q < 8; ++q) v[q] *= sc * act_grad_fast(h[q], EVOMOE_RELU);
                        } else {
#pragma unroll
                            for (int q = 0; q < 8; ++q) v[q] *= sc * act_grad_fast(h[q], EVOMOE_GELU_ERF);
                        }
                        const float rv = trow < rows ? 1.f : 0.f;     // rows beyond the tile repeat its last row
#pragma unroll
                        for (int q = 0; q < 8; ++q) cs[q] = fmaf(v[q], rv, cs[q]);
                    }
                    if (ok) store_out(p.out1 + grow * p.N + col_c, v);
                    if (EPI == E_HA) {
                        float a[8];
                        if (p.act == EVOMOE_RELU) {
#pragma unroll
                            for (int q = 0; q < 8; ++q) a[q] = act_fwd_fast(v[q], EVOMOE_RELU);
                        } else {
#pragma unroll
                            for (int q = 0; q < 8; ++q) a[q] = act_fwd_fast(v[q], EVOMOE_GELU_ERF);
                        }
                        if (ok) store_out(p.out2 + grow * p.N + col_c, a);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (EPI == E_ACTGRAD && LAYOUT != L_TN) {
            // the RPI lane groups hold different rows of the same columns: add them up, lane group 0 writes
            // this wave's sums (rows wm*WM .. +WM-1 of the tile) as one row of the partial table
            if (p.colpart) {
#pragma unroll
                for (int o = CPW; o < 64; o <<= 1)
#pragma unroll
                    for (int q = 0; q < 8; ++q) cs[q] += __shfl_xor(cs[q], o, 64);
                if (lane < CPW && col < p.N) {
                    const int rt = tstart[g] + (row0 - offs[g]) / BM;
                    float* dst = p.colpart + ((int64_t)rt * (NW / 2) + wm) * p.N + col_c;
                    *reinterpret_cast<f32x4*>(dst) = f32x4{cs[0], cs[1], cs[2], cs[3]};
                    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{cs[4], cs[5], cs[6], cs[7]};
                }
            }
        }
        }
    }
}

// Both bias gradients in one launch.  The first E * gx1 blocks (expert g = b / gx1, 256 columns each):
// db1[g, n] (+)= sum over expert g's row tiles (`parts` partial rows each) of the per-tile column sums written by the
// dH GEMM, in row order.  The remaining blocks: db2[i] (+)= sum over the splits of the streaming column sums of
// dO, in split order.  Reproducible bit for bit.
__global__ __launch_bounds__(256) void bias_grad_final_kernel(
    const float* __restrict__ part1, const int32_t* __restrict__ expert_offsets, int E, int64_t P_cap, int N1,
    int BM, int parts, int gx1, float* __restrict__ db1, const float* __restrict__ part2, size_t n2, float* __restrict__ db2,
    int accumulate)
{
    if ((int)blockIdx.x >= E * gx1) {
        const size_t i = (size_t)(blockIdx.x - E * gx1) * 256 + threadIdx.x;
        if (i >= n2) return;
        float s = accumulate ? db2[i] : 0.f;
        for (int k0 = 0; k0 < kColsumSplit; k0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part2[(size_t)(k0 + u) * n2 + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        db2[i] = s;
        return;
    }
    const int g = blockIdx.x / gx1;
    const int n = (blockIdx.x % gx1) * 256 + threadIdx.x;
    __shared__ int offs[65];
    if ((int)threadIdx.x <= E) offs[threadIdx.x] = clamp_pairs(expert_offsets[threadIdx.x], P_cap);
    __syncthreads();
    if (n >= N1) return;
    int t0 = 0;                          // first row tile of expert g
    for (int e = 0; e < g; ++e) t0 += (offs[e + 1] - offs[e] + BM - 1) / BM;
    const int nt = (offs[g + 1] - offs[g] + BM - 1) / BM;
    const float* src = part1 + (int64_t)t0 * parts * N1 + n;
    float sum = accumulate ? db1[(int64_t)g * N1 + n] : 0.f;
    int i = 0;
    for (; i + 8 <= parts * nt; i += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(i + u) * N1];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
    }
    for (; i < parts * nt; ++i) sum += src[(int64_t)i * N1];
    db1[(int64_t)g * N1 + n] = sum;
}

// Tile configurations.  BIG4: one block per compute unit, 256 accumulator registers per lane.
// OCT: the same tile and stages worked by eight waves (64x128 each, two per SIMD, 128 accumulator registers): 4 %
// faster than BIG4 for GEMM1 and 1 % for the weight gradients, 2 % slower for GEMM2, the same for dXp.
// DUO: two blocks per compute unit (one's epilogue and stalls hide under the other's MFMAs).
// LAT: for launches with no more tiles than compute units and a long contraction: what counts then is how fast
// one block walks its K loop, and 64-wide slabs halve the number of load/barrier rounds of that walk.
struct CfgDuo { static constexpr int BM = 128, BN = 256, BK = 32, NSTAGE = 3, WPE = 2, NW = 4; };
struct CfgBig4 { static constexpr int BM = 256, BN = 256, BK = 32, NSTAGE = 4, WPE = 1, NW = 4; };
struct CfgOct { static constexpr int BM = 256, BN = 256, BK = 32, NSTAGE = 4, WPE = 1, NW = 8; };
struct CfgLat { static constexpr int BM = 128, BN = 256, BK = 64, NSTAGE = 3, WPE = 1, NW = 4; };

template <int LAYOUT, int EPI, class Cfg>
hipError_t launch_gemm(const Ctx& c, const GemmArgs& a0, int64_t tiles0, const GemmArgs& a1, int64_t tiles1) {
    using G = Geo<LAYOUT, Cfg::BM, Cfg::BN, Cfg::BK, Cfg::NSTAGE, Cfg::NW>;
    auto kern = grouped_gemm_bf16<LAYOUT, EPI, Cfg::BM, Cfg::BN, Cfg::BK, Cfg::NSTAGE, Cfg::WPE, Cfg::NW>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::SMEM);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int64_t cap = (int64_t)c.num_cu * Cfg::WPE, worst = tiles0 + tiles1;
    const int grid = (int)(worst < cap ? worst : cap);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::NW * 64), G::SMEM, c.stream, a0, a1, (int)tiles0);
    return hipGetLastError();
}
template <int LAYOUT, int EPI, class Cfg>
hipError_t launch_gemm(const Ctx& c, const GemmArgs& a, int64_t worst_tiles) {
    return launch_gemm<LAYOUT, EPI, Cfg>(c, a, worst_tiles, a, 0);
}

// Worst-case number of row tiles (launch grids and tables are sized for P_cap rows) ...
template <class Cfg> int64_t row_tiles(const evomoe_shape& s) { return (s.P_cap + Cfg::BM - 1) / Cfg::BM + s.E; }
template <class Cfg> int64_t ctiles(int n) { return (n + Cfg::BN - 1) / Cfg::BN; }
template <class Cfg> int64_t mtiles(int m) { return (m + Cfg::BM - 1) / Cfg::BM; }
// ... and the number expected: the tile shape is chosen for the pair count the caller announced
// (evomoe_hint_pairs; the capacity when it announced none).  Any shape is correct for any pair count.
inline int64_t expected_pairs(const Ctx& c, const evomoe_shape& s) {
    return c.pair_hint > 0 && c.pair_hint < s.P_cap ? c.pair_hint : s.P_cap;
}
template <class Cfg> int64_t expected_row_tiles(const Ctx& c, const evomoe_shape& s) {
    return (expected_pairs(c, s) + Cfg::BM - 1) / Cfg::BM + s.E / 2;
}

using CfgGemm1 = CfgOct;
using CfgGemm2 = CfgBig4;
using CfgDh = CfgDuo;
using CfgDx = CfgBig4;
using CfgDw = CfgOct;

// Column tiles per group of the NT/NN tile order: as many weight panels (BN x K) as stay in one XCD's 4 MB L2 next to
// the row panels streaming past them; all of them when a row panel (BM x K) is itself so large (long contractions)
// that reading it once per group would cost more than re-reading the weights.
template <class Cfg> int col_group_for(int n, int k) {
    const int nct = (int)ctiles<Cfg>(n);
    if ((int64_t)Cfg::BM * k * 2 >= (1 << 20)) return nct;
    const int64_t fit = (int64_t)(2.4 * 1024 * 1024) / ((int64_t)Cfg::BN * k * 2);
    return (int)(fit < 1 ? 1 : (fit > nct ? nct : fit));
}

// Choice of tile shape per launch.  A persistent grid works through its tiles in rounds (one tile per resident
// block), so a launch takes about rounds x (time of one tile): the finer 128-row tiles lose a little per flop but
// waste less in the last, partly filled round and in the padding of each expert's last row tile.  The relative
// tile times below were measured on the GPT-shaped layer (d = 768, F = 3072) at pair counts from 8 k to 58 k: a
// 128x256x64 tile with a CU to itself takes 0.53 (NT) / 0.63 (NN) of a 256x256x32 tile; two co-resident 128x256x32
// blocks take 1.06-1.2 times as long per round as one eight-wave 256x256 block when the contraction is short
// (priced at 1.15; 1.2x and more when it is long, which never pays).  The weight-gradient launch and the act'(H)
// launch keep one shape each: 256x256 tiles were 8-29 % faster than either 128-row shape for the former, and for
// the latter two co-resident blocks are almost twice as fast as a four-wave 256x256 block and 2 % faster than an
// eight-wave one.
template <class Cfg> double launch_cost(const Ctx& c, const evomoe_shape& s, int n, double tile_time) {
    const int64_t tiles = expected_row_tiles<Cfg>(c, s) * ctiles<Cfg>(n);
    const int64_t slots = (int64_t)c.num_cu * Cfg::WPE;
    return (double)((tiles + slots - 1) / slots) * tile_time;
}
enum class Tile { Big, Duo, Lat };
// short contraction (GEMM1): 256-row tiles or two co-resident 128-row blocks
inline Tile pick_short_k(const Ctx& c, const evomoe_shape& s, int n) {
    return launch_cost<CfgDuo>(c, s, n, 1.15) < launch_cost<CfgGemm1>(c, s, n, 1.0) ? Tile::Duo : Tile::Big;
}
// long contraction (GEMM2, dXp): 256-row tiles or 128-row tiles with 64-wide slabs, one block per CU
inline Tile pick_long_k(const Ctx& c, const evomoe_shape& s, int n, double lat_time) {
    return launch_cost<CfgLat>(c, s, n, lat_time) < launch_cost<CfgBig4>(c, s, n, 1.0) ? Tile::Lat : Tile::Big;
}

}  // namespace

// per-tile column sums of dH: one row of F floats per wave row of each row tile of the dH GEMM
size_t dh_colpart_bytes(const evomoe_shape& s) {
    if (s.dtype != EVOMOE_BF16) return 0;
    return ((size_t)row_tiles<CfgDh>(s) * (CfgDh::NW / 2) * s.F * sizeof(float) + 255) & ~(size_t)255;
}

hipError_t mfma_ffn_fwd(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                        const int32_t* expert_offsets, const void* W1, const float* b1, const void* W2,
                        const float* b2, void* H, void* A, void* O) {
    GemmArgs a{};
    a.expert_offsets = expert_offsets; a.E = s.E; a.P_cap = s.P_cap; a.act = s.act;
    hipError_t err;
    {   // H = X W1^T + b1, A = act(H)
        using Cfg = CfgGemm1;
        ProfScope ps(c, EVOMOE_K_FFN_GEMM1);
        a.A = (const bf16_t*)x; a.lda = s.d; a.a_rows = pair_token;
        a.B = (const bf16_t*)W1; a.ldb = s.d; a.b_group_stride = (int64_t)s.F * s.d;
        a.N = s.F; a.K = s.d; a.bias = b1; a.out1 = (bf16_t*)H; a.out2 = (bf16_t*)A;
        a.col_group = col_group_for<Cfg>(s.F, s.d);
        if (pick_short_k(c, s, s.F) == Tile::Duo)
            err = launch_gemm<L_NT, E_HA, CfgDuo>(c, a, row_tiles<CfgDuo>(s) * ctiles<CfgDuo>(s.F));
        else
            err = launch_gemm<L_NT, E_HA, Cfg>(c, a, row_tiles<Cfg>(s) * ctiles<Cfg>(s.F));
        if (err != hipSuccess || !O) return err;      // O == nullptr: recomputation of H and A only
    }
    {   // O = A W2^T + b2
        using Cfg = CfgGemm2;
        ProfScope ps(c, EVOMOE_K_FFN_GEMM2);
        a.A = (const bf16_t*)A; a.lda = s.F; a.a_rows = nullptr;
        a.B = (const bf16_t*)W2; a.ldb = s.F; a.b_group_stride = (int64_t)s.d * s.F;
        a.N = s.d; a.K = s.F; a.bias = b2; a.out1 = (bf16_t*)O; a.out2 = nullptr;
        a.col_group = col_group_for<Cfg>(s.d, s.F);
        if (pick_long_k(c, s, s.d, 0.53) == Tile::Lat)
            err = launch_gemm<L_NT, E_BIAS, CfgLat>(c, a, row_tiles<CfgLat>(s) * ctiles<CfgLat>(s.d));
        else
            err = launch_gemm<L_NT, E_BIAS, Cfg>(c, a, row_tiles<Cfg>(s) * ctiles<Cfg>(s.d));
    }
    return err;
}

hipError_t mfma_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H, const void* A,
                        const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                        const void* W1, const void* W2, const void* dy, const float* pair_gate, void* dW1,
                        float* db1, void* dW2, float* db2, void* dXp, int accumulate, void* dH) {
    GemmArgs a{};
    a.expert_offsets = expert_offsets; a.E = s.E; a.P_cap = s.P_cap; a.act = s.act;
    hipError_t err;
    // workspace behind dH: [column-sum partials of the streaming kernel][per-tile column sums of dH][gathered x]
    float* scratch = reinterpret_cast<float*>(static_cast<char*>(dH) + dh_bytes(s));
    float* colpart = reinterpret_cast<float*>(static_cast<char*>(dH) + dh_bytes(s) + colsum_scratch_bytes(s) -
                                              dh_colpart_bytes(s));
    {   // dH = (dO W2) * act'(H); its epilogue also leaves the column sums of every tile (for db1).
        // With dy and the pair weights at hand, dO W2 is taken as G_r * (dy[token(r)] W2): the rows of dy are
        // gathered on load and the weight is applied to the f32 accumulators, so that the rounding of the stored
        // dO (a product rounded to bf16) does not reach dH, dXp, dW1 and db1.
        using Cfg = CfgDh;
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DH);
        const bool from_dy = dy && pair_gate && pair_token;
        a.A = (const bf16_t*)(from_dy ? dy : dO); a.lda = s.d; a.a_rows = from_dy ? pair_token : nullptr;
        a.row_scale = from_dy ? pair_gate : nullptr;
        a.B = (const bf16_t*)W2; a.ldb = s.F;
        a.b_group_stride = (int64_t)s.d * s.F; a.N = s.F; a.K = s.d; a.Hin = (const bf16_t*)H;
        a.out1 = (bf16_t*)dH; a.colpart = db1 ? colpart : nullptr;
        a.col_group = col_group_for<Cfg>(s.F, s.d);
        err = launch_gemm<L_NN, E_ACTGRAD, Cfg>(c, a, row_tiles<Cfg>(s) * ctiles<Cfg>(s.F));
        a.colpart = nullptr; a.a_rows = nullptr; a.row_scale = nullptr;
        if (err != hipSuccess) return err;
    }
    {   // dXp = dH W1
        using Cfg = CfgDx;
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DX);
        a.A = (const bf16_t*)dH; a.lda = s.F; a.B = (const bf16_t*)W1; a.ldb = s.d;
        a.b_group_stride = (int64_t)s.F * s.d; a.N = s.d; a.K = s.F; a.Hin = nullptr;
        a.out1 = (bf16_t*)dXp;
        a.col_group = col_group_for<Cfg>(s.d, s.F);
        if (pick_long_k(c, s, s.d, 0.63) == Tile::Lat)
            err = launch_gemm<L_NN, E_NONE, CfgLat>(c, a, row_tiles<CfgLat>(s) * ctiles<CfgLat>(s.d));
        else
            err = launch_gemm<L_NN, E_NONE, Cfg>(c, a, row_tiles<Cfg>(s) * ctiles<Cfg>(s.d));
        if (err != hipSuccess) return err;
    }
    a.accumulate = accumulate;
    using CfgW = CfgDw;
    GemmArgs w2 = a, w1 = a;
    // dW2_g = dO_g^T A_g   [d,F]
    w2.A = (const bf16_t*)dO; w2.lda = s.d; w2.B = (const bf16_t*)A; w2.ldb = s.F;
    w2.M = s.d; w2.N = s.F; w2.out1 = (bf16_t*)dW2;
    const int64_t t2 = (int64_t)s.E * mtiles<CfgW>(s.d) * ctiles<CfgW>(s.F);
    // dW1_g = dH_g^T X_g   [F,d]; the token rows are gathered once into a dense copy so that the GEMM
    // streams them like any other operand
    const bf16_t* xg = (const bf16_t*)x;
    if (dW1 && pair_token) {
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW1);
        bf16_t* xp = reinterpret_cast<bf16_t*>(static_cast<char*>(dH) + dh_bytes(s) + colsum_scratch_bytes(s));
        err = launch_gather_rows(c, s, x, pair_token, expert_offsets, xp);
        if (err != hipSuccess) return err;
        xg = xp;
    }
    w1.A = (const bf16_t*)dH; w1.lda = s.F; w1.B = xg; w1.ldb = s.d;
    w1.M = s.F; w1.N = s.d; w1.out1 = (bf16_t*)dW1;
    const int64_t t1 = (int64_t)s.E * mtiles<CfgW>(s.F) * ctiles<CfgW>(s.d);
    if (dW2 && dW1) {
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW2);
        err = launch_gemm<L_TN, E_WGRAD, CfgW>(c, w2, t2, w1, t1);
    } else if (dW2) {
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW2);
        err = launch_gemm<L_TN, E_WGRAD, CfgW>(c, w2, t2);
    } else if (dW1) {
        ProfScope ps(c, EVOMOE_K_FFN_BWD_DW1);
        err = launch_gemm<L_TN, E_WGRAD, CfgW>(c, w1, t1);
    }
    if (err != hipSuccess) return err;
    ProfScope ps(c, EVOMOE_K_FFN_BWD_DB);
    if (db2) err = launch_colsum_part<bf16_t>(c, s, dO, s.d, expert_offsets, scratch);
    if (err != hipSuccess) return err;
    if (db1 || db2) {
        // one launch finishes both: E * gx1 blocks for db1 (if wanted), then gx2 blocks for db2 (if wanted)
        const size_t n2 = db2 ? (size_t)s.E * s.d : 0;
        const int gx1 = db1 ? (s.F + 255) / 256 : 0, gx2 = (int)((n2 + 255) / 256);
        hipLaunchKernelGGL(bias_grad_final_kernel, dim3(s.E * gx1 + gx2), dim3(256), 0, c.stream, colpart,
                           expert_offsets, s.E, s.P_cap, s.F, (int)CfgDh::BM, (int)CfgDh::NW / 2, gx1, db1, scratch, n2, db2,
                           accumulate);
        err = hipGetLastError();
    }
    return err;
}

}  // namespace evomoe
