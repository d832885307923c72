// Launchers shared between the expert-FFN translation units.  Internal to the library.
#pragma once
#include "kernels.h"

namespace evomoe {

template <typename TX>
hipError_t simple_ffn_fwd(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                          const int32_t* expert_offsets, const void* W1, const float* b1,
                          const void* W2, const float* b2, void* H, void* A, void* O);
template <typename TX>
hipError_t simple_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H,
                          const void* A, const void* x, const int32_t* pair_token,
                          const int32_t* expert_offsets, const void* W1, const void* W2, void* dW1,
                          float* db1, void* dW2, float* db2, void* dXp, int accumulate, void* dH);
template <typename TX>
hipError_t launch_colsum(const Ctx& c, const evomoe_shape& s, const void* Mx, int N,
                         const int32_t* expert_offsets, float* db, int accumulate, float* scratch);
// the streaming column sums split every expert's rows into this many ranges: part[split][g][n], added in order
constexpr int kColsumSplit = 32;
// first pass only: leaves part[kColsumSplit][E][N] in scratch
template <typename TX>
hipError_t launch_colsum_part(const Ctx& c, const evomoe_shape& s, const void* Mx, int N,
                              const int32_t* expert_offsets, float* scratch);
// [partials of the streaming column sums][bf16 layer: per-tile column sums of dH]; a multiple of 256
size_t colsum_scratch_bytes(const evomoe_shape& s);
size_t dh_colpart_bytes(const evomoe_shape& s);       // the second part alone (0 for a float32 layer)
// the backward workspace is [dH : P_cap x F elements, rounded up to 256 B][bias-gradient partial sums]
inline size_t dh_bytes(const evomoe_shape& s) {
    const size_t esz = s.dtype == EVOMOE_BF16 ? 2 : 4;
    return ((size_t)s.P_cap * s.F * esz + 255) & ~(size_t)255;
}

// bf16 matrix-core path (ffn_mfma.hip)
hipError_t mfma_ffn_fwd(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                        const int32_t* expert_offsets, const void* W1, const float* b1, const void* W2,
                        const float* b2, void* H, void* A, void* O);
hipError_t mfma_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H, const void* A,
                        const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                        const void* W1, const void* W2, const void* dy, const float* pair_gate, void* dW1,
                        float* db1, void* dW2, float* db2, void* dXp, int accumulate, void* dH);

}  // namespace evomoe
