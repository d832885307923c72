// Expert FFNs: choice of kernel family per storage type.
#include "ffn_internal.h"

namespace evomoe {

size_t ffn_bwd_workspace_bytes(const evomoe_shape& s) {
    // [dH][bias-gradient partials][gathered copy of x for the dW1 GEMM (bf16 layer)]
    const size_t xp = s.dtype == EVOMOE_BF16 ? (size_t)s.P_cap * s.d * 2 : 0;
    return dh_bytes(s) + colsum_scratch_bytes(s) + xp;
}

hipError_t launch_expert_ffn(const Ctx& c, const evomoe_shape& s, const void* x,
                             const int32_t* pair_token, const int32_t* expert_offsets, const void* W1,
                             const float* b1, const void* W2, const float* b2, void* H, void* A, void* O) {
    if (s.dtype == EVOMOE_BF16)
        return mfma_ffn_fwd(c, s, x, pair_token, expert_offsets, W1, b1, W2, b2, H, A, O);
    return simple_ffn_fwd<float>(c, s, x, pair_token, expert_offsets, W1, b1, W2, b2, H, A, O);
}

hipError_t launch_expert_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H,
                                 const void* A, const void* x, const int32_t* pair_token,
                                 const int32_t* expert_offsets, const void* W1, const void* W2,
                                 const void* dy, const float* pair_gate,
                                 void* dW1, float* db1, void* dW2, float* db2, void* dXp,
                                 int accumulate, void* workspace) {
    if (s.dtype == EVOMOE_BF16)
        return mfma_ffn_bwd(c, s, dO, H, A, x, pair_token, expert_offsets, W1, W2, dy, pair_gate, dW1, db1,
                            dW2, db2, dXp, accumulate, workspace);
    return simple_ffn_bwd<float>(c, s, dO, H, A, x, pair_token, expert_offsets, W1, W2, dW1, db1, dW2,
                                 db2, dXp, accumulate, workspace);
}

// Recompute variant: workspace = [H : P_cap x F][A : P_cap x F][the plain backward's workspace].
static size_t act_bytes(const evomoe_shape& s) { return dh_bytes(s); }
size_t ffn_bwd_recompute_workspace_bytes(const evomoe_shape& s) {
    return 2 * act_bytes(s) + ffn_bwd_workspace_bytes(s);
}
hipError_t launch_expert_ffn_bwd_recompute(const Ctx& c, const evomoe_shape& s, const void* dO, const void* x,
                                           const int32_t* pair_token, const int32_t* expert_offsets,
                                           const void* W1, const float* b1, const void* W2, const void* dy,
                                           const float* pair_gate, void* dW1,
                                           float* db1, void* dW2, float* db2, void* dXp, int accumulate,
                                           void* workspace) {
    char* w = static_cast<char*>(workspace);
    void* H = w;
    void* A = w + act_bytes(s);
    void* rest = w + 2 * act_bytes(s);
    hipError_t err = launch_expert_ffn(c, s, x, pair_token, expert_offsets, W1, b1, W2, nullptr, H, A, nullptr);
    if (err != hipSuccess) return err;
    return launch_expert_ffn_bwd(c, s, dO, H, A, x, pair_token, expert_offsets, W1, W2, dy, pair_gate, dW1, db1,
                                 dW2, db2, dXp, accumulate, rest);
}

}  // namespace evomoe
