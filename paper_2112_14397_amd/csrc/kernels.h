// Host-side launchers of the gfx950 kernels (one per step of the layer).  Internal to the library.
#pragma once
#include "common.h"

namespace evomoe {

// gate.hip
hipError_t launch_dts_gate(const Ctx& c, const evomoe_shape& s, const void* x, const float* Wg,
                           const float* bg, const float* noise, float tau, float threshold,
                           float* gprime, float* gate_w, uint64_t* mask_bits, int32_t* counts,
                           int32_t* k_per_token, int32_t* block_hist);
hipError_t launch_dts_gate_bwd(const Ctx& c, const evomoe_shape& s, const float* dG_pairs,
                               const int32_t* tok_off, const int32_t* tok_rows, const float* gprime,
                               const uint64_t* mask_bits, float tau, const void* x, const float* Wg,
                               float* dWg, float* dbg, void* dx, void* workspace,
                               const float* dgprime_coef = nullptr, float coef_scale = 0.f);
size_t gate_bwd_workspace_bytes(const evomoe_shape& s);
// balance loss: scratch holds balance_blocks(s) * E floats of per-block column sums of g'
int balance_blocks(const evomoe_shape& s);
hipError_t launch_balance_loss(const Ctx& c, const evomoe_shape& s, const float* gprime, const int32_t* counts,
                               float alpha, float* loss, float* dgprime_coef);

// dispatch.hip
hipError_t launch_dispatch(const Ctx& c, const evomoe_shape& s, const uint64_t* mask_bits,
                           const float* scores, const int32_t* block_hist, int32_t* expert_offsets,
                           int32_t* pair_token, float* pair_gate, int32_t* tok_off, int32_t* tok_rows,
                           int64_t* num_pairs, const void* x, void* x_perm, int32_t* hist_scratch);
int dispatch_blocks(const evomoe_shape& s);     // 256-token groups: rows of a block_hist table
// device address, on `device` (which must be current), of the library's static histogram table
hipError_t static_hist_table(int device, int32_t** table);
hipError_t launch_gather_rows(const Ctx& c, const evomoe_shape& s, const void* x, const int32_t* pair_token,
                              const int32_t* expert_offsets, void* x_perm);   // x_perm[r,:] = x[pair_token[r],:]
hipError_t launch_dispatch_bwd(const Ctx& c, const evomoe_shape& s, const void* dXp,
                               const int32_t* tok_off, const int32_t* tok_rows, void* dx);

// diversify.hip
hipError_t launch_diversify(const Ctx& c, const evomoe_shape& s, const void* W1s, const float* b1s, const void* W2s,
                            const float* b2s, uint64_t seed, float mask_ratio, void* W1, float* b1, void* W2,
                            float* b2);

// combine.hip
hipError_t launch_combine(const Ctx& c, const evomoe_shape& s, const void* O, const float* pair_gate,
                          const int32_t* tok_off, const int32_t* tok_rows, void* y);
hipError_t launch_combine_bwd(const Ctx& c, const evomoe_shape& s, const void* dy, const void* O,
                              const float* pair_gate, const int32_t* pair_token,
                              const int32_t* expert_offsets, void* dO, float* dG_pairs);

// ffn.hip
hipError_t launch_expert_ffn(const Ctx& c, const evomoe_shape& s, const void* x,
                             const int32_t* pair_token, const int32_t* expert_offsets, const void* W1,
                             const float* b1, const void* W2, const float* b2, void* H, void* A, void* O);
hipError_t launch_expert_ffn_bwd(const Ctx& c, const evomoe_shape& s, const void* dO, const void* H,
                                 const void* A, const void* x, const int32_t* pair_token,
                                 const int32_t* expert_offsets, const void* W1, const void* W2,
                                 const void* dy, const float* pair_gate,
                                 void* dW1, float* db1, void* dW2, float* db2, void* dXp,
                                 int accumulate, void* workspace);
size_t ffn_bwd_workspace_bytes(const evomoe_shape& s);
size_t ffn_bwd_recompute_workspace_bytes(const evomoe_shape& s);
hipError_t launch_expert_ffn_bwd_recompute(const Ctx& c, const evomoe_shape& s, const void* dO, const void* x,
                                           const int32_t* pair_token, const int32_t* expert_offsets,
                                           const void* W1, const float* b1, const void* W2, const void* dy,
                                           const float* pair_gate, void* dW1,
                                           float* db1, void* dW2, float* db2, void* dXp, int accumulate,
                                           void* workspace);

}  // namespace evomoe
