// C ABI of the DTS-Gate MoE layer: argument validation, context, and hand-off to the kernel launchers.
#include <new>

#include "kernels.h"

using namespace evomoe;

struct evomoe_ctx {
    Ctx c;
};

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

evomoe_status check_shape(const evomoe_shape* s) {
    if (!s) return EVOMOE_EINVAL;
    if (s->T <= 0 || s->d <= 0 || s->E <= 0 || s->F <= 0 || s->P_cap <= 0) return EVOMOE_EINVAL;
    if (s->dtype != EVOMOE_F32 && s->dtype != EVOMOE_BF16) return EVOMOE_EINVAL;
    if (s->act != EVOMOE_RELU && s->act != EVOMOE_GELU_ERF) return EVOMOE_EINVAL;
    if (s->E > 64) return EVOMOE_EUNSUPPORTED;
    const int vec = s->dtype == EVOMOE_BF16 ? 8 : 4;
    if (s->d % vec || s->F % vec) return EVOMOE_EUNSUPPORTED;
    if ((int64_t)s->T * s->E > INT32_MAX || s->P_cap > INT32_MAX) return EVOMOE_EUNSUPPORTED;
    return EVOMOE_OK;
}

// Extra limits of the bf16 expert FFN: its MFMA kernels address operands as a 64-bit tile base plus 32-bit
// byte offsets per lane, and their k-contiguous tiles need at least one full 64-wide slab.
evomoe_status check_ffn_shape(const evomoe_shape* s) {
    if (s->dtype != EVOMOE_BF16) return EVOMOE_OK;
    const int64_t lim = (int64_t)1 << 32, wide = s->d > s->F ? s->d : s->F;
    if (s->d < 64 || s->F < 64 || s->T >= (1 << 24)) return EVOMOE_EUNSUPPORTED;
    if ((int64_t)s->T * wide * 2 >= lim || (int64_t)s->d * s->F * 2 >= lim) return EVOMOE_EUNSUPPORTED;
    return EVOMOE_OK;
}

#define REQUIRE_PTR(p) \
    do { if (!(p) || !aligned16(p)) return EVOMOE_EINVAL; } while (0)
#define OPTIONAL_PTR(p) \
    do { if ((p) && !aligned16(p)) return EVOMOE_EINVAL; } while (0)
#define CHECK_CTX_SHAPE()                                  \
    do {                                                   \
        if (!ctx) return EVOMOE_EINVAL;                    \
        evomoe_status st_ = check_shape(shape);            \
        if (st_ != EVOMOE_OK) return st_;                  \
    } while (0)

evomoe_status from_hip(hipError_t e) { return e == hipSuccess ? EVOMOE_OK : EVOMOE_EHIP; }

// Make sure the context's histogram scratch holds `elems` ints (grows with a device allocation).
evomoe_status ensure_scratch(Ctx& c, size_t elems) {
    if (elems <= c.block_counts_elems) return EVOMOE_OK;
    if (c.block_counts) {
        if (hipStreamSynchronize(c.stream) != hipSuccess) return EVOMOE_EHIP;
        if (hipFree(c.block_counts) != hipSuccess) return EVOMOE_EHIP;
        c.block_counts = nullptr;
        c.block_counts_elems = 0;
    }
    size_t want = elems < 65536 ? 65536 : elems;
    if (hipMalloc(&c.block_counts, want * sizeof(int32_t)) != hipSuccess) return EVOMOE_EHIP;
    c.block_counts_elems = want;
    return EVOMOE_OK;
}

// Scratch of the bf16 gate (split copy of W_g); grows with a device allocation when a larger d*E shows up.
evomoe_status ensure_wg_planes(Ctx& c, size_t bytes) {
    if (bytes <= c.wg_planes_bytes) return EVOMOE_OK;
    if (c.wg_planes) {
        if (hipStreamSynchronize(c.stream) != hipSuccess) return EVOMOE_EHIP;
        if (hipFree(c.wg_planes) != hipSuccess) return EVOMOE_EHIP;
        c.wg_planes = nullptr;
        c.wg_planes_bytes = 0;
    }
    const size_t want = bytes < (1u << 20) ? (1u << 20) : bytes;
    if (hipMalloc(&c.wg_planes, want) != hipSuccess) return EVOMOE_EHIP;
    c.wg_planes_bytes = want;
    return EVOMOE_OK;
}

}  // namespace

extern "C" {

evomoe_status evomoe_create(evomoe_ctx** ctx_out, void* hip_stream) {
    if (!ctx_out) return EVOMOE_EINVAL;
    *ctx_out = nullptr;
    evomoe_ctx* ctx = new (std::nothrow) evomoe_ctx();
    if (!ctx) return EVOMOE_EHIP;
    Ctx& c = ctx->c;
    c.stream = (hipStream_t)hip_stream;
    c.block_counts = nullptr;
    c.block_counts_elems = 0;
    c.wg_planes = nullptr;
    c.wg_planes_bytes = 0;
    c.status_dev = nullptr;
    c.prof = nullptr;
    c.pair_hint = 0;
    hipDeviceProp_t prop;
    int32_t* small = nullptr;
    if (hipGetDevice(&c.device) != hipSuccess || hipGetDeviceProperties(&prop, c.device) != hipSuccess ||
        hipMalloc(&small, 256) != hipSuccess) {
        delete ctx;
        return EVOMOE_EHIP;
    }
    c.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // device address of the static histogram table of evomoe_dispatch_static, looked up once per device
    c.static_hist = nullptr;
    (void)static_hist_table(c.device, &c.static_hist);
    c.status_dev = small;          // [0] status flag
    if (hipMemsetAsync(small, 0, 256, c.stream) != hipSuccess ||
        ensure_scratch(c, 65536) != EVOMOE_OK) {
        (void)hipFree(small);
        delete ctx;
        return EVOMOE_EHIP;
    }
    *ctx_out = ctx;
    return EVOMOE_OK;
}

evomoe_status evomoe_destroy(evomoe_ctx* ctx) {
    if (!ctx) return EVOMOE_EINVAL;
    (void)hipStreamSynchronize(ctx->c.stream);
    if (ctx->c.block_counts) (void)hipFree(ctx->c.block_counts);
    if (ctx->c.wg_planes) (void)hipFree(ctx->c.wg_planes);
    if (ctx->c.status_dev) (void)hipFree(ctx->c.status_dev);
    if (ctx->c.prof) {
        for (int i = 0; i < ctx->c.prof->cap; ++i) {
            (void)hipEventDestroy(ctx->c.prof->rec[i].start);
            (void)hipEventDestroy(ctx->c.prof->rec[i].stop);
        }
        delete[] ctx->c.prof->rec;
        delete ctx->c.prof;
    }
    delete ctx;
    return EVOMOE_OK;
}

const char* evomoe_status_string(evomoe_status s) {
    switch (s) {
        case EVOMOE_OK: return "ok";
        case EVOMOE_EINVAL: return "invalid argument";
        case EVOMOE_EUNSUPPORTED: return "unsupported shape";
        case EVOMOE_ECAPACITY: return "number of selected pairs exceeds P_cap";
        case EVOMOE_EWORKSPACE: return "workspace missing or too small";
        case EVOMOE_EHIP: return "HIP runtime error";
        case EVOMOE_ESTATIC: return "shape exceeds the static scratch of the entry point that allocates nothing "
                                    "(ceil(T/256) * E > 65536)";
    }
    return "unknown status";
}

size_t evomoe_workspace_bytes(const evomoe_shape* shape) {
    if (check_shape(shape) != EVOMOE_OK) return 0;
    const size_t a = ffn_bwd_workspace_bytes(*shape), b = gate_bwd_workspace_bytes(*shape);
    const size_t m = a > b ? a : b;
    return (m + 255) & ~(size_t)255;
}

evomoe_status evomoe_dts_gate(evomoe_ctx* ctx, const evomoe_shape* shape, const void* x,
                              const float* Wg, const float* bg, const float* noise, float tau,
                              float threshold, float* gprime, float* gate_w, uint64_t* mask_bits,
                              int32_t* counts, int32_t* k_per_token, int32_t* block_hist) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(x); REQUIRE_PTR(Wg); REQUIRE_PTR(gprime); REQUIRE_PTR(mask_bits); REQUIRE_PTR(counts);
    OPTIONAL_PTR(bg); OPTIONAL_PTR(noise); OPTIONAL_PTR(gate_w); OPTIONAL_PTR(k_per_token); OPTIONAL_PTR(block_hist);
    if (!(tau > 0.f) || !(threshold >= 0.f)) return EVOMOE_EINVAL;
    if (shape->dtype == EVOMOE_BF16) {
        evomoe_status st = ensure_wg_planes(ctx->c, (size_t)3 * 64 * ((shape->d + 31) / 32 * 32) * sizeof(uint16_t));
        if (st != EVOMOE_OK) return st;
    }
    return from_hip(launch_dts_gate(ctx->c, *shape, x, Wg, bg, noise, tau, threshold, gprime, gate_w,
                                    mask_bits, counts, k_per_token, block_hist));
}

evomoe_status evomoe_dts_gate_top1(evomoe_ctx* ctx, const evomoe_shape* shape, const void* x,
                                   const float* Wg, const float* bg, const float* noise, float tau,
                                   float* gprime, float* gate_w, uint64_t* mask_bits, int32_t* counts,
                                   int32_t* k_per_token, int32_t* block_hist) {
    // No score exceeds a threshold above 1, so every token takes the arg-max rule of the threshold gate
    // (lowest index on ties): exactly Algorithm 2's Top-1 branch, with the un-renormalised weight g'.
    return evomoe_dts_gate(ctx, shape, x, Wg, bg, noise, tau, 2.0f, gprime, gate_w, mask_bits, counts,
                           k_per_token, block_hist);
}

evomoe_status evomoe_balance_loss(evomoe_ctx* ctx, const evomoe_shape* shape, const float* gprime,
                                  const int32_t* counts, float alpha, float* loss, float* dgprime_coef) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(gprime); REQUIRE_PTR(counts);
    if (!loss || (reinterpret_cast<uintptr_t>(loss) & 3u)) return EVOMOE_EINVAL;
    if (dgprime_coef && (reinterpret_cast<uintptr_t>(dgprime_coef) & 3u)) return EVOMOE_EINVAL;
    evomoe_status st = ensure_scratch(ctx->c, (size_t)balance_blocks(*shape) * shape->E);
    if (st != EVOMOE_OK) return st;
    return from_hip(launch_balance_loss(ctx->c, *shape, gprime, counts, alpha, loss, dgprime_coef));
}

evomoe_status evomoe_dispatch(evomoe_ctx* ctx, const evomoe_shape* shape, const uint64_t* mask_bits,
                              const float* scores, int32_t* expert_offsets,
                              int32_t* pair_token, float* pair_gate, int32_t* tok_off, int32_t* tok_rows,
                              int64_t* num_pairs, const void* x, void* x_perm, const int32_t* block_hist) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(mask_bits); REQUIRE_PTR(scores); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(pair_token);
    REQUIRE_PTR(pair_gate); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(num_pairs);
    OPTIONAL_PTR(x); OPTIONAL_PTR(x_perm); OPTIONAL_PTR(block_hist);
    if (x_perm && !x) return EVOMOE_EINVAL;
    if (!block_hist) {
        const size_t nblk = dispatch_blocks(*shape);
        evomoe_status st = ensure_scratch(ctx->c, nblk * shape->E + nblk);
        if (st != EVOMOE_OK) return st;
    }
    return from_hip(launch_dispatch(ctx->c, *shape, mask_bits, scores, block_hist, expert_offsets, pair_token,
                                    pair_gate, tok_off, tok_rows, num_pairs, x, x_perm, ctx->c.block_counts));
}

evomoe_status evomoe_dispatch_static(evomoe_ctx* ctx, const evomoe_shape* shape, const uint64_t* mask_bits,
                                     const float* scores, int32_t* expert_offsets,
                                     int32_t* pair_token, float* pair_gate, int32_t* tok_off, int32_t* tok_rows,
                                     int64_t* num_pairs, const void* x, void* x_perm) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(mask_bits); REQUIRE_PTR(scores); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(pair_token);
    REQUIRE_PTR(pair_gate); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(num_pairs);
    OPTIONAL_PTR(x); OPTIONAL_PTR(x_perm);
    if (x_perm && !x) return EVOMOE_EINVAL;
    if ((size_t)dispatch_blocks(*shape) * shape->E > (size_t)kStaticHistEntries) return EVOMOE_ESTATIC;
    if (!ctx->c.static_hist) return EVOMOE_EHIP;      // the address lookup at evomoe_create failed
    return from_hip(launch_dispatch(ctx->c, *shape, mask_bits, scores, nullptr, expert_offsets, pair_token,
                                    pair_gate, tok_off, tok_rows, num_pairs, x, x_perm, ctx->c.static_hist));
}

evomoe_status evomoe_expert_ffn(evomoe_ctx* ctx, const evomoe_shape* shape, const void* x,
                                const int32_t* pair_token, const int32_t* expert_offsets,
                                const void* W1, const float* b1, const void* W2, const float* b2,
                                void* H, void* A, void* O) {
    CHECK_CTX_SHAPE();
    if (evomoe_status fs = check_ffn_shape(shape); fs != EVOMOE_OK) return fs;
    REQUIRE_PTR(x); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(W1); REQUIRE_PTR(W2);
    REQUIRE_PTR(H); REQUIRE_PTR(A); REQUIRE_PTR(O);
    OPTIONAL_PTR(pair_token); OPTIONAL_PTR(b1); OPTIONAL_PTR(b2);
    return from_hip(launch_expert_ffn(ctx->c, *shape, x, pair_token, expert_offsets, W1, b1, W2, b2, H, A, O));
}

evomoe_status evomoe_combine(evomoe_ctx* ctx, const evomoe_shape* shape, const void* O,
                             const float* pair_gate, const int32_t* tok_off, const int32_t* tok_rows,
                             void* y) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(O); REQUIRE_PTR(pair_gate); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(y);
    return from_hip(launch_combine(ctx->c, *shape, O, pair_gate, tok_off, tok_rows, y));
}

evomoe_status evomoe_combine_bwd(evomoe_ctx* ctx, const evomoe_shape* shape, const void* dy,
                                 const void* O, const float* pair_gate, const int32_t* pair_token,
                                 const int32_t* expert_offsets, void* dO, float* dG_pairs) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(dy); REQUIRE_PTR(O); REQUIRE_PTR(pair_gate); REQUIRE_PTR(pair_token);
    REQUIRE_PTR(expert_offsets); REQUIRE_PTR(dO); REQUIRE_PTR(dG_pairs);
    return from_hip(launch_combine_bwd(ctx->c, *shape, dy, O, pair_gate, pair_token, expert_offsets, dO, dG_pairs));
}

evomoe_status evomoe_expert_ffn_bwd(evomoe_ctx* ctx, const evomoe_shape* shape, const void* dO,
                                    const void* H, const void* A, const void* x,
                                    const int32_t* pair_token, const int32_t* expert_offsets,
                                    const void* W1, const void* W2, const void* dy, const float* pair_gate,
                                    void* dW1, float* db1, void* dW2,
                                    float* db2, void* dXp, int accumulate, void* workspace,
                                    size_t workspace_bytes) {
    CHECK_CTX_SHAPE();
    if (evomoe_status fs = check_ffn_shape(shape); fs != EVOMOE_OK) return fs;
    REQUIRE_PTR(dO); REQUIRE_PTR(H); REQUIRE_PTR(A); REQUIRE_PTR(x); REQUIRE_PTR(expert_offsets);
    REQUIRE_PTR(W1); REQUIRE_PTR(W2); REQUIRE_PTR(dXp);
    OPTIONAL_PTR(pair_token); OPTIONAL_PTR(dW1); OPTIONAL_PTR(db1); OPTIONAL_PTR(dW2); OPTIONAL_PTR(db2);
    OPTIONAL_PTR(dy); OPTIONAL_PTR(pair_gate);
    if ((dy != nullptr) != (pair_gate != nullptr) || (dy && !pair_token)) return EVOMOE_EINVAL;
    if (!workspace || !aligned16(workspace) || workspace_bytes < ffn_bwd_workspace_bytes(*shape))
        return EVOMOE_EWORKSPACE;
    return from_hip(launch_expert_ffn_bwd(ctx->c, *shape, dO, H, A, x, pair_token, expert_offsets, W1,
                                          W2, dy, pair_gate, dW1, db1, dW2, db2, dXp, accumulate, workspace));
}

evomoe_status evomoe_dispatch_bwd(evomoe_ctx* ctx, const evomoe_shape* shape, const void* dXp,
                                  const int32_t* tok_off, const int32_t* tok_rows, void* dx) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(dXp); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(dx);
    return from_hip(launch_dispatch_bwd(ctx->c, *shape, dXp, tok_off, tok_rows, dx));
}

evomoe_status evomoe_dts_gate_bwd(evomoe_ctx* ctx, const evomoe_shape* shape, const float* dG_pairs,
                                  const int32_t* tok_off, const int32_t* tok_rows, const float* gprime,
                                  const uint64_t* mask_bits, float tau, const void* x, const float* Wg,
                                  float* dWg, float* dbg, void* dx, void* workspace,
                                  size_t workspace_bytes) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(dG_pairs); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(gprime);
    REQUIRE_PTR(mask_bits); REQUIRE_PTR(x); REQUIRE_PTR(Wg); REQUIRE_PTR(dWg); REQUIRE_PTR(dx);
    OPTIONAL_PTR(dbg);
    if (!(tau > 0.f)) return EVOMOE_EINVAL;
    if (!workspace || !aligned16(workspace) || workspace_bytes < gate_bwd_workspace_bytes(*shape))
        return EVOMOE_EWORKSPACE;
    return from_hip(launch_dts_gate_bwd(ctx->c, *shape, dG_pairs, tok_off, tok_rows, gprime, mask_bits,
                                        tau, x, Wg, dWg, dbg, dx, workspace));
}

evomoe_status evomoe_dts_gate_bwd_balance(evomoe_ctx* ctx, const evomoe_shape* shape, const float* dG_pairs,
                                          const int32_t* tok_off, const int32_t* tok_rows, const float* gprime,
                                          const uint64_t* mask_bits, float tau, const void* x, const float* Wg,
                                          const float* dgprime_coef, float loss_scale, float* dWg, float* dbg,
                                          void* dx, void* workspace, size_t workspace_bytes) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(dG_pairs); REQUIRE_PTR(tok_off); REQUIRE_PTR(tok_rows); REQUIRE_PTR(gprime);
    REQUIRE_PTR(mask_bits); REQUIRE_PTR(x); REQUIRE_PTR(Wg); REQUIRE_PTR(dWg); REQUIRE_PTR(dx);
    OPTIONAL_PTR(dbg);
    if (dgprime_coef && (reinterpret_cast<uintptr_t>(dgprime_coef) & 3u)) return EVOMOE_EINVAL;
    if (!(tau > 0.f)) return EVOMOE_EINVAL;
    if (!workspace || !aligned16(workspace) || workspace_bytes < gate_bwd_workspace_bytes(*shape))
        return EVOMOE_EWORKSPACE;
    return from_hip(launch_dts_gate_bwd(ctx->c, *shape, dG_pairs, tok_off, tok_rows, gprime, mask_bits,
                                        tau, x, Wg, dWg, dbg, dx, workspace, dgprime_coef, loss_scale));
}

size_t evomoe_workspace_bytes_recompute(const evomoe_shape* shape) {
    if (check_shape(shape) != EVOMOE_OK) return 0;
    const size_t a = ffn_bwd_recompute_workspace_bytes(*shape), b = gate_bwd_workspace_bytes(*shape);
    const size_t m = a > b ? a : b;
    return (m + 255) & ~(size_t)255;
}

evomoe_status evomoe_expert_ffn_bwd_recompute(evomoe_ctx* ctx, const evomoe_shape* shape, const void* dO,
                                              const void* x, const int32_t* pair_token,
                                              const int32_t* expert_offsets, const void* W1, const float* b1,
                                              const void* W2, const void* dy, const float* pair_gate,
                                              void* dW1, float* db1, void* dW2, float* db2,
                                              void* dXp, int accumulate, void* workspace,
                                              size_t workspace_bytes) {
    CHECK_CTX_SHAPE();
    if (evomoe_status fs = check_ffn_shape(shape); fs != EVOMOE_OK) return fs;
    REQUIRE_PTR(dO); REQUIRE_PTR(x); REQUIRE_PTR(expert_offsets); REQUIRE_PTR(W1); REQUIRE_PTR(W2);
    REQUIRE_PTR(dXp);
    OPTIONAL_PTR(dy); OPTIONAL_PTR(pair_gate);
    if ((dy != nullptr) != (pair_gate != nullptr) || (dy && !pair_token)) return EVOMOE_EINVAL;
    OPTIONAL_PTR(pair_token); OPTIONAL_PTR(b1); OPTIONAL_PTR(dW1); OPTIONAL_PTR(db1); OPTIONAL_PTR(dW2);
    OPTIONAL_PTR(db2);
    if (!workspace || !aligned16(workspace) || workspace_bytes < ffn_bwd_recompute_workspace_bytes(*shape))
        return EVOMOE_EWORKSPACE;
    return from_hip(launch_expert_ffn_bwd_recompute(ctx->c, *shape, dO, x, pair_token, expert_offsets, W1, b1,
                                                    W2, dy, pair_gate, dW1, db1, dW2, db2, dXp, accumulate,
                                                    workspace));
}

evomoe_status evomoe_schedule(int64_t iteration, int64_t T_S, int64_t T_D, float tau_hi, float tau_lo,
                              evomoe_phase* phase_out) {
    if (!phase_out || iteration < 0 || T_S < 0 || T_D < 0 || !(tau_hi > 0.f) || !(tau_lo > 0.f))
        return EVOMOE_EINVAL;
    if (iteration < T_S) {
        phase_out->stage = 1; phase_out->top1 = 0; phase_out->tau = NAN;
        return EVOMOE_OK;
    }
    const int64_t j = iteration - T_S;
    phase_out->stage = 2;
    if (j < T_D) {
        phase_out->top1 = 0;
        phase_out->tau = T_D == 1 ? tau_hi
                                  : (float)((double)tau_hi - ((double)tau_hi - (double)tau_lo) * ((double)j / (double)(T_D - 1)));
    } else {
        phase_out->top1 = 1;
        phase_out->tau = tau_lo;
    }
    return EVOMOE_OK;
}

evomoe_status evomoe_num_pairs(evomoe_ctx* ctx, const int64_t* num_pairs, int64_t* num_pairs_host) {
    if (!ctx || !num_pairs || !num_pairs_host) return EVOMOE_EINVAL;
    int32_t flag = 0;
    if (hipMemcpyAsync(num_pairs_host, num_pairs, sizeof(int64_t), hipMemcpyDeviceToHost, ctx->c.stream) != hipSuccess ||
        hipMemcpyAsync(&flag, ctx->c.status_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->c.stream) != hipSuccess ||
        hipStreamSynchronize(ctx->c.stream) != hipSuccess)
        return EVOMOE_EHIP;
    if (flag & 1) {
        if (hipMemsetAsync(ctx->c.status_dev, 0, sizeof(int32_t), ctx->c.stream) != hipSuccess) return EVOMOE_EHIP;
        return EVOMOE_ECAPACITY;
    }
    return EVOMOE_OK;
}

evomoe_status evomoe_diversify(evomoe_ctx* ctx, const evomoe_shape* shape, const void* W1_shared,
                               const float* b1_shared, const void* W2_shared, const float* b2_shared,
                               uint64_t seed, float mask_ratio, void* W1, float* b1, void* W2, float* b2) {
    CHECK_CTX_SHAPE();
    REQUIRE_PTR(W1_shared); REQUIRE_PTR(W2_shared); REQUIRE_PTR(W1); REQUIRE_PTR(W2);
    OPTIONAL_PTR(b1_shared); OPTIONAL_PTR(b2_shared); OPTIONAL_PTR(b1); OPTIONAL_PTR(b2);
    if ((b1_shared != nullptr) != (b1 != nullptr) || (b2_shared != nullptr) != (b2 != nullptr)) return EVOMOE_EINVAL;
    if (!(mask_ratio >= 0.f) || !(mask_ratio <= 1.f)) return EVOMOE_EINVAL;
    if ((int64_t)shape->d * shape->F >= ((int64_t)1 << 48)) return EVOMOE_EUNSUPPORTED;
    return from_hip(launch_diversify(ctx->c, *shape, W1_shared, b1_shared, W2_shared, b2_shared, seed, mask_ratio,
                                     W1, b1, W2, b2));
}

evomoe_status evomoe_hint_pairs(evomoe_ctx* ctx, int64_t expected_pairs) {
    if (!ctx) return EVOMOE_EINVAL;
    ctx->c.pair_hint = expected_pairs > 0 ? expected_pairs : 0;
    return EVOMOE_OK;
}

evomoe_status evomoe_profile_select(evomoe_ctx* ctx, int kernel_id) {
    if (!ctx) return EVOMOE_EINVAL;
    if (kernel_id != EVOMOE_K_ALL && kernel_id != EVOMOE_K_NONE && (kernel_id < 0 || kernel_id >= EVOMOE_K_COUNT))
        return EVOMOE_EINVAL;
    Ctx& c = ctx->c;
    if (!c.prof) {
        if (kernel_id == EVOMOE_K_NONE) return EVOMOE_OK;
        Prof* p = new (std::nothrow) Prof();
        if (!p) return EVOMOE_EHIP;
        p->cap = 16384;
        p->used = 0;
        p->rec = new (std::nothrow) ProfRecord[p->cap];
        if (!p->rec) { delete p; return EVOMOE_EHIP; }
        for (int i = 0; i < p->cap; ++i) {
            if (hipEventCreate(&p->rec[i].start) != hipSuccess || hipEventCreate(&p->rec[i].stop) != hipSuccess) {
                p->cap = i;
                break;
            }
        }
        c.prof = p;
    }
    c.prof->select = kernel_id;
    return EVOMOE_OK;
}

evomoe_status evomoe_profile_read(evomoe_ctx* ctx, double* total_ms_host, int64_t* launches_host) {
    if (!ctx || !total_ms_host || !launches_host) return EVOMOE_EINVAL;
    for (int i = 0; i < EVOMOE_K_COUNT; ++i) { total_ms_host[i] = 0.0; launches_host[i] = 0; }
    Ctx& c = ctx->c;
    if (!c.prof) return EVOMOE_OK;
    if (hipStreamSynchronize(c.stream) != hipSuccess) return EVOMOE_EHIP;
    for (int i = 0; i < c.prof->used; ++i) {
        float ms = 0.f;
        const ProfRecord& r = c.prof->rec[i];
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return EVOMOE_EHIP;
        total_ms_host[r.id] += ms;
        launches_host[r.id] += 1;
    }
    c.prof->used = 0;
    return EVOMOE_OK;
}

}  // extern "C"
