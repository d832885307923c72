// Internal helpers shared by the gfx950 kernels of the DTS-Gate MoE layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/evomoe.h"

namespace evomoe {

constexpr int kWave = 64;                 // CDNA wavefront
constexpr int kDispatchTokens = 256;      // tokens per dispatch block (one thread per token)
constexpr int kStaticHistEntries = 65536; // ints in the static histogram table (256 KB per GPU): 1024 blocks x 64 experts
constexpr int kMaxDevices = 64;

typedef __bf16 bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float -> bf16, round-to-nearest-even, through the hardware conversion (v_cvt_pk_bf16_f32: two per instruction)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const bf16x2 v = {(bf16_t)lo, (bf16_t)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;   // elements per 16-byte vector
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
    // 16-byte vector of kVec elements -> floats
    __device__ static __forceinline__ void load_vec(const float* p, float* out) {
        f32x4 v = *reinterpret_cast<const f32x4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
    __device__ static __forceinline__ void store_vec(float* p, const float* in) {
        f32x4 v = {in[0], in[1], in[2], in[3]};
        *reinterpret_cast<f32x4*>(p) = v;
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static __forceinline__ float load(const bf16_t* p) {
        return bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(p));
    }
    __device__ static __forceinline__ void store(bf16_t* p, float v) {
        *reinterpret_cast<uint16_t*>(p) = (uint16_t)f32_to_bf16_bits(v);
    }
    __device__ static __forceinline__ void load_vec(const bf16_t* p, float* out) {
        u32x4 v = *reinterpret_cast<const u32x4*>(p);
        out[0] = lo_bf16(v.x); out[1] = hi_bf16(v.x);
        out[2] = lo_bf16(v.y); out[3] = hi_bf16(v.y);
        out[4] = lo_bf16(v.z); out[5] = hi_bf16(v.z);
        out[6] = lo_bf16(v.w); out[7] = hi_bf16(v.w);
    }
    __device__ static __forceinline__ void store_vec(bf16_t* p, const float* in) {
        u32x4 v = {pack_bf16x2(in[0], in[1]), pack_bf16x2(in[2], in[3]),
                   pack_bf16x2(in[4], in[5]), pack_bf16x2(in[6], in[7])};
        *reinterpret_cast<u32x4*>(p) = v;
    }
};

// Activation of Eq. ffn (ReLU) and of the experiments (exact GeLU x*Phi(x)); derivatives with ReLU'(0)=0.
__device__ __forceinline__ float act_fwd(float h, int act) {
    if (act == EVOMOE_RELU) return h > 0.f ? h : 0.f;
    return 0.5f * h * (1.0f + erff(h * 0.70710678118654752440f));
}
__device__ __forceinline__ float act_grad(float h, int act) {
    if (act == EVOMOE_RELU) return h > 0.f ? 1.f : 0.f;
    float Phi = 0.5f * (1.0f + erff(h * 0.70710678118654752440f));
    float phi = 0.39894228040143267794f * __expf(-0.5f * h * h);
    return Phi + h * phi;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Number of rows the per-pair kernels may touch: P clamped to the buffers' capacity.
__device__ __forceinline__ int clamp_pairs(int P, int64_t P_cap) {
    return (int64_t)P > P_cap ? (int)P_cap : P;
}

// Optional per-kernel timing with HIP events on the context's stream (measurement aid).
struct ProfRecord { int id; hipEvent_t start, stop; };
struct Prof {
    int select;                       // evomoe_kernel_id, EVOMOE_K_ALL or EVOMOE_K_NONE
    ProfRecord* rec;                  // pool
    int used, cap;
};

struct Ctx {
    hipStream_t stream;
    int device;
    int num_cu;
    int64_t pair_hint;        // pair count announced by the caller (0 = none): picks tile shapes, nothing else
    int32_t* status_dev;      // [1] device flag: bit0 = capacity overflow
    int32_t* block_counts;    // scratch for per-block expert histograms
    int32_t* static_hist;     // this device's address of the static table of evomoe_dispatch_static (or null)
    size_t block_counts_elems;
    uint16_t* wg_planes;      // bf16 gate: W_g split into three bf16 terms, in MFMA fragment order
    size_t wg_planes_bytes;
    Prof* prof;
};

// Brackets the kernel launches issued during its lifetime with two events when kernel `id` is selected.
struct ProfScope {
    const Ctx& c;
    ProfRecord* r;
    ProfScope(const Ctx& ctx, int id) : c(ctx), r(nullptr) {
        Prof* p = ctx.prof;
        if (!p || p->select == EVOMOE_K_NONE || (p->select != EVOMOE_K_ALL && p->select != id)) return;
        if (p->used >= p->cap) return;
        r = &p->rec[p->used++];
        r->id = id;
        (void)hipEventRecord(r->start, ctx.stream);
    }
    ~ProfScope() { if (r) (void)hipEventRecord(r->stop, c.stream); }
};

}  // namespace evomoe
