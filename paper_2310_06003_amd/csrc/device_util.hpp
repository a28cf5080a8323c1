// Device-side building blocks of libparo (gfx950): launch-shape and cache-policy knobs, vector
// types, dtype conversions, streaming loads and stores, the block-wide fp64 sum.  Included by
// kernels.hip only; everything lives in that translation unit's anonymous namespace.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "plan.hpp"

namespace {


// Launch-shape and cache-policy knobs (the defaults are the measured best on MI355X).
#ifndef PARO_NT_FOLD
#define PARO_NT_FOLD 1              // streaming (non-temporal) loads for the contributions
#endif
#ifndef PARO_NT_STATE
#define PARO_NT_STATE 0             // ... for g, p, m, v
#endif
#ifndef PARO_NT_GSTORE
#define PARO_NT_GSTORE 1            // ... stores of the reduced gradient in sweep 1
#endif
#ifndef PARO_TPBK_FOLD
#define PARO_TPBK_FOLD 2            // 0: persistent grid-stride blocks; k > 0: block b takes tiles [b*k, b*k + k)
#endif
#ifndef PARO_TPBK_ADAM
#define PARO_TPBK_ADAM 1
#endif
#ifndef PARO_G_TRANSPOSE
#define PARO_G_TRANSPOSE 1          // sweep 1 stores the gradient with whole-wave contiguous 1 KB store instructions
#endif
#ifndef PARO_BLOCKS_PER_CU
#define PARO_BLOCKS_PER_CU 8
#endif
#ifndef PARO_FOLD4
#define PARO_FOLD4 1        // sweep 1, chunk layout: the 4-elements-per-thread kernel
#endif
#ifndef PARO_FOLD4_TPB
#define PARO_FOLD4_TPB 64   // its block size (one wave)
#endif
#ifndef PARO_FOLD4_WAVES_PER_CU
#define PARO_FOLD4_WAVES_PER_CU 14   // blocks (waves) of it in flight per compute unit; 0 = no limit
#endif
#ifndef PARO_FUSED4_WAVES_PER_CU
#define PARO_FUSED4_WAVES_PER_CU 10
#endif
#ifndef PARO_HOP_WAVES_PER_CU
#define PARO_HOP_WAVES_PER_CU 0
#endif
#ifndef PARO_COPY_WAVES_PER_CU
#define PARO_COPY_WAVES_PER_CU 0
#endif
#ifndef PARO_ADAM4_WAVES_PER_CU
#define PARO_ADAM4_WAVES_PER_CU 12
#endif
#ifndef PARO_ADAM4
#define PARO_ADAM4 1        // sweep 2 without a decay mask: the 4-elements-per-thread kernel
#endif
#ifndef PARO_NT_ADAM4
#define PARO_NT_ADAM4 3     // its cache policy: bit 0 streaming loads, bit 1 streaming stores
#endif
#ifndef PARO_ADAM4_TPB
#define PARO_ADAM4_TPB 64   // its block size (one wave)
#endif
#ifndef PARO_BATCH_BF16
#define PARO_BATCH_BF16 16
#endif
#ifndef PARO_TPB
#define PARO_TPB 256
#endif

constexpr int TPB = PARO_TPB;        // threads per block
constexpr int EPT = 8;              // elements per thread per tile
constexpr int TILE = TPB * EPT;     // 2048 with 256 threads
constexpr int BLOCKS_PER_CU = PARO_BLOCKS_PER_CU;
constexpr int FINALIZE_CHUNK = 2048;  // partials per block in the first level of the final sum

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// P device pointers in fold order.  Lives in the kernel-argument segment and is
// only ever indexed with wave-uniform indices, i.e. read with scalar loads.
struct SrcTable {
    const void *p[PARO_MAX_RANKS];
};

struct AdamConsts {
    float beta1, beta2, omb1, omb2, eps, step_size, sqrt_bc2, decay, wd, grad_scale, max_norm;
    int adamw, skip_nonfinite, pack_dtype;
};

// What the kernels need to map an element of the flat buffer to its tensor.
struct TensorMap {
    const int64_t *nz_off;      // [n_nz + 1]
    const int32_t *nz_tensor;   // [n_nz]
    const uint8_t *dtype;       // [T]
    const uint8_t *no_decay;    // [T]
    int n_nz;
    int64_t total;              // Psi
};

// ---------------------------------------------------------------- small helpers
__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp16 <-> fp32: the hardware conversions (exact upwards, round-to-nearest-even downwards)
__device__ __forceinline__ float f16_bits_to_f32(unsigned int h16) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h16);
}
__device__ __forceinline__ unsigned int f32_to_f16_bits(float f) {
    return (unsigned int)__builtin_bit_cast(unsigned short, (_Float16)f);
}
// the two 16-bit values of a word, as fp32, for a 2-byte gradient dtype
template <int DT>
__device__ __forceinline__ float cvt_lo(unsigned int w) {
    return DT == PARO_F16 ? f16_bits_to_f32(w & 0xFFFFu) : bf16_lo(w);
}
template <int DT>
__device__ __forceinline__ float cvt_hi(unsigned int w) {
    return DT == PARO_F16 ? f16_bits_to_f32(w >> 16) : bf16_hi(w);
}
template <int DT>
__device__ __forceinline__ void unpack16x8(const u32x4 &q, float x[8]) {
    x[0] = cvt_lo<DT>(q.x); x[1] = cvt_hi<DT>(q.x); x[2] = cvt_lo<DT>(q.y); x[3] = cvt_hi<DT>(q.y);
    x[4] = cvt_lo<DT>(q.z); x[5] = cvt_hi<DT>(q.z); x[6] = cvt_lo<DT>(q.w); x[7] = cvt_hi<DT>(q.w);
}
__device__ __forceinline__ float cvt16(unsigned int h16, int dt) {
    return dt == PARO_F16 ? f16_bits_to_f32(h16) : __uint_as_float(h16 << 16);
}

__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;      // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Pointers that were themselves loaded from memory carry no address space; these are device
// (global) addresses by contract, so say so and get global rather than flat loads.
template <class V>
__device__ __forceinline__ const __attribute__((address_space(1))) V *global_ptr(uintptr_t a) {
    return reinterpret_cast<const __attribute__((address_space(1))) V *>(a);
}
template <bool NT, class V>
__device__ __forceinline__ V ld_as(const __attribute__((address_space(1))) V *p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT, class V>
__device__ __forceinline__ V ld_as(const V *p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <class Ptr>
__device__ __forceinline__ auto ld_contrib(Ptr p) { return ld_as<PARO_NT_FOLD != 0>(p); }
template <class V>
__device__ __forceinline__ V ld_state(const V *p) { return ld_as<PARO_NT_STATE != 0>(p); }
template <bool NT, class V>
__device__ __forceinline__ void st_as(V *p, V v) {
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

template <bool NT = (PARO_NT_STATE != 0)>
__device__ __forceinline__ void load8_f32(const float *p, float x[8]) {
    f32x4 a = ld_as<NT>(reinterpret_cast<const f32x4 *>(p));
    f32x4 b = ld_as<NT>(reinterpret_cast<const f32x4 *>(p + 4));
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

template <bool NT = false>
__device__ __forceinline__ void store8_f32(float *p, const float x[8]) {
    f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
    st_as<NT>(reinterpret_cast<f32x4 *>(p), a);
    st_as<NT>(reinterpret_cast<f32x4 *>(p + 4), b);
}

// the low-precision copy of 8 parameters: bf16 or fp16 (block-uniform choice)
__device__ __forceinline__ void store8_lowp(uint16_t *p, const float x[8], int pack_dtype) {
    u32x4 w;
    if (pack_dtype == PARO_F16) {
        w.x = f32_to_f16_bits(x[0]) | (f32_to_f16_bits(x[1]) << 16);
        w.y = f32_to_f16_bits(x[2]) | (f32_to_f16_bits(x[3]) << 16);
        w.z = f32_to_f16_bits(x[4]) | (f32_to_f16_bits(x[5]) << 16);
        w.w = f32_to_f16_bits(x[6]) | (f32_to_f16_bits(x[7]) << 16);
    } else {
        w.x = f32_to_bf16_rne(x[0]) | (f32_to_bf16_rne(x[1]) << 16);
        w.y = f32_to_bf16_rne(x[2]) | (f32_to_bf16_rne(x[3]) << 16);
        w.z = f32_to_bf16_rne(x[4]) | (f32_to_bf16_rne(x[5]) << 16);
        w.w = f32_to_bf16_rne(x[6]) | (f32_to_bf16_rne(x[7]) << 16);
    }
    *reinterpret_cast<u32x4 *>(p) = w;
}

// Stores the wave's 512 results so that each of the two store instructions writes 1 KB of
// consecutive addresses (lane l writes elements 4l..4l+3, then 256+4l..256+4l+3 of the wave's
// span) instead of every other 16 bytes.  x[0..7] are the lane's elements 8l..8l+7; the values
// travel between lanes by shuffles.  wave_base = address of the wave's first element.
template <bool NT>
__device__ __forceinline__ void store8_f32_wave_contiguous(float *wave_base, const float x[8]) {
    const int lane = threadIdx.x & 63;
    const int src_a = lane >> 1, src_b = 32 + (lane >> 1);
    const bool odd = lane & 1;
    float a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo_a = __shfl(x[i], src_a, 64), hi_a = __shfl(x[4 + i], src_a, 64);
        const float lo_b = __shfl(x[i], src_b, 64), hi_b = __shfl(x[4 + i], src_b, 64);
        a[i] = odd ? hi_a : lo_a;
        b[i] = odd ? hi_b : lo_b;
    }
    f32x4 va = {a[0], a[1], a[2], a[3]}, vb = {b[0], b[1], b[2], b[3]};
    st_as<NT>(reinterpret_cast<f32x4 *>(wave_base + 4 * lane), va);
    st_as<NT>(reinterpret_cast<f32x4 *>(wave_base + 256 + 4 * lane), vb);
}

// Sum over the block, valid in thread 0.  Fixed shape: lanes by shuffles, then
// the waves in order.
template <int NTHREADS = TPB>
__device__ __forceinline__ double block_sum(double v) {
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    if constexpr (NTHREADS == 64) {
        return v;
    } else {
        __shared__ double s_wave[NTHREADS / 64];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        if (lane == 0) s_wave[wave] = v;
        __syncthreads();
        double r = 0.0;
        if (threadIdx.x == 0) {
            r = s_wave[0];
            for (int w = 1; w < NTHREADS / 64; ++w) r += s_wave[w];
        }
        __syncthreads();
        return r;
    }
}

template <class Ld>
__device__ __forceinline__ int64_t ld_lean_off(const Ld &ld) {
    if constexpr (Ld::kTensor) return ld.lean_byte_off; else return 0;
}

template <class Ld>
__device__ __forceinline__ int ld_lean_dt(const Ld &ld) {
    if constexpr (Ld::kTensor) return ld.lean_dt; else return PARO_BF16;
}

// Compile-time loop: the body sees its index as a constant, so arrays indexed by it stay in
// registers whatever the size of the body.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Where the thread's 8 elements live: tensor (-1 = padding) and offset inside it.
struct Where8 {
    int tens[8];
    int64_t toff[8];
    bool one_tensor;       // all 8 in one tensor (then tens[0], toff[0] describe them)
    int first_dt;          // dtype of tens[0] (meaningful when tens[0] >= 0)
};

}  // namespace
