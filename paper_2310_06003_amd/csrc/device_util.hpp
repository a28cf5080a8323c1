// Device-side building blocks of libparo (gfx950): launch-shape and cache-policy knobs, vector
// types, dtype conversions, streaming loads and stores, the wave-wide fp64 sum.  Included by
// kernels.hip only; everything lives in that translation unit's anonymous namespace.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "plan.hpp"

namespace {

// Cache-policy and occupancy knobs (the defaults are the measured best on MI355X).
// Everything is touched once: loads are streaming (nt) loads.  Cache policy of the stores, as the
// instruction's bits: 1 = sc0, 2 = nt, 16 = sc1 (0 = default policy): streaming at system scope
// (nt sc1), which the mixed read/write sweeps like 2 % better than nt alone.
#ifndef PARO_POL_G_ST
#define PARO_POL_G_ST 18            // the reduced gradient out of sweep 1
#endif
#ifndef PARO_POL_STATE_ST
#define PARO_POL_STATE_ST 18        // p, m, v and the packed parameters out of them
#endif
#ifndef PARO_POL_LIGHT_ST
#define PARO_POL_LIGHT_ST 18
#endif
#ifndef PARO_BATCH
#define PARO_BATCH 16               // contributions loaded before the first is consumed
#endif
#ifndef PARO_LANE_BATCH
#define PARO_LANE_BATCH 4          // ... in a block with a tensor boundary inside (element loads; more costs registers for nothing)
#endif
// One-wave blocks in flight per compute unit (0 = as many as fit).  The mixed read/write sweeps
// run faster with fewer requests outstanding than the registers would allow.  For the fold the
// budget is in loads: a wave has min(P, PARO_BATCH) of them in flight, so with P = 16 the numbers
// below mean 14 waves per compute unit for sweep 1 and 10 for the single sweep (whose waves also
// load 3 state vectors); with fewer contributions per wave, more waves.
#ifndef PARO_FOLD_LOADS_PER_CU
#define PARO_FOLD_LOADS_PER_CU 224
#endif
#ifndef PARO_FUSED_LOADS_PER_CU
#define PARO_FUSED_LOADS_PER_CU 190
#endif
#ifndef PARO_ADAM_WAVES_PER_CU
#define PARO_ADAM_WAVES_PER_CU 12
#endif
#ifndef PARO_ADAM_MASK_WAVES_PER_CU
#define PARO_ADAM_MASK_WAVES_PER_CU 16   // with a decay mask: a table look-up per wave to hide as well
#endif
// Sweep 1 in the tensor layout.  What decides is the list: a chunk made of a few large tensors
// ("large": at least PARO_DENSE_BLOCKS_PER_TENSOR blocks per tensor piece in the chunk, on average)
// behaves like the chunk layout - its look-ups hit the scalar cache - and keeps the chunk layout's
// shape and budget.  A chunk cut into many small pieces has waves that spend part of their life on
// look-ups with no data in flight: it is launched without the throttle, and with at most
// PARO_PAIR_MAX_RANKS contributions and at least PARO_PAIR_MIN_BLOCKS blocks a wave takes two
// consecutive blocks under a budget twice the chunk layout's (see k_reduce4t; the two shapes cross
// near 50 M elements: a smaller launch wants as many waves as it can get).
#ifndef PARO_PAIR_MAX_RANKS
#define PARO_PAIR_MAX_RANKS 8
#endif
#ifndef PARO_PAIR_MIN_BLOCKS
#define PARO_PAIR_MIN_BLOCKS 196608
#endif
#ifndef PARO_FOLD_T_LOADS_PER_CU
#define PARO_FOLD_T_LOADS_PER_CU 448
#endif
#ifndef PARO_DENSE_BLOCKS_PER_TENSOR
#define PARO_DENSE_BLOCKS_PER_TENSOR 1024
#endif
#ifndef PARO_FOLD_TM_LOADS_PER_CU
#define PARO_FOLD_TM_LOADS_PER_CU 100000
#endif
#ifndef PARO_FUSED_T_LOADS_PER_CU      // the single sweep over many small tensors
#define PARO_FUSED_T_LOADS_PER_CU 100000
#endif
#ifndef PARO_MIN_WAVES_PER_CU
#define PARO_MIN_WAVES_PER_CU 8     // the throttle never goes below this
#endif
#ifndef PARO_HOP_WAVES_PER_CU
#define PARO_HOP_WAVES_PER_CU 0
#endif
#ifndef PARO_COPY_WAVES_PER_CU
#define PARO_COPY_WAVES_PER_CU 0
#endif

constexpr int WAVE = 64;              // threads of a block: every sweep kernel runs in one-wave blocks
constexpr int EPT = 4;                // elements per thread
constexpr int PIECE = WAVE * EPT;     // elements per block
constexpr int TILE = PARO_TILE;       // granularity of the plan's per-block table
constexpr int FINALIZE_TPB = 256;     // threads of the kernel that adds the partial sums
constexpr int FINALIZE_CHUNK = 2048;  // partials per block in its first level
static_assert(TILE == PIECE, "the per-tile table has one entry per block");

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

// What a launch needs to map its elements to tensors.
struct TensorMap {
    const int64_t *nz_off;      // [n_nz + 1] flat start of every non-empty tensor, then Psi
    const int32_t *nz_tensor;   // [n_nz]
    const uint8_t *nz_dtype;    // [n_nz] gradient dtype of that tensor
    const uint8_t *dtype;       // [T]
    const uint8_t *no_decay;    // [T]
    int n_nz;
    int64_t total;              // Psi
    int64_t begin;              // flat index of the launch's element 0
    const paro_tile_info *tile_tab;   // the per-tile table of the launch's chunk, or null
};

// Lane of the thread in its wave (the sweep kernels run in one-wave blocks).
__device__ __forceinline__ unsigned lane_id() { return threadIdx.x & (WAVE - 1); }

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
__device__ __forceinline__ float cvt16(unsigned int h16, int dt) {
    return dt == PARO_F16 ? f16_bits_to_f32(h16) : __uint_as_float(h16 << 16);
}

__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;      // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// two parameters rounded to the low-precision format, packed into one word
__device__ __forceinline__ unsigned int pack2_lowp(float a, float b, int pack_dtype) {
    if (pack_dtype == PARO_F16) return f32_to_f16_bits(a) | (f32_to_f16_bits(b) << 16);
    return f32_to_bf16_rne(a) | (f32_to_bf16_rne(b) << 16);
}

// Pointers that were themselves loaded from memory carry no address space; these are device
// (global) addresses by contract, so say so and get global rather than flat loads.
template <class V>
__device__ __forceinline__ const __attribute__((address_space(1))) V *global_ptr(uintptr_t a) {
    return reinterpret_cast<const __attribute__((address_space(1))) V *>(a);
}
// Streaming (non-temporal) load of something read once.
template <class V>
__device__ __forceinline__ V ld_nt(const V *p) { return __builtin_nontemporal_load(p); }
template <class V>
__device__ __forceinline__ V ld_nt(const __attribute__((address_space(1))) V *p) { return __builtin_nontemporal_load(p); }

// ---- stores through per-wave buffer descriptors.  A block's stores to one array go through a
// descriptor that covers exactly the block's piece of it (a wave-uniform base address and a byte
// count): the instruction then carries its cache policy as an immediate - which a plain store
// cannot express beyond "non-temporal" - and the hardware drops whatever falls outside the piece.
// (Loads stay plain streaming loads: building a descriptor per contribution cost the fold 5 %.)
typedef __amdgpu_buffer_rsrc_t wave_buf;
__device__ __forceinline__ wave_buf wave_buffer(const void *base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
template <int POL>
__device__ __forceinline__ void buf_store8(u32x2 v, wave_buf b, unsigned off) {
    __builtin_amdgcn_raw_buffer_store_b64(v, b, (int)off, 0, POL);
}
template <int POL>
__device__ __forceinline__ void buf_store16(u32x4 v, wave_buf b, unsigned off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, b, (int)off, 0, POL);
}
__device__ __forceinline__ u32x4 as_u32x4(float a, float b, float c, float d) {
    return u32x4{__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
}

// A value that is the same in every lane, marked as such for the compiler (scalar registers,
// scalar branches, scalar loads of what it indexes).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform(int64_t v) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Sum over the wave, valid in lane 0.  Fixed shape (shuffles by 32, 16, ... 1).
__device__ __forceinline__ double wave_sum(double v) {
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    return v;
}

// Sum over a block of FINALIZE_TPB threads, valid in thread 0: lanes by shuffles, then the waves in order.
__device__ __forceinline__ double block_sum(double v) {
    __shared__ double s_wave[FINALIZE_TPB / 64];
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) s_wave[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) {
        r = s_wave[0];
        for (int w = 1; w < FINALIZE_TPB / 64; ++w) r += s_wave[w];
    }
    return r;
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

}  // namespace
