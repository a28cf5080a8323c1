// Device side of libparo for gfx950 (MI355X): the streaming kernels of the
// Update stage (paper Sec. 3.2) and the entry points that launch them.
//
// Everything here is bound by HBM bandwidth: per shard parameter the method
// moves 2P bytes of bf16 contributions and 26-34 bytes of fp32 state, against
// P adds and ~20 flops.  So the kernels are plain sweeps built around 16-byte
// coalesced accesses with many independent loads in flight per thread; there
// is no dense contraction and hence no MFMA.
//
//   tile      2048 consecutive elements (256 threads x 8 elements)
//   grid      one block per run of consecutive tiles (2 for the fold, 1 for
//             Adam), dispatched in address order: on MI355X this beat
//             persistent grid-stride blocks by 8-15 % for these mixed
//             read/write streams (measured; both shapes are kept behind
//             PARO_TPBK_*)
//   caches    contributions are read once: streaming (non-temporal) loads;
//             the reduced gradient is written with streaming stores, each
//             store instruction of a wave covering 1 KB of consecutive
//             addresses (values change lanes by shuffles first); p, m, v use
//             the default policy (streaming hints made sweep 2 slower)
//   fold      the P contributions of an element are added in a fixed order
//             (never re-associated, never contracted into FMAs) so the result
//             is bit-identical to a reduce-scatter ring run in that order
//   norm      squares are exact in fp64; per-thread fp64 sums -> wave shuffles
//             -> LDS -> one partial per block -> a one-block kernel adds the
//             partials in a fixed order.  No atomics: run-to-run identical.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

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
// the four waves in order.
__device__ __forceinline__ double block_sum(double v) {
    __shared__ double s_wave[TPB / 64];
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) s_wave[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) {
        r = s_wave[0];
        for (int w = 1; w < TPB / 64; ++w) r += s_wave[w];
    }
    __syncthreads();
    return r;
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

// ------------------------------------------------------------------- loaders
// A loader hands the fold the 8 values that contribution k (in fold order)
// holds for the thread's 8 elements.

struct TileSegs;

// Contributions are arrays in shard coordinates, all bf16 or all fp32.
template <int DT>
struct ChunkLoader {
    static constexpr bool kTensor = false;
    // contributions loaded before the first is consumed (16 bytes each for bf16, 32 for fp32)
    static constexpr int kBatch = DT != PARO_F32 ? PARO_BATCH_BF16 : 8;
    struct Raw { u32x4 a, b; };
    int64_t e;                                   // first of the thread's 8 elements
    __device__ __forceinline__ void prepare(int64_t e0, const Where8 &) { e = e0; }
    __device__ __forceinline__ void begin_tile(const TileSegs &, const SrcTable &, int, uintptr_t *) {}
    __device__ __forceinline__ bool lean() const { return false; }
    template <bool SLOW>
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        if (DT != PARO_F32) {
            r.a = ld_contrib(reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(src.p[k]) + e));
        } else {
            const u32x4 *q = reinterpret_cast<const u32x4 *>(static_cast<const float *>(src.p[k]) + e);
            r.a = ld_contrib(q);
            r.b = ld_contrib(q + 1);
        }
    }
    template <bool SLOW>
    __device__ __forceinline__ void unpack(const SrcTable &, int, const Raw &r, float x[8]) const {
        if (DT != PARO_F32) {
            unpack16x8<DT>(r.a, x);
        } else {
            x[0] = __uint_as_float(r.a.x); x[1] = __uint_as_float(r.a.y);
            x[2] = __uint_as_float(r.a.z); x[3] = __uint_as_float(r.a.w);
            x[4] = __uint_as_float(r.b.x); x[5] = __uint_as_float(r.b.y);
            x[6] = __uint_as_float(r.b.z); x[7] = __uint_as_float(r.b.w);
        }
    }
};

// Largest k in [0, n_entries) with tab[k] <= f, for a sorted table with
// tab[0] <= f; the 64 lanes of a wave probe 64 places per round.
__device__ __forceinline__ int wave_search(const int64_t *tab, int n_entries, int64_t f, int lane) {
    int lo = 0, hi = n_entries;
    while (hi - lo > 1) {
        const int step = (hi - lo + 63) / 64;
        const int idx = lo + lane * step;
        const bool le = idx < hi && tab[idx] <= f;
        const int cnt = __popcll(__ballot(le));        // the lanes that hold form a prefix
        lo = lo + (cnt - 1) * step;
        hi = min(hi, lo + step);
    }
    return lo;
}

// The slice of the tensor-offset table that covers one tile, staged in LDS, so
// that the ragged side of the work (which tensor, which offset) costs LDS
// lookups instead of dependent global loads.
struct TileSegs {
    int64_t *s_off;        // [TILE + 2], tile-relative starts of the segments, then the end of the last
    int *s_head;           // [2]: index of the first segment in the table, segment count
    TensorMap tm;
    int64_t range_begin;   // flat index of shard element 0
    const paro_tile_info *tile_tab;   // per-tile summary of this launch's range, or null
    // set by begin_tile when the table says the whole tile lies in one tensor (then nothing is staged)
    int single_tensor;
    int64_t single_toff;
    int single_dt;

    __device__ __forceinline__ void begin_tile(int64_t tile_start) {
        const int64_t f0 = range_begin + tile_start;
        const int64_t f_end = min(f0 + (int64_t)TILE, tm.total);
        single_tensor = -1;
        int k_known = -1;
        if (tile_tab) {
            const paro_tile_info info = tile_tab[tile_start / TILE];     // same address for the whole block
            if (info.tensor >= 0) {
                single_tensor = info.tensor;
                single_toff = info.toff;
                single_dt = info.first_seg;                     // for such tiles the field holds the dtype
                return;
            }
            k_known = info.first_seg;
        }
        __syncthreads();                                   // the previous tile's readers are done
        if (threadIdx.x < 64) {
            int k_lo = tm.n_nz;
            if (k_known >= 0)
                k_lo = k_known;
            else if (f0 < tm.total)
                k_lo = wave_search(tm.nz_off, tm.n_nz + 1, f0, threadIdx.x);
            if (threadIdx.x == 0) {
                s_head[0] = k_lo;
                s_head[1] = 0;
            }
        }
        __syncthreads();
        const int k_lo = s_head[0];
        // segments are at least one element long, so a tile sees at most TILE of them
        for (int base = 0; base <= TILE; base += TPB) {
            const int c = base + threadIdx.x;
            int64_t val = INT64_MAX;
            if (c <= TILE && k_lo + c <= tm.n_nz) {
                val = tm.nz_off[k_lo + c];
                s_off[c] = val - f0;
                if (val < f_end) atomicMax(&s_head[1], c + 1);
            }
            // stop once a whole round lies at or past the end of the tile
            const int more = __syncthreads_or(val < f_end);
            if (!more) break;
        }
    }
    __device__ __forceinline__ int count() const { return s_head[1]; }
    __device__ __forceinline__ int first() const { return s_head[0]; }
    // segment (tile-local index) holding tile-relative element rel, or -1 for padding
    __device__ __forceinline__ int find(int rel) const {
        const int n = s_head[1];
        if (n == 0 || (int64_t)rel >= s_off[n]) return -1;
        int lo = 0, hi = n;                                 // s_off[lo] <= rel < s_off[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_off[mid] <= rel) lo = mid; else hi = mid;
        }
        return lo;
    }
};

__device__ __forceinline__ void locate8(const TileSegs &segs, int rel0, Where8 &w) {
    if (segs.single_tensor >= 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w.tens[i] = segs.single_tensor;
            w.toff[i] = segs.single_toff + rel0 + i;
        }
        w.one_tensor = true;
        w.first_dt = segs.single_dt;
        return;
    }
    int c = segs.find(rel0);
    const int n = segs.count();
    const int c_first = c;
    if (c >= 0 && (int64_t)(rel0 + 7) < segs.s_off[c + 1]) {      // the usual case: all 8 in one segment
        const int t = segs.tm.nz_tensor[segs.first() + c];
        const int64_t toff = (int64_t)rel0 - segs.s_off[c];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w.tens[i] = t;
            w.toff[i] = toff + i;
        }
        w.one_tensor = true;
        w.first_dt = segs.tm.dtype[t];
        return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rel = rel0 + i;
        if (c >= 0) {
            while (c < n && segs.s_off[c + 1] <= rel) ++c;
            if (c >= n) c = -1;                            // ran into the padding
        }
        if (c >= 0) {
            w.tens[i] = segs.tm.nz_tensor[segs.first() + c];
            w.toff[i] = (int64_t)rel - segs.s_off[c];
        } else {
            w.tens[i] = -1;
            w.toff[i] = 0;
        }
    }
    w.one_tensor = c_first >= 0 && c == c_first;
    w.first_dt = w.tens[0] >= 0 ? segs.tm.dtype[w.tens[0]] : PARO_BF16;
}

// Contributions are per-tensor gradients: source k is a device array of T
// pointers.  Elements map to tensors through the staged offsets.
//
// Fast path (the thread's 8 elements lie in one tensor): the source address has
// whatever alignment the tensor's base and offset give it, so the thread loads the
// 16-byte-aligned blocks that cover its 16 (bf16) or 32 (fp32) bytes - two or three
// vector loads, the extra one shared with the neighbouring lane through the L1 - and
// shifts the words into place.  An aligned 16-byte block that holds at least one valid
// byte never crosses a page, so the over-read at either end of a tensor stays inside
// mapped memory.  Slow path (a tensor boundary or padding inside the 8): element loads.
struct TensorLoader {
    static constexpr bool kTensor = true;
    static constexpr int kBatch = 4;
    struct Raw { u32x4 a, b, c, meta; };      // meta.x = byte offset of the first wanted byte in block a
    const uint8_t *dtype;  // [T]
    Where8 w;
    const uintptr_t *s_ptr;   // LDS: the P base pointers of the tile's tensor, when the tile lies in one tensor
    bool staged;
    bool lean_;               // ... and it is a 2-byte dtype and every source's first byte is 16-byte aligned
    int lean_dt;
    int64_t lean_byte_off;    // byte offset of the tile's first element inside the tensor

    __device__ __forceinline__ bool lean() const { return lean_; }

    __device__ __forceinline__ void prepare(int64_t, const Where8 &where) { w = where; }

    // When the whole tile lies in one tensor, fetch that tensor's P base pointers once per block
    // (thread k fetches source k's) instead of once per thread and batch: the pointer look-up
    // then costs one round trip per tile, off the critical path of the data loads.
    __device__ __forceinline__ void begin_tile(const TileSegs &segs, const SrcTable &src, int P, uintptr_t *lds_ptr) {
        s_ptr = lds_ptr;
        staged = segs.single_tensor >= 0;                  // uniform over the block
        lean_ = false;
        if (!staged) return;
        lean_byte_off = segs.single_toff * 2;
        __syncthreads();                                   // the previous tile's readers are done
        bool aligned = segs.single_dt != PARO_F32;
        lean_dt = segs.single_dt;
        for (int k = threadIdx.x; k < P; k += TPB) {
            const uintptr_t b = reinterpret_cast<uintptr_t>(static_cast<const void *const *>(src.p[k])[segs.single_tensor]);
            lds_ptr[k] = b;
            aligned = aligned && ((b + (uintptr_t)lean_byte_off) & 15) == 0;
        }
        lean_ = __syncthreads_and(aligned);                // also publishes the pointers
    }

    template <bool SLOW>
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        if (SLOW && !w.one_tensor) return;
        const int t = w.tens[0];
        const bool is_bf16 = w.first_dt != PARO_F32;        // "2-byte dtype": bf16 or fp16
        const uintptr_t base = staged ? s_ptr[k]
                                      : reinterpret_cast<uintptr_t>(static_cast<const void *const *>(src.p[k])[t]);
        const uintptr_t addr = base + (uintptr_t)w.toff[0] * (is_bf16 ? 2 : 4);
        const uintptr_t al = addr & ~(uintptr_t)15;
        const unsigned int shift = (unsigned int)(addr & 15);
        r.meta = u32x4{shift, 0u, 0u, 0u};
        const bool need_b = !is_bf16 || shift != 0;
        const bool need_c = !is_bf16 && shift != 0;
        r.a = ld_contrib(global_ptr<u32x4>(al));
        if (need_b) r.b = ld_contrib(global_ptr<u32x4>(al + 16));
        if (need_c) r.c = ld_contrib(global_ptr<u32x4>(al + 32));
    }

    static __device__ __forceinline__ unsigned int sel4(unsigned int q, unsigned int w0, unsigned int w1,
                                                        unsigned int w2, unsigned int w3) {
        return q == 0 ? w0 : q == 1 ? w1 : q == 2 ? w2 : w3;
    }

    template <bool SLOW>
    __device__ __forceinline__ void unpack(const SrcTable &src, int k, const Raw &r, float x[8]) const {
        if (SLOW && !w.one_tensor) {
            const void *const *ptrs = static_cast<const void *const *>(src.p[k]);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float val = 0.0f;                           // padding contributes +0
                const int t = w.tens[i];
                if (t >= 0) {
                    const void *b = ptrs[t];
                    const int dt = dtype[t];
                    if (dt != PARO_F32)
                        val = cvt16(static_cast<const uint16_t *>(b)[w.toff[i]], dt);
                    else
                        val = static_cast<const float *>(b)[w.toff[i]];
                }
                x[i] = val;
            }
            return;
        }
        const unsigned int shift = r.meta.x;
        const unsigned int q = shift >> 2;                  // first word that holds wanted bytes
        if (w.first_dt != PARO_F32) {
            const bool f16 = w.first_dt == PARO_F16;
            const bool half = (shift & 2) != 0;             // the run starts in the upper half of its first word
            static_for<0, 4>([&](auto j) {
                const unsigned int v0 = sel4(q, word<j>(r), word<j + 1>(r), word<j + 2>(r), word<j + 3>(r));
                const unsigned int v1 = sel4(q, word<j + 1>(r), word<j + 2>(r), word<j + 3>(r), word<j + 4>(r));
                const unsigned int wd = half ? (v0 >> 16) | (v1 << 16) : v0;
                x[2 * j] = f16 ? cvt_lo<PARO_F16>(wd) : bf16_lo(wd);
                x[2 * j + 1] = f16 ? cvt_hi<PARO_F16>(wd) : bf16_hi(wd);
            });
        } else {
            static_for<0, 8>([&](auto j) {
                x[j] = __uint_as_float(sel4(q, word<j>(r), word<j + 1>(r), word<j + 2>(r), word<j + 3>(r)));
            });
        }
    }

    // J-th 32-bit word of the three loaded blocks, J a compile-time constant (no array, so
    // nothing the compiler could turn into an indexed access to memory)
    template <int J>
    static __device__ __forceinline__ unsigned int word(const Raw &r) {
        static_assert(J >= 0 && J < 12, "word index");
        if constexpr (J < 4) return J == 0 ? r.a.x : J == 1 ? r.a.y : J == 2 ? r.a.z : r.a.w;
        else if constexpr (J < 8) return J == 4 ? r.b.x : J == 5 ? r.b.y : J == 6 ? r.b.z : r.b.w;
        else return J == 8 ? r.c.x : J == 9 ? r.c.y : J == 10 ? r.c.z : r.c.w;
    }
};

// The tile lies in one tensor of a 2-byte dtype and every source is 16-byte aligned there: the
// same loads as the chunk layout, base pointers taken from LDS.
template <int DT>
struct Staged16Loader {
    static constexpr bool kTensor = false;
    static constexpr int kBatch = PARO_BATCH_BF16;
    struct Raw { u32x4 a; };
    const uintptr_t *s_ptr;
    int64_t byte_off;          // of the thread's first element inside the tensor
    template <bool SLOW>
    __device__ __forceinline__ void load(const SrcTable &, int k, Raw &r) const {
        r.a = ld_contrib(global_ptr<u32x4>(s_ptr[k] + (uintptr_t)byte_off));
    }
    template <bool SLOW>
    __device__ __forceinline__ void unpack(const SrcTable &, int, const Raw &r, float x[8]) const {
        unpack16x8<DT>(r.a, x);
    }
};

// ---------------------------------------------------------------------- fold
// X[i] = contributions added in table order: runs of group_len into a partial A
// (left to right), partials into X (left to right).  The first value of a run
// and the first partial are copied, not added to zero (that would lose -0).
// SLOW (tensor layout only): some thread of the wave has a tensor boundary inside its 8
// elements; contributions are then taken one at a time, each thread on its own path.
template <class Ld, bool SLOW>
__device__ __forceinline__ void fold8(const Ld &ld, const SrcTable &src, int P, int group_len, float X[8]) {
    float A[8];
    int pos = 0;
    bool first_group = true;
    constexpr int FOLD_BATCH = SLOW ? 1 : Ld::kBatch;
    for (int k0 = 0; k0 < P; k0 += FOLD_BATCH) {
        typename Ld::Raw raw[FOLD_BATCH];
        static_for<0, FOLD_BATCH>([&](auto b) {
            if (k0 + b < P) ld.template load<SLOW>(src, k0 + b, raw[b]);
        });
        static_for<0, FOLD_BATCH>([&](auto b) {
            if (k0 + b < P) {
                float x[8];
                ld.template unpack<SLOW>(src, k0 + b, raw[b], x);
                if (pos == 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) A[i] = x[i];
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) A[i] = A[i] + x[i];
                }
                if (++pos == group_len) {
                    pos = 0;
                    if (first_group) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) X[i] = A[i];
                        first_group = false;
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i) X[i] = X[i] + A[i];
                    }
                }
            }
        });
    }
}

// ---------------------------------------------------------------------- Adam
// sc = grad_scale * clip coefficient, from the global sum of squares.
__device__ __forceinline__ float scale_from_norm(const AdamConsts &a, const double *total_sumsq) {
    double coef = 1.0;
    if (a.max_norm > 0.0f) {
        const double norm = (double)a.grad_scale * sqrt(*total_sumsq);
        const double c = (double)a.max_norm / (norm + 1e-6);
        coef = c < 1.0 ? c : 1.0;
    }
    return (float)((double)a.grad_scale * coef);
}

// One element.  Every operation is a separate fp32 rounding, in this order
// (the library is compiled without FMA contraction).
__device__ __forceinline__ void adam1(const AdamConsts &a, float sc, bool decays, float g, float &p, float &m,
                                      float &v) {
    float gh = sc * g;
    if (!a.adamw && decays) gh = gh + a.wd * p;
    const float t1 = a.beta1 * m, t2 = a.omb1 * gh;
    m = t1 + t2;
    const float t3 = a.beta2 * v, t4 = gh * gh;
    const float t5 = a.omb2 * t4;
    v = t3 + t5;
    float den = sqrtf(v) / a.sqrt_bc2;
    den = den + a.eps;
    const float q = m / den;
    const float upd = a.step_size * q;
    if (a.adamw && decays) {
        const float pd = p * a.decay;
        p = pd - upd;
    } else {
        p = p - upd;
    }
}

// Which tiles a block takes: TPBK == 0: grid-stride (persistent blocks); TPBK > 0: a run of
// TPBK consecutive tiles.
#define TILE_LOOP(TPBK, tile, ntiles)                                                                       \
    for (int64_t tile = (TPBK) ? (int64_t)blockIdx.x * (TPBK) : (int64_t)blockIdx.x,                        \
                 tile##_end = (TPBK) ? min((int64_t)(ntiles), tile + (TPBK)) : (int64_t)(ntiles),           \
                 tile##_step = (TPBK) ? 1 : (int64_t)gridDim.x;                                             \
         tile < tile##_end; tile += tile##_step)

// --------------------------------------------------------------------- kernels
// Sweep 1: g = fold of the contributions; optional per-block partial of sum g^2.
template <class Ld, bool SUMSQ>
__global__ __launch_bounds__(TPB) void k_reduce(Ld ld, const SrcTable src, int P, int group_len, int64_t n,
                                                float *__restrict__ g, double *__restrict__ partials,
                                                TileSegs segs) {
    __shared__ int64_t s_off[Ld::kTensor ? TILE + 2 : 1];
    __shared__ int s_head[2];
    __shared__ uintptr_t s_ptr[Ld::kTensor ? PARO_MAX_RANKS : 1];
    segs.s_off = s_off;
    segs.s_head = s_head;
    double acc = 0.0;
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_FOLD, tile, ntiles) {
        if (Ld::kTensor) {
            segs.begin_tile(tile * TILE);
            ld.begin_tile(segs, src, P, s_ptr);
        }
        const int rel0 = threadIdx.x * EPT;
        const int64_t e = tile * TILE + rel0;
        if (e < n) {
            Where8 w;
            if (Ld::kTensor) locate8(segs, rel0, w);
            ld.prepare(e, w);
            float X[8];
            if (Ld::kTensor && ld.lean()) {
                if (ld_lean_dt(ld) == PARO_F16) {
                    Staged16Loader<PARO_F16> lean{s_ptr, ld_lean_off(ld) + (int64_t)rel0 * 2};
                    fold8<Staged16Loader<PARO_F16>, false>(lean, src, P, group_len, X);
                } else {
                    Staged16Loader<PARO_BF16> lean{s_ptr, ld_lean_off(ld) + (int64_t)rel0 * 2};
                    fold8<Staged16Loader<PARO_BF16>, false>(lean, src, P, group_len, X);
                }
            } else if (Ld::kTensor && !__all(w.one_tensor)) {
                fold8<Ld, true>(ld, src, P, group_len, X);
            } else {
                fold8<Ld, false>(ld, src, P, group_len, X);
            }
            // n is a multiple of 8 but a wave's 512-element span may be cut by the end of the range;
            // only whole spans take the transposed path (the test is wave-uniform)
            const int64_t wave_first = tile * TILE + (threadIdx.x & ~63) * EPT;
            if (PARO_G_TRANSPOSE && wave_first + 64 * EPT <= n)
                store8_f32_wave_contiguous<PARO_NT_GSTORE != 0>(g + wave_first, X);
            else
                store8_f32<PARO_NT_GSTORE != 0>(g + e, X);
            if (SUMSQ) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc += (double)X[i] * (double)X[i];
            }
        }
    }
    if (SUMSQ) {
        const double s = block_sum(acc);
        if (threadIdx.x == 0) partials[blockIdx.x] = s;
    }
}

// Adds partials in a fixed order: block b takes the slice [b*chunk, b*chunk + chunk) of the n
// values; thread t adds its slice's elements t, t+T, t+2T, ... (eight loads in flight at a time,
// added in index order); then the fixed block tree.  Launched as many-blocks -> one block.
__global__ __launch_bounds__(TPB) void k_finalize(const double *__restrict__ partials, int n, int chunk, double *out) {
    const int lo = blockIdx.x * chunk, hi = min(n, lo + chunk);
    double acc = 0.0;
    for (int k0 = lo + threadIdx.x; k0 < hi; k0 += 8 * TPB) {
        double x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = (k0 + u * TPB < hi) ? partials[k0 + u * TPB] : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    const double s = block_sum(acc);
    if (threadIdx.x == 0) out[blockIdx.x] = s;
}

// Sweep 2: Adam on the stored gradient, optionally packing bf16 parameters and
// optionally with a per-tensor weight-decay mask.
template <bool PACK, bool MASK>
__global__ __launch_bounds__(TPB) void k_adam(const AdamConsts a, const double *__restrict__ total_sumsq,
                                              const float *__restrict__ g, float *__restrict__ p,
                                              float *__restrict__ m, float *__restrict__ v,
                                              uint16_t *__restrict__ dst, int64_t n, TileSegs segs) {
    __shared__ int64_t s_off[MASK ? TILE + 2 : 1];
    __shared__ int s_head[2];
    segs.s_off = s_off;
    segs.s_head = s_head;
    // an overflowed (non-finite) gradient makes its sum of squares non-finite: the whole step is skipped
    if (a.skip_nonfinite && !isfinite(*total_sumsq)) return;
    const float sc = scale_from_norm(a, total_sumsq);
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_ADAM, tile, ntiles) {
        if (MASK) segs.begin_tile(tile * TILE);
        const int rel0 = threadIdx.x * EPT;
        const int64_t e = tile * TILE + rel0;
        if (e < n) {
            bool decays[8];
            if (MASK) {
                Where8 w;
                locate8(segs, rel0, w);
#pragma unroll
                for (int i = 0; i < 8; ++i) decays[i] = w.tens[i] < 0 || segs.tm.no_decay[w.tens[i]] == 0;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) decays[i] = true;
            }
            float gg[8], pp[8], mm[8], vv[8];
            load8_f32(g + e, gg);
            load8_f32(p + e, pp);
            load8_f32(m + e, mm);
            load8_f32(v + e, vv);
#pragma unroll
            for (int i = 0; i < 8; ++i) adam1(a, sc, decays[i], gg[i], pp[i], mm[i], vv[i]);
            store8_f32(p + e, pp);
            store8_f32(m + e, mm);
            store8_f32(v + e, vv);
            if (PACK) store8_lowp(dst + e, pp, a.pack_dtype);
        }
    }
}

// Single sweep when nothing has to wait for the norm: fold, Adam and pack; the
// reduced gradient never goes to memory.
template <class Ld, bool MASK>
__global__ __launch_bounds__(TPB) void k_fused(Ld ld, const SrcTable src, int P, int group_len, int64_t n,
                                               const AdamConsts a, float *__restrict__ p, float *__restrict__ m,
                                               float *__restrict__ v, uint16_t *__restrict__ dst, TileSegs segs) {
    constexpr bool NEED_SEGS = Ld::kTensor || MASK;
    __shared__ int64_t s_off[NEED_SEGS ? TILE + 2 : 1];
    __shared__ int s_head[2];
    __shared__ uintptr_t s_ptr[Ld::kTensor ? PARO_MAX_RANKS : 1];
    segs.s_off = s_off;
    segs.s_head = s_head;
    const float sc = a.grad_scale;                     // no clipping on this path
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_FOLD, tile, ntiles) {
        if (NEED_SEGS) segs.begin_tile(tile * TILE);
        if (Ld::kTensor) ld.begin_tile(segs, src, P, s_ptr);
        const int rel0 = threadIdx.x * EPT;
        const int64_t e = tile * TILE + rel0;
        if (e < n) {
            Where8 w;
            if (NEED_SEGS) locate8(segs, rel0, w);
            ld.prepare(e, w);
            float pp[8], mm[8], vv[8], X[8];
            load8_f32(p + e, pp);
            load8_f32(m + e, mm);
            load8_f32(v + e, vv);
            if (Ld::kTensor && ld.lean()) {
                if (ld_lean_dt(ld) == PARO_F16) {
                    Staged16Loader<PARO_F16> lean{s_ptr, ld_lean_off(ld) + (int64_t)rel0 * 2};
                    fold8<Staged16Loader<PARO_F16>, false>(lean, src, P, group_len, X);
                } else {
                    Staged16Loader<PARO_BF16> lean{s_ptr, ld_lean_off(ld) + (int64_t)rel0 * 2};
                    fold8<Staged16Loader<PARO_BF16>, false>(lean, src, P, group_len, X);
                }
            } else if (Ld::kTensor && !__all(w.one_tensor)) {
                fold8<Ld, true>(ld, src, P, group_len, X);
            } else {
                fold8<Ld, false>(ld, src, P, group_len, X);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                bool decays = true;
                if (MASK) decays = w.tens[i] < 0 || segs.tm.no_decay[w.tens[i]] == 0;
                adam1(a, sc, decays, X[i], pp[i], mm[i], vv[i]);
            }
            store8_f32(p + e, pp);
            store8_f32(m + e, mm);
            store8_f32(v + e, vv);
            store8_lowp(dst + e, pp, a.pack_dtype);
        }
    }
}

// Low-precision pack alone.
__global__ __launch_bounds__(TPB) void k_pack(const float *__restrict__ p, uint16_t *__restrict__ dst, int64_t n,
                                              int pack_dtype) {
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_ADAM, tile, ntiles) {
        const int64_t e = tile * TILE + threadIdx.x * EPT;
        if (e < n) {
            float pp[8];
            load8_f32(p + e, pp);
            store8_lowp(dst + e, pp, pack_dtype);
        }
    }
}

// One ring hop / one accumulation: out = a + b, element by element in fp32.
template <int DT>
__device__ __forceinline__ void hop_load8(const void *a, int64_t e, float x[8]) {
    if (DT != PARO_F32) {
        const u32x4 q = ld_contrib(reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(a) + e));
        unpack16x8<DT>(q, x);
    } else {
        load8_f32<false>(static_cast<const float *>(a) + e, x);
    }
}
template <int DT>
__device__ __forceinline__ float hop_load1(const void *a, int64_t i) {
    return DT != PARO_F32 ? cvt16(static_cast<const uint16_t *>(a)[i], DT) : static_cast<const float *>(a)[i];
}

template <int DA, int DB>
__global__ __launch_bounds__(TPB) void k_hop(const void *a, const void *b, float *out, int64_t n) {
    const int64_t e = ((int64_t)blockIdx.x * TPB + threadIdx.x) * EPT;
    if (e + EPT <= n) {
        float x[8], y[8];
        hop_load8<DA>(a, e, x);
        hop_load8<DB>(b, e, y);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = x[i] + y[i];
        store8_f32(out + e, x);
    } else {
        for (int64_t i = e; i < n; ++i) out[i] = hop_load1<DA>(a, i) + hop_load1<DB>(b, i);   // last, partial group
    }
}

// Plain copy of n 16-byte units (an all-gather message landing in the parameter buffer).
__global__ __launch_bounds__(TPB) void k_copy16(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) dst[i] = ld_contrib(src + i);
}

}  // namespace

// =========================================================================
// host side: validation and launches
// =========================================================================
namespace {

using paro::fail;

#define PARO_HIP(expr)                                                                             \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(PARO_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

int check_ptr(const void *p, const char *what) {
    if (!p) return fail(PARO_EINVAL, std::string(what) + " is NULL");
    if (reinterpret_cast<uintptr_t>(p) & 15) return fail(PARO_EALIGN, std::string(what) + " is not 16-byte aligned");
    return PARO_OK;
}

template <class T>
int upload(T **dst, const T *src, size_t n) {
    PARO_HIP(hipMalloc(reinterpret_cast<void **>(dst), (n ? n : 1) * sizeof(T)));
    if (n) PARO_HIP(hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice));
    return PARO_OK;
}

// Creates the plan's device tables on the current device, once.
int ensure_device(paro_plan_t *pl) {
    std::lock_guard<std::mutex> lock(pl->dev_mutex);
    int dev = -1;
    PARO_HIP(hipGetDevice(&dev));
    if (pl->dev.device >= 0) {
        if (pl->dev.device != dev)
            return fail(PARO_EINVAL, "the plan's device tables live on another device than the current one");
        return PARO_OK;
    }
    paro_device_tables d;
    PARO_HIP(hipDeviceGetAttribute(&d.n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if (d.n_cu < 1) d.n_cu = 256;
    int rc;
    if ((rc = upload(&d.nz_off, pl->nz_off.data(), pl->nz_off.size()))) return rc;
    if ((rc = upload(&d.nz_tensor, pl->nz_tensor.data(), pl->nz_tensor.size()))) return rc;
    if ((rc = upload(&d.dtype, pl->dtype.data(), pl->dtype.size()))) return rc;
    if ((rc = upload(&d.no_decay, pl->no_decay.data(), pl->no_decay.size()))) return rc;
    // per-tile summaries for chunk-aligned launches over the tensor layout (16 B per 2048 elements)
    d.tiles_per_chunk = (pl->L + TILE - 1) / TILE;
    if (pl->T > 1 && (int64_t)pl->P * d.tiles_per_chunk <= (int64_t)4 << 20) {
        std::vector<paro_tile_info> tab((size_t)pl->P * d.tiles_per_chunk);
        const int64_t n_nz = (int64_t)pl->nz_tensor.size();
        for (int c = 0; c < pl->P; ++c) {
            for (int64_t i = 0; i < d.tiles_per_chunk; ++i) {
                const int64_t f0 = (int64_t)c * pl->L + i * TILE;
                const int64_t f1 = std::min(f0 + (int64_t)TILE, (int64_t)(c + 1) * pl->L);   // end of the tile
                paro_tile_info &ti = tab[(size_t)c * d.tiles_per_chunk + i];
                ti.toff = 0;
                ti.tensor = -1;
                ti.first_seg = (int32_t)n_nz;
                if (f0 >= pl->total) continue;
                const int64_t k = std::upper_bound(pl->nz_off.begin(), pl->nz_off.end(), f0) - pl->nz_off.begin() - 1;
                ti.first_seg = (int32_t)k;
                if (f1 <= pl->nz_off[k + 1]) {
                    ti.tensor = pl->nz_tensor[k];
                    ti.toff = f0 - pl->nz_off[k];
                    ti.first_seg = pl->dtype[ti.tensor];          // single-tensor tiles: the field carries the dtype
                }
            }
        }
        if ((rc = upload(&d.tile_tab, tab.data(), tab.size()))) return rc;
    }
    // one partial per block of the largest sweep-1 launch (a launch covers one chunk of L elements)
    // (a launch covers one chunk of L elements), followed by room for the second-level sums
    int64_t n_part = (pl->L + TILE - 1) / TILE;
    if (n_part < PARO_MAX_PARTIALS) n_part = PARO_MAX_PARTIALS;
    d.n_partials = n_part;
    const int64_t n_level2 = (n_part + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
    PARO_HIP(hipMalloc(reinterpret_cast<void **>(&d.partials), (n_part + n_level2) * sizeof(double)));
    d.device = dev;
    pl->dev = d;
    return PARO_OK;
}

// Blocks of a launch over n elements, for a kernel that takes tpbk tiles per block (0 = persistent).
int grid_for(const paro_plan_t *pl, int64_t n, int tpbk) {
    const int64_t ntiles = (n + TILE - 1) / TILE;
    if (tpbk > 0) {
        const int64_t nb = (ntiles + tpbk - 1) / tpbk;
        return (int)(nb < 1 ? 1 : nb);
    }
    int64_t cap = (int64_t)pl->dev.n_cu * BLOCKS_PER_CU;
    if (cap > PARO_MAX_PARTIALS) cap = PARO_MAX_PARTIALS;
    return (int)(ntiles < cap ? (ntiles < 1 ? 1 : ntiles) : cap);
}

TileSegs segs_for(const paro_plan_t *pl, int64_t range_begin, bool chunk_launch) {
    TileSegs s;
    s.s_off = nullptr;
    s.s_head = nullptr;
    s.tm.nz_off = pl->dev.nz_off;
    s.tm.nz_tensor = pl->dev.nz_tensor;
    s.tm.dtype = pl->dev.dtype;
    s.tm.no_decay = pl->dev.no_decay;
    s.tm.n_nz = (int)pl->nz_tensor.size();
    s.tm.total = pl->total;
    s.range_begin = range_begin;
    s.tile_tab = nullptr;
    s.single_tensor = -1;
    s.single_toff = 0;
    s.single_dt = PARO_BF16;
    // the per-tile table is laid out per chunk: usable when the launch starts on a chunk boundary
    // and stays inside that chunk
    if (pl->dev.tile_tab && chunk_launch && range_begin % pl->L == 0)
        s.tile_tab = pl->dev.tile_tab + (range_begin / pl->L) * pl->dev.tiles_per_chunk;
    return s;
}

int check_common(const paro_plan_t *pl, int rank, const char *fn) {
    if (!pl) return fail(PARO_EINVAL, std::string(fn) + ": plan is NULL");
    if (rank < 0 || rank >= pl->P) return fail(PARO_ERANGE, std::string(fn) + ": rank out of range");
    return PARO_OK;
}

int check_contrib(const paro_plan_t *pl, const void *const *contrib, int layout, const char *fn) {
    if (!contrib) return fail(PARO_EINVAL, std::string(fn) + ": contrib is NULL");
    if (layout != PARO_CHUNK && layout != PARO_TENSORS) return fail(PARO_EINVAL, std::string(fn) + ": bad layout");
    if (layout == PARO_CHUNK && !pl->uniform_dtype)
        return fail(PARO_EINVAL, std::string(fn) + ": chunk layout needs one gradient dtype for all tensors");
    for (int q = 0; q < pl->P; ++q) {
        if (!contrib[q]) return fail(PARO_EINVAL, std::string(fn) + ": a contribution pointer is NULL");
        if (layout == PARO_CHUNK && (reinterpret_cast<uintptr_t>(contrib[q]) & 15))
            return fail(PARO_EALIGN, std::string(fn) + ": a contribution is not 16-byte aligned");
        if (layout == PARO_TENSORS && (reinterpret_cast<uintptr_t>(contrib[q]) & 7))
            return fail(PARO_EALIGN, std::string(fn) + ": a pointer table is not 8-byte aligned");
    }
    return PARO_OK;
}

int adam_consts(const paro_adam_t *hp, AdamConsts *a, const char *fn) {
    if (!hp) return fail(PARO_EINVAL, std::string(fn) + ": hp is NULL");
    if (hp->step < 1) return fail(PARO_EINVAL, std::string(fn) + ": step must be >= 1");
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f && hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(PARO_EINVAL, std::string(fn) + ": betas must lie in [0, 1)");
    // element-independent scalars: formed in fp64 from the fp32 hyper-parameters, rounded once
    const double b1 = hp->beta1, b2 = hp->beta2;
    const float bc1 = (float)(1.0 - std::pow(b1, (double)hp->step));
    const float bc2 = (float)(1.0 - std::pow(b2, (double)hp->step));
    a->beta1 = hp->beta1;
    a->beta2 = hp->beta2;
    a->omb1 = (float)(1.0 - b1);
    a->omb2 = (float)(1.0 - b2);
    a->eps = hp->eps;
    a->step_size = (float)((double)hp->lr / (double)bc1);
    a->sqrt_bc2 = (float)std::sqrt((double)bc2);
    a->decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);
    a->wd = hp->weight_decay;
    a->grad_scale = hp->grad_scale;
    a->max_norm = hp->max_norm;
    a->adamw = hp->adamw ? 1 : 0;
    a->skip_nonfinite = hp->skip_nonfinite ? 1 : 0;
    a->pack_dtype = PARO_BF16;         // the entry points overwrite it with the plan's
    return PARO_OK;
}

// Pointer table of a chunk in fold order.  Chunk layout: pointers advanced to the
// chunk's first element inside the update range.
void src_table(const paro_plan_t *pl, int chunk, const void *const *contrib, int layout, int64_t chunk_off_in_range,
               SrcTable *tab, int *group_len) {
    int32_t order[PARO_MAX_RANKS];
    int32_t gl = 0;
    paro::fold_order(pl, chunk, order, &gl);
    const int64_t esize = pl->dtype[0] == PARO_F32 ? 4 : 2;
    for (int k = 0; k < pl->P; ++k) {
        const char *base = static_cast<const char *>(contrib[order[k]]);
        tab->p[k] = layout == PARO_CHUNK ? base + chunk_off_in_range * esize : base;
    }
    for (int k = pl->P; k < PARO_MAX_RANKS; ++k) tab->p[k] = nullptr;
    *group_len = gl;
}

template <bool SUMSQ>
void launch_reduce(const paro_plan_t *pl, int layout, const SrcTable &tab, int group_len, int64_t flat_begin, float *g,
                   hipStream_t st) {
    const int64_t n = pl->L;
    const int grid = grid_for(pl, n, PARO_TPBK_FOLD);
    TileSegs segs = segs_for(pl, flat_begin, true);
    double *partials = pl->dev.partials;
    if (layout == PARO_TENSORS) {
        TensorLoader ld;
        ld.dtype = pl->dev.dtype;
        hipLaunchKernelGGL((k_reduce<TensorLoader, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, g,
                           partials, segs);
    } else if (pl->dtype[0] == PARO_BF16) {
        ChunkLoader<PARO_BF16> ld{0};
        hipLaunchKernelGGL((k_reduce<ChunkLoader<PARO_BF16>, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, g, partials, segs);
    } else if (pl->dtype[0] == PARO_F16) {
        ChunkLoader<PARO_F16> ld{0};
        hipLaunchKernelGGL((k_reduce<ChunkLoader<PARO_F16>, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, g, partials, segs);
    } else {
        ChunkLoader<PARO_F32> ld{0};
        hipLaunchKernelGGL((k_reduce<ChunkLoader<PARO_F32>, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, g, partials, segs);
    }
}

template <bool MASK>
void launch_fused(const paro_plan_t *pl, int layout, const SrcTable &tab, int group_len, int64_t flat_begin,
                  const AdamConsts &a, float *p, float *m, float *v, uint16_t *dst, hipStream_t st) {
    const int64_t n = pl->L;
    const int grid = grid_for(pl, n, PARO_TPBK_FOLD);
    TileSegs segs = segs_for(pl, flat_begin, true);
    if (layout == PARO_TENSORS) {
        TensorLoader ld;
        ld.dtype = pl->dev.dtype;
        hipLaunchKernelGGL((k_fused<TensorLoader, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, a,
                           p, m, v, dst, segs);
    } else if (pl->dtype[0] == PARO_BF16) {
        ChunkLoader<PARO_BF16> ld{0};
        hipLaunchKernelGGL((k_fused<ChunkLoader<PARO_BF16>, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, a, p, m, v, dst, segs);
    } else if (pl->dtype[0] == PARO_F16) {
        ChunkLoader<PARO_F16> ld{0};
        hipLaunchKernelGGL((k_fused<ChunkLoader<PARO_F16>, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, a, p, m, v, dst, segs);
    } else {
        ChunkLoader<PARO_F32> ld{0};
        hipLaunchKernelGGL((k_fused<ChunkLoader<PARO_F32>, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P,
                           group_len, n, a, p, m, v, dst, segs);
    }
}

// Sweep 1 over the whole update range, chunk by chunk; the sum of squares covers
// the rank's own chunk only.
int do_reduce(paro_plan_t *pl, int rank, const void *const *contrib, int layout, float *grad_out, double *sumsq_out,
              hipStream_t st) {
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    const int own = paro::chunk_of_rank(pl, rank);
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {
        SrcTable tab;
        int gl;
        const int64_t lo = c * pl->L - ob;
        src_table(pl, (int)c, contrib, layout, lo, &tab, &gl);
        if (c == own && sumsq_out)
            launch_reduce<true>(pl, layout, tab, gl, c * pl->L, grad_out + lo, st);
        else
            launch_reduce<false>(pl, layout, tab, gl, c * pl->L, grad_out + lo, st);
        PARO_HIP(hipGetLastError());
    }
    if (sumsq_out) {
        const int n_part = grid_for(pl, pl->L, PARO_TPBK_FOLD);
        if (n_part > 2 * FINALIZE_CHUNK) {       // two levels: slices of 2048 partials, then their sums
            const int nb = (n_part + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
            double *level2 = pl->dev.partials + pl->dev.n_partials;
            hipLaunchKernelGGL(k_finalize, dim3(nb), dim3(TPB), 0, st, pl->dev.partials, n_part, FINALIZE_CHUNK, level2);
            PARO_HIP(hipGetLastError());
            hipLaunchKernelGGL(k_finalize, dim3(1), dim3(TPB), 0, st, level2, nb, nb, sumsq_out);
        } else {
            hipLaunchKernelGGL(k_finalize, dim3(1), dim3(TPB), 0, st, pl->dev.partials, n_part, n_part, sumsq_out);
        }
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

int do_adam(paro_plan_t *pl, int rank, const AdamConsts &a, const float *grad, const double *total_sumsq, float *p,
            float *m, float *v, uint16_t *dst /* nullable: no pack */, hipStream_t st) {
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    const int grid = grid_for(pl, on, PARO_TPBK_ADAM);
    TileSegs segs = segs_for(pl, ob, false);
    const bool mask = pl->any_no_decay;
    if (dst && mask)
        hipLaunchKernelGGL((k_adam<true, true>), dim3(grid), dim3(TPB), 0, st, a, total_sumsq, grad, p, m, v, dst, on, segs);
    else if (dst)
        hipLaunchKernelGGL((k_adam<true, false>), dim3(grid), dim3(TPB), 0, st, a, total_sumsq, grad, p, m, v, dst, on, segs);
    else if (mask)
        hipLaunchKernelGGL((k_adam<false, true>), dim3(grid), dim3(TPB), 0, st, a, total_sumsq, grad, p, m, v, dst, on, segs);
    else
        hipLaunchKernelGGL((k_adam<false, false>), dim3(grid), dim3(TPB), 0, st, a, total_sumsq, grad, p, m, v, dst, on, segs);
    PARO_HIP(hipGetLastError());
    return PARO_OK;
}

}  // namespace

extern "C" {

void paro_plan_destroy(paro_plan_t *pl) {
    if (!pl) return;
    if (pl->dev.device >= 0) {
        // frees are best effort: the plan may outlive the HIP runtime at process exit
        (void)hipFree(pl->dev.nz_off);
        (void)hipFree(pl->dev.nz_tensor);
        (void)hipFree(pl->dev.dtype);
        (void)hipFree(pl->dev.no_decay);
        (void)hipFree(pl->dev.partials);
        if (pl->dev.tile_tab) (void)hipFree(pl->dev.tile_tab);
    }
    delete pl;
}

int paro_reduce_shard(paro_plan_t *pl, int rank, const void *const *contrib, int layout, float *grad_out,
                      double *sumsq_out, void *stream) {
    int rc;
    if ((rc = check_common(pl, rank, "paro_reduce_shard"))) return rc;
    if ((rc = check_contrib(pl, contrib, layout, "paro_reduce_shard"))) return rc;
    if ((rc = check_ptr(grad_out, "paro_reduce_shard: grad_out"))) return rc;
    if (sumsq_out && (reinterpret_cast<uintptr_t>(sumsq_out) & 7))
        return fail(PARO_EALIGN, "paro_reduce_shard: sumsq_out is not 8-byte aligned");
    if ((rc = ensure_device(pl))) return rc;
    return do_reduce(pl, rank, contrib, layout, grad_out, sumsq_out, static_cast<hipStream_t>(stream));
}

int paro_adam_shard(paro_plan_t *pl, int rank, const paro_adam_t *hp, const float *grad, const double *total_sumsq,
                    float *p, float *m, float *v, uint16_t *dst_base, void *stream) {
    int rc;
    AdamConsts a;
    if ((rc = check_common(pl, rank, "paro_adam_shard"))) return rc;
    if ((rc = adam_consts(hp, &a, "paro_adam_shard"))) return rc;
    if ((rc = check_ptr(grad, "paro_adam_shard: grad"))) return rc;
    if ((rc = check_ptr(p, "paro_adam_shard: p"))) return rc;
    if ((rc = check_ptr(m, "paro_adam_shard: m"))) return rc;
    if ((rc = check_ptr(v, "paro_adam_shard: v"))) return rc;
    if ((a.max_norm > 0.0f || a.skip_nonfinite) && !total_sumsq)
        return fail(PARO_EINVAL, "paro_adam_shard: clipping and skip_nonfinite need total_sumsq");
    a.pack_dtype = pl->pack_dtype;
    if (dst_base && (reinterpret_cast<uintptr_t>(dst_base) & 15))
        return fail(PARO_EALIGN, "paro_adam_shard: dst_base is not 16-byte aligned");
    if ((rc = ensure_device(pl))) return rc;
    uint16_t *dst = nullptr;
    if (dst_base) {
        int64_t dl, so, sl;
        paro_pack_slot(pl, rank, &dl, &so, &sl);
        dst = dst_base + so;
    }
    return do_adam(pl, rank, a, grad, total_sumsq, p, m, v, dst, static_cast<hipStream_t>(stream));
}

int paro_pack_params(paro_plan_t *pl, int rank, const float *p, uint16_t *dst_base, void *stream) {
    int rc;
    if ((rc = check_common(pl, rank, "paro_pack_params"))) return rc;
    if ((rc = check_ptr(p, "paro_pack_params: p"))) return rc;
    if ((rc = check_ptr(dst_base, "paro_pack_params: dst_base"))) return rc;
    if ((rc = ensure_device(pl))) return rc;
    int64_t dl, so, sl;
    paro_pack_slot(pl, rank, &dl, &so, &sl);
    hipLaunchKernelGGL(k_pack, dim3(grid_for(pl, sl, PARO_TPBK_ADAM)), dim3(TPB), 0, static_cast<hipStream_t>(stream), p,
                       dst_base + so, sl, pl->pack_dtype);
    PARO_HIP(hipGetLastError());
    return PARO_OK;
}

int paro_step_fused(paro_plan_t *pl, int rank, const void *const *contrib, int layout, const paro_adam_t *hp,
                    float *grad_scratch, double *sumsq_scratch, float *p, float *m, float *v, uint16_t *dst_base,
                    void *stream) {
    int rc;
    AdamConsts a;
    if ((rc = check_common(pl, rank, "paro_step_fused"))) return rc;
    if ((rc = check_contrib(pl, contrib, layout, "paro_step_fused"))) return rc;
    if ((rc = adam_consts(hp, &a, "paro_step_fused"))) return rc;
    if ((rc = check_ptr(p, "paro_step_fused: p"))) return rc;
    if ((rc = check_ptr(m, "paro_step_fused: m"))) return rc;
    if ((rc = check_ptr(v, "paro_step_fused: v"))) return rc;
    if ((rc = check_ptr(dst_base, "paro_step_fused: dst_base"))) return rc;
    a.pack_dtype = pl->pack_dtype;
    const bool clip = a.max_norm > 0.0f || a.skip_nonfinite;       // both need the norm before the update
    if (clip) {
        if ((rc = check_ptr(grad_scratch, "paro_step_fused: grad_scratch"))) return rc;
        if (!sumsq_scratch || (reinterpret_cast<uintptr_t>(sumsq_scratch) & 7))
            return fail(sumsq_scratch ? PARO_EALIGN : PARO_EINVAL, "paro_step_fused: clipping and skip_nonfinite need sumsq_scratch");
    }
    if ((rc = ensure_device(pl))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t dl, so, sl, ob, on;
    paro_pack_slot(pl, rank, &dl, &so, &sl);
    uint16_t *dst = dst_base + so;
    if (clip) {
        if ((rc = do_reduce(pl, rank, contrib, layout, grad_scratch, sumsq_scratch, st))) return rc;
        return do_adam(pl, rank, a, grad_scratch, sumsq_scratch, p, m, v, dst, st);
    }
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {
        SrcTable tab;
        int gl;
        const int64_t lo = c * pl->L - ob;
        src_table(pl, (int)c, contrib, layout, lo, &tab, &gl);
        if (pl->any_no_decay)
            launch_fused<true>(pl, layout, tab, gl, c * pl->L, a, p + lo, m + lo, v + lo, dst + lo, st);
        else
            launch_fused<false>(pl, layout, tab, gl, c * pl->L, a, p + lo, m + lo, v + lo, dst + lo, st);
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

}  // extern "C"


// ---- ring hops and scheduled transfers ----------------------------------------
namespace {
int launch_hop(const void *a, int da, const void *b, int db, float *out, int64_t n, hipStream_t st) {
    if (n <= 0) return PARO_OK;
    const int64_t groups = (n + EPT - 1) / EPT;
    const int grid = (int)((groups + TPB - 1) / TPB);
#define PARO_HOP_CASE(A, B)                                                                                   \
    if (da == A && db == B) hipLaunchKernelGGL((k_hop<A, B>), dim3(grid), dim3(TPB), 0, st, a, b, out, n)
    PARO_HOP_CASE(PARO_BF16, PARO_BF16); PARO_HOP_CASE(PARO_BF16, PARO_F32); PARO_HOP_CASE(PARO_BF16, PARO_F16);
    PARO_HOP_CASE(PARO_F32, PARO_BF16);  PARO_HOP_CASE(PARO_F32, PARO_F32);  PARO_HOP_CASE(PARO_F32, PARO_F16);
    PARO_HOP_CASE(PARO_F16, PARO_BF16);  PARO_HOP_CASE(PARO_F16, PARO_F32);  PARO_HOP_CASE(PARO_F16, PARO_F16);
#undef PARO_HOP_CASE
    PARO_HIP(hipGetLastError());
    return PARO_OK;
}
}  // namespace

extern "C" {

int paro_ring_hop(paro_plan_t *pl, const void *partial_in, int in_dtype, const void *local, int local_dtype, float *out,
                  int64_t n, void *stream) {
    int rc;
    if (!pl) return fail(PARO_EINVAL, "paro_ring_hop: plan is NULL");
    if (n < 0) return fail(PARO_EINVAL, "paro_ring_hop: n is negative");
    if (in_dtype < PARO_BF16 || in_dtype > PARO_F16 || local_dtype < PARO_BF16 || local_dtype > PARO_F16)
        return fail(PARO_EINVAL, "paro_ring_hop: bad dtype");
    if ((rc = check_ptr(partial_in, "paro_ring_hop: partial_in"))) return rc;
    if ((rc = check_ptr(local, "paro_ring_hop: local"))) return rc;
    if ((rc = check_ptr(out, "paro_ring_hop: out"))) return rc;
    if ((in_dtype != PARO_F32 && static_cast<const void *>(out) == partial_in) ||
        (local_dtype != PARO_F32 && static_cast<const void *>(out) == local))
        return fail(PARO_EINVAL, "paro_ring_hop: out may only alias an fp32 operand");
    if ((rc = ensure_device(pl))) return rc;
    return launch_hop(partial_in, in_dtype, local, local_dtype, out, n, static_cast<hipStream_t>(stream));
}

int64_t paro_collective_step(paro_plan_t *pl, int rank, int sched, int collective, int phase, int ring, int step,
                             void *const *bufs, void *stream) {
    int rc;
    if ((rc = check_common(pl, rank, "paro_collective_step"))) return rc;
    if (!bufs) return fail(PARO_EINVAL, "paro_collective_step: bufs is NULL");
    for (int q = 0; q < pl->P; ++q)
        if ((rc = check_ptr(bufs[q], "paro_collective_step: a buffer"))) return rc;
    const int64_t count = paro_schedule(pl, rank, sched, collective, nullptr, 0);
    if (count < 0) return count;
    std::vector<paro_msg_t> msgs((size_t)count);
    if (count && paro_schedule(pl, rank, sched, collective, msgs.data(), count) < 0) return PARO_EINVAL;
    if ((rc = ensure_device(pl))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t received = 0;
    for (const paro_msg_t &m : msgs) {
        if (m.phase != phase || m.ring != ring || m.step != step) continue;
        if (collective == PARO_RS) {
            const float *from = static_cast<const float *>(bufs[m.recv_from]) + m.recv_off;
            float *mine = static_cast<float *>(bufs[rank]) + m.recv_off;
            if ((rc = launch_hop(from, PARO_F32, mine, PARO_F32, mine, m.recv_len, st))) return rc;
        } else {
            const uint16_t *from = static_cast<const uint16_t *>(bufs[m.recv_from]) + m.recv_off;
            uint16_t *mine = static_cast<uint16_t *>(bufs[rank]) + m.recv_off;
            const int64_t n16 = m.recv_len / 8;             // ranges are whole chunks: multiples of 8 elements
            const int grid = (int)((n16 + TPB - 1) / TPB);
            if (n16 > 0) {
                hipLaunchKernelGGL(k_copy16, dim3(grid), dim3(TPB), 0, st, reinterpret_cast<const u32x4 *>(from),
                                   reinterpret_cast<u32x4 *>(mine), n16);
                PARO_HIP(hipGetLastError());
            }
        }
        received += m.recv_len;
    }
    return received;
}

}  // extern "C"
