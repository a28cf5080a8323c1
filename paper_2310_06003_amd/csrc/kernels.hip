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
#include <new>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "plan.hpp"

#include "device_util.hpp"
#include "loaders.hpp"

namespace {

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

// Which tiles a block takes: a run of TPBK consecutive tiles of the launch's range, or, when the
// launch comes with a list of tiles, a run of TPBK entries of that list.
#define TILE_LOOP(TPBK, tile, ntiles, list, n_list)                                                          \
    for (int64_t it_ = (int64_t)blockIdx.x * (TPBK),                                                         \
                 it_end_ = min((list) ? (int64_t)(n_list) : (int64_t)(ntiles), it_ + (TPBK)), tile = 0;      \
         it_ < it_end_ && ((tile = (list) ? (int64_t)(list)[it_] : it_), true); ++it_)

// --------------------------------------------------------------------- kernels
// Sweep 1: g = fold of the contributions; optional per-block partial of sum g^2.
template <class Ld, bool SUMSQ>
__global__ __launch_bounds__(TPB) void k_reduce(Ld ld, const SrcTable src, int P, int group_len, int64_t n,
                                                float *__restrict__ g, double *__restrict__ partials,
                                                TileSegs segs, const int32_t *__restrict__ tile_list, int n_list) {
    __shared__ int64_t s_off[Ld::kTensor ? TILE + 2 : 1];
    __shared__ int s_head[2];
    __shared__ uintptr_t s_ptr[Ld::kTensor ? PARO_MAX_RANKS : 1];
    segs.s_off = s_off;
    segs.s_head = s_head;
    double acc = 0.0;
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_FOLD, tile, ntiles, tile_list, n_list) {
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

// Sweep 1 for the chunk layout: 4 elements per thread in one-wave blocks.  Every load
// instruction of a wave covers 512 (2-byte dtypes) or 1024 consecutive bytes, the store 1 KB,
// and the many short-lived waves interleave reads and writes more finely than 8-element
// threads in 256-thread blocks did (measured: 3-4 % faster at P = 16).
template <int DT, bool SUMSQ>
__global__ __launch_bounds__(PARO_FOLD4_TPB) void k_reduce4(const SrcTable src, int P, int group_len, int64_t n,
                                                            float *__restrict__ g, double *__restrict__ partials) {
    const int64_t e = ((int64_t)blockIdx.x * PARO_FOLD4_TPB + threadIdx.x) * 4;     // n is a multiple of 8
    double acc = 0.0;
    if (e < n) {
        Chunk4Loader<DT> ld{e};
        float X[4];
        fold8<Chunk4Loader<DT>, false>(ld, src, P, group_len, X);
        st_as<PARO_NT_GSTORE != 0>(reinterpret_cast<f32x4 *>(g + e), f32x4{X[0], X[1], X[2], X[3]});
        if (SUMSQ) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc += (double)X[i] * (double)X[i];
        }
    }
    if (SUMSQ) {
        const double s = block_sum<PARO_FOLD4_TPB>(acc);
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
                                              uint16_t *__restrict__ dst, int64_t n, TileSegs segs,
                                              const int32_t *__restrict__ tile_list, int n_list) {
    __shared__ int64_t s_off[MASK ? TILE + 2 : 1];
    __shared__ int s_head[2];
    segs.s_off = s_off;
    segs.s_head = s_head;
    // an overflowed (non-finite) gradient makes its sum of squares non-finite: the whole step is skipped
    if (a.skip_nonfinite && !isfinite(*total_sumsq)) return;
    const float sc = scale_from_norm(a, total_sumsq);
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_ADAM, tile, ntiles, tile_list, n_list) {
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

// ---- 4 elements per thread, one-wave blocks: the shape of the sweeps that need no per-element
// look-up (chunk layout, no tensor exempt from weight decay).  Every load and store instruction
// of a wave covers 1 KB of consecutive addresses (512 B for 2-byte data) - whole cache lines,
// which is what lets the streaming policy be used both ways without partial-line writes.
constexpr bool ADAM4_LNT = (PARO_NT_ADAM4 & 1) != 0, ADAM4_SNT = (PARO_NT_ADAM4 & 2) != 0;

struct State4 { f32x4 p, m, v; };

__device__ __forceinline__ State4 load_state4(const float *p, const float *m, const float *v, int64_t e) {
    State4 s;
    s.p = ld_as<ADAM4_LNT>(reinterpret_cast<const f32x4 *>(p + e));
    s.m = ld_as<ADAM4_LNT>(reinterpret_cast<const f32x4 *>(m + e));
    s.v = ld_as<ADAM4_LNT>(reinterpret_cast<const f32x4 *>(v + e));
    return s;
}

// Adam on the thread's 4 elements, state and (optionally) the low-precision copy written back.
template <bool PACK>
__device__ __forceinline__ void update4(const AdamConsts &a, float sc, bool decays, const float gg[4], const State4 &s,
                                        float *p, float *m, float *v, uint16_t *dst, int64_t e) {
    float pp[4] = {s.p.x, s.p.y, s.p.z, s.p.w}, mm[4] = {s.m.x, s.m.y, s.m.z, s.m.w},
          vv[4] = {s.v.x, s.v.y, s.v.z, s.v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) adam1(a, sc, decays, gg[i], pp[i], mm[i], vv[i]);
    st_as<ADAM4_SNT>(reinterpret_cast<f32x4 *>(p + e), f32x4{pp[0], pp[1], pp[2], pp[3]});
    st_as<ADAM4_SNT>(reinterpret_cast<f32x4 *>(m + e), f32x4{mm[0], mm[1], mm[2], mm[3]});
    st_as<ADAM4_SNT>(reinterpret_cast<f32x4 *>(v + e), f32x4{vv[0], vv[1], vv[2], vv[3]});
    if (PACK) {
        u32x2 w;
        if (a.pack_dtype == PARO_F16) {
            w.x = f32_to_f16_bits(pp[0]) | (f32_to_f16_bits(pp[1]) << 16);
            w.y = f32_to_f16_bits(pp[2]) | (f32_to_f16_bits(pp[3]) << 16);
        } else {
            w.x = f32_to_bf16_rne(pp[0]) | (f32_to_bf16_rne(pp[1]) << 16);
            w.y = f32_to_bf16_rne(pp[2]) | (f32_to_bf16_rne(pp[3]) << 16);
        }
        st_as<ADAM4_SNT>(reinterpret_cast<u32x2 *>(dst + e), w);
    }
}

// Sweep 2 without a decay mask.
template <bool PACK>
__global__ __launch_bounds__(PARO_ADAM4_TPB) void k_adam4(const AdamConsts a, const double *__restrict__ total_sumsq,
                                                          const float *__restrict__ g, float *__restrict__ p,
                                                          float *__restrict__ m, float *__restrict__ v,
                                                          uint16_t *__restrict__ dst, int64_t n) {
    if (a.skip_nonfinite && !isfinite(*total_sumsq)) return;
    const float sc = scale_from_norm(a, total_sumsq);
    const int64_t e = ((int64_t)blockIdx.x * PARO_ADAM4_TPB + threadIdx.x) * 4;      // n is a multiple of 8
    if (e >= n) return;
    const f32x4 G = ld_as<ADAM4_LNT>(reinterpret_cast<const f32x4 *>(g + e));
    const State4 s = load_state4(p, m, v, e);
    const float gg[4] = {G.x, G.y, G.z, G.w};
    update4<PACK>(a, sc, true, gg, s, p, m, v, dst, e);
}

// Single sweep (no clipping), chunk layout, no decay mask: fold, Adam and pack.
template <int DT>
__global__ __launch_bounds__(PARO_FOLD4_TPB) void k_fused4(const SrcTable src, int P, int group_len, int64_t n,
                                                           const AdamConsts a, float *__restrict__ p,
                                                           float *__restrict__ m, float *__restrict__ v,
                                                           uint16_t *__restrict__ dst) {
    const int64_t e = ((int64_t)blockIdx.x * PARO_FOLD4_TPB + threadIdx.x) * 4;
    if (e >= n) return;
    const State4 s = load_state4(p, m, v, e);
    Chunk4Loader<DT> ld{e};
    float X[4];
    fold8<Chunk4Loader<DT>, false>(ld, src, P, group_len, X);
    update4<true>(a, a.grad_scale, true, X, s, p, m, v, dst, e);
}

// ---- the one-wave shape for work that depends on the tensor an element belongs to (tensor
// layout, weight-decay mask).  The plan's per-tile table says, for every 2048-element tile of a
// chunk, whether it lies inside one tensor (then the 8 one-wave blocks of the tile know their
// tensor and offset without any search), is all padding, or holds a tensor boundary.  Boundary
// tiles are left to the tile-at-a-time kernels, which then run over the plan's list of such
// tiles only; the blocks here return at once for them.
struct Piece {
    int tensor;        // >= 0: the block's 256 elements lie in this tensor; -1: boundary tile; -2: padding
    int dt;            // the tensor's gradient dtype
    int64_t toff;      // offset of the block's first element inside the tensor
};

__device__ __forceinline__ Piece piece_of(const paro_tile_info *__restrict__ tile_tab, int64_t e0) {
    const paro_tile_info info = tile_tab[e0 / TILE];           // one address for the whole wave
    Piece pc;
    pc.tensor = __builtin_amdgcn_readfirstlane(info.tensor);  // tell the compiler: wave-uniform
    pc.dt = __builtin_amdgcn_readfirstlane(info.first_seg);
    const int64_t toff = info.toff + (e0 % TILE);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)toff);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uint64_t)toff >> 32));
    pc.toff = (int64_t)(((uint64_t)hi << 32) | lo);
    return pc;
}

// 4 elements per thread out of one tensor's per-rank gradients.  ALIGNED: every rank's first byte
// for this block is 8-byte (2-byte dtypes) or 16-byte (fp32) aligned, so one vector load fetches
// the thread's 4 values; otherwise element loads.
template <int DT, bool ALIGNED>
struct Tensor4Loader {
    static constexpr bool kTensor = false;
    static constexpr int kElems = 4;
    static constexpr int kBatch = PARO_BATCH_BF16;
    using Raw = std::conditional_t<DT == PARO_F32, u32x4, u32x2>;
    int tensor;
    int64_t byte_off;          // of the thread's first element inside the tensor
    template <bool SLOW>
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t base = static_cast<const uintptr_t *>(src.p[k])[tensor] + (uintptr_t)byte_off;
        if constexpr (ALIGNED) {
            r = ld_contrib(global_ptr<Raw>(base));
        } else if constexpr (DT != PARO_F32) {
            const auto *h = global_ptr<uint16_t>(base);
            r.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
            r.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
        } else {
            const auto *w = global_ptr<unsigned int>(base);
            r = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
    template <bool SLOW>
    __device__ __forceinline__ void unpack(const SrcTable &s, int k, const Raw &r, float x[4]) const {
        Chunk4Loader<DT>{0}.template unpack<SLOW>(s, k, r, x);
    }
};

template <int DT>
__device__ __forceinline__ void fold_piece_dt(const Piece &pc, const SrcTable &src, int P, int group_len, float X[4]) {
    constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    constexpr uintptr_t NEED = DT == PARO_F32 ? 15 : 7;
    bool aligned = true;                                         // wave-uniform
    for (int k = 0; k < P; ++k) {
        const uintptr_t b = static_cast<const uintptr_t *>(src.p[k])[pc.tensor];
        aligned = aligned && ((b + (uintptr_t)pc.toff * ESIZE) & NEED) == 0;
    }
    const int64_t byte_off = (pc.toff + (int64_t)threadIdx.x * 4) * ESIZE;
    if (aligned) {
        Tensor4Loader<DT, true> ld{pc.tensor, byte_off};
        fold8<Tensor4Loader<DT, true>, false>(ld, src, P, group_len, X);
    } else {
        Tensor4Loader<DT, false> ld{pc.tensor, byte_off};
        fold8<Tensor4Loader<DT, false>, false>(ld, src, P, group_len, X);
    }
}

// The ordered fold for a block whose elements lie in one tensor (pc.tensor >= 0).
__device__ __forceinline__ void fold_piece(const Piece &pc, const SrcTable &src, int P, int group_len, float X[4]) {
    if (pc.dt == PARO_BF16) fold_piece_dt<PARO_BF16>(pc, src, P, group_len, X);
    else if (pc.dt == PARO_F16) fold_piece_dt<PARO_F16>(pc, src, P, group_len, X);
    else fold_piece_dt<PARO_F32>(pc, src, P, group_len, X);
}

// Sweep 1, tensor layout, tiles that lie in one tensor or in the padding.  Every block writes its
// partial sum (0 for a block that leaves its tile to the boundary-tile launch).
template <bool SUMSQ>
__global__ __launch_bounds__(64) void k_reduce4t(const SrcTable src, int P, int group_len, int64_t n,
                                                 float *__restrict__ g, double *__restrict__ partials,
                                                 const paro_tile_info *__restrict__ tile_tab) {
    const int64_t e0 = (int64_t)blockIdx.x * 256, e = e0 + (int64_t)threadIdx.x * 4;
    const Piece pc = piece_of(tile_tab, e0);
    double acc = 0.0;
    if (pc.tensor != -1 && e < n) {
        float X[4] = {0.0f, 0.0f, 0.0f, 0.0f};                   // padding: the sum of zeros
        if (pc.tensor >= 0) fold_piece(pc, src, P, group_len, X);
        st_as<PARO_NT_GSTORE != 0>(reinterpret_cast<f32x4 *>(g + e), f32x4{X[0], X[1], X[2], X[3]});
        if (SUMSQ) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc += (double)X[i] * (double)X[i];
        }
    }
    if (SUMSQ) {
        const double s = block_sum<64>(acc);
        if (threadIdx.x == 0) partials[blockIdx.x] = s;
    }
}

// Sweep 2 with a weight-decay mask, same tiles.
template <bool PACK>
__global__ __launch_bounds__(64) void k_adam4m(const AdamConsts a, const double *__restrict__ total_sumsq,
                                               const float *__restrict__ g, float *__restrict__ p,
                                               float *__restrict__ m, float *__restrict__ v,
                                               uint16_t *__restrict__ dst, int64_t n,
                                               const paro_tile_info *__restrict__ tile_tab,
                                               const uint8_t *__restrict__ no_decay) {
    if (a.skip_nonfinite && !isfinite(*total_sumsq)) return;
    const float sc = scale_from_norm(a, total_sumsq);
    const int64_t e0 = (int64_t)blockIdx.x * 256, e = e0 + (int64_t)threadIdx.x * 4;
    if (e >= n) return;
    const Piece pc = piece_of(tile_tab, e0);
    if (pc.tensor == -1) return;
    const bool decays = pc.tensor < 0 || no_decay[pc.tensor] == 0;      // padding decays (and stays 0)
    const f32x4 G = ld_as<ADAM4_LNT>(reinterpret_cast<const f32x4 *>(g + e));
    const State4 s = load_state4(p, m, v, e);
    const float gg[4] = {G.x, G.y, G.z, G.w};
    update4<PACK>(a, sc, decays, gg, s, p, m, v, dst, e);
}

// Single sweep (no clipping) for the tensor layout and / or a weight-decay mask, same tiles.
// TENSORS: contributions are per-tensor gradients; else arrays in shard coordinates of dtype DT.
template <bool TENSORS, int DT, bool MASK>
__global__ __launch_bounds__(64) void k_fused4t(const SrcTable src, int P, int group_len, int64_t n, const AdamConsts a,
                                                float *__restrict__ p, float *__restrict__ m, float *__restrict__ v,
                                                uint16_t *__restrict__ dst,
                                                const paro_tile_info *__restrict__ tile_tab,
                                                const uint8_t *__restrict__ no_decay) {
    const int64_t e0 = (int64_t)blockIdx.x * 256, e = e0 + (int64_t)threadIdx.x * 4;
    if (e >= n) return;
    const Piece pc = piece_of(tile_tab, e0);
    if (pc.tensor == -1) return;
    const bool decays = !MASK || pc.tensor < 0 || no_decay[pc.tensor] == 0;
    const State4 s = load_state4(p, m, v, e);
    float X[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (TENSORS) {
        if (pc.tensor >= 0) fold_piece(pc, src, P, group_len, X);
    } else {
        Chunk4Loader<DT> ld{e};
        fold8<Chunk4Loader<DT>, false>(ld, src, P, group_len, X);
    }
    update4<true>(a, a.grad_scale, decays, X, s, p, m, v, dst, e);
}

// Single sweep when nothing has to wait for the norm: fold, Adam and pack; the
// reduced gradient never goes to memory.
template <class Ld, bool MASK>
__global__ __launch_bounds__(TPB) void k_fused(Ld ld, const SrcTable src, int P, int group_len, int64_t n,
                                               const AdamConsts a, float *__restrict__ p, float *__restrict__ m,
                                               float *__restrict__ v, uint16_t *__restrict__ dst, TileSegs segs,
                                               const int32_t *__restrict__ tile_list, int n_list) {
    constexpr bool NEED_SEGS = Ld::kTensor || MASK;
    __shared__ int64_t s_off[NEED_SEGS ? TILE + 2 : 1];
    __shared__ int s_head[2];
    __shared__ uintptr_t s_ptr[Ld::kTensor ? PARO_MAX_RANKS : 1];
    segs.s_off = s_off;
    segs.s_head = s_head;
    const float sc = a.grad_scale;                     // no clipping on this path
    const int64_t ntiles = (n + TILE - 1) / TILE;
    TILE_LOOP(PARO_TPBK_FOLD, tile, ntiles, tile_list, n_list) {
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

// Low-precision pack alone: one-wave blocks, 4 elements per thread.
__global__ __launch_bounds__(64) void k_pack(const float *__restrict__ p, uint16_t *__restrict__ dst, int64_t n,
                                             int pack_dtype) {
    const int64_t e = ((int64_t)blockIdx.x * 64 + threadIdx.x) * 4;          // n is a multiple of 8
    if (e >= n) return;
    const f32x4 P = ld_as<true>(reinterpret_cast<const f32x4 *>(p + e));
    u32x2 w;
    if (pack_dtype == PARO_F16) {
        w.x = f32_to_f16_bits(P.x) | (f32_to_f16_bits(P.y) << 16);
        w.y = f32_to_f16_bits(P.z) | (f32_to_f16_bits(P.w) << 16);
    } else {
        w.x = f32_to_bf16_rne(P.x) | (f32_to_bf16_rne(P.y) << 16);
        w.y = f32_to_bf16_rne(P.z) | (f32_to_bf16_rne(P.w) << 16);
    }
    st_as<true>(reinterpret_cast<u32x2 *>(dst + e), w);
}

// One ring hop / one accumulation: out = a + b, element by element in fp32.  One-wave blocks,
// 4 elements per thread, streaming loads and stores.
template <int DT>
__device__ __forceinline__ void hop_load4(const void *a, int64_t e, float x[4]) {
    if (DT != PARO_F32) {
        const u32x2 q = ld_as<true>(reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(a) + e));
        x[0] = cvt_lo<DT>(q.x); x[1] = cvt_hi<DT>(q.x); x[2] = cvt_lo<DT>(q.y); x[3] = cvt_hi<DT>(q.y);
    } else {
        const f32x4 q = ld_as<true>(reinterpret_cast<const f32x4 *>(static_cast<const float *>(a) + e));
        x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
    }
}
template <int DT>
__device__ __forceinline__ float hop_load1(const void *a, int64_t i) {
    return DT != PARO_F32 ? cvt16(static_cast<const uint16_t *>(a)[i], DT) : static_cast<const float *>(a)[i];
}

template <int DA, int DB>
__global__ __launch_bounds__(64) void k_hop(const void *a, const void *b, float *out, int64_t n) {
    const int64_t e = ((int64_t)blockIdx.x * 64 + threadIdx.x) * 4;
    if (e + 4 <= n) {
        float x[4], y[4];
        hop_load4<DA>(a, e, x);
        hop_load4<DB>(b, e, y);
        st_as<true>(reinterpret_cast<f32x4 *>(out + e), f32x4{x[0] + y[0], x[1] + y[1], x[2] + y[2], x[3] + y[3]});
    } else {
        for (int64_t i = e; i < n; ++i) out[i] = hop_load1<DA>(a, i) + hop_load1<DB>(b, i);   // last, partial group
    }
}

// Plain copy of n 16-byte units (an all-gather message landing in the parameter buffer).
__global__ __launch_bounds__(64) void k_copy16(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (i < n) st_as<true>(dst + i, ld_as<true>(src + i));
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

// Blocks of the 4-elements-per-thread fold over n elements.
int fold4_grid(int64_t n) {
    const int64_t per_block = 4 * (int64_t)PARO_FOLD4_TPB;
    const int64_t nb = (n + per_block - 1) / per_block;
    return (int)(nb < 1 ? 1 : nb);
}

// Occupancy throttle for the one-wave-block sweeps: on this part the mixed read/write sweeps run
// faster with 12-14 waves per compute unit in flight than with the 32 the registers would allow
// (fewer requests fighting over DRAM pages).  The launch asks for dynamic LDS it never touches,
// sized so that only `waves_per_cu` blocks fit on a compute unit.
unsigned throttle_lds(const paro_plan_t *pl, int waves_per_cu) {
    if (waves_per_cu <= 0) return 0;
    unsigned bytes = (unsigned)(pl->dev.lds_per_cu / waves_per_cu) / 256u * 256u;
    return bytes > 65536u ? 65536u : bytes;
}

template <class T>
int upload(T **dst, const T *src, size_t n) {
    PARO_HIP(hipMalloc(reinterpret_cast<void **>(dst), (n ? n : 1) * sizeof(T)));
    if (n) PARO_HIP(hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice));
    return PARO_OK;
}

void free_tables(paro_device_tables &d) {
    // best effort: at process exit the runtime may already be gone
    (void)hipFree(d.nz_off);
    (void)hipFree(d.nz_tensor);
    (void)hipFree(d.dtype);
    (void)hipFree(d.no_decay);
    (void)hipFree(d.tile_tab);
    (void)hipFree(d.slow_tiles);
    (void)hipFree(d.partials);
    d = paro_device_tables();
}

int fill_tables(const paro_plan_t *pl, paro_device_tables &d) {
    int rc;
    if ((rc = upload(&d.nz_off, pl->nz_off.data(), pl->nz_off.size()))) return rc;
    if ((rc = upload(&d.nz_tensor, pl->nz_tensor.data(), pl->nz_tensor.size()))) return rc;
    if ((rc = upload(&d.dtype, pl->dtype.data(), pl->dtype.size()))) return rc;
    if ((rc = upload(&d.no_decay, pl->no_decay.data(), pl->no_decay.size()))) return rc;
    d.tiles_per_chunk = (pl->L + TILE - 1) / TILE;
    // one partial per block of the largest sweep-1 launch (a launch covers one chunk of L elements),
    // followed by room for the second-level sums
    // (the one-wave fold's blocks, then the blocks of a launch over the boundary tiles)
    int64_t n_part = fold4_grid(pl->L) + (pl->L + TILE - 1) / TILE;
    if (n_part < PARO_MAX_PARTIALS) n_part = PARO_MAX_PARTIALS;
    d.n_partials = n_part;
    const int64_t n_level2 = (n_part + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
    PARO_HIP(hipMalloc(reinterpret_cast<void **>(&d.partials), (n_part + n_level2) * sizeof(double)));
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
    PARO_HIP(hipDeviceGetAttribute(&d.lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev));
    if (d.lds_per_cu < 65536) d.lds_per_cu = 65536;
    const int rc = fill_tables(pl, d);
    if (rc != PARO_OK) {
        free_tables(d);                    // nothing half-built stays behind
        return rc;
    }
    d.device = dev;
    pl->dev = d;
    return PARO_OK;
}

// Builds, once, the per-tile table and the per-chunk lists of boundary tiles (for calls that work
// tensor by tensor: the tensor layout, a weight-decay mask).  Too large a table (more than 4 Mi
// tiles) is not built; the callers then use the kernels that search.
int ensure_tile_table(paro_plan_t *pl) {
    std::lock_guard<std::mutex> lock(pl->dev_mutex);
    paro_device_tables &d = pl->dev;
    if (d.tile_tab_tried) return PARO_OK;
    d.tile_tab_tried = true;
    if ((int64_t)pl->P * d.tiles_per_chunk > (int64_t)4 << 20) return PARO_OK;
    std::vector<paro_tile_info> tab;
    std::vector<int32_t> slow;
    try {
        tab.resize((size_t)pl->P * d.tiles_per_chunk);
        d.slow_start.assign((size_t)pl->P + 1, 0);
        const int64_t n_nz = (int64_t)pl->nz_tensor.size();
        for (int c = 0; c < pl->P; ++c) {
            d.slow_start[c] = (int64_t)slow.size();
            for (int64_t i = 0; i < d.tiles_per_chunk; ++i) {
                const int64_t f0 = (int64_t)c * pl->L + i * TILE;
                const int64_t f1 = std::min(f0 + (int64_t)TILE, (int64_t)(c + 1) * pl->L);   // end of the tile
                paro_tile_info &ti = tab[(size_t)c * d.tiles_per_chunk + i];
                ti.toff = 0;
                ti.tensor = -2;
                ti.first_seg = (int32_t)n_nz;
                if (f0 >= pl->total) continue;
                const int64_t k = std::upper_bound(pl->nz_off.begin(), pl->nz_off.end(), f0) - pl->nz_off.begin() - 1;
                if (f1 <= pl->nz_off[k + 1]) {
                    ti.tensor = pl->nz_tensor[k];
                    ti.toff = f0 - pl->nz_off[k];
                    ti.first_seg = pl->dtype[ti.tensor];
                } else {
                    ti.tensor = -1;
                    ti.first_seg = (int32_t)k;
                    slow.push_back((int32_t)i);
                }
            }
        }
        d.slow_start[pl->P] = (int64_t)slow.size();
    } catch (const std::bad_alloc &) {
        return fail(PARO_ENOMEM, "out of host memory while building the per-tile table");
    }
    int rc;
    if ((rc = upload(&d.slow_tiles, slow.data(), slow.size()))) return rc;
    if ((rc = upload(&d.tile_tab, tab.data(), tab.size()))) {
        (void)hipFree(d.slow_tiles);
        d.slow_tiles = nullptr;
        return rc;
    }
    return PARO_OK;
}

// Blocks of a launch over n_tiles tiles, for a kernel that takes tpbk tiles per block.
int grid_for_tiles(int64_t n_tiles, int tpbk) {
    const int64_t nb = (n_tiles + tpbk - 1) / tpbk;
    return (int)(nb < 1 ? 1 : nb);
}
int grid_for(int64_t n, int tpbk) { return grid_for_tiles((n + TILE - 1) / TILE, tpbk); }

// Chunk c's part of the per-tile table and of the list of boundary tiles (null / 0 without a table).
struct ChunkTiles {
    const paro_tile_info *tab = nullptr;
    const int32_t *slow = nullptr;
    int n_slow = 0;
};
ChunkTiles chunk_tiles(const paro_plan_t *pl, int64_t c) {
    ChunkTiles ct;
    if (!pl->dev.tile_tab) return ct;
    ct.tab = pl->dev.tile_tab + c * pl->dev.tiles_per_chunk;
    ct.slow = pl->dev.slow_tiles + pl->dev.slow_start[(size_t)c];
    ct.n_slow = (int)(pl->dev.slow_start[(size_t)c + 1] - pl->dev.slow_start[(size_t)c]);
    return ct;
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

#define PARO_BY_DTYPE(dt, CALL)            \
    do {                                   \
        if ((dt) == PARO_BF16) {           \
            constexpr int DT = PARO_BF16;  \
            CALL;                          \
        } else if ((dt) == PARO_F16) {     \
            constexpr int DT = PARO_F16;   \
            CALL;                          \
        } else {                           \
            constexpr int DT = PARO_F32;   \
            CALL;                          \
        }                                  \
    } while (0)

// Launches sweep 1 over chunk c; returns the number of per-block partial sums it writes.
template <bool SUMSQ>
int launch_reduce(const paro_plan_t *pl, int layout, const SrcTable &tab, int group_len, int64_t c, float *g,
                  hipStream_t st) {
    const int64_t n = pl->L;
    double *partials = pl->dev.partials;
    const int g4 = fold4_grid(n);
    const unsigned lds = throttle_lds(pl, PARO_FOLD4_WAVES_PER_CU);
    if (layout == PARO_CHUNK) {
        PARO_BY_DTYPE(pl->dtype[0], hipLaunchKernelGGL((k_reduce4<DT, SUMSQ>), dim3(g4), dim3(PARO_FOLD4_TPB), lds, st, tab,
                                                       pl->P, group_len, n, g, partials));
        return g4;
    }
    TensorLoader ld;
    ld.dtype = pl->dev.dtype;
    TileSegs segs = segs_for(pl, c * pl->L, true);
    const ChunkTiles ct = chunk_tiles(pl, c);
    if (!ct.tab) {                        // no per-tile table: the searching kernel over every tile
        const int grid = grid_for(n, PARO_TPBK_FOLD);
        hipLaunchKernelGGL((k_reduce<TensorLoader, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, g,
                           partials, segs, nullptr, 0);
        return grid;
    }
    hipLaunchKernelGGL((k_reduce4t<SUMSQ>), dim3(g4), dim3(64), lds, st, tab, pl->P, group_len, n, g, partials, ct.tab);
    if (ct.n_slow == 0) return g4;
    const int grid = grid_for_tiles(ct.n_slow, PARO_TPBK_FOLD);
    hipLaunchKernelGGL((k_reduce<TensorLoader, SUMSQ>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, g,
                       partials + g4, segs, ct.slow, ct.n_slow);
    return g4 + grid;
}

// Launches the single sweep (no clipping) over chunk c.
template <bool MASK>
void launch_fused(const paro_plan_t *pl, int layout, const SrcTable &tab, int group_len, int64_t c, const AdamConsts &a,
                  float *p, float *m, float *v, uint16_t *dst, hipStream_t st) {
    const int64_t n = pl->L;
    const int g4 = fold4_grid(n);
    const unsigned lds = throttle_lds(pl, PARO_FUSED4_WAVES_PER_CU);
    if (layout == PARO_CHUNK && !MASK) {
        PARO_BY_DTYPE(pl->dtype[0], hipLaunchKernelGGL((k_fused4<DT>), dim3(g4), dim3(PARO_FOLD4_TPB), lds, st, tab, pl->P,
                                                       group_len, n, a, p, m, v, dst));
        return;
    }
    TileSegs segs = segs_for(pl, c * pl->L, true);
    const ChunkTiles ct = chunk_tiles(pl, c);
    // the tile-at-a-time kernel: over every tile without a table, else over the boundary tiles
    const int n_list = ct.tab ? ct.n_slow : 0;
    const int grid = ct.tab ? grid_for_tiles(ct.n_slow, PARO_TPBK_FOLD) : grid_for(n, PARO_TPBK_FOLD);
    const uint8_t *no_decay = pl->dev.no_decay;
    if (layout == PARO_TENSORS) {
        if (ct.tab)
            hipLaunchKernelGGL((k_fused4t<true, PARO_BF16, MASK>), dim3(g4), dim3(64), lds, st, tab, pl->P, group_len, n, a, p,
                               m, v, dst, ct.tab, no_decay);
        if (ct.tab && n_list == 0) return;
        TensorLoader ld;
        ld.dtype = pl->dev.dtype;
        hipLaunchKernelGGL((k_fused<TensorLoader, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, a,
                           p, m, v, dst, segs, ct.slow, n_list);
        return;
    }
    if (ct.tab)
        PARO_BY_DTYPE(pl->dtype[0], hipLaunchKernelGGL((k_fused4t<false, DT, MASK>), dim3(g4), dim3(64), lds, st, tab, pl->P,
                                                       group_len, n, a, p, m, v, dst, ct.tab, no_decay));
    if (ct.tab && n_list == 0) return;
    PARO_BY_DTYPE(pl->dtype[0], {
        ChunkLoader<DT> ld{0};
        hipLaunchKernelGGL((k_fused<ChunkLoader<DT>, MASK>), dim3(grid), dim3(TPB), 0, st, ld, tab, pl->P, group_len, n, a, p,
                           m, v, dst, segs, ct.slow, n_list);
    });
}

// Sweep 1 over the whole update range, chunk by chunk; the sum of squares covers
// the rank's own chunk only.
int do_reduce(paro_plan_t *pl, int rank, const void *const *contrib, int layout, float *grad_out, double *sumsq_out,
              hipStream_t st) {
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    const int own = paro::chunk_of_rank(pl, rank);
    int n_part = 0;                      // partial sums written by the launches over the rank's own chunk
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {
        SrcTable tab;
        int gl;
        const int64_t lo = c * pl->L - ob;
        src_table(pl, (int)c, contrib, layout, lo, &tab, &gl);
        if (c == own && sumsq_out)
            n_part = launch_reduce<true>(pl, layout, tab, gl, c, grad_out + lo, st);
        else
            launch_reduce<false>(pl, layout, tab, gl, c, grad_out + lo, st);
        PARO_HIP(hipGetLastError());
    }
    if (sumsq_out) {
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

template <bool PACK>
int launch_adam(paro_plan_t *pl, int rank, const AdamConsts &a, const float *grad, const double *total_sumsq, float *p,
                float *m, float *v, uint16_t *dst, hipStream_t st) {
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    const unsigned lds = throttle_lds(pl, PARO_ADAM4_WAVES_PER_CU);
    if (!pl->any_no_decay) {
        const int64_t nb = (on / 4 + PARO_ADAM4_TPB - 1) / PARO_ADAM4_TPB;
        hipLaunchKernelGGL((k_adam4<PACK>), dim3((unsigned)nb), dim3(PARO_ADAM4_TPB), lds, st, a, total_sumsq, grad, p, m, v,
                           dst, on);
        PARO_HIP(hipGetLastError());
        return PARO_OK;
    }
    if (!pl->dev.tile_tab) {              // no per-tile table: the searching kernel over the whole range
        hipLaunchKernelGGL((k_adam<PACK, true>), dim3(grid_for(on, PARO_TPBK_ADAM)), dim3(TPB), 0, st, a, total_sumsq, grad,
                           p, m, v, dst, on, segs_for(pl, ob, false), nullptr, 0);
        PARO_HIP(hipGetLastError());
        return PARO_OK;
    }
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {      // the table is laid out chunk by chunk
        const int64_t lo = c * pl->L - ob;
        const ChunkTiles ct = chunk_tiles(pl, c);
        uint16_t *d = dst ? dst + lo : nullptr;
        hipLaunchKernelGGL((k_adam4m<PACK>), dim3(fold4_grid(pl->L)), dim3(64), lds, st, a, total_sumsq, grad + lo, p + lo,
                           m + lo, v + lo, d, pl->L, ct.tab, pl->dev.no_decay);
        PARO_HIP(hipGetLastError());
        if (ct.n_slow == 0) continue;
        hipLaunchKernelGGL((k_adam<PACK, true>), dim3(grid_for_tiles(ct.n_slow, PARO_TPBK_ADAM)), dim3(TPB), 0, st, a,
                           total_sumsq, grad + lo, p + lo, m + lo, v + lo, d, pl->L, segs_for(pl, c * pl->L, true), ct.slow,
                           ct.n_slow);
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

int do_adam(paro_plan_t *pl, int rank, const AdamConsts &a, const float *grad, const double *total_sumsq, float *p,
            float *m, float *v, uint16_t *dst /* nullable: no pack */, hipStream_t st) {
    return dst ? launch_adam<true>(pl, rank, a, grad, total_sumsq, p, m, v, dst, st)
               : launch_adam<false>(pl, rank, a, grad, total_sumsq, p, m, v, dst, st);
}

}  // namespace

extern "C" {

void paro_plan_destroy(paro_plan_t *pl) {
    if (!pl) return;
    if (pl->dev.device >= 0) free_tables(pl->dev);
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
    if (layout == PARO_TENSORS && (rc = ensure_tile_table(pl))) return rc;
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
    if (pl->any_no_decay && (rc = ensure_tile_table(pl))) return rc;
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
    const int64_t nb = (sl / 4 + 63) / 64;
    hipLaunchKernelGGL(k_pack, dim3((unsigned)(nb < 1 ? 1 : nb)), dim3(64), throttle_lds(pl, PARO_COPY_WAVES_PER_CU),
                       static_cast<hipStream_t>(stream), p, dst_base + so, sl, pl->pack_dtype);
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
    if ((layout == PARO_TENSORS || pl->any_no_decay) && (rc = ensure_tile_table(pl))) return rc;
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
            launch_fused<true>(pl, layout, tab, gl, c, a, p + lo, m + lo, v + lo, dst + lo, st);
        else
            launch_fused<false>(pl, layout, tab, gl, c, a, p + lo, m + lo, v + lo, dst + lo, st);
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

}  // extern "C"


// ---- ring hops and scheduled transfers ----------------------------------------
namespace {
int launch_hop(const paro_plan_t *pl, const void *a, int da, const void *b, int db, float *out, int64_t n,
               hipStream_t st) {
    if (n <= 0) return PARO_OK;
    const int64_t groups = (n + 3) / 4;
    const unsigned grid = (unsigned)((groups + 63) / 64);
    const unsigned lds = throttle_lds(pl, PARO_HOP_WAVES_PER_CU);
#define PARO_HOP_CASE(A, B)                                                                                   \
    if (da == A && db == B) hipLaunchKernelGGL((k_hop<A, B>), dim3(grid), dim3(64), lds, st, a, b, out, n)
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
    return launch_hop(pl, partial_in, in_dtype, local, local_dtype, out, n, static_cast<hipStream_t>(stream));
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
    std::vector<paro_msg_t> msgs;
    try {
        msgs.resize((size_t)count);
    } catch (const std::bad_alloc &) {
        return fail(PARO_ENOMEM, "paro_collective_step: out of host memory");
    }
    if (count && paro_schedule(pl, rank, sched, collective, msgs.data(), count) < 0) return PARO_EINVAL;
    if ((rc = ensure_device(pl))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t received = 0;
    for (const paro_msg_t &m : msgs) {
        if (m.phase != phase || m.ring != ring || m.step != step) continue;
        if (collective == PARO_RS) {
            const float *from = static_cast<const float *>(bufs[m.recv_from]) + m.recv_off;
            float *mine = static_cast<float *>(bufs[rank]) + m.recv_off;
            if ((rc = launch_hop(pl, from, PARO_F32, mine, PARO_F32, mine, m.recv_len, st))) return rc;
        } else {
            const uint16_t *from = static_cast<const uint16_t *>(bufs[m.recv_from]) + m.recv_off;
            uint16_t *mine = static_cast<uint16_t *>(bufs[rank]) + m.recv_off;
            const int64_t n16 = m.recv_len / 8;             // ranges are whole chunks: multiples of 8 elements
            const unsigned grid = (unsigned)((n16 + 63) / 64);
            if (n16 > 0) {
                hipLaunchKernelGGL(k_copy16, dim3(grid), dim3(64), throttle_lds(pl, PARO_COPY_WAVES_PER_CU), st,
                                   reinterpret_cast<const u32x4 *>(from), reinterpret_cast<u32x4 *>(mine), n16);
                PARO_HIP(hipGetLastError());
            }
        }
        received += m.recv_len;
    }
    return received;
}

}  // extern "C"
