// Device side of libparo for gfx950 (MI355X): the streaming kernels of the
// Update stage (paper Sec. 3.2) and the entry points that launch them.
//
// Everything here is bound by HBM bandwidth: per shard parameter the method
// moves 2P bytes of bf16 contributions and 26-34 bytes of fp32 state, against
// P adds and ~20 flops.  So the kernels are plain sweeps with many independent
// loads in flight per thread; there is no dense contraction and hence no MFMA.
//
//   shape     every sweep runs in one-wave blocks (64 threads) of 256 consecutive
//             elements, 4 per thread: each load or store instruction of a wave
//             covers 512 B - 1 KB of consecutive addresses (whole cache lines), and
//             the many short-lived waves, dealt round-robin to the 8 XCDs in
//             address order, interleave reads and writes finely.  On MI355X this
//             beat 256-thread blocks of 8-element threads by 8-11 %, and those had
//             beaten persistent grid-stride blocks by 8-15 %.
//   occupancy the heavy sweeps ask for unused dynamic LDS so that only 10-14 waves
//             run per compute unit: fewer requests outstanding fight less over
//             DRAM pages (another 3-6 %).  The tensor layout over many small
//             tensors wants the opposite - its waves wait on look-ups with no
//             data in flight - and gets two blocks per wave (few contributions)
//             or every wave the registers allow.
//   caches    everything is touched once: streaming (non-temporal) loads; stores
//             through per-wave buffer descriptors, which let the instruction say
//             "streaming, system scope" (nt sc1: 2 % better than nt alone).
//   fold      the P contributions of an element are added in a fixed order
//             (never re-associated, never contracted into FMAs) so the result
//             is bit-identical to a reduce-scatter ring run in that order
//   norm      squares are exact in fp64; per-thread fp64 sums -> wave shuffles
//             -> one partial per block -> a small kernel adds the partials in a
//             fixed order, in two levels.  No atomics: run-to-run identical.
//   tensors   the tensor layout and the weight-decay mask need the tensor an
//             element belongs to: a per-block table (built once per chunk) answers
//             with a single look-up; a block with a tensor boundary inside finds
//             its elements' tensors with one load per lane and a search across
//             the lanes' registers.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <new>
#include <cstdlib>
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

struct State4 { u32x4 p, m, v; };

// elements of the block at e0 that lie inside a launch of n elements
__device__ __forceinline__ unsigned piece_elems(int64_t e0, int64_t n) {
    return (unsigned)min((int64_t)PIECE, n - e0);
}

__device__ __forceinline__ State4 load_state4(const float *p, const float *m, const float *v, int64_t e) {
    State4 s;
    s.p = ld_nt(reinterpret_cast<const u32x4 *>(p + e));
    s.m = ld_nt(reinterpret_cast<const u32x4 *>(m + e));
    s.v = ld_nt(reinterpret_cast<const u32x4 *>(v + e));
    return s;
}

// Adam on the thread's 4 elements; state and (optionally) the low-precision copy written back.
template <bool PACK>
__device__ __forceinline__ void update4(const AdamConsts &a, float sc, const bool decays[4], const float gg[4],
                                        const State4 &s, float *p, float *m, float *v, uint16_t *dst, int64_t e0,
                                        unsigned elems) {
    float pp[4] = {__uint_as_float(s.p.x), __uint_as_float(s.p.y), __uint_as_float(s.p.z), __uint_as_float(s.p.w)},
          mm[4] = {__uint_as_float(s.m.x), __uint_as_float(s.m.y), __uint_as_float(s.m.z), __uint_as_float(s.m.w)},
          vv[4] = {__uint_as_float(s.v.x), __uint_as_float(s.v.y), __uint_as_float(s.v.z), __uint_as_float(s.v.w)};
#pragma unroll
    for (int i = 0; i < 4; ++i) adam1(a, sc, decays[i], gg[i], pp[i], mm[i], vv[i]);
    constexpr int ST = PARO_POL_STATE_ST;
    buf_store16<ST>(as_u32x4(pp[0], pp[1], pp[2], pp[3]), wave_buffer(p + e0, elems * 4), lane_id() * 16);
    buf_store16<ST>(as_u32x4(mm[0], mm[1], mm[2], mm[3]), wave_buffer(m + e0, elems * 4), lane_id() * 16);
    buf_store16<ST>(as_u32x4(vv[0], vv[1], vv[2], vv[3]), wave_buffer(v + e0, elems * 4), lane_id() * 16);
    if (PACK) {
        const u32x2 w = {pack2_lowp(pp[0], pp[1], a.pack_dtype), pack2_lowp(pp[2], pp[3], a.pack_dtype)};
        buf_store8<ST>(w, wave_buffer(dst + e0, elems * 2), lane_id() * 8);
    }
}

// Which of the thread's 4 elements take weight decay (padding does, and stays 0).  loc: from
// locate4 when the block holds a boundary.
__device__ __forceinline__ void decay_flags(const TensorMap &tm, const Piece &pc, const Located &loc, bool decays[4]) {
    if (pc.tensor != -1) {
        const bool d = pc.tensor < 0 || tm.no_decay[pc.tensor] == 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) decays[i] = d;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) decays[i] = loc.tens[i] < 0 || tm.no_decay[loc.tens[i]] == 0;
    }
}

// The thread's first element; n (the launch's length) is a multiple of 8, so a thread's 4
// elements are all inside the range or all outside.
__device__ __forceinline__ int64_t block_first() { return (int64_t)blockIdx.x * PIECE; }

// Where a block of sweep 1 puts its partial sum.  Blocks are dealt round-robin to the 8 XCDs, each
// with an L2 of its own: giving every XCD its own run of slots lets each L2 collect whole lines of
// partials before writing them back (slot = blockIdx would make every line a patchwork of 8-byte
// writes from 8 caches).  The grid of such a launch is a multiple of 8.
__device__ __forceinline__ unsigned partial_slot() { return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3); }

__device__ __forceinline__ double sumsq4(const float X[4]) {
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc += (double)X[i] * (double)X[i];
    return acc;
}

// --------------------------------------------------------------------- kernels

__device__ __forceinline__ void store_g4(float *g, int64_t e0, unsigned elems, const float X[4]) {
    buf_store16<PARO_POL_G_ST>(as_u32x4(X[0], X[1], X[2], X[3]), wave_buffer(g + e0, elems * 4), lane_id() * 16);
}

// Sweep 1, chunk layout: g = fold of the contributions; optional per-block partial of sum g^2.
template <int DT, bool SUMSQ>
__global__ __launch_bounds__(WAVE) void k_reduce4(const SrcTable src, int P, int group_len, int64_t n,
                                                  float *__restrict__ g, double *__restrict__ partials) {
    const int64_t e0 = block_first(), e = e0 + lane_id() * EPT;
    double acc = 0.0;
    if (e < n) {
        const unsigned elems = piece_elems(e0, n);
        Chunk4Loader<DT> ld{e};
        float X[4];
        fold4(ld, src, P, group_len, X);
        store_g4(g, e0, elems, X);
        if (SUMSQ) acc = sumsq4(X);
    }
    if (SUMSQ) {
        const double s = wave_sum(acc);
        if (lane_id() == 0) partials[partial_slot()] = s;
    }
}

// Sweep 1, tensor layout: one block of 256 elements starting at e0 < n.  Every lane of the wave takes part.
template <bool SUMSQ, int KB>
__device__ __forceinline__ void reduce_piece_t(const TensorMap &tm, const Piece &pc, const SrcTable &src, int P,
                                               int group_len, int64_t n, int64_t e0, float *g, double &acc) {
    const int64_t e = e0 + lane_id() * EPT;
    Located loc;
    if (pc.tensor == -1) locate4(tm, pc.seg, tm.begin + e0, lane_id() * EPT, loc);     // the whole wave
    if (e < n) {
        const unsigned elems = piece_elems(e0, n);
        float X[4] = {0.0f, 0.0f, 0.0f, 0.0f};           // padding: the sum of zeros
        if (pc.tensor != -2) fold_tensors<KB>(pc, loc, src, P, group_len, X);
        store_g4(g, e0, elems, X);
        if (SUMSQ) acc += sumsq4(X);
    }
}

// A wave takes PPW consecutive blocks.  PPW = 2 is for few contributions (P <= 8) over many small tensors: where both
// blocks lie inside one tensor - the usual case - the wave folds them as one stream of 512
// elements per contribution: one look-up and twice the bytes in flight per wave; the cache line
// that the two blocks share (a block does not start on a line inside its tensor) is fetched once.
// KB: contributions loaded before the first is consumed (8 when launched for P <= 8 only: fewer
// registers, more waves).
template <bool SUMSQ, int PPW, int KB>
__global__ __launch_bounds__(WAVE) void k_reduce4t(const SrcTable src, int P, int group_len, int64_t n,
                                                   float *__restrict__ g, double *__restrict__ partials,
                                                   const TensorMap tm) {
    const int64_t e0 = (int64_t)blockIdx.x * (PPW * PIECE);
    double acc = 0.0;
    if (e0 < n) {                                            // wave-uniform
        bool done = false;
        if constexpr (PPW == 2) {
            if (e0 + 2 * PIECE <= n) {                       // two whole blocks
                const Piece pa = piece_of(tm, e0, n), pb = piece_of(tm, e0 + PIECE, n);
                if (pa.tensor >= 0 && pb.tensor == pa.tensor) {                         // ... inside one tensor
                    float X[8];
                    fold_tensor_pair(pa, src, P, group_len, X);
                    const wave_buf out = wave_buffer(g + e0, 2 * PIECE * 4);
                    buf_store16<PARO_POL_G_ST>(as_u32x4(X[0], X[1], X[2], X[3]), out, lane_id() * 16);
                    buf_store16<PARO_POL_G_ST>(as_u32x4(X[4], X[5], X[6], X[7]), out, PIECE * 4 + lane_id() * 16);
                    if (SUMSQ) acc = sumsq4(X) + sumsq4(X + 4);
                    done = true;
                }
            }
        }
        if (!done) {                                         // block by block (one copy of the code: no unrolling)
#pragma unroll 1
            for (int j = 0; j < PPW; ++j) {
                const int64_t ej = e0 + (int64_t)j * PIECE;
                if (ej < n)
                    reduce_piece_t<SUMSQ, KB>(tm, piece_of(tm, ej, n), src, P, group_len, n, ej, g, acc);
            }
        }
    }
    if (SUMSQ) {
        const double s = wave_sum(acc);
        if (lane_id() == 0) partials[partial_slot()] = s;
    }
}

// Adds partials in a fixed order: block b takes the slice [b*chunk, b*chunk + chunk) of the n
// values; thread t adds its slice's elements t, t+T, t+2T, ... (eight loads in flight at a time,
// added in index order); then the fixed block tree.  Launched as many-blocks -> one block.
__global__ __launch_bounds__(FINALIZE_TPB) void k_finalize(const double *__restrict__ partials, int n, int chunk,
                                                           double *out) {
    const int lo = blockIdx.x * chunk, hi = min(n, lo + chunk);
    double acc = 0.0;
    for (int k0 = lo + threadIdx.x; k0 < hi; k0 += 8 * FINALIZE_TPB) {
        double x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = (k0 + u * FINALIZE_TPB < hi) ? partials[k0 + u * FINALIZE_TPB] : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    const double s = block_sum(acc);
    if (threadIdx.x == 0) out[blockIdx.x] = s;
}

// Sweep 2: Adam on the stored gradient, optionally packing the low-precision parameters.
// MASK: some tensors are exempt from weight decay.
template <bool PACK, bool MASK>
__global__ __launch_bounds__(WAVE) void k_adam4(const AdamConsts a, const double *__restrict__ total_sumsq,
                                                const float *__restrict__ g, float *__restrict__ p,
                                                float *__restrict__ m, float *__restrict__ v,
                                                uint16_t *__restrict__ dst, int64_t n, const TensorMap tm) {
    // an overflowed (non-finite) gradient makes its sum of squares non-finite: the whole step is skipped
    if (a.skip_nonfinite && !isfinite(*total_sumsq)) return;
    const float sc = scale_from_norm(a, total_sumsq);
    const int64_t e0 = block_first(), e = e0 + lane_id() * EPT;
    if (e0 >= n) return;
    bool decays[4] = {true, true, true, true};
    Piece pc;
    Located loc;
    if (MASK) {
        pc = piece_of(tm, e0, n);
        if (pc.tensor == -1) locate4(tm, pc.seg, tm.begin + e0, lane_id() * EPT, loc);     // the whole wave
    }
    if (e >= n) return;
    const unsigned elems = piece_elems(e0, n);
    const u32x4 G = ld_nt(reinterpret_cast<const u32x4 *>(g + e));
    const State4 s = load_state4(p, m, v, e);
    if (MASK) decay_flags(tm, pc, loc, decays);
    const float gg[4] = {__uint_as_float(G.x), __uint_as_float(G.y), __uint_as_float(G.z), __uint_as_float(G.w)};
    update4<PACK>(a, sc, decays, gg, s, p, m, v, dst, e0, elems);
}

// Single sweep when nothing has to wait for the norm (no clipping): fold, Adam and pack; the
// reduced gradient never goes to memory.  TENSORS: contributions are per-tensor gradients; else
// arrays in shard coordinates of dtype DT.
template <bool TENSORS, int DT, bool MASK>
__global__ __launch_bounds__(WAVE) void k_fused4(const SrcTable src, int P, int group_len, int64_t n,
                                                 const AdamConsts a, float *__restrict__ p, float *__restrict__ m,
                                                 float *__restrict__ v, uint16_t *__restrict__ dst,
                                                 const TensorMap tm) {
    const int64_t e0 = block_first(), e = e0 + lane_id() * EPT;
    if (e0 >= n) return;
    Piece pc;
    Located loc;
    if (TENSORS || MASK) {
        pc = piece_of(tm, e0, n);
        if (pc.tensor == -1) locate4(tm, pc.seg, tm.begin + e0, lane_id() * EPT, loc);     // the whole wave
    }
    if (e >= n) return;
    const unsigned elems = piece_elems(e0, n);
    const State4 s = load_state4(p, m, v, e);
    float X[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (TENSORS) {
        if (pc.tensor != -2) fold_tensors(pc, loc, src, P, group_len, X);
    } else {
        Chunk4Loader<DT> ld{e};
        fold4(ld, src, P, group_len, X);
    }
    bool decays[4] = {true, true, true, true};
    if (MASK) decay_flags(tm, pc, loc, decays);
    update4<true>(a, a.grad_scale, decays, X, s, p, m, v, dst, e0, elems);
}

// Low-precision pack alone.
__global__ __launch_bounds__(WAVE) void k_pack(const float *__restrict__ p, uint16_t *__restrict__ dst, int64_t n,
                                               int pack_dtype) {
    const int64_t e0 = block_first(), e = e0 + lane_id() * EPT;
    if (e >= n) return;
    const unsigned elems = piece_elems(e0, n);
    const u32x4 P = ld_nt(reinterpret_cast<const u32x4 *>(p + e));
    const u32x2 w = {pack2_lowp(__uint_as_float(P.x), __uint_as_float(P.y), pack_dtype),
                     pack2_lowp(__uint_as_float(P.z), __uint_as_float(P.w), pack_dtype)};
    buf_store8<PARO_POL_LIGHT_ST>(w, wave_buffer(dst + e0, elems * 2), lane_id() * 8);
}

// One ring hop / one accumulation: out = a + b, element by element in fp32.  n may be any
// length: the descriptors cover the block's whole groups of 4 elements, the thread that holds
// the last, partial group takes it element by element.
template <int DT>
__device__ __forceinline__ void hop_load4(const void *a, int64_t e, float x[4]) {
    constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    using Raw = typename Chunk4Loader<DT>::Raw;
    Chunk4Loader<DT>::to_f32(ld_nt(reinterpret_cast<const Raw *>(static_cast<const char *>(a) + e * ESIZE)), x);
}
template <int DT>
__device__ __forceinline__ float hop_load1(const void *a, int64_t i) {
    return DT != PARO_F32 ? cvt16(static_cast<const uint16_t *>(a)[i], DT) : static_cast<const float *>(a)[i];
}

template <int DA, int DB>
__global__ __launch_bounds__(WAVE) void k_hop(const void *a, const void *b, float *out, int64_t n) {
    const int64_t e0 = block_first(), e = e0 + lane_id() * EPT;
    const unsigned whole = piece_elems(e0, n) & ~3u;       // elements of the block in whole groups of 4
    if (e + EPT <= n) {
        float x[4], y[4];
        hop_load4<DA>(a, e, x);
        hop_load4<DB>(b, e, y);
        buf_store16<PARO_POL_LIGHT_ST>(as_u32x4(x[0] + y[0], x[1] + y[1], x[2] + y[2], x[3] + y[3]),
                                       wave_buffer(out + e0, whole * 4), lane_id() * 16);
    } else {
        for (int64_t i = e; i < n; ++i) out[i] = hop_load1<DA>(a, i) + hop_load1<DB>(b, i);
    }
}

// Plain copy of n 16-byte units (an all-gather message landing in the parameter buffer).
__global__ __launch_bounds__(WAVE) void k_copy16(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n) {
    const int64_t i0 = (int64_t)blockIdx.x * WAVE;
    if (i0 + threadIdx.x >= n) return;
    const unsigned bytes = (unsigned)min((int64_t)WAVE, n - i0) * 16;
    const u32x4 v = ld_nt(src + i0 + threadIdx.x);
    buf_store16<PARO_POL_LIGHT_ST>(v, wave_buffer(dst + i0, bytes), lane_id() * 16);
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

// One-wave blocks of a sweep over n elements, ppw pieces per wave.
unsigned piece_grid(int64_t n, int ppw = 1) {
    const int64_t nb = (n + (int64_t)PIECE * ppw - 1) / ((int64_t)PIECE * ppw);
    return (unsigned)(nb < 1 ? 1 : nb);
}

// Occupancy throttle for the one-wave-block sweeps: on this part the mixed read/write sweeps run
// faster with 10-14 waves per compute unit in flight than with the 32 the registers would allow
// (fewer requests fighting over DRAM pages).  The launch asks for dynamic LDS it never touches,
// sized so that only `waves_per_cu` blocks fit on a compute unit.
unsigned throttle_lds(int lds_per_cu, int waves_per_cu) {
    if (waves_per_cu <= 0) return 0;
    unsigned bytes = (unsigned)(lds_per_cu / waves_per_cu) / 256u * 256u;
    return bytes > 65536u ? 65536u : bytes;
}

// Waves per compute unit that keep about `loads_per_cu` loads in flight when a wave issues
// `per_wave` loads at a time; 0 (no limit) when that is all that fit anyway.
int fold_waves(int per_wave, int loads_per_cu) {
    const int waves = loads_per_cu / per_wave;
    return waves >= 32 ? 0 : std::max(waves, PARO_MIN_WAVES_PER_CU);
}
// Loads a wave of the fold has in flight: a batch of contributions, for each block it takes.
int fold_loads(int P, int blocks_per_wave = 1) { return std::min(P, PARO_BATCH) * blocks_per_wave; }

// What a launch needs from the device besides the caller's buffers: the LDS size behind the
// occupancy throttle and the scratch array of partial sums (per-block sums of a sweep-1 launch,
// then `level2`, the second-level sums).  Either the plan's own allocation or the library's
// static array.
struct Scratch {
    int lds_per_cu;
    double *partials;
    double *level2;
    double *chunk_sums;    // [PARO_MAX_RANKS] one sum per chunk of an update range of several chunks
    bool plan_tables;      // the plan's device tables (offset tables, per-tile tables) exist
};

Scratch plan_scratch(const paro_plan_t *pl) {
    double *level2 = pl->dev.partials + pl->dev.n_partials;
    const int64_t n_level2 = (pl->dev.n_partials + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
    return Scratch{pl->dev.lds_per_cu, pl->dev.partials, level2, level2 + n_level2, true};
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
    (void)hipFree(d.nz_dtype);
    (void)hipFree(d.dtype);
    (void)hipFree(d.no_decay);
    for (paro_tile_info *t : d.tile_tab) (void)hipFree(t);
    (void)hipFree(d.partials);
    d = paro_device_tables();
}

int fill_tables(const paro_plan_t *pl, paro_device_tables &d) {
    int rc;
    if ((rc = upload(&d.nz_off, pl->nz_off.data(), pl->nz_off.size()))) return rc;
    if ((rc = upload(&d.nz_tensor, pl->nz_tensor.data(), pl->nz_tensor.size()))) return rc;
    std::vector<uint8_t> nz_dtype(pl->nz_tensor.size());
    for (size_t k = 0; k < nz_dtype.size(); ++k) nz_dtype[k] = pl->dtype[(size_t)pl->nz_tensor[k]];
    if ((rc = upload(&d.nz_dtype, nz_dtype.data(), nz_dtype.size()))) return rc;
    if ((rc = upload(&d.dtype, pl->dtype.data(), pl->dtype.size()))) return rc;
    if ((rc = upload(&d.no_decay, pl->no_decay.data(), pl->no_decay.size()))) return rc;
    d.tiles_per_chunk = (pl->L + TILE - 1) / TILE;
    d.tile_tab.assign((size_t)pl->P, nullptr);
    d.tile_tab_tried.assign((size_t)pl->P, 0);
    // one partial per block of a sweep-1 launch (a launch covers one chunk of L elements),
    // followed by room for the second-level sums
    int64_t n_part = ((int64_t)piece_grid(pl->L) + 7) & ~(int64_t)7;
    if (n_part < PARO_MIN_PARTIALS) n_part = PARO_MIN_PARTIALS;
    d.n_partials = n_part;
    const int64_t n_level2 = (n_part + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
    PARO_HIP(hipMalloc(reinterpret_cast<void **>(&d.partials), (n_part + n_level2 + PARO_MAX_RANKS) * sizeof(double)));
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
    // LDS per compute unit, for the occupancy throttle; 160 KB on gfx950 if the runtime does not say
    if (hipDeviceGetAttribute(&d.lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess ||
        d.lds_per_cu < 65536) {
        (void)hipGetLastError();
        d.lds_per_cu = 160 * 1024;
    }
    const int rc = fill_tables(pl, d);
    if (rc != PARO_OK) {
        free_tables(d);                    // nothing half-built stays behind
        return rc;
    }
    d.device = dev;
    pl->dev = d;
    return PARO_OK;
}

// Builds, once per chunk, the per-tile tables of the chunks of a rank's update range (for calls
// that work tensor by tensor: the tensor layout, a weight-decay mask).  Too large a table (more
// than 4 Mi tiles per chunk, or what the environment variable PARO_TILE_TABLE_MAX_TILES says) is
// not built; the kernels then search the offset table for every block.
int ensure_tile_tables(paro_plan_t *pl, int rank) {
    std::lock_guard<std::mutex> lock(pl->dev_mutex);
    paro_device_tables &d = pl->dev;
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    int64_t max_tiles = (int64_t)4 << 20;                   // 64 MB of table
    if (const char *env = std::getenv("PARO_TILE_TABLE_MAX_TILES")) max_tiles = std::atoll(env);
    const int64_t n_nz = (int64_t)pl->nz_tensor.size();
    std::vector<paro_tile_info> tab;
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {
        if (d.tile_tab_tried[(size_t)c]) continue;
        if (d.tiles_per_chunk > max_tiles) {
            d.tile_tab_tried[(size_t)c] = 1;         // decided: this chunk works without a table
            continue;
        }
        try {
            tab.resize((size_t)d.tiles_per_chunk);
        } catch (const std::bad_alloc &) {
            return fail(PARO_ENOMEM, "out of host memory while building the per-tile table");
        }
        for (int64_t i = 0; i < d.tiles_per_chunk; ++i) {
            const int64_t f0 = c * pl->L + i * TILE;
            const int64_t f1 = std::min(f0 + (int64_t)TILE, (c + 1) * pl->L);   // end of the tile
            paro_tile_info &ti = tab[(size_t)i];
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
            }
        }
        paro_tile_info *dev_tab = nullptr;
        const int rc = upload(&dev_tab, tab.data(), tab.size());
        if (rc != PARO_OK) {                         // the next call tries again (and reports again)
            (void)hipFree(dev_tab);
            return rc;
        }
        d.tile_tab[(size_t)c] = dev_tab;
        d.tile_tab_tried[(size_t)c] = 1;
    }
    return PARO_OK;
}

// The map from elements to tensors for a launch whose element 0 is flat index `begin`.  The
// per-tile tables are per chunk: they serve launches that start on a chunk boundary and stay
// inside that chunk.
TensorMap map_for(const paro_plan_t *pl, const Scratch &sc, int64_t begin, bool one_chunk) {
    TensorMap tm;
    if (!sc.plan_tables) {                  // launches that never look at tensors (chunk layout, no decay mask)
        tm.nz_off = nullptr;
        tm.nz_tensor = nullptr;
        tm.nz_dtype = tm.dtype = tm.no_decay = nullptr;
        tm.n_nz = 0;
        tm.total = pl->total;
        tm.begin = begin;
        tm.tile_tab = nullptr;
        return tm;
    }
    tm.nz_off = pl->dev.nz_off;
    tm.nz_tensor = pl->dev.nz_tensor;
    tm.nz_dtype = pl->dev.nz_dtype;
    tm.dtype = pl->dev.dtype;
    tm.no_decay = pl->dev.no_decay;
    tm.n_nz = (int)pl->nz_tensor.size();
    tm.total = pl->total;
    tm.begin = begin;
    tm.tile_tab = nullptr;
    if (one_chunk && begin % pl->L == 0) tm.tile_tab = pl->dev.tile_tab[(size_t)(begin / pl->L)];
    return tm;
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

// Whether chunk c is cut into many small pieces of tensors (fewer than PARO_DENSE_BLOCKS_PER_TENSOR
// blocks per piece on average) rather than a few large ones.
bool many_small_tensors(const paro_plan_t *pl, int64_t c) {
    const int64_t f0 = c * pl->L, f1 = std::min((c + 1) * pl->L, pl->total);
    if (f0 >= f1) return false;                                             // all padding
    const auto first = std::upper_bound(pl->nz_off.begin(), pl->nz_off.end(), f0) - 1;
    const auto last = std::lower_bound(pl->nz_off.begin(), pl->nz_off.end(), f1);
    const int64_t pieces = last - first;
    return (int64_t)piece_grid(pl->L) < pieces * PARO_DENSE_BLOCKS_PER_TENSOR;
}

// Launches sweep 1 over chunk c; returns the number of per-block partial sums it writes.
template <bool SUMSQ>
int launch_reduce(const paro_plan_t *pl, const Scratch &sc, int layout, const SrcTable &tab, int group_len, int64_t c,
                  float *g, hipStream_t st) {
    const int64_t n = pl->L;
    double *partials = sc.partials;
    if (layout == PARO_CHUNK) {
        const unsigned grid = (piece_grid(n) + 7u) & ~7u;       // a multiple of 8: see partial_slot()
        const unsigned lds = throttle_lds(sc.lds_per_cu, fold_waves(fold_loads(pl->P), PARO_FOLD_LOADS_PER_CU));
        PARO_BY_DTYPE(pl->dtype[0], hipLaunchKernelGGL((k_reduce4<DT, SUMSQ>), dim3(grid), dim3(WAVE), lds, st, tab, pl->P,
                                                       group_len, n, g, partials));
        return (int)grid;
    }
    const TensorMap tm = map_for(pl, sc, c * pl->L, true);
    // What decides is the list.  A chunk cut into many small pieces of tensors: its waves wait for their look-ups
    // with no data in flight, and want more bytes in flight per wave and per compute unit (no throttle; with few
    // contributions and a launch that fills the GPU many times over, two blocks per wave).  A few large tensors:
    // the look-ups hit the scalar cache and the launch behaves like the chunk layout's, budget included; only with
    // 4 contributions or fewer does a wave with one block have too little in flight beside its look-ups.
    const bool small = many_small_tensors(pl, c);
    int64_t pair_min_blocks = PARO_PAIR_MIN_BLOCKS;
    const char *env = std::getenv("PARO_PAIR_MIN_BLOCKS");                  // for tests: pairs on any list from this size on
    if (env) pair_min_blocks = std::atoll(env);
    if (pl->P <= PARO_PAIR_MAX_RANKS && (small || env || 2 * pl->P <= PARO_PAIR_MAX_RANKS) &&
        (int64_t)piece_grid(n) >= pair_min_blocks) {
        const unsigned grid = (piece_grid(n, 2) + 7u) & ~7u;
        const unsigned lds = throttle_lds(
            sc.lds_per_cu, fold_waves(fold_loads(pl->P, 2), small ? PARO_FOLD_T_LOADS_PER_CU : PARO_FOLD_LOADS_PER_CU));
        hipLaunchKernelGGL((k_reduce4t<SUMSQ, 2, 8>), dim3(grid), dim3(WAVE), lds, st, tab, pl->P, group_len, n, g, partials, tm);
        return (int)grid;
    }
    const unsigned grid = (piece_grid(n) + 7u) & ~7u;
    const unsigned lds =
        throttle_lds(sc.lds_per_cu, fold_waves(fold_loads(pl->P), small ? PARO_FOLD_TM_LOADS_PER_CU : PARO_FOLD_LOADS_PER_CU));
    if (pl->P <= PARO_PAIR_MAX_RANKS)                                       // a batch of 8 contributions: fewer registers
        hipLaunchKernelGGL((k_reduce4t<SUMSQ, 1, 8>), dim3(grid), dim3(WAVE), lds, st, tab, pl->P, group_len, n, g, partials, tm);
    else
        hipLaunchKernelGGL((k_reduce4t<SUMSQ, 1, PARO_BATCH>), dim3(grid), dim3(WAVE), lds, st, tab, pl->P, group_len, n, g,
                           partials, tm);
    return (int)grid;
}

// Launches the single sweep (no clipping) over chunk c.
template <bool MASK>
void launch_fused(const paro_plan_t *pl, const Scratch &sc, int layout, const SrcTable &tab, int group_len, int64_t c,
                  const AdamConsts &a, float *p, float *m, float *v, uint16_t *dst, hipStream_t st) {
    const int64_t n = pl->L;
    const bool small = layout == PARO_TENSORS && many_small_tensors(pl, c);
    const int waves = fold_waves(fold_loads(pl->P) + 3, small ? PARO_FUSED_T_LOADS_PER_CU : PARO_FUSED_LOADS_PER_CU);
    const TensorMap tm = map_for(pl, sc, c * pl->L, true);
    const unsigned grid = piece_grid(n), lds = throttle_lds(sc.lds_per_cu, waves);
    if (layout == PARO_TENSORS)
        hipLaunchKernelGGL((k_fused4<true, PARO_BF16, MASK>), dim3(grid), dim3(WAVE), lds, st, tab, pl->P, group_len, n, a, p, m,
                           v, dst, tm);
    else
        PARO_BY_DTYPE(pl->dtype[0], hipLaunchKernelGGL((k_fused4<false, DT, MASK>), dim3(grid), dim3(WAVE), lds, st, tab,
                                                       pl->P, group_len, n, a, p, m, v, dst, tm));
}

// Adds the n_part partial sums a sweep-1 launch left in the scratch array into *out (device).
int finalize_partials(const Scratch &sc, int n_part, double *out, hipStream_t st) {
    if (n_part > 2 * FINALIZE_CHUNK) {       // two levels: slices of 2048 partials, then their sums
        const int nb = (n_part + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
        hipLaunchKernelGGL(k_finalize, dim3(nb), dim3(FINALIZE_TPB), 0, st, sc.partials, n_part, FINALIZE_CHUNK, sc.level2);
        PARO_HIP(hipGetLastError());
        hipLaunchKernelGGL(k_finalize, dim3(1), dim3(FINALIZE_TPB), 0, st, sc.level2, nb, nb, out);
    } else {
        hipLaunchKernelGGL(k_finalize, dim3(1), dim3(FINALIZE_TPB), 0, st, sc.partials, n_part, n_part, out);
    }
    PARO_HIP(hipGetLastError());
    return PARO_OK;
}

// Sweep 1 over the whole update range, chunk by chunk.  The sum of squares covers the rank's own
// chunk only (so that the ranks' values add up to the model's) - or, with norm_over_range, every
// chunk of the update range: one sum per chunk, added in chunk order.
int do_reduce(const paro_plan_t *pl, const Scratch &sc, int rank, const void *const *contrib, int layout, float *grad_out,
              double *sumsq_out, bool norm_over_range, hipStream_t st) {
    int rc;
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    const int own = paro::chunk_of_rank(pl, rank);
    const int64_t c0 = ob / pl->L, c1 = (ob + on) / pl->L;
    const bool per_chunk = sumsq_out && norm_over_range && c1 - c0 > 1;
    for (int64_t c = c0; c < c1; ++c) {
        SrcTable tab;
        int gl;
        const int64_t lo = c * pl->L - ob;
        src_table(pl, (int)c, contrib, layout, lo, &tab, &gl);
        if (sumsq_out && (per_chunk || c == own)) {
            const int n_part = launch_reduce<true>(pl, sc, layout, tab, gl, c, grad_out + lo, st);
            PARO_HIP(hipGetLastError());
            // the next launch reuses the scratch array: this chunk's partials are added up first
            if ((rc = finalize_partials(sc, n_part, per_chunk ? sc.chunk_sums + (c - c0) : sumsq_out, st))) return rc;
        } else {
            launch_reduce<false>(pl, sc, layout, tab, gl, c, grad_out + lo, st);
            PARO_HIP(hipGetLastError());
        }
    }
    if (per_chunk) {
        const int nc = (int)(c1 - c0);
        hipLaunchKernelGGL(k_finalize, dim3(1), dim3(FINALIZE_TPB), 0, st, sc.chunk_sums, nc, nc, sumsq_out);
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

template <bool PACK>
int launch_adam(const paro_plan_t *pl, const Scratch &sc, int rank, const AdamConsts &a, const float *grad,
                const double *total_sumsq, float *p, float *m, float *v, uint16_t *dst, hipStream_t st) {
    int64_t ob, on;
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    if (!pl->any_no_decay) {
        const unsigned lds = throttle_lds(sc.lds_per_cu, PARO_ADAM_WAVES_PER_CU);
        hipLaunchKernelGGL((k_adam4<PACK, false>), dim3(piece_grid(on)), dim3(WAVE), lds, st, a, total_sumsq, grad, p, m, v,
                           dst, on, map_for(pl, sc, ob, false));
        PARO_HIP(hipGetLastError());
        return PARO_OK;
    }
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {      // chunk by chunk: each has its own per-tile table
        const int64_t lo = c * pl->L - ob;
        const unsigned lds = throttle_lds(sc.lds_per_cu, PARO_ADAM_MASK_WAVES_PER_CU);
        hipLaunchKernelGGL((k_adam4<PACK, true>), dim3(piece_grid(pl->L)), dim3(WAVE), lds, st, a, total_sumsq, grad + lo,
                           p + lo, m + lo, v + lo, dst ? dst + lo : nullptr, pl->L, map_for(pl, sc, c * pl->L, true));
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

int do_adam(const paro_plan_t *pl, const Scratch &sc, int rank, const AdamConsts &a, const float *grad,
            const double *total_sumsq, float *p, float *m, float *v, uint16_t *dst /* nullable: no pack */, hipStream_t st) {
    return dst ? launch_adam<true>(pl, sc, rank, a, grad, total_sumsq, p, m, v, dst, st)
               : launch_adam<false>(pl, sc, rank, a, grad, total_sumsq, p, m, v, dst, st);
}

// The launches of the fused step, arguments already checked: two sweeps when the update waits for
// the norm (clipping, skip on overflow), else one.
int launch_step(const paro_plan_t *pl, const Scratch &sc, int rank, const void *const *contrib, int layout,
                const AdamConsts &a, float *grad_scratch, double *sumsq_scratch, float *p, float *m, float *v,
                uint16_t *dst_base, hipStream_t st) {
    int rc;
    int64_t dl, so, sl, ob, on;
    paro_pack_slot(pl, rank, &dl, &so, &sl);
    uint16_t *dst = dst_base + so;
    if (a.max_norm > 0.0f || a.skip_nonfinite) {
        // the norm this rank can form on its own: over everything it updates (its update range)
        if ((rc = do_reduce(pl, sc, rank, contrib, layout, grad_scratch, sumsq_scratch, true, st))) return rc;
        return do_adam(pl, sc, rank, a, grad_scratch, sumsq_scratch, p, m, v, dst, st);
    }
    paro::letter_range(pl, rank, pl->letters[2], &ob, &on);
    for (int64_t c = ob / pl->L; c < (ob + on) / pl->L; ++c) {
        SrcTable tab;
        int gl;
        const int64_t lo = c * pl->L - ob;
        src_table(pl, (int)c, contrib, layout, lo, &tab, &gl);
        if (pl->any_no_decay)
            launch_fused<true>(pl, sc, layout, tab, gl, c, a, p + lo, m + lo, v + lo, dst + lo, st);
        else
            launch_fused<false>(pl, sc, layout, tab, gl, c, a, p + lo, m + lo, v + lo, dst + lo, st);
        PARO_HIP(hipGetLastError());
    }
    return PARO_OK;
}

// ---- the library's own scratch, for the entry point that allocates nothing --------------------
// Partial sums of squares of one sweep-1 launch over a chunk of at most PARO_STATIC_MAX_CHUNK
// elements (one per block of 256), followed by the second-level sums.  Every device the library
// runs on holds its own copy of this array, at its own address, until the process ends.
constexpr int64_t STATIC_PARTIALS = PARO_STATIC_MAX_CHUNK / PIECE;
constexpr int64_t STATIC_LEVEL2 = (STATIC_PARTIALS + FINALIZE_CHUNK - 1) / FINALIZE_CHUNK;
static __device__ __align__(256) double scratch[STATIC_PARTIALS + STATIC_LEVEL2 + PARO_MAX_RANKS];

constexpr int MAX_DEVICES = 64;
struct StaticScratch {
    std::mutex mutex;
    double *ptr[MAX_DEVICES] = {};       // device address of `scratch` on each device, once asked for
    int lds_per_cu[MAX_DEVICES] = {};
};
StaticScratch g_static;

// The current device's copy of `scratch`.  In host code the array's name is only a handle for the
// runtime: its device address comes from hipGetSymbolAddress, once per device with that device
// current, and that address is what kernels, copies and fills get.  Allocates nothing.
int static_scratch(Scratch *out) {
    int dev = -1;
    PARO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(PARO_EINVAL, "paro_step_fused_static: device index out of range");
    std::lock_guard<std::mutex> lock(g_static.mutex);
    if (!g_static.ptr[dev]) {
        double *ptr = nullptr;
        PARO_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) return fail(PARO_EHIP, "hipGetSymbolAddress gave no address for the static scratch array");
        int lds = 0;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess ||
            lds < 65536) {
            (void)hipGetLastError();
            lds = 160 * 1024;
        }
        g_static.lds_per_cu[dev] = lds;
        g_static.ptr[dev] = ptr;
    }
    *out = Scratch{g_static.lds_per_cu[dev], g_static.ptr[dev], g_static.ptr[dev] + STATIC_PARTIALS,
                   g_static.ptr[dev] + STATIC_PARTIALS + STATIC_LEVEL2, false};
    return PARO_OK;
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
    if (layout == PARO_TENSORS && (rc = ensure_tile_tables(pl, rank))) return rc;
    return do_reduce(pl, plan_scratch(pl), rank, contrib, layout, grad_out, sumsq_out, false, static_cast<hipStream_t>(stream));
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
    if (pl->any_no_decay && (rc = ensure_tile_tables(pl, rank))) return rc;
    uint16_t *dst = nullptr;
    if (dst_base) {
        int64_t dl, so, sl;
        paro_pack_slot(pl, rank, &dl, &so, &sl);
        dst = dst_base + so;
    }
    return do_adam(pl, plan_scratch(pl), rank, a, grad, total_sumsq, p, m, v, dst, static_cast<hipStream_t>(stream));
}

int paro_pack_params(paro_plan_t *pl, int rank, const float *p, uint16_t *dst_base, void *stream) {
    int rc;
    if ((rc = check_common(pl, rank, "paro_pack_params"))) return rc;
    if ((rc = check_ptr(p, "paro_pack_params: p"))) return rc;
    if ((rc = check_ptr(dst_base, "paro_pack_params: dst_base"))) return rc;
    if ((rc = ensure_device(pl))) return rc;
    int64_t dl, so, sl;
    paro_pack_slot(pl, rank, &dl, &so, &sl);
    hipLaunchKernelGGL(k_pack, dim3(piece_grid(sl)), dim3(WAVE), throttle_lds(pl->dev.lds_per_cu, PARO_COPY_WAVES_PER_CU),
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
    if ((layout == PARO_TENSORS || pl->any_no_decay) && (rc = ensure_tile_tables(pl, rank))) return rc;
    return launch_step(pl, plan_scratch(pl), rank, contrib, layout, a, grad_scratch, sumsq_scratch, p, m, v, dst_base,
                       static_cast<hipStream_t>(stream));
}

int paro_step_fused_static(const paro_plan_t *pl, int rank, const void *const *contrib, const paro_adam_t *hp,
                           float *grad_scratch, double *sumsq_scratch, float *p, float *m, float *v,
                           uint16_t *dst_base, void *stream) {
    const char *fn = "paro_step_fused_static";
    int rc;
    AdamConsts a;
    if ((rc = check_common(pl, rank, fn))) return rc;
    if (pl->any_no_decay)
        return fail(PARO_EINVAL, std::string(fn) + ": a weight-decay mask needs the plan's device tables; use paro_step_fused");
    if (pl->L > PARO_STATIC_MAX_CHUNK)
        return fail(PARO_ERANGE, std::string(fn) + ": the plan's chunk of " + std::to_string(pl->L) +
                                     " elements exceeds PARO_STATIC_MAX_CHUNK (" +
                                     std::to_string((long long)PARO_STATIC_MAX_CHUNK) + ")");
    if ((rc = check_contrib(pl, contrib, PARO_CHUNK, fn))) return rc;
    if ((rc = adam_consts(hp, &a, fn))) return rc;
    if ((rc = check_ptr(p, "paro_step_fused_static: p"))) return rc;
    if ((rc = check_ptr(m, "paro_step_fused_static: m"))) return rc;
    if ((rc = check_ptr(v, "paro_step_fused_static: v"))) return rc;
    if ((rc = check_ptr(dst_base, "paro_step_fused_static: dst_base"))) return rc;
    a.pack_dtype = pl->pack_dtype;
    if (a.max_norm > 0.0f || a.skip_nonfinite) {
        if ((rc = check_ptr(grad_scratch, "paro_step_fused_static: grad_scratch"))) return rc;
        if (!sumsq_scratch || (reinterpret_cast<uintptr_t>(sumsq_scratch) & 7))
            return fail(sumsq_scratch ? PARO_EALIGN : PARO_EINVAL,
                        std::string(fn) + ": clipping and skip_nonfinite need sumsq_scratch");
    }
    Scratch sc;
    if ((rc = static_scratch(&sc))) return rc;
    return launch_step(pl, sc, rank, contrib, PARO_CHUNK, a, grad_scratch, sumsq_scratch, p, m, v, dst_base,
                       static_cast<hipStream_t>(stream));
}

}  // extern "C"


// ---- ring hops and scheduled transfers ----------------------------------------
namespace {
int launch_hop(const paro_plan_t *pl, const void *a, int da, const void *b, int db, float *out, int64_t n,
               hipStream_t st) {
    if (n <= 0) return PARO_OK;
    const unsigned grid = piece_grid(n);
    const unsigned lds = throttle_lds(pl->dev.lds_per_cu, PARO_HOP_WAVES_PER_CU);
#define PARO_HOP_CASE(A, B)                                                                                   \
    if (da == A && db == B) hipLaunchKernelGGL((k_hop<A, B>), dim3(grid), dim3(WAVE), lds, st, a, b, out, n)
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
            const unsigned grid = (unsigned)((n16 + WAVE - 1) / WAVE);
            if (n16 > 0) {
                hipLaunchKernelGGL(k_copy16, dim3(grid), dim3(WAVE), throttle_lds(pl->dev.lds_per_cu, PARO_COPY_WAVES_PER_CU), st,
                                   reinterpret_cast<const u32x4 *>(from), reinterpret_cast<u32x4 *>(mine), n16);
                PARO_HIP(hipGetLastError());
            }
        }
        received += m.recv_len;
    }
    return received;
}

}  // extern "C"
