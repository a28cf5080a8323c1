// How the fold gets its operands - the chunk layout (arrays in shard coordinates) and the tensor
// layout (per-tensor gradients, found through the plan's per-tile table or by searching its offset
// table) - and the ordered fold itself.  Every sweep kernel runs in one-wave blocks of 256
// elements, 4 per thread.  Included by kernels.hip only.
#pragma once

#include "device_util.hpp"

namespace {

// ------------------------------------------------------------------- loaders
// A loader hands the fold the 4 values that contribution k (in fold order) holds for the
// thread's 4 elements: load() issues the memory operations, unpack() turns what came back into
// fp32.  kBatch contributions are loaded before the first is consumed.

// Contributions are arrays in shard coordinates, all of one dtype: an 8-byte load per
// contribution for the 2-byte dtypes (a wave instruction covers 512 consecutive bytes), a
// 16-byte load for fp32.
template <int DT>
struct Chunk4Loader {
    static constexpr int kBatch = PARO_BATCH;
    static constexpr int kElems = 4;
    static constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    using Raw = std::conditional_t<DT == PARO_F32, u32x4, u32x2>;
    int64_t e;                                   // first of the thread's 4 elements
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        r = ld_nt(reinterpret_cast<const Raw *>(static_cast<const char *>(src.p[k]) + e * ESIZE));
    }
    static __device__ __forceinline__ void to_f32(const Raw &r, float x[4]) {
        if constexpr (DT != PARO_F32) {
            x[0] = cvt_lo<DT>(r.x); x[1] = cvt_hi<DT>(r.x); x[2] = cvt_lo<DT>(r.y); x[3] = cvt_hi<DT>(r.y);
        } else {
            x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
            x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
        }
    }
    __device__ __forceinline__ void unpack(const Raw &r, float x[4]) const { to_f32(r, x); }
};

// Largest k in [0, n_entries) with tab[k] <= f, for a sorted table with
// tab[0] <= f; the 64 lanes of the wave probe 64 places per round.
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

// What a block knows about its 256 elements.
struct Piece {
    int tensor;        // >= 0: all of them lie in this tensor; -1: a tensor boundary (or the end of the
                       // data) falls inside; -2: all padding
    int dt;            // tensor >= 0: its gradient dtype
    int64_t toff;      // tensor >= 0: offset of the block's first element inside the tensor
    int seg;           // tensor == -1: index, in the table of non-empty tensors, of the one that
                       // holds the block's first element
};

// e0: the block's first element (< n, the launch's length).  With the per-tile table a block
// inside a single-tensor or all-padding tile needs one look-up; otherwise the wave searches the
// offset table (below the tile's first segment when the table gives it, else from the start).
// Everything returned is wave-uniform.
__device__ __forceinline__ Piece piece_of(const TensorMap &tm, int64_t e0, int64_t n) {
    Piece pc;
    pc.tensor = -2;
    pc.dt = PARO_BF16;
    pc.toff = 0;
    pc.seg = 0;
    const int64_t f0 = tm.begin + e0;
    int k_lo = 0, k_hi = tm.n_nz + 1;
    if (tm.tile_tab) {
        const paro_tile_info info = tm.tile_tab[e0 / TILE];                 // one address for the whole wave
        const int t = uniform(info.tensor);
        if (t != -1) {
            pc.tensor = t;
            pc.dt = uniform(info.first_seg);
            pc.toff = uniform(info.toff);
            return pc;
        }
        pc.tensor = -1;                                               // a boundary inside: the table names the first segment
        pc.seg = uniform(info.first_seg);
        return pc;
    }
    if (f0 >= tm.total) return pc;                                    // padding
    const int k = uniform(k_lo + wave_search(tm.nz_off + k_lo, k_hi - k_lo, f0, (int)lane_id()));
    const int64_t piece_end = tm.begin + min(e0 + (int64_t)PIECE, n);
    if (tm.nz_off[k + 1] >= piece_end) {
        pc.tensor = tm.nz_tensor[k];
        pc.dt = tm.dtype[pc.tensor];
        pc.toff = f0 - tm.nz_off[k];
    } else {
        pc.tensor = -1;
        pc.seg = k;
    }
    return pc;
}

// For a block with a boundary inside: tensor (-1 = padding), gradient dtype and offset inside the
// tensor of each of the thread's 4 elements.  EVERY lane of the wave must call this (lanes past the
// end of the launch included): the search runs across the lanes' registers.
//   f0: flat index of the block's first element, which lies in segment seg (nz_off[seg] <= f0);
//   x0: position of the thread's first element inside the block (4 * lane).
// Lane l fetches the l-th segment start after seg, as a position relative to the block (PIECE or
// more = beyond the block): one load per lane instead of a binary search through memory per lane.
// An element's segment is seg + the number of those starts at or before it, found by a binary
// search over the 64 lanes' values with shuffles.  Only a block with more than 64 starts inside
// (tensors of 1-3 elements in a row) walks the table in memory instead.
struct Located {
    int tens[4];
    int dt[4];
    int64_t toff[4];
};
__device__ __forceinline__ void locate4(const TensorMap &tm, int seg, int64_t f0, int x0, Located &loc) {
    const int lane = (int)lane_id();
    const int idx = seg + 1 + lane;                                    // nz_off[n_nz] = Psi: where padding starts
    int R = PIECE;
    if (idx <= tm.n_nz) R = (int)min(tm.nz_off[idx] - f0, (int64_t)PIECE);
    const int64_t first_start = tm.nz_off[seg];                        // wave-uniform: a scalar load
    if (uniform(__shfl(R, WAVE - 1, WAVE)) >= PIECE) {                 // the 64 starts cover the block
        int lo = 0, hi = WAVE - 1;                                     // starts at or before x0: a number in [lo, hi]
#pragma unroll                                                         // (not 64: lane 63's start lies beyond the block)
        for (int it = 0; it < 6; ++it) {                               // 64 candidates -> 1
            const int mid = (lo + hi) >> 1;
            const int r = __shfl(R, mid, WAVE);
            if (r <= x0) lo = mid + 1; else hi = mid;
        }
        int c = lo;                                                    // < 64: the last start lies beyond the block
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i > 0 && __shfl(R, c, WAVE) <= x0 + i) ++c;            // starts are distinct: at most one step
            const int before = __shfl(R, max(c - 1, 0), WAVE);         // start of the element's segment, if c > 0
            const int s = seg + c;
            loc.toff[i] = c == 0 ? f0 + x0 + i - first_start : (int64_t)(x0 + i - before);
            if (s < tm.n_nz) {
                loc.tens[i] = tm.nz_tensor[s];
                loc.dt[i] = tm.nz_dtype[s];
            } else {
                loc.tens[i] = -1;
                loc.dt[i] = PARO_BF16;
                loc.toff[i] = 0;
            }
        }
        return;
    }
    // more than 64 segment starts inside the block: per-lane search through the table
    const int64_t f = f0 + x0;
    int lo = seg, hi = min(seg + PIECE + 1, tm.n_nz + 1);             // nz_off[lo] <= f; nz_off[n_nz] = Psi
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tm.nz_off[mid] <= f) lo = mid; else hi = mid;
    }
    int c = lo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (c < tm.n_nz && tm.nz_off[c + 1] <= f + i) ++c;            // at most one step per element
        if (c < tm.n_nz) {
            loc.tens[i] = tm.nz_tensor[c];
            loc.dt[i] = tm.nz_dtype[c];
            loc.toff[i] = f + i - tm.nz_off[c];
        } else {
            loc.tens[i] = -1;
            loc.dt[i] = PARO_BF16;
            loc.toff[i] = 0;
        }
    }
}

// Contributions are per-tensor gradients (source k is a device array of T pointers) and the
// block's elements lie in one tensor.  Where a source's first byte for this block is 8-byte
// (2-byte dtypes) or 16-byte (fp32) aligned, one vector load fetches the thread's 4 values, as
// in the chunk layout; else element loads.  The test is wave-uniform, source by source.
template <int DT, int KB = PARO_BATCH>
struct Tensor4Loader {
    static constexpr int kBatch = (DT == PARO_F32 && KB > 8) ? KB / 2 : KB;     // 32 registers of loads in flight at most
    static constexpr int kElems = 4;
    static constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    using Raw = typename Chunk4Loader<DT>::Raw;
    int tensor;
    int64_t piece_byte_off;    // of the block's first element inside the tensor
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t b0 = static_cast<const uintptr_t *>(src.p[k])[tensor] + (uintptr_t)piece_byte_off;
        const uintptr_t mine = b0 + (uintptr_t)lane_id() * (4 * ESIZE);
        if ((b0 & (4 * ESIZE - 1)) == 0) {
            r = ld_nt(global_ptr<Raw>(mine));
        } else if constexpr (DT != PARO_F32) {
            const auto *h = global_ptr<uint16_t>(mine);
            r.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
            r.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
        } else {
            const auto *w = global_ptr<unsigned int>(mine);
            r = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
    __device__ __forceinline__ void unpack(const Raw &r, float x[4]) const { Chunk4Loader<DT>::to_f32(r, x); }
};

// Two consecutive blocks inside one tensor, folded by one wave (sweep 1 with few contributions:
// the wave then has as many loads in flight as with many, and one look-up serves 512 elements).
// The thread's elements 0-3 lie in the first block, 4-7 in the second, 256 elements further on.
template <int DT>
struct Tensor8Loader {
    static constexpr int kBatch = DT == PARO_F32 ? 4 : 8;     // 32 registers of loads in flight either way
    static constexpr int kElems = 8;
    static constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    using Raw4 = typename Chunk4Loader<DT>::Raw;
    struct Raw { Raw4 a, b; };
    int tensor;
    int64_t piece_byte_off;    // of the first block's first element inside the tensor
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t b0 = static_cast<const uintptr_t *>(src.p[k])[tensor] + (uintptr_t)piece_byte_off;
        const uintptr_t mine = b0 + (uintptr_t)lane_id() * (4 * ESIZE);
        constexpr uintptr_t NEXT = (uintptr_t)PIECE * ESIZE;
        if ((b0 & (4 * ESIZE - 1)) == 0) {
            r.a = ld_nt(global_ptr<Raw4>(mine));
            r.b = ld_nt(global_ptr<Raw4>(mine + NEXT));
        } else if constexpr (DT != PARO_F32) {
            const auto *h = global_ptr<uint16_t>(mine), *h2 = global_ptr<uint16_t>(mine + NEXT);
            r.a.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
            r.a.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
            r.b.x = (unsigned)h2[0] | ((unsigned)h2[1] << 16);
            r.b.y = (unsigned)h2[2] | ((unsigned)h2[3] << 16);
        } else {
            const auto *w = global_ptr<unsigned int>(mine), *w2 = global_ptr<unsigned int>(mine + NEXT);
            r.a = u32x4{w[0], w[1], w[2], w[3]};
            r.b = u32x4{w2[0], w2[1], w2[2], w2[3]};
        }
    }
    __device__ __forceinline__ void unpack(const Raw &r, float x[8]) const {
        Chunk4Loader<DT>::to_f32(r.a, x);
        Chunk4Loader<DT>::to_f32(r.b, x + 4);
    }
};

// ... and a tensor boundary (or the end of the data) falls inside the block: every element has
// its own tensor, dtype and offset; element loads.  Padding contributes +0.  A source's base
// pointer is fetched per element only where the thread's elements lie in different tensors.
struct Lane4Loader {
    static constexpr int kBatch = PARO_LANE_BATCH;
    static constexpr int kElems = 4;
    struct Raw { unsigned int bits[4]; };
    Located at;
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t *ptrs = static_cast<const uintptr_t *>(src.p[k]);
        uintptr_t b = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r.bits[i] = 0u;
            if (at.tens[i] >= 0) {
                if (i == 0 || at.tens[i] != at.tens[i - 1]) b = ptrs[at.tens[i]];
                if (at.dt[i] != PARO_F32)
                    r.bits[i] = global_ptr<uint16_t>(b)[at.toff[i]];
                else
                    r.bits[i] = global_ptr<unsigned int>(b)[at.toff[i]];
            }
        }
    }
    __device__ __forceinline__ void unpack(const Raw &r, float x[4]) const {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            x[i] = at.tens[i] < 0 ? 0.0f
                                  : at.dt[i] != PARO_F32 ? cvt16(r.bits[i], at.dt[i]) : __uint_as_float(r.bits[i]);
    }
};

// ---------------------------------------------------------------------- fold
// X[i] = contributions added in table order: runs of group_len into a partial A
// (left to right), partials into X (left to right).  The first value of a run
// and the first partial are copied, not added to zero (that would lose -0).
// A thread folds Ld::kElems elements (4, or 8 when the wave takes two blocks).
template <class Ld>
__device__ __forceinline__ void fold4(const Ld &ld, const SrcTable &src, int P, int group_len, float *X) {
    constexpr int NE = Ld::kElems;
    float A[NE];
    int pos = 0;
    bool first_group = true;
    constexpr int B = Ld::kBatch;
    for (int k0 = 0; k0 < P; k0 += B) {
        typename Ld::Raw raw[B];
        static_for<0, B>([&](auto b) {
            if (k0 + b < P) ld.load(src, k0 + b, raw[b]);
        });
        static_for<0, B>([&](auto b) {
            if (k0 + b < P) {
                float x[NE];
                ld.unpack(raw[b], x);
                if (pos == 0) {
#pragma unroll
                    for (int i = 0; i < NE; ++i) A[i] = x[i];
                } else {
#pragma unroll
                    for (int i = 0; i < NE; ++i) A[i] = A[i] + x[i];
                }
                if (++pos == group_len) {
                    pos = 0;
                    if (first_group) {
#pragma unroll
                        for (int i = 0; i < NE; ++i) X[i] = A[i];
                        first_group = false;
                    } else {
#pragma unroll
                        for (int i = 0; i < NE; ++i) X[i] = X[i] + A[i];
                    }
                }
            }
        });
    }
}

// The ordered fold of the thread's 4 elements out of per-tensor gradients, for a block that is
// not all padding.  loc: from locate4 when the block holds a boundary (pc.tensor == -1).
// KB: contributions loaded before the first is consumed (a kernel that is only launched for few
// contributions says so, and saves the registers).
template <int KB = PARO_BATCH>
__device__ __forceinline__ void fold_tensors(const Piece &pc, const Located &loc, const SrcTable &src, int P,
                                             int group_len, float X[4]) {
    if (pc.tensor >= 0) {
        if (pc.dt == PARO_BF16) {
            Tensor4Loader<PARO_BF16, KB> ld{pc.tensor, pc.toff * 2};
            fold4(ld, src, P, group_len, X);
        } else if (pc.dt == PARO_F16) {
            Tensor4Loader<PARO_F16, KB> ld{pc.tensor, pc.toff * 2};
            fold4(ld, src, P, group_len, X);
        } else {
            Tensor4Loader<PARO_F32, KB> ld{pc.tensor, pc.toff * 4};
            fold4(ld, src, P, group_len, X);
        }
    } else {
        Lane4Loader ld{loc};
        fold4(ld, src, P, group_len, X);
    }
}

// ... of the thread's 8 elements in two consecutive blocks that lie in one tensor (pc: the first).
__device__ __forceinline__ void fold_tensor_pair(const Piece &pc, const SrcTable &src, int P, int group_len, float X[8]) {
    if (pc.dt == PARO_BF16) {
        Tensor8Loader<PARO_BF16> ld{pc.tensor, pc.toff * 2};
        fold4(ld, src, P, group_len, X);
    } else if (pc.dt == PARO_F16) {
        Tensor8Loader<PARO_F16> ld{pc.tensor, pc.toff * 2};
        fold4(ld, src, P, group_len, X);
    } else {
        Tensor8Loader<PARO_F32> ld{pc.tensor, pc.toff * 4};
        fold4(ld, src, P, group_len, X);
    }
}

}  // namespace
