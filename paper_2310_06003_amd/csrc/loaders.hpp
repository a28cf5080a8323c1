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
        const paro_tile_info info = tm.tile_tab[e0 / TILE];           // one address for the whole wave
        const int t = uniform(info.tensor);
        if (t != -1) {
            pc.tensor = t;
            pc.dt = uniform(info.first_seg);
            pc.toff = uniform(info.toff) + (e0 % TILE);
            return pc;
        }
        k_lo = uniform(info.first_seg);                               // the tile's first segment
        k_hi = min(k_hi, k_lo + TILE + 1);                            // segments are at least one element long
    }
    if (f0 >= tm.total) return pc;                                    // padding
    const int k = uniform(k_lo + wave_search(tm.nz_off + k_lo, k_hi - k_lo, f0, threadIdx.x));
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

// For a block with a boundary inside: tensor (-1 = padding) and offset of each of the thread's 4
// elements, f being the flat index of the first.  The block's first element lies in segment seg,
// and 256 elements meet at most 256 further segments.
__device__ __forceinline__ void locate4(const TensorMap &tm, int seg, int64_t f, int tens[4], int64_t toff[4]) {
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
            tens[i] = tm.nz_tensor[c];
            toff[i] = f + i - tm.nz_off[c];
        } else {
            tens[i] = -1;
            toff[i] = 0;
        }
    }
}

// Contributions are per-tensor gradients (source k is a device array of T pointers) and the
// block's elements lie in one tensor.  Where a source's first byte for this block is 8-byte
// (2-byte dtypes) or 16-byte (fp32) aligned, one vector load fetches the thread's 4 values, as
// in the chunk layout; else element loads.  The test is wave-uniform, source by source.
template <int DT>
struct Tensor4Loader {
    static constexpr int kBatch = PARO_BATCH;
    static constexpr int ESIZE = DT == PARO_F32 ? 4 : 2;
    using Raw = typename Chunk4Loader<DT>::Raw;
    int tensor;
    int64_t piece_byte_off;    // of the block's first element inside the tensor
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t b0 = static_cast<const uintptr_t *>(src.p[k])[tensor] + (uintptr_t)piece_byte_off;
        const uintptr_t mine = b0 + (uintptr_t)threadIdx.x * (4 * ESIZE);
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

// ... and a tensor boundary (or the end of the data) falls inside the block: every element has
// its own tensor, dtype and offset; element loads.  Padding contributes +0.
struct Lane4Loader {
    static constexpr int kBatch = PARO_LANE_BATCH;
    struct Raw { unsigned int bits[4]; };
    int tens[4];
    int dt[4];
    int64_t toff[4];
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        const uintptr_t *ptrs = static_cast<const uintptr_t *>(src.p[k]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r.bits[i] = 0u;
            if (tens[i] >= 0) {
                const uintptr_t b = ptrs[tens[i]];
                if (dt[i] != PARO_F32)
                    r.bits[i] = global_ptr<uint16_t>(b)[toff[i]];
                else
                    r.bits[i] = global_ptr<unsigned int>(b)[toff[i]];
            }
        }
    }
    __device__ __forceinline__ void unpack(const Raw &r, float x[4]) const {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            x[i] = tens[i] < 0 ? 0.0f : dt[i] != PARO_F32 ? cvt16(r.bits[i], dt[i]) : __uint_as_float(r.bits[i]);
    }
};

// ---------------------------------------------------------------------- fold
// X[i] = contributions added in table order: runs of group_len into a partial A
// (left to right), partials into X (left to right).  The first value of a run
// and the first partial are copied, not added to zero (that would lose -0).
template <class Ld>
__device__ __forceinline__ void fold4(const Ld &ld, const SrcTable &src, int P, int group_len, float X[4]) {
    float A[4];
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
                float x[4];
                ld.unpack(raw[b], x);
                if (pos == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) A[i] = x[i];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) A[i] = A[i] + x[i];
                }
                if (++pos == group_len) {
                    pos = 0;
                    if (first_group) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) X[i] = A[i];
                        first_group = false;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) X[i] = X[i] + A[i];
                    }
                }
            }
        });
    }
}

// The ordered fold of the thread's 4 elements out of per-tensor gradients, for a block that is
// not all padding.  e: the thread's first element.
__device__ __forceinline__ void fold_tensors(const TensorMap &tm, const Piece &pc, int64_t e, const SrcTable &src, int P,
                                             int group_len, float X[4]) {
    if (pc.tensor >= 0) {
        if (pc.dt == PARO_BF16) {
            Tensor4Loader<PARO_BF16> ld{pc.tensor, pc.toff * 2};
            fold4(ld, src, P, group_len, X);
        } else if (pc.dt == PARO_F16) {
            Tensor4Loader<PARO_F16> ld{pc.tensor, pc.toff * 2};
            fold4(ld, src, P, group_len, X);
        } else {
            Tensor4Loader<PARO_F32> ld{pc.tensor, pc.toff * 4};
            fold4(ld, src, P, group_len, X);
        }
    } else {
        Lane4Loader ld;
        locate4(tm, pc.seg, tm.begin + e, ld.tens, ld.toff);
#pragma unroll
        for (int i = 0; i < 4; ++i) ld.dt[i] = ld.tens[i] >= 0 ? tm.dtype[ld.tens[i]] : PARO_BF16;
        fold4(ld, src, P, group_len, X);
    }
}

}  // namespace
