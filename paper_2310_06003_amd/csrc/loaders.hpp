// How the fold gets its operands: the chunk layout (arrays in shard coordinates) and the tensor
// layout (per-tensor gradients found through the plan's offset table, staged per tile in LDS),
// and the ordered fold itself.  Included by kernels.hip only.
#pragma once

#include "device_util.hpp"

namespace {

// ------------------------------------------------------------------- loaders
// A loader hands the fold the 8 values that contribution k (in fold order)
// holds for the thread's 8 elements.

struct TileSegs;

// Contributions are arrays in shard coordinates, all of one dtype (bf16, fp16 or fp32).
template <int DT>
struct ChunkLoader {
    static constexpr bool kTensor = false;
    static constexpr int kElems = 8;
    // contributions loaded before the first is consumed (16 bytes each for the 2-byte dtypes, 32 for fp32)
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

// The same contributions taken 4 elements per thread: an 8-byte load per contribution for the
// 2-byte dtypes (a wave instruction covers 512 consecutive bytes), a 16-byte load for fp32.
template <int DT>
struct Chunk4Loader {
    static constexpr bool kTensor = false;
    static constexpr int kElems = 4;
    static constexpr int kBatch = PARO_BATCH_BF16;
    using Raw = std::conditional_t<DT == PARO_F32, u32x4, u32x2>;
    int64_t e;                                   // first of the thread's 4 elements
    template <bool SLOW>
    __device__ __forceinline__ void load(const SrcTable &src, int k, Raw &r) const {
        if constexpr (DT != PARO_F32)
            r = ld_contrib(reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(src.p[k]) + e));
        else
            r = ld_contrib(reinterpret_cast<const u32x4 *>(static_cast<const float *>(src.p[k]) + e));
    }
    template <bool SLOW>
    __device__ __forceinline__ void unpack(const SrcTable &, int, const Raw &r, float x[4]) const {
        if constexpr (DT != PARO_F32) {
            x[0] = cvt_lo<DT>(r.x); x[1] = cvt_hi<DT>(r.x); x[2] = cvt_lo<DT>(r.y); x[3] = cvt_hi<DT>(r.y);
        } else {
            x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
            x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
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
    static constexpr int kElems = 8;
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
    static constexpr int kElems = 8;
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
// (named for its first use: it folds Ld::kElems elements per thread)
// X[i] = contributions added in table order: runs of group_len into a partial A
// (left to right), partials into X (left to right).  The first value of a run
// and the first partial are copied, not added to zero (that would lose -0).
// SLOW (tensor layout only): some thread of the wave has a tensor boundary inside its 8
// elements; contributions are then taken one at a time, each thread on its own path.
template <class Ld, bool SLOW>
__device__ __forceinline__ void fold8(const Ld &ld, const SrcTable &src, int P, int group_len, float X[Ld::kElems]) {
    constexpr int E = Ld::kElems;                // elements per thread: 8, or 4 for the 4-element loaders
    float A[E];
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
                float x[E];
                ld.template unpack<SLOW>(src, k0 + b, raw[b], x);
                if (pos == 0) {
#pragma unroll
                    for (int i = 0; i < E; ++i) A[i] = x[i];
                } else {
#pragma unroll
                    for (int i = 0; i < E; ++i) A[i] = A[i] + x[i];
                }
                if (++pos == group_len) {
                    pos = 0;
                    if (first_group) {
#pragma unroll
                        for (int i = 0; i < E; ++i) X[i] = A[i];
                        first_group = false;
                    } else {
#pragma unroll
                        for (int i = 0; i < E; ++i) X[i] = X[i] + A[i];
                    }
                }
            }
        });
    }
}

}  // namespace
