// Internal definition of the plan object (host side) shared by plan.cpp and the
// device entry points.  Not part of the public interface.
#pragma once
#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "paro.h"

#ifndef PARO_TILE_ELEMS
#define PARO_TILE_ELEMS 256
#endif
constexpr int PARO_TILE = PARO_TILE_ELEMS;      // elements per tile of the per-tile table (a multiple of 256)

// What a tile (PARO_TILE consecutive elements: by default one block's 256) of a chunk looks like,
// precomputed so that the kernels do not have to search: tensor >= 0: the whole tile lies inside that tensor, its first element at
// offset toff, first_seg = the tensor's gradient dtype; tensor == -1: the tile holds a tensor
// boundary (or ends in padding), first_seg = index of its first non-empty tensor; tensor == -2:
// the tile is all padding.
struct paro_tile_info {
    int64_t toff;
    int32_t tensor;
    int32_t first_seg;
};

struct paro_device_tables {
    int device = -1;
    int lds_per_cu = 0;             // bytes of LDS a compute unit has (for the occupancy throttle)
    int64_t *nz_off = nullptr;      // [n_nz + 1] flat start of every non-empty tensor, then Psi
    int32_t *nz_tensor = nullptr;   // [n_nz]     index of that tensor in the caller's list
    uint8_t *nz_dtype = nullptr;    // [n_nz]     its gradient dtype
    uint8_t *dtype = nullptr;       // [T]
    uint8_t *no_decay = nullptr;    // [T]
    // per chunk, built at the first call that works on the chunk tensor by tensor (tensor layout,
    // weight-decay mask):
    std::vector<paro_tile_info *> tile_tab;   // [P] the chunk's [tiles_per_chunk] table, or null
    std::vector<uint8_t> tile_tab_tried;      // [P] the decision for the chunk has been made
    int64_t tiles_per_chunk = 0;
    double *partials = nullptr;     // per-block partial sums of squares, then the second-level sums
    int64_t n_partials = 0;         // capacity of the first level
};

struct paro_plan_s {
    int P = 0, G = 0, g = 0;
    char letters[4] = {0, 0, 0, 0};     // parameter, gradient, optimizer state
    int sched = PARO_RING;
    int pack_dtype = PARO_BF16;         // dtype of the packed low-precision parameters
    int64_t align = 8;
    int64_t T = 0;
    std::vector<int64_t> sizes;         // [T]
    std::vector<int64_t> off;           // [T + 1]
    std::vector<uint8_t> dtype;         // [T]
    std::vector<uint8_t> no_decay;      // [T]
    bool uniform_dtype = true;
    bool any_no_decay = false;
    int64_t total = 0;                  // Psi
    int64_t L = 0;                      // chunk length
    std::vector<int64_t> nz_off;        // non-empty tensors only (see paro_device_tables)
    std::vector<int32_t> nz_tensor;

    std::mutex dev_mutex;
    paro_device_tables dev;             // filled on the first device call
};

enum { PARO_MIN_PARTIALS = 4096 };   // smallest partial-sum scratch

namespace paro {
int fail(int code, const std::string &msg);     // records the thread's last error, returns code
inline int group_of(const paro_plan_t *pl, int rank) { return rank / pl->G; }
inline int local_of(const paro_plan_t *pl, int rank) { return rank % pl->G; }
inline int chunk_of_rank(const paro_plan_t *pl, int rank) {
    return local_of(pl, rank) * pl->g + group_of(pl, rank);
}
inline int owner_of_chunk(const paro_plan_t *pl, int chunk) {
    return (chunk % pl->g) * pl->G + chunk / pl->g;
}
// [begin, begin+len) of a rank's range for a sharding letter
void letter_range(const paro_plan_t *pl, int rank, char letter, int64_t *begin, int64_t *len);
// ranks in fold order for a chunk, and the run length of the first-level sums
void fold_order(const paro_plan_t *pl, int chunk, int32_t *ranks, int32_t *group_len);
}  // namespace paro
