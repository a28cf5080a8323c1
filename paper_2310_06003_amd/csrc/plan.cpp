// Host side of libparo: strategy validation, flat layout, ownership, fold order
// and collective message tables.  Integer work only; needs no GPU.
//
// Paper references: Sec. 3.1.1 (three sharding states), Sec. 3.1.3 (Principle 1
// -> the 14 strategies of Table 1), Table 2 (per-GPU sizes Psi/N and Psi/M),
// Sec. 3.4 (Ring, H-Ring, HO-Ring).
#include "plan.hpp"

#include <algorithm>
#include <cstring>
#include <functional>
#include <new>

namespace {
thread_local std::string g_last_error;

int fineness(char c) {          // coarse -> fine, Sec. 3.1.1
    switch (c) {
        case 'N': return 0;
        case 'I': return 1;
        case 'G': return 2;
        default: return -1;
    }
}

bool rank_ok(const paro_plan_t *pl, int rank) { return pl && rank >= 0 && rank < pl->P; }

// A ring of n members; this member sits at position idx.  unit(k) lists the
// chunks associated with ring position k (what position k ends up owning in a
// reduce-scatter / starts out with in an all-gather).  Step s of a
// reduce-scatter sends the partial of unit(idx - s) and receives unit(idx - s - 1);
// step s of an all-gather sends unit(idx - s + 1) and receives unit(idx - s).
struct RingPass {
    int n, idx, to, from, ring_id, phase;
    std::function<std::vector<int>(int)> unit;
};

void coalesce(std::vector<int> chunks, int64_t L, std::vector<std::pair<int64_t, int64_t>> *out) {
    std::sort(chunks.begin(), chunks.end());
    out->clear();
    for (int c : chunks) {
        int64_t o = (int64_t)c * L;
        if (!out->empty() && out->back().first + out->back().second == o)
            out->back().second += L;
        else
            out->push_back({o, L});
    }
}

void emit_pass(const RingPass &rp, int collective, int64_t L, std::vector<paro_msg_t> *msgs) {
    auto mod = [&](int x) { return ((x % rp.n) + rp.n) % rp.n; };
    std::vector<std::pair<int64_t, int64_t>> s, r;
    for (int step = 1; step < rp.n; ++step) {
        int su = collective == PARO_RS ? mod(rp.idx - step) : mod(rp.idx - step + 1);
        int ru = collective == PARO_RS ? mod(rp.idx - step - 1) : mod(rp.idx - step);
        coalesce(rp.unit(su), L, &s);
        coalesce(rp.unit(ru), L, &r);
        for (size_t n = 0; n < s.size() && n < r.size(); ++n) {
            paro_msg_t m;
            std::memset(&m, 0, sizeof m);
            m.phase = rp.phase;
            m.step = step;
            m.ring = rp.ring_id;
            m.send_to = rp.to;
            m.recv_from = rp.from;
            m.send_off = s[n].first;
            m.send_len = s[n].second;
            m.recv_off = r[n].first;
            m.recv_len = r[n].second;
            msgs->push_back(m);
        }
    }
}
}  // namespace

namespace paro {
int fail(int code, const std::string &msg) {
    g_last_error = msg;
    return code;
}

void letter_range(const paro_plan_t *pl, int rank, char letter, int64_t *begin, int64_t *len) {
    if (letter == 'G') {
        *begin = (int64_t)chunk_of_rank(pl, rank) * pl->L;
        *len = pl->L;
    } else if (letter == 'I') {
        *begin = (int64_t)local_of(pl, rank) * pl->g * pl->L;
        *len = (int64_t)pl->g * pl->L;
    } else {
        *begin = 0;
        *len = (int64_t)pl->P * pl->L;
    }
}

void fold_order(const paro_plan_t *pl, int chunk, int32_t *ranks, int32_t *group_len) {
    const int P = pl->P, G = pl->G, g = pl->g;
    const int owner = owner_of_chunk(pl, chunk);
    int n = 0;
    if (pl->sched == PARO_RING) {
        // the partial sum leaves the owner's successor and ends at the owner
        for (int k = 1; k <= P; ++k) ranks[n++] = (owner + k) % P;
        *group_len = P;
        return;
    }
    // hierarchical: inside each group the ring over local indices ends at the
    // owner's local index; the group partials travel the inter-group ring,
    // which ends at the owner's group
    const int oj = owner / G, oi = owner % G;
    for (int dj = 1; dj <= g; ++dj) {
        const int grp = (oj + dj) % g;
        for (int di = 1; di <= G; ++di) ranks[n++] = grp * G + (oi + di) % G;
    }
    *group_len = G;
}
}  // namespace paro

using namespace paro;

extern "C" {

const char *paro_last_error(void) { return g_last_error.c_str(); }

int paro_strategy_legal(const char *s) {
    if (!s || std::strlen(s) != 3) return 0;
    int fp = fineness(s[0]), fg = fineness(s[1]), fo = fineness(s[2]);
    if (fp < 0 || fg < 0 || fo < 0) return 0;
    return (fo >= fp && fo >= fg) ? 1 : 0;
}

int paro_plan(int P, int G, const char *strategy, const int64_t *tensor_sizes, int64_t n_tensors,
              const paro_plan_opts_t *opts, paro_plan_t **out) {
    if (!out) return fail(PARO_EINVAL, "paro_plan: out is NULL");
    *out = nullptr;
    if (P < 1 || P > PARO_MAX_RANKS) return fail(PARO_EINVAL, "paro_plan: P must be in [1, 256]");
    if (G < 1 || P % G != 0) return fail(PARO_EINVAL, "paro_plan: G must be >= 1 and divide P");
    if (!tensor_sizes || n_tensors < 1) return fail(PARO_EINVAL, "paro_plan: need at least one tensor");
    if (!strategy || std::strlen(strategy) != 3 || fineness(strategy[0]) < 0 || fineness(strategy[1]) < 0 ||
        fineness(strategy[2]) < 0)
        return fail(PARO_ESTRATEGY, "paro_plan: strategy must be three letters out of N, I, G");
    if (!paro_strategy_legal(strategy))
        return fail(PARO_ESTRATEGY,
                    "paro_plan: optimizer state must be sharded at least as finely as parameters and gradients");
    int sched = PARO_SCHED_DEFAULT;
    int64_t align = 8;
    int pack_dtype = PARO_BF16;
    if (opts) {
        pack_dtype = opts->pack_dtype;
        if (pack_dtype != PARO_BF16 && pack_dtype != PARO_F16)
            return fail(PARO_EINVAL, "paro_plan: pack_dtype must be PARO_BF16 or PARO_F16");
        sched = opts->sched;
        if (opts->align_elems != 0) align = opts->align_elems;
        if (sched < PARO_SCHED_DEFAULT || sched > PARO_HORING) return fail(PARO_EINVAL, "paro_plan: bad sched");
        if (align < 8 || align % 8 != 0)
            return fail(PARO_EINVAL, "paro_plan: align_elems must be a positive multiple of 8");
    }
    paro_plan_t *pl = new (std::nothrow) paro_plan_t;
    if (!pl) return fail(PARO_ENOMEM, "paro_plan: out of host memory");
    try {
        pl->P = P;
        pl->G = G;
        pl->g = P / G;
        std::memcpy(pl->letters, strategy, 3);
        pl->sched = sched == PARO_SCHED_DEFAULT ? ((G > 1 && G < P) ? PARO_HORING : PARO_RING) : sched;
        pl->align = align;
        pl->pack_dtype = pack_dtype;
        pl->T = n_tensors;
        pl->sizes.assign(tensor_sizes, tensor_sizes + n_tensors);
        pl->off.resize(n_tensors + 1);
        pl->dtype.assign(n_tensors, PARO_BF16);
        pl->no_decay.assign(n_tensors, 0);
        int64_t acc = 0;
        for (int64_t t = 0; t < n_tensors; ++t) {
            if (tensor_sizes[t] < 0) {
                delete pl;
                return fail(PARO_EINVAL, "paro_plan: negative tensor size");
            }
            pl->off[t] = acc;
            acc += tensor_sizes[t];
            if (opts && opts->grad_dtype) {
                if (opts->grad_dtype[t] > PARO_F16) {
                    delete pl;
                    return fail(PARO_EINVAL, "paro_plan: bad grad_dtype");
                }
                pl->dtype[t] = opts->grad_dtype[t];
            }
            if (opts && opts->no_decay) pl->no_decay[t] = opts->no_decay[t] ? 1 : 0;
            if (tensor_sizes[t] > 0) {
                pl->nz_off.push_back(pl->off[t]);
                pl->nz_tensor.push_back((int32_t)t);
            }
        }
        pl->off[n_tensors] = acc;
        pl->nz_off.push_back(acc);
        if (acc < 1) {
            delete pl;
            return fail(PARO_EINVAL, "paro_plan: the tensors hold no element");
        }
        pl->total = acc;
        int64_t per = (acc + P - 1) / P;
        pl->L = (per + align - 1) / align * align;
        pl->uniform_dtype = std::all_of(pl->dtype.begin(), pl->dtype.end(),
                                        [&](uint8_t d) { return d == pl->dtype[0]; });
        pl->any_no_decay = std::any_of(pl->no_decay.begin(), pl->no_decay.end(), [](uint8_t d) { return d != 0; });
    } catch (const std::bad_alloc &) {
        delete pl;
        return fail(PARO_ENOMEM, "paro_plan: out of host memory");
    }
    *out = pl;
    return PARO_OK;
}

int64_t paro_total(const paro_plan_t *pl) { return pl ? pl->total : (int64_t)PARO_EINVAL; }
int64_t paro_shard_len(const paro_plan_t *pl) { return pl ? pl->L : (int64_t)PARO_EINVAL; }
int64_t paro_padded_total(const paro_plan_t *pl) { return pl ? (int64_t)pl->P * pl->L : (int64_t)PARO_EINVAL; }
int paro_sched(const paro_plan_t *pl) { return pl ? pl->sched : PARO_EINVAL; }

int paro_chunk_of_rank(const paro_plan_t *pl, int rank) {
    if (!rank_ok(pl, rank)) return fail(PARO_ERANGE, "paro_chunk_of_rank: rank out of range");
    return chunk_of_rank(pl, rank);
}

int paro_owner_of_chunk(const paro_plan_t *pl, int chunk) {
    if (!pl || chunk < 0 || chunk >= pl->P) return fail(PARO_ERANGE, "paro_owner_of_chunk: chunk out of range");
    return owner_of_chunk(pl, chunk);
}

int paro_range(const paro_plan_t *pl, int rank, char state, int64_t *begin, int64_t *len) {
    if (!rank_ok(pl, rank)) return fail(PARO_ERANGE, "paro_range: rank out of range");
    if (!begin || !len) return fail(PARO_EINVAL, "paro_range: NULL output");
    int which = state == 'P' ? 0 : state == 'G' ? 1 : state == 'O' ? 2 : -1;
    if (which < 0) return fail(PARO_EINVAL, "paro_range: state must be 'P', 'G' or 'O'");
    letter_range(pl, rank, pl->letters[which], begin, len);
    return PARO_OK;
}

int64_t paro_segments(const paro_plan_t *pl, int rank, paro_seg_t *out, int64_t cap) {
    if (!rank_ok(pl, rank)) return fail(PARO_ERANGE, "paro_segments: rank out of range");
    if (cap < 0 || (cap > 0 && !out)) return fail(PARO_EINVAL, "paro_segments: bad output array");
    int64_t b, n;
    letter_range(pl, rank, pl->letters[2], &b, &n);
    const int64_t e = std::min(b + n, pl->total);
    int64_t count = 0;
    if (b >= e) return 0;
    // first non-empty tensor whose end lies past b
    size_t k = std::upper_bound(pl->nz_off.begin(), pl->nz_off.end(), b) - pl->nz_off.begin() - 1;
    for (; k + 1 < pl->nz_off.size() && pl->nz_off[k] < e; ++k) {
        int64_t lo = std::max(b, pl->nz_off[k]), hi = std::min(e, pl->nz_off[k + 1]);
        if (count < cap) out[count] = paro_seg_t{pl->nz_tensor[k], lo - pl->nz_off[k], lo - b, hi - lo};
        ++count;
    }
    return count;
}

int paro_fold_order(const paro_plan_t *pl, int chunk, int32_t *ranks, int32_t *group_len) {
    if (!pl || chunk < 0 || chunk >= pl->P) return fail(PARO_ERANGE, "paro_fold_order: chunk out of range");
    if (!ranks || !group_len) return fail(PARO_EINVAL, "paro_fold_order: NULL output");
    fold_order(pl, chunk, ranks, group_len);
    return PARO_OK;
}

int64_t paro_schedule(const paro_plan_t *pl, int rank, int sched, int collective, paro_msg_t *out, int64_t cap) {
    if (!rank_ok(pl, rank)) return fail(PARO_ERANGE, "paro_schedule: rank out of range");
    if (cap < 0 || (cap > 0 && !out)) return fail(PARO_EINVAL, "paro_schedule: bad output array");
    if (collective != PARO_RS && collective != PARO_AG) return fail(PARO_EINVAL, "paro_schedule: bad collective");
    if (sched == PARO_SCHED_DEFAULT) sched = pl->sched;
    if (sched < PARO_RING || sched > PARO_HORING) return fail(PARO_EINVAL, "paro_schedule: bad sched");
    const int P = pl->P, G = pl->G, g = pl->g;
    const int j = rank / G, i = rank % G;
    std::vector<paro_msg_t> msgs;
    try {
        RingPass flat{P, rank, (rank + 1) % P, (rank + P - 1) % P, 0, 1,
                      [&](int k) { return std::vector<int>{chunk_of_rank(pl, k)}; }};
        const int ito = j * G + (i + 1) % G, ifrom = j * G + (i + G - 1) % G;
        const int xto = ((j + 1) % g) * G + i, xfrom = ((j + g - 1) % g) * G + i;
        // units of the intra-group ring (position = local index b)
        auto whole_block = [&](int b) {
            std::vector<int> v;
            for (int jj = 0; jj < g; ++jj) v.push_back(b * g + jj);
            return v;
        };
        auto own_group_chunk = [&](int b) { return std::vector<int>{b * g + j}; };
        auto other_groups_chunks = [&](int b) {
            std::vector<int> v;
            for (int jj = 0; jj < g; ++jj)
                if (jj != j) v.push_back(b * g + jj);
            return v;
        };
        // unit of the inter-group ring (position = group index k), inside block i
        auto group_chunk = [&](int k) { return std::vector<int>{i * g + k}; };

        if (sched == PARO_RING) {
            emit_pass(flat, collective, pl->L, &msgs);
        } else if (sched == PARO_HRING) {
            if (collective == PARO_RS) {
                emit_pass({G, i, ito, ifrom, 0, 1, whole_block}, PARO_RS, pl->L, &msgs);
                emit_pass({g, j, xto, xfrom, 1, 2, group_chunk}, PARO_RS, pl->L, &msgs);
            } else {
                emit_pass({g, j, xto, xfrom, 1, 1, group_chunk}, PARO_AG, pl->L, &msgs);
                emit_pass({G, i, ito, ifrom, 0, 2, whole_block}, PARO_AG, pl->L, &msgs);
            }
        } else {  // HO-Ring
            if (collective == PARO_AG) {
                emit_pass({G, i, ito, ifrom, 0, 1, own_group_chunk}, PARO_AG, pl->L, &msgs);
                emit_pass({g, j, xto, xfrom, 1, 1, group_chunk}, PARO_AG, pl->L, &msgs);
                if (g > 1) emit_pass({G, i, ito, ifrom, 0, 2, other_groups_chunks}, PARO_AG, pl->L, &msgs);
            } else {
                if (g > 1) emit_pass({G, i, ito, ifrom, 0, 1, other_groups_chunks}, PARO_RS, pl->L, &msgs);
                emit_pass({G, i, ito, ifrom, 0, 2, own_group_chunk}, PARO_RS, pl->L, &msgs);
                emit_pass({g, j, xto, xfrom, 1, 2, group_chunk}, PARO_RS, pl->L, &msgs);
            }
        }
    } catch (const std::bad_alloc &) {
        return fail(PARO_ENOMEM, "paro_schedule: out of host memory");
    }
    for (int64_t n = 0; n < (int64_t)msgs.size() && n < cap; ++n) out[n] = msgs[n];
    return (int64_t)msgs.size();
}

int paro_cost(const char *strategy, double psi, double psit, int N, int M, int s, int K, int sched, paro_cost_t *out) {
    if (!out) return fail(PARO_EINVAL, "paro_cost: out is NULL");
    if (!paro_strategy_legal(strategy)) return fail(PARO_ESTRATEGY, "paro_cost: strategy is not one of Table 1's");
    if (N < 1 || M < 1 || N % M != 0 || s < 1 || K < 0 || !(psi > 0) || !(psit >= 0) || psit > psi)
        return fail(PARO_EINVAL, "paro_cost: need N >= 1, M | N, s >= 1, K >= 0, 0 <= Psi' <= Psi");
    if (sched < PARO_SCHED_DEFAULT || sched > PARO_HORING) return fail(PARO_EINVAL, "paro_cost: bad sched");
    const bool ring = sched == PARO_RING || (sched == PARO_SCHED_DEFAULT && !(M > 1 && M < N));
    const double g = (double)N / M, n = N, m = M, sd = s;
    std::memset(out, 0, sizeof *out);
    auto div = [&](char c) { return c == 'N' ? 1.0 : c == 'I' ? m : n; };
    out->mem_param = 2.0 * psi / div(strategy[0]);
    out->mem_grad = 2.0 * psit / div(strategy[1]);
    out->mem_os = (double)K * psit / div(strategy[2]);

    struct Vol { double intra, inter; };
    // one collective over all N GPUs on x elements (messages of x/N)
    auto global = [&](double x) -> Vol {
        if (ring) {
            const double links_inter = g > 1 ? g : 0;          // the flat ring crosses a group border g times
            return {(n - links_inter) * x / n * (n - 1), links_inter * x / n * (n - 1)};
        }
        return {n * x / m * (m - 1), n * x / n * (g - 1)};     // HO-Ring / H-Ring
    };
    auto intra_group = [&](double x) -> Vol { return {n * x / m * (m - 1), 0.0}; };
    auto inter_group = [&](double x) -> Vol { return {0.0, n * x / n * (g - 1)}; };
    auto add = [](double &a, double &b, Vol v, double times) { a += v.intra * times; b += v.inter * times; };

    const char sp = strategy[0], sg = strategy[1], so = strategy[2];
    // parameters are gathered before use in forward and in backward, every micro-batch (Sec. 3.1.1)
    if (sp == 'I') {
        add(out->fwd_ag_intra, out->fwd_ag_inter, intra_group(psi), sd);
        add(out->bwd_ag_intra, out->bwd_ag_inter, intra_group(psi), sd);
    } else if (sp == 'G') {
        add(out->fwd_ag_intra, out->fwd_ag_inter, global(psi), sd);
        add(out->bwd_ag_intra, out->bwd_ag_inter, global(psi), sd);
    }
    // sharded gradients are reduce-scattered every micro-batch
    if (sg == 'I') add(out->bwd_rs_intra, out->bwd_rs_inter, intra_group(psit), sd);
    if (sg == 'G') add(out->bwd_rs_intra, out->bwd_rs_inter, global(psit), sd);
    // update stage, once per mini-batch: bring the gradients to the optimizer state's sharding ...
    if (sg == 'N') {                                   // unsharded gradients: all-reduce (ZeRO-1 row, bold)
        add(out->upd_g_intra, out->upd_g_inter, global(psit), 2.0);
    } else if (sg == 'I' && so == 'G') {               // PaRO-IIG / NIG rows
        add(out->upd_g_intra, out->upd_g_inter, inter_group(psit), 1.0);
    } else if (sg == 'I' && so == 'I') {               // MiCS row: all-reduce of the group shard across groups
        out->upd_g_inter += 2.0 * g * psit / m * (g - 1);
        out->upd_g_intra += 2.0 * (n - g) * psit / m * (g - 1);
    }
    // ... and the updated parameters back to the parameters' sharding
    if (sp == 'N' && so == 'G') add(out->upd_ag_intra, out->upd_ag_inter, global(psi), 1.0);
    if (sp == 'I' && so == 'G') add(out->upd_ag_intra, out->upd_ag_inter, inter_group(psi), 1.0);
    if (sp == 'N' && so == 'I') add(out->upd_ag_intra, out->upd_ag_inter, intra_group(psi), 1.0);

    static const struct { const char *s; int rec[4]; int printed; } table1[] = {
        {"NNN", {1, 1, 1, 1}, 0}, {"NNI", {1, 1, 1, 1}, 0}, {"NNG", {1, 1, 1, 0}, 1}, {"NII", {1, 1, 1, 0}, 0},
        {"NIG", {1, 1, 1, 0}, 1}, {"NGG", {1, 1, 1, 0}, 1}, {"INI", {0, 0, 0, 1}, 0}, {"ING", {0, 1, 1, 0}, 0},
        {"III", {0, 0, 1, 0}, 1}, {"IIG", {1, 1, 0, 0}, 1}, {"IGG", {1, 1, 1, 0}, 1}, {"GNG", {0, 1, 1, 1}, 0},
        {"GIG", {0, 1, 1, 0}, 0}, {"GGG", {1, 1, 1, 0}, 1}};
    for (const auto &row : table1)
        if (std::strcmp(row.s, strategy) == 0) {
            for (int c = 0; c < 4; ++c) out->recommended[c] = row.rec[c];
            out->derived = row.printed ? 0 : 1;
        }
    return PARO_OK;
}

double paro_two_step_saving(double psi, int N, int M, int s) {
    if (N < 1 || M < 1 || N % M != 0 || s < 1) return 0.0;
    return psi * (s - 1) * ((double)N / M - 1) / N;
}

int paro_pack_slot(const paro_plan_t *pl, int rank, int64_t *dst_len, int64_t *slot_off, int64_t *slot_len) {
    if (!rank_ok(pl, rank)) return fail(PARO_ERANGE, "paro_pack_slot: rank out of range");
    if (!dst_len || !slot_off || !slot_len) return fail(PARO_EINVAL, "paro_pack_slot: NULL output");
    int64_t pb, pn, ob, on;
    letter_range(pl, rank, pl->letters[0], &pb, &pn);
    letter_range(pl, rank, pl->letters[2], &ob, &on);
    *dst_len = pn;
    *slot_off = ob - pb;      // Principle 1 makes the update range a sub-range of the parameter range
    *slot_len = on;
    return PARO_OK;
}

}  // extern "C"
