/*
 * libparo - the one-GPU share of a PaRO training step's Update stage, for
 * AMD MI355X (gfx950).
 *
 * Paper: "Rethinking Memory and Communication Costs for Efficient Large
 * Language Model Training" (PaRO + HO-Ring).  This library does the per-GPU
 * work of the Update stage of a PaRO training step (Sec. 3.2, the walk-throughs
 * of PaRO-IGG / IIG / NIG): after the last micro-batch the reduce-scatter leaves
 * every rank with the summed gradients of its own shard; the rank runs Adam on
 * the optimizer state of that shard, and the new parameters leave in 16 bits
 * for the all-gather that follows.
 *
 *   paro_plan           who owns what (Sec. 3.1.1 sharding states, Table 1
 *                       strategies), in which order the reduce-scatter adds the
 *                       ranks' contributions (Sec. 3.4 Ring / H-Ring / HO-Ring),
 *                       and where the packed parameters go;
 *   paro_reduce_shard   sums the P contributions to this rank's range in that
 *                       order (fp32), and the sum of squares of the result;
 *   paro_adam_shard     mixed-precision Adam on the range (Sec. 3.1.2: fp32
 *                       master copy + two moments = 12 bytes/param), with
 *                       optional global-norm clipping;
 *   paro_pack_params    rounds the master parameters to bf16 into the
 *                       all-gather buffer;
 *   paro_step_fused     the three in two sweeps over memory (one when not
 *                       clipping).
 *
 * Peer ranks are simulated: their contributions are buffers in this GPU's
 * memory.  No collective is issued.
 *
 * NAMING.  P = number of ranks in the cluster (the paper's N), G = ranks per
 * group (the paper's M), g = P / G groups.  Rank r is local index i = r % G of
 * group j = r / G.  A strategy is three letters, parameter / gradient /
 * optimizer state, each 'N' (not sharded), 'I' (sharded inside the group,
 * replicated across groups) or 'G' (sharded over all ranks) - Table 1.
 *
 * LAYOUT.  The tensors are laid end to end into a flat buffer of
 * Psi = sum(sizes) elements, cut into P chunks of
 * L = align * ceil(ceil(Psi / P) / align) elements; elements at and past Psi
 * are padding (their gradient is 0; their state stays 0).  Block b (0 <= b < G)
 * is chunks [b*g, (b+1)*g): the intra-group shard of local index b.  Chunk
 * i*g + j belongs to rank (group j, local i).  A rank's range for a state is its
 * chunk ('G'), its block ('I') or everything ('N').  Its UPDATE RANGE is the
 * range of its optimizer state; grad_out, p, m and v below are arrays over the
 * update range ("shard coordinates": element 0 = first element of the range).
 *
 * CONVENTIONS.  Every function returns PARO_OK (0) or a negative error code and
 * never throws or aborts; paro_last_error() gives the text of the calling
 * thread's last failure.  The caller owns every buffer it passes in.  The
 * library owns the plan: its host tables, and - created on the first device
 * call, on the device that is current then - device memory for the tensor
 * offset tables and a scratch array of partial sums (8 bytes per 256 elements
 * of a chunk); the first call for a rank that uses the tensor layout or a
 * weight-decay mask adds a per-tile table for each chunk of that rank's update
 * range (16 bytes per 256 elements, built when the chunk has at most 4 Mi
 * tiles, or at most PARO_TILE_TABLE_MAX_TILES when that environment variable
 * is set; without it the kernels search; PARO_PAIR_MIN_BLOCKS, also read at
 * every call, makes sweep 1 of the tensor layout give a wave two blocks from
 * that many blocks on, whatever the tensor list, instead of from the built-in
 * size on for lists of many small tensors - both exist for tests).  Those first calls allocate and copy
 * synchronously - make them outside any stream capture; every later call only
 * enqueues kernels and can be captured.  Device
 * functions only enqueue work on `stream` (a hipStream_t passed as void*; NULL =
 * the default stream) and never synchronise; a launch error is reported by the
 * call that launched.  Calls that run concurrently on ONE plan (different
 * streams) race on the plan's scratch array; use one plan per stream.  Host
 * queries are thread-safe; a plan is immutable after creation.  "device" /
 * "host" below says where a pointer must point.
 */
#ifndef PARO_H
#define PARO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct paro_plan_s paro_plan_t; /* opaque */

enum { PARO_OK = 0, PARO_EINVAL = -1, PARO_ESTRATEGY = -2, PARO_ERANGE = -3, PARO_ENOMEM = -4,
       PARO_EHIP = -5, PARO_EALIGN = -6 };
enum { PARO_SCHED_DEFAULT = -1, PARO_RING = 0, PARO_HRING = 1, PARO_HORING = 2 };
enum { PARO_BF16 = 0, PARO_F32 = 1, PARO_F16 = 2 }; /* dtype of gradient contributions / packed parameters */
enum { PARO_CHUNK = 0, PARO_TENSORS = 1 };     /* how the contributions are laid out */
enum { PARO_RS = 0, PARO_AG = 1 };             /* reduce-scatter, all-gather */
enum { PARO_MAX_RANKS = 256 };                 /* largest P */

typedef struct {
    int32_t sched;              /* PARO_SCHED_DEFAULT: HO-Ring when 1 < G < P, else ring */
    int32_t align_elems;        /* 0 = default 8; otherwise a positive multiple of 8 */
    const uint8_t *grad_dtype;  /* host [n_tensors] of PARO_BF16/PARO_F32/PARO_F16, or NULL = all bf16 */
    const uint8_t *no_decay;    /* host [n_tensors], nonzero = exempt from weight decay, or NULL */
    int32_t pack_dtype;         /* low-precision parameter format: PARO_BF16 (0, default) or PARO_F16 */
    int32_t reserved_;          /* 0 */
} paro_plan_opts_t;

/* a piece of a tensor inside a range */
typedef struct { int64_t tensor, tensor_off, shard_off, len; } paro_seg_t;

/* one contiguous range of one message of a collective; offsets in elements of
 * the padded flat buffer.  Entries with equal (phase, ring, step) make up one
 * logical message; the n-th such entry of the sender pairs with the n-th of
 * the receiver. */
typedef struct {
    int32_t phase, step, ring /* 0 intra-group (or the flat ring), 1 inter-group */, send_to, recv_from;
    int32_t pad_;
    int64_t send_off, send_len, recv_off, recv_len;
} paro_msg_t;

/* Adam hyper-parameters (Kingma & Ba, Algorithm 1; the paper only names the
 * optimizer).  step is 1 on the first update.  grad_scale multiplies the summed
 * gradient (1/P gives the mean).  max_norm > 0 clips by global L2 norm:
 *   coef = min(1, max_norm / (grad_scale * sqrt(total_sumsq) + 1e-6)).
 * adamw != 0: decoupled decay  p <- p*(1 - lr*wd) - step;  adamw == 0: classic
 * L2 (wd*p is added to the gradient before the moments).
 * skip_nonfinite != 0 (fp16 training with loss scaling; the paper says only
 * "mixed precision"): when total_sumsq is not finite - some gradient overflowed -
 * the update leaves p, m, v and the packed parameters untouched; the caller
 * reads the scalar, halves its loss scale and goes on.  The un-scaling by the
 * loss scale S is folded into grad_scale (1 / (P * S) for the mean). */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay, grad_scale, max_norm;
    int32_t step, adamw, skip_nonfinite;
} paro_adam_t;

/* ---- plan (host only; needs no GPU) -------------------------------------- */

/* 1 if the three letters satisfy Principle 1 (Sec. 3.1.3: the optimizer state
 * is sharded at least as finely as parameters and as gradients) - the 14 rows
 * of Table 1 - else 0. */
int paro_strategy_legal(const char *strategy);

/* Builds a plan.  tensor_sizes: host [n_tensors], each >= 0, sum >= 1.
 * Errors: P < 1, P > PARO_MAX_RANKS, G < 1, P % G != 0, n_tensors < 1, a negative
 * size, a bad option -> PARO_EINVAL; strategy not in Table 1 -> PARO_ESTRATEGY.
 * On success *out owns the plan; free it with paro_plan_destroy. */
int paro_plan(int P, int G, const char *strategy, const int64_t *tensor_sizes, int64_t n_tensors,
              const paro_plan_opts_t *opts /* nullable */, paro_plan_t **out);
void paro_plan_destroy(paro_plan_t *plan);

int64_t paro_total(const paro_plan_t *plan);        /* Psi */
int64_t paro_shard_len(const paro_plan_t *plan);    /* L */
int64_t paro_padded_total(const paro_plan_t *plan); /* P * L */
int paro_sched(const paro_plan_t *plan);            /* the resolved schedule kind */

/* Chunk owned by a rank under global sharding ('G', Sec. 3.1.1), and its inverse.
 * With the N GPUs in g groups of M (Sec. 3.4, Fig. 4) rank (group j, local index i)
 * owns chunk i*g + j: the g chunks of local index i's intra-group shard ('I':
 * Psi/M elements, Table 2) are dealt to the ranks with that local index, one per
 * group, so that the inter-group reduce-scatter of PaRO-IIG / NIG and the
 * inter-group all-gather of PaRO-IGG / IIG (Sec. 3.2) work inside one intra-group
 * shard.  The figures that would show the assignment are not in the text: this
 * nesting is the reading taken.  Returns < 0 (an error code) for a rank or chunk
 * out of range. */
int paro_chunk_of_rank(const paro_plan_t *plan, int rank);
int paro_owner_of_chunk(const paro_plan_t *plan, int chunk);

/* Range a rank holds of state 'P' (parameters), 'G' (gradients) or 'O'
 * (optimizer state = the update range), in elements of the padded flat buffer,
 * from the state's sharding letter (Sec. 3.1.1): 'N' everything, 'I' the rank's
 * block of g*L elements (Psi/M of Table 2), 'G' its chunk of L (Psi/N).  *len
 * times the bytes per element is Table 2's entry when P divides Psi.
 * PARO_ERANGE for a bad rank, PARO_EINVAL for another state letter. */
int paro_range(const paro_plan_t *plan, int rank, char state, int64_t *begin, int64_t *len);

/* Pieces of tensors inside the rank's update range, in order (the model state is
 * sharded as one flat sequence of parameters, Sec. 3.1.1 / Table 2, so a range
 * cuts through tensors wherever it falls); writes at most cap entries to out
 * (host, may be NULL when cap == 0) and returns the full count, or a negative
 * error.  Empty tensors and padding give no piece. */
int64_t paro_segments(const paro_plan_t *plan, int rank, paro_seg_t *out, int64_t cap);

/* order in which the reduce-scatter adds the P ranks' contributions to a chunk
 * (Sec. 3.4): ranks[0..P) (host) lists them; consecutive runs of *group_len
 * are summed left to right into partials, the partials left to right.  The flat
 * ring gives *group_len == P; the chunk's owner always comes last. */
int paro_fold_order(const paro_plan_t *plan, int chunk, int32_t *ranks, int32_t *group_len);

/* message table of a rank for a reduce-scatter (PARO_RS) or all-gather
 * (PARO_AG) under schedule kind `sched` (PARO_SCHED_DEFAULT = the plan's own).
 * Same cap / count convention as paro_segments.  Ring: Sec. 3.4 "traditional
 * Ring"; H-Ring: two sequential steps (intra-group first for a reduce-scatter,
 * last for an all-gather); HO-Ring: phase 1 = both rings at once on the rank's
 * own chunk, phase 2 = intra-group ring passing on what the inter-group ring
 * delivered (all-gather), and the reverse in time for a reduce-scatter. */
int64_t paro_schedule(const paro_plan_t *plan, int rank, int sched, int collective, paro_msg_t *out,
                      int64_t cap);

/* Where paro_pack_params writes.  The Update stage ends with every rank's new
 * low-precision parameters being all-gathered into the range its parameter
 * sharding keeps (Sec. 3.2: across groups for PaRO-IGG / IIG, over all ranks for
 * PaRO-NIG, not at all when parameters are sharded like the optimizer state): the
 * rank's parameter buffer has *dst_len elements (its 'P' range) and the update
 * range sits at *slot_off in it, *slot_len long - the send slot of that
 * all-gather, in place. */
int paro_pack_slot(const paro_plan_t *plan, int rank, int64_t *dst_len, int64_t *slot_off,
                   int64_t *slot_len);

/* ---- device work ------------------------------------------------------------
 * contrib: HOST array of P pointers, indexed by rank (contrib[rank] is this
 * rank's own gradient).
 *   PARO_CHUNK:   contrib[q] -> DEVICE array over the update range, 16-byte
 *                 aligned, all of one dtype (every tensor of the plan must have
 *                 the same grad_dtype).
 *   PARO_TENSORS: contrib[q] -> DEVICE array of n_tensors DEVICE pointers, the
 *                 q-th rank's full gradient of each tensor (dtype per tensor as
 *                 planned; each naturally aligned - 8-byte (2-byte dtypes) or
 *                 16-byte (fp32) alignment of the data a rank contributes to
 *                 the range lets the kernels use vector loads, anything less
 *                 costs element loads; empty tensors may be NULL).
 * grad_out, p, m, v: DEVICE fp32 arrays over the update range, 16-byte aligned.
 * PARO_EALIGN for a misaligned pointer, PARO_EINVAL for a NULL one. */

/* grad_out[e] = the P contributions to element e added in the fold order of
 * e's chunk; *sumsq_out (DEVICE double, overwritten; NULL = not wanted) = sum of grad_out[e]^2
 * over the rank's OWN chunk only, so that adding the ranks' values counts every
 * element of the model once. */
int paro_reduce_shard(paro_plan_t *plan, int rank, const void *const *contrib, int layout,
                      float *grad_out, double *sumsq_out, void *stream);

/* Adam over the update range, in place on p, m, v.  total_sumsq: DEVICE double
 * = the sum over all ranks of their sumsq_out (read when hp->max_norm > 0; may
 * be NULL otherwise).  dst_base: NULL, or the buffer of paro_pack_params - then
 * the updated parameters are also packed, in the same sweep. */
int paro_adam_shard(paro_plan_t *plan, int rank, const paro_adam_t *hp, const float *grad,
                    const double *total_sumsq, float *p, float *m, float *v, uint16_t *dst_base,
                    void *stream);

/* dst_base[slot_off + e] = p[e] rounded to nearest even in the plan's pack_dtype
 * (bf16, or fp16 with overflow to infinity), over the update range.  dst_base: DEVICE uint16 array of dst_len elements (paro_pack_slot),
 * 16-byte aligned. */
int paro_pack_params(paro_plan_t *plan, int rank, const float *p, uint16_t *dst_base, void *stream);

/* reduce + clip + Adam + pack.  With hp->max_norm > 0 or hp->skip_nonfinite it
 * is paro_reduce_shard followed by paro_adam_shard with dst_base: sweep 1 writes
 * the reduced gradient to grad_scratch (DEVICE fp32 over the update range) and a
 * sum of squares to *sumsq_scratch (DEVICE double); sweep 2 takes that sum as the
 * total, clips, updates and packs.  The sum is the norm this rank can form on its
 * own (the cross-rank sum a deployment inserts between the sweeps has no peer
 * here): over the rank's whole UPDATE RANGE - its own chunk when the optimizer
 * state is sharded over all ranks ('G': the same value paro_reduce_shard gives);
 * every chunk of its block or of the model when it is sharded inside the group
 * only or not at all ('I', 'N': one sum per chunk, added in chunk order), so that
 * every replica of a range clips, or skips an overflowed step, alike - and with
 * 'N' it is the model's true norm.  With neither clipping nor skipping one sweep
 * does everything, the gradient is never stored, and both scratch pointers may
 * be NULL. */
int paro_step_fused(paro_plan_t *plan, int rank, const void *const *contrib, int layout,
                    const paro_adam_t *hp, float *grad_scratch, double *sumsq_scratch, float *p,
                    float *m, float *v, uint16_t *dst_base, void *stream);

/* paro_step_fused for callers that cannot allocate device memory at the call: code
 * under HIP graph capture whose first call would fall inside the capture, tight
 * serving or training loops and harnesses that forbid hipMalloc.  Same work, same
 * results, same buffer arguments as paro_step_fused with layout PARO_CHUNK, but the
 * per-block partial sums of the norm go to a static device array inside the library
 * (32 MiB + 16 KiB, held by every GPU the library runs on until the process ends)
 * instead of the plan's device allocation: this call never allocates or frees
 * device memory, never synchronises, and does not touch the plan's device tables
 * (the plan may never have seen a device call).  Limits: chunk layout only; no
 * weight-decay mask (PARO_EINVAL: it needs the plan's device tables); a chunk of
 * at most PARO_STATIC_MAX_CHUNK elements (PARO_ERANGE beyond).  All calls on one
 * GPU share that GPU's array, whatever their plan or stream: calls that overlap in
 * time on one GPU race on it - serialise them on one stream.  Nothing in the array
 * has to start at zero (every launch overwrites what it later reads). */
enum { PARO_STATIC_MAX_CHUNK = 1 << 30 };
int paro_step_fused_static(const paro_plan_t *plan, int rank, const void *const *contrib,
                           const paro_adam_t *hp, float *grad_scratch, double *sumsq_scratch, float *p,
                           float *m, float *v, uint16_t *dst_base, void *stream);

/* ---- the steps around the Update stage: ring hops and scheduled transfers -----
 * One hop of a reduce-scatter ring (Sec. 3.4: each GPU passes the partial sum on
 * to the next one after adding its own contribution), and the same operation as
 * micro-batch gradient accumulation (Sec. 3.3: the gradients of each
 * micro-batch are reduce-scattered inside the group and accumulated; one
 * inter-group reduce-scatter follows the last micro-batch):
 *   out[e] = partial_in[e] + local[e]   for 0 <= e < n, one fp32 add per element.
 * partial_in and local are DEVICE arrays of dtype in_dtype / local_dtype
 * (PARO_BF16, PARO_F32 or PARO_F16), out is DEVICE fp32 and may be the same array as an
 * fp32 partial_in or local (in-place accumulation).  All 16-byte aligned. */
int paro_ring_hop(paro_plan_t *plan, const void *partial_in, int in_dtype, const void *local, int local_dtype,
                  float *out, int64_t n, void *stream);

/* The receive side of one step of rank `rank` in a simulated collective: for every
 * entry of paro_schedule(plan, rank, sched, collective) with the given (phase,
 * ring, step),
 *   PARO_RS: bufs[rank][recv range] = bufs[recv_from][same range] + bufs[rank][recv range]   (fp32)
 *   PARO_AG: bufs[rank][recv range] = bufs[recv_from][same range]                            (bf16)
 * bufs: HOST array of P DEVICE pointers, rank q's padded flat buffer of
 * paro_padded_total elements (fp32 working buffers for a reduce-scatter, bf16
 * parameter buffers for an all-gather).  Playing every rank's steps in schedule
 * order on one stream (inside a phase: ring 0 before ring 1) reproduces the
 * collective: after a reduce-scatter rank r's own chunk of bufs[r] holds the sum
 * in the fold order of paro_fold_order; after an all-gather every buffer is
 * complete.  Returns the number of elements received (>= 0) or an error. */
int64_t paro_collective_step(paro_plan_t *plan, int rank, int sched, int collective, int phase, int ring,
                             int step, void *const *bufs, void *stream);

/* ---- cost model (host only): the paper's Tables 1-3 and Eq. 1 as a function ------
 * Memory per GPU in bytes (Table 2: 2*Psi/d, 2*Psi'/d, K*Psi'/d with d = 1, M, N for
 * N / I / G) and communication volume in ELEMENTS, summed over all GPUs, for one
 * mini-batch of s micro-batches (Table 3), split into intra-group and inter-group
 * traffic.  sched picks the global collective: PARO_RING gives the flat-ring rows
 * (ZeRO-1/2/3), PARO_HORING (or PARO_HRING, same volumes) the HO-Ring rows (PaRO-IGG
 * backward reduce-scatter, PaRO-NIG update all-gather); PARO_SCHED_DEFAULT = HO-Ring when
 * 1 < M < N.  Rows the paper prints (NNG, NGG, GGG, III, IGG, IIG, NIG) are reproduced as
 * printed, including the all-reduce of ZeRO-1 and MiCS; the other strategies follow the
 * same rules (Sec. 3.1.1) and are marked derived = 1.  recommended[c] is Table 1's mark for
 * column c (0: Psi' = Psi, 1: Psi' >= Psi/6, 2: Psi' < Psi/6, 3: PEFT). */
typedef struct {
    double mem_param, mem_grad, mem_os;
    double fwd_ag_intra, fwd_ag_inter;      /* forward all-gather of parameters */
    double bwd_ag_intra, bwd_ag_inter;      /* backward all-gather of parameters */
    double bwd_rs_intra, bwd_rs_inter;      /* backward reduce-scatter of gradients */
    double upd_g_intra, upd_g_inter;        /* update stage: reduce-scatter / all-reduce of gradients */
    double upd_ag_intra, upd_ag_inter;      /* update stage: all-gather of parameters */
    int32_t recommended[4];
    int32_t derived;
} paro_cost_t;

/* N GPUs in groups of M (M divides N), s >= 1 micro-batches, K bytes of optimizer state
 * per trainable parameter (12 for mixed-precision Adam, Sec. 3.1.2).  PARO_ESTRATEGY for a
 * strategy outside Table 1, PARO_EINVAL for bad numbers. */
int paro_cost(const char *strategy, double psi, double psi_trainable, int N, int M, int s, int K, int sched,
              paro_cost_t *out);

/* Eq. 1: elements a GPU no longer sends when the global reduce-scatter of every
 * micro-batch is replaced by an intra-group one per micro-batch plus one inter-group one
 * per mini-batch: Psi * (s - 1) * (g - 1) / N. */
double paro_two_step_saving(double psi, int N, int M, int s);

/* text of the calling thread's last error ("" if none); valid until that
 * thread's next failing call */
const char *paro_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PARO_H */
