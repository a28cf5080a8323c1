"""CPU oracle, part 1: sharding plan, collective schedules and their literal
simulation.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package; only tests/, the smoke check and the benchmark's cpu_baseline leg do.
It shares no code with the HIP library.

Notation.  The paper (Sec. 3.1) writes N for the number of GPUs, M for the
GPUs per group, g = N / M for the number of groups, and uses the letters
P / G / OS for parameter / gradient / optimizer state.  This code follows the
benchmark's naming instead: ``P`` = number of ranks (paper N), ``G`` = ranks per
group (paper M), ``g = P // G`` groups.  A strategy is three letters ordered
parameter / gradient / optimizer-state, each N (no sharding), I (intra-group)
or G (global) as in Table 1.

Readings of the paper taken here (each is pinned by a test, or declared
unpinned):
  * consecutive ranks share a group (Table 3's flat-ring rows count exactly g
    inter-group links out of N, true only for consecutive grouping);
  * every ring sends to the next index and receives from the previous one
    (Sec. 3.4, "to the next GPU").  The direction is a convention: the mirror
    image only permutes the order of the additions.  PARITY UNPINNED by the
    paper.
  * chunk <-> owner map: nested (see ``chunk_of_rank``) so that the range a
    rank holds under global sharding lies inside the range it holds under
    intra-group sharding - what the inter-group reduce-scatter of an
    intra-group shard (Sec. 3.2, PaRO-IIG) and the inter-group all-gather
    completing an intra-group parameter shard (PaRO-IGG) need;
  * H-Ring (Sec. 3.4 gives no order): reduce-scatter runs the intra-group ring
    first and the inter-group ring second, all-gather the reverse;
  * HO-Ring reduce-scatter (only the all-gather is described in Sec. 3.4) is
    the all-gather run backwards in time.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

RING, HRING, HORING = 0, 1, 2
RS, AG = 0, 1
_FINENESS = {"N": 0, "I": 1, "G": 2}          # Sec. 3.1.1: N coarser than I coarser than G


# ---------------------------------------------------------------- strategies
def strategy_legal(s: str) -> bool:
    """Principle 1 (Sec. 3.1.3): the optimizer state is sharded at least as
    finely as the parameters and as the gradients."""
    if len(s) != 3 or any(c not in _FINENESS for c in s):
        return False
    fp, fg, fo = (_FINENESS[c] for c in s)
    return fo >= fp and fo >= fg


def all_legal_strategies() -> List[str]:
    return [a + b + c for a in "NIG" for b in "NIG" for c in "NIG" if strategy_legal(a + b + c)]


# -------------------------------------------------------------------- layout
@dataclass(frozen=True)
class Layout:
    P: int
    G: int
    sizes: Tuple[int, ...]
    align: int
    offsets: Tuple[int, ...]     # flat start of each tensor, plus the total at the end
    total: int                   # Psi: number of real elements
    L: int                       # chunk length (elements); padded total = P * L

    @property
    def g(self) -> int:
        return self.P // self.G


def layout(P: int, G: int, sizes: Sequence[int], align: int = 8) -> Layout:
    """Tensors are laid end to end (no per-tensor padding); the flat buffer is
    cut into P equal chunks of L = align * ceil(ceil(Psi / P) / align) elements
    (Table 2: a globally sharded state is Psi / N per GPU); elements past Psi
    are padding."""
    if P < 1 or G < 1 or P % G or align < 1 or len(sizes) < 1 or any(s < 0 for s in sizes):
        raise ValueError("bad cluster shape or sizes")
    off = [0]
    for s in sizes:
        off.append(off[-1] + int(s))
    total = off[-1]
    per = -(-total // P)
    L = max(align, -(-per // align) * align)
    return Layout(P, G, tuple(int(s) for s in sizes), align, tuple(off), total, L)


def group_of(rank: int, G: int) -> Tuple[int, int]:
    """(group index j, local index i) of a rank: consecutive ranks share a group."""
    return rank // G, rank % G


def chunk_of_rank(rank: int, P: int, G: int) -> int:
    """Chunk owned by a rank under global sharding.  The flat buffer is first
    cut into G blocks (block i belongs to local index i of every group: the
    intra-group shard of size Psi / M), and block i is cut into g chunks, the
    j-th of which belongs to group j."""
    g = P // G
    j, i = group_of(rank, G)
    return i * g + j


def owner_of_chunk(chunk: int, P: int, G: int) -> int:
    g = P // G
    return (chunk % g) * G + chunk // g


def state_range(lay: Layout, rank: int, letter: str) -> Tuple[int, int]:
    """(begin, length), in elements of the padded flat buffer, of what a rank
    holds of a state sharded with the given letter (Sec. 3.1.1)."""
    j, i = group_of(rank, lay.G)
    if letter == "G":
        return chunk_of_rank(rank, lay.P, lay.G) * lay.L, lay.L
    if letter == "I":
        return i * lay.g * lay.L, lay.g * lay.L
    if letter == "N":
        return 0, lay.P * lay.L
    raise ValueError(letter)


def segments(lay: Layout, begin: int, length: int) -> List[Tuple[int, int, int, int]]:
    """Pieces of tensors inside flat [begin, begin+length): tuples
    (tensor, offset inside the tensor, offset inside the range, length).
    Empty tensors and padding produce no piece."""
    out = []
    end = begin + length
    for t, size in enumerate(lay.sizes):
        lo = max(begin, lay.offsets[t])
        hi = min(end, lay.offsets[t] + size)
        if hi > lo:
            out.append((t, lo - lay.offsets[t], lo - begin, hi - lo))
    return out


def pack_slot(lay: Layout, rank: int, strategy: str) -> Tuple[int, int, int]:
    """(length of the low-precision parameter buffer the rank holds, offset of
    its updated range inside it, length of that range).  The updated range is
    the optimizer-state range; the buffer is the parameter-state range, which
    contains it under Principle 1."""
    pb, pl = state_range(lay, rank, strategy[0])
    ob, ol = state_range(lay, rank, strategy[2])
    assert pb <= ob and ob + ol <= pb + pl
    return pl, ob - pb, ol


# ---------------------------------------------------------------- fold order
def default_sched(P: int, G: int) -> int:
    return HORING if 1 < G < P else RING


def fold_order(P: int, G: int, sched: int, chunk: int) -> Tuple[List[int], int]:
    """Order in which the P contributions to a chunk are added by the
    reduce-scatter that delivers it to its owner, as (ranks, group_len):
    consecutive runs of group_len ranks are summed left to right into a partial,
    and the partials are then summed left to right.

    Flat ring (Sec. 3.4): the partial sum starts at the owner's successor and
    travels round the ring; the owner adds its own contribution last.
    H-Ring / HO-Ring: inside every group the ring over the local indices ends at
    the owner's local index; the group partials then travel round the
    inter-group ring, which ends at the owner's group.  HO-Ring differs from
    H-Ring only in which transfers overlap in time (Sec. 3.4), so the
    additions are the same."""
    g = P // G
    owner = owner_of_chunk(chunk, P, G)
    if sched == RING:
        return [(owner + k) % P for k in range(1, P + 1)], P
    if sched not in (HRING, HORING):
        raise ValueError(sched)
    j, i = group_of(owner, G)
    ranks = []
    for k in range(1, g + 1):
        jj = (j + k) % g
        ranks += [jj * G + (i + l) % G for l in range(1, G + 1)]
    return ranks, G


# ------------------------------------------------------------------ schedules
@dataclass(frozen=True)
class Msg:
    phase: int      # 1 or 2
    step: int       # 1-based inside (phase, ring)
    ring: int       # 0 intra-group ring, 1 inter-group ring (flat ring: 0)
    send_to: int
    recv_from: int
    send_off: int   # element offsets into the padded flat buffer
    send_len: int
    recv_off: int
    recv_len: int


def _ranges_of_chunks(chunks: Sequence[int], L: int) -> List[Tuple[int, int]]:
    """Sorted chunk indices -> maximal contiguous (offset, length) ranges."""
    out: List[Tuple[int, int]] = []
    for c in sorted(chunks):
        if out and out[-1][0] + out[-1][1] == c * L:
            out[-1] = (out[-1][0], out[-1][1] + L)
        else:
            out.append((c * L, L))
    return out


def _emit(out, phase, step, ring, to, frm, send_chunks, recv_chunks, L):
    s = _ranges_of_chunks(send_chunks, L)
    r = _ranges_of_chunks(recv_chunks, L)
    assert len(s) == len(r)
    for (so, sl), (ro, rl) in zip(s, r):
        out.append(Msg(phase, step, ring, to, frm, so, sl, ro, rl))


def schedule(lay: Layout, sched: int, rank: int, collective: int) -> List[Msg]:
    """Every message a rank sends / receives, one entry per contiguous range.
    A reduce-scatter message carries partial sums that the receiver adds to
    what it holds for the same range; an all-gather message is stored as is.
    Entries with equal (phase, ring, step) form one logical message."""
    P, G, L = lay.P, lay.G, lay.L
    g = P // G
    j, i = group_of(rank, G)
    out: List[Msg] = []
    if sched == RING:
        nxt, prv = (rank + 1) % P, (rank - 1) % P
        for k in range(1, P):
            if collective == RS:
                sc = chunk_of_rank((rank - k) % P, P, G)
                rc = chunk_of_rank((rank - k - 1) % P, P, G)
            else:
                sc = chunk_of_rank((rank - k + 1) % P, P, G)
                rc = chunk_of_rank((rank - k) % P, P, G)
            _emit(out, 1, k, 0, nxt, prv, [sc], [rc], L)
        return out

    intra_to, intra_from = j * G + (i + 1) % G, j * G + (i - 1) % G
    inter_to, inter_from = ((j + 1) % g) * G + i, ((j - 1) % g) * G + i
    block = lambda b: [b * g + jj for jj in range(g)]                 # noqa: E731
    others = lambda b: [b * g + jj for jj in range(g) if jj != j]     # noqa: E731

    if sched == HRING and collective == RS:
        for k in range(1, G):                       # intra ring, whole blocks
            _emit(out, 1, k, 0, intra_to, intra_from, block((i - k) % G), block((i - k - 1) % G), L)
        for k in range(1, g):                       # inter ring, one chunk
            _emit(out, 2, k, 1, inter_to, inter_from,
                  [i * g + (j - k) % g], [i * g + (j - k - 1) % g], L)
    elif sched == HRING and collective == AG:
        for k in range(1, g):
            _emit(out, 1, k, 1, inter_to, inter_from,
                  [i * g + (j - k + 1) % g], [i * g + (j - k) % g], L)
        for k in range(1, G):
            _emit(out, 2, k, 0, intra_to, intra_from, block((i - k + 1) % G), block((i - k) % G), L)
    elif sched == HORING and collective == AG:
        # phase 1: the rank's own chunk goes round both rings at once
        for k in range(1, G):
            _emit(out, 1, k, 0, intra_to, intra_from,
                  [((i - k + 1) % G) * g + j], [((i - k) % G) * g + j], L)
        for k in range(1, g):
            _emit(out, 1, k, 1, inter_to, inter_from,
                  [i * g + (j - k + 1) % g], [i * g + (j - k) % g], L)
        # phase 2: what the inter-group ring delivered goes round the group
        if g > 1:
            for k in range(1, G):
                _emit(out, 2, k, 0, intra_to, intra_from,
                      others((i - k + 1) % G), others((i - k) % G), L)
    elif sched == HORING and collective == RS:
        # phase 1: inside each group, reduce the chunks owned by other groups
        if g > 1:
            for k in range(1, G):
                _emit(out, 1, k, 0, intra_to, intra_from,
                      others((i - k) % G), others((i - k - 1) % G), L)
        # phase 2: inter-group ring on the group partials, while the intra-group
        # ring reduces the chunks this group owns
        for k in range(1, G):
            _emit(out, 2, k, 0, intra_to, intra_from,
                  [((i - k) % G) * g + j], [((i - k - 1) % G) * g + j], L)
        for k in range(1, g):
            _emit(out, 2, k, 1, inter_to, inter_from,
                  [i * g + (j - k) % g], [i * g + (j - k - 1) % g], L)
    else:
        raise ValueError((sched, collective))
    return out


def simulate(lay: Layout, sched: int, collective: int, bufs: List[np.ndarray], phases=None) -> None:
    """Literal message passing over P simulated ranks, in place.  bufs[r] is
    rank r's padded flat fp32 buffer (P*L elements).  Reduce-scatter: bufs[r]
    starts as rank r's own gradient and ends with the fully reduced chunk of
    rank r in its chunk range.  All-gather: bufs[r] starts with rank r's chunk
    in place and ends complete.

    Rings that overlap in time inside one phase touch disjoint ranges, except
    for the last inter-group step of the HO-Ring reduce-scatter, whose received
    partial is added to the group's own partial of the same chunk; that add
    needs the intra-group ring of the phase to be finished, so a phase is played
    ring 0 first, then ring 1.  phases: play only these phases (e.g. {1} of an
    H-Ring reduce-scatter = the intra-group reduce-scatter alone)."""
    P = lay.P
    table = [schedule(lay, sched, r, collective) for r in range(P)]
    keys = sorted({(m.phase, m.ring, m.step) for ms in table for m in ms
                   if phases is None or m.phase in phases})
    for key in keys:
        sel = [[m for m in table[r] if (m.phase, m.ring, m.step) == key] for r in range(P)]
        wire = {}
        for r in range(P):                          # everybody sends first ...
            for n, m in enumerate(sel[r]):
                wire[(r, m.send_to, n)] = bufs[r][m.send_off:m.send_off + m.send_len].copy()
        for r in range(P):                          # ... then everybody receives
            for n, m in enumerate(sel[r]):
                data = wire.pop((m.recv_from, r, n))
                assert data.shape[0] == m.recv_len
                dst = bufs[r][m.recv_off:m.recv_off + m.recv_len]
                if collective == RS:
                    dst[:] = data + dst             # fp32 + fp32, one IEEE add per element
                else:
                    dst[:] = data
        assert not wire, "a message was sent that nobody received"


def volumes(lay: Layout, sched: int, rank: int, collective: int) -> Tuple[int, int]:
    """(intra-group, inter-group) elements sent by a rank.  For the flat ring a
    link is inter-group when it joins ranks of different groups."""
    intra = inter = 0
    for m in schedule(lay, sched, rank, collective):
        crosses = group_of(m.send_to, lay.G)[0] != group_of(rank, lay.G)[0]
        if crosses:
            inter += m.send_len
        else:
            intra += m.send_len
    return intra, inter


def accumulate_two_step(lay: Layout, micro_batches: List[List[np.ndarray]]) -> List[np.ndarray]:
    """Gradient accumulation with the grouped two-step reduce-scatter (Sec. 3.3,
    PaRO-IIG / NIG): micro_batches[b][r] is rank r's padded flat fp32 gradient of
    micro-batch b.  Every micro-batch is reduce-scattered inside the groups (the
    intra-group ring of the H-Ring schedule); each rank adds the block it receives
    to its persistent gradient shard (the first micro-batch is stored, the later
    ones are added, in order); after the last micro-batch one inter-group
    reduce-scatter runs on the accumulated blocks.  Returns, per rank, the reduced
    chunk it owns."""
    P, L = lay.P, lay.L
    acc: List[np.ndarray] = []
    for b, grads in enumerate(micro_batches):
        bufs = [g.copy() for g in grads]
        simulate(lay, HRING, RS, bufs, phases={1})
        for r in range(P):
            lo, n = state_range(lay, r, "I")
            if b == 0:
                acc.append(bufs[r][lo:lo + n].copy())
            else:
                acc[r] = acc[r] + bufs[r][lo:lo + n]          # fp32 + fp32
    work = []
    for r in range(P):
        w = np.zeros(P * L, np.float32)
        lo, n = state_range(lay, r, "I")
        w[lo:lo + n] = acc[r]
        work.append(w)
    simulate(lay, HRING, RS, work, phases={2})
    out = []
    for r in range(P):
        c = chunk_of_rank(r, P, lay.G)
        out.append(work[r][c * L:(c + 1) * L].copy())
    return out
