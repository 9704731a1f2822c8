"""Plain CPU oracle: reshard training state by gathering every source shard into
the full logical tensors and re-splitting them for the target world.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.  No blocking, no
fusion, no descriptor planning: this file is the *definition* of the result.

What the paper fixes (LiveR, Section 4.6 and Appendix A.2):
  * the state is a set of logical tensors plus a sharding specification that is
    independent of rank numbering (Abstract Resource View, Section 4.6.1);
  * a reshard is correct iff the union of all shards is the same before and
    after (Appendix A.2.1, Eq. 1) and every element of the global state appears
    exactly once in the new configuration (Section 4.6, constraint 1);
  * the paper's own check gathers the global tensors before and after and
    compares them element by element, with deviation exactly zero (Section 6.6).
So the result has a plain definition: gather, then split.  This file writes that
definition out.

What the paper does NOT fix, and the readings taken here (each is a convention of
Megatron-style mixed-parallel training, stated so a reader can check it by eye):
  R1  logical tensors are stored row-major as [out_features, in_features].
  R2  column-parallel linears (q/k/v, gate/up, embeddings, lm_head) are split in
      contiguous blocks of dim 0; row-parallel linears (o, down) in contiguous
      blocks of dim 1; norms, position embeddings and the biases of row-parallel
      linears are replicated on every TP rank.
  R3  q, k, v live in ONE fused physical parameter per rank, grouped per
      kv-head group g: [q rows of the group ; k rows of g ; v rows of g], groups
      in ascending order (MHA: per head [q_h; k_h; v_h]).
  R3b if TP > n_kv (TP a multiple of n_kv), kv group g is REPLICATED on the
      r = TP/n_kv ranks g*r .. g*r+r-1; rank g*r+j holds the j-th r-th of the
      group's q rows, then all k rows of g, then all v rows of g.  A gather reads
      k and v from the rank with j = 0.
  R4  with a gated FFN, gate and up live in one physical parameter per rank as
      [gate rows of this rank ; up rows of this rank].
  R5  a (tp, pp) rank's parameters are flattened row-major and packed back to
      back, in forward order, into one flat buffer; the bf16 and fp32 buffers
      use the same element offsets.
  R5b with bucket_elems = B > 0 the flat buffer is a sequence of BUCKETS (as a
      distributed optimizer's gradient / parameter buffer is): parameters are
      appended in order and a bucket closes after the parameter that brings it
      to >= B elements; the last bucket takes the rest.  B = 0: one bucket.
  R6  every bucket is zero-padded to a multiple of DP*pad_multiple elements (the
      flat buffer then has N_pad elements).  PARAM (bf16) is a full N_pad copy on
      every DP rank; MASTER / ADAM_M / ADAM_V (fp32) are split evenly PER BUCKET:
      DP rank d owns the d-th DP-th of every bucket and its buffer is the
      concatenation of those slices (one bucket: [d*S, (d+1)*S), S = N_pad/DP).
  R7  where a value exists more than once in the source world, the copy that is
      read is the one with the lowest coordinate (dp=0, tp=0, first stage).
  R8  with tied embeddings and PP>1 the last stage holds a second physical copy
      of the word embedding (same TP split) after the final norm.
  R9  stage pp owns layers [pp*L/PP, (pp+1)*L/PP).  With an interleaved schedule
      (vpp > 1 model chunks per stage, as in the interleaved 1F1B the paper's
      Section 4.7 mentions) the layers are cut into PP*vpp groups of c layers and
      stage pp owns groups pp, pp+PP, pp+2*PP, ...; they sit in its flat buffer in
      that order.  Embeddings stay on stage 0, final norm / head on stage PP-1.
  R9c uneven split: pp_first / pp_last give the layer count of the first / last
      stage (the stages that also hold the embedding / the head); the other stages
      share the remaining layers evenly.
  R10 fp32 -> bf16 is round-to-nearest-even on the upper 16 bits; NaN keeps sign
      and upper payload and gets the quiet bit.
  R11b with vocab_multiple = m > 0 the vocabulary dimension of embed.word / lm_head
      is padded per world to V_p = ceil(V / (m*TP)) * m*TP rows (what Megatron's
      make-vocab-size-divisible-by does), so V_p changes with TP.  Every rank
      holds V_p/TP rows; rows with global index >= V are padding: written +0 in
      the target, never read from the source.  Logical tensors keep V rows.
  R12 buffer-table index of a rank is tp + TP*(dp + DP*pp).
  R13 mixture of experts (n_experts = E > 0; Appendix A.2.3 says the view extends
      along the expert dimension): every layer's FFN becomes a router
      (router.w [E, H], a dense parameter replicated over TP) plus E experts with
      their own gate/up/down weights.  With expert parallelism EP (EP divides DP
      and E) DP rank d belongs to expert-parallel index d % EP and holds experts
      [ep*E/EP, (ep+1)*E/EP) of its stage, each split over TP like a dense FFN.
      Expert parameters form a SECOND flat buffer per rank (kinds 4..7), laid out
      layer by layer, expert by expert (fc1, fc2), with the same bucket / padding
      rules, but replicated and optimizer-sharded over the DP/EP ranks that hold
      the same experts (d = ep, ep + EP, ...), in that order; the copy that is read
      is the first of them.  Dense parameters (kinds 0..3) are unaffected by EP.

All data are handled as raw bit patterns (uint16 for bf16, uint32 for fp32):
resharding moves bits, it never interprets them (except rne_bf16).

Pins (tests/test_oracle_*.py): closed-form sizes, index-encoded tensors against
formulas typed out in the test, brute-force per-element ownership on tiny models,
identity / round trip / composition, the TP4->TP8 worked example of Section
4.6.1, and torch's CPU float->bfloat16 conversion for rne_bf16.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, Iterable, List, Optional, Tuple

import numpy as np

PARAM, MASTER, ADAM_M, ADAM_V = 0, 1, 2, 3
KINDS = (PARAM, MASTER, ADAM_M, ADAM_V)
# R13: the expert parameters of a mixture-of-experts model live in buffers of their own, kinds 4..7
EXPERT_PARAM, EXPERT_MASTER, EXPERT_ADAM_M, EXPERT_ADAM_V = 4, 5, 6, 7
EXPERT_KINDS = (EXPERT_PARAM, EXPERT_MASTER, EXPERT_ADAM_M, EXPERT_ADAM_V)
WORD = {k: (np.uint16 if k % 4 == 0 else np.uint32) for k in range(8)}


@dataclass(frozen=True)
class ModelSpec:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    ffn: int
    vocab: int
    max_pos: int = 0          # 0: no learned position embedding
    glu: bool = False         # gated FFN (SwiGLU): gate + up
    norm_bias: bool = False   # LayerNorm (with bias) instead of RMSNorm
    linear_bias: bool = False
    tied_embed: bool = False  # no lm_head; output layer reuses embed.word
    n_experts: int = 0        # R13: > 0 = mixture of experts (ffn = hidden size of ONE expert's FFN)


@dataclass(frozen=True)
class Layout:
    tp: int
    pp: int
    dp: int
    pad_multiple: int = 128
    vpp: int = 1              # R9b: model chunks per stage (interleaved pipeline schedule)
    vocab_multiple: int = 0   # R11b: pad the vocabulary to a multiple of vocab_multiple*TP rows; 0 = no padding
    pp_first: int = 0         # R9c: layers on the first / last stage (0 = even share); the other
    pp_last: int = 0          #      stages split the remaining layers evenly
    bucket_elems: int = 0     # R5b: flat buffer cut into buckets of at least this many elements (0 = one bucket)
    ep: int = 1               # R13: expert-parallel size (divides DP and n_experts)

    @property
    def n_ranks(self) -> int:
        return self.tp * self.pp * self.dp

    def rank(self, tp: int, pp: int, dp: int) -> int:       # R12
        return tp + self.tp * (dp + self.dp * pp)


def _kv_split_ok(spec: ModelSpec, tp: int) -> bool:
    """kv groups split evenly over TP, or (R3b) each kv group replicated over TP/n_kv ranks."""
    if spec.n_kv_heads % tp == 0:
        return True
    r = tp // spec.n_kv_heads
    return tp % spec.n_kv_heads == 0 and (spec.n_q_heads // spec.n_kv_heads) % r == 0


def padded_vocab(spec: ModelSpec, lay: Layout) -> int:       # R11b
    if not lay.vocab_multiple:
        return spec.vocab
    q = lay.vocab_multiple * lay.tp
    return -(-spec.vocab // q) * q


def check_supported(spec: ModelSpec, lay: Layout) -> None:
    ok = (lay.vpp >= 1 and _stage_counts(spec, lay) is not None and spec.hidden % spec.n_q_heads == 0
          and spec.n_q_heads % spec.n_kv_heads == 0 and _kv_split_ok(spec, lay.tp)
          and spec.ffn % lay.tp == 0 and (spec.vocab % lay.tp == 0 or lay.vocab_multiple > 0)
          and lay.vocab_multiple >= 0 and lay.bucket_elems >= 0
          and min(lay.tp, lay.pp, lay.dp, lay.pad_multiple, lay.ep) >= 1
          and ((lay.dp % lay.ep == 0 and spec.n_experts % lay.ep == 0) if spec.n_experts else lay.ep == 1))
    if not ok:
        raise ValueError(f"unsupported combination {spec} {lay}")


# --------------------------------------------------------------------------- R1
def logical_tensors(spec: ModelSpec) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape of every logical tensor, in forward order."""
    H, F, V = spec.hidden, spec.ffn, spec.vocab
    hd = H // spec.n_q_heads
    Q, KV = spec.n_q_heads * hd, spec.n_kv_heads * hd
    t: Dict[str, Tuple[int, ...]] = {"embed.word": (V, H)}
    if spec.max_pos:
        t["embed.pos"] = (spec.max_pos, H)
    for l in range(spec.n_layers):
        p = f"L{l}."
        t[p + "ln1.w"] = (H,)
        if spec.norm_bias:
            t[p + "ln1.b"] = (H,)
        t[p + "q.w"], t[p + "k.w"], t[p + "v.w"] = (Q, H), (KV, H), (KV, H)
        if spec.linear_bias:
            t[p + "q.b"], t[p + "k.b"], t[p + "v.b"] = (Q,), (KV,), (KV,)
        t[p + "o.w"] = (H, Q)
        if spec.linear_bias:
            t[p + "o.b"] = (H,)
        t[p + "ln2.w"] = (H,)
        if spec.norm_bias:
            t[p + "ln2.b"] = (H,)
        if spec.n_experts:                           # R13: router + one FFN per expert
            t[p + "router.w"] = (spec.n_experts, H)
        for q in ([p + f"x{e}." for e in range(spec.n_experts)] if spec.n_experts else [p]):
            if spec.glu:
                t[q + "gate.w"] = (F, H)
            t[q + "up.w"] = (F, H)
            if spec.linear_bias:
                if spec.glu:
                    t[q + "gate.b"] = (F,)
                t[q + "up.b"] = (F,)
            t[q + "down.w"] = (H, F)
            if spec.linear_bias:
                t[q + "down.b"] = (H,)
    t["final_norm.w"] = (H,)
    if spec.norm_bias:
        t["final_norm.b"] = (H,)
    if not spec.tied_embed:
        t["lm_head.w"] = (V, H)
    return t


# ------------------------------------------------------------- physical params
@dataclass(frozen=True)
class Block:
    """local[loc] holds logical[name][idx] (tuples of slices).  canonical: may a
    gather read this block from this rank (R7)?"""
    name: str
    idx: Tuple[slice, ...]
    loc: Tuple[slice, ...]
    canonical: bool = True


@dataclass
class PhysParam:
    name: str
    shape: Tuple[int, ...]
    blocks: List[Block]
    canonical: bool           # R7: is this rank's copy the one a gather reads?
    offset: int = 0           # element offset in the (tp, pp) flat buffer

    @property
    def size(self) -> int:
        return int(np.prod(self.shape))


@dataclass
class StageView:
    params: List[PhysParam]
    n_local: int              # end of the last parameter (interior bucket padding included)
    n_pad: int
    S: int                    # elements of one DP rank's fp32 buffers = N_pad / len(dp_ranks)
    buckets: List[Tuple[int, int]] = field(default_factory=list)   # (start, padded size) in flat coordinates
    dp_ranks: List[int] = field(default_factory=list)   # DP coordinates sharing this flat buffer, in slice order


def _rows(a: int, b: int) -> Tuple[slice, ...]:
    return (slice(a, b),)


def _cols(a: int, b: int) -> Tuple[slice, ...]:
    return (slice(None), slice(a, b))


_ALL: Tuple[slice, ...] = (slice(None),)


def _stage_counts(spec: ModelSpec, lay: Layout) -> Optional[List[int]]:
    """Layers per stage, or None if the split is not possible (R9, R9c)."""
    L, PP = spec.n_layers, lay.pp
    if lay.pp_first < 0 or lay.pp_last < 0 or min(lay.tp, lay.pp, lay.dp) < 1:
        return None
    if not lay.pp_first and not lay.pp_last:
        return [L // PP] * PP if L % (PP * lay.vpp) == 0 else None
    fixed = (1 if lay.pp_first else 0) + (1 if lay.pp_last else 0)
    rest, others = L - lay.pp_first - lay.pp_last, PP - fixed
    if lay.vpp != 1 or others < 0 or rest < 0 or (others == 0 and rest != 0) or (others > 0 and rest % others):
        return None
    counts = [rest // others if others else 0] * PP
    if lay.pp_first:
        counts[0] = lay.pp_first
    if lay.pp_last:
        counts[-1] = lay.pp_last
    return counts if min(counts) >= 1 else None


def stage_layers(spec: ModelSpec, lay: Layout, pp: int) -> List[int]:
    """Layers held by stage pp, in the order they sit in its flat buffer (R9)."""
    if lay.pp_first or lay.pp_last:                  # R9c: uneven first / last stage
        counts = _stage_counts(spec, lay)
        return list(range(sum(counts[:pp]), sum(counts[:pp + 1])))
    c = spec.n_layers // (lay.pp * lay.vpp)          # layers per model chunk
    return [l for v in range(lay.vpp) for l in range((v * lay.pp + pp) * c, (v * lay.pp + pp + 1) * c)]


def stage_view(spec: ModelSpec, lay: Layout, tp: int, pp: int, ep: Optional[int] = None) -> StageView:
    """Ordered physical parameters of rank column (tp, pp) -- R2..R5, R8, R9.
    ep = None: the dense parameters (kinds 0..3).  ep = e: the expert parameters (kinds 4..7) held by the
    ranks of expert-parallel index e (R13)."""
    check_supported(spec, lay)
    shapes = logical_tensors(spec)
    TP = lay.tp
    hd = spec.hidden // spec.n_q_heads
    qpg = spec.n_q_heads // spec.n_kv_heads          # q heads per kv group
    g_loc = spec.n_kv_heads // TP                    # kv groups per TP rank
    out: List[PhysParam] = []

    def replicated(name: str) -> None:               # R2: full copy on every tp
        out.append(PhysParam(name, shapes[name], [Block(name, _ALL, _ALL)], tp == 0))

    def split0(phys: str, name: str, canonical: bool = True) -> None:   # R2 column-parallel
        n = shapes[name][0] // TP
        out.append(PhysParam(phys, (n,) + shapes[name][1:],
                             [Block(name, _rows(tp * n, (tp + 1) * n), _ALL)], canonical))

    def vocab_split(phys: str, name: str, canonical: bool = True) -> None:   # R2 + R11b
        n = padded_vocab(spec, lay) // TP            # rows per rank, padding included
        lo, hi = tp * n, min((tp + 1) * n, spec.vocab)
        blocks = [Block(name, _rows(lo, hi), _rows(0, hi - lo))] if hi > lo else []
        out.append(PhysParam(phys, (n,) + shapes[name][1:], blocks, canonical))

    def split1(phys: str, name: str) -> None:        # R2 row-parallel
        r, c = shapes[name]
        n = c // TP
        out.append(PhysParam(phys, (r, n), [Block(name, _cols(tp * n, (tp + 1) * n), _ALL)], True))

    def fused_qkv(p: str, suffix: str) -> None:      # R3
        tail = shapes[p + "q." + suffix][1:]
        blocks, row = [], 0
        if g_loc == 0:                               # R3b: TP > n_kv, kv group replicated on r ranks
            r = TP // spec.n_kv_heads
            g, j, nq = tp // r, tp % r, (qpg // r) * hd
            for nm, lo, n, canon in ((p + "q." + suffix, g * qpg * hd + j * nq, nq, True),
                                     (p + "k." + suffix, g * hd, hd, j == 0),
                                     (p + "v." + suffix, g * hd, hd, j == 0)):
                blocks.append(Block(nm, _rows(lo, lo + n), _rows(row, row + n), canon))
                row += n
        for j in range(g_loc):
            g = tp * g_loc + j
            for nm, lo, n in ((p + "q." + suffix, g * qpg * hd, qpg * hd),
                              (p + "k." + suffix, g * hd, hd),
                              (p + "v." + suffix, g * hd, hd)):
                blocks.append(Block(nm, _rows(lo, lo + n), _rows(row, row + n)))
                row += n
        out.append(PhysParam(p + "qkv." + suffix, (row,) + tail, blocks, True))

    def fc1(p: str, suffix: str, phys: str) -> None:  # R4
        if not spec.glu:
            split0(phys + "fc1." + suffix, p + "up." + suffix)
            return
        n = spec.ffn // TP
        tail = shapes[p + "up." + suffix][1:]
        out.append(PhysParam(phys + "fc1." + suffix, (2 * n,) + tail,
                             [Block(p + "gate." + suffix, _rows(tp * n, (tp + 1) * n), _rows(0, n)),
                              Block(p + "up." + suffix, _rows(tp * n, (tp + 1) * n), _rows(n, 2 * n))],
                             True))

    def ffn(p: str, phys: str) -> None:              # fc1 (+bias), fc2 (+bias) of the FFN whose tensors start with p
        fc1(p, "w", phys)
        if spec.linear_bias:
            fc1(p, "b", phys)
        split1(phys + "fc2.w", p + "down.w")
        if spec.linear_bias:
            replicated(p + "down.b")

    if ep is not None:                               # R13: expert buffer: layer by layer, expert by expert
        per = spec.n_experts // lay.ep
        for l in stage_layers(spec, lay, pp):
            for e in range(ep * per, (ep + 1) * per):
                ffn(f"L{l}.x{e}.", f"L{l}.x{e}.")
        return _finish(out, lay, [ep + lay.ep * j for j in range(lay.dp // lay.ep)])

    if pp == 0:
        vocab_split("embed.word", "embed.word")
        if spec.max_pos:
            replicated("embed.pos")
    for l in stage_layers(spec, lay, pp):
        p = f"L{l}."
        replicated(p + "ln1.w")
        if spec.norm_bias:
            replicated(p + "ln1.b")
        fused_qkv(p, "w")
        if spec.linear_bias:
            fused_qkv(p, "b")
        split1(p + "o.w", p + "o.w")
        if spec.linear_bias:
            replicated(p + "o.b")
        replicated(p + "ln2.w")
        if spec.norm_bias:
            replicated(p + "ln2.b")
        if spec.n_experts:
            replicated(p + "router.w")
        else:
            ffn(p, p)
    if pp == lay.pp - 1:
        replicated("final_norm.w")
        if spec.norm_bias:
            replicated("final_norm.b")
        if not spec.tied_embed:
            vocab_split("lm_head.w", "lm_head.w")
        elif lay.pp > 1:                             # R8: second copy, never the one read
            vocab_split("embed.word(tied copy)", "embed.word", canonical=False)

    return _finish(out, lay, list(range(lay.dp)))


def _finish(out: List[PhysParam], lay: Layout, dp_ranks: List[int]) -> StageView:
    """Assign flat offsets (R5), close and pad buckets (R5b, R6)."""
    quantum = len(dp_ranks) * lay.pad_multiple       # R6
    buckets: List[Tuple[int, int]] = []
    off = start = end = 0
    for i, prm in enumerate(out):                    # R5: back to back, no per-param padding
        prm.offset = off
        off = end = off + prm.size
        if (lay.bucket_elems and off - start >= lay.bucket_elems) or i == len(out) - 1:     # R5b: bucket closes
            off = start + -(-(off - start) // quantum) * quantum
            buckets.append((start, off - start))
            start = off
    return StageView(out, end, off, off // len(dp_ranks), buckets, dp_ranks)


def kinds_of(spec: ModelSpec) -> Tuple[int, ...]:
    return KINDS + EXPERT_KINDS if spec.n_experts else KINDS


def columns(lay: Layout, kind: int):
    """(tp, pp, ep) of every flat buffer of `kind`: ep is None for the dense kinds."""
    for pp in range(lay.pp):
        for tp in range(lay.tp):
            for ep in (range(lay.ep) if kind >= EXPERT_PARAM else (None,)):
                yield tp, pp, ep


def buffer_elems(spec: ModelSpec, lay: Layout, tp: int, pp: int, kind: int, dp: int = 0) -> int:
    sv = stage_view(spec, lay, tp, pp, dp % lay.ep if kind >= EXPERT_PARAM else None)
    return sv.n_pad if kind % 4 == 0 else sv.S


# ------------------------------------------------------------------ flat access
Reader = Callable[[int, int, int, int], np.ndarray]   # (rank, kind, lo, hi) -> elements [lo, hi)


def dict_reader(bufs: Dict[Tuple[int, int], np.ndarray]) -> Reader:
    return lambda rank, kind, lo, hi: bufs[(rank, kind)][lo:hi]


def dp_pieces(sv: StageView, lay: Layout, lo: int, hi: int) -> List[Tuple[int, int, int, int]]:
    """Where flat elements [lo, hi) of a rank column live in the fp32 buffers (R6):
    [(dp rank, offset in that rank's buffer, flat offset, count)] in flat order.
    Each bucket is cut into equal slices, one per DP rank sharing the buffer
    (sv.dp_ranks); a rank's buffer is the concatenation of its slice of every bucket."""
    out, prefix, group = [], 0, sv.dp_ranks
    for b0, nb in sv.buckets:
        sb = nb // len(group)
        for j, d in enumerate(group):
            a, b = max(lo, b0 + j * sb), min(hi, b0 + (j + 1) * sb)
            if a < b:
                out.append((d, prefix + a - b0 - j * sb, a, b - a))
        prefix += sb
    return out


def read_flat(read: Reader, lay: Layout, sv: StageView, tp: int, pp: int, kind: int, lo: int, hi: int,
              dp_replica: Optional[int] = None) -> np.ndarray:
    """Elements [lo, hi) of the flat buffer `sv` of rank column (tp, pp), kind `kind`.

    bf16 kinds: taken from replica `dp_replica` (default: the first rank that holds
    the buffer, R7).  fp32 kinds: concatenation of the pieces held by the DP ranks
    (dp_pieces)."""
    if kind % 4 == 0:
        return np.asarray(read(lay.rank(tp, pp, sv.dp_ranks[0] if dp_replica is None else dp_replica), kind, lo, hi))
    parts = [np.asarray(read(lay.rank(tp, pp, d), kind, loc, loc + n)) for d, loc, _, n in dp_pieces(sv, lay, lo, hi)]
    return np.concatenate(parts) if parts else np.empty(0, WORD[kind])


# ----------------------------------------------------------------------- gather
def gather_logical(spec: ModelSpec, lay: Layout, kind: int, read: Reader,
                   names: Optional[Iterable[str]] = None, check: bool = True) -> Dict[str, np.ndarray]:
    """Full logical tensors (all, or `names`) of `kind` from a sharded world.

    Each canonical physical parameter is cut out of its rank's flat buffer,
    reshaped to its local shape and assigned into the logical tensors block by
    block.  With `check`, every logical element must be assigned exactly once
    (Appendix A.2.1, Eq. 1: the shards of a configuration tile the tensor)."""
    shapes = logical_tensors(spec)
    want = set(shapes) if names is None else set(names)
    mine = lambda n: (".x" in n) == (kind >= EXPERT_PARAM)   # expert tensors live in kinds 4..7, the others in 0..3
    logical = {n: np.zeros(shapes[n], WORD[kind]) for n in shapes if n in want and mine(n)}
    hits = {n: np.zeros(shapes[n], np.uint8) for n in logical} if check else None
    for tp, pp, ep in columns(lay, kind):
        sv = stage_view(spec, lay, tp, pp, ep)
        for prm in sv.params:
            if not prm.canonical or not any(b.name in logical and b.canonical for b in prm.blocks):
                continue
            local = read_flat(read, lay, sv, tp, pp, kind, prm.offset, prm.offset + prm.size).reshape(prm.shape)
            for b in prm.blocks:
                if b.name in logical and b.canonical:
                    logical[b.name][b.idx] = local[b.loc]
                    if hits is not None:
                        hits[b.name][b.idx] += 1
    if hits is not None:
        for n, h in hits.items():
            if not (h == 1).all():
                raise AssertionError(f"logical tensor {n}: not every element gathered exactly once")
    return logical


# ------------------------------------------------------------------------ split
def build_shard(prm: PhysParam, logical: Dict[str, np.ndarray], dtype) -> np.ndarray:
    """Local shard of one physical parameter, cut out of the logical tensors
    (elements no block covers -- vocabulary padding -- stay +0)."""
    local = np.zeros(prm.shape, dtype)
    for b in prm.blocks:
        local[b.loc] = logical[b.name][b.idx]
    return local


def split_logical(spec: ModelSpec, lay: Layout, kind: int,
                  logical: Dict[str, np.ndarray]) -> Dict[Tuple[int, int], np.ndarray]:
    """Every rank's buffer of `kind` for world `lay`; padding is +0 (R6)."""
    out: Dict[Tuple[int, int], np.ndarray] = {}
    for tp, pp, ep in columns(lay, kind):
        sv = stage_view(spec, lay, tp, pp, ep)
        flat = np.zeros(sv.n_pad, WORD[kind])
        for prm in sv.params:
            flat[prm.offset:prm.offset + prm.size] = build_shard(prm, logical, WORD[kind]).ravel()
        n = len(sv.dp_ranks)
        for j, dp in enumerate(sv.dp_ranks):
            if kind % 4 == 0:
                out[(lay.rank(tp, pp, dp), kind)] = flat.copy()
            else:                                    # this rank's slice of every bucket, concatenated
                out[(lay.rank(tp, pp, dp), kind)] = np.concatenate(
                    [flat[b0 + j * (nb // n):b0 + (j + 1) * (nb // n)] for b0, nb in sv.buckets])
    return out


# ------------------------------------------------------------------------- cast
def rne_bf16(u: np.ndarray) -> np.ndarray:
    """fp32 bit patterns -> bf16 bit patterns, round to nearest even (R10)."""
    u = np.asarray(u, np.uint32)
    wide = u.astype(np.uint64)
    rounded = ((wide + 0x7FFF + ((wide >> 16) & 1)) >> 16).astype(np.uint16)
    is_nan = (u & 0x7FFFFFFF) > 0x7F800000
    quiet = ((u >> 16) | 0x0040).astype(np.uint16)
    return np.where(is_nan, quiet, rounded)


# ---------------------------------------------------------------------- reshard
def reshard_state(spec: ModelSpec, src: Layout, dst: Layout,
                  src_bufs: Dict[Tuple[int, int], np.ndarray], derive_bf16: bool = False,
                  kinds: Optional[Iterable[int]] = None) -> Dict[Tuple[int, int], np.ndarray]:
    """The whole result: gather under `src`, split under `dst`, kind by kind.

    derive_bf16: target PARAM is rne_bf16 of the gathered MASTER tensors (the
    element with the same logical index), not a copy of the source PARAM."""
    read = dict_reader(src_bufs)
    out: Dict[Tuple[int, int], np.ndarray] = {}
    for kind in (kinds_of(spec) if kinds is None else kinds):
        if kind % 4 == 0 and derive_bf16:              # PARAM from MASTER, EXPERT_PARAM from EXPERT_MASTER
            master = gather_logical(spec, src, kind + 1, read)
            logical = {n: rne_bf16(a) for n, a in master.items()}
        else:
            logical = gather_logical(spec, src, kind, read)
        out.update(split_logical(spec, dst, kind, logical))
    return out


def expected_shards(spec: ModelSpec, lay: Layout, logical: Dict[str, np.ndarray],
                    tps: Optional[Iterable[int]] = None, pps: Optional[Iterable[int]] = None, kind: int = PARAM):
    """For a subset of logical tensors: yield (tp, pp, stage_view, param, shard)
    for every physical parameter of world `lay` (optionally only rank columns
    tps x pps) built only from that subset.  Lets a caller verify a few tensors
    of a very large state one at a time.  `kind` selects the buffer family: a
    dense kind walks the dense buffers, an expert kind the expert buffers of
    every expert-parallel index (the stage view names the DP ranks that share it)."""
    have = set(logical)
    tps, pps = (None if tps is None else set(tps)), (None if pps is None else set(pps))
    for tp, pp, ep in columns(lay, kind):
        if (tps is not None and tp not in tps) or (pps is not None and pp not in pps):
            continue
        sv = stage_view(spec, lay, tp, pp, ep)
        for prm in sv.params:
            if prm.blocks and all(b.name in have for b in prm.blocks):
                yield tp, pp, sv, prm, build_shard(prm, logical, logical[prm.blocks[0].name].dtype)


__all__ = ["PARAM", "MASTER", "ADAM_M", "ADAM_V", "KINDS", "EXPERT_PARAM", "EXPERT_MASTER", "EXPERT_ADAM_M",
           "EXPERT_ADAM_V", "EXPERT_KINDS", "kinds_of", "columns", "WORD", "ModelSpec", "Layout",
           "check_supported", "padded_vocab", "logical_tensors", "Block", "PhysParam", "StageView", "stage_layers", "stage_view",
           "buffer_elems", "Reader", "dict_reader", "dp_pieces", "read_flat", "gather_logical", "build_shard",
           "split_logical", "rne_bf16", "reshard_state", "expected_shards"]
