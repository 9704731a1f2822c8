"""Shared test helpers (CPU side)."""
import numpy as np

import liver_synth as synth
import oracle
import ownership as own

NAN16, NAN32 = 0x7FC1, 0x7FC00001          # sentinels written into SOURCE padding


def cfg_objects(name):
    cfg = synth.CONFIGS[name]
    spec = oracle.ModelSpec(**cfg["spec"])
    src = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    dst = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["dst"])
    return cfg, spec, src, dst


def buffers_of(spec, lay):
    """(kind base, ep) of every flat-buffer family of world `lay`: (0, None) for the dense parameters and, for a
    mixture-of-experts model, (4, e) for the expert buffer of every expert-parallel index e."""
    yield 0, None
    if spec.n_experts:
        for e in range(lay.ep):
            yield 4, e


def _scatter(spec, lay, bufs, tp, pp, base, ep, positions, fn16, fn32):
    """Apply fn16 / fn32 (in place, on index arrays) to the given flat positions of one flat buffer of rank
    column (tp, pp) in every device buffer that holds them: all bf16 replicas, and the owning rank's fp32 buffers."""
    dp_of, local_of = own.shard_location(spec, lay, pp, ep)
    group = range(lay.dp) if ep is None else range(ep, lay.dp, lay.ep)
    for j, dp in enumerate(group):
        r = lay.rank(tp, pp, dp)
        if (r, base) in bufs:
            fn16(bufs[(r, base)], positions, j)
        mine = local_of[positions[dp_of[positions] == dp]]
        for k in (base + 1, base + 2, base + 3):
            if (r, k) in bufs:
                fn32(bufs[(r, k)], mine)


def poison_pads(spec, lay, bufs):
    """Overwrite every padding element of world `lay` (bucket padding, tail padding, vocabulary padding rows)
    with NaN sentinels: source padding must never be read by a reshard."""
    def f16(a, pos, j):
        a[pos] = NAN16

    def f32(a, pos):
        a[pos] = NAN32
    for base, ep in buffers_of(spec, lay):
        for pp in range(lay.pp):
            for tp in range(lay.tp):
                names, _, _ = own.column_ownership(spec, lay, tp, pp, ep)
                _scatter(spec, lay, bufs, tp, pp, base, ep, np.flatnonzero(np.equal(names, None)), f16, f32)
    return bufs


def make_world(spec, lay, state, poison=True, kinds=None):
    """Shard a logical state {kind: {name: array}} into world `lay`."""
    bufs = {}
    for k in (oracle.kinds_of(spec) if kinds is None else kinds):
        bufs.update(oracle.split_logical(spec, lay, k, state[k % 4]))
    return poison_pads(spec, lay, bufs) if poison else bufs


def corrupt_replicas(spec, lay, bufs):
    """Flip bits in every copy a gather must NOT read, located by the ownership formulas (not by the oracle):
    TP-replicated parameters on tp > 0, replicated k / v heads, the tied embedding copy, all padding, and the
    whole bf16 buffer of every replica but the first."""
    def f16(a, pos, j):
        if j > 0:
            a ^= 0x00FF
        else:
            a[pos] ^= 0x5555

    def f32(a, pos):
        a[pos] ^= 0x55555555
    for base, ep in buffers_of(spec, lay):
        for pp in range(lay.pp):
            for tp in range(lay.tp):
                names, _, canon = own.column_ownership(spec, lay, tp, pp, ep)
                _scatter(spec, lay, bufs, tp, pp, base, ep, np.flatnonzero(~canon | np.equal(names, None)), f16, f32)
    return bufs


def assert_same(a, b, what=""):
    assert set(a) == set(b), (what, sorted(set(a) ^ set(b))[:8])
    for key in a:
        x, y = np.asarray(a[key]), np.asarray(b[key])
        assert x.shape == y.shape and x.dtype == y.dtype, (what, key, x.shape, y.shape, x.dtype, y.dtype)
        if not np.array_equal(x, y):
            bad = np.flatnonzero(x != y)
            raise AssertionError(f"{what} buffer {key}: {bad.size} mismatches, first at {bad[:5]}: "
                                 f"{x[bad[:5]]} vs {y[bad[:5]]}")


def brute_reshard(spec, src, dst, src_bufs, derive=False):
    """Element-by-element reshard in pure Python, from the ownership formulas
    alone (tiny models only).  Independent of the oracle's slicing."""
    value = {k: {} for k in range(4)}           # by kind % 4: tensor names tell dense and expert tensors apart
    for base, ep in buffers_of(spec, src):
        for pp in range(src.pp):
            dp_of, local_of = own.shard_location(spec, src, pp, ep)
            first = 0 if ep is None else ep      # the bf16 copy that is read: the first rank holding the buffer
            for tp in range(src.tp):
                names, idx, canon = own.column_ownership(spec, src, tp, pp, ep)
                for k in range(len(names)):
                    if not canon[k] or names[k] is None:
                        continue
                    key = (names[k], int(idx[k]))
                    assert key not in value[0], ("owned twice", key)
                    value[0][key] = src_bufs[(src.rank(tp, pp, first), base)][k]
                    for kind in (1, 2, 3):
                        value[kind][key] = src_bufs[(src.rank(tp, pp, int(dp_of[k])), base + kind)][local_of[k]]
    if derive:
        value[0] = {key: _rne_scalar(int(v)) for key, v in value[1].items()}
    out = {}
    for base, ep in buffers_of(spec, dst):
        for pp in range(dst.pp):
            npad = own.n_pad(spec, dst, pp, ep)
            dp_of, local_of = own.shard_location(spec, dst, pp, ep)
            group = list(range(dst.dp)) if ep is None else list(range(ep, dst.dp, dst.ep))
            for tp in range(dst.tp):
                names, idx, _ = own.column_ownership(spec, dst, tp, pp, ep)
                for dp in group:
                    r = dst.rank(tp, pp, dp)
                    out[(r, base)] = np.zeros(npad, np.uint16)
                    for kind in (1, 2, 3):
                        out[(r, base + kind)] = np.zeros(npad // len(group), np.uint32)
                for k in range(len(names)):
                    if names[k] is None:            # padding stays +0
                        continue
                    key = (names[k], int(idx[k]))
                    for dp in group:
                        out[(dst.rank(tp, pp, dp), base)][k] = value[0][key]
                    for kind in (1, 2, 3):
                        out[(dst.rank(tp, pp, int(dp_of[k])), base + kind)][local_of[k]] = value[kind][key]
    return out


def _rne_scalar(u):
    """fp32 bits -> bf16 bits for one value, by comparing the two neighbours
    (not the add-and-shift trick): nearest, ties to the even upper half."""
    if (u & 0x7FFFFFFF) > 0x7F800000:
        return (u >> 16) | 0x0040
    lo = u >> 16
    rem = u & 0xFFFF
    if rem > 0x8000 or (rem == 0x8000 and (lo & 1)):
        lo += 1                     # carries into the exponent -> next binade / Inf, as it should
    return lo & 0xFFFF


def tiny_state(spec, seed=1):
    """Random distinct-ish bit patterns for a tiny model (all kinds independent)."""
    rng = np.random.default_rng(seed)
    shapes = oracle.logical_tensors(spec)
    st = {k: {} for k in oracle.KINDS}           # state[kind % 4][name]: expert tensors are told apart by name
    for name, shape in shapes.items():
        st[oracle.PARAM][name] = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
        for k in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
            st[k][name] = rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)
    return st
