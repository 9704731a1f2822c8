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


def poison_pads(spec, lay, bufs):
    """Overwrite the padding of every buffer of world `lay` with NaN sentinels
    (source padding must never be read by a reshard)."""
    for pp in range(lay.pp):
        nl = own.n_local(spec, lay.tp, lay.pp, pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last)
        npad = own.n_pad(spec, lay.tp, lay.pp, lay.dp, lay.pad_multiple, pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last)
        S = npad // lay.dp
        for tp in range(lay.tp):
            for dp in range(lay.dp):
                r = lay.rank(tp, pp, dp)
                if (r, oracle.PARAM) in bufs:
                    bufs[(r, oracle.PARAM)][nl:npad] = NAN16
                lo = max(nl - dp * S, 0)
                for k in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
                    if (r, k) in bufs and lo < S:
                        bufs[(r, k)][lo:S] = NAN32
    return bufs


def make_world(spec, lay, state, poison=True, kinds=oracle.KINDS):
    """Shard a logical state {kind: {name: array}} into world `lay`."""
    bufs = {}
    for k in kinds:
        bufs.update(oracle.split_logical(spec, lay, k, state[k]))
    return poison_pads(spec, lay, bufs) if poison else bufs


def corrupt_replicas(spec, lay, bufs):
    """Flip bits in every copy a gather must NOT read, located by the ownership
    formulas (not by the oracle): TP-replicated parameters on tp > 0, the tied
    embedding copy, PARAM replicas with dp > 0, and vocabulary padding rows."""
    for pp in range(lay.pp):
        nl = own.n_local(spec, lay.tp, lay.pp, pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last)
        S = own.n_pad(spec, lay.tp, lay.pp, lay.dp, lay.pad_multiple, pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last) // lay.dp
        for tp in range(lay.tp):
            names, _, canon = own.column_ownership(spec, lay.tp, lay.pp, tp, pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last)
            bad = np.flatnonzero(~canon | np.equal(names, None))       # copies, and vocabulary padding
            for dp in range(lay.dp):
                r = lay.rank(tp, pp, dp)
                if dp > 0:
                    bufs[(r, oracle.PARAM)][:nl] ^= 0x00FF
                else:
                    bufs[(r, oracle.PARAM)][bad] ^= 0x5555
                mine = bad[(bad >= dp * S) & (bad < (dp + 1) * S)] - dp * S
                for k in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
                    bufs[(r, k)][mine] ^= 0x55555555
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
    value = {k: {} for k in oracle.KINDS}
    for pp in range(src.pp):
        npad = own.n_pad(spec, src.tp, src.pp, src.dp, src.pad_multiple, pp, src.vpp, src.vocab_multiple, src.pp_first, src.pp_last)
        S = npad // src.dp
        for tp in range(src.tp):
            names, idx, canon = own.column_ownership(spec, src.tp, src.pp, tp, pp, src.vpp, src.vocab_multiple, src.pp_first, src.pp_last)
            for k in range(len(names)):
                if not canon[k] or names[k] is None:
                    continue
                key = (names[k], int(idx[k]))
                assert key not in value[oracle.PARAM], ("owned twice", key)
                value[oracle.PARAM][key] = src_bufs[(src.rank(tp, pp, 0), oracle.PARAM)][k]
                d = k // S
                for kind in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
                    value[kind][key] = src_bufs[(src.rank(tp, pp, d), kind)][k - d * S]
    if derive:
        value[oracle.PARAM] = {key: _rne_scalar(int(v)) for key, v in value[oracle.MASTER].items()}
    out = {}
    for pp in range(dst.pp):
        npad = own.n_pad(spec, dst.tp, dst.pp, dst.dp, dst.pad_multiple, pp, dst.vpp, dst.vocab_multiple, dst.pp_first, dst.pp_last)
        S = npad // dst.dp
        for tp in range(dst.tp):
            names, idx, _ = own.column_ownership(spec, dst.tp, dst.pp, tp, pp, dst.vpp, dst.vocab_multiple, dst.pp_first, dst.pp_last)
            flat = {kind: np.zeros(npad, oracle.WORD[kind]) for kind in oracle.KINDS}
            for k in range(len(names)):
                if names[k] is None:            # vocabulary padding stays +0
                    continue
                key = (names[k], int(idx[k]))
                for kind in oracle.KINDS:
                    flat[kind][k] = value[kind][key]
            for dp in range(dst.dp):
                r = dst.rank(tp, pp, dp)
                out[(r, oracle.PARAM)] = flat[oracle.PARAM].copy()
                for kind in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
                    out[(r, kind)] = flat[kind][dp * S:(dp + 1) * S].copy()
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
    st = {k: {} for k in oracle.KINDS}
    for name, shape in shapes.items():
        st[oracle.PARAM][name] = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
        for k in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
            st[k][name] = rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)
    return st
