"""Per-element ownership, typed out as integer arithmetic (test tool).

For element `k` of physical parameter `phys` on TP rank `tp`, which logical
tensor and which row-major index inside it does that element hold?  These are
the closed forms of the layout conventions (column-parallel: contiguous rows;
row-parallel: a strip of every row; fused QKV grouped per kv-head group; gated
FFN stored as [gate rows ; up rows] per rank).  Nothing here slices arrays or
calls the oracle: it exists so that the oracle's slicing can be checked against
formulas a reader can verify with pencil and paper.
"""
import numpy as np


def dims(spec):
    H = spec.hidden
    hd = H // spec.n_q_heads
    return H, hd, spec.n_q_heads * hd, spec.n_kv_heads * hd, spec.ffn, spec.vocab


def layer_param_sizes(spec, TP, l):
    """[(physical name, element count)] of one transformer layer on one TP rank."""
    H, hd, Q, KV, F, V = dims(spec)
    p = f"L{l}."
    out = [(p + "ln1.w", H)]
    if spec.norm_bias:
        out.append((p + "ln1.b", H))
    # kv groups split over TP; if TP > n_kv every rank holds Q/TP q rows plus ONE whole k and v head
    qkv_rows = (Q + 2 * KV) // TP if spec.n_kv_heads % TP == 0 else Q // TP + 2 * hd
    out.append((p + "qkv.w", qkv_rows * H))
    if spec.linear_bias:
        out.append((p + "qkv.b", qkv_rows))
    out.append((p + "o.w", H * Q // TP))
    if spec.linear_bias:
        out.append((p + "o.b", H))
    out.append((p + "ln2.w", H))
    if spec.norm_bias:
        out.append((p + "ln2.b", H))
    if spec.n_experts:                      # mixture of experts: the dense buffer holds only the router
        out.append((p + "router.w", spec.n_experts * H))
    else:
        out += ffn_param_sizes(spec, TP, p)
    return out


def ffn_param_sizes(spec, TP, p):
    """fc1 (+bias), fc2 (+bias) of the FFN whose physical names start with p."""
    H, hd, Q, KV, F, V = dims(spec)
    n_fc1 = 2 * F if spec.glu else F
    out = [(p + "fc1.w", n_fc1 * H // TP)]
    if spec.linear_bias:
        out.append((p + "fc1.b", n_fc1 // TP))
    out.append((p + "fc2.w", H * F // TP))
    if spec.linear_bias:
        out.append((p + "down.b", H))
    return out


def group_size(lay, ep=None):
    """Ranks sharing one flat buffer: all DP ranks for the dense buffers, DP/EP for the expert buffers."""
    return lay.dp if ep is None else lay.dp // lay.ep


def stage_layer_list(spec, lay, pp):
    PP, vpp, first, last = lay.pp, lay.vpp, lay.pp_first, lay.pp_last
    if first or last:
        return list(range(*uneven_stage_range(spec.n_layers, PP, pp, first, last)))
    c = spec.n_layers // (PP * vpp)          # layers per model chunk; stage pp holds chunks pp, pp+PP, ...
    return [l for v in range(vpp) for l in range((v * PP + pp) * c, (v * PP + pp) * c + c)]


def vocab_rows(spec, TP, vm=0):
    """Rows of embed.word / lm_head per TP rank; vm > 0 pads the vocabulary to a multiple of vm*TP."""
    V = spec.vocab
    return V // TP if not vm else (V + vm * TP - 1) // (vm * TP) * vm


def uneven_stage_range(L, PP, pp, first, last):
    """[lo, hi) of the layers of stage pp when the first / last stage hold `first` / `last` layers
    (0 = not fixed) and the remaining stages share the rest evenly."""
    n_other = PP - (first > 0) - (last > 0)
    per = (L - first - last) // n_other if n_other else 0
    count = lambda p: first if (p == 0 and first) else last if (p == PP - 1 and last) else per
    lo = sum(count(p) for p in range(pp))
    return lo, lo + count(pp)


def stage_param_sizes(spec, lay, pp, ep=None):
    """[(physical name, element count)] of stage pp on one TP rank, in flat-buffer order.
    `lay` is any object with tp, pp, dp, pad_multiple, vpp, vocab_multiple, pp_first, pp_last, bucket_elems, ep.
    ep = None: the dense buffer.  ep = e: the expert buffer of expert-parallel index e (experts
    e*E/EP .. (e+1)*E/EP - 1 of every layer of the stage, layer by layer)."""
    H, hd, Q, KV, F, V = dims(spec)
    TP, PP, vpp, vm, first, last = lay.tp, lay.pp, lay.vpp, lay.vocab_multiple, lay.pp_first, lay.pp_last
    if ep is not None:
        per = spec.n_experts // lay.ep
        return [x for l in stage_layer_list(spec, lay, pp) for e in range(ep * per, ep * per + per)
                for x in ffn_param_sizes(spec, TP, f"L{l}.x{e}.")]
    out = []
    if pp == 0:
        out.append(("embed.word", vocab_rows(spec, TP, vm) * H))
        if spec.max_pos:
            out.append(("embed.pos", spec.max_pos * H))
    for l in stage_layer_list(spec, lay, pp):
        out += layer_param_sizes(spec, TP, l)
    if pp == PP - 1:
        out.append(("final_norm.w", H))
        if spec.norm_bias:
            out.append(("final_norm.b", H))
        if not spec.tied_embed:
            out.append(("lm_head.w", vocab_rows(spec, TP, vm) * H))
        elif PP > 1:
            out.append(("embed.word(tied copy)", vocab_rows(spec, TP, vm) * H))
    return out


def bucket_table(spec, lay, pp, ep=None):
    """[(start, used, padded)] of the buckets of stage pp's flat buffer.  Parameters are appended in order; a
    bucket closes after the parameter that brings it to >= bucket_elems elements (bucket_elems 0: one bucket);
    every bucket is zero-padded to a multiple of DP*pad_multiple elements."""
    sizes = stage_param_sizes(spec, lay, pp, ep)
    q = group_size(lay, ep) * lay.pad_multiple
    out, start, used = [], 0, 0
    for i, (_, n) in enumerate(sizes):
        used += n
        if (lay.bucket_elems and used >= lay.bucket_elems) or i == len(sizes) - 1:
            padded = (used + q - 1) // q * q
            out.append((start, used, padded))
            start, used = start + padded, 0
    return out


def n_local(spec, lay, pp, ep=None):
    """End of the last parameter in the flat buffer (interior bucket padding included)."""
    start, used, _ = bucket_table(spec, lay, pp, ep)[-1]
    return start + used


def n_pad(spec, lay, pp, ep=None):
    start, _, padded = bucket_table(spec, lay, pp, ep)[-1]
    return start + padded


def shard_location(spec, lay, pp, ep=None):
    """(dp_of, local_of): for every flat position 0..N_pad-1 of the fp32 buffers, the DP rank that holds it and
    its offset in that rank's buffer.  Each bucket is cut into equal slices, one per rank sharing the buffer
    (all DP ranks; for an expert buffer the DP ranks ep, ep+EP, ...); a rank's buffer is the concatenation of
    its slice of every bucket."""
    npad = n_pad(spec, lay, pp, ep)
    dp_of, local_of = np.zeros(npad, np.int64), np.zeros(npad, np.int64)
    prefix, g = 0, group_size(lay, ep)
    for start, _, padded in bucket_table(spec, lay, pp, ep):
        Sb = padded // g
        k = np.arange(padded, dtype=np.int64)
        dp_of[start:start + padded] = k // Sb if ep is None else ep + lay.ep * (k // Sb)
        local_of[start:start + padded] = prefix + k % Sb
        prefix += Sb
    return dp_of, local_of


def owner(spec, lay, tp, phys, k):
    """(names, idx): logical tensor name and row-major logical index of local
    elements k (int64 array) of physical parameter `phys` on TP rank `tp`."""
    H, hd, Q, KV, F, V = dims(spec)
    TP, vm = lay.tp, lay.vocab_multiple
    k = np.asarray(k, np.int64)
    base = phys.split("(")[0]
    pre = base[:base.index(".") + 1] if base.startswith("L") else ""
    if base[len(pre):].startswith("x"):                          # expert FFN: "L3.x5.fc1.w"
        pre = base[:base.index(".", len(pre)) + 1]
    leaf = base[len(pre):]
    names = np.empty(k.shape, dtype=object)

    if leaf in ("ln1.w", "ln1.b", "ln2.w", "ln2.b", "o.b", "down.b", "final_norm.w",
                "final_norm.b", "embed.pos", "router.w"):        # replicated
        names[:] = base
        return names, k
    if leaf in ("embed.word", "lm_head.w"):                      # column-parallel [V, H], maybe padded
        idx = tp * vocab_rows(spec, TP, vm) * H + k
        names[:] = base
        names[idx >= V * H] = None                               # vocabulary padding: owns nothing
        return names, np.where(idx >= V * H, 0, idx)
    if leaf == "o.w":                                            # row-parallel [H, Q]
        w = Q // TP
        names[:] = base
        return names, (k // w) * Q + tp * w + k % w
    if leaf == "fc2.w":                                          # row-parallel [H, F]
        w = F // TP
        names[:] = pre + "down.w"
        return names, (k // w) * F + tp * w + k % w
    if leaf in ("qkv.w", "qkv.b"):
        C = H if leaf == "qkv.w" else 1
        sfx = leaf[-1]
        qpg = spec.n_q_heads // spec.n_kv_heads
        g_loc = spec.n_kv_heads // TP
        i, j = k // C, k % C
        if g_loc == 0:                      # kv group g replicated on r = TP/n_kv ranks; this is its part `part`
            r = TP // spec.n_kv_heads
            g, part, nq = tp // r, tp % r, (qpg // r) * hd
            is_q, is_k = i < nq, (i >= nq) & (i < nq + hd)
            row = np.where(is_q, g * qpg * hd + part * nq + i, np.where(is_k, g * hd + (i - nq), g * hd + (i - nq - hd)))
            names[:] = pre + "v." + sfx
            names[is_k] = pre + "k." + sfx
            names[is_q] = pre + "q." + sfx
            return names, row * C + j
        G = (qpg + 2) * hd
        g = tp * g_loc + i // G
        w = i % G
        is_q, is_k = w < qpg * hd, (w >= qpg * hd) & (w < (qpg + 1) * hd)
        row = np.where(is_q, g * qpg * hd + w,
                       np.where(is_k, g * hd + (w - qpg * hd), g * hd + (w - (qpg + 1) * hd)))
        names[:] = pre + "v." + sfx
        names[is_k] = pre + "k." + sfx
        names[is_q] = pre + "q." + sfx
        return names, row * C + j
    if leaf in ("fc1.w", "fc1.b"):
        C = H if leaf == "fc1.w" else 1
        sfx = leaf[-1]
        n = F // TP
        i, j = k // C, k % C
        if not spec.glu:
            names[:] = pre + "up." + sfx
            return names, (tp * n + i) * C + j
        is_gate = i < n
        row = np.where(is_gate, tp * n + i, tp * n + i - n)
        names[:] = pre + "up." + sfx
        names[is_gate] = pre + "gate." + sfx
        return names, row * C + j
    raise KeyError(phys)


def column_ownership(spec, lay, tp, pp, ep=None):
    """For flat positions 0..N_pad-1 of rank column (tp, pp): (names, idx, canonical).

    names[k] is None where the position holds padding (bucket padding, tail padding, vocabulary padding rows).
    canonical[k] is False where the element is a replica that a gather must not read: TP-replicated
    parameters on tp > 0, replicated k / v heads on all but the first rank of their group, and the
    tied-embedding copy."""
    TP = lay.tp
    npad = n_pad(spec, lay, pp, ep)
    names = np.full(npad, None, dtype=object)
    idx = np.zeros(npad, np.int64)
    canon = np.zeros(npad, bool)
    sizes = stage_param_sizes(spec, lay, pp, ep)
    q = group_size(lay, ep) * lay.pad_multiple
    pos, used = 0, 0
    for phys, n in sizes:
        nm, ix = owner(spec, lay, tp, phys, np.arange(n, dtype=np.int64))
        leaf = phys.split(".", 1)[1] if phys.startswith("L") else phys
        if leaf.startswith("x"):
            leaf = leaf.split(".", 1)[1]
        replicated = leaf in ("ln1.w", "ln1.b", "ln2.w", "ln2.b", "o.b", "down.b", "final_norm.w",
                              "final_norm.b", "embed.pos", "router.w")
        ok = np.full(n, not (replicated and tp > 0) and "(tied copy)" not in phys)
        if leaf in ("qkv.w", "qkv.b") and spec.n_kv_heads % TP and tp % (TP // spec.n_kv_heads):
            ok &= np.char.endswith(nm.astype(str), ("q." + leaf[-1]))      # replicated k / v: read from part 0 only
        names[pos:pos + n], idx[pos:pos + n], canon[pos:pos + n] = nm, ix, ok
        pos, used = pos + n, used + n
        if lay.bucket_elems and used >= lay.bucket_elems:                  # bucket closes: skip its padding
            pos, used = pos + (-used) % q, 0
    return names, idx, canon
