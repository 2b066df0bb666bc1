"""Scalar-loop evaluation of the decoder block, in Python floats, for tiny shapes.

An independent statement of the same definition the oracle follows, used only to pin the
oracle: nested loops over tokens, heads, keys and features with explicit [out][in] weight
indexing, math.exp / math.cos / math.sin, and a contiguous per-sequence cache (no paging).
"""
import math


def rmsnorm_row(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    return [x[j] * g[j] / math.sqrt(ms + eps) for j in range(len(x))]


def layernorm_row(x, g, b, eps):
    """Variance through the plain two-moment formula E[x^2] - E[x]^2 (the tensor code sums squared deviations)."""
    n = len(x)
    mean = sum(x) / n
    var = sum(v * v for v in x) / n - mean * mean
    return [(x[j] - mean) / math.sqrt(var + eps) * g[j] + (b[j] if b is not None else 0.0) for j in range(n)]


def norm_row(shape, x, g, b):
    if getattr(shape, "norm_kind", "rms") == "layer":
        return layernorm_row(x, g, b, shape.rms_eps)
    return rmsnorm_row(x, g, shape.rms_eps)


def gelu_scalar(z, form):
    """Phi(z) through the complementary error function, and the tanh form written with exponentials."""
    if form == "gelu_erf":
        return z * 0.5 * math.erfc(-z / math.sqrt(2.0))
    t = math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)
    return z / (1.0 + math.exp(-2.0 * t))            # 0.5 (1 + tanh t) = 1 / (1 + exp(-2 t))


def matvec(w, x):
    """w[out][in] times x[in]."""
    return [sum(w[o][i] * x[i] for i in range(len(x))) for o in range(len(w))]


def scaled_frequency(freq, scaling):
    """In terms of turns over the trained length L (turns = L * freq / 2 pi): more than `high` turns - unchanged; fewer
    than `low` - divided by the factor; in between - the weight of the unchanged frequency rises linearly with the turns."""
    if scaling is None:
        return freq
    if scaling[0] == "linear":
        return freq / scaling[1]
    _, f, low, high, length = scaling
    turns = length * freq / (2.0 * math.pi)
    if turns > high:
        return freq
    if turns < low:
        return freq / f
    keep = (turns - low) / (high - low)
    return keep * freq + (1.0 - keep) * freq / f


def rope_head(u, p, theta, rotary_dim=0, interleaved=False, scaling=None):
    """rotary_dim > 0: only u[:rotary_dim] rotates (as a head of that size), the rest is copied.
    interleaved: element 2i is rotated with element 2i + 1 instead of element i with element i + d/2."""
    if rotary_dim and rotary_dim < len(u):
        return rope_head(u[:rotary_dim], p, theta, 0, interleaved, scaling) + list(u[rotary_dim:])
    d = len(u)
    half = d // 2
    y = [0.0] * d
    for i in range(half):
        ang = p * scaled_frequency(theta ** (-2.0 * i / d), scaling)
        c, s = math.cos(ang), math.sin(ang)
        a, b = (2 * i, 2 * i + 1) if interleaved else (i, i + half)
        y[a] = u[a] * c - u[b] * s
        y[b] = u[b] * c + u[a] * s
    return y


def layer_one_sequence(shape, w, rows, pos, cache_k, cache_v):
    """rows: list of [H] new-token inputs; cache_k/v: lists of [nkv][d] for the cached context
    (extended in place).  Returns the list of [H] outputs."""
    nq, nkv, d, hdim = shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.hidden
    g = nq // nkv
    ctx = len(cache_k)
    qs = []
    for n, x in enumerate(rows):
        a = norm_row(shape, x, w["norm1"], w.get("norm1_bias"))
        qkv = matvec(w["wqkv"], a)
        if w.get("bqkv") is not None:
            qkv = [u + b for u, b in zip(qkv, w["bqkv"])]
        qh = [qkv[h * d:(h + 1) * d] for h in range(nq)]
        kh = [qkv[(nq + r) * d:(nq + r + 1) * d] for r in range(nkv)]
        if w.get("qnorm") is not None:            # per-head norm of queries and keys, before the rotation
            qh = [rmsnorm_row(u, w["qnorm"], shape.rms_eps) for u in qh]
            kh = [rmsnorm_row(u, w["knorm"], shape.rms_eps) for u in kh]
        rd, il = getattr(shape, "rotary_dim", 0), getattr(shape, "rope_interleaved", False)
        sc = getattr(shape, "rope_scaling", None)
        if w.get("alibi") is None:
            q = [rope_head(u, pos[n], shape.rope_theta, rd, il, sc) for u in qh]
            k = [rope_head(u, pos[n], shape.rope_theta, rd, il, sc) for u in kh]
        else:                                     # linear biases: nothing rotates
            q, k = qh, kh
        v = [qkv[(nq + nkv + r) * d:(nq + nkv + r + 1) * d] for r in range(nkv)]
        cache_k.append(k)
        cache_v.append(v)
        qs.append(q)
    outs = []
    for n, x in enumerate(rows):
        o = []
        for h in range(nq):
            r = h // g
            last = ctx + n                       # causal: keys 0..ctx+n inclusive
            e = [sum(qs[n][h][c] * cache_k[j][r][c] for c in range(d)) / math.sqrt(d) for j in range(last + 1)]
            if w.get("alibi") is not None:       # each key is penalised by its distance from the query
                e = [e[j] - w["alibi"][h] * (last - j) for j in range(last + 1)]
            mx = max(e)
            wts = [math.exp(v_ - mx) for v_ in e]
            z = sum(wts)
            o.extend(sum(wts[j] / z * cache_v[j][r][c] for j in range(last + 1)) for c in range(d))
        proj = matvec(w["wo"], o)
        if w.get("bo") is not None:
            proj = [proj[j] + w["bo"][j] for j in range(hdim)]
        parallel = getattr(shape, "parallel_block", False)
        mlp_in = x if parallel else [x[j] + proj[j] for j in range(hdim)]
        if w.get("norm2") is None:               # the block's one norm feeds both branches
            b = norm_row(shape, x, w["norm1"], w.get("norm1_bias"))
        else:
            b = norm_row(shape, mlp_in, w["norm2"], w.get("norm2_bias"))
        up = matvec(w["wup"], b)
        kind = getattr(shape, "mlp_kind", "swiglu")
        if kind == "swiglu":
            gate = matvec(w["wgate"], b)
            m = [gate[f] / (1.0 + math.exp(-gate[f])) * up[f] for f in range(len(gate))]
        else:
            if w.get("bup") is not None:
                up = [up[f] + w["bup"][f] for f in range(len(up))]
            m = [gelu_scalar(u, kind) for u in up]
        dn = matvec(w["wdown"], m)
        if w.get("bdown") is not None:
            dn = [dn[j] + w["bdown"][j] for j in range(hdim)]
        outs.append([x[j] + proj[j] + dn[j] for j in range(hdim)])
    return outs


def round_to_bfloat16(x):
    """A Python float rounded to the nearest bfloat16 (ties to even), by way of float32 - the route a
    float64 tensor takes when it is stored into a bfloat16 cache."""
    import struct
    bits = struct.unpack("<I", struct.pack("<f", x))[0]
    if (bits & 0x7F800000) == 0x7F800000:                 # inf / nan: keep the top half
        return struct.unpack("<f", struct.pack("<I", bits & 0xFFFF0000))[0]
    bits += 0x7FFF + ((bits >> 16) & 1)
    return struct.unpack("<f", struct.pack("<I", bits & 0xFFFF0000))[0]


def layer_one_sequence_rounded_cache(shape, w, rows, pos, cache_k, cache_v, store=round_to_bfloat16):
    """The same block when the cache is a store of a narrower type: every new key (after the rotation)
    and value passes through `store` on its way into the cache, and attention - of the chunk that
    wrote them too - reads the cache."""
    nq, nkv, d, hdim = shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.hidden
    g = nq // nkv
    ctx = len(cache_k)
    qs = []
    for n, x in enumerate(rows):
        a = rmsnorm_row(x, w["norm1"], shape.rms_eps)
        qkv = matvec(w["wqkv"], a)
        q = [rope_head(qkv[h * d:(h + 1) * d], pos[n], shape.rope_theta) for h in range(nq)]
        k = [rope_head(qkv[(nq + r) * d:(nq + r + 1) * d], pos[n], shape.rope_theta) for r in range(nkv)]
        v = [qkv[(nq + nkv + r) * d:(nq + nkv + r + 1) * d] for r in range(nkv)]
        cache_k.append([[store(e) for e in head] for head in k])
        cache_v.append([[store(e) for e in head] for head in v])
        qs.append(q)
    outs = []
    for n, x in enumerate(rows):
        o = []
        for h in range(nq):
            r = h // g
            last = ctx + n
            e = [sum(qs[n][h][c] * cache_k[j][r][c] for c in range(d)) / math.sqrt(d) for j in range(last + 1)]
            mx = max(e)
            wts = [math.exp(v_ - mx) for v_ in e]
            z = sum(wts)
            o.extend(sum(wts[j] / z * cache_v[j][r][c] for j in range(last + 1)) for c in range(d))
        proj = matvec(w["wo"], o)
        hrow = [x[j] + proj[j] for j in range(hdim)]
        b = rmsnorm_row(hrow, w["norm2"], shape.rms_eps)
        gate = matvec(w["wgate"], b)
        up = matvec(w["wup"], b)
        m = [gate[f] / (1.0 + math.exp(-gate[f])) * up[f] for f in range(len(gate))]
        dn = matvec(w["wdown"], m)
        outs.append([hrow[j] + dn[j] for j in range(hdim)])
    return outs
