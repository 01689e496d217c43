"""Oracle-side shard plan, per-step partial attention and log-sum-exp merge.

TEST INFRASTRUCTURE ONLY; independent of the HIP library (no shared code, no import).

The paper only says that context parallelism splits each sequence evenly over the
d ranks of its group (Sec. 4.3, memory estimation) and that d may be any positive
integer (Sec. 4.2).  The load-balanced reading used by this build:

  * degree 1: the sequence is one chunk on its base rank;
  * degree d > 1: 2d zigzag chunks, the first (L mod 2d) chunks one token longer;
    group-local rank i owns chunk i ("early") and chunk 2d-1-i ("late");
  * ring step s of rank i uses the keys/values owned by rank j = (i - s) mod d, i.e.
    chunks j and 2d-1-j, of which a query chunk a sees those with index <= a;
  * inside a (query chunk, key chunk) pair a key is visible iff k_pos <= q_pos.

Mixed masks (Sec. 4.3, time estimation: some tokens of a multimodal sequence attend in full):
`spans` is a list of (seq, start, length); tokens of one span see each other in both directions,
every other pair stays causal.  Then a query chunk may also see keys of a LATER chunk (a span that
crosses the chunk border), so the work items are found from the visibility predicate itself: a key
chunk is a segment of an item iff at least one (query row, key) pair of the two chunks is visible.
The per-row form the kernels use -- row i sees exactly the keys 0 .. q_limit[i], key j is seen by
exactly the rows k_from[j] .. L-1 -- is DERIVED here by brute force from the predicate, and the
tests check that the visible sets really are such intervals.  eta_k of Eq. 8 is the number of
visible pairs of sequence k over its causal count, minus one.

Everything here is integer-exact or fp64 numpy, written for clarity.
"""
from __future__ import annotations

import numpy as np

CHUNK_DTYPE = np.dtype([("seq", "<i4"), ("rank", "<i4"), ("chunk", "<i4"),
                        ("seq_start", "<i4"), ("len", "<i4"), ("local_off", "<i4")])
WORK_DTYPE = np.dtype([("seq", "<i4"), ("rank", "<i4"), ("step", "<i4"),
                       ("q_local_off", "<i4"), ("q_seq_start", "<i4"), ("q_len", "<i4"),
                       ("n_seg", "<i4"), ("k_seq_start", "<i4", (2,)), ("k_len", "<i4", (2,))])
assert CHUNK_DTYPE.itemsize == 24 and WORK_DTYPE.itemsize == 44


def chunk_bounds(L: int, d: int):
    """(start, len) of every chunk of a length-L sequence at degree d."""
    if d == 1:
        return [(0, L)]
    n = 2 * d
    b, r = divmod(L, n)
    out, start = [], 0
    for c in range(n):
        ln = b + (1 if c < r else 0)
        out.append((start, ln))
        start += ln
    return out


def owner(c: int, d: int) -> int:
    """group-local rank that owns chunk c"""
    if d == 1:
        return 0
    return c if c < d else 2 * d - 1 - c


def span_ids(seq_lens, spans):
    """int32 [T]: index (in `spans`) of the span that holds each packed token, -1 for none."""
    cu = np.concatenate([[0], np.cumsum([int(x) for x in seq_lens])])
    sid = np.full(int(cu[-1]), -1, np.int32)
    for n, (k, st, ln) in enumerate(spans or []):
        assert 0 <= st and ln >= 1 and st + ln <= int(seq_lens[k])
        assert (sid[cu[k] + st: cu[k] + st + ln] == -1).all(), "spans overlap"
        sid[cu[k] + st: cu[k] + st + ln] = n
    return sid


def visible_matrix(q_pos, k_pos, sid_q=None, sid_k=None):
    """bool [nq, nk]: key visible to query, by definition (positions inside one sequence)."""
    q_pos, k_pos = np.asarray(q_pos)[:, None], np.asarray(k_pos)[None, :]
    vis = k_pos <= q_pos
    if sid_q is not None:
        sq, sk = np.asarray(sid_q)[:, None], np.asarray(sid_k)[None, :]
        vis = vis | ((sq >= 0) & (sq == sk))
    return vis


def mask_tables(seq_lens, spans, chunks, rank):
    """(q_limit [tq] int32, k_from [T] int32, eta [K] float64), each by brute force over the predicate:
    q_limit[row] = last key position the rank's local row sees, k_from[t] = first query position of the
    sequence that sees pool token t, eta[k] = visible pairs / causal pairs - 1."""
    seq_lens = [int(x) for x in seq_lens]
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    sid = span_ids(seq_lens, spans)
    lim_seq, k_from, eta = [], np.zeros(int(cu[-1]), np.int32), np.zeros(len(seq_lens))
    for k, L in enumerate(seq_lens):
        pos = np.arange(L)
        s = sid[cu[k]:cu[k + 1]]
        vis = visible_matrix(pos, pos, s, s)
        lim_seq.append(np.array([np.nonzero(vis[i])[0].max() for i in range(L)], np.int32))
        k_from[cu[k]:cu[k + 1]] = [np.nonzero(vis[:, j])[0].min() for j in range(L)]
        eta[k] = vis.sum() / (L * (L + 1) // 2) - 1.0
    mine = chunks[chunks["rank"] == rank]
    q_limit = np.zeros(int(mine["len"].sum()), np.int32)
    for ch in mine:
        a, n, lo = int(ch["seq_start"]), int(ch["len"]), int(ch["local_off"])
        q_limit[lo:lo + n] = lim_seq[int(ch["seq"])][a:a + n]
    return q_limit, k_from, eta


def shard_plan(seq_lens, cp_degree, base_rank=None, spans=None):
    """Returns (chunks, work) as structured arrays in the library's order:
    chunks by (rank, seq, chunk); work by (rank, step, seq, q_seq_start)."""
    seq_lens = [int(x) for x in seq_lens]
    sid_all = span_ids(seq_lens, spans) if spans else None
    cu_all = np.concatenate([[0], np.cumsum(seq_lens)])

    def sees(k, qa, kb):
        """does any row of chunk qa see any key of chunk kb (sequence k)?"""
        if qa["len"] == 0 or kb["len"] == 0:
            return False
        qp = np.arange(qa["seq_start"], qa["seq_start"] + qa["len"])
        kp = np.arange(kb["seq_start"], kb["seq_start"] + kb["len"])
        s = sid_all[cu_all[k]:cu_all[k + 1]]
        return bool(visible_matrix(qp, kp, s[qp], s[kp]).any())

    cp_degree = [int(x) for x in cp_degree]
    base = [0] * len(seq_lens) if base_rank is None else [int(x) for x in base_rank]
    chunks = []
    for k, (L, d) in enumerate(zip(seq_lens, cp_degree)):
        for c, (st, ln) in enumerate(chunk_bounds(L, d)):
            chunks.append(dict(seq=k, rank=base[k] + owner(c, d), chunk=c, seq_start=st, len=ln))
    chunks.sort(key=lambda x: (x["rank"], x["seq"], x["chunk"]))
    running = {}
    for ch in chunks:
        ch["local_off"] = running.get(ch["rank"], 0)
        running[ch["rank"]] = ch["local_off"] + ch["len"]
    by_key = {(ch["seq"], ch["chunk"]): ch for ch in chunks}

    work = []
    for k, d in enumerate(cp_degree):
        n = 1 if d == 1 else 2 * d
        for i in range(d):
            q_chunks = [0] if d == 1 else [i, 2 * d - 1 - i]
            for s in range(d):
                j = (i - s) % d
                kv_chunks = [0] if d == 1 else sorted([j, 2 * d - 1 - j])
                for a in q_chunks:
                    qa = by_key[(k, a)]
                    if qa["len"] == 0:
                        continue
                    if sid_all is None:
                        segs = [by_key[(k, b)] for b in kv_chunks if b <= a and by_key[(k, b)]["len"] > 0]
                    else:
                        segs = [by_key[(k, b)] for b in kv_chunks if sees(k, qa, by_key[(k, b)])]
                    if not segs:
                        continue
                    ks = [sg["seq_start"] for sg in segs] + [0] * (2 - len(segs))
                    kl = [sg["len"] for sg in segs] + [0] * (2 - len(segs))
                    work.append(dict(seq=k, rank=base[k] + i, step=s, q_local_off=qa["local_off"],
                                     q_seq_start=qa["seq_start"], q_len=qa["len"], n_seg=len(segs),
                                     k_seq_start=ks, k_len=kl))
        assert n == len(chunk_bounds(seq_lens[k], d))
    work.sort(key=lambda x: (x["rank"], x["step"], x["seq"], x["q_seq_start"]))

    ca = np.zeros(len(chunks), CHUNK_DTYPE)
    for idx, ch in enumerate(chunks):
        for f in CHUNK_DTYPE.names:
            ca[idx][f] = ch[f]
    wa = np.zeros(len(work), WORK_DTYPE)
    for idx, w in enumerate(work):
        for f in WORK_DTYPE.names:
            wa[idx][f] = w[f]
    return ca, wa


def rank_rows(chunks, cu_seqlens, rank):
    """Global token ids of the rows a rank owns, in its local (packed) order."""
    rows = []
    for ch in chunks[chunks["rank"] == rank]:
        t0 = int(cu_seqlens[ch["seq"]]) + int(ch["seq_start"])
        rows.append(np.arange(t0, t0 + int(ch["len"]), dtype=np.int64))
    return np.concatenate(rows) if rows else np.zeros(0, np.int64)


def rank_pairs(work, rank) -> int:
    """Number of visible (query, key) pairs in a rank's work items: for a query at
    position qp and a key segment [k0, k0+kl) the visible keys are k0..min(k0+kl-1, qp)."""
    total = 0
    for w in work[work["rank"] == rank]:
        qp = np.arange(int(w["q_seq_start"]), int(w["q_seq_start"]) + int(w["q_len"]), dtype=np.int64)
        for sgi in range(int(w["n_seg"])):
            k0, kl = int(w["k_seq_start"][sgi]), int(w["k_len"][sgi])
            total += int(np.clip(np.minimum(k0 + kl - 1, qp) - k0 + 1, 0, None).sum())
    return total


# ----------------------------------------------------------------------------
# fp64 partial attention over an explicit key set, and the merge of partials
# ----------------------------------------------------------------------------
def partial_attn(qf, kf, vf, q_pos, k_pos, scale, sid_q=None, sid_k=None):
    """qf [nq,Hq,D], kf/vf [nk,Hkv,D] float64; positions inside the sequence.
    Softmax over the visible keys only (k_pos <= q_pos, or the same span id when ids are given).
    Returns O [nq,Hq,D], LSE [nq,Hq]; a row with no visible key gets O = 0, LSE = -inf."""
    nq, hq, D = qf.shape
    hkv = kf.shape[1]
    G = hq // hkv
    kx = np.repeat(kf, G, axis=1)
    vx = np.repeat(vf, G, axis=1)
    s = scale * np.einsum("ihc,jhc->hij", qf, kx)
    vis = visible_matrix(q_pos, k_pos, sid_q, sid_k)[None]
    s = np.where(vis, s, -np.inf)
    m = s.max(axis=2, keepdims=True)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    p = np.where(vis, np.exp(s - m_safe), 0.0)
    l = p.sum(axis=2, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(l > 0, m_safe + np.log(l), -np.inf)[:, :, 0]
        pn = np.where(l > 0, p / l, 0.0)
    O = np.einsum("hij,jhc->ihc", pn, vx)
    return O, lse.T.copy()


def rank_partials(qbits_f64, kf, vf, cu_seqlens, chunks, work, rank, scale, span_id=None):
    """Per-step partials of one rank from its work items.
    qbits_f64: unsharded Q [T,Hq,D] float64.  Returns O_part [n_parts,tq,Hq,D],
    LSE_part [n_parts,tq,Hq] with O=0 / LSE=-inf where a row has no key in that step."""
    mine = work[work["rank"] == rank]
    my_chunks = chunks[chunks["rank"] == rank]
    tq = int(my_chunks["len"].sum())
    n_parts = int(mine["step"].max()) + 1 if len(mine) else 1
    hq, D = qbits_f64.shape[1], qbits_f64.shape[2]
    O = np.zeros((n_parts, tq, hq, D))
    LSE = np.full((n_parts, tq, hq), -np.inf)
    for w in mine:
        t0 = int(cu_seqlens[w["seq"]])
        q0, ql, lo = int(w["q_seq_start"]), int(w["q_len"]), int(w["q_local_off"])
        q_pos = np.arange(q0, q0 + ql)
        k_pos = np.concatenate([np.arange(int(w["k_seq_start"][sgi]), int(w["k_seq_start"][sgi]) + int(w["k_len"][sgi]))
                                for sgi in range(int(w["n_seg"]))])
        sq = None if span_id is None else span_id[t0 + q_pos]
        sk = None if span_id is None else span_id[t0 + k_pos]
        o, lse = partial_attn(qbits_f64[t0 + q_pos], kf[t0 + k_pos], vf[t0 + k_pos], q_pos, k_pos, scale, sq, sk)
        O[int(w["step"]), lo:lo + ql] = o
        LSE[int(w["step"]), lo:lo + ql] = lse
    return O, LSE


def lse_merge(O_part, LSE_part):
    """LSE = ln sum_s exp(LSE_s);  O = sum_s exp(LSE_s - LSE) O_s.  A part with
    LSE_s = -inf has weight 0; all parts -inf gives O = 0, LSE = -inf."""
    m = LSE_part.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(LSE_part - m_safe[None])           # exp(-inf) = 0
    tot = w.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(tot > 0, m_safe + np.log(tot), -np.inf)
        wn = np.where(tot[None] > 0, w / tot[None], 0.0)
    O = (wn[..., None] * O_part).sum(axis=0)
    return O, lse
