"""CPU oracle for DEER's draft-verify step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the path computes.  It is imported only by the
tests, by the smoke check and by the benchmark's CPU-baseline leg; the product path never
calls it, and it shares no code with the HIP kernels.  Arithmetic is numpy in a caller-chosen
dtype (float64 by default; float32 for the multi-billion-parameter shapes).

What follows the paper, and where:
  * block drafting  y^_{j+1:j+k} ~ q_theta(. | x_{1:j}), all k positions from ONE drafter pass,
    each position's marginal independent of the other drafted tokens  (Sec. 3.2, first
    display; the "independent of previously drafted tokens" identity in the same section);
  * acceptance probability alpha_i = min(1, p_AR(y^_{j+i} | x_{1:j+i-1}) / q_theta(y^_{j+i} |
    x_{1:j}))  (Sec. 3.2, Eq. "accept"; Appendix, Lemma, step 2);
  * on rejection the token is drawn from the normalised residual max(0, p - q) / (1 - gamma)
    (Sec. 3.2, Eq. "resample"; Appendix, definition of p_res and gamma);
  * the decoding loop  (Algorithm 1).

Readings taken where the paper is silent or ambiguous (each is listed in the design notes):
  R1  The inner loop stops at the first rejection: the verifier's p_i for later i were
      conditioned on the draft prefix, which is no longer the realised prefix, and the Lemma
      conditions on the realised prefix.
  R2  No bonus token: the verifier sees k rows [x_j, y^_1 .. y^_{k-1}] and yields p_1..p_k; the
      largest accepted length is k (Table 4 reports max accepted length = block size).
  R3  The drafter is a decoder whose committed tokens attend causally (so their K,V can be
      cached append-only) and whose k MASK rows see every committed token and each other.
  R4  The MASK row at position j+i predicts token x_{j+i} (same position, no shift), as in the
      masked-denoising loss of Sec. 3.1 Eq. 1-2.
  R5  One temperature T scales both models' logits; T=0 is the one-hot limit, where the rule
      becomes: accept while y^_i equals the target's argmax, then emit that argmax.
  R6  Categorical draws use Gumbel-max over a counter-based generator (splitmix64 finaliser),
      ties to the lowest index.

Parity pins live in tests/test_oracle_*.py (losslessness at T=0 against plain greedy decoding,
k=1 reduction, exact enumeration of the one-step Lemma and of the sequence-level Theorem on
tabular models, RoPE/GQA/MoE reductions, closed-form acceptance rate).  The paper prints no
worked numeric example, so no value is pinned against the paper's tables ("parity unpinned"
against the printed tables: every one of them needs trained weights and datasets).
"""
from __future__ import annotations

import numpy as np

# =============================================================================================
# elementary pieces
# =============================================================================================


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def silu(x):
    return x / (1.0 + np.exp(-x))


def log_softmax(z):
    """Row-wise log softmax (last axis) with the usual max shift."""
    m = np.max(z, axis=-1, keepdims=True)
    s = z - m
    return s - np.log(np.sum(np.exp(s), axis=-1, keepdims=True))


def softmax(z):
    return np.exp(log_softmax(z))


def argmax_lowest(v):
    """Index of the maximum; the lowest index among equal maxima."""
    return int(np.argmax(v))  # numpy returns the first occurrence


def rope(x, pos, base):
    """Rotary embedding, rotate-half pairing (i, i + hd/2), angle = pos * base^(-2i/hd).

    x: [R][H][hd]; pos: [R] integer positions."""
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=np.float64)
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * i / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def round_to_bf16(x):
    """Nearest bfloat16 (8 significand bits, ties to even), returned in x's dtype.  Storage
    format only; finite inputs."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    keep = u >> np.uint64(16)
    rest = u & np.uint64(0xFFFF)
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint64(1)) == 1))
    keep = (keep + up.astype(np.uint64)) << np.uint64(16)
    return keep.astype(np.uint32).view(np.float32).reshape(f.shape).astype(x.dtype)


def gqa_attention(q, keys, vals, allowed):
    """Softmax attention with grouped K/V heads.

    q[R][Hq][hd], keys/vals[C][Hkv][hd], allowed[R][C] bool.  Query head h uses K/V head
    h // (Hq/Hkv).  Scores are q.k / sqrt(hd); disallowed pairs get weight 0."""
    R, Hq, hd = q.shape
    group = Hq // keys.shape[1]
    o = np.empty_like(q)
    for hq in range(Hq):
        hk = hq // group
        sc = (q[:, hq, :] @ keys[:, hk, :].T) / np.sqrt(q.dtype.type(hd))
        sc = np.where(allowed, sc, -np.inf)
        o[:, hq, :] = softmax(sc) @ vals[:, hk, :]
    return o


# =============================================================================================
# the two transformers
# =============================================================================================


class KVCache:
    """Per-layer K,V rows of the committed tokens, slot t holding 0-indexed position t."""

    def __init__(self, shape, capacity, dtype):
        dims = (shape.n_layers, capacity, shape.n_kv_heads, shape.head_dim)
        self.K = np.zeros(dims, dtype=dtype)
        self.V = np.zeros(dims, dtype=dtype)
        self.n = 0

    def truncate(self, n):
        assert 0 <= n <= self.n
        self.n = n


class Decoder:
    """Pre-norm decoder-only transformer: RMSNorm, GQA attention with RoPE, SwiGLU FFN (dense or
    top-k-of-E mixture), untied LM head.  RMSNorm gains are 1.  No biases.

    `weights(name, layer, expert)` returns the tensor in [in][out] orientation (embedding
    [vocab][d]) as exact values of the stored model; it may generate them on demand."""

    def __init__(self, shape, weights, dtype=np.float64, kv_storage=None):
        """kv_storage: None (K,V rows kept in the compute dtype) or "bf16": every K,V row is
        rounded to bfloat16 when it is produced, the way a bf16 KV cache stores it (the
        workloads with bf16 weights also state a bf16 cache); arithmetic stays in `dtype`."""
        self.s = shape
        self.w = weights
        self.dtype = dtype
        self.kv_storage = kv_storage

    def _w(self, name, layer=-1, expert=-1):
        return np.asarray(self.w(name, layer, expert), dtype=self.dtype)

    # -- feed-forward -------------------------------------------------------------------------
    def _ffn_dense(self, f, wg, wu, wd):
        return (silu(f @ wg) * (f @ wu)) @ wd

    def _ffn(self, f, layer):
        s = self.s
        if not s.n_experts:
            return self._ffn_dense(f, self._w("wg", layer), self._w("wu", layer), self._w("wd", layer))
        # mixture: softmax over all experts, take the top_k (ties -> lowest index), renormalise
        probs = softmax(f @ self._w("router", layer))
        out = np.zeros_like(f)
        order = np.argsort(-probs, axis=-1, kind="stable")[:, : s.top_k]
        cache = {}
        for r in range(f.shape[0]):
            sel = order[r]
            wsel = probs[r, sel] / np.sum(probs[r, sel])
            for e, we in zip(sel, wsel):
                e = int(e)
                if e not in cache:
                    cache[e] = (self._w("wg", layer, e), self._w("wu", layer, e), self._w("wd", layer, e))
                out[r] += we * self._ffn_dense(f[r:r + 1], *cache[e])[0]
        return out

    # -- one pass over R new rows ----------------------------------------------------------------
    def forward(self, ids, pos, cache, allowed_new, keep, logits_rows=None):
        """Run R rows through the model.

        ids[R], pos[R]: token ids and 0-indexed positions of the new rows.
        cache: KVCache holding cache.n committed rows, all visible to every new row.
        allowed_new[R][R] (bool): new row r may attend to new row c.
        keep (int): the first `keep` new rows' K,V are appended to the cache afterwards.
        logits_rows: indices of rows whose logits are wanted (default: all).
        Returns logits [len(logits_rows)][vocab]."""
        s, dt = self.s, self.dtype
        R = len(ids)
        n_old = cache.n
        h = self._w("embed")[np.asarray(ids)]
        ones = np.ones(s.d_model, dtype=dt)
        allowed = np.concatenate([np.ones((R, n_old), dtype=bool), np.asarray(allowed_new, dtype=bool)], axis=1)
        for l in range(s.n_layers):
            a = rmsnorm(h, ones, s.rms_eps)
            q = (a @ self._w("wq", l)).reshape(R, s.n_q_heads, s.head_dim)
            k = (a @ self._w("wk", l)).reshape(R, s.n_kv_heads, s.head_dim)
            v = (a @ self._w("wv", l)).reshape(R, s.n_kv_heads, s.head_dim)
            q = rope(q, pos, s.rope_base)
            k = rope(k, pos, s.rope_base)
            if self.kv_storage == "bf16":
                k, v = round_to_bf16(k), round_to_bf16(v)
            keys = np.concatenate([cache.K[l, :n_old], k], axis=0)
            vals = np.concatenate([cache.V[l, :n_old], v], axis=0)
            o = gqa_attention(q, keys, vals, allowed)
            h = h + o.reshape(R, -1) @ self._w("wo", l)
            f = rmsnorm(h, ones, s.rms_eps)
            h = h + self._ffn(f, l)
            cache.K[l, n_old:n_old + keep] = k[:keep]
            cache.V[l, n_old:n_old + keep] = v[:keep]
        cache.n = n_old + keep
        rows = np.arange(R) if logits_rows is None else np.asarray(logits_rows)
        if len(rows) == 0:
            return np.zeros((0, s.vocab), dtype=dt)
        return rmsnorm(h[rows], ones, s.rms_eps) @ self._w("lm_head")


def causal_mask(R):
    return np.tril(np.ones((R, R), dtype=bool))


def drafter_block_mask(m, k):
    """m committed-but-not-yet-cached rows followed by k MASK rows (reading R3): committed rows
    are causal among themselves and never see MASK rows; MASK rows see everything."""
    R = m + k
    a = np.zeros((R, R), dtype=bool)
    a[:m, :m] = np.tril(np.ones((m, m), dtype=bool))
    a[m:, :] = True
    return a


# =============================================================================================
# random numbers: counter-based, specified here, implemented independently on each side
# =============================================================================================
_M64 = (1 << 64) - 1
TAG_DRAFT, TAG_ACCEPT, TAG_RESID = 1, 2, 3


def mix64(z):
    """splitmix64's output finaliser on uint64 arrays (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def row_key(seed, tag, seq, pos):
    """Key of the random stream used for (purpose tag, sequence, absolute 0-indexed position)."""
    with np.errstate(over="ignore"):
        a = mix64(np.uint64(seed & _M64) + np.uint64(0x9E3779B97F4A7C15) * np.uint64(tag))
        b = mix64(a ^ ((np.uint64(seq) << np.uint64(40)) + np.uint64(pos)))
    return b


def uniforms(key, idx):
    """u in (0,1): the top 23 bits of mix64(key + (idx+1)*golden), centred: (r + 0.5) / 2^23."""
    with np.errstate(over="ignore"):
        bits = mix64(np.uint64(key) + np.uint64(0x9E3779B97F4A7C15) * (np.asarray(idx, dtype=np.uint64) + np.uint64(1)))
    r = (bits >> np.uint64(41)).astype(np.float64)
    return (r + 0.5) / 8388608.0


class CounterRng:
    """The generator both sides implement.  `accept` draws u ~ U(0,1) and applies the test
    u <= alpha of Algorithm 1 in log space; `categorical` is Gumbel-max over log-weights."""

    def __init__(self, seed, seq=0, dtype=np.float64):
        self.seed, self.seq, self.dtype = int(seed), int(seq), dtype

    def accept(self, log_alpha, pos):
        u = uniforms(row_key(self.seed, TAG_ACCEPT, self.seq, pos), 0)
        return bool(np.log(u) <= log_alpha)

    def _gumbel(self, tag, pos, n):
        u = uniforms(row_key(self.seed, tag, self.seq, pos), np.arange(n))
        return (-np.log(-np.log(u))).astype(self.dtype)

    def categorical(self, logw, pos, tag):
        """argmax_v (logw_v + Gumbel_v); entries with logw = -inf can never win."""
        return argmax_lowest(np.asarray(logw, dtype=self.dtype) + self._gumbel(tag, pos, len(logw)))


# =============================================================================================
# the acceptance rule
# =============================================================================================


def log_alpha(logp_y, logq_y):
    """log of alpha = min(1, p(y)/q(y))  (Sec. 3.2 Eq. "accept")."""
    return min(0.0, float(logp_y) - float(logq_y))


def residual_logweights(logp, logq):
    """log max(0, p - q), elementwise (Sec. 3.2 Eq. "resample"); -inf where p <= q.

    If p <= q everywhere (gamma = 1, so the branch is unreachable in exact arithmetic) the
    Appendix allows any definition; p itself is used."""
    p, q = np.exp(logp), np.exp(logq)
    d = p - q
    if not np.any(d > 0):
        return np.array(logp, copy=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        return np.where(d > 0, np.log(np.where(d > 0, d, 1.0)), -np.inf)


def residual_distribution(logp, logq):
    """Normalised residual (p - min(p,q)) / (1 - gamma)  (Appendix, definition of p_res)."""
    lw = residual_logweights(logp, logq)
    w = np.exp(lw - np.max(lw))
    return w / np.sum(w)


def accept_block_sampling(logp, logq, yhat, rng, pos0, bonus=False):
    """Lines "for i = 1..k" of Algorithm 1 under reading R1 (stop at the first rejection).

    logp[k][V] = log p_AR(. | x_{1:j+i-1}) with the draft prefix, logq[k][V] = log q_theta(. |
    x_{1:j}); yhat[k] the drafted tokens; pos0 = 0-indexed position of y^_1 (= j).
    Returns (a, correction): a accepted drafts, then the residual sample, or None if a == k.

    bonus (an extension beside Algorithm 1, off by default): logp has a (k+1)-th row, log p_AR(. |
    x_{1:j}, y^_1..y^_k), and when all k drafts are accepted one more token is drawn from it.  No draft
    stands at that position, so the residual of Eq. "resample" with q = 0 is p itself; the Appendix
    Theorem's induction step applies unchanged (a draw from p given an exactly distributed prefix)."""
    k = len(yhat)
    for i in range(k):
        y = int(yhat[i])
        if rng.accept(log_alpha(logp[i, y], logq[i, y]), pos0 + i):
            continue
        c = rng.categorical(residual_logweights(logp[i], logq[i]), pos0 + i, TAG_RESID)
        return i, int(c)
    if bonus:
        return k, int(rng.categorical(logp[k], pos0 + k, TAG_RESID))
    return k, None


def accept_block_greedy(target_argmax, yhat, bonus=False):
    """T = 0 limit (reading R5): q is one-hot at y^_i and p one-hot at the target's argmax, so
    alpha_i = [y^_i == argmax] and the residual is one-hot at the argmax.  With bonus, target_argmax
    has k+1 entries and the last one is committed after k accepted drafts."""
    k = len(yhat)
    for i in range(k):
        if int(yhat[i]) != int(target_argmax[i]):
            return i, int(target_argmax[i])
    if bonus:
        return k, int(target_argmax[k])
    return k, None


# =============================================================================================
# model interface used by the loop, and its transformer realisation
# =============================================================================================


class TransformerPair:
    """One sequence's state: committed tokens x, target cache (x_{1:j-1}), drafter cache.

    Invariant (reading R2): the target cache holds every committed token except the last one,
    which is "pending" - it is the first row of the next verify pass.  The drafter cache holds
    the committed tokens it has ingested; the rest ride along with the next draft pass."""

    def __init__(self, target: Decoder, drafter: Decoder, mask_id, capacity):
        self.t, self.d = target, drafter
        self.mask_id = int(mask_id)
        self.tc = KVCache(target.s, capacity, target.dtype)
        self.dc = KVCache(drafter.s, capacity, drafter.dtype)
        self.x = []

    def prefill(self, prompt):
        self.x = [int(t) for t in prompt]
        n = len(self.x)
        self.tc.n = 0
        self.dc.n = 0
        if n > 1:
            self.t.forward(self.x[:-1], np.arange(n - 1), self.tc, causal_mask(n - 1), n - 1, logits_rows=[])
        self.d.forward(self.x, np.arange(n), self.dc, causal_mask(n), n, logits_rows=[])

    def draft_logits(self, k, fixed=()):
        """z^d_i, i=1..k: one drafter pass over the not-yet-cached committed rows plus k block rows.
        The block rows hold the MASK id, except the first len(fixed) ones, which hold the tokens `fixed`
        (a partially filled block, see draft_block_multipass); every block row sees the whole block."""
        j = len(self.x)
        m = j - self.dc.n
        ids = self.x[self.dc.n:] + [int(t) for t in fixed] + [self.mask_id] * (k - len(fixed))
        pos = np.arange(self.dc.n, j + k)
        return self.d.forward(ids, pos, self.dc, drafter_block_mask(m, k), m, logits_rows=np.arange(m, m + k))

    def verify_logits(self, yhat, bonus=False):
        """z^t_i, i=1..k: one target pass over rows [x_j, y^_1 .. y^_{k-1}], causal in the block.
        All k rows' K,V are written; commit() rolls the cache length back.
        bonus: the last draft y^_k is a row too (k+1 rows), so the pass also yields z^t_{k+1}."""
        j = len(self.x)
        k = len(yhat)
        assert self.tc.n == j - 1
        ids = [self.x[-1]] + [int(t) for t in (yhat if bonus else yhat[:-1])]
        n = len(ids)
        return self.t.forward(ids, np.arange(j - 1, j - 1 + n), self.tc, causal_mask(n), n)

    def commit(self, tokens):
        """Append the committed tokens; the target cache rolls back to (new length - 1)."""
        self.x.extend(int(t) for t in tokens)
        self.tc.truncate(len(self.x) - 1)

    def prefix(self):
        return list(self.x)


def multipass_bounds(k, n_passes):
    """Positions fixed after pass s = 1..n_passes of a multi-pass draft: the first ceil(k * s / n_passes)."""
    return [-((-k * s) // n_passes) for s in range(n_passes + 1)]


def draft_block_multipass(pair, k, T, rng, n_passes):
    """Block regeneration (Sec. "Generative Capabilities": the drafter takes a partially masked block and fills
    in the rest) used as a multi-pass draft: pass s sees the tokens fixed so far at the first hi_{s-1} block
    positions and MASK at the others, and fixes positions hi_{s-1} .. hi_s - 1 (left to right, equal shares).
    Position i's token and the logits that define its law q_i are those of the pass that fixed it, so q_i
    depends on x_{1:j} and on drafts at EARLIER positions only - the condition under which the acceptance rule
    of Eq. "accept"/"resample" stays exact.  n_passes = 1 is the one-pass draft of Sec. 3.2.
    Returns (tokens[k], logits[k][V])."""
    j = len(pair.prefix())
    hi = multipass_bounds(k, n_passes)
    yhat, rows = [], []
    for s in range(1, n_passes + 1):
        if hi[s] == hi[s - 1]:
            continue
        z = pair.draft_logits(k, yhat)
        for i in range(hi[s - 1], hi[s]):
            rows.append(z[i])
            yhat.append(argmax_lowest(z[i]) if T == 0.0 else rng.categorical(z[i] / T, j + i, TAG_DRAFT))
    return yhat, np.stack(rows)


def deer_iteration(pair, k, T, rng, eos_id=-1, draft_override=None, bonus=False, n_draft_passes=1):
    """One pass of Algorithm 1's while-body.  Returns a dict with the drafted block, accepted
    length a, committed tokens, and the two logit blocks (for parity checks).

    draft_override: tokens to use instead of the drafter's own pick (tests inject blocks that
    force a given accepted length; random-init drafters are almost never accepted at T=0).
    bonus: verify k+1 rows and commit a (k+1)-th target token after k accepted drafts."""
    j = len(pair.prefix())
    if n_draft_passes > 1:
        yhat, zd = draft_block_multipass(pair, k, T, rng, n_draft_passes)
    else:
        zd = pair.draft_logits(k)
        if T == 0.0:
            yhat = [argmax_lowest(zd[i]) for i in range(k)]
        else:
            yhat = [rng.categorical(zd[i] / T, j + i, TAG_DRAFT) for i in range(k)]
    if draft_override is not None:
        yhat = [int(t) for t in draft_override]
    zt = pair.verify_logits(yhat, bonus)
    if T == 0.0:
        a, c = accept_block_greedy([argmax_lowest(zt[i]) for i in range(len(zt))], yhat, bonus)
    else:
        a, c = accept_block_sampling(log_softmax(zt / T), log_softmax(zd / T), yhat, rng, j, bonus)
    committed = list(yhat[:a]) + ([] if c is None else [c])
    if eos_id >= 0 and eos_id in committed:
        committed = committed[: committed.index(eos_id) + 1]
    pair.commit(committed)
    return dict(draft=yhat, accept_len=a, committed=committed, draft_logits=zd, target_logits=zt)


def deer_decode(pair, prompt, k, T, n_new, rng, eos_id=-1, bonus=False):
    """Algorithm 1: repeat draft -> verify -> accept until n_new tokens (or EOS) are committed."""
    pair.prefill(prompt)
    out, accepts = [], []
    while len(out) < n_new:
        it = deer_iteration(pair, k, T, rng, eos_id, bonus=bonus)
        out.extend(it["committed"])
        accepts.append(it["accept_len"])
        if eos_id >= 0 and eos_id in it["committed"]:
            break
    return out[:n_new], accepts


# =============================================================================================
# the plain definitions the method must reproduce
# =============================================================================================


def ar_decode(target: Decoder, prompt, n_new, T=0.0, rng=None, capacity=None):
    """Ordinary autoregressive decoding of the target, one token per forward pass: greedy at
    T=0, ancestral sampling (same Gumbel-max generator, TAG_RESID unused) otherwise."""
    x = [int(t) for t in prompt]
    cap = capacity or (len(x) + n_new + 1)
    cache = KVCache(target.s, cap, target.dtype)
    z = target.forward(x, np.arange(len(x)), cache, causal_mask(len(x)), len(x), logits_rows=[len(x) - 1])[0]
    out = []
    for _ in range(n_new):
        if T == 0.0:
            t = argmax_lowest(z)
        else:
            t = rng.categorical(z / T, len(x), TAG_DRAFT)
        out.append(t)
        x.append(t)
        z = target.forward([t], [len(x) - 1], cache, causal_mask(1), 1)[0]
    return out


# =============================================================================================
# the same loop over abstract conditional tables (used by the enumeration pins)
# =============================================================================================


def deer_iteration_tabular(prefix, k, target_logp, drafter_logq, rng, bonus=False, n_draft_passes=1):
    """Algorithm 1's while-body with the two models given as functions:
    target_logp(prefix_list) -> log p_AR(. | prefix); drafter_logq(prefix_list, i) -> log
    q_theta(x_{j+i} = . | x_{1:j}), i = 1..k.  rng supplies draft_token / accept / residual.
    n_draft_passes > 1: pass s conditions the drafter on the drafts fixed so far, given to it as an extended
    prefix: position i (past hi_{s-1} fixed ones) has the law drafter_logq(prefix + fixed, i - hi_{s-1})."""
    j = len(prefix)
    hi = multipass_bounds(k, n_draft_passes)
    yhat, logq = [], []
    for s in range(1, n_draft_passes + 1):
        fixed = list(yhat)
        for i in range(hi[s - 1], hi[s]):
            logq.append(drafter_logq(list(prefix) + fixed, i + 1 - len(fixed)))
            yhat.append(rng.categorical(logq[i], j + i, TAG_DRAFT))
    logq = np.stack(logq)
    logp = np.stack([target_logp(list(prefix) + yhat[:i]) for i in range(k + (1 if bonus else 0))])
    a, c = accept_block_sampling(logp, logq, yhat, rng, j, bonus)
    return list(yhat[:a]) + ([] if c is None else [c]), a
