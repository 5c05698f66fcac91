"""CPU oracle for the greedy self-speculative decode round with DEL statistics.

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, independent implementation
used only by the tests, by the smoke check and by the benchmark's CPU-baseline
leg.  It shares no code with the HIP library and is never on a product path.

What it computes, and the passage of the paper (DEL, arXiv 2504.05598) each part
follows:

* decoder forward, h^l = Transformer_l(h^{l-1}), token = argmax LM-Head(h^L)
  (Section 2, "Auto-regressive decoding").  The paper treats the block as a
  black box; the block here is the pre-norm Llama block (RMSNorm, rotary
  embedding in the rotate-half pairing, grouped-query causal attention with
  scale 1/sqrt(head_dim), SwiGLU feed-forward, no biases).
* greedy speculative acceptance: compare top-1 of draft and target
  (Section 2, "Speculative decoding", greedy special case).
* early-exit self-speculation: draft with the first E layers + LM head, verify
  with the remaining layers, shared KV cache (Section 2, "Early-exit
  self-speculative decoding"; Section 1 on reusing hidden states).
* shadow tokens, first-mismatch index u_r, matched counts c_r^l
  (Section 4.2), decayed sums S and acceptance rates alpha_l (Eq. 2),
  Token-per-Layer (Eq. 1) and the arg-max selection of (E, gamma)
  (Section 4.3; Algorithm 1, DEL_Update).

Precision: every floating-point step runs in `dtype` (float64 by default;
float32 is offered for the full-size shapes).  Weights are the bf16 (or fp32)
values widened exactly.  Two decisions are taken in the kernel's precision so
that both sides decide alike: keys and values are rounded to the KV-cache
dtype when they are stored, and logits are rounded to fp32 before the arg-max
(lowest index wins a tie).

Readings of points the paper leaves open (all "parity unpinned" by the paper;
the pins in tests/ cover the mathematics around them):
  R1  alpha_l = S(c^l) / S(n) with n_r = u_r + 1, the number of valid positions
      (Section 4.2 calls the denominator the length of the valid context).
  R2  u_r compares the draft layer E with layer L (text of Section 4.2; the
      listing's superscript is taken as a typo).
  R3  the last drafted token runs the first E layers once more so that
      gamma+1 exit states exist; verify then runs layers E+1..L on gamma+1 rows.
  R5  the final RMSNorm gain is applied before the LM head at every exit layer.
  R6  prefill enters the statistics as one pseudo-round over the last
      min(32, P) prompt positions, each layer's shadow token compared with
      layer L's.
  R8  arg-max ties: smallest layer, then smallest d (strict > while scanning
      l ascending, d ascending).
  R9  TPL's numerator is evaluated as the sum over i of alpha^i (the form given
      below Eq. 1), which is also defined at alpha = 1.
  R18 dynamic draft-exiting (Section 4.4, Eq. 3; Algorithm 1 loop): the confidence
      of a token is its soft-max probability at temperature 1; drafting runs up
      to d_max steps and stops before appending a token whose confidence is
      below tau_E; the hidden state of the stopping step is the round's last
      row.  In Eq. 3 the mismatched count is n - c (reading R1) and a ratio
      whose denominator is zero (no matched, or no mismatched, token seen yet)
      counts as 0.
  R19 speculative sampling (Section 2, "Speculative decoding"; Appendix on the
      inference setup: temperature and top_p).  The paper names temperature and
      top_p and leaves their definition to the sampling library; here a logits
      row becomes a distribution by soft-max of logits/temperature, then the
      nucleus: tokens ordered by falling logit (lower id first among equals),
      the shortest leading run whose mass reaches top_p is kept and
      renormalised.  A uniform number r in [0, 1) picks the first token, in
      token-id order, whose cumulative probability exceeds r.  A drafted token
      x is accepted when r * q(x) < p(x), which accepts with probability
      min(1, p(x)/q(x)); after the first rejection the next token comes from
      max(0, p - q) renormalised, and after gamma acceptances from p at the
      last position.  The uniform numbers are inputs (gamma for the drafts,
      gamma for the acceptances, one for the last token).  All of this runs in
      fp64 on the fp32-rounded logits.
  R21 dynamic draft-exiting under sampling: the confidence of a draft step is, as
      in R18, the temperature-1 soft-max probability of the exit layer's greedy
      token (the quantity tau_l is built from); a step below tau_E stops the
      drafting before its token is drawn.
  R20 statistics under sampling: shadow tokens are greedy at every layer,
      layer L included (Section 4.2 obtains them by greedy decoding), u_r is
      the number of drafted tokens the sampling rule accepted, and c^l, tcs^l,
      fcs^l compare layer l's shadow tokens with layer L's over rows 0..u_r.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import math
import torch


# --------------------------------------------------------------------------
# DEL policy: statistics and selection (Sections 4.1-4.3, Eq. 1, Eq. 2)
# --------------------------------------------------------------------------

def decayed_sum(a: Sequence[float], omega: float) -> float:
    """S(a) = sum_{i=0}^{r-1} omega^(r-i-1) a[i]  (Section 4.2)."""
    r = len(a)
    total = 0.0
    for i in range(r):
        total += (omega ** (r - i - 1)) * float(a[i])
    return total


def tpl(alpha: float, l: int, d: int, n_layers: int) -> float:
    """Token-per-Layer, Eq. 1, with the numerator as sum_{i=0}^{d} alpha^i."""
    num = 0.0
    p = 1.0
    for _ in range(d + 1):
        num += p
        p *= alpha
    return num / (d * l + n_layers)


def select_exit_and_length(alpha: Sequence[float], n_layers: int, d_max: int) -> Tuple[int, int]:
    """(E, gamma) = argmax over l in [1, L), d in [0, d_max] of TPL(l, d).

    alpha is indexed by layer number (alpha[0] unused).  Section 4.3.
    """
    best = -1.0
    best_l, best_d = 1, 0
    for l in range(1, n_layers):
        for d in range(0, d_max + 1):
            v = tpl(alpha[l], l, d, n_layers)
            if v > best:
                best, best_l, best_d = v, l, d
    return best_l, best_d


def first_mismatch(draft_layer_tokens: Sequence[int], target_tokens: Sequence[int], gamma: int) -> int:
    """u_r: first i in [0, gamma) where the draft and the target token differ, else gamma.

    Position gamma holds no drafted token, so it cannot reject (Section 2).
    """
    for i in range(gamma):
        if int(draft_layer_tokens[i]) != int(target_tokens[i]):
            return i
    return gamma


def confidence_sums(shadow: Sequence[Sequence[int]], conf: Sequence[Sequence[float]],
                    target: Sequence[int], u: int) -> Tuple[List[float], List[float]]:
    """tcs^l, fcs^l: confidence of layer l's shadow tokens at positions 0..u, summed over the
    matched and over the mismatched ones (Section 4.4); index 0 unused."""
    tcs, fcs = [0.0], [0.0]
    for l in range(1, len(shadow)):
        t = f = 0.0
        for i in range(u + 1):
            if int(shadow[l][i]) == int(target[i]):
                t += float(conf[l][i])
            else:
                f += float(conf[l][i])
        tcs.append(t)
        fcs.append(f)
    return tcs, fcs


def matched_counts(shadow: Sequence[Sequence[int]], target: Sequence[int], u: int) -> List[int]:
    """c^l = sum_{i=0}^{u} 1(shadow[l][i] == target[i]); index 0 unused (Section 4.2)."""
    out = [0]
    for l in range(1, len(shadow)):
        out.append(sum(1 for i in range(u + 1) if int(shadow[l][i]) == int(target[i])))
    return out


# --------------------------------------------------------------------------
# Speculative sampling (Section 2, "Speculative decoding"; reading R19)
# --------------------------------------------------------------------------

def tempered_nucleus(logits: torch.Tensor, temperature: float, top_p: float) -> torch.Tensor:
    """Distribution a logits row is sampled from: soft-max(logits / temperature) restricted to the
    nucleus of mass top_p and renormalised.  fp64 on the fp32-rounded logits."""
    assert temperature > 0.0 and 0.0 < top_p
    z = logits.reshape(-1).to(torch.float32).to(torch.float64)
    p = torch.softmax(z / temperature, dim=0)
    if top_p >= 1.0:
        return p
    order = torch.sort(-z, stable=True).indices          # falling logit, lower id first among equals
    cum = torch.cumsum(p[order], dim=0)
    reached = torch.nonzero(cum >= top_p)
    k = int(reached[0, 0]) if reached.numel() else z.numel() - 1
    kept = order[:k + 1]
    out = torch.zeros_like(p)
    out[kept] = p[kept]
    return out / out.sum()


def inverse_cdf(p: torch.Tensor, r: float) -> int:
    """First token, in id order, whose cumulative mass exceeds r times the total mass."""
    assert 0.0 <= r < 1.0
    cdf = torch.cumsum(p.to(torch.float64), dim=0)
    over = torch.nonzero(cdf > r * cdf[-1])
    if over.numel():
        return int(over[0, 0])
    return int(torch.nonzero(p > 0)[-1, 0])


def residual_distribution(p: torch.Tensor, q: torch.Tensor) -> torch.Tensor:
    """max(0, p - q), renormalised: what a rejected position is resampled from."""
    res = torch.clamp(p - q, min=0.0)
    total = res.sum()
    return res / total if float(total) > 0.0 else p.clone()


def speculative_accept(drafts: Sequence[int], q: Sequence[torch.Tensor], p: Sequence[torch.Tensor],
                       r_accept: Sequence[float], r_last: float) -> Tuple[int, int, torch.Tensor]:
    """Acceptance of gamma = len(drafts) drafted tokens.  q[i] is the distribution drafts[i] was drawn
    from, p[0..gamma] the target's distributions.  Returns (u, token, dist): u drafted tokens are
    accepted and `token`, drawn from `dist` with r_last, follows them."""
    gamma = len(drafts)
    assert len(q) == gamma and len(p) == gamma + 1 and len(r_accept) >= gamma
    for i in range(gamma):
        x = int(drafts[i])
        if not float(r_accept[i]) * float(q[i][x]) < float(p[i][x]):
            dist = residual_distribution(p[i], q[i])
            return i, inverse_cdf(dist, r_last), dist
    return gamma, inverse_cdf(p[gamma], r_last), p[gamma]


class DelStats:
    """Per-round lists c, n and the quantities derived from them."""

    def __init__(self, n_layers: int, omega: float, d_max: int):
        self.L = n_layers
        self.omega = omega
        self.d_max = d_max
        self.c_hist: List[List[int]] = []   # one [L+1] list per round
        self.n_hist: List[int] = []
        self.u_hist: List[int] = []
        self.tcs_hist: List[List[float]] = []   # confidence summed over matched shadow tokens
        self.fcs_hist: List[List[float]] = []   # ... over mismatched ones

    def append(self, c: Sequence[int], n: int, u: int,
               tcs: Optional[Sequence[float]] = None, fcs: Optional[Sequence[float]] = None) -> None:
        assert len(c) == self.L + 1
        self.c_hist.append([int(x) for x in c])
        self.n_hist.append(int(n))
        self.u_hist.append(int(u))
        self.tcs_hist.append([float(x) for x in (tcs if tcs is not None else [0.0] * (self.L + 1))])
        self.fcs_hist.append([float(x) for x in (fcs if fcs is not None else [0.0] * (self.L + 1))])

    def S_tcs(self, l: int) -> float:
        return decayed_sum([t[l] for t in self.tcs_hist], self.omega)

    def S_fcs(self, l: int) -> float:
        return decayed_sum([t[l] for t in self.fcs_hist], self.omega)

    def tau(self) -> List[float]:
        """Dynamic threshold, Eq. 3: midpoint of the decayed mean confidence of matched and of
        mismatched shadow tokens; a ratio with a zero denominator counts as 0."""
        out = [0.0]
        sn = self.S_n()
        for l in range(1, self.L + 1):
            sc = self.S_c(l)
            sm = sn - sc                       # S(n - c): S is linear
            a = self.S_tcs(l) / sc if sc > 0.0 else 0.0
            b = self.S_fcs(l) / sm if sm > 0.0 else 0.0
            out.append(0.5 * (a + b))
        return out

    def S_c(self, l: int) -> float:
        return decayed_sum([c[l] for c in self.c_hist], self.omega)

    def S_n(self) -> float:
        return decayed_sum(self.n_hist, self.omega)

    def alpha(self) -> List[float]:
        sn = self.S_n()
        return [0.0] + [self.S_c(l) / sn for l in range(1, self.L + 1)]

    def select(self) -> Tuple[int, int]:
        return select_exit_and_length(self.alpha(), self.L, self.d_max)


# --------------------------------------------------------------------------
# Decoder arithmetic
# --------------------------------------------------------------------------

def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x * torch.rsqrt(ms + eps) * gain


def rope_rotate(x: torch.Tensor, positions: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary embedding, rotate-half pairing: element j pairs with j + hd/2.

    x: [rows, heads, hd]; positions: [rows] absolute positions.
    angle(p, j) = p * theta^(-2j/hd) for j in [0, hd/2).
    """
    hd = x.shape[-1]
    half = hd // 2
    j = torch.arange(half, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * j / hd)
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]
    cos = torch.cos(ang).to(x.dtype)[:, None, :]
    sin = torch.sin(ang).to(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


@dataclass
class RoundRecord:
    E: int
    gamma: int
    T_before: int
    draft_ids: List[int]
    target_ids: List[int]            # x^L_{t..t+gamma}
    u: int
    n: int
    out_tokens: List[int]            # x^L_t .. x^L_{t+u}
    shadow: List[List[int]]          # [L+1][gamma+1]; row 0 unused (zeros)
    gaps: List[List[float]]          # top-2 logit gap of every shadow arg-max
    c: List[int]                     # [L+1]
    alpha: List[float]               # after the update
    S_c: List[float]
    S_n: float
    next_E: int
    next_gamma: int
    hidden: Optional[torch.Tensor] = None   # [L+1, gamma+1, d] if kept
    conf: Optional[List[List[float]]] = None        # confidence of every shadow token [L+1][gamma+1]
    draft_conf: Optional[List[float]] = None        # confidence of each draft step taken (incl. a stopping one)
    stopped_early: bool = False                     # the draft loop broke on low confidence
    tcs: Optional[List[float]] = None
    fcs: Optional[List[float]] = None
    tau: Optional[List[float]] = None               # thresholds after the update
    S_tcs: Optional[List[float]] = None
    S_fcs: Optional[List[float]] = None
    # speculative sampling only (reading R19): the distributions every decision was taken from
    q_dists: Optional[List[torch.Tensor]] = None    # [gamma] draft distributions
    p_dists: Optional[List[torch.Tensor]] = None    # [gamma+1] target distributions
    last_dist: Optional[torch.Tensor] = None        # what the round's last token was drawn from
    uniforms: Optional[List[float]] = None


@dataclass
class PrefillRecord:
    first_token: int
    first_gap: float
    window: int
    shadow: List[List[int]]          # [L+1][window]
    gaps: List[List[float]]
    c: List[int]
    alpha: List[float]
    next_E: int
    next_gamma: int
    hidden: Optional[torch.Tensor] = None   # [L+1, window, d]
    conf: Optional[List[List[float]]] = None
    tau: Optional[List[float]] = None


class Oracle:
    """Decoder + KV cache + self-speculative round + DEL statistics."""

    def __init__(self, cfg, weights: Dict[Tuple[int, str], torch.Tensor],
                 dtype: torch.dtype = torch.float64, kv_dtype: Optional[str] = None,
                 max_context: Optional[int] = None, cache_widened: bool = True):
        self.cfg = cfg
        self.w = weights
        self.dtype = dtype
        self.kv_dtype = kv_dtype or ("bf16" if cfg.weight_dtype == "bf16" else "fp32")
        self.L = cfg.n_layers
        self.max_context = max_context or cfg.max_context
        self._cache: Dict[Tuple[int, str], torch.Tensor] = {}
        self._cache_on = cache_widened
        self.reset()

    # ---- state ----
    def reset(self) -> None:
        c = self.cfg
        shape = (self.max_context, c.n_kv_heads, c.head_dim)
        self.K = [None] + [torch.zeros(shape, dtype=self.dtype) for _ in range(self.L)]
        self.V = [None] + [torch.zeros(shape, dtype=self.dtype) for _ in range(self.L)]
        self.T = 0
        self.pending: Optional[int] = None
        self.stats = DelStats(self.L, c.omega, c.d_max)

    def W(self, layer: int, kind: str) -> torch.Tensor:
        if kind == "lm_head" and self.cfg.tied_embeddings:
            layer, kind = -1, "embed"
        key = (layer, kind)
        if key in self._cache:
            return self._cache[key]
        t = self.w[key].to(self.dtype)
        if kind.endswith("norm"):
            t = t.reshape(-1)
        if self._cache_on:
            self._cache[key] = t
        return t

    def _store_round(self, x: torch.Tensor) -> torch.Tensor:
        """Round to the KV-cache storage type (the kernel stores bf16 from fp32)."""
        if self.kv_dtype == "bf16":
            return x.to(torch.float32).to(torch.bfloat16).to(self.dtype)
        return x.to(torch.float32).to(self.dtype)

    # ---- model pieces ----
    def embed(self, token: int) -> torch.Tensor:
        return self.w[(-1, "embed")][int(token)].to(self.dtype)

    def layer(self, l: int, h: torch.Tensor, pos0: int) -> torch.Tensor:
        """Transformer_l on rows h [m, d] at positions pos0..pos0+m-1; l in 1..L.

        Appends the rows' keys and values to the cache of layer l; row i attends
        to cache rows 0..pos0+i.
        """
        c = self.cfg
        li = l - 1
        m = h.shape[0]
        nq, nkv, hd = c.n_q_heads, c.n_kv_heads, c.head_dim
        group = nq // nkv
        a = rmsnorm(h, self.W(li, "attn_norm"), c.rms_eps)
        q = (a @ self.W(li, "wq").T).view(m, nq, hd)
        k = (a @ self.W(li, "wk").T).view(m, nkv, hd)
        v = (a @ self.W(li, "wv").T).view(m, nkv, hd)
        pos = torch.arange(pos0, pos0 + m)
        q = rope_rotate(q, pos, c.rope_theta)
        k = rope_rotate(k, pos, c.rope_theta)
        self.K[l][pos0:pos0 + m] = self._store_round(k)
        self.V[l][pos0:pos0 + m] = self._store_round(v)
        n_ctx = pos0 + m
        keys = self.K[l][:n_ctx]                      # [n_ctx, nkv, hd]
        vals = self.V[l][:n_ctx]
        keys = keys.repeat_interleave(group, dim=1)   # q head j reads kv head j // group
        vals = vals.repeat_interleave(group, dim=1)
        scores = torch.einsum("mhd,thd->hmt", q, keys) / math.sqrt(hd)
        t_idx = torch.arange(n_ctx)[None, None, :]
        allowed = t_idx <= pos[None, :, None]
        scores = scores.masked_fill(~allowed, float("-inf"))
        p = torch.softmax(scores, dim=-1)
        o = torch.einsum("hmt,thd->mhd", p, vals).reshape(m, nq * hd)
        h1 = h + o @ self.W(li, "wo").T
        b = rmsnorm(h1, self.W(li, "ffn_norm"), c.rms_eps)
        act = silu(b @ self.W(li, "wg").T) * (b @ self.W(li, "wu").T)
        return h1 + act @ self.W(li, "wd").T

    def logits(self, h: torch.Tensor) -> torch.Tensor:
        """LM head applied after the final RMSNorm; h [rows, d] -> [rows, vocab]."""
        x = rmsnorm(h, self.W(-1, "final_norm"), self.cfg.rms_eps)
        return x @ self.W(-1, "lm_head").T

    def head(self, h: torch.Tensor) -> Tuple[List[int], List[float]]:
        """Greedy token and top-2 logit gap per row."""
        ids, gaps, _ = self.head_conf(h)
        return ids, gaps

    def head_conf(self, h: torch.Tensor) -> Tuple[List[int], List[float], List[float]]:
        """Greedy token, top-2 logit gap and confidence (soft-max probability of the greedy
        token, Section 4.4) per row."""
        lg = self.logits(h)
        lg32 = lg.to(torch.float32)
        lse = torch.logsumexp(lg, dim=-1)
        ids, gaps, conf = [], [], []
        for r in range(lg32.shape[0]):
            row = lg32[r]
            top = row.max()
            idx = int(torch.nonzero(row == top)[0, 0])   # lowest index on ties
            two = torch.topk(lg[r], 2).values
            ids.append(idx)
            gaps.append(float(two[0] - two[1]))
            conf.append(float(torch.exp(lg[r, idx] - lse[r])))
        return ids, gaps, conf

    # ---- prefill ----
    def prefill(self, prompt: Sequence[int], keep_hidden: bool = False) -> PrefillRecord:
        self.reset()
        P = len(prompt)
        assert 0 < P <= self.max_context
        h = torch.stack([self.embed(t) for t in prompt])
        w = min(self.cfg.prefill_window, P)
        hid = torch.zeros((self.L + 1, w, self.cfg.d_model), dtype=self.dtype)
        hid[0] = h[P - w:]
        for l in range(1, self.L + 1):
            h = self.layer(l, h, 0)
            hid[l] = h[P - w:]
        self.T = P
        self._last_row = hid[self.L, w - 1].clone()
        shadow = [[0] * w]
        gaps = [[0.0] * w]
        conf = [[0.0] * w]
        for l in range(1, self.L + 1):
            ids, g, cf = self.head_conf(hid[l])
            shadow.append(ids)
            gaps.append(g)
            conf.append(cf)
        target = shadow[self.L]
        c = matched_counts(shadow, target, w - 1)
        tcs, fcs = confidence_sums(shadow, conf, target, w - 1)
        self.stats.append(c, w, w - 1, tcs, fcs)
        first = target[w - 1]
        self.pending = first
        E, gamma = self.stats.select()
        return PrefillRecord(first, gaps[self.L][w - 1], w, shadow, gaps, c,
                             self.stats.alpha(), E, gamma, hid if keep_hidden else None,
                             conf, self.stats.tau())

    # ---- one self-speculative round ----
    def round(self, E: int, gamma: int, keep_hidden: bool = False,
              tau: Optional[float] = None) -> RoundRecord:
        """One self-speculative round.  tau = None: draft exactly `gamma` tokens.  Otherwise
        dynamic draft-exiting (Section 4.4; Algorithm 1 loop): draft up to `gamma` (= d_max)
        tokens and stop, before appending, at the first token whose confidence is below tau."""
        L, d = self.L, self.cfg.d_model
        assert 1 <= E <= L and 0 <= gamma
        assert self.pending is not None, "prefill first"
        T = self.T
        assert T + gamma + 1 <= self.max_context
        hid = torch.zeros((L + 1, gamma + 1, d), dtype=self.dtype)
        # draft: auto-regressive steps through the first E layers
        drafts: List[int] = []
        draft_conf: List[float] = []
        stopped = False
        tok = self.pending
        for i in range(gamma):
            h = self.embed(tok)[None, :]
            hid[0, i] = h[0]
            for l in range(1, E + 1):
                h = self.layer(l, h, T + i)
                hid[l, i] = h[0]
            ids, _, cf = self.head_conf(hid[E, i][None, :])
            draft_conf.append(cf[0])
            if tau is not None and cf[0] < tau:
                stopped = True                  # not appended; row i is the round's last row
                break
            drafts.append(ids[0])
            tok = ids[0]
        if stopped:
            gamma = len(drafts)
            hid = hid[:, :gamma + 1].clone()
        else:
            # the last pending token passes the first E layers (no head needed)
            h = self.embed(tok)[None, :]
            hid[0, gamma] = h[0]
            for l in range(1, E + 1):
                h = self.layer(l, h, T + gamma)
                hid[l, gamma] = h[0]
        # verify: the gamma+1 exit states pass the remaining layers together
        rows = hid[E].clone()
        for l in range(E + 1, L + 1):
            rows = self.layer(l, rows, T)
            hid[l] = rows
        # shadow tokens of every layer (layer L's are the target's tokens)
        shadow = [[0] * (gamma + 1)]
        gaps = [[0.0] * (gamma + 1)]
        conf = [[0.0] * (gamma + 1)]
        for l in range(1, L + 1):
            ids, g, cf = self.head_conf(hid[l])
            shadow.append(ids)
            gaps.append(g)
            conf.append(cf)
        target = shadow[L]
        u = first_mismatch(drafts, target, gamma)
        n = u + 1
        out = target[:u + 1]
        c = matched_counts(shadow, target, u)
        tcs, fcs = confidence_sums(shadow, conf, target, u)
        self.stats.append(c, n, u, tcs, fcs)
        alpha = self.stats.alpha()
        nE, ng = self.stats.select()
        self.T = T + u + 1
        self.pending = out[-1]
        return RoundRecord(E, gamma, T, drafts, target, u, n, out, shadow, gaps, c, alpha,
                           [0.0] + [self.stats.S_c(l) for l in range(1, L + 1)],
                           self.stats.S_n(), nE, ng, hid if keep_hidden else None,
                           conf, draft_conf, stopped, tcs, fcs, self.stats.tau(),
                           [0.0] + [self.stats.S_tcs(l) for l in range(1, L + 1)],
                           [0.0] + [self.stats.S_fcs(l) for l in range(1, L + 1)])

    # ---- speculative sampling (Section 2; readings R19, R20) ----
    def sample_first(self, temperature: float, top_p: float, r: float) -> Tuple[int, torch.Tensor]:
        """Replace the greedy first token of the prefill by one drawn from the target's
        distribution at the last prompt position."""
        dist = tempered_nucleus(self.logits(self._last_row[None, :])[0], temperature, top_p)
        tok = inverse_cdf(dist, r)
        self.pending = tok
        return tok, dist

    def round_sample(self, E: int, gamma: int, temperature: float, top_p: float,
                     uniforms: Sequence[float], keep_hidden: bool = False,
                     tau: Optional[float] = None) -> RoundRecord:
        """One self-speculative round with sampled drafts and the sampling acceptance rule.
        uniforms: gamma numbers for the drafts, gamma for the acceptances, one for the last token.
        tau: dynamic draft-exiting on top (reading R21): `gamma` is then the cap on the draft length,
        and drafting stops, before a token is drawn, at the first step whose confidence is below tau;
        the uniform numbers keep their places (draft i uses uniforms[i], acceptance i uniforms[gamma+i])."""
        L, d = self.L, self.cfg.d_model
        assert 1 <= E <= L and 0 <= gamma and len(uniforms) >= 2 * gamma + 1
        assert self.pending is not None, "prefill first"
        T = self.T
        assert T + gamma + 1 <= self.max_context
        r_draft = [float(x) for x in uniforms[:gamma]]
        r_acc = [float(x) for x in uniforms[gamma:2 * gamma]]
        r_last = float(uniforms[2 * gamma])
        hid = torch.zeros((L + 1, gamma + 1, d), dtype=self.dtype)
        drafts: List[int] = []
        q_dists: List[torch.Tensor] = []
        draft_conf: List[float] = []
        stopped = False
        tok = self.pending
        for i in range(gamma + 1):
            h = self.embed(tok)[None, :]
            hid[0, i] = h[0]
            for l in range(1, E + 1):
                h = self.layer(l, h, T + i)
                hid[l, i] = h[0]
            if i < gamma:
                if tau is not None:
                    _, _, cf = self.head_conf(hid[E, i][None, :])
                    draft_conf.append(cf[0])
                    if cf[0] < tau:
                        stopped = True          # nothing drawn; row i is the round's last row
                        break
                qd = tempered_nucleus(self.logits(hid[E, i][None, :])[0], temperature, top_p)
                tok = inverse_cdf(qd, r_draft[i])
                q_dists.append(qd)
                drafts.append(tok)
        if stopped:
            gamma = len(drafts)
            hid = hid[:, :gamma + 1].clone()
        rows = hid[E].clone()
        for l in range(E + 1, L + 1):
            rows = self.layer(l, rows, T)
            hid[l] = rows
        shadow = [[0] * (gamma + 1)]
        gaps = [[0.0] * (gamma + 1)]
        conf = [[0.0] * (gamma + 1)]
        for l in range(1, L + 1):
            ids, g, cf = self.head_conf(hid[l])
            shadow.append(ids)
            gaps.append(g)
            conf.append(cf)
        target = shadow[L]
        lgL = self.logits(hid[L])
        p_dists = [tempered_nucleus(lgL[i], temperature, top_p) for i in range(gamma + 1)]
        u, last, last_dist = speculative_accept(drafts, q_dists, p_dists, r_acc, r_last)
        n = u + 1
        out = drafts[:u] + [last]
        c = matched_counts(shadow, target, u)
        tcs, fcs = confidence_sums(shadow, conf, target, u)
        self.stats.append(c, n, u, tcs, fcs)
        alpha = self.stats.alpha()
        nE, ng = self.stats.select()
        self.T = T + u + 1
        self.pending = last
        return RoundRecord(E, gamma, T, drafts, target, u, n, out, shadow, gaps, c, alpha,
                           [0.0] + [self.stats.S_c(l) for l in range(1, L + 1)],
                           self.stats.S_n(), nE, ng, hid if keep_hidden else None,
                           conf, draft_conf if tau is not None else None, stopped, tcs, fcs, self.stats.tau(),
                           [0.0] + [self.stats.S_tcs(l) for l in range(1, L + 1)],
                           [0.0] + [self.stats.S_fcs(l) for l in range(1, L + 1)],
                           q_dists, p_dists, last_dist, [float(x) for x in uniforms])

    # ---- reference definitions used by the pins ----
    def vanilla_step(self) -> int:
        """One auto-regressive step of the full model on the pending token."""
        h = self.embed(self.pending)[None, :]
        for l in range(1, self.L + 1):
            h = self.layer(l, h, self.T)
        ids, _ = self.head(h)
        self.T += 1
        self.pending = ids[0]
        return ids[0]

    def forward_nocache(self, tokens: Sequence[int]) -> torch.Tensor:
        """All-layer hidden states [L+1, n, d] of a full causal forward, no cache reuse.

        Uses a scratch oracle so the caller's cache is untouched.
        """
        tmp = Oracle(self.cfg, self.w, self.dtype, self.kv_dtype,
                     max_context=max(len(tokens), 1), cache_widened=False)
        tmp._cache = self._cache
        h = torch.stack([tmp.embed(t) for t in tokens])
        out = [h]
        for l in range(1, self.L + 1):
            h = tmp.layer(l, h, 0)
            out.append(h)
        return torch.stack(out)


def generate_vanilla(oracle: Oracle, prompt: Sequence[int], n_tokens: int) -> List[int]:
    """Greedy auto-regressive decoding of the full model: the definition of the right tokens."""
    rec = oracle.prefill(prompt)
    toks = [rec.first_token]
    while len(toks) < n_tokens:
        toks.append(oracle.vanilla_step())
    return toks


def generate_fixed(oracle: Oracle, prompt: Sequence[int], n_tokens: int, E: int, gamma: int,
                   ) -> Tuple[List[int], List[RoundRecord]]:
    """Self-speculative decoding with a fixed (E, gamma); gamma is clamped near the end."""
    rec = oracle.prefill(prompt)
    toks = [rec.first_token]
    recs = []
    while len(toks) < n_tokens:
        g = min(gamma, n_tokens - len(toks) - 1)
        r = oracle.round(E, g)
        recs.append(r)
        toks.extend(r.out_tokens)
    return toks, recs


def generate_del(oracle: Oracle, prompt: Sequence[int], n_tokens: int, keep_hidden: bool = False,
                 ) -> Tuple[List[int], PrefillRecord, List[RoundRecord]]:
    """Self-speculative decoding with DEL choosing (E, gamma) every round (Algorithm 1
    without the confidence-threshold break: the paper's DEL-E ablation variant)."""
    pre = oracle.prefill(prompt, keep_hidden)
    toks = [pre.first_token]
    E, gamma = pre.next_E, pre.next_gamma
    recs = []
    while len(toks) < n_tokens:
        g = min(gamma, n_tokens - len(toks) - 1)
        r = oracle.round(E, g, keep_hidden)
        recs.append(r)
        toks.extend(r.out_tokens)
        E, gamma = r.next_E, r.next_gamma
    return toks, pre, recs


def generate_del_full(oracle: Oracle, prompt: Sequence[int], n_tokens: int, keep_hidden: bool = False,
                      ) -> Tuple[List[int], PrefillRecord, List[RoundRecord]]:
    """Algorithm 1 in full: DEL selects the exit layer every round and the draft loop runs up to
    d_max steps, stopping at the first token whose confidence is below tau_E (Section 4.4)."""
    pre = oracle.prefill(prompt, keep_hidden)
    toks = [pre.first_token]
    E, tau = pre.next_E, pre.tau[pre.next_E]
    recs = []
    while len(toks) < n_tokens:
        cap = min(oracle.cfg.d_max, n_tokens - len(toks) - 1)
        r = oracle.round(E, cap, keep_hidden, tau=tau)
        recs.append(r)
        toks.extend(r.out_tokens)
        E, tau = r.next_E, r.tau[r.next_E]
    return toks, pre, recs


def generate_sample(oracle: Oracle, prompt: Sequence[int], n_tokens: int, temperature: float, top_p: float,
                    uniforms_for, keep_hidden: bool = False, schedule=None, dynamic: bool = False,
                    ) -> Tuple[List[int], PrefillRecord, List[RoundRecord]]:
    """Speculative sampling with DEL choosing (E, gamma) every round (or schedule(round) if given).
    uniforms_for(k, count) returns the uniform numbers of draw k: k = 0 is the first token (one
    number), k = r + 1 is round r (2 * gamma + 1 numbers).  dynamic: draft-exiting on top
    (Algorithm 1 in full): gamma is d_max and the draft loop stops on tau_E."""
    pre = oracle.prefill(prompt, keep_hidden)
    first, _ = oracle.sample_first(temperature, top_p, float(uniforms_for(0, 1)[0]))
    toks = [first]
    E, gamma = pre.next_E, pre.next_gamma
    recs = []
    while len(toks) < n_tokens:
        if schedule is not None:
            E, gamma = schedule(len(recs))
        g = min(oracle.cfg.d_max if dynamic else gamma, n_tokens - len(toks) - 1)
        tau = (recs[-1].tau[E] if recs else pre.tau[E]) if dynamic else None
        r = oracle.round_sample(E, g, temperature, top_p, uniforms_for(len(recs) + 1, 2 * g + 1), keep_hidden,
                                tau=tau)
        recs.append(r)
        toks.extend(r.out_tokens)
        E, gamma = r.next_E, r.next_gamma
    return toks, pre, recs


def empirical_tpl(records: Sequence[RoundRecord], n_layers: int) -> float:
    """eTPL = generated tokens / loaded layers, with gamma*E + L layers per round
    (Section 4.1 cost estimate; Appendix B.4)."""
    tokens = sum(len(r.out_tokens) for r in records)
    layers = sum(r.gamma * r.E + n_layers for r in records)
    return tokens / layers


def load_weights(cfg, device="cpu") -> Dict[Tuple[int, str], torch.Tensor]:
    """All tensors of a synthetic model from the shared seeded generator."""
    from synthdata import gen_tensor, iter_tensor_specs
    out = {}
    for layer, kind in iter_tensor_specs(cfg):
        t = gen_tensor(cfg, layer, kind, device=device)
        out[(layer, kind)] = t.cpu()
    return out
