"""CPU oracle, part 2: the HiViS draft-verify cycle (float64, numpy): greedy (temperature 0)
and, at the end of the file, with tokens drawn at a temperature T > 0 (speculative sampling).

TEST INFRASTRUCTURE ONLY (see oracle/model.py).  Follows Algorithm 1 of the paper
("Residual-Aided Drafting and Verification Process") step by step, in its notation:

  prefill   f_fused^{1:l}, x_{l+1}  <-  Prefill(M_p; e_visual^{1:v}, e_text^{1:l})
  fusion    e^_{j+1} = f^j w1 + Embed(x_{j+1}) w2          (section 3.2, fusion formula)
  residual  every input row built from a TRUE target feature gets r^0 w; the input row
            built from the drafter's own i-th hidden state f'_{l+i} gets r^i w, and r^3
            is reused beyond (Algorithm 1 steps 2-3; Eq. (1)-(2); section 4 training setup)
  draft     lambda (= K here) serial drafter steps, greedy token from the shared LM head
  verify    one target pass over [x_{l+1}, x'_{l+2..l+1+K}] against the full visual+text cache
  accept    longest prefix of drafts equal to the target's greedy tokens, plus the target's
            own next token (section 2.1)
  roll      the accepted positions' TRUE features re-condition the drafter (section 3.3:
            each drafting round starts from fused features supplied by the target)

`rho` below is the folded vector r^i w (r^i is a row vector broadcast over rows and w
is constant at inference, so only the product matters).

Readings taken where the paper is silent are listed in the design notes of this
repository; the ones that shape this file: f_fused is taken AFTER the target's final
norm (it lives in LM-head input space, as the drafter's f' does); drafter positions are
text-local (0..l-1); the drafter's speculative KV rows are discarded after each
verification and rebuilt from true features; the last draft step builds no further input.

`greedy_reference` is the plain definition the method must reproduce exactly at T=0:
ordinary one-token-at-a-time greedy decoding of the target.
"""
import numpy as np

from .model import F64, Target, Drafter, argmax_lowest


def fuse(f, e, fuse_w, rho):
    """Visual-injected text embedding: f w1 + e w2 + rho, with fuse_w = [w1; w2] ([2d][d])."""
    f = np.asarray(f, F64)
    e = np.asarray(e, F64)
    d = f.shape[-1]
    W = np.asarray(fuse_w, F64)
    return f @ W[:d] + e @ W[d:] + np.asarray(rho, F64)


def accept_length(drafts, target_tokens):
    """n = number of leading drafts d_1..d_n with d_i == t_i (t_i = target's greedy token
    for the same position); the first mismatch rejects itself and everything after it."""
    n = 0
    for d_i, t_i in zip(drafts, target_tokens):
        if int(d_i) != int(t_i):
            break
        n += 1
    return n


class HivisOracle:
    """State of one sequence: target, drafter, the text so far, and the drafter's pending
    hidden state f'_1 that the next draft round starts from."""

    def __init__(self, cfg, weights):
        self.cfg = cfg
        self.w = weights
        self.target = Target(cfg, weights)
        self.drafter = Drafter(cfg, weights)
        self.v = 0
        self.text = []            # x_1 .. x_{l+1}: all text tokens known so far (last one not yet in the target cache)
        self.f_next = None        # f'_1 of the coming round: drafter output at its last true-feature row
        self.l = 0                # number of text tokens inside the target cache == drafter KV length between rounds

    # -- helpers -------------------------------------------------------------------
    def rho(self, i):
        return np.asarray(self.w["resid_rho"], F64)[min(i, self.cfg.n_resid - 1)]

    def _refeed(self, feats, next_tokens, start_pos):
        """Drafter rows built from TRUE features feats[j] and the embedding of the token that
        follows each of them; residual r^0 on every row."""
        u = fuse(feats, self.target.embed(next_tokens), self.w["fuse_w"], self.rho(0))
        out = self.drafter.forward(u, start_pos)
        return out[-1]

    # -- Algorithm 1, inputs line + steps 1-2 --------------------------------------------
    def prefill(self, vis_embeds, text_ids, pick=None):
        """Target prefill over [visual ; text]; returns x_{l+1} (emitted) and the logits
        that chose it.  Then the drafter is prefilled over the l text positions only.
        pick: optional function logits -> token replacing the greedy choice of x_{l+1}
        (temperature sampling, or following another implementation's token)."""
        vis = np.asarray(vis_embeds, F64)
        ids = [int(t) for t in text_ids]
        self.v = vis.shape[0]
        l = len(ids)
        x = np.concatenate([vis, self.target.embed(ids)], axis=0)
        f_all = self.target.forward(x, 0)
        f = f_all[self.v:]                                   # f_fused^{1:l}: text rows only
        logits = self.target.logits(f[-1])
        x_next = int(argmax_lowest(logits)) if pick is None else int(pick(logits))
        self.text = ids + [x_next]
        self.l = l
        # e^_{2:l+1} = f^{1:l} w1 + e^{2:l+1} w2, all rows carry r^0
        self.f_next = self._refeed(f, self.text[1:], 0)
        return x_next, logits

    # -- Algorithm 1, the drafting loop ------------------------------------------------
    def draft(self, K, follow=None):
        """K chain drafts.  Returns (tokens [K], logits [K][V]).  If `follow` is given, its
        tokens are fed forward instead of this oracle's own argmax (the logits returned are
        still this oracle's), so that a second implementation's trajectory can be tracked."""
        assert self.drafter.kv_len == self.l
        f_prev = self.f_next
        tokens, logits_all = [], []
        for i in range(1, K + 1):
            logits = self.target.logits(f_prev)              # shared LM head, applied to f' directly
            d_i = int(argmax_lowest(logits))
            logits_all.append(logits)
            tokens.append(d_i)
            used = d_i if follow is None else int(follow[i - 1])
            if follow is not None:
                tokens[-1] = used
            if i < K:
                u = fuse(f_prev, self.target.embed([used])[0], self.w["fuse_w"], self.rho(i))
                f_prev = self.drafter.forward(u[None, :], self.l + i - 1)[0]
        return tokens, np.stack(logits_all)

    # -- Algorithm 1, parallel verification --------------------------------------------
    def verify(self, drafts):
        """Target pass over rows [x_{l+1}, d_1..d_K] at positions v+l .. v+l+K.
        Returns (g [K+1][d], logits [K+1][V], t [K+1]) with t[i] the greedy token after row i."""
        rows = [self.text[-1]] + [int(t) for t in drafts]
        g = self.target.forward(self.target.embed(rows), self.v + self.l)
        logits = self.target.logits(g)
        return g, logits, [int(t) for t in argmax_lowest(logits)]

    # -- acceptance + roll-forward -----------------------------------------------------
    def accept(self, drafts, g, t, force=None):
        """n, emitted tokens (d_1..d_n, t_{n+1}); then roll the state forward.
        force=(n, emitted) replaces this oracle's own decision (follow mode)."""
        K = len(drafts)
        n = accept_length(drafts, t[:K])
        emitted = [int(x) for x in drafts[:n]] + [t[n]]
        if force is not None:
            n, emitted = int(force[0]), [int(x) for x in force[1]]
        # target keeps rows of x_{l+1}, d_1..d_n ; the rejected rows are dropped
        self.target.truncate(self.v + self.l + n + 1)
        # drafter: speculative rows dropped, n+1 rows rebuilt from the true features g_0..g_n
        self.drafter.truncate(self.l)
        self.text = self.text + emitted
        nxt = self.text[self.l + 1: self.l + n + 2]          # tokens following rows l+1 .. l+n+1
        self.f_next = self._refeed(g[: n + 1], nxt, self.l)
        self.l += n + 1
        return n, emitted

    def cycle(self, K, planted=None, follow_drafts=None, force=None):
        """One draft-verify-accept round.  planted: use these drafts instead of drafting
        (the drafter state is untouched by drafting then).  Returns a dict of everything a
        parity test wants to look at."""
        if planted is not None:
            drafts, dlogits = [int(t) for t in planted], None
        else:
            drafts, dlogits = self.draft(K, follow=follow_drafts)
        g, vlogits, t = self.verify(drafts)
        n, emitted = self.accept(drafts, g, t, force=force)
        return {"drafts": drafts, "draft_logits": dlogits, "g": g, "verify_logits": vlogits,
                "target_tokens": t, "n": n, "emitted": emitted}


def greedy_reference(cfg, weights, vis_embeds, text_ids, n_tokens):
    """Plain definition of the output at T=0: prefill the target, then decode one token at
    a time, always taking the argmax.  Returns (tokens [n_tokens], logits [n_tokens][V])."""
    tgt = Target(cfg, weights)
    vis = np.asarray(vis_embeds, F64)
    x = np.concatenate([vis, tgt.embed(text_ids)], axis=0)
    f = tgt.forward(x, 0)[-1]
    tokens, logits_all = [], []
    pos = x.shape[0]
    for _ in range(n_tokens):
        logits = tgt.logits(f)
        tok = int(argmax_lowest(logits))
        tokens.append(tok)
        logits_all.append(logits)
        f = tgt.forward(tgt.embed([tok]), pos)[0]
        pos += 1
    return tokens, np.stack(logits_all)


def top2_gap(logits):
    """Difference between the largest and second-largest logit of each row."""
    part = np.partition(np.asarray(logits, F64), -2, axis=-1)
    return part[..., -1] - part[..., -2]


# ---- temperature sampling (speculative sampling) -------------------------------------------------
# Section 2.1 of the paper describes the verification at T > 0 in words: the target accepts the
# consecutive candidates that agree with its distribution, rejects the first mismatch and
# everything after it, resamples the next token "accordingly", and samples from its own
# distribution if every candidate was accepted.  The rule behind those words is the speculative
# sampling rule of the works the section cites (Leviathan et al. 2023; Chen et al. 2023), restated
# here: a candidate x drawn from the drafter's distribution q is accepted with probability
# min(1, p(x) / q(x)); on the first rejection the replacement is drawn from the normalised
# positive part of p - q.  With that rule every emitted token is distributed exactly as a sample
# of the target alone (tests/test_oracle_sampling.py pins this).
# The uniform random numbers are INPUTS (so that two implementations can be compared draw by draw).

def softmax_temperature(logits, T):
    """softmax(logits / T) along the last axis, float64."""
    z = np.asarray(logits, F64) / float(T)
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def sample_inverse_cdf(weights, u):
    """Index drawn from non-negative weights (not necessarily normalised) by inversion: the
    smallest j whose running sum exceeds u * total, for u in [0, 1).  If rounding leaves no such
    j, the last index with a positive weight."""
    w = np.asarray(weights, F64)
    c = np.cumsum(w)
    j = int(np.searchsorted(c, float(u) * c[-1], side="right"))
    if j >= w.shape[0]:
        j = int(np.max(np.nonzero(w > 0)[0]))
    return j


def speculative_accept(p, q, drafts, u_accept, u_resample):
    """p: [K+1][V] target distributions after rows 0..K; q: [K][V] drafter distributions the
    drafts were drawn from; drafts: [K].  Returns (n, token): the number of accepted drafts and
    the token that follows them (replacement at the first rejection, or a sample of p[K])."""
    K = len(drafts)
    for i in range(K):
        x = int(drafts[i])
        if float(u_accept[i]) * q[i][x] < p[i][x]:          # u < min(1, p/q)
            continue
        resid = np.maximum(p[i] - q[i], 0.0)
        if not np.any(resid > 0):                             # p == q everywhere: nothing to correct
            resid = p[i]
        return i, sample_inverse_cdf(resid, u_resample)
    return K, sample_inverse_cdf(p[K], u_resample)


class HivisSamplingOracle(HivisOracle):
    """The same cycle with tokens drawn at temperature T instead of taken greedily.  prefill()
    keeps the greedy first token; prefill_sample() draws it from the target's distribution too."""

    def prefill_sample(self, vis_embeds, text_ids, T, u, follow=None):
        """Prefill with x_{l+1} drawn from softmax(logits / T) with uniform u (or `follow`'s token fed
        forward instead, the returned token still being this oracle's own draw)."""
        drawn = {}

        def pick(logits):
            drawn["x"] = sample_inverse_cdf(softmax_temperature(logits, T), u)
            return drawn["x"] if follow is None else int(follow)

        _, logits = self.prefill(vis_embeds, text_ids, pick=pick)
        return drawn["x"], logits

    def draft_sample(self, K, T, u, follow=None):
        """K chain drafts, draft i drawn from softmax(logits_i / T) with uniform u[i].
        Returns (tokens [K], logits [K][V]).  `follow` as in draft()."""
        assert self.drafter.kv_len == self.l
        f_prev = self.f_next
        tokens, logits_all = [], []
        for i in range(1, K + 1):
            logits = self.target.logits(f_prev)
            d_i = sample_inverse_cdf(softmax_temperature(logits, T), u[i - 1])
            used = d_i if follow is None else int(follow[i - 1])
            logits_all.append(logits)
            tokens.append(used)
            if i < K:
                uu = fuse(f_prev, self.target.embed([used])[0], self.w["fuse_w"], self.rho(i))
                f_prev = self.drafter.forward(uu[None, :], self.l + i - 1)[0]
        return tokens, np.stack(logits_all)

    def accept_sample(self, drafts, draft_logits, g, verify_logits, T, u_accept, u_resample, force=None):
        """Stochastic acceptance, then the same roll-forward as accept()."""
        p = softmax_temperature(verify_logits, T)
        q = softmax_temperature(draft_logits, T)
        n, tok = speculative_accept(p, q, drafts, u_accept, u_resample)
        emitted = [int(x) for x in drafts[:n]] + [int(tok)]
        if force is not None:
            n, emitted = int(force[0]), [int(x) for x in force[1]]
        self.target.truncate(self.v + self.l + n + 1)
        self.drafter.truncate(self.l)
        self.text = self.text + emitted
        nxt = self.text[self.l + 1: self.l + n + 2]
        self.f_next = self._refeed(g[: n + 1], nxt, self.l)
        self.l += n + 1
        return n, emitted

    def cycle_sample(self, K, T, u_draft, u_accept, u_resample, follow_drafts=None, force=None):
        """One draft-verify-accept round at temperature T."""
        drafts, dlogits = self.draft_sample(K, T, u_draft, follow=follow_drafts)
        g, vlogits, _ = self.verify(drafts)
        n, emitted = self.accept_sample(drafts, dlogits, g, vlogits, T, u_accept, u_resample, force=force)
        return {"drafts": drafts, "draft_logits": dlogits, "g": g, "verify_logits": vlogits, "n": n, "emitted": emitted}


def sampling_reference(cfg, weights, vis_embeds, text_ids, n_tokens, T, u, sample_first=False):
    """Plain definition at T > 0: prefill the target, then decode one token at a time, each drawn
    from softmax(logits / T) with u[k]; the first token is greedy (as prefill() does) unless
    sample_first (as prefill_sample() does)."""
    tgt = Target(cfg, weights)
    vis = np.asarray(vis_embeds, F64)
    x = np.concatenate([vis, tgt.embed(text_ids)], axis=0)
    f = tgt.forward(x, 0)[-1]
    tokens = []
    pos = x.shape[0]
    for k in range(n_tokens):
        logits = tgt.logits(f)
        tok = int(argmax_lowest(logits)) if (k == 0 and not sample_first) else sample_inverse_cdf(softmax_temperature(logits, T), u[k])
        tokens.append(tok)
        f = tgt.forward(tgt.embed([tok]), pos)[0]
        pos += 1
    return tokens
