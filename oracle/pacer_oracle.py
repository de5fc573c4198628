"""Plain CPU oracle for one Pacer adaptive speculative-decoding step.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this module.  It shares no code with the HIP library and
never calls it; every input (weights, prompts, seeds) is handed in by the caller.

All arithmetic is numpy float64 (weights arrive as exactly representable bf16/fp32
values and are widened on use).  The one exception is the stop decision of Alg. 1,
which is an integer outcome of floating point: the block mean and the threshold are
evaluated in float32 in index order, the precision the GPU kernel decides in.

What follows the paper, and where:
  * model forward / autoregressive generation ........ Sec. 2.1, Eq. 1 and Eq. 2
  * drafting, target verification ..................... Sec. 2.2, Eq. 3 and Eq. 4
  * acceptance rule, residual resampling, bonus token . Sec. 2.2, Eq. 5; Alg. 1 (verification part)
  * blockwise drafting and pre-verification ........... Sec. 3.2, Eq. 6 and Eq. 7
  * halting test, threshold growth, gamma = k*b ....... Sec. 3.2 last paragraph; Alg. 1 (inner loop)
  * the whole step .................................... Appendix A, Alg. 1

The paper fixes neither the network architecture nor the sampler; the readings used
here (Llama-style decoder, one decoder layer of draft width for M_B with a 2-class head,
learned additive draft-position table with row 0 = 0 for prefix rows, threshold reset
at every outer step, gamma_max cap, Gumbel-max sampling on a counter-based generator,
beta-coupled effective target logits) are listed with their reasons in the design notes
of the repository.

Pins (tests/test_oracle_*.py, all CPU):
  decoder forward ........ an independent Llama implementation (transformers' LlamaForCausalLM,
                           float64) loaded with the same weights; from-scratch full-prefix
                           recomputation against the KV-cached path; RoPE shift invariance
  verify pass ............ row i equals the i-th of gamma+1 sequential single-token passes
  greedy procedure ....... output equals target-only greedy decoding of the effective target,
                           for every b, gamma_max, beta and forced stop pattern
  acceptance rule ........ exact enumeration of the emitted-token law on tiny vocabularies
                           (equals p), chi-square of the sampled path, n-gram law against
                           autoregressive sampling with adversarial stop decisions
  halting / threshold .... closed form t0*rho^(k-1), gamma = k*b, the scenario counts printed
                           in the caption of Fig. 1 and the forward-count identities of the
                           forward-pass table (tests/golden/)
  rollback ............... caches after a step equal a fresh prefill of the committed prefix
  M_B block pass ......... b-row causal pass equals b single-row passes
PARITY UNPINNED: M_B against the paper's *trained* layer (no weights or alpha-hat values are
printed anywhere in the paper), and the paper's tokens/s and tau (need its models and data).
"""
import numpy as np

from . import philox

F64 = np.float64
F32 = np.float32

GREEDY = 0
SAMPLE = 1


class ModelCfg:
    def __init__(self, n_layers, d_model, n_heads, head_dim, d_ffn, vocab,
                 rope_theta=10000.0, rms_eps=1e-5):
        self.n_layers = n_layers
        self.d_model = d_model
        self.n_heads = n_heads
        self.head_dim = head_dim
        self.d_ffn = d_ffn
        self.vocab = vocab
        self.rope_theta = rope_theta
        self.rms_eps = rms_eps
        assert n_heads * head_dim == d_model


def _a(w):
    return np.asarray(w, dtype=F64)


# ----------------------------------------------------------------------------- model
def rmsnorm(x, g, eps):
    """x * g / sqrt(mean(x^2) + eps) over the last axis."""
    x = _a(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _a(g)


def rope(x, pos, theta):
    """Rotary position embedding, rotate-half pairing (j, j + hd/2).
    x: [R, H, hd]; pos: [R] absolute positions."""
    R, H, hd = x.shape
    half = hd // 2
    inv_freq = theta ** (-(np.arange(half, dtype=F64) * 2.0 / hd))
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]      # [R, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(z):
    z = _a(z)
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


class KVCache:
    """Per-layer key/value rows for positions 0..n-1 (row p = token at absolute position p)."""

    def __init__(self, n_layers, width, max_seq):
        self.K = [np.zeros((max_seq, width), dtype=F64) for _ in range(n_layers)]
        self.V = [np.zeros((max_seq, width), dtype=F64) for _ in range(n_layers)]
        self.n = 0

    def truncate(self, n):
        assert 0 <= n <= self.n
        self.n = n


def _attention_rows(q, K, V, pos, H, hd):
    """q: [R, H*hd] (already rotated); K, V: cache arrays; row r attends to keys 0..pos[r].
    Per head: softmax(Q K^T / sqrt(hd) + causal mask) V, the masked-matrix form of Eq. 2."""
    R = q.shape[0]
    pos = np.asarray(pos, dtype=np.int64)
    n = int(pos.max()) + 1
    out = np.zeros((R, H * hd), dtype=F64)
    scale = 1.0 / np.sqrt(float(hd))
    hidden = np.arange(n)[None, :] > pos[:, None]          # [R, n]: keys after the row's own position
    for h in range(H):
        cols = slice(h * hd, (h + 1) * hd)
        s = (q[:, cols] @ K[:n, cols].T) * scale           # [R, n]
        s[hidden] = -np.inf
        out[:, cols] = softmax(s) @ V[:n, cols]
    return out


def decoder_layer(x, pos, lw, K, V, cfg, kv_only=False):
    """One pre-norm Llama-style layer on rows x [R, d] at absolute positions pos [R].
    Writes the rows' keys/values into K, V at those positions.  kv_only: stop after that."""
    R = x.shape[0]
    H, hd = cfg.n_heads, cfg.head_dim
    a = rmsnorm(x, lw["attn_norm"], cfg.rms_eps)
    k = rope((a @ _a(lw["wk"]).T).reshape(R, H, hd), pos, cfg.rope_theta).reshape(R, -1)
    v = a @ _a(lw["wv"]).T
    for r in range(R):
        K[int(pos[r])] = k[r]
        V[int(pos[r])] = v[r]
    if kv_only:
        return None
    q = rope((a @ _a(lw["wq"]).T).reshape(R, H, hd), pos, cfg.rope_theta).reshape(R, -1)
    o = _attention_rows(q, K, V, pos, H, hd)
    x = x + o @ _a(lw["wo"]).T
    m = rmsnorm(x, lw["ffn_norm"], cfg.rms_eps)
    x = x + (silu(m @ _a(lw["wg"]).T) * (m @ _a(lw["wu"]).T)) @ _a(lw["wd"]).T
    return x


def lm_forward(w, cfg, tokens, cache):
    """Parallel forward (Eq. 2) of the rows `tokens` placed at positions cache.n, cache.n+1, ...
    against the cache; appends their K/V.  Returns (hidden [R, d] after the final norm,
    logits [R, V])."""
    tokens = np.asarray(tokens, dtype=np.int64)
    R = tokens.shape[0]
    pos = cache.n + np.arange(R)
    x = _a(w["embed"][tokens])
    for l in range(cfg.n_layers):
        x = decoder_layer(x, pos, w["layers"][l], cache.K[l], cache.V[l], cfg)
    cache.n += R
    h = rmsnorm(x, w["final_norm"], cfg.rms_eps)
    return h, h @ _a(w["head"]).T


def mb_forward(mb, cfg, u, cache, kv_only=False):
    """Pre-verification layer M_B (Eq. 7) on rows u [R, d] = h + e placed at positions
    cache.n.. ; one decoder layer over its own KV cache, final norm, 2-class head,
    alpha-hat = softmax(z)[1].  kv_only rows (prefix rows) only extend the cache."""
    R = u.shape[0]
    pos = cache.n + np.arange(R)
    x = decoder_layer(_a(u), pos, mb["layer"], cache.K[0], cache.V[0], cfg, kv_only=kv_only)
    cache.n += R
    if kv_only:
        return None
    z = rmsnorm(x, mb["final_norm"], cfg.rms_eps) @ _a(mb["cls"]).T       # [R, 2]
    return softmax(z)[:, 1]


# ------------------------------------------------------------------ acceptance (Eq. 5)
def accept_prob(p, q, y):
    """alpha_i of Eq. 5 for draft token y."""
    return 1.0 if p[y] >= q[y] else p[y] / q[y]


def residual_dist(p, q):
    """norm(max(0, p - q)); falls back to p when p == q everywhere (no residual mass)."""
    w = np.maximum(0.0, p - q)
    s = w.sum()
    return p.copy() if s <= 0.0 else w / s


def gumbel_argmax(logw, u):
    """argmax_v(logw_v + Gumbel(u_v)); lowest index wins ties."""
    with np.errstate(divide="ignore"):
        return int(np.argmax(logw + philox.gumbel(u)))


def first_rejection(ratios, r):
    """n = min({i-1 : r_i > p_i[y_i]/q_i[y_i]} U {gamma})  (Alg. 1)."""
    for i in range(len(ratios)):
        if r[i] > ratios[i]:
            return i
    return len(ratios)


# ------------------------------------------------------------------------ the procedure
class PacerOracle:
    """Alg. 1 around three models with KV caches.  State between steps: the committed
    tokens x_0..x_{N-1}; all three caches hold positions 0..N-2."""

    def __init__(self, target, cfg_t, draft, cfg_d, mb, block, gamma_max, t0, rho, beta,
                 mode=GREEDY, seed=0, seq=0, max_seq=4096, use_preverify=True,
                 halting="mean"):
        self.wT, self.cT, self.wD, self.cD, self.wB = target, cfg_t, draft, cfg_d, mb
        self.b, self.gamma_max = int(block), int(gamma_max)
        self.t0, self.rho, self.beta = F32(t0), F32(rho), float(beta)
        self.mode, self.seed, self.seq = mode, seed, seq
        self.use_preverify = use_preverify
        self.halting = halting
        self.kvT = KVCache(cfg_t.n_layers, cfg_t.d_model, max_seq)
        self.kvD = KVCache(cfg_d.n_layers, cfg_d.d_model, max_seq)
        self.kvB = KVCache(1, cfg_d.d_model, max_seq)
        self.tokens = []
        self.step_idx = 0
        self.n_draft_fwd = 0       # the k*b drafting forwards
        self.n_bonus_fwd = 0       # extra draft forward when every draft was accepted
        self.n_target_fwd = 0
        self.n_pv_calls = 0

    # -- model calls (overridable by counting tests) --
    def _target_rows(self, toks):
        self.n_target_fwd += 1
        return lm_forward(self.wT, self.cT, toks, self.kvT)[1]

    def _draft_one(self, tok):
        h, lg = lm_forward(self.wD, self.cD, [tok], self.kvD)
        return h[0], lg[0]

    def _preverify(self, hs, i):
        e = _a(self.wB["posemb"])[i:i + len(hs)]
        self.n_pv_calls += 1
        return mb_forward(self.wB, self.cD, np.stack(hs) + e, self.kvB)

    def _mb_prefix_rows(self, hs):
        if self.wB is not None and len(hs):
            mb_forward(self.wB, self.cD, np.stack(hs), self.kvB, kv_only=True)   # e_0 = 0

    # -- prompt ingestion (support; Alg. 1 takes the prefix as given) --
    def prefill(self, prompt):
        assert not self.tokens and len(prompt) >= 1
        self.tokens = [int(t) for t in prompt]
        if len(prompt) > 1:
            lm_forward(self.wT, self.cT, prompt[:-1], self.kvT)
            h, _ = lm_forward(self.wD, self.cD, prompt[:-1], self.kvD)
            self._mb_prefix_rows(list(h))

    def _pick(self, logits, row, purpose):
        if self.mode == GREEDY:
            return int(np.argmax(logits))
        u = philox.vocab_uniforms(self.seed, self.seq, self.step_idx, row, purpose, len(logits))
        return gumbel_argmax(logits, u)

    def _halt(self, alpha, t):
        """Stop test of Alg. 1, decided in float32.  'mean' is the paper's criterion; 'any'
        and 'last' are the stricter alternatives of Sec. 5.2."""
        a32 = alpha.astype(F32)
        if self.halting == "mean":
            s = F32(0.0)
            for v in a32:
                s = F32(s + v)
            return bool(F32(s / F32(len(a32))) <= t), float(F32(s / F32(len(a32))))
        if self.halting == "any":
            return bool(np.any(a32 <= t)), float(a32.min())
        return bool(a32[-1] <= t), float(a32[-1])

    def step(self, force_stop=None, fixed_gamma=None):
        """One outer iteration of Alg. 1.  force_stop(round_k, alpha) -> bool overrides the
        halting test (any rule that looks only at draft-side quantities keeps the output law).
        fixed_gamma: vanilla speculative decoding with that window, no pre-verification."""
        N = len(self.tokens)
        b = self.b
        t = self.t0                       # threshold restarts at t0 every step
        i = 1                             # draft position of the next block's first token
        y, dlog, hid, alphas, rounds = [], [], [], [], []
        cur = self.tokens[-1]
        while True:
            nblk = b if fixed_gamma is None else fixed_gamma
            hs = []
            for _ in range(nblk):                                   # Eq. 6: b draft forwards
                h, lg = self._draft_one(cur)
                self.n_draft_fwd += 1
                cur = self._pick(lg, len(y) + 1, philox.PURPOSE_DRAFT)
                y.append(cur)
                dlog.append(lg)
                hs.append(h)
            hid.extend(hs)
            if fixed_gamma is not None or not self.use_preverify:
                if self.wB is not None:
                    self._mb_prefix_rows(hs)
                if fixed_gamma is not None or len(y) + b > self.gamma_max:
                    break
                continue
            alpha = self._preverify(hs, i)                          # Eq. 7
            alphas.extend(alpha)
            i += b
            stop, stat = self._halt(alpha, t)
            if force_stop is not None:
                stop = bool(force_stop(len(rounds), alpha))
            capped = len(y) + b > self.gamma_max
            rounds.append({"t": float(t), "stat": stat, "stop": stop, "capped": capped})
            if stop or capped:
                break
            t = F32(t * self.rho)
        gamma = len(y)

        # Eq. 4: one target pass over [x_{N-1}, y_1..y_gamma]
        tlog = self._target_rows([self.tokens[-1]] + y)
        dl = np.stack(dlog)
        eff = tlog[:gamma] + self.beta * dl                          # rows 1..gamma
        if self.mode == GREEDY:
            am = np.argmax(eff, axis=-1)
            n = 0
            while n < gamma and am[n] == y[n]:
                n += 1
            ratios, r = None, None
        else:
            P = softmax(eff)
            Q = softmax(dl)
            ratios = np.array([P[k, y[k]] / Q[k, y[k]] for k in range(gamma)])
            r = np.array([philox.scalar_uniform(self.seed, self.seq, self.step_idx, k + 1,
                                                philox.PURPOSE_ACCEPT) for k in range(gamma)])
            n = first_rejection(ratios, r)

        bonus_dlog = None
        if n == gamma:
            # all accepted: the draft has not yet seen y_gamma; this forward also supplies the
            # draft logits that the beta-coupled bonus row needs
            h, bonus_dlog = self._draft_one(y[-1])
            self.n_bonus_fwd += 1
            self._mb_prefix_rows([h])
            row = tlog[gamma] + self.beta * bonus_dlog
            if self.mode == GREEDY:
                z = int(np.argmax(row))
            else:
                u = philox.vocab_uniforms(self.seed, self.seq, self.step_idx, gamma + 1,
                                          philox.PURPOSE_NEXT, len(row))
                z = gumbel_argmax(np.log(softmax(row)), u)
        else:
            if self.mode == GREEDY:
                z = int(am[n])
            else:
                pp = residual_dist(P[n], Q[n])
                u = philox.vocab_uniforms(self.seed, self.seq, self.step_idx, n + 1,
                                          philox.PURPOSE_NEXT, len(pp))
                with np.errstate(divide="ignore"):
                    z = gumbel_argmax(np.log(pp), u)

        self.tokens.extend(y[:n] + [z])
        keep = len(self.tokens) - 1
        self.kvT.truncate(keep)
        self.kvD.truncate(keep)
        if self.wB is not None:
            self.kvB.truncate(keep)
        self.step_idx += 1
        return {"gamma": gamma, "n": n, "z": z, "draft_tokens": y, "draft_logits": dl,
                "bonus_draft_logits": bonus_dlog, "hidden": np.stack(hid),
                "alpha": np.array(alphas), "rounds": rounds, "target_logits": tlog,
                "ratios": ratios, "r": r}

    def generate(self, n_new, **kw):
        start = len(self.tokens)
        recs = []
        while len(self.tokens) - start < n_new:
            recs.append(self.step(**kw))
        return self.tokens[start:start + n_new], recs


def ar_decode(target, cfg_t, draft, cfg_d, beta, prompt, n_new, mode=GREEDY, seed=0, seq=0,
              max_seq=4096, return_logits=False):
    """Eq. 1 on the effective target: logits_T(prefix) + beta * logits_D(prefix), one token per
    forward.  Sampling mode draws token k with Gumbel noise keyed by (step=k, row=0)."""
    kvT = KVCache(cfg_t.n_layers, cfg_t.d_model, max_seq)
    kvD = KVCache(cfg_d.n_layers, cfg_d.d_model, max_seq)
    toks = [int(t) for t in prompt]
    if len(toks) > 1:
        lm_forward(target, cfg_t, toks[:-1], kvT)
        if beta != 0.0:
            lm_forward(draft, cfg_d, toks[:-1], kvD)
    out, logs = [], []
    for k in range(n_new):
        row = lm_forward(target, cfg_t, [toks[-1]], kvT)[1][0]
        if beta != 0.0:
            row = row + beta * lm_forward(draft, cfg_d, [toks[-1]], kvD)[1][0]
        if mode == GREEDY:
            z = int(np.argmax(row))
        else:
            u = philox.vocab_uniforms(seed, seq, k, 0, philox.PURPOSE_NEXT, len(row))
            z = gumbel_argmax(row, u)
        toks.append(z)
        out.append(z)
        logs.append(row)
    return (out, np.stack(logs)) if return_logits else out
