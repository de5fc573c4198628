"""Host-side driver around the C ABI: uploads and binds a model pair, owns the torch buffers
the library borrows, and runs the outer loop of Alg. 1 (Appendix A) by issuing the four hot
calls.  No arithmetic of the method happens here: the loop only reads the stop flag and the
accept result that the kernels produced.
"""
import torch

from . import binding as B


def _dev(t, dtype=None):
    t = t.to("cuda", non_blocking=False)
    return t if dtype is None else t.to(dtype)


class Session:
    def __init__(self, w, target, draft, preverify, max_seq, max_batch=1, t0=None, rho=None,
                 block=None, gamma_max=None, halting=B.HALT_MEAN, kv_fill=None):
        """w: workload description (synth.workload); target/draft/preverify: weight dicts
        (linear weights [out, in]; any device).  kv_fill: byte value the KV buffers are filled with
        before they are handed over (tests: the library must not depend on their contents)."""
        assert torch.cuda.is_available(), "the Pacer hot path needs a GPU"
        self.w = w
        self.dtype = w["dtype"]
        self.block = block or w["block"]
        self.gamma_max = gamma_max or w["gamma_max"]
        self.G1 = self.gamma_max + 1
        max_seq = (max_seq + 31) // 32 * 32          # the f16 KV layout wants whole 32-key groups
        self.max_seq, self.max_batch = max_seq, max_batch
        self.stream = torch.cuda.current_stream().cuda_stream
        self.keep = []                      # tensors the library borrows
        self.not_finite = torch.zeros(1, dtype=torch.int32, device="cuda")   # weights that do not fit a half float
        cfg_t = B.model_cfg(w["target"] | {"n_layers": len(target["layers"])}, max_seq, self.dtype)
        cfg_d = B.model_cfg(w["draft"], max_seq, self.dtype)
        pv = B.PvCfg(self.block, self.gamma_max, t0 if t0 is not None else w["t0"],
                     rho if rho is not None else w["rho"], halting)
        self.ctx = B.pacer_create(cfg_t, cfg_d, pv, max_batch, self.stream)
        self.V = w["target"]["vocab"]
        self.dD = w["draft"]["d_model"]
        self._bind_lm(B.TARGET, target)
        self._bind_lm(B.DRAFT, draft, share=target if draft["embed"] is target["embed"] else None)
        self._bind_layer(B.PREVERIFY, 0, preverify["layer"])
        self._bind_f32(B.PREVERIFY, B.T_FINAL_NORM, 0, preverify["final_norm"])
        self._bind_f32(B.PREVERIFY, B.T_POSEMB, 0, preverify["posemb"])
        self._bind_f32(B.PREVERIFY, B.T_CLS, 0, preverify["cls"])
        bad = int(self.not_finite.item())
        if bad:
            raise B.PacerError(B.EINVAL, f"{bad} weights are not finite as half floats (|w| > 65504, inf or NaN)")
        for which in (B.TARGET, B.DRAFT, B.PREVERIFY):
            kv = torch.empty(B.pacer_kv_bytes(self.ctx, which), dtype=torch.uint8, device="cuda")
            if kv_fill is not None:
                kv.fill_(kv_fill)
            self.keep.append(kv)
            B.pacer_bind_kv(self.ctx, which, kv)
        self.ws = torch.empty(B.pacer_workspace_bytes(self.ctx) + 256, dtype=torch.uint8, device="cuda")
        off = (-self.ws.data_ptr()) % 256
        self.ws_view = self.ws[off:]
        B.pacer_bind_workspace(self.ctx, self.ws_view)
        self.logits = torch.zeros(max_batch, self.G1, self.V, dtype=torch.float32, device="cuda")
        self.alpha = torch.zeros(max_batch, self.block, dtype=torch.float32, device="cuda")
        self.stop = torch.zeros(max_batch, dtype=torch.int32, device="cuda")
        self.n_acc = torch.zeros(max_batch, dtype=torch.int32, device="cuda")
        self.next_tok = torch.zeros(max_batch, dtype=torch.int32, device="cuda")
        self.step_idx = [0] * max_batch
        self.counts = dict(draft=0, target=0, preverify=0)
        self.timers = None                  # dict name -> [(start_event, stop_event)] when timing calls
        self.launches = {}                  # dict name -> [kernels enqueued by the call] while timing calls
        torch.cuda.synchronize()

    # ---- weight upload -------------------------------------------------------------------
    def _matrix(self, parts, tid, head_dim=0):
        """row-major [out, in] pieces -> the library's format for this dtype (device tensor)."""
        if self.dtype == "bf16":
            src = torch.cat([_dev(p, torch.bfloat16) for p in parts], dim=0).contiguous()
            dst = torch.empty_like(src)
            B.pacer_pack_weight(dst, src, tid, head_dim, self.not_finite, self.stream)
            torch.cuda.synchronize()
            del src
            return dst
        return torch.cat([_dev(p, torch.float32) for p in parts], dim=0).contiguous()

    def _bind_f32(self, which, tid, layer, t):
        t = _dev(t, torch.float32).contiguous()
        self.keep.append(t)
        B.pacer_bind(self.ctx, which, tid, layer, t)

    def _bind_mat(self, which, tid, layer, parts):
        hd = (self.w["target"] if which == B.TARGET else self.w["draft"])["head_dim"]
        t = self._matrix(parts, tid, hd)
        self.keep.append(t)
        B.pacer_bind(self.ctx, which, tid, layer, t)
        return t

    def _bind_layer(self, which, l, lw):
        self._bind_f32(which, B.T_ATTN_NORM, l, lw["attn_norm"])
        self._bind_mat(which, B.T_WQKV, l, [lw["wq"], lw["wk"], lw["wv"]])
        self._bind_mat(which, B.T_WO, l, [lw["wo"]])
        self._bind_f32(which, B.T_FFN_NORM, l, lw["ffn_norm"])
        self._bind_mat(which, B.T_WGU, l, [lw["wg"], lw["wu"]])
        self._bind_mat(which, B.T_WD, l, [lw["wd"]])

    def _bind_lm(self, which, m, share=None):
        for l, lw in enumerate(m["layers"]):
            self._bind_layer(which, l, lw)
        self._bind_f32(which, B.T_FINAL_NORM, 0, m["final_norm"])
        if share is not None:
            emb, head = self._shared
        else:
            edt = torch.bfloat16 if self.dtype == "bf16" else torch.float32
            emb = _dev(m["embed"], edt).contiguous()
            head = self._matrix([m["head"]], B.T_HEAD)
            self._shared = (emb, head)
        self.keep += [emb, head]
        B.pacer_bind(self.ctx, which, B.T_EMBED, 0, emb)
        B.pacer_bind(self.ctx, which, B.T_HEAD, 0, head)

    # ---- taps ----------------------------------------------------------------------------
    def _peek(self, seq, what, dtype):
        p, nb = B.pacer_peek(self.ctx, seq, what)
        off = p - self.ws_view.data_ptr()
        return self.ws_view[off:off + nb].view(dtype)

    def draft_logits(self, seq=0):
        return self._peek(seq, B.PEEK_DRAFT_LOGITS, torch.float32).view(self.G1, self.V)

    def draft_hidden(self, seq=0):
        return self._peek(seq, B.PEEK_DRAFT_HIDDEN, torch.float32).view(self.G1, self.dD)

    def draft_tokens(self, seq=0):
        return self._peek(seq, B.PEEK_DRAFT_TOKENS, torch.int32)

    def tokens(self, seq=0):
        n = B.pacer_get_state(self.ctx, seq)["len"]
        return self._peek(seq, B.PEEK_TOKENS, torch.int32)[:n].tolist()

    # ---- per-call timing (benchmarks) ------------------------------------------------------
    def _call(self, name, fn, *a):
        if self.timers is None:
            return fn(*a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n0 = B.pacer_launch_count(self.ctx)
        e0.record()
        out = fn(*a)
        e1.record()
        self.timers.setdefault(name, []).append((e0, e1))
        self.launches.setdefault(name, []).append(B.pacer_launch_count(self.ctx) - n0)
        return out

    def read_timers(self):
        torch.cuda.synchronize()
        out = {k: [a.elapsed_time(b) for a, b in v] for k, v in (self.timers or {}).items()}
        self.timers = {} if self.timers is not None else None
        return out

    def read_launches(self):
        out, self.launches = self.launches, {}
        return out

    # ---- decoding --------------------------------------------------------------------------
    def prefill(self, prompt, seq=0):
        t = torch.as_tensor(prompt, dtype=torch.int32).to("cuda")
        B.pacer_prefill(self.ctx, seq, t)
        torch.cuda.current_stream().synchronize()
        self.step_idx[seq] = 0

    def step(self, mode=B.GREEDY, beta=None, seed=0, seq=0, force_stop=None, fixed_gamma=None,
             record=False):
        """One outer iteration of Alg. 1 for one sequence.  force_stop(round, alpha) overrides the
        stop flag; fixed_gamma drafts that many tokens without pre-verification (vanilla SD);
        fixed_gamma = 0 is plain autoregressive decoding through the same kernels."""
        beta = self.w["beta"] if beta is None else beta
        ctx, seqs, ctr = self.ctx, [seq], self.step_idx[seq]
        B.pacer_begin_step(ctx, seq)
        rec = dict(alpha=[], stops=[]) if record else None
        gamma, rnd = 0, 0
        if fixed_gamma is not None:
            for _ in range(fixed_gamma):
                self._call("draft_step", B.pacer_draft_step, ctx, seqs, mode, seed, ctr)
            gamma = fixed_gamma
            self.counts["draft"] += gamma
        elif not record and force_stop is None and self.timers is None:
            # the whole inner loop of Alg. 1 in one library call (same kernels and flags as the loop below)
            gamma = B.pacer_draft_window(ctx, seqs, mode, seed, ctr, self.alpha, self.stop)[0]
            self.counts["draft"] += gamma
            self.counts["preverify"] += gamma // self.block
        else:
            while True:
                for _ in range(self.block):
                    self._call("draft_step", B.pacer_draft_step, ctx, seqs, mode, seed, ctr)
                gamma += self.block
                self.counts["draft"] += self.block
                forced = None
                if force_stop is not None:
                    # a pattern that does not look at alpha is forced inside the library (the kernel writes the
                    # forced flag); one that does is applied here, after the read-back
                    try:
                        forced = force_stop(rnd, None)
                    except TypeError:
                        forced = None
                    if forced is not None:
                        B.pacer_force_stop(ctx, seq, 1 if forced else 0)
                self._call("preverify_block", B.pacer_preverify_block, ctx, seqs, self.alpha, self.stop)
                self.counts["preverify"] += 1
                stop = bool(B.pacer_wait_stop(ctx, seqs)[0])       # the only read-back of the drafting loop
                if record:
                    rec["alpha"] += self.alpha[0].tolist()
                    rec["stops"].append(stop)
                if force_stop is not None and forced is None:
                    stop = bool(force_stop(rnd, self.alpha[0].tolist()))
                rnd += 1
                if stop or gamma + self.block > self.gamma_max:
                    break
        self._call("verify", B.pacer_verify, ctx, seqs, None, self.logits)
        self.counts["target"] += 1
        self._call("accept_rollback", B.pacer_accept_rollback, ctx, seqs, mode, [beta], seed, ctr, self.logits,
                   self.n_acc, self.next_tok)
        st = self._call("collect_result", B.pacer_get_state, ctx, seq)   # the bonus-row part runs here when every draft was accepted
        self.step_idx[seq] += 1
        out = dict(gamma=gamma, n=st["n_accepted"], z=st["next_token"], len=st["len"])
        if record:
            out.update(rec)
            out["draft_tokens"] = self.draft_tokens(seq)[:gamma].tolist()
            out["draft_logits"] = self.draft_logits(seq)[:gamma + 1].clone()
            out["hidden"] = self.draft_hidden(seq)[:gamma + 1].clone()
            out["target_logits"] = self.logits[0, :gamma + 1].clone()
        return out

    def step_batch(self, seqs, mode=B.GREEDY, betas=None, seed=0, fixed_gamma=None, record=False):
        """One outer iteration of Alg. 1 for several sequences in lock step: sequences whose block
        fails pre-verification (or that reach gamma_max) drop out of the drafting loop, the others
        go on; one ragged verify and one accept call serve all of them."""
        betas = [self.w["beta"]] * len(seqs) if betas is None else list(betas)
        ctx, ctr = self.ctx, self.step_idx[seqs[0]]
        assert all(self.step_idx[s] == ctr for s in seqs), "lock-step sequences share the step counter"
        for s in seqs:
            B.pacer_begin_step(ctx, s)
        gamma = {s: 0 for s in seqs}
        recs = {s: dict(alpha=[], stops=[]) for s in seqs}
        active = list(seqs)
        if fixed_gamma is not None:
            for _ in range(fixed_gamma):
                self._call("draft_step", B.pacer_draft_step, ctx, active, mode, seed, ctr)
            gamma = {s: fixed_gamma for s in seqs}
            self.counts["draft"] += fixed_gamma * len(seqs)
            active = []
        elif not record and self.timers is None:
            gs = B.pacer_draft_window(ctx, active, mode, seed, ctr, self.alpha, self.stop)
            gamma = dict(zip(seqs, gs))
            self.counts["draft"] += sum(gs)
            self.counts["preverify"] += sum(g // self.block for g in gs)
            active = []
        while active:
            for _ in range(self.block):
                self._call("draft_step", B.pacer_draft_step, ctx, active, mode, seed, ctr)
            self.counts["draft"] += self.block * len(active)
            self._call("preverify_block", B.pacer_preverify_block, ctx, active, self.alpha, self.stop)
            self.counts["preverify"] += len(active)
            stops = B.pacer_wait_stop(ctx, active)
            alphas = self.alpha[:len(active)].tolist() if record else None
            nxt = []
            for i, s in enumerate(active):
                gamma[s] += self.block
                if record:
                    recs[s]["alpha"] += alphas[i]
                    recs[s]["stops"].append(bool(stops[i]))
                if not stops[i] and gamma[s] + self.block <= self.gamma_max:
                    nxt.append(s)
            active = nxt
        self._call("verify", B.pacer_verify, ctx, seqs, None, self.logits)
        self.counts["target"] += 1
        self._call("accept_rollback", B.pacer_accept_rollback, ctx, seqs, mode, betas, seed, ctr, self.logits,
                   self.n_acc, self.next_tok)
        out = []
        for i, s in enumerate(seqs):
            st = B.pacer_get_state(ctx, s)
            self.step_idx[s] += 1
            r = dict(gamma=gamma[s], n=st["n_accepted"], z=st["next_token"], len=st["len"])
            if record:
                g = gamma[s]
                r.update(recs[s])
                r["draft_tokens"] = self.draft_tokens(s)[:g].tolist()
                r["draft_logits"] = self.draft_logits(s)[:g + 1].clone()
                r["hidden"] = self.draft_hidden(s)[:g + 1].clone()
                r["target_logits"] = self.logits[i, :g + 1].clone()
            out.append(r)
        return out

    def generate(self, n_new, seq=0, **kw):
        start = B.pacer_get_state(self.ctx, seq)["len"]
        recs = []
        while B.pacer_get_state(self.ctx, seq)["len"] - start < n_new:
            recs.append(self.step(seq=seq, **kw))
        return self.tokens(seq)[start:start + n_new], recs

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize()
            B.pacer_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
