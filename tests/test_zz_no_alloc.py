"""The allocation-free acceptance entry point against pacer_accept_rollback, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2602_01274_amd import binding as B
from paper_2602_01274_amd import synth

pytestmark = pytest.mark.gpu


def _drafted_and_verified(s, seq, gamma, mode, seed):
    ctr = s.step_idx[seq]
    B.pacer_begin_step(s.ctx, seq)
    for _ in range(gamma):
        B.pacer_draft_step(s.ctx, [seq], mode, seed, ctr)
    B.pacer_verify(s.ctx, [seq], None, s.logits)
    return ctr


@pytest.mark.parametrize("mode", [B.GREEDY, B.SAMPLE])
def test_accept_noalloc_matches_accept_rollback(mode):
    """pacer_accept_noalloc (scratch in the library's device image, no workspace, no allocation) must give the n and
    the new token of pacer_accept_rollback on the same logits, bit for bit: two calls in a row on one stream, the
    second with a smaller window (the shared scratch then still holds the first call's rows), on a pair whose
    vocabulary spans all 16 chunks; strong coupling makes all-accepted steps (bonus row) occur, weak coupling rejections."""
    from paper_2602_01274_amd.engine import Session
    w = synth.workload("mid")
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=2)
    s = Session(w, tgt, drf, mb, max_seq=256)
    V = w["target"]["vocab"]
    s.prefill(synth.make_prompt(V, 40, 1).tolist())
    stream = torch.cuda.current_stream().cuda_stream
    out_n = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    out_z = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    seen = set()
    for gamma, beta in ((12, 3.0), (4, 3.0), (8, 12.0), (3, 12.0), (12, 0.5), (1, 12.0), (2, 1.0), (1, 1.0), (1, 0.0), (1, 1.0), (1, 0.5)):
        ctr = _drafted_and_verified(s, 0, gamma, mode, 11)
        B.pacer_accept_rollback(s.ctx, [0], mode, [beta], 11, ctr, s.logits, s.n_acc, s.next_tok)
        st = B.pacer_get_state(s.ctx, 0)
        n, z = st["n_accepted"], st["next_token"]
        # the rings still hold this step's draft logits (row gamma: the bonus forward's, if it ran) and tokens
        tl = s.logits[0, :gamma + 1].contiguous()
        dl = s.draft_logits(0)[:gamma + 1].contiguous()
        dt = s.draft_tokens(0)[:gamma].contiguous()
        bonus = n == gamma
        B.pacer_accept_noalloc(tl, dl, dt, gamma, bonus, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
        torch.cuda.synchronize()
        assert (int(out_n.item()), int(out_z.item())) == (n, z), (gamma, beta, n, z)
        if not bonus:
            # without the bonus row a rejection gives the same result, and with it too (the row is then skipped)
            B.pacer_accept_noalloc(tl, dl, dt, gamma, True, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
            torch.cuda.synchronize()
            assert (int(out_n.item()), int(out_z.item())) == (n, z)
        else:
            B.pacer_accept_noalloc(tl, dl, dt, gamma, False, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
            torch.cuda.synchronize()
            assert (int(out_n.item()), int(out_z.item())) == (gamma, -1)
        seen.add(bonus)
        s.step_idx[0] += 1
    assert seen == {True, False}, "both a rejection and an all-accepted step must have occurred"
    with pytest.raises(B.PacerError) as e:
        B.pacer_accept_noalloc(tl, dl, dt, 32, True, V, mode, 1.0, 0, 0, 0, out_n, out_z, stream)
    assert e.value.code == B.EOVERFLOW
    s.close()
