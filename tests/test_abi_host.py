"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and validates
arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    so = os.path.join(ROOT, "paper_2602_01274_amd", "libpacer.so")
    if not os.path.exists(so):
        import __graft_entry__ as g
        g.build()
    import paper_2602_01274_amd.binding as b
    return b


def test_library_exports_every_declared_symbol(B):
    hdr = open(os.path.join(ROOT, "include", "pacer.h")).read()
    declared = set(re.findall(r"\b(pacer_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(B._lib, name) is not None


def _cfgs(B, **over):
    t = dict(n_layers=2, d_model=128, n_heads=2, head_dim=64, d_ffn=256, vocab=64, rope_theta=1e4, rms_eps=1e-5)
    t.update(over)
    return B.model_cfg(t, 64, "bf16"), B.model_cfg(dict(t, n_layers=1), 64, "bf16")


def test_create_validates_shapes(B):
    t, d = _cfgs(B)
    ctx = B.pacer_create(t, d, B.PvCfg(2, 8, 0.5, 1.05, 0), 1, 0)
    assert B.pacer_workspace_bytes(ctx) > 0
    assert B.pacer_kv_bytes(ctx, B.TARGET) == 1 * 2 * 2 * 64 * 128 * 2
    B.pacer_destroy(ctx)
    bad = [
        (dict(head_dim=32), B.PvCfg(2, 8, 0.5, 1.05, 0), 1),       # unsupported head size
        (dict(d_model=120), B.PvCfg(2, 8, 0.5, 1.05, 0), 1),       # heads * head_dim != d_model
        (dict(d_ffn=250), B.PvCfg(2, 8, 0.5, 1.05, 0), 1),         # bf16 needs multiples of 32
        (dict(), B.PvCfg(3, 8, 0.5, 1.05, 0), 1),                  # gamma_max not a multiple of b
        (dict(), B.PvCfg(0, 8, 0.5, 1.05, 0), 1),
        (dict(), B.PvCfg(2, 8, 0.5, 1.05, 0), 17),                 # batch too large
        (dict(), B.PvCfg(2, 8, 0.5, 0.0, 0), 1),                   # rho must be positive
        (dict(), B.PvCfg(2, 8, 0.5, 1.05, 3), 1),                  # unknown halting rule
    ]
    for over, pv, mb in bad:
        t, d = _cfgs(B, **over)
        with pytest.raises(B.PacerError) as e:
            B.pacer_create(t, d, pv, mb, 0)
        assert e.value.code == B.EINVAL


def test_calls_out_of_order_and_bad_arguments_fail_on_the_host(B):
    import numpy as np
    t, d = _cfgs(B)
    ctx = B.pacer_create(t, d, B.PvCfg(2, 8, 0.5, 1.05, 0), 2, 0)

    class Fake:            # a host buffer posing as a tensor: bind only records the pointer
        def __init__(self, nbytes):
            self.a = np.zeros(nbytes + 512, dtype=np.uint8)
            self.n = nbytes
        def data_ptr(self):
            return (self.a.ctypes.data + 255) // 256 * 256
        def numel(self):
            return self.n
        def element_size(self):
            return 1
    with pytest.raises(B.PacerError) as e:
        B.pacer_bind(ctx, B.TARGET, B.T_WO, 0, Fake(100))
    assert e.value.code == B.EINVAL and "expects" in str(e.value)
    with pytest.raises(B.PacerError) as e:
        B.pacer_bind(ctx, B.TARGET, B.T_WO, 5, Fake(128 * 128 * 2))
    assert e.value.code == B.EINVAL
    with pytest.raises(B.PacerError) as e:
        B.pacer_bind(ctx, B.TARGET, B.T_CLS, 0, Fake(2 * 128 * 4))     # M_B-only tensor
    assert e.value.code == B.EINVAL
    keep = Fake(128 * 128 * 2)
    B.pacer_bind(ctx, B.TARGET, B.T_WO, 1, keep)
    with pytest.raises(B.PacerError) as e:
        B.pacer_bind_kv(ctx, B.DRAFT, Fake(10))
    assert e.value.code == B.EINVAL
    # nothing bound yet: every hot call reports a state error, never reaches the GPU
    for call in (lambda: B.pacer_begin_step(ctx, 0),
                 lambda: B.pacer_draft_step(ctx, [0], B.GREEDY, 0, 0),
                 lambda: B.pacer_verify(ctx, [0], None, Fake(8)),
                 lambda: B.pacer_prefill(ctx, 0, Fake(8))):
        with pytest.raises(B.PacerError) as e:
            call()
        assert e.value.code == B.ESTATE
    assert "workspace" in B.pacer_last_error(ctx)
    st = B.pacer_get_state(ctx, 1)
    assert st["len"] == 0 and st["n_accepted"] == -1
    with pytest.raises(B.PacerError) as e:
        B.pacer_get_state(ctx, 2)
    assert e.value.code == B.EINVAL
    B.pacer_destroy(ctx)


def test_launch_plan_of_the_few_tile_projections(B):
    """Tiles per block and K slices across blocks for the target's O and down projections: the
    measured choices at the three model widths, and bounds that hold for any size."""
    for rows in (5, 13, 17, 32):
        assert B.pacer_launch_plan(4096, 11008, rows, 2) == (2, 2)      # 7B down: 256 tiles, 256 blocks
        assert B.pacer_launch_plan(5120, 13824, rows, 2) == (4, 3)      # 13B down: 320 tiles, 240 blocks
        assert B.pacer_launch_plan(7168, 19200, rows, 2) == (4, 2)      # 33B down: 448 tiles, 224 blocks
        if rows <= 17:
            assert B.pacer_launch_plan(4096, 4096, rows, 1) == (1, 1)   # 7B O, hi only: its operand is small
    assert B.pacer_launch_plan(768, 768, 4, 1) == (1, 1)                # K below 2048: never split
    for n_out in range(16, 8192, 16 * 7):
        for n_in in (2048, 4096, 11008, 19200):
            for rows in (1, 9, 17, 32):
                for parts in (1, 2):
                    nt, ksb = B.pacer_launch_plan(n_out, n_in, rows, parts)
                    tiles = n_out // 16
                    groups = -(-tiles // nt)
                    assert 1 <= ksb <= 3 and 1 <= nt <= 4 and ksb <= max(nt, 1)
                    assert groups <= 512                                   # arrival counters in the workspace
                    assert groups * ksb * nt * 2 * 256 <= 1 << 20 or ksb == 1   # partial tiles fit their 4 MiB
                    assert n_in // 32 // ksb >= 8                          # every slice has K steps for all 8 waves
    for bad in ((8, 4096, 4, 1), (4096, 100, 4, 1), (4096, 4096, 0, 1), (4096, 4096, 33, 1), (4096, 4096, 4, 3), (16 * 512, 4096, 4, 1)):
        with pytest.raises(B.PacerError):
            B.pacer_launch_plan(*bad)


def test_accept_noalloc_validates_on_the_host(B):
    """The allocation-free acceptance call checks its arguments before it touches a GPU: null pointers, modes,
    and a window beyond the fixed scratch's capacity (refused with PACER_EOVERFLOW and a message naming the limit)."""
    import numpy as np

    class Fake:
        def __init__(self, nbytes):
            self.a = np.zeros(nbytes, dtype=np.uint8)
        def data_ptr(self):
            return self.a.ctypes.data
    f = Fake(64)
    ok = dict(dev_target_logits=f, dev_draft_logits=f, dev_draft_tokens=f, gamma=4, bonus_row=1, vocab=64, mode=B.GREEDY,
              beta=1.0, rng_seed=0, rng_ctr=0, seq=0, dev_n=f, dev_z=f, stream=0)
    for over, code in ((dict(dev_target_logits=None), B.EINVAL), (dict(dev_draft_tokens=None), B.EINVAL),
                       (dict(dev_z=None), B.EINVAL), (dict(mode=2), B.EINVAL), (dict(gamma=-1), B.EINVAL),
                       (dict(seq=16), B.EINVAL), (dict(vocab=0), B.EINVAL), (dict(gamma=0, bonus_row=0), B.EINVAL),
                       (dict(gamma=32), B.EOVERFLOW), (dict(gamma=1000), B.EOVERFLOW)):
        with pytest.raises(B.PacerError) as e:
            B.pacer_accept_noalloc(**dict(ok, **over))
        assert e.value.code == code, over
        if code == B.EOVERFLOW:
            assert "PACER_NOALLOC_MAX_GAMMA = 31" in str(e.value)


def test_force_stop_and_launch_count_validate_arguments(B):
    t, d = _cfgs(B)
    ctx = B.pacer_create(t, d, B.PvCfg(2, 8, 0.5, 1.05, 0), 2, 0)
    B.pacer_force_stop(ctx, 1, 1)
    B.pacer_force_stop(ctx, 1, -1)
    for seq, flag in ((2, 1), (-1, 0), (0, 2), (0, -2)):
        with pytest.raises(B.PacerError) as e:
            B.pacer_force_stop(ctx, seq, flag)
        assert e.value.code == B.EINVAL
    assert B.pacer_launch_count(ctx) == 0
    B.pacer_destroy(ctx)
