"""ctypes binding of libpacer.so (include/pacer.h): argument marshalling only.

Every function here has the name of the C entry point it calls and does nothing but convert
arguments (torch tensors -> device pointers, python lists -> C arrays) and raise on a non-zero
status.  PyTorch supplies device memory and the stream; all arithmetic runs in the library's
HIP kernels.  There is no fallback: if the library has not been built, importing this module
raises.
"""
import ctypes as C
import os

import torch  # imported first: the library resolves libamdhip64 to the runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
# PACER_LIB: another build of the same library (e.g. one compiled with -DPACER_FENCED_HANDOVER, to compare)
LIB_PATH = os.environ.get("PACER_LIB") or os.path.join(_HERE, "libpacer.so")

OK, EINVAL, ESTATE, EOVERFLOW, EHIP, ENUMERIC = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
TARGET, DRAFT, PREVERIFY = 0, 1, 2
GREEDY, SAMPLE = 0, 1
HALT_MEAN, HALT_ANY, HALT_LAST = 0, 1, 2
T_EMBED, T_FINAL_NORM, T_HEAD, T_ATTN_NORM, T_WQKV, T_WO, T_FFN_NORM, T_WGU, T_WD, T_POSEMB, T_CLS = range(11)
PEEK_DRAFT_LOGITS, PEEK_DRAFT_HIDDEN, PEEK_DRAFT_TOKENS, PEEK_TOKENS = range(4)

EXPORTS = [
    "pacer_create", "pacer_destroy", "pacer_last_error", "pacer_pack_weight", "pacer_bind",
    "pacer_kv_bytes", "pacer_bind_kv", "pacer_workspace_bytes", "pacer_bind_workspace",
    "pacer_prefill", "pacer_force_commit", "pacer_begin_step", "pacer_draft_step",
    "pacer_preverify_block", "pacer_wait_stop", "pacer_verify", "pacer_accept_rollback", "pacer_get_state",
    "pacer_peek", "pacer_profile_enable", "pacer_profile_read", "pacer_launch_plan", "pacer_accept_noalloc",
    "pacer_force_stop", "pacer_launch_count", "pacer_stream_probe",
    "pacer_draft_window",
]


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("max_seq", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32)]


class PvCfg(C.Structure):
    _fields_ = [("block", C.c_int32), ("gamma_max", C.c_int32), ("t0", C.c_float), ("rho", C.c_float),
                ("halting", C.c_int32)]


class PacerError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"pacer error {code}: {msg}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
    sig = {
        "pacer_create": (i32, [C.POINTER(vp), C.POINTER(ModelCfg), C.POINTER(ModelCfg), C.POINTER(PvCfg), i32, vp]),
        "pacer_destroy": (None, [vp]),
        "pacer_last_error": (C.c_char_p, [vp]),
        "pacer_pack_weight": (i32, [vp, vp, i32, i32, i32, i32, vp, vp]),
        "pacer_bind": (i32, [vp, i32, i32, i32, vp, u64]),
        "pacer_kv_bytes": (u64, [vp, i32]),
        "pacer_bind_kv": (i32, [vp, i32, vp, u64]),
        "pacer_workspace_bytes": (u64, [vp]),
        "pacer_bind_workspace": (i32, [vp, vp, u64]),
        "pacer_prefill": (i32, [vp, i32, vp, i32]),
        "pacer_force_commit": (i32, [vp, i32, i32, C.POINTER(i32), i32]),
        "pacer_begin_step": (i32, [vp, i32]),
        "pacer_draft_step": (i32, [vp, C.POINTER(i32), i32, i32, u64, u64]),
        "pacer_preverify_block": (i32, [vp, C.POINTER(i32), i32, vp, vp]),
        "pacer_wait_stop": (i32, [vp, C.POINTER(i32), i32, C.POINTER(i32)]),
        "pacer_verify": (i32, [vp, C.POINTER(i32), i32, C.POINTER(i32), vp]),
        "pacer_accept_rollback": (i32, [vp, C.POINTER(i32), i32, i32, C.POINTER(C.c_float), u64, u64, vp, vp, vp]),
        "pacer_get_state": (i32, [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(i32), C.POINTER(i32)]),
        "pacer_peek": (i32, [vp, i32, i32, C.POINTER(vp), C.POINTER(u64)]),
        "pacer_profile_enable": (i32, [vp, i32]),
        "pacer_launch_plan": (i32, [i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]),
        "pacer_profile_read": (i32, [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "pacer_stream_probe": (i32, [vp, u64, i32, vp, vp]),
        "pacer_draft_window": (i32, [vp, C.POINTER(i32), i32, i32, u64, u64, vp, vp, C.POINTER(i32)]),
        "pacer_force_stop": (i32, [vp, i32, i32]),
        "pacer_launch_count": (i32, [vp, C.POINTER(C.c_int64)]),
        "pacer_accept_noalloc": (i32, [vp, vp, vp, i32, i32, i32, i32, C.c_float, u64, u64, i32, vp, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()


def _chk(ctx, rc):
    if rc != OK:
        msg = _lib.pacer_last_error(ctx).decode() if ctx else "invalid arguments"
        raise PacerError(rc, msg)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _i32s(v):
    return (C.c_int32 * len(v))(*v)


def model_cfg(shape, max_seq, dtype):
    return ModelCfg(shape["n_layers"], shape["d_model"], shape["n_heads"], shape["head_dim"],
                    shape["d_ffn"], shape["vocab"], max_seq, shape["rope_theta"], shape["rms_eps"],
                    BF16 if dtype == "bf16" else F32)


def pacer_create(target, draft, pv, max_batch, stream):
    ctx = C.c_void_p()
    rc = _lib.pacer_create(C.byref(ctx), C.byref(target), C.byref(draft), C.byref(pv), max_batch, C.c_void_p(stream))
    _chk(None, rc)
    return ctx


def pacer_destroy(ctx):
    _lib.pacer_destroy(ctx)


def pacer_last_error(ctx):
    return _lib.pacer_last_error(ctx).decode()


def pacer_pack_weight(dst, src, tensor_id, head_dim, dev_not_finite, stream):
    n_out, n_in = src.shape
    _chk(None, _lib.pacer_pack_weight(_ptr(dst), _ptr(src), n_out, n_in, tensor_id, head_dim, _ptr(dev_not_finite),
                                      C.c_void_p(stream)))


def pacer_bind(ctx, which, tensor_id, layer, t):
    _chk(ctx, _lib.pacer_bind(ctx, which, tensor_id, layer, _ptr(t), t.numel() * t.element_size()))


def pacer_kv_bytes(ctx, which):
    return int(_lib.pacer_kv_bytes(ctx, which))


def pacer_bind_kv(ctx, which, t):
    _chk(ctx, _lib.pacer_bind_kv(ctx, which, _ptr(t), t.numel() * t.element_size()))


def pacer_workspace_bytes(ctx):
    return int(_lib.pacer_workspace_bytes(ctx))


def pacer_bind_workspace(ctx, t):
    _chk(ctx, _lib.pacer_bind_workspace(ctx, _ptr(t), t.numel() * t.element_size()))


def pacer_prefill(ctx, seq, dev_tokens):
    _chk(ctx, _lib.pacer_prefill(ctx, seq, _ptr(dev_tokens), dev_tokens.numel()))


def pacer_force_commit(ctx, seq, start, tokens):
    _chk(ctx, _lib.pacer_force_commit(ctx, seq, start, _i32s(tokens), len(tokens)))


def pacer_begin_step(ctx, seq):
    _chk(ctx, _lib.pacer_begin_step(ctx, seq))


def pacer_draft_step(ctx, seqs, mode, rng_seed, rng_ctr):
    _chk(ctx, _lib.pacer_draft_step(ctx, _i32s(seqs), len(seqs), mode, rng_seed, rng_ctr))


def pacer_draft_window(ctx, seqs, mode, rng_seed, rng_ctr, dev_alpha, dev_stop):
    out = (C.c_int32 * len(seqs))()
    _chk(ctx, _lib.pacer_draft_window(ctx, _i32s(seqs), len(seqs), mode, rng_seed, rng_ctr, _ptr(dev_alpha), _ptr(dev_stop), out))
    return list(out)


def pacer_preverify_block(ctx, seqs, dev_alpha, dev_stop):
    _chk(ctx, _lib.pacer_preverify_block(ctx, _i32s(seqs), len(seqs), _ptr(dev_alpha), _ptr(dev_stop)))


def pacer_stream_probe(src, sink, stream, repeat=1):
    rc = _lib.pacer_stream_probe(_ptr(src), src.numel() * src.element_size(), repeat, _ptr(sink), C.c_void_p(stream))
    if rc != OK:
        raise PacerError(rc, _lib.pacer_last_error(None).decode())


def pacer_force_stop(ctx, seq, flag):
    _chk(ctx, _lib.pacer_force_stop(ctx, seq, flag))


def pacer_launch_count(ctx):
    n = C.c_int64()
    _chk(ctx, _lib.pacer_launch_count(ctx, C.byref(n)))
    return n.value


def pacer_wait_stop(ctx, seqs):
    out = (C.c_int32 * len(seqs))()
    _chk(ctx, _lib.pacer_wait_stop(ctx, _i32s(seqs), len(seqs), out))
    return list(out)


def pacer_verify(ctx, seqs, gamma_override, dev_logits):
    go = None if gamma_override is None else _i32s(gamma_override)
    _chk(ctx, _lib.pacer_verify(ctx, _i32s(seqs), len(seqs), go, _ptr(dev_logits)))


def pacer_accept_rollback(ctx, seqs, mode, beta, rng_seed, rng_ctr, dev_logits, dev_n, dev_z):
    b = (C.c_float * len(beta))(*beta)
    _chk(ctx, _lib.pacer_accept_rollback(ctx, _i32s(seqs), len(seqs), mode, b, rng_seed, rng_ctr,
                                         _ptr(dev_logits), _ptr(dev_n), _ptr(dev_z)))


def pacer_accept_noalloc(dev_target_logits, dev_draft_logits, dev_draft_tokens, gamma, bonus_row, vocab, mode, beta,
                         rng_seed, rng_ctr, seq, dev_n, dev_z, stream):
    rc = _lib.pacer_accept_noalloc(_ptr(dev_target_logits), _ptr(dev_draft_logits), _ptr(dev_draft_tokens), gamma,
                                   1 if bonus_row else 0, vocab, mode, beta, rng_seed, rng_ctr, seq, _ptr(dev_n), _ptr(dev_z),
                                   C.c_void_p(stream))
    if rc != OK:
        raise PacerError(rc, _lib.pacer_last_error(None).decode())


def pacer_get_state(ctx, seq):
    g, ln, n, z = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    t = C.c_float()
    _chk(ctx, _lib.pacer_get_state(ctx, seq, C.byref(g), C.byref(ln), C.byref(t), C.byref(n), C.byref(z)))
    return dict(gamma=g.value, len=ln.value, t=t.value, n_accepted=n.value, next_token=z.value)


def pacer_peek(ctx, seq, what):
    p, nb = C.c_void_p(), C.c_uint64()
    _chk(ctx, _lib.pacer_peek(ctx, seq, what, C.byref(p), C.byref(nb)))
    return p.value, nb.value


def pacer_launch_plan(n_out, n_in, rows, operand_parts):
    nt, ksb = C.c_int32(), C.c_int32()
    rc = _lib.pacer_launch_plan(n_out, n_in, rows, operand_parts, C.byref(nt), C.byref(ksb))
    if rc != OK:
        raise PacerError(rc, "pacer_launch_plan: bad arguments")
    return nt.value, ksb.value


def pacer_profile_enable(ctx, on):
    _chk(ctx, _lib.pacer_profile_enable(ctx, 1 if on else 0))


def pacer_profile_read(ctx):
    n, ms, by = C.c_int64(), C.c_double(), C.c_double()
    _chk(ctx, _lib.pacer_profile_read(ctx, C.byref(n), C.byref(ms), C.byref(by)))
    return n.value, ms.value, by.value
