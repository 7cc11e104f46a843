"""Thin ctypes binding of libsd.so (argument marshalling only).

Every step of the hot path runs in the HIP library; this module converts
Python / torch arguments to the plain pointers and sizes of include/sd.h.
PyTorch provides device memory and the stream, nothing else.  Importing this
module fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsd.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2211_17192_amd.build` first")
lib = C.CDLL(LIB_PATH)

SD_OK, SD_EINVAL, SD_ESTATE, SD_ERANGE, SD_ENOMEM, SD_EHIP = range(6)
SD_F32, SD_BF16 = 0, 1
SD_MAX_GAMMA = 15
SD_FLAG_GRAPH, SD_FLAG_PROFILE, SD_FLAG_BETA, SD_FLAG_SCATTER_PAGES, SD_FLAG_SEPARATE_CROSS_Q = 1, 2, 4, 8, 16
STATUS_NAMES = ["SD_OK", "SD_EINVAL", "SD_ESTATE", "SD_ERANGE", "SD_ENOMEM", "SD_EHIP"]


class SdError(RuntimeError):
    def __init__(self, status, msg=""):
        self.status = status
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {msg}")


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


lib.sd_spec_sample_scratch_bytes.restype = C.c_size_t
lib.sd_spec_sample_scratch_bytes.argtypes = [C.c_int32, C.c_int32]
lib.sd_spec_sample.restype = C.c_int
lib.sd_spec_sample.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]


class _Sampling(C.Structure):
    _fields_ = [("lenience", C.c_float), ("top_k", C.c_int32), ("top_p", C.c_float)]


lib.sd_spec_sample_ex.restype = C.c_int
lib.sd_spec_sample_ex.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                                     C.POINTER(_Sampling), C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_void_p, C.c_void_p]
lib.sd_spec_sample_static.restype = C.c_int
lib.sd_spec_sample_static.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                                         C.POINTER(_Sampling), C.c_void_p, C.c_void_p, C.c_void_p,
                                                         C.c_void_p]
SD_SPEC_SAMPLE_STATIC_MAX_ROWS = 256
lib.sd_choose_gamma.restype = C.c_int
lib.sd_choose_gamma.argtypes = [C.c_double, C.c_double, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double)]


def choose_gamma(alpha: float, c: float, gamma_max: int):
    """sd_choose_gamma: (gamma, predicted improvement factor).  Host arithmetic only."""
    g, v = C.c_int32(0), C.c_double(0.0)
    st = lib.sd_choose_gamma(float(alpha), float(c), int(gamma_max), C.byref(g), C.byref(v))
    if st != SD_OK:
        raise SdError(st, "sd_choose_gamma")
    return g.value, v.value


def spec_sample_scratch(rows: int, gamma: int) -> torch.Tensor:
    n = lib.sd_spec_sample_scratch_bytes(rows, gamma)
    if n == 0:
        raise SdError(SD_EINVAL, "rows / gamma out of range")
    return torch.zeros(n, dtype=torch.uint8, device="cuda")


def spec_sample(p_logits, q_logits, x, r, s, temperature: float, scratch=None, out_n=None, out_t=None,
                lenience=None, beta=None, top_k=0, top_p=0.0):
    """sd_spec_sample on cuda tensors: p_logits [rows, gamma+1, V] fp32, q_logits
    [rows, gamma, V] fp32, x [rows, gamma] int32, r [rows, gamma] fp32, s [rows] fp32.
    Returns device tensors (n [rows], t [rows]); asynchronous on the current stream.
    With lenience or beta (a [rows, gamma] fp32 cuda tensor that receives the
    acceptance probabilities) the call goes to sd_spec_sample_ex."""
    rows, g1, V = p_logits.shape
    gamma = g1 - 1
    for t_, dt in ((p_logits, torch.float32), (q_logits, torch.float32), (x, torch.int32)):
        assert t_.is_cuda and t_.is_contiguous() and t_.dtype == dt
    assert q_logits.shape == (rows, gamma, V) and x.shape == (rows, gamma)
    if scratch is None:
        scratch = spec_sample_scratch(rows, gamma)
    if out_n is None:
        out_n = torch.empty(rows, dtype=torch.int32, device="cuda")
        out_t = torch.empty(rows, dtype=torch.int32, device="cuda")
    if lenience is None and beta is None and not top_k and not top_p:
        st = lib.sd_spec_sample(_ptr(p_logits), _ptr(q_logits), _ptr(x), _ptr(r), _ptr(s), rows, gamma, V,
                                float(temperature), _ptr(out_n), _ptr(out_t), _ptr(scratch), _stream())
    else:
        if beta is not None:
            assert beta.is_cuda and beta.is_contiguous() and beta.dtype == torch.float32 and beta.shape == (rows, gamma)
        opt = _Sampling(1.0 if lenience is None else float(lenience), int(top_k), float(top_p))
        st = lib.sd_spec_sample_ex(_ptr(p_logits), _ptr(q_logits), _ptr(x), _ptr(r), _ptr(s), rows, gamma, V,
                                   float(temperature), C.byref(opt), _ptr(out_n), _ptr(out_t),
                                   _ptr(beta) if beta is not None else None, _ptr(scratch), _stream())
    if st != SD_OK:
        raise SdError(st, "sd_spec_sample")
    return out_n, out_t


def spec_sample_static(p_logits, q_logits, x, r, s, temperature: float, out_n, out_t, lenience=None, beta=None,
                       top_k=0, top_p=0.0):
    """sd_spec_sample_static: as spec_sample, with the library's own fixed scratch array.  The
    outputs are the caller's tensors (nothing is allocated here either)."""
    rows, g1, V = p_logits.shape
    gamma = g1 - 1
    for t_, dt in ((p_logits, torch.float32), (q_logits, torch.float32), (x, torch.int32), (out_n, torch.int32),
                   (out_t, torch.int32)):
        assert t_.is_cuda and t_.is_contiguous() and t_.dtype == dt
    assert q_logits.shape == (rows, gamma, V) and x.shape == (rows, gamma) and out_n.numel() == rows and out_t.numel() == rows
    if beta is not None:
        assert beta.is_cuda and beta.is_contiguous() and beta.dtype == torch.float32 and beta.shape == (rows, gamma)
    opt = _Sampling(1.0 if lenience is None else float(lenience), int(top_k), float(top_p))
    st = lib.sd_spec_sample_static(_ptr(p_logits), _ptr(q_logits), _ptr(x), _ptr(r), _ptr(s), rows, gamma, V,
                                   float(temperature), C.byref(opt), _ptr(out_n), _ptr(out_t),
                                   _ptr(beta) if beta is not None else None, _stream())
    if st != SD_OK:
        raise SdError(st, (lib.sd_last_error(None) or b"").decode())
    return out_n, out_t


# --------------------------------------------------------------------------
# the model API
# --------------------------------------------------------------------------
class _ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("arch", "n_layers", "d_model", "n_heads", "n_kv_heads", "d_head",
                                         "d_ff", "vocab", "max_len", "enc_len", "rel_buckets", "rel_max_dist")] + \
               [("rope_theta", C.c_float), ("logit_scale", C.c_float), ("norm_eps", C.c_float), ("dtype", C.c_int32)]


class _Tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dev", C.c_void_p), ("ndim", C.c_int32), ("shape", C.c_int64 * 4),
                ("dtype", C.c_int32)]


class _RuntimeCfg(C.Structure):
    _fields_ = [("batch", C.c_int32), ("max_gamma", C.c_int32), ("page_size", C.c_int32),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
                ("flags", C.c_int32)]


class _Stats(C.Structure):
    _fields_ = [("draft_ms", C.c_double), ("verify_ms", C.c_double), ("accept_ms", C.c_double),
                ("steps", C.c_int64), ("tokens", C.c_int64), ("accepted", C.c_int64), ("fallbacks", C.c_int64),
                ("ffn_in_ms_sum", C.c_double), ("ffn_in_launches", C.c_int64),
                ("tested", C.c_int64), ("beta_sum", C.c_double), ("beta_count", C.c_int64)]


lib.sd_workspace_bytes.restype = C.c_size_t
lib.sd_workspace_bytes.argtypes = [C.POINTER(_ModelCfg), C.POINTER(_ModelCfg), C.POINTER(_RuntimeCfg)]
lib.sd_load_models.restype = C.c_int
lib.sd_load_models.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_ModelCfg), C.POINTER(_Tensor), C.c_int32,
                               C.POINTER(_ModelCfg), C.POINTER(_Tensor), C.c_int32, C.POINTER(_RuntimeCfg)]
lib.sd_prefill.restype = C.c_int
lib.sd_prefill.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p]
lib.sd_step.restype = C.c_int
lib.sd_step.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_float,
                        C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.sd_step_baseline.restype = C.c_int
lib.sd_step_baseline.argtypes = [C.c_void_p, C.c_float, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
lib.sd_reset.restype = C.c_int
lib.sd_reset.argtypes = [C.c_void_p, C.c_int32]
lib.sd_free.restype = None
lib.sd_free.argtypes = [C.c_void_p]
lib.sd_last_error.restype = C.c_char_p
lib.sd_last_error.argtypes = [C.c_void_p]
lib.sd_debug_logits.restype = C.c_int
lib.sd_debug_logits.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_float), C.c_size_t]
lib.sd_get_stats.restype = C.c_int
lib.sd_get_stats.argtypes = [C.c_void_p, C.POINTER(_Stats)]
lib.sd_set_flags.restype = C.c_int
lib.sd_set_flags.argtypes = [C.c_void_p, C.c_int32]
lib.sd_time_ffn_in.restype = C.c_int
lib.sd_time_ffn_in.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
lib.sd_time_forward.restype = C.c_int
lib.sd_time_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
SD_OP = {"qkv": 1, "attn": 2, "o": 4, "cross_q": 8, "cross_attn": 16, "cross_o": 32, "ffn_in": 64, "ffn_out": 128,
         "head": 256}
lib.sd_time_stream_read.restype = C.c_int
lib.sd_time_stream_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
lib.sd_set_sampling.restype = C.c_int
lib.sd_set_sampling.argtypes = [C.c_void_p, C.POINTER(_Sampling)]
lib.sd_set_table_draft.restype = C.c_int
lib.sd_set_table_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
lib.sd_set_copy_draft.restype = C.c_int
lib.sd_set_copy_draft.argtypes = [C.c_void_p, C.c_int32]
lib.sd_measure_cost.restype = C.c_int
lib.sd_measure_cost.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
lib.sd_autotune_gamma.restype = C.c_int
lib.sd_autotune_gamma.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]


def _cfg_struct(cfg: dict) -> _ModelCfg:
    s = _ModelCfg()
    for k in ("arch", "n_layers", "d_model", "n_heads", "n_kv_heads", "d_head", "d_ff", "vocab", "max_len",
              "enc_len", "rel_buckets", "rel_max_dist"):
        setattr(s, k, int(cfg[k]))
    s.rope_theta = float(cfg["rope_theta"])
    s.logit_scale = float(cfg["logit_scale"])
    s.norm_eps = float(cfg["norm_eps"])
    s.dtype = SD_BF16 if cfg["dtype"] == "bf16" else SD_F32
    return s


def _tensor_array(w: dict, keep: list):
    arr = (_Tensor * len(w))()
    for i, (name, t) in enumerate(w.items()):
        assert t.is_cuda and t.is_contiguous(), name
        nb = name.encode()
        keep.append(nb)
        arr[i].name = nb
        arr[i].dev = t.data_ptr()
        arr[i].ndim = t.dim()
        for j, v in enumerate(t.shape):
            arr[i].shape[j] = int(v)
        arr[i].dtype = SD_BF16 if t.dtype == torch.bfloat16 else SD_F32
    return arr


class SpecDecoder:
    """One (Mp, Mq) pair bound with sd_load_models.  Weights are dicts name -> cuda tensor."""

    def __init__(self, cfg_p: dict, w_p: dict, cfg_q: dict, w_q: dict, max_gamma: int = 7,
                 page_size: int = 16, flags: int = 0, batch: int = 1):
        self._ctx = C.c_void_p()
        self.cfg_p, self.cfg_q = cfg_p, cfg_q
        self.batch = int(batch)
        cp, cq = _cfg_struct(cfg_p), _cfg_struct(cfg_q)
        rt = _RuntimeCfg(batch=self.batch, max_gamma=max_gamma, page_size=page_size, workspace=None,
                         workspace_bytes=0, stream=None, flags=flags)
        need = lib.sd_workspace_bytes(C.byref(cp), C.byref(cq), C.byref(rt))
        if need == 0:
            raise SdError(SD_EINVAL, "invalid model / runtime configuration")
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        rt.workspace, rt.workspace_bytes = base, need
        keep = []
        tp, tq = _tensor_array(w_p, keep), _tensor_array(w_q, keep)
        torch.cuda.synchronize()                      # weights were produced on torch's streams
        st = lib.sd_load_models(C.byref(self._ctx), C.byref(cp), tp, len(w_p), C.byref(cq), tq, len(w_q),
                                C.byref(rt))
        if st != SD_OK:
            raise SdError(st, (lib.sd_last_error(None) or b"").decode())
        self.vocab = int(cfg_p["vocab"])
        self.workspace_bytes = need

    def _check(self, st):
        if st != SD_OK:
            raise SdError(st, (lib.sd_last_error(self._ctx) or b"").decode())

    def prefill(self, prompt, enc_p=None, enc_q=None, row: int = 0):
        p = np.ascontiguousarray(np.asarray(prompt, dtype=np.int32))
        torch.cuda.synchronize()
        self._check(lib.sd_prefill(self._ctx, int(row), p.ctypes.data_as(C.POINTER(C.c_int32)), len(p),
                                   _ptr(enc_p), _ptr(enc_q)))

    def step(self, gamma: int, temperature: float, uniforms=None, prefix=None):
        """One run of Algorithm 1.  batch 1: uniforms [2*gamma+1] -> (n, tokens).
        batch B > 1: uniforms [B, 2*gamma+1] -> list of (n, tokens), one per sequence."""
        B = self.batch
        out = (C.c_int32 * (B * (gamma + 1)))()
        n = (C.c_int32 * B)()
        u = None
        if uniforms is not None:
            ua = np.ascontiguousarray(np.asarray(uniforms, dtype=np.float32))
            assert ua.shape == ((2 * gamma + 1,) if B == 1 else (B, 2 * gamma + 1))
            u = ua.ctypes.data_as(C.POINTER(C.c_float))
        pp, pl = None, 0
        if prefix is not None:
            pa = np.ascontiguousarray(np.asarray(prefix, dtype=np.int32))
            pp, pl = pa.ctypes.data_as(C.POINTER(C.c_int32)), len(pa)
        self._check(lib.sd_step(self._ctx, pp, pl, gamma, float(temperature), u, out, n))
        res = [(n[b], [out[b * (gamma + 1) + i] for i in range(n[b] + 1)]) for b in range(B)]
        return res[0] if B == 1 else res

    def step_baseline(self, temperature: float, uniform=None):
        """One standard decoding step: a token (batch 1) or a list of tokens, one per sequence."""
        B = self.batch
        tok = (C.c_int32 * B)()
        u = None
        if uniform is not None:
            ua = np.ascontiguousarray(np.asarray(uniform, dtype=np.float32).reshape(B))
            u = ua.ctypes.data_as(C.POINTER(C.c_float))
        self._check(lib.sd_step_baseline(self._ctx, float(temperature), u, tok))
        return tok[0] if B == 1 else [tok[b] for b in range(B)]

    def logits(self, which: int, rows: int) -> np.ndarray:
        out = np.empty((rows, self.vocab), dtype=np.float32)
        self._check(lib.sd_debug_logits(self._ctx, which, out.ctypes.data_as(C.POINTER(C.c_float)), out.size))
        return out

    def stats(self) -> dict:
        s = _Stats()
        self._check(lib.sd_get_stats(self._ctx, C.byref(s)))
        return {k: getattr(s, k) for k, _ in _Stats._fields_}

    def time_ffn_in(self, rows: int, reps: int = 20) -> float:
        """Mean duration (microseconds) of one launch of Mp's FFN-in GEMM over `rows` rows."""
        us = C.c_double(0.0)
        self._check(lib.sd_time_ffn_in(self._ctx, int(rows), int(reps), C.byref(us)))
        return us.value

    def time_forward(self, which: int, rows: int, skip_ops: int = 0, reps: int = 20) -> float:
        """Microseconds of one graph-replayed forward of Mp (which 0) or Mq (1) over `rows` rows with
        the launches in skip_ops (SD_OP bits) left out."""
        us = C.c_double(0.0)
        self._check(lib.sd_time_forward(self._ctx, int(which), int(rows), int(skip_ops), int(reps), C.byref(us)))
        return us.value

    def stream_read_GBps(self, which: int = 0, reps: int = 10) -> float:
        """GB/s of a pure read of the model's resident weights (the chip's ceiling for the GEMMs' access shape)."""
        us, nb = C.c_double(0.0), C.c_double(0.0)
        self._check(lib.sd_time_stream_read(self._ctx, int(which), int(reps), C.byref(us), C.byref(nb)))
        return nb.value / us.value / 1e3

    def set_flags(self, flags: int):
        self._check(lib.sd_set_flags(self._ctx, int(flags)))

    def set_sampling(self, lenience: float = 1.0, top_k: int = 0, top_p: float = 0.0):
        opt = _Sampling(float(lenience), int(top_k), float(top_p))
        self._check(lib.sd_set_sampling(self._ctx, C.byref(opt)))

    def set_table_draft(self, table=None, row_of=None):
        """Draft from an n-gram table (cuda fp32 [rows, vocab]; row_of: cuda int32 [vocab] or None
        for a unigram model) instead of Mq; None goes back to Mq.  The tensors are kept alive here."""
        if table is None:
            self._check(lib.sd_set_table_draft(self._ctx, None, None, 0))
            self._draft = None
            return
        assert table.is_cuda and table.is_contiguous() and table.dtype == torch.float32 and table.shape[1] == self.vocab
        if row_of is not None:
            assert row_of.is_cuda and row_of.is_contiguous() and row_of.dtype == torch.int32 and row_of.numel() == self.vocab
        torch.cuda.synchronize()
        self._check(lib.sd_set_table_draft(self._ctx, _ptr(table), _ptr(row_of) if row_of is not None else None,
                                           int(table.shape[0])))
        self._draft = (table, row_of)

    def set_copy_draft(self, match: int = 0):
        """Draft by copying from the context: the token after the most recent earlier occurrence
        of the last `match` tokens (else the table draft / the uniform model); 0 turns it off."""
        self._check(lib.sd_set_copy_draft(self._ctx, int(match)))

    def measure_cost(self, reps: int = 20):
        """(microseconds of one Mq draft step, microseconds of one standard Mp decoding step)."""
        a, b = C.c_double(0.0), C.c_double(0.0)
        self._check(lib.sd_measure_cost(self._ctx, int(reps), C.byref(a), C.byref(b)))
        return a.value, b.value

    def autotune_gamma(self, reps: int = 20) -> dict:
        g = C.c_int32(0)
        a, c, v = C.c_double(0.0), C.c_double(0.0), C.c_double(0.0)
        self._check(lib.sd_autotune_gamma(self._ctx, int(reps), C.byref(g), C.byref(a), C.byref(c), C.byref(v)))
        return {"gamma": g.value, "alpha": a.value, "c": c.value, "improvement": v.value}

    def reset(self, row: int = -1):
        self._check(lib.sd_reset(self._ctx, int(row)))

    def close(self):
        if self._ctx:
            lib.sd_free(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
