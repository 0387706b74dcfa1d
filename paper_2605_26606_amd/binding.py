"""ctypes binding of the C ABI in include/pc.h: argument marshalling only.

Every function takes torch tensors (device memory) or numpy arrays (host
memory) exactly where the header says "device" or "host", checks dtype and
contiguity, and passes raw pointers.  There is no fallback: if the library
is not built, importing any entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpc.so")

PC_OPT_USE_GRAPH = 1
PC_OPT_FORCE_SIMT = 2
PC_OPT_TIME_NEXT_STEP = 3
PC_OPT_FUSE_DECODE = 4
PC_KERNEL_ATTN_DECODE, PC_KERNEL_GEMM_QKV, PC_KERNEL_GEMM_WO = 0, 1, 2
PC_KERNEL_GEMM_GATE_UP, PC_KERNEL_GEMM_DOWN, PC_KERNEL_GEMM_LM_HEAD = 3, 4, 5
_DTYPES = {"fp32": 0, "bf16": 1}


class PcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("pc error %d: %s" % (code, msg))
        self.code = code


class _ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff", "vocab")] \
        + [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("act_dtype", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] \
        + [(n, C.POINTER(C.c_void_p)) for n in
           ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class _SchedConfig(C.Structure):
    _fields_ = [("p_lower", C.c_float), ("p_upper", C.c_float), ("p_solve", C.c_float), ("b_t", C.c_int32),
                ("max_delay", C.c_int32)]


PC_SCHED_STATS = ("step", "buffered_now", "pilot_batches", "prompts_seen", "buffered", "committed", "aged_out",
                  "evictions", "short_steps", "multi_round_steps")


class _CacheConfig(C.Structure):
    _fields_ = [("block_size", C.c_int32), ("kv_pool_bytes", C.c_int64), ("max_slots", C.c_int32),
                ("max_ctx", C.c_int32), ("max_batch_rows", C.c_int32)]


_lib = None


def library() -> C.CDLL:
    """The loaded HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2605_26606_amd.build` "
                              "(there is no CPU fallback)" % _LIB_PATH)
        lib = C.CDLL(_LIB_PATH)
        vp, i32, i64, f32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_uint64
        lib.pc_last_error.restype = C.c_char_p
        lib.pc_last_error.argtypes = []
        sigs = {
            "pc_create": [C.POINTER(_ModelConfig), C.POINTER(_Weights), C.POINTER(_CacheConfig), C.POINTER(vp)],
            "pc_destroy": [vp],
            "pc_set_option": [vp, i32, i32],
            "pc_kv_blocks": [vp, C.POINTER(i64), C.POINTER(i64)],
            "pc_slots": [vp, C.POINTER(i64), C.POINTER(i64)],
            "pc_timing_read": [vp, C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(i64), i32],
            "pc_prefill_shared": [vp, vp, vp, i32, vp, vp, vp],
            "pc_fork": [vp, vp, i32, i32, vp, vp],
            "pc_fork_need": [vp, vp, i32, i32, vp],
            "pc_decode_step": [vp, vp, vp, i32, vp, vp],
            "pc_decode_step_static": [vp, vp, vp, i32, vp, vp],
            "pc_release": [vp, vp, i32, i32],
            "pc_score": [vp, vp, vp, vp, i32, f32, vp, vp],
            "pc_sample": [vp, vp, i32, i32, f32, f32, u64, vp, vp, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp],
            "pc_saturation_count": [vp, C.POINTER(i64), i32],
            "pc_group_stats": [vp, vp, i32, vp, vp, vp, vp, vp],
            "pc_select_commit": [vp, i32, f32, f32, f32, i32, vp, vp, vp, vp, vp, vp],
            "pc_select_commit_var": [vp, vp, i32, f32, f32, f32, f32, i32, vp, vp, vp, vp, vp, vp],
            "pc_advantages": [vp, vp, i32, f32, vp, vp, vp, vp],
            "pc_sched_create": [C.POINTER(_SchedConfig), C.POINTER(vp)],
            "pc_sched_destroy": [vp],
            "pc_sched_pilot": [vp, vp, vp, vp, i32, vp, vp, vp],
            "pc_sched_commit": [vp, vp, vp, vp, vp, vp, vp, i32, vp],
            "pc_sched_evicted": [vp, vp, i32, vp],
            "pc_sched_stats": [vp, vp],
        }
        for name, args in sigs.items():
            fn = getattr(lib, name)
            fn.argtypes = args
            fn.restype = i32
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise PcError(rc, library().pc_last_error().decode("utf-8", "replace"))


def _dev(t: Optional[torch.Tensor], dtype, name: str):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _host_i32(a, name: str) -> np.ndarray:
    arr = np.ascontiguousarray(np.asarray(a), dtype=np.int32)
    if arr.ndim != 1:
        raise ValueError("%s must be one-dimensional" % name)
    return arr


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    return stream.cuda_stream or None


class Context:
    """Owns a pc_ctx.  `weights` is a dict of device tensors laid out as
    workloads.make_weights produces them; they are kept alive here."""

    def __init__(self, model, weights: dict, block_size: int = 64, kv_pool_bytes: int = 1 << 30,
                 max_slots: int = 1024, max_ctx: int = 2048, max_batch_rows: int = 4096, act_dtype: str = "default"):
        lib = library()
        self.model = model
        self.vocab = int(model.vocab)
        # the library copies the per-layer matrices into its own layout: only these three must outlive the
        # context (the caller is free to drop its per-layer tensors after this constructor returns)
        self._weights = {k: weights[k] for k in ("tok_embed", "lm_head", "final_norm")}
        mc = _ModelConfig(model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads, model.head_dim,
                          model.d_ff, model.vocab, model.rms_eps, model.rope_theta, _DTYPES[model.dtype],
                          {"default": 0, "bf16": 1, "f16": 2}[act_dtype])
        tdt = torch.float32 if model.dtype == "fp32" else torch.bfloat16
        L = model.n_layers

        def arr(name, dt):
            ts = weights[name]
            if len(ts) != L:
                raise ValueError("weights[%s] needs %d layers" % (name, L))
            return (C.c_void_p * L)(*[_dev(t, dt, name) for t in ts])

        self._arrays = {n: arr(n, tdt) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")}
        self._arrays.update({n: arr(n, torch.float32) for n in ("attn_norm", "ffn_norm")})
        w = _Weights(_dev(weights["tok_embed"], tdt, "tok_embed"), _dev(weights["lm_head"], tdt, "lm_head"),
                     _dev(weights["final_norm"], torch.float32, "final_norm"),
                     *[C.cast(self._arrays[n], C.POINTER(C.c_void_p)) for n in
                       ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")])
        cc = _CacheConfig(block_size, kv_pool_bytes, max_slots, max_ctx, max_batch_rows)
        self.max_slots, self.max_batch_rows = int(max_slots), int(max_batch_rows)
        h = C.c_void_p()
        _check(lib.pc_create(C.byref(mc), C.byref(w), C.byref(cc), C.byref(h)))
        self._h = h
        self._arrays = None

    @property
    def handle(self):
        if self._h is None:
            raise RuntimeError("context destroyed")
        return self._h

    def close(self):
        if getattr(self, "_h", None) is not None:
            library().pc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pc_set_option(ctx: Context, option: int, value: int):
    _check(library().pc_set_option(ctx.handle, option, value))


def pc_timing_read(ctx: Context, reset: bool = True):
    """(total_ms, launches, empty_ms, empty_pairs) over the event pairs recorded since the last
    reset (the "empty" pairs bracket nothing: the cost of the bracket); synchronises."""
    ms, n, ems, en = C.c_double(), C.c_int64(), C.c_double(), C.c_int64()
    _check(library().pc_timing_read(ctx.handle, C.byref(ms), C.byref(n), C.byref(ems), C.byref(en),
                                    1 if reset else 0))
    return ms.value, n.value, ems.value, en.value


def pc_saturation_count(ctx: Context, reset: bool = False) -> int:
    """Values clamped to the IEEE-half range on their way into activations or the KV cache since the last
    reset (0 unless the model's activations leave +-65504); synchronises the device."""
    n = C.c_int64()
    _check(library().pc_saturation_count(ctx.handle, C.byref(n), 1 if reset else 0))
    return n.value


def pc_kv_blocks(ctx: Context):
    f, t = C.c_int64(), C.c_int64()
    _check(library().pc_kv_blocks(ctx.handle, C.byref(f), C.byref(t)))
    return f.value, t.value


def pc_slots(ctx: Context):
    f, t = C.c_int64(), C.c_int64()
    _check(library().pc_slots(ctx.handle, C.byref(f), C.byref(t)))
    return f.value, t.value


def pc_prefill_shared(ctx: Context, prompt_tokens: torch.Tensor, cu_lens, last_logits: torch.Tensor, stream=None):
    """prompt_tokens: device int32 (packed); cu_lens: host int32 [P+1];
    last_logits: device fp32 [P, vocab] (written).  Returns handles (numpy int32 [P])."""
    cu = _host_i32(cu_lens, "cu_lens")
    P = len(cu) - 1
    if P < 0:
        raise ValueError("cu_lens needs at least one entry")
    if P > 0 and prompt_tokens.numel() < int(cu[-1]):
        raise ValueError("prompt_tokens shorter than cu_lens[-1]")
    if last_logits is not None and P > 0 and tuple(last_logits.shape) != (P, ctx.vocab):
        raise ValueError("last_logits must be [P, vocab]")
    handles = np.zeros(max(P, 1), np.int32)
    _check(library().pc_prefill_shared(ctx.handle, _dev(prompt_tokens, torch.int32, "prompt_tokens"),
                                       cu.ctypes.data, P, handles.ctypes.data,
                                       _dev(last_logits, torch.float32, "last_logits"), _stream_ptr(stream)))
    return handles[:P]


def pc_fork(ctx: Context, prompt_handle, max_new_tokens: int, stream=None) -> np.ndarray:
    ph = _host_i32(prompt_handle, "prompt_handle")
    out = np.zeros(max(len(ph), 1), np.int32)
    _check(library().pc_fork(ctx.handle, ph.ctypes.data, len(ph), int(max_new_tokens), out.ctypes.data,
                             _stream_ptr(stream)))
    return out[:len(ph)]


def pc_fork_need(ctx: Context, prompt_handle, max_new_tokens: int) -> np.ndarray:
    """KV blocks a fork of each handle would take (int64 [n]); changes nothing."""
    ph = _host_i32(prompt_handle, "prompt_handle")
    out = np.zeros(max(len(ph), 1), np.int64)
    _check(library().pc_fork_need(ctx.handle, ph.ctypes.data, len(ph), int(max_new_tokens), out.ctypes.data))
    return out[:len(ph)]


def pc_decode_step(ctx: Context, seq, tokens_in: torch.Tensor, logits: torch.Tensor, stream=None):
    s = seq if (isinstance(seq, np.ndarray) and seq.dtype == np.int32 and seq.flags.c_contiguous and seq.ndim == 1) \
        else _host_i32(seq, "seq")
    n = len(s)
    if n and (tokens_in.numel() < n or logits.numel() < n * ctx.vocab):
        raise ValueError("tokens_in / logits too small for %d sequences" % n)
    _check(library().pc_decode_step(ctx.handle, s.ctypes.data, _dev(tokens_in, torch.int32, "tokens_in"), n,
                                    _dev(logits, torch.float32, "logits"), _stream_ptr(stream)))


def pc_decode_step_static(ctx: Context, seq, tokens_in: torch.Tensor, logits: torch.Tensor, stream=None):
    """pc_decode_step without any device allocation: eager launches, scratch in the library's static array."""
    s = seq if (isinstance(seq, np.ndarray) and seq.dtype == np.int32 and seq.flags.c_contiguous and seq.ndim == 1) \
        else _host_i32(seq, "seq")
    n = len(s)
    if n and (tokens_in.numel() < n or logits.numel() < n * ctx.vocab):
        raise ValueError("tokens_in / logits too small for %d sequences" % n)
    _check(library().pc_decode_step_static(ctx.handle, s.ctypes.data, _dev(tokens_in, torch.int32, "tokens_in"), n,
                                           _dev(logits, torch.float32, "logits"), _stream_ptr(stream)))


def pc_score(ctx: Context, tokens: torch.Tensor, cu_lens, prompt_len, temperature: float, logprob_out: torch.Tensor,
             stream=None):
    """log pi(o_t | q, o_<t) of every completion token of the packed sequences (device int32 `tokens`,
    host `cu_lens` [S+1] and `prompt_len` [S]) into `logprob_out` (device fp32, packed)."""
    cu = _host_i32(cu_lens, "cu_lens")
    pl = _host_i32(prompt_len, "prompt_len")
    S = len(cu) - 1
    if len(pl) != S:
        raise ValueError("prompt_len must have one entry per sequence")
    n_out = int((np.diff(cu) - pl).sum()) if S > 0 else 0
    if S > 0 and (tokens.numel() < cu[-1] or logprob_out.numel() < n_out):
        raise ValueError("tokens or logprob_out is too small")
    _check(library().pc_score(ctx.handle, _dev(tokens, torch.int32, "tokens"), cu.ctypes.data, pl.ctypes.data, S,
                              float(temperature), _dev(logprob_out, torch.float32, "logprob_out"),
                              _stream_ptr(stream)))


def pc_release(ctx: Context, ids, kind: int):
    a = _host_i32(ids, "ids")
    _check(library().pc_release(ctx.handle, a.ctypes.data, len(a), int(kind)))


def pc_sample(logits: torch.Tensor, logit_row: Optional[torch.Tensor], n: int, vocab: int, temperature: float,
              seed: int, seq_uid: torch.Tensor, step: Optional[torch.Tensor], step_base: int, eos_id: int,
              eos_logit_bias: float, tokens_out: torch.Tensor, logprob_out: Optional[torch.Tensor] = None,
              finished: Optional[torch.Tensor] = None, stream=None, top_p: float = 1.0,
              hist_tokens: Optional[torch.Tensor] = None, hist_logprob: Optional[torch.Tensor] = None,
              hist_index: Optional[torch.Tensor] = None):
    for t, name in ((seq_uid, "seq_uid"), (tokens_out, "tokens_out"), (logit_row, "logit_row"), (step, "step"),
                    (logprob_out, "logprob_out"), (finished, "finished"), (hist_index, "hist_index")):
        if t is not None and t.numel() < n:
            raise ValueError("%s has fewer than n entries" % name)
    if hist_index is None:
        for t, name in ((hist_tokens, "hist_tokens"), (hist_logprob, "hist_logprob")):
            if t is not None and t.numel() < n:
                raise ValueError("%s has fewer than n entries" % name)
    if logit_row is None and logits.numel() < n * vocab:
        raise ValueError("logits has fewer than n rows")
    _check(library().pc_sample(_dev(logits, torch.float32, "logits"), _dev(logit_row, torch.int32, "logit_row"),
                               int(n), int(vocab), float(temperature), float(top_p), int(seed) & (2 ** 64 - 1),
                               _dev(seq_uid, torch.int64, "seq_uid"), _dev(step, torch.int32, "step"), int(step_base),
                               int(eos_id), float(eos_logit_bias), _dev(tokens_out, torch.int32, "tokens_out"),
                               _dev(logprob_out, torch.float32, "logprob_out"),
                               _dev(finished, torch.uint8, "finished"),
                               _dev(hist_tokens, torch.int32, "hist_tokens"),
                               _dev(hist_logprob, torch.float32, "hist_logprob"),
                               _dev(hist_index, torch.int32, "hist_index"), _stream_ptr(stream)))


def pc_group_stats(rewards: torch.Tensor, group_off: torch.Tensor, n_pos=None, n_tot=None, mean=None, var=None,
                   stream=None):
    P = group_off.numel() - 1
    for t, name in ((n_pos, "n_pos"), (n_tot, "n_tot"), (mean, "mean"), (var, "var")):
        if t is not None and t.numel() < P:
            raise ValueError("%s has fewer than P entries" % name)
    _check(library().pc_group_stats(_dev(rewards, torch.float32, "rewards"), _dev(group_off, torch.int32, "group_off"),
                                    P, _dev(n_pos, torch.int32, "n_pos"), _dev(n_tot, torch.int32, "n_tot"),
                                    _dev(mean, torch.float32, "mean"), _dev(var, torch.float32, "var"),
                                    _stream_ptr(stream)))


def pc_select_commit(p_hat: torch.Tensor, P: int, p_lower: float, p_upper: float, p_solve: float, b_t: int,
                     cls, evict, commit_idx, surplus_idx, counts, stream=None):
    for t, name, need in ((p_hat, "p_hat", P), (cls, "cls", P), (evict, "evict", P), (commit_idx, "commit_idx", P),
                          (surplus_idx, "surplus_idx", P), (counts, "counts", 4)):
        if t is not None and t.numel() < need:
            raise ValueError("%s too small" % name)
    _check(library().pc_select_commit(_dev(p_hat, torch.float32, "p_hat"), int(P), float(p_lower), float(p_upper),
                                      float(p_solve), int(b_t), _dev(cls, torch.uint8, "cls"),
                                      _dev(evict, torch.uint8, "evict"), _dev(commit_idx, torch.int32, "commit_idx"),
                                      _dev(surplus_idx, torch.int32, "surplus_idx"),
                                      _dev(counts, torch.int32, "counts"), _stream_ptr(stream)))


def pc_select_commit_var(mean: torch.Tensor, var: torch.Tensor, P: int, var_hard: float, var_easy: float,
                         mean_pivot: float, mean_solve: float, b_t: int, cls, evict, commit_idx, surplus_idx, counts,
                         stream=None):
    for t, name, need in ((mean, "mean", P), (var, "var", P), (cls, "cls", P), (evict, "evict", P),
                          (commit_idx, "commit_idx", P), (surplus_idx, "surplus_idx", P), (counts, "counts", 4)):
        if t is not None and t.numel() < need:
            raise ValueError("%s too small" % name)
    _check(library().pc_select_commit_var(_dev(mean, torch.float32, "mean"), _dev(var, torch.float32, "var"), int(P),
                                          float(var_hard), float(var_easy), float(mean_pivot), float(mean_solve),
                                          int(b_t), _dev(cls, torch.uint8, "cls"), _dev(evict, torch.uint8, "evict"),
                                          _dev(commit_idx, torch.int32, "commit_idx"),
                                          _dev(surplus_idx, torch.int32, "surplus_idx"),
                                          _dev(counts, torch.int32, "counts"), _stream_ptr(stream)))


def pc_advantages(rewards: torch.Tensor, group_off: torch.Tensor, eps: float, adv: torch.Tensor, mu=None, sigma=None,
                  stream=None):
    P = group_off.numel() - 1
    if adv.numel() < rewards.numel():
        raise ValueError("adv smaller than rewards")
    _check(library().pc_advantages(_dev(rewards, torch.float32, "rewards"), _dev(group_off, torch.int32, "group_off"),
                                   P, float(eps), _dev(adv, torch.float32, "adv"), _dev(mu, torch.float32, "mu"),
                                   _dev(sigma, torch.float32, "sigma"), _stream_ptr(stream)))


class Scheduler:
    """Multi-step scheduling state (pc_sched_*): host arrays in, host arrays out."""

    def __init__(self, p_lower: float, p_upper: float, p_solve: float, b_t: int, max_delay: int):
        cfg = _SchedConfig(float(p_lower), float(p_upper), float(p_solve), int(b_t), int(max_delay))
        h = C.c_void_p()
        _check(library().pc_sched_create(C.byref(cfg), C.byref(h)))
        self.handle = h
        self.b_t = int(b_t)

    def close(self):
        if self.handle is not None:
            library().pc_sched_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def pilot(self, prompt_uid, tag, p_hat):
        """One sampling batch at the current step -> (cls u8 [n], evict u8 [n], counts i32 [4])."""
        uid = np.ascontiguousarray(prompt_uid, dtype=np.int64)
        tg = None if tag is None else np.ascontiguousarray(tag, dtype=np.int64)
        ph = np.ascontiguousarray(p_hat, dtype=np.float32)
        n = len(uid)
        if len(ph) != n or (tg is not None and len(tg) != n):
            raise ValueError("prompt_uid, tag and p_hat must have the same length")
        cls, ev, counts = np.zeros(max(n, 1), np.uint8), np.zeros(max(n, 1), np.uint8), np.zeros(4, np.int32)
        _check(library().pc_sched_pilot(self.handle, uid.ctypes.data, None if tg is None else tg.ctypes.data,
                                        ph.ctypes.data, n, cls.ctypes.data, ev.ctypes.data, counts.ctypes.data))
        return cls[:n], ev[:n], counts

    def commit(self):
        """Commit selection, age-out, t <- t+1 -> ((uid, tag, age), (aged uid, aged tag))."""
        cap = int(self.stats()["buffered_now"])
        kmax = max(1, min(self.b_t, cap))          # never more than the buffer holds
        uid, tg, age = np.zeros(kmax, np.int64), np.zeros(kmax, np.int64), np.zeros(kmax, np.int32)
        auid, atg = np.zeros(max(cap, 1), np.int64), np.zeros(max(cap, 1), np.int64)
        k, a = C.c_int32(0), C.c_int32(0)
        _check(library().pc_sched_commit(self.handle, uid.ctypes.data, tg.ctypes.data, age.ctypes.data,
                                         C.addressof(k), auid.ctypes.data, atg.ctypes.data, cap, C.addressof(a)))
        return (uid[:k.value], tg[:k.value], age[:k.value]), (auid[:a.value], atg[:a.value])

    def evicted(self, prompt_uid) -> np.ndarray:
        uid = np.ascontiguousarray(prompt_uid, dtype=np.int64)
        out = np.zeros(max(len(uid), 1), np.uint8)
        _check(library().pc_sched_evicted(self.handle, uid.ctypes.data, len(uid), out.ctypes.data))
        return out[:len(uid)]

    def stats(self) -> dict:
        out = np.zeros(len(PC_SCHED_STATS), np.int64)
        _check(library().pc_sched_stats(self.handle, out.ctypes.data))
        return dict(zip(PC_SCHED_STATS, out.tolist()))
