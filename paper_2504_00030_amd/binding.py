"""ctypes binding of libspecdecode.so: argument marshalling only.

Every step of the speculative-decoding path runs in the library's HIP kernels;
PyTorch appears only as the owner of device memory (weight tensors) and of the
stream.  Loading fails loudly when the library has not been built
(`python -m paper_2504_00030_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "libspecdecode.so")

SPEC_OK, SPEC_EINVAL, SPEC_ESTATE, SPEC_ENOMEM, SPEC_EHIP, SPEC_ECAP, SPEC_ENOTIMPL = 0, -1, -2, -3, -4, -5, -6
SPEC_F32, SPEC_BF16, SPEC_Q8 = 0, 1, 2
ACCEPT_NATURAL, ACCEPT_FORCED = 0, 1
PATH_AUTO, PATH_WAVEDOT, PATH_MFMA = 0, 1, 2
GT_EXPAND_A, GT_LITERAL, GT_SHORT_TERM = 0, 1, 2

# every symbol include/spec.h and include/gammatune.h declare
EXPORTS = [
    "spec_init", "spec_prefill", "spec_prefill_ragged", "spec_debug_set_step", "spec_draft", "spec_draft_batch", "spec_verify", "spec_accept",
    "spec_set_forced_alpha", "spec_set_early_stop", "spec_generate", "spec_read_tokens", "spec_debug_logits",
    "spec_debug_drafted", "spec_debug_read", "spec_debug_fill_kv", "spec_debug_write_kv", "spec_debug_set_block_table", "spec_device_bytes", "spec_profile_kernel", "spec_profile_read", "spec_profile_read_class", "spec_debug_verify_rows", "spec_destroy",
    "spec_strerror", "spec_last_error", "spec_k_gemv", "spec_k_gemv_tiled", "spec_k_gemm_tiled", "spec_k_retile_q8", "spec_k_gemv_tiled_q8", "spec_k_gemm_tiled_q8", "spec_k_retile", "spec_k_copy", "spec_k_philox", "spec_k_accept", "spec_k_accept_static",
    "gammatune_init", "gammatune_update",
]


class SpecShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "dtype")] + [
        ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


_PP = C.POINTER(C.c_void_p)


class SpecWeights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP), ("w_gate", _PP),
                ("w_up", _PP), ("w_down", _PP), ("attn_norm", _PP), ("ffn_norm", _PP), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p),
                ("wq_scale", _PP), ("wk_scale", _PP), ("wv_scale", _PP), ("wo_scale", _PP), ("w_gate_scale", _PP),
                ("w_up_scale", _PP), ("w_down_scale", _PP), ("lm_head_scale", C.c_void_p)]


class SpecConfig(C.Structure):
    _fields_ = [("batch", C.c_int32), ("max_seq", C.c_int32), ("page_tokens", C.c_int32), ("gamma_max", C.c_int32),
                ("temperature", C.c_float), ("seed", C.c_uint64), ("accept_mode", C.c_int32), ("gemv_path", C.c_int32),
                ("use_graphs", C.c_int32), ("attn_chunk", C.c_int32), ("hip_stream", C.c_void_p)]


class SpecGenStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("steps", "generated", "accepted", "drafted", "gamma_sum", "seq_steps")]


class GtParams(C.Structure):
    _fields_ = [("eta", C.c_double), ("delta", C.c_int32), ("gamma_min", C.c_int32), ("gamma_max", C.c_int32),
                ("reading", C.c_int32)]


class GtState(C.Structure):
    _fields_ = [("gamma_bar", C.c_double), ("gamma", C.c_int32), ("p", GtParams)]


class SpecError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: error {code}" + (f" ({detail})" if detail else ""))


_lib = None


def load() -> C.CDLL:
    """Load the shared library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2504_00030_amd.build`")
    lib = C.CDLL(LIB_PATH)
    i32p, f32p = C.POINTER(C.c_int32), C.POINTER(C.c_float)
    lib.spec_init.argtypes = [C.POINTER(SpecShape), C.POINTER(SpecWeights), C.POINTER(SpecShape), C.POINTER(SpecWeights),
                              C.POINTER(SpecConfig), C.POINTER(C.c_void_p)]
    lib.spec_prefill.argtypes = [C.c_void_p, i32p, C.c_int32]
    lib.spec_prefill_ragged.argtypes = [C.c_void_p, i32p, C.c_int32, i32p]
    lib.spec_debug_set_step.argtypes = [C.c_void_p, C.c_int32, i32p]
    lib.spec_draft.argtypes = [C.c_void_p, C.c_int32]
    lib.spec_draft_batch.argtypes = [C.c_void_p, i32p]
    lib.spec_verify.argtypes = [C.c_void_p, C.c_int32]
    lib.spec_accept.argtypes = [C.c_void_p, i32p, i32p, i32p]
    lib.spec_set_forced_alpha.argtypes = [C.c_void_p, f32p, C.c_int32]
    lib.spec_set_early_stop.argtypes = [C.c_void_p, C.c_float]
    lib.spec_read_tokens.argtypes = [C.c_void_p, C.c_int32, i32p, C.c_int32, i32p]
    lib.spec_debug_logits.argtypes = [C.c_void_p, C.c_int32, f32p, C.c_int64, i32p]
    lib.spec_debug_drafted.argtypes = [C.c_void_p, C.c_int32, i32p, C.c_int32, i32p]
    lib.spec_debug_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64]
    lib.spec_debug_fill_kv.argtypes = [C.c_void_p, C.c_int32, C.c_uint64]
    lib.spec_debug_write_kv.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                        C.c_void_p]
    lib.spec_debug_set_block_table.argtypes = [C.c_void_p, i32p]
    lib.spec_profile_kernel.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.spec_profile_read.argtypes = [C.c_void_p, i32p, C.POINTER(C.c_double)]
    lib.spec_profile_read_class.argtypes = [C.c_void_p, C.c_int32, C.c_int32, i32p, C.POINTER(C.c_double)]
    lib.spec_debug_verify_rows.argtypes = [C.c_void_p, C.c_int32]
    lib.spec_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(SpecGenStats)]
    lib.spec_device_bytes.argtypes = [C.c_void_p]
    lib.spec_device_bytes.restype = C.c_int64
    lib.spec_destroy.argtypes = [C.c_void_p]
    lib.spec_destroy.restype = None
    lib.spec_strerror.argtypes = [C.c_int]
    lib.spec_strerror.restype = C.c_char_p
    lib.spec_last_error.argtypes = [C.c_void_p]
    lib.spec_last_error.restype = C.c_char_p
    lib.spec_k_gemv.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                C.c_void_p]
    lib.spec_k_gemv_tiled.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                      C.c_void_p]
    lib.spec_k_gemm_tiled.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int64, C.c_void_p]
    lib.spec_k_retile_q8.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spec_k_gemv_tiled_q8.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                         C.c_void_p]
    lib.spec_k_gemm_tiled_q8.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                         C.c_void_p, C.c_int64, C.c_void_p]
    lib.spec_k_retile.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spec_k_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.spec_k_philox.argtypes = [C.c_uint64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spec_k_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_uint64,
                                  C.c_int32, C.c_void_p, C.c_void_p]
    lib.spec_k_accept_static.argtypes = lib.spec_k_accept.argtypes
    lib.gammatune_init.argtypes = [C.POINTER(GtState), C.POINTER(GtParams), C.c_int32]
    lib.gammatune_update.argtypes = [C.POINTER(GtState), C.c_int32, C.c_int32]
    lib.gammatune_update.restype = C.c_int32
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().spec_strerror(code).decode()


# ---- controller ---------------------------------------------------------------------------------------
class GammaTune:
    """gammatune_init / gammatune_update on a caller-owned gt_state."""

    def __init__(self, eta=0.25, delta=1, gamma_min=1, gamma_max=8, gamma0=4, reading=GT_EXPAND_A):
        self._lib = load()
        self.state = GtState()
        p = GtParams(eta, delta, gamma_min, gamma_max, reading)
        rc = self._lib.gammatune_init(C.byref(self.state), C.byref(p), gamma0)
        if rc != 0:
            raise SpecError(rc, "gammatune_init")

    @property
    def gamma(self) -> int:
        return int(self.state.gamma)

    @property
    def gamma_bar(self) -> float:
        return float(self.state.gamma_bar)

    def update(self, accepted: int, drafted: Optional[int] = None) -> int:
        d = self.state.gamma if drafted is None else drafted
        g = self._lib.gammatune_update(C.byref(self.state), int(accepted), int(d))
        if g < 0:
            raise SpecError(g, "gammatune_update")
        return int(g)


class FixedGamma:
    def __init__(self, gamma: int):
        self.gamma = int(gamma)

    def update(self, accepted: int, drafted: Optional[int] = None) -> int:
        return self.gamma


# ---- engine -------------------------------------------------------------------------------------------
def _shape_struct(ms) -> SpecShape:
    return SpecShape(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab,
                     {"bf16": SPEC_BF16, "q8": SPEC_Q8}.get(ms.dtype, SPEC_F32), ms.rope_theta, ms.rms_eps)


def _weights_struct(W: Dict, keep: list) -> SpecWeights:
    """W: dict of torch tensors on the GPU (see synth.make_weights). Only data_ptr() is taken."""
    def arr(ts):
        a = (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
        keep.append(a)
        return C.cast(a, _PP)
    for k, v in W.items():
        for t in (v if isinstance(v, list) else [v]):
            if not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"weight {k} must be a contiguous GPU tensor")
    def sc(k):  # scales of 8-bit weights (synth.quantize_weights); absent for the other storage types
        return arr(W[k + "_scale"]) if (k + "_scale") in W else None
    return SpecWeights(W["tok_embed"].data_ptr(), arr(W["wq"]), arr(W["wk"]), arr(W["wv"]), arr(W["wo"]),
                       arr(W["w_gate"]), arr(W["w_up"]), arr(W["w_down"]), arr(W["attn_norm"]), arr(W["ffn_norm"]),
                       W["final_norm"].data_ptr(), W["lm_head"].data_ptr(), sc("wq"), sc("wk"), sc("wv"), sc("wo"), sc("w_gate"),
                       sc("w_up"), sc("w_down"), W["lm_head_scale"].data_ptr() if "lm_head_scale" in W else None)


class SpecEngine:
    """spec_init ... spec_destroy.  Keeps references to the weight tensors so they outlive the context."""

    def __init__(self, target_shape, target_w: Dict, draft_shape, draft_w: Dict, *, batch=1, max_seq=512, gamma_max=8,
                 temperature=0.0, seed=0, accept_mode=ACCEPT_NATURAL, page_tokens=64, gemv_path=PATH_AUTO,
                 use_graphs=False, attn_chunk=0, stream: int = 0):
        self._lib = load()
        self._keep = [target_w, draft_w]
        ts, ds = _shape_struct(target_shape), _shape_struct(draft_shape)
        tw, dw = _weights_struct(target_w, self._keep), _weights_struct(draft_w, self._keep)
        cfg = SpecConfig(batch, max_seq, page_tokens, gamma_max, temperature, seed, accept_mode, gemv_path,
                         1 if use_graphs else 0, attn_chunk, stream)
        self.batch, self.max_seq, self.gamma_max, self.vocab = batch, max_seq, gamma_max, target_shape.vocab
        self._ctx = C.c_void_p()
        rc = self._lib.spec_init(C.byref(ts), C.byref(tw), C.byref(ds), C.byref(dw), C.byref(cfg), C.byref(self._ctx))
        if rc != 0:
            raise SpecError(rc, "spec_init", self._lib.spec_last_error(None).decode())

    def _chk(self, rc: int, where: str):
        if rc != 0:
            raise SpecError(rc, where, self._lib.spec_last_error(self._ctx).decode())

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.spec_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens: np.ndarray):
        t = np.ascontiguousarray(tokens, dtype=np.int32).reshape(self.batch, -1)
        self._chk(self._lib.spec_prefill(self._ctx, t.ctypes.data_as(C.POINTER(C.c_int32)), t.shape[1]), "spec_prefill")

    def prefill_ragged(self, seqs):
        """seqs: list of token lists, one per sequence."""
        lens = np.array([len(t) for t in seqs], dtype=np.int32)
        n_max = int(lens.max())
        t = np.zeros((self.batch, n_max), dtype=np.int32)
        for b, q in enumerate(seqs):
            t[b, : len(q)] = q
        self._chk(self._lib.spec_prefill_ragged(self._ctx, t.ctypes.data_as(C.POINTER(C.c_int32)), n_max,
                                                lens.ctypes.data_as(C.POINTER(C.c_int32))), "spec_prefill_ragged")

    def set_step(self, step: int, prompt_lens):
        p = np.ascontiguousarray(prompt_lens, dtype=np.int32)
        self._chk(self._lib.spec_debug_set_step(self._ctx, int(step), p.ctypes.data_as(C.POINTER(C.c_int32))),
                  "spec_debug_set_step")

    def draft(self, gamma):
        if np.isscalar(gamma):
            self._chk(self._lib.spec_draft(self._ctx, int(gamma)), "spec_draft")
        else:
            g = np.ascontiguousarray(gamma, dtype=np.int32)
            self._chk(self._lib.spec_draft_batch(self._ctx, g.ctypes.data_as(C.POINTER(C.c_int32))), "spec_draft_batch")

    def verify(self, gamma: int):
        self._chk(self._lib.spec_verify(self._ctx, int(gamma)), "spec_verify")

    def accept(self):
        A = np.zeros(self.batch, dtype=np.int32)
        y = np.zeros(self.batch, dtype=np.int32)
        k = np.zeros(self.batch, dtype=np.int32)
        p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
        self._chk(self._lib.spec_accept(self._ctx, p(A), p(y), p(k)), "spec_accept")
        return A, y, k

    def set_forced_alpha(self, alpha: Sequence[float]):
        a = np.ascontiguousarray(alpha, dtype=np.float32)
        self._chk(self._lib.spec_set_forced_alpha(self._ctx, a.ctypes.data_as(C.POINTER(C.c_float)), a.shape[0]),
                  "spec_set_forced_alpha")

    def set_early_stop(self, tau: float):
        self._chk(self._lib.spec_set_early_stop(self._ctx, float(tau)), "spec_set_early_stop")

    def set_block_table(self, table: np.ndarray):
        t = np.ascontiguousarray(table, dtype=np.int32)
        self._chk(self._lib.spec_debug_set_block_table(self._ctx, t.ctypes.data_as(C.POINTER(C.c_int32))),
                  "spec_debug_set_block_table")

    def read_tokens(self, b: int = 0) -> np.ndarray:
        out = np.zeros(self.max_seq, dtype=np.int32)
        n = C.c_int32()
        self._chk(self._lib.spec_read_tokens(self._ctx, b, out.ctypes.data_as(C.POINTER(C.c_int32)), self.max_seq,
                                             C.byref(n)), "spec_read_tokens")
        return out[: n.value].copy()

    def debug_logits(self, which: int) -> np.ndarray:
        cap = self.batch * (self.gamma_max + 1) * self.vocab
        out = np.empty(cap, dtype=np.float32)
        rows = C.c_int32()
        self._chk(self._lib.spec_debug_logits(self._ctx, which, out.ctypes.data_as(C.POINTER(C.c_float)), cap,
                                              C.byref(rows)), "spec_debug_logits")
        return out[: self.batch * rows.value * self.vocab].reshape(self.batch, rows.value, self.vocab).copy()

    def debug_drafted(self, b: int = 0) -> list:
        out = np.zeros(self.gamma_max, dtype=np.int32)
        n = C.c_int32()
        self._chk(self._lib.spec_debug_drafted(self._ctx, b, out.ctypes.data_as(C.POINTER(C.c_int32)), self.gamma_max,
                                               C.byref(n)), "spec_debug_drafted")
        return out[: n.value].tolist()

    def debug_read(self, model: int, which: int, n: int, dtype=np.float32) -> np.ndarray:
        out = np.zeros(n, dtype=dtype)
        self._chk(self._lib.spec_debug_read(self._ctx, model, which, out.ctypes.data_as(C.c_void_p), out.nbytes),
                  "spec_debug_read")
        return out

    def fill_kv(self, length: int, seed: int = 0):
        self._chk(self._lib.spec_debug_fill_kv(self._ctx, int(length), int(seed)), "spec_debug_fill_kv")

    def write_kv(self, model: int, layer: int, seq: int, pos0: int, k, v):
        """k, v: numpy float32 [n][n_kv_heads][head_dim]."""
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        self._chk(self._lib.spec_debug_write_kv(self._ctx, model, layer, seq, pos0, k.shape[0], k.ctypes.data, v.ctypes.data),
                  "spec_debug_write_kv")

    def profile_kernel(self, model: int, kind: int):
        self._chk(self._lib.spec_profile_kernel(self._ctx, model, kind), "spec_profile_kernel")

    def profile_read(self):
        n = C.c_int32()
        ms = C.c_double()
        self._chk(self._lib.spec_profile_read(self._ctx, C.byref(n), C.byref(ms)), "spec_profile_read")
        return n.value, ms.value

    def profile_read_class(self, model: int, kind: int):
        n = C.c_int32()
        ms = C.c_double()
        self._chk(self._lib.spec_profile_read_class(self._ctx, model, kind, C.byref(n), C.byref(ms)), "spec_profile_read_class")
        return n.value, ms.value

    def verify_rows(self, rows: int):
        self._chk(self._lib.spec_debug_verify_rows(self._ctx, int(rows)), "spec_debug_verify_rows")

    def device_bytes(self) -> int:
        return int(self._lib.spec_device_bytes(self._ctx))

    def run(self, n_generate: int, controllers: List) -> dict:
        """spec_generate: the decode loop in native code (after prefill).  controllers: one GammaTune per sequence
        (their states are updated), or FixedGamma objects of one common gamma."""
        st = SpecGenStats()
        if all(isinstance(c, GammaTune) for c in controllers):
            arr = (GtState * self.batch)(*[c.state for c in controllers])
            rc = self._lib.spec_generate(self._ctx, arr, 0, int(n_generate), C.byref(st))
            for c, s_ in zip(controllers, arr):
                c.state.gamma_bar, c.state.gamma = s_.gamma_bar, s_.gamma
        else:
            rc = self._lib.spec_generate(self._ctx, None, int(controllers[0].gamma), int(n_generate), C.byref(st))
        self._chk(rc, "spec_generate")
        return dict(generated=int(st.generated), spec_steps=int(st.steps), accepted=int(st.accepted), drafted=int(st.drafted),
                    gamma_sum=int(st.gamma_sum), seq_steps=int(st.seq_steps))

    def generate(self, prompts: np.ndarray, n_generate: int, controllers: List, keep_logits: bool = False):
        """Host loop of speculative decoding: draft -> verify -> accept -> controller update, until every
        sequence holds n_generate new tokens; like spec_generate, a sequence that has them rides along with
        gamma = 1 and its controller is left alone (trace["live"] marks the sequences still counted).
        Returns (tokens [B][n_prompt + n_generate], trace)."""
        prompts = np.asarray(prompts, dtype=np.int32).reshape(self.batch, -1)
        n0 = prompts.shape[1]
        self.prefill(prompts)
        gen = np.zeros(self.batch, dtype=np.int64)
        trace = []
        while gen.min() < n_generate:
            live = gen < n_generate
            gammas = np.array([c.gamma if live[b] else 1 for b, c in enumerate(controllers)], dtype=np.int32)
            self.draft(gammas if self.batch > 1 else int(gammas[0]))
            gmax = int(gammas.max())
            self.verify(gmax)
            rec = {"gamma": gammas.copy(), "live": live.copy()}
            if keep_logits:
                rec["q_logits"] = self.debug_logits(0)
            A, y, k = self.accept()
            if keep_logits:
                rec["p_logits"] = self.debug_logits(1)
            rec.update(A=A.copy(), y=y.copy(), k=k.copy())
            trace.append(rec)
            for b, c in enumerate(controllers):
                if live[b]:
                    c.update(int(A[b]), int(k[b]))
            gen += A + 1
        toks = np.stack([self.read_tokens(b)[: n0 + n_generate] for b in range(self.batch)])
        return toks, trace


# ---- single kernels -----------------------------------------------------------------------------------
def k_gemv(w, x, y, path=PATH_WAVEDOT, stream: int = 0, N=None, K=None):
    """y[R][N] = x[R][K] . W[N][K]^T on GPU tensors (w: fp32 or bf16, x/y fp32)."""
    import torch
    dtype = SPEC_BF16 if w.dtype == torch.bfloat16 else SPEC_F32
    N = w.shape[0] if N is None else N
    K = w.shape[1] if K is None else K
    rc = load().spec_k_gemv(w.data_ptr(), dtype, N, K, x.data_ptr(), x.shape[0], y.data_ptr(), path, stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_gemv")


def k_gemv_tiled(w_tiled, N, K, x_bf16, y, cfg: int = 0, stream: int = 0, x_lo=None):
    """x_bf16: [R][K] bf16, or [2][R][K] with x_lo = x_bf16[1] (both terms in one allocation)."""
    rc = load().spec_k_gemv_tiled(w_tiled.data_ptr(), N, K, x_bf16.data_ptr(), None if x_lo is None else x_lo.data_ptr(),
                                  y.shape[0], y.data_ptr(), cfg, stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_gemv_tiled")


def k_gemm_tiled(w_tiled, N, K, x, y, cfg: int = 0, stream: int = 0, workspace=None):
    """x: fp32 [R][K]; y: fp32 [R][N]; the dense-contraction kernel with the plain epilogue.  workspace: a device
    tensor for the partial results when K is shared out over workgroups (cfg = 1000 * shares + shape)."""
    ws = None if workspace is None else workspace.data_ptr()
    nb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spec_k_gemm_tiled(w_tiled.data_ptr(), N, K, x.data_ptr(), y.shape[0], y.data_ptr(), cfg, ws, nb, stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_gemm_tiled")


def k_retile_q8(w_q8, out, stream: int = 0):
    rc = load().spec_k_retile_q8(w_q8.data_ptr(), w_q8.shape[0], w_q8.shape[1], out.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_retile_q8")


def k_gemv_tiled_q8(w_tiled, w_scale, N, K, x_bf16, y, stream: int = 0, x_lo=None):
    rc = load().spec_k_gemv_tiled_q8(w_tiled.data_ptr(), w_scale.data_ptr(), N, K, x_bf16.data_ptr(),
                                     None if x_lo is None else x_lo.data_ptr(), y.shape[0], y.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_gemv_tiled_q8")


def k_gemm_tiled_q8(w_tiled, w_scale, N, K, x, y, cfg: int = 0, stream: int = 0, workspace=None):
    ws = None if workspace is None else workspace.data_ptr()
    nb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().spec_k_gemm_tiled_q8(w_tiled.data_ptr(), w_scale.data_ptr(), N, K, x.data_ptr(), y.shape[0], y.data_ptr(), cfg,
                                     ws, nb, stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_gemm_tiled_q8")


def k_retile(w, out, stream: int = 0):
    rc = load().spec_k_retile(w.data_ptr(), w.shape[0], w.shape[1], out.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_retile")


def k_copy(dst, src, stream: int = 0):
    rc = load().spec_k_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_copy")


def k_philox(seed: int, ctr, out, stream: int = 0):
    rc = load().spec_k_philox(seed, ctr.data_ptr(), ctr.shape[0], out.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_philox")


def k_accept(p_logits, q_logits, drafted, temperature: float, seed: int, step: int, result, stream: int = 0):
    k = q_logits.shape[0]
    rc = load().spec_k_accept(p_logits.data_ptr(), q_logits.data_ptr(), drafted.data_ptr(), k, p_logits.shape[1],
                              temperature, seed, step, result.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_accept")


def k_accept_static(p_logits, q_logits, drafted, temperature: float, seed: int, step: int, result, stream: int = 0):
    """spec_k_accept_static: as k_accept, scratch in the library's fixed device array, asynchronous on `stream`."""
    k = q_logits.shape[0]
    rc = load().spec_k_accept_static(p_logits.data_ptr(), q_logits.data_ptr(), drafted.data_ptr(), k, p_logits.shape[1],
                                     temperature, seed, step, result.data_ptr(), stream)
    if rc != 0:
        raise SpecError(rc, "spec_k_accept_static", load().spec_last_error(None).decode())
