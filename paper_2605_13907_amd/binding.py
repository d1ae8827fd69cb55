"""ctypes binding of the C ABI in include/ais.h.

Argument marshalling only: tensors are checked (device, dtype, contiguity), their
device pointers and the current HIP stream are handed to the library, and outputs
are allocated with torch.  Every step of the path runs in the library's kernels;
there is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libais_gfx950.so")

AIS_BF16, AIS_F32 = 0, 1
AIS_K_LOGPROB, AIS_K_DLOGITS, AIS_K_COPY, AIS_K_FP8_QUANT, AIS_K_FP8_DEQUANT, AIS_K_FP8_LOGPROB = range(6)
AIS_K_FUSED = 6
AIS_K_LM_HEAD = 7
AIS_K_LM_HEAD_GRAD = 8
AIS_STATUS_LIVE_OVERFLOW = 4
STATUS_BAD_TOKEN, STATUS_BAD_CU = 1, 2

ERRORS = {
    0: "AIS_OK", -1: "AIS_ERR_NULL", -2: "AIS_ERR_SIZE", -3: "AIS_ERR_STRIDE", -4: "AIS_ERR_ALIGN",
    -5: "AIS_ERR_PARAM", -6: "AIS_ERR_GROUP", -7: "AIS_ERR_DTYPE", -8: "AIS_ERR_HIP", -9: "AIS_ERR_NOMEM",
    -10: "AIS_ERR_SCRATCH",
}
STATIC_SCRATCH_BYTES = 1 << 20


class AisParams(C.Structure):
    _fields_ = [("C", C.c_float), ("delta", C.c_float), ("gamma", C.c_float), ("eps_std", C.c_float),
                ("beta_var", C.c_float), ("clip_eps", C.c_float), ("adv_mode", C.c_int),
                ("alpha_override", C.c_float), ("inv_temperature", C.c_float), ("beta_kl", C.c_float)]


class AisDiag(C.Structure):
    _fields_ = [("n_valid", C.c_longlong), ("mean_w", C.c_double), ("var_w", C.c_double), ("cv2", C.c_double),
                ("ess_ratio", C.c_double), ("dbar", C.c_double), ("std_a", C.c_double), ("std_aw", C.c_double),
                ("dsigma", C.c_double), ("alpha_ess", C.c_double), ("alpha_mis", C.c_double),
                ("alpha_var", C.c_double), ("alpha", C.c_double), ("clip_frac", C.c_double),
                ("kl_roll_train", C.c_double), ("mean_abs_dp", C.c_double), ("status", C.c_int), ("reserved", C.c_int)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_ if name != "reserved"}


class AisError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib().ais_strerror(code).decode() if _LIB is not None else ""
        super().__init__(f"{where}: {ERRORS.get(code, code)} ({msg})")


_LIB = None

# every symbol include/ais.h declares: (name, restype, argtypes)
_P, _LL, _I, _F = C.c_void_p, C.c_longlong, C.c_int, C.c_float
SYMBOLS = {
    "ais_create": (_I, [C.POINTER(_P), _I, _P]),
    "ais_destroy": (_I, [_P]),
    "ais_set_stream": (_I, [_P, _P]),
    "ais_params_default": (None, [C.POINTER(AisParams)]),
    "ais_strerror": (C.c_char_p, [_I]),
    "ais_last_hip_error": (_I, [_P]),
    "ais_status": (_I, [_P, C.POINTER(_I), _I]),
    "ais_version": (_I, []),
    "ais_token_logprob": (_I, [_P, _P, _I, _LL, _LL, _LL, _P, _P, _F, _P, _P]),
    "ais_diagnostics": (_I, [_P, _P, _P, _P, _LL, _P, _I, _I, _P, C.POINTER(AisParams), _P, _P, _P]),
    "ais_diagnostics_static": (_I, [_P, _P, _P, _P, _LL, _P, _I, _I, _P, C.POINTER(AisParams), _P, _P, _P]),
    "ais_grpo_loss_grad": (_I, [_P, _P, _I, _LL, _LL, _LL, _P, _P, _P, _I, _P, _P, _P, _P, _P, _P, _P, _P,
                                C.POINTER(AisParams), _P, _P, _P]),
    "ais_token_logprob_softmax_grad": (_I, [_P, _P, _I, _LL, _LL, _LL, _P, _P, _F, _P, _P, _P]),
    "ais_grpo_row_scale": (_I, [_P, _P, _P, _P, _P, _P, _LL, _P, _I, _P, _P, _P, C.POINTER(AisParams), _P, _P, _P]),
    "ais_fp8_quantize_rows": (_I, [_P, _P, _I, _LL, _LL, _LL, _P, _LL, _P]),
    "ais_fp8_dequantize_rows": (_I, [_P, _P, _LL, _P, _LL, _LL, _P, _I, _LL]),
    "ais_fp8_rollout_logprob": (_I, [_P, _P, _I, _LL, _LL, _LL, _P, _P, _P]),
    "ais_lm_head_logprob": (_I, [_P, _P, _LL, _P, _LL, _I, _LL, _LL, _LL, _P, _P, _F, _P, _P]),
    "ais_lm_head_grad": (_I, [_P, _P, _LL, _P, _LL, _I, _LL, _LL, _LL, _P, _P, _P, _P, _F, _LL, _LL, _P, _P]),
    "ais_profile": (_I, [_P, _I]),
    "ais_profile_read": (_I, [_P, _I, C.POINTER(_F), C.POINTER(_I)]),
    "ais_copy": (_I, [_P, _P, _P, _LL]),
}


def _lib():
    """The loaded library.  Raises if it has not been built: there is no other implementation to fall back on."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_13907_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def default_params(**overrides) -> AisParams:
    p = AisParams()
    _lib().ais_params_default(C.byref(p))
    for k, v in overrides.items():
        if not hasattr(p, k):
            raise AttributeError(k)
        setattr(p, k, v)
    return p


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return AIS_BF16
    if t.dtype == torch.float32:
        return AIS_F32
    raise TypeError(f"logits must be bfloat16 or float32, not {t.dtype}")


def _ptr(t: Optional[torch.Tensor], dtype=None, numel=None, name="tensor", device=None):
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if device is not None and t.device != device:
        raise ValueError(f"{name} is on {t.device}, expected {device}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name}: expected {numel} elements, got {t.numel()}")
    return C.c_void_p(t.data_ptr())


def _dev_ptr(t: torch.Tensor, device: torch.device, name: str):
    """Device pointer of a buffer whose layout the caller has already checked: it must live on the context's GPU
    (a host or foreign pointer handed to a kernel is a GPU memory fault, not an error code)."""
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch.Tensor")
    if not t.is_cuda or t.device != device:
        raise ValueError(f"{name} is on {t.device}, expected {device}")
    return C.c_void_p(t.data_ptr())


def _logits_geometry(logits: torch.Tensor, device: Optional[torch.device] = None, name: str = "logits"):
    if not isinstance(logits, torch.Tensor):
        raise TypeError(f"{name} must be a torch.Tensor")
    if logits.dim() != 2 or logits.stride(1) != 1 and logits.shape[1] > 1:
        raise ValueError(f"{name} must be [n_rows, vocab] with unit stride along the vocabulary")
    if device is not None and (not logits.is_cuda or logits.device != device):
        raise ValueError(f"{name} is on {logits.device}, expected {device}")
    n_rows, vocab = logits.shape
    row_stride = logits.stride(0) if n_rows > 1 else max(vocab, logits.stride(0))
    return n_rows, vocab, row_stride


class AisContext:
    """One library context bound to a GPU; launches on torch's current stream of that GPU."""

    def __init__(self, device: Optional[torch.device] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("AisContext needs a GPU")
        self.device = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
        if self.device.index is None:
            self.device = torch.device("cuda", torch.cuda.current_device())
        self._lib = _lib()
        h = C.c_void_p()
        rc = self._lib.ais_create(C.byref(h), self.device.index, self._stream())
        if rc != 0:
            raise AisError(rc, "ais_create")
        self._h = h

    def _stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def _sync_stream(self):
        rc = self._lib.ais_set_stream(self._h, self._stream())
        if rc != 0:
            raise AisError(rc, "ais_set_stream")

    def close(self):
        if getattr(self, "_h", None) is not None:
            self._lib.ais_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ the three calls
    def token_logprob(self, logits, token_ids, valid=None, inv_temperature: float = 1.0):
        """-> (logp [R] fp32, lse [R] fp32).  See ais_token_logprob in include/ais.h."""
        dev = self.device
        n_rows, vocab, row_stride = _logits_geometry(logits, dev)
        logp = torch.empty(n_rows, dtype=torch.float32, device=dev)
        lse = torch.empty(n_rows, dtype=torch.float32, device=dev)
        self._sync_stream()
        rc = self._lib.ais_token_logprob(
            self._h, C.c_void_p(logits.data_ptr()), _dtype_code(logits), n_rows, vocab, row_stride,
            _ptr(token_ids, torch.int32, n_rows, "token_ids", dev), _ptr(valid, torch.uint8, n_rows, "valid", dev),
            float(inv_temperature), _ptr(logp), _ptr(lse))
        if rc != 0:
            raise AisError(rc, "ais_token_logprob")
        return logp, lse

    def diagnostics(self, logp_train, logp_roll, valid, cu_rows, rewards, group_size: int,
                    params: Optional[AisParams] = None, static_scratch: bool = False, out=None):
        """-> (adv [B] fp32, count [B] int32, diag: uint8 tensor holding one ais_diag on the device).
        static_scratch: call ais_diagnostics_static (no device allocation inside the library); out: the three
        output tensors to write into instead of new ones (so that the binding allocates nothing either)."""
        p = params or default_params()
        dev = self.device
        n_rows = logp_train.numel()
        n_resp = rewards.numel()
        if out is None:
            adv = torch.empty(n_resp, dtype=torch.float32, device=dev)
            count = torch.empty(n_resp, dtype=torch.int32, device=dev)
            diag = torch.zeros(C.sizeof(AisDiag), dtype=torch.uint8, device=dev)
        else:
            adv, count, diag = out
            _ptr(adv, torch.float32, n_resp, "adv", dev), _ptr(count, torch.int32, n_resp, "count", dev)
            _ptr(diag, torch.uint8, C.sizeof(AisDiag), "diag", dev)
        self._sync_stream()
        fn = self._lib.ais_diagnostics_static if static_scratch else self._lib.ais_diagnostics
        rc = fn(
            self._h, _ptr(logp_train, torch.float32, n_rows, "logp_train", dev),
            _ptr(logp_roll, torch.float32, n_rows, "logp_roll", dev), _ptr(valid, torch.uint8, n_rows, "valid", dev),
            n_rows, _ptr(cu_rows, torch.int64, n_resp + 1, "cu_rows", dev), n_resp, int(group_size),
            _ptr(rewards, torch.float32, n_resp, "rewards", dev), C.byref(p), _ptr(adv), _ptr(count), _ptr(diag))
        if rc != 0:
            raise AisError(rc, "ais_diagnostics_static" if static_scratch else "ais_diagnostics")
        return adv, count, diag

    def grpo_loss_grad(self, logits, token_ids, valid, cu_rows, logp_train, lse, logp_roll, adv, count, diag,
                       params: Optional[AisParams] = None, logp_old=None, logp_ref=None, dlogits=None,
                       want_wtilde: bool = True):
        """-> (loss: fp64 tensor [1] on the device, wtilde [R] fp32 or None, dlogits like logits).
        Pass dlogits=logits to overwrite the logits in place."""
        p = params or default_params()
        dev = self.device
        n_rows, vocab, row_stride = _logits_geometry(logits, dev)
        n_resp = adv.numel()
        if dlogits is None:
            dlogits = torch.empty_strided(logits.shape, logits.stride(), dtype=logits.dtype, device=dev)
        elif dlogits.dtype != logits.dtype or dlogits.shape != logits.shape or dlogits.stride() != logits.stride():
            raise ValueError("dlogits must have the dtype, shape and strides of logits")
        _dev_ptr(dlogits, dev, "dlogits")
        wtilde = torch.empty(n_rows, dtype=torch.float32, device=dev) if want_wtilde else None
        loss = torch.empty(1, dtype=torch.float64, device=dev)
        self._sync_stream()
        rc = self._lib.ais_grpo_loss_grad(
            self._h, C.c_void_p(logits.data_ptr()), _dtype_code(logits), n_rows, vocab, row_stride,
            _ptr(token_ids, torch.int32, n_rows, "token_ids", dev), _ptr(valid, torch.uint8, n_rows, "valid", dev),
            _ptr(cu_rows, torch.int64, n_resp + 1, "cu_rows", dev), n_resp,
            _ptr(logp_train, torch.float32, n_rows, "logp_train", dev), _ptr(lse, torch.float32, n_rows, "lse", dev),
            _ptr(logp_roll, torch.float32, n_rows, "logp_roll", dev),
            _ptr(logp_old, torch.float32, n_rows, "logp_old", dev),
            _ptr(logp_ref, torch.float32, n_rows, "logp_ref", dev),
            _ptr(adv, torch.float32, n_resp, "adv", dev), _ptr(count, torch.int32, n_resp, "count", dev),
            _ptr(diag, torch.uint8, C.sizeof(AisDiag), "diag", dev), C.byref(p), _ptr(wtilde), _ptr(loss),
            C.c_void_p(dlogits.data_ptr()))
        if rc != 0:
            raise AisError(rc, "ais_grpo_loss_grad")
        return loss, wtilde, dlogits

    def step(self, batch, params: Optional[AisParams] = None, logp_old=None, logp_ref=None, in_place=False):
        """The whole path on one workloads.RolloutBatch: the three calls back to back on one stream."""
        p = params or default_params()
        logp, lse = self.token_logprob(batch.logits, batch.token_ids, batch.valid, p.inv_temperature)
        # Alg. 1 estimates the coefficient from log pi_train at the checkpoint that generated the rollout
        adv, count, diag = self.diagnostics(logp if logp_old is None else logp_old, batch.logp_roll, batch.valid,
                                            batch.cu_rows, batch.rewards, batch.shape.group_size, p)
        loss, wtilde, dz = self.grpo_loss_grad(batch.logits, batch.token_ids, batch.valid, batch.cu_rows, logp, lse,
                                               batch.logp_roll, adv, count, diag, p, logp_old, logp_ref,
                                               dlogits=batch.logits if in_place else None)
        return dict(logp=logp, lse=lse, adv=adv, count=count, diag=diag, loss=loss, wtilde=wtilde, dlogits=dz)

    # ------------------------------------------------------------------ one-sweep variant
    def token_logprob_softmax_grad(self, logits, token_ids, valid=None, inv_temperature: float = 1.0, sgrad=None):
        """-> (logp, lse, sgrad) with sgrad[n, v] = softmax_v - 1[v = y_n]; pass sgrad=logits for in place."""
        dev = self.device
        n_rows, vocab, row_stride = _logits_geometry(logits, dev)
        logp = torch.empty(n_rows, dtype=torch.float32, device=dev)
        lse = torch.empty(n_rows, dtype=torch.float32, device=dev)
        if sgrad is None:
            sgrad = torch.empty_strided(logits.shape, logits.stride(), dtype=logits.dtype, device=dev)
        elif sgrad.dtype != logits.dtype or sgrad.shape != logits.shape or sgrad.stride() != logits.stride():
            raise ValueError("sgrad must have the dtype, shape and strides of logits")
        _dev_ptr(sgrad, dev, "sgrad")
        self._sync_stream()
        rc = self._lib.ais_token_logprob_softmax_grad(
            self._h, C.c_void_p(logits.data_ptr()), _dtype_code(logits), n_rows, vocab, row_stride,
            _ptr(token_ids, torch.int32, n_rows, "token_ids", dev), _ptr(valid, torch.uint8, n_rows, "valid", dev),
            float(inv_temperature), _ptr(logp), _ptr(lse), C.c_void_p(sgrad.data_ptr()))
        if rc != 0:
            raise AisError(rc, "ais_token_logprob_softmax_grad")
        return logp, lse, sgrad

    def grpo_row_scale(self, logp_train, logp_roll, valid, cu_rows, adv, count, diag,
                       params: Optional[AisParams] = None, logp_old=None, logp_ref=None):
        """-> (loss [1] fp64, wtilde [R], g [R]) with dlogits[n, :] = g[n] * sgrad[n, :]."""
        p = params or default_params()
        dev = self.device
        n_rows, n_resp = logp_train.numel(), adv.numel()
        wtilde = torch.empty(n_rows, dtype=torch.float32, device=dev)
        g = torch.empty(n_rows, dtype=torch.float32, device=dev)
        loss = torch.empty(1, dtype=torch.float64, device=dev)
        self._sync_stream()
        rc = self._lib.ais_grpo_row_scale(
            self._h, _ptr(logp_train, torch.float32, n_rows, "logp_train", dev),
            _ptr(logp_roll, torch.float32, n_rows, "logp_roll", dev),
            _ptr(logp_old, torch.float32, n_rows, "logp_old", dev),
            _ptr(logp_ref, torch.float32, n_rows, "logp_ref", dev), _ptr(valid, torch.uint8, n_rows, "valid", dev),
            n_rows, _ptr(cu_rows, torch.int64, n_resp + 1, "cu_rows", dev), n_resp,
            _ptr(adv, torch.float32, n_resp, "adv", dev), _ptr(count, torch.int32, n_resp, "count", dev),
            _ptr(diag, torch.uint8, C.sizeof(AisDiag), "diag", dev), C.byref(p), _ptr(wtilde), _ptr(loss), _ptr(g))
        if rc != 0:
            raise AisError(rc, "ais_grpo_row_scale")
        return loss, wtilde, g

    def step_one_sweep(self, batch, params: Optional[AisParams] = None, logp_old=None, logp_ref=None, in_place=False):
        """The path with each logits row read once: direction s and per-row scale g instead of dlogits."""
        p = params or default_params()
        logp, lse, s = self.token_logprob_softmax_grad(batch.logits, batch.token_ids, batch.valid, p.inv_temperature,
                                                       sgrad=batch.logits if in_place else None)
        adv, count, diag = self.diagnostics(logp if logp_old is None else logp_old, batch.logp_roll, batch.valid,
                                            batch.cu_rows, batch.rewards, batch.shape.group_size, p)
        loss, wtilde, g = self.grpo_row_scale(logp, batch.logp_roll, batch.valid, batch.cu_rows, adv, count, diag, p,
                                              logp_old, logp_ref)
        return dict(logp=logp, lse=lse, adv=adv, count=count, diag=diag, loss=loss, wtilde=wtilde, sgrad=s, g=g)

    # ------------------------------------------------------------------ FP8 rollout perturbation
    def fp8_quantize_rows(self, logits):
        """-> (codes [R, V] uint8, scale [R] fp32).  See ais_fp8_quantize_rows in include/ais.h."""
        n_rows, vocab, row_stride = _logits_geometry(logits, self.device)
        codes = torch.empty((n_rows, vocab), dtype=torch.uint8, device=self.device)
        scale = torch.empty(n_rows, dtype=torch.float32, device=self.device)
        self._sync_stream()
        rc = self._lib.ais_fp8_quantize_rows(self._h, C.c_void_p(logits.data_ptr()), _dtype_code(logits), n_rows,
                                             vocab, row_stride, _ptr(codes), vocab, _ptr(scale))
        if rc != 0:
            raise AisError(rc, "ais_fp8_quantize_rows")
        return codes, scale

    def fp8_dequantize_rows(self, codes, scale, dtype=torch.float32):
        """-> z_r [R, V] of `dtype` (float32 or bfloat16)."""
        if codes.dim() != 2 or codes.stride(1) != 1 and codes.shape[1] > 1:
            raise ValueError("codes must be [n_rows, vocab] with unit stride along the vocabulary")
        if codes.dtype != torch.uint8:
            raise TypeError(f"codes: expected torch.uint8, got {codes.dtype}")
        codes_ptr = _dev_ptr(codes, self.device, "codes")
        n_rows, vocab = codes.shape
        out = torch.empty((n_rows, vocab), dtype=dtype, device=self.device)
        self._sync_stream()
        rc = self._lib.ais_fp8_dequantize_rows(self._h, codes_ptr,
                                               codes.stride(0) if n_rows > 1 else vocab,
                                               _ptr(scale, torch.float32, n_rows, "scale", self.device), n_rows,
                                               vocab, _ptr(out), _dtype_code(out), vocab)
        if rc != 0:
            raise AisError(rc, "ais_fp8_dequantize_rows")
        return out

    def fp8_rollout_logprob(self, logits, token_ids, valid=None):
        """-> logp_roll [R] fp32: log-softmax of the FP8 round trip of each row at the sampled token."""
        n_rows, vocab, row_stride = _logits_geometry(logits, self.device)
        out = torch.empty(n_rows, dtype=torch.float32, device=self.device)
        self._sync_stream()
        rc = self._lib.ais_fp8_rollout_logprob(
            self._h, C.c_void_p(logits.data_ptr()), _dtype_code(logits), n_rows, vocab, row_stride,
            _ptr(token_ids, torch.int32, n_rows, "token_ids", self.device),
            _ptr(valid, torch.uint8, n_rows, "valid", self.device), _ptr(out))
        if rc != 0:
            raise AisError(rc, "ais_fp8_rollout_logprob")
        return out

    # ------------------------------------------------------------------ log-probs without materialised logits
    def lm_head_logprob(self, hidden, weight, token_ids, valid=None, inv_temperature: float = 1.0):
        """-> (logp [R] fp32, lse [R] fp32) from hidden [R, D] and weight [V, D], both bf16."""
        for name, t in (("hidden", hidden), ("weight", weight)):
            if t.dim() != 2 or t.stride(1) != 1:
                raise ValueError(f"{name} must be 2-D with unit stride along d_model")
            if t.dtype != torch.bfloat16:
                raise ValueError(f"{name} must be bfloat16")
            _dev_ptr(t, self.device, name)
        n_rows, d_model = hidden.shape
        vocab = weight.shape[0]
        if weight.shape[1] != d_model:
            raise ValueError("hidden and weight disagree on d_model")
        dev = self.device
        logp = torch.empty(n_rows, dtype=torch.float32, device=dev)
        lse = torch.empty(n_rows, dtype=torch.float32, device=dev)
        self._sync_stream()
        rc = self._lib.ais_lm_head_logprob(
            self._h, C.c_void_p(hidden.data_ptr()), hidden.stride(0) if n_rows > 1 else max(d_model, hidden.stride(0)),
            C.c_void_p(weight.data_ptr()), weight.stride(0) if vocab > 1 else max(d_model, weight.stride(0)),
            AIS_BF16, n_rows, d_model, vocab, _ptr(token_ids, torch.int32, n_rows, "token_ids", dev),
            _ptr(valid, torch.uint8, n_rows, "valid", dev), float(inv_temperature), _ptr(logp), _ptr(lse))
        if rc != 0:
            raise AisError(rc, "ais_lm_head_logprob")
        return logp, lse

    def lm_head_grad(self, hidden, weight, token_ids, lse, logp, coeff, inv_temperature: float = 1.0,
                     chunk_vocab: int = 0, n_live_max: int = -1):
        """-> (dhidden [R, D] fp32, dweight [V, D] fp32): gradient of the loss w.r.t. the read-out's operands from the
        per-row coefficient (the g of grpo_row_scale) and the lse / logp of lm_head_logprob; the [R, V] logits and
        their gradient never exist as a whole.  n_live_max: a bound the caller vouches for on the number of rows with a
        non-zero coefficient (-1: none): the work then follows that number.  See ais_lm_head_grad in include/ais.h."""
        for name, t in (("hidden", hidden), ("weight", weight)):
            if t.dim() != 2 or t.stride(1) != 1:
                raise ValueError(f"{name} must be 2-D with unit stride along d_model")
            if t.dtype != torch.bfloat16:
                raise ValueError(f"{name} must be bfloat16")
            _dev_ptr(t, self.device, name)
        n_rows, d_model = hidden.shape
        vocab = weight.shape[0]
        if weight.shape[1] != d_model:
            raise ValueError("hidden and weight disagree on d_model")
        dev = self.device
        ptrs = [_ptr(token_ids, torch.int32, n_rows, "token_ids", dev), _ptr(lse, torch.float32, n_rows, "lse", dev),
                _ptr(logp, torch.float32, n_rows, "logp", dev), _ptr(coeff, torch.float32, n_rows, "coeff", dev)]
        dhidden = torch.empty((n_rows, d_model), dtype=torch.float32, device=dev)
        dweight = torch.empty((vocab, d_model), dtype=torch.float32, device=dev)
        self._sync_stream()
        rc = self._lib.ais_lm_head_grad(
            self._h, C.c_void_p(hidden.data_ptr()), hidden.stride(0) if n_rows > 1 else max(d_model, hidden.stride(0)),
            C.c_void_p(weight.data_ptr()), weight.stride(0) if vocab > 1 else max(d_model, weight.stride(0)),
            AIS_BF16, n_rows, d_model, vocab, *ptrs, float(inv_temperature), int(chunk_vocab), int(n_live_max),
            _ptr(dhidden), _ptr(dweight))
        if rc != 0:
            raise AisError(rc, "ais_lm_head_grad")
        return dhidden, dweight

    # ------------------------------------------------------------------ helpers
    def read_diag(self, diag: torch.Tensor) -> dict:
        """Copies the device ais_diag to the host (synchronises)."""
        raw = bytes(diag.cpu().numpy().tobytes())
        return AisDiag.from_buffer_copy(raw).as_dict()

    def status(self, clear: bool = True) -> int:
        out = C.c_int(0)
        rc = self._lib.ais_status(self._h, C.byref(out), 1 if clear else 0)
        if rc != 0:
            raise AisError(rc, "ais_status")
        return out.value

    def profile(self, enable: bool):
        self._sync_stream()
        rc = self._lib.ais_profile(self._h, 1 if enable else 0)
        if rc != 0:
            raise AisError(rc, "ais_profile")

    def profile_read(self, which: int):
        ms, n = C.c_float(0), C.c_int(0)
        rc = self._lib.ais_profile_read(self._h, which, C.byref(ms), C.byref(n))
        if rc != 0:
            raise AisError(rc, "ais_profile_read")
        return ms.value, n.value

    def copy(self, dst: torch.Tensor, src: torch.Tensor):
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes:
            raise ValueError("size mismatch")
        if not (src.is_contiguous() and dst.is_contiguous()):
            raise ValueError("copy needs contiguous tensors")
        _dev_ptr(dst, self.device, "dst")
        _dev_ptr(src, self.device, "src")
        self._sync_stream()
        rc = self._lib.ais_copy(self._h, C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes)
        if rc != 0:
            raise AisError(rc, "ais_copy")
