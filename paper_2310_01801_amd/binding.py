"""Thin Python binding of libfastgen.so (ctypes): argument marshalling only.

Every step of the path runs inside the HIP library; PyTorch only supplies device memory and
the stream. There is no fallback: if the library has not been built (``python -m
paper_2310_01801_amd.build``) loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastgen.so")

FG_OK, FG_EINVAL, FG_ENOMEM, FG_EHIP, FG_ESTATE, FG_ECAP = range(6)
FG_F32, FG_BF16 = 0, 1
FG_COMP_SPECIAL, FG_COMP_PUNCT, FG_COMP_FREQUENT, FG_COMP_LOCAL = 1, 2, 4, 8
STATUS_NAMES = ("FG_OK", "FG_EINVAL", "FG_ENOMEM", "FG_EHIP", "FG_ESTATE", "FG_ECAP")

EXPORTED = (
    "fastgen_workspace_bytes", "fastgen_create", "fastgen_destroy", "fastgen_profile",
    "fastgen_compact", "fastgen_decode_step", "fastgen_decode_step_probe", "fastgen_export_state", "fastgen_last_error",
    "fastgen_version", "fastgen_enable_timing", "fastgen_read_timing", "fastgen_profile_static", "fastgen_classify",
)
PHASES = ("sweep1", "sweep2", "select", "compact", "decode_attn", "decode_update")


class FgConfig(ctypes.Structure):
    _fields_ = [
        ("num_units", ctypes.c_int32), ("num_seqs", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("prompt_len", ctypes.c_int32), ("max_new_tokens", ctypes.c_int32),
        ("T", ctypes.c_double), ("r_l", ctypes.c_double), ("r_f", ctypes.c_double),
        ("softmax_scale", ctypes.c_float), ("forced_policy", ctypes.c_int32),
        ("cache_tokens", ctypes.c_int64), ("family", ctypes.c_int32 * 4), ("group_size", ctypes.c_int32),
    ]


class FastGenError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2310_01801_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, cp = ctypes.c_void_p, ctypes.POINTER(FgConfig)
    lib.fastgen_workspace_bytes.restype = ctypes.c_size_t
    lib.fastgen_workspace_bytes.argtypes = [cp]
    lib.fastgen_create.restype = ctypes.c_int
    lib.fastgen_create.argtypes = [cp, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    lib.fastgen_destroy.restype = ctypes.c_int
    lib.fastgen_destroy.argtypes = [vp]
    lib.fastgen_profile.restype = ctypes.c_int
    lib.fastgen_profile.argtypes = [vp] * 9
    lib.fastgen_profile_static.restype = ctypes.c_int
    lib.fastgen_profile_static.argtypes = [cp] + [vp] * 8
    lib.fastgen_classify.restype = ctypes.c_int
    lib.fastgen_classify.argtypes = [vp, ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                     ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, vp, vp]
    lib.fastgen_compact.restype = ctypes.c_int
    lib.fastgen_compact.argtypes = [vp] * 4
    lib.fastgen_decode_step.restype = ctypes.c_int
    lib.fastgen_decode_step.argtypes = [vp] * 7
    lib.fastgen_decode_step_probe.restype = ctypes.c_int
    lib.fastgen_decode_step_probe.argtypes = [vp] * 8
    lib.fastgen_export_state.restype = ctypes.c_int
    lib.fastgen_export_state.argtypes = [vp] * 9
    lib.fastgen_last_error.restype = ctypes.c_char_p
    lib.fastgen_last_error.argtypes = [vp]
    lib.fastgen_enable_timing.restype = ctypes.c_int
    lib.fastgen_enable_timing.argtypes = [vp, ctypes.c_int]
    lib.fastgen_read_timing.restype = ctypes.c_int
    lib.fastgen_read_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.fastgen_version.restype = ctypes.c_char_p
    lib.fastgen_version.argtypes = []
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_config(num_units: int, num_seqs: int, head_dim: int, dtype: torch.dtype, prompt_len: int,
                max_new_tokens: int, T: float, r_l: float, r_f: float, softmax_scale: float = 0.0,
                forced_policy: int = -1, cache_tokens: int = 0, family=None,
                group_size: int = 1) -> FgConfig:
    """family: None (the family of Eq. 2) or four FG_COMP_* masks for policy ids 0..3."""
    code = {torch.float32: FG_F32, torch.bfloat16: FG_BF16}[dtype]
    fam = (ctypes.c_int32 * 4)(*(family if family is not None else (0, 0, 0, 0)))
    return FgConfig(num_units, num_seqs, head_dim, code, prompt_len, max_new_tokens, T, r_l, r_f,
                    softmax_scale, forced_policy, cache_tokens, fam, group_size)


def fastgen_workspace_bytes(cfg: FgConfig) -> int:
    return int(load_library().fastgen_workspace_bytes(ctypes.byref(cfg)))


def fastgen_classify(token_ids: torch.Tensor, special_ids, punct_ids,
                     token_class: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Class bytes (FG_CLASS_* bits) of int32 token ids on the device; the id lists are host
    sequences of at most 64 ids each."""
    lib = load_library()
    assert token_ids.dtype == torch.int32
    if token_class is None:
        token_class = torch.empty(token_ids.shape, dtype=torch.uint8, device=token_ids.device)
    sp = (ctypes.c_int32 * max(1, len(special_ids)))(*[int(x) for x in special_ids])
    pu = (ctypes.c_int32 * max(1, len(punct_ids)))(*[int(x) for x in punct_ids])
    st = lib.fastgen_classify(_ptr(token_ids), token_ids.numel(), sp, len(special_ids), pu, len(punct_ids),
                              _ptr(token_class), _stream())
    if st != FG_OK:
        raise FastGenError(st, lib.fastgen_last_error(None).decode())
    return token_class


def fastgen_profile_static(cfg: FgConfig, Q: torch.Tensor, K: torch.Tensor, token_class: torch.Tensor,
                           policy: torch.Tensor, recovery: torch.Tensor, kept_count: torch.Tensor,
                           lse: Optional[torch.Tensor] = None) -> None:
    """fastgen_profile without a context or a workspace (the library's static scratch array).
    The caller passes the output tensors: this wrapper allocates nothing either."""
    lib = load_library()
    st = lib.fastgen_profile_static(ctypes.byref(cfg), _ptr(Q), _ptr(K), _ptr(token_class), _ptr(lse),
                                    _ptr(policy), _ptr(recovery), _ptr(kept_count), _stream())
    if st != FG_OK:
        raise FastGenError(st, lib.fastgen_last_error(None).decode())


class FastGen:
    """One context over a torch-allocated workspace. Methods mirror the C entry points."""

    def __init__(self, cfg: FgConfig, device: str = "cuda:0", workspace: Optional[torch.Tensor] = None):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = fastgen_workspace_bytes(cfg)
        if nbytes == 0:
            raise FastGenError(FG_EINVAL, "invalid configuration")
        if workspace is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert workspace.numel() * workspace.element_size() >= nbytes
        self.workspace = workspace
        self._ctx = ctypes.c_void_p()
        st = self.lib.fastgen_create(ctypes.byref(cfg), self.workspace.data_ptr(), nbytes,
                                     ctypes.byref(self._ctx))
        if st != FG_OK:
            raise FastGenError(st, "fastgen_create failed")
        self.tdtype = torch.float32 if cfg.dtype == FG_F32 else torch.bfloat16

    def close(self) -> None:
        if self._ctx:
            self.lib.fastgen_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int) -> None:
        if st != FG_OK:
            raise FastGenError(st, self.lib.fastgen_last_error(self._ctx).decode())

    def fastgen_enable_timing(self, enable=True) -> None:
        """True/1: time every kernel group; N > 1: the prompt phases and every N-th decode step."""
        self._check(self.lib.fastgen_enable_timing(self._ctx, int(enable)))

    def fastgen_read_timing(self) -> Dict[str, Tuple[float, int]]:
        ms = (ctypes.c_double * len(PHASES))()
        cnt = (ctypes.c_int64 * len(PHASES))()
        self._check(self.lib.fastgen_read_timing(self._ctx, ms, cnt))
        return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(PHASES)}

    # -- stage 1
    def fastgen_profile(self, Q: torch.Tensor, K: torch.Tensor, token_class: torch.Tensor,
                        lse: Optional[torch.Tensor] = None
                        ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        U = self.cfg.num_units
        policy = torch.empty(U, dtype=torch.int32, device=self.device)
        recovery = torch.empty((U, 5), dtype=torch.float64, device=self.device)
        kept = torch.empty((U, 5), dtype=torch.int32, device=self.device)
        self._check(self.lib.fastgen_profile(self._ctx, _ptr(Q), _ptr(K), _ptr(token_class), _ptr(lse),
                                             _ptr(policy), _ptr(recovery), _ptr(kept), _stream()))
        return policy, recovery, kept

    def fastgen_compact(self, K: torch.Tensor, V: torch.Tensor) -> None:
        self._check(self.lib.fastgen_compact(self._ctx, _ptr(K), _ptr(V), _stream()))

    # -- stage 2
    def fastgen_decode_step(self, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                            class_new: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty((self.cfg.num_units * max(1, self.cfg.group_size), self.cfg.head_dim),
                              dtype=self.tdtype, device=self.device)
        self._check(self.lib.fastgen_decode_step(self._ctx, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                 _ptr(class_new), _ptr(out), _stream()))
        return out

    def fastgen_decode_step_probe(self, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                                  class_new: torch.Tensor, out: Optional[torch.Tensor] = None
                                  ) -> Tuple[torch.Tensor, torch.Tensor]:
        if out is None:
            out = torch.empty((self.cfg.num_units * max(1, self.cfg.group_size), self.cfg.head_dim),
                              dtype=self.tdtype, device=self.device)
        rho = torch.empty((self.cfg.num_units, 5), dtype=torch.float64, device=self.device)
        self._check(self.lib.fastgen_decode_step_probe(self._ctx, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                       _ptr(class_new), _ptr(out), _ptr(rho), _stream()))
        return out, rho

    def fastgen_export_state(self, rows: bool = False, lengths_only: bool = False) -> Dict[str, torch.Tensor]:
        U, d = self.cfg.num_units, self.cfg.head_dim
        lengths = torch.empty(U, dtype=torch.int32, device=self.device)
        offsets = torch.empty(U + 1, dtype=torch.int64, device=self.device)
        status = torch.zeros(1, dtype=torch.int32, device=self.device)
        # first the lengths, to size the packed outputs
        self._check(self.lib.fastgen_export_state(self._ctx, _ptr(lengths), _ptr(offsets), None, None,
                                                  None, None, _ptr(status), _stream()))
        if lengths_only:
            return dict(lengths=lengths, offsets=offsets, status=status)
        total = int(offsets[-1].item())
        positions = torch.empty(max(total, 1), dtype=torch.int32, device=self.device)
        scores = torch.empty(max(total, 1), dtype=torch.float64, device=self.device)
        keys = values = None
        if rows:
            keys = torch.empty((max(total, 1), d), dtype=self.tdtype, device=self.device)
            values = torch.empty_like(keys)
        self._check(self.lib.fastgen_export_state(self._ctx, _ptr(lengths), _ptr(offsets), _ptr(positions),
                                                  _ptr(scores), _ptr(keys), _ptr(values), _ptr(status),
                                                  _stream()))
        return dict(lengths=lengths, offsets=offsets, positions=positions[:total], scores=scores[:total],
                    keys=None if keys is None else keys[:total],
                    values=None if values is None else values[:total], status=status)
