"""Thin ctypes binding of libmtpc (include/mtpc.h): argument marshalling only.

Every step of the head runs in the HIP library; PyTorch is used for device
buffers and the current stream.  There is no CPU fallback: if the shared library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtpc.so")

FF, CP, HMM, BTREE = 0, 1, 2, 3
FAMILY = {"ff": FF, "cp": CP, "hmm": HMM, "btree": BTREE}
OP_LOGLIK, OP_MARGINALS, OP_SAMPLE, OP_VERIFY, OP_BACKWARD, OP_TABLE, OP_WINDOWS = 0, 1, 2, 3, 4, 5, 6
VERIFY_SAMPLING, VERIFY_GREEDY = 0, 1
MARG_PREFIX, MARG_UNIVARIATE = 0, 1
SCORE_JOINT, SCORE_PREFIX = 0, 1
F32, BF16 = 0, 1


class MtpcError(RuntimeError):
    pass


class mtpc_head(C.Structure):
    _fields_ = [("B", C.c_int32), ("d", C.c_int32), ("n", C.c_int32), ("r", C.c_int32),
                ("v", C.c_int32), ("dtype", C.c_int32),
                ("h", C.c_void_p), ("ld_h", C.c_int64), ("W", C.c_void_p), ("Wsum", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
                ("W_stage_major", C.c_void_p), ("W_stage_bytes", C.c_int32)]


class mtpc_sumlayers(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("layer_stride", C.c_int64), ("batch_stride", C.c_int64),
                ("R", C.c_void_p), ("R_layer_stride", C.c_int64)]


EXPORTS = [
    "mtpc_status_string", "mtpc_workspace_bytes",
    "mtpc_ff_loglik", "mtpc_cp_loglik", "mtpc_hmm_loglik", "mtpc_btree_loglik",
    "mtpc_ff_marginals", "mtpc_cp_marginals", "mtpc_hmm_marginals", "mtpc_btree_marginals",
    "mtpc_ff_sample", "mtpc_cp_sample", "mtpc_hmm_sample", "mtpc_btree_sample",
    "mtpc_ff_verify", "mtpc_cp_verify", "mtpc_hmm_verify", "mtpc_btree_verify",
    "mtpc_ff_window_scores", "mtpc_cp_window_scores", "mtpc_hmm_window_scores", "mtpc_btree_window_scores",
    "mtpc_ff_table_scores", "mtpc_cp_table_scores", "mtpc_hmm_table_scores", "mtpc_btree_table_scores",
    "mtpc_ff_greedy_draft", "mtpc_cp_greedy_draft", "mtpc_hmm_greedy_draft", "mtpc_btree_greedy_draft",
    "mtpc_ff_loss_backward", "mtpc_cp_loss_backward", "mtpc_hmm_loss_backward", "mtpc_btree_loss_backward",
    "mtpc_philox_uniforms", "mtpc_profile_unembed", "mtpc_profile_circuit", "mtpc_sample_static", "mtpc_pack_weights",
]

_lib = None


def lib() -> C.CDLL:
    """Load libmtpc.so (built by __graft_entry__.build()); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MtpcError(f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        hp, lp, ip, fp = C.POINTER(mtpc_head), C.POINTER(mtpc_sumlayers), C.c_void_p, C.c_void_p
        L.mtpc_status_string.restype = C.c_char_p
        L.mtpc_status_string.argtypes = [C.c_int]
        L.mtpc_workspace_bytes.restype = C.c_size_t
        L.mtpc_workspace_bytes.argtypes = [C.c_int32, C.c_int32, hp, lp, C.c_int32, C.c_int32]
        for fam in ("ff", "cp"):
            getattr(L, f"mtpc_{fam}_loglik").argtypes = [hp, ip, fp]
            getattr(L, f"mtpc_{fam}_marginals").argtypes = [hp, ip, C.c_int32, fp]
            getattr(L, f"mtpc_{fam}_sample").argtypes = [hp, C.c_int32, C.c_uint64, C.c_uint32, ip, ip, fp, fp]
            getattr(L, f"mtpc_{fam}_verify").argtypes = [hp, fp, ip, fp, fp, C.c_int32, C.c_uint64, C.c_uint32, ip, ip]
            getattr(L, f"mtpc_{fam}_greedy_draft").argtypes = [hp, ip, ip, fp, fp]
            getattr(L, f"mtpc_{fam}_table_scores").argtypes = [hp, fp, ip, C.c_int32, C.c_int32, fp]
            getattr(L, f"mtpc_{fam}_window_scores").argtypes = [hp, ip, C.c_int32, ip, C.c_int32, C.c_int32, fp]
        for fam in ("hmm", "btree"):
            getattr(L, f"mtpc_{fam}_loglik").argtypes = [hp, lp, ip, fp]
            getattr(L, f"mtpc_{fam}_marginals").argtypes = [hp, lp, ip, C.c_int32, fp]
            getattr(L, f"mtpc_{fam}_sample").argtypes = [hp, lp, C.c_int32, C.c_uint64, C.c_uint32, ip, ip, fp, fp]
            getattr(L, f"mtpc_{fam}_verify").argtypes = [hp, lp, fp, ip, fp, fp, C.c_int32, C.c_uint64, C.c_uint32, ip, ip]
            getattr(L, f"mtpc_{fam}_greedy_draft").argtypes = [hp, lp, ip, ip, fp, fp]
            getattr(L, f"mtpc_{fam}_table_scores").argtypes = [hp, lp, fp, ip, C.c_int32, C.c_int32, fp]
            getattr(L, f"mtpc_{fam}_window_scores").argtypes = [hp, lp, ip, C.c_int32, ip, C.c_int32, C.c_int32, fp]
        L.mtpc_ff_loss_backward.argtypes = [hp, ip, fp, fp, fp, fp]
        L.mtpc_cp_loss_backward.argtypes = [hp, ip, fp, fp, fp, fp, fp]
        L.mtpc_hmm_loss_backward.argtypes = [hp, lp, ip, fp, fp, fp, fp, fp, fp, fp]
        L.mtpc_btree_loss_backward.argtypes = [hp, lp, ip, fp, fp, fp, fp, fp, fp, fp]
        L.mtpc_philox_uniforms.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_uint64, C.c_uint32,
                                           fp, C.c_void_p]
        L.mtpc_sample_static.argtypes = [C.c_int32, hp, lp, C.c_int32, C.c_uint64, C.c_uint32, ip, ip, fp, fp]
        L.mtpc_pack_weights.argtypes = [hp, C.c_void_p]
        L.mtpc_profile_unembed.argtypes = [C.c_void_p, C.c_void_p]
        L.mtpc_profile_unembed.restype = None
        L.mtpc_profile_circuit.argtypes = [C.c_void_p, C.c_void_p]
        L.mtpc_profile_circuit.restype = None
        for name in EXPORTS:
            if name not in ("mtpc_status_string", "mtpc_workspace_bytes", "mtpc_profile_unembed", "mtpc_profile_circuit"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        raise MtpcError(f"libmtpc: {lib().mtpc_status_string(status).decode()} (status {status})")


def n_latents(family: str, n: int) -> int:
    return {"ff": 0, "cp": 1, "hmm": n, "btree": n - 1}[family]


class Head:
    """Device-resident parameters of one head plus a reusable workspace."""

    def __init__(self, family: str, h: torch.Tensor, W: torch.Tensor, Wsum: Optional[torch.Tensor] = None,
                 layers: Optional[torch.Tensor] = None, R: Optional[torch.Tensor] = None):
        """layers: fp32 logits [L,r,r] / [1,r,r] / [B,L,r,r]; with R ([L,r,r,d] or [1,r,r,d], dtype of h)
        the layer logits are computed from h inside the library and `layers` (3-dim) is the bias."""
        assert family in FAMILY
        assert h.is_cuda and W.is_cuda and h.dim() == 2 and W.dim() == 4
        assert h.dtype == W.dtype and h.dtype in (torch.float32, torch.bfloat16)
        assert h.stride(1) == 1 and W.is_contiguous()
        self.family = family
        self.h, self.W, self.Wsum = h, W, Wsum
        self.B, self.d = h.shape
        self.n, self.r, self.v, d2 = W.shape
        assert d2 == self.d
        if Wsum is not None:
            assert Wsum.is_cuda and Wsum.is_contiguous() and Wsum.dtype == h.dtype and tuple(Wsum.shape) == (self.r, self.d)
        self.layers = layers
        self._sl = None
        if layers is not None:
            assert layers.is_cuda and layers.dtype == torch.float32 and layers.is_contiguous()
            need = self.n - 1 if family == "hmm" else self.n - 2
            if layers.dim() == 3:          # [L, r, r], L == need or 1 (homogeneous)
                L, bs = layers.shape[0], 0
            else:                          # [B, L, r, r] contextual
                assert layers.shape[0] == self.B
                L, bs = layers.shape[1], layers.shape[1] * self.r * self.r
            assert L in (need, 1) and tuple(layers.shape[-2:]) == (self.r, self.r)
            ls = self.r * self.r if (L == need and need > 0) else 0
            if L == 1 and need > 1:
                ls = 0
            self._sl = mtpc_sumlayers(layers.data_ptr(), ls, bs, None, 0)
        self.R = R
        if R is not None:
            need = self.n - 1 if family == "hmm" else self.n - 2
            assert R.is_cuda and R.is_contiguous() and R.dtype == h.dtype and R.dim() == 4
            assert R.shape[0] in (need, 1) and tuple(R.shape[1:]) == (self.r, self.r, self.d)
            assert layers is None or layers.dim() == 3
            rls = self.r * self.r * self.d if (R.shape[0] == need and need > 1) else 0
            if self._sl is None:
                self._sl = mtpc_sumlayers(None, 0, 0, R.data_ptr(), rls)
            else:
                self._sl.R, self._sl.R_layer_stride = R.data_ptr(), rls
        self._ws = None
        self.W_stage_major = None
        self.W_stage_bytes = 0

    def pack_W(self, stage_bytes: Optional[int] = None) -> None:
        """Make the stage-major copy of W (for serving, W fixed) and use it from now on: the pass over
        all of W reads it instead of W's rows.  The stage size has to be the one that pass uses for this
        head's batch (the default): 128 bytes up to 64 positions, 64 bytes above.  Costs one more buffer
        of the size of W."""
        buf = torch.empty_like(self.W)
        hd = self._head(256)
        hd.W_stage_major = None
        hd.W_stage_bytes = stage_bytes if stage_bytes is not None else (128 if self.B <= 64 else 64)
        _check(lib().mtpc_pack_weights(C.byref(hd), buf.data_ptr()))
        self.W_stage_major, self.W_stage_bytes = buf, hd.W_stage_bytes

    # ---- plumbing --------------------------------------------------------
    def _head(self, ws_bytes: int) -> mtpc_head:
        if self._ws is None or self._ws.numel() < ws_bytes:
            self._ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=self.h.device)
        hd = mtpc_head()
        hd.B, hd.d, hd.n, hd.r, hd.v = self.B, self.d, self.n, self.r, self.v
        hd.dtype = BF16 if self.h.dtype == torch.bfloat16 else F32
        hd.h, hd.ld_h = self.h.data_ptr(), self.h.stride(0)
        hd.W = self.W.data_ptr()
        hd.Wsum = self.Wsum.data_ptr() if self.Wsum is not None else None
        hd.workspace, hd.workspace_bytes = self._ws.data_ptr(), self._ws.numel()
        hd.stream = torch.cuda.current_stream(self.h.device).cuda_stream
        hd.W_stage_major = self.W_stage_major.data_ptr() if self.W_stage_major is not None else None
        hd.W_stage_bytes = self.W_stage_bytes
        return hd

    def _layers_ref(self):
        return C.byref(self._sl) if self._sl is not None else None

    def workspace_bytes(self, op: int, S: int = 1, mode: int = 0) -> int:
        probe = mtpc_head()
        probe.B, probe.d, probe.n, probe.r, probe.v = self.B, self.d, self.n, self.r, self.v
        return lib().mtpc_workspace_bytes(FAMILY[self.family], op, C.byref(probe), self._layers_ref(), S, mode)

    def _call(self, name, hd, *args):
        fn = getattr(lib(), f"mtpc_{self.family}_{name}")
        if self.family in ("hmm", "btree"):
            return fn(C.byref(hd), self._layers_ref(), *args)
        return fn(C.byref(hd), *args)

    # ---- operations ------------------------------------------------------
    def loglik(self, targets: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        assert targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous()
        assert tuple(targets.shape) == (self.B, self.n)
        if out is None:
            out = torch.empty(self.B, dtype=torch.float32, device=self.h.device)
        hd = self._head(self.workspace_bytes(OP_LOGLIK))
        _check(self._call("loglik", hd, targets.data_ptr(), out.data_ptr()))
        return out

    def prefix_marginals(self, targets: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        assert targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous()
        assert tuple(targets.shape) == (self.B, self.n)
        if out is None:
            out = torch.empty(self.B, self.n, dtype=torch.float32, device=self.h.device)
        hd = self._head(self.workspace_bytes(OP_MARGINALS, mode=MARG_PREFIX))
        _check(self._call("marginals", hd, targets.data_ptr(), MARG_PREFIX, out.data_ptr()))
        return out

    def univariate_marginals(self, out: Optional[torch.Tensor] = None, keep_table: bool = True) -> torch.Tensor:
        """[B,n,v] log marginal of every token.  keep_table=False hands the library a workspace without
        room for the table of input units (B n r v floats): the mixture is then formed in registers."""
        if out is None:
            out = torch.empty(self.B, self.n, self.v, dtype=torch.float32, device=self.h.device)
        need = self.workspace_bytes(OP_MARGINALS, mode=MARG_UNIVARIATE)
        hd = self._head(need)
        if not keep_table and self.r > 1:
            hd.workspace_bytes = max(need - 4 * self.B * self.n * self.r * self.v, 16)
        _check(self._call("marginals", hd, None, MARG_UNIVARIATE, out.data_ptr()))
        return out

    def sample(self, S: int, seed: int, offset: int = 0, want_latents: bool = True,
               want_prefix: bool = False, out=None, logphi: Optional[torch.Tensor] = None):
        """Returns (drafts [B,S,n] int32, latents [B,S,n_lat] int32 or None, prefix_logq [B,S,n] or None).
        logphi: optional fp32 [B,n,r,v] buffer that receives the normalised input units (for verify)."""
        dev = self.h.device
        if out is None:
            drafts = torch.empty(self.B, S, self.n, dtype=torch.int32, device=dev)
            nl = n_latents(self.family, self.n)
            lat = torch.empty(self.B, S, nl, dtype=torch.int32, device=dev) if want_latents else None
            pl = torch.empty(self.B, S, self.n, dtype=torch.float32, device=dev) if want_prefix else None
        else:
            drafts, lat, pl = out
        hd = self._head(self.workspace_bytes(OP_SAMPLE, S=S))
        _check(self._call("sample", hd, S, seed, offset, drafts.data_ptr(),
                          lat.data_ptr() if lat is not None and lat.numel() > 0 else None,
                          pl.data_ptr() if pl is not None else None,
                          self._phi_ptr(logphi)))
        return drafts, lat, pl

    def sample_static(self, S: int, seed: int, offset: int, drafts: torch.Tensor, latents: Optional[torch.Tensor] = None,
                      prefix_logq: Optional[torch.Tensor] = None, logphi: Optional[torch.Tensor] = None) -> None:
        """sample() through the entry point that allocates nothing: every buffer is the caller's, the
        scratch is the library's static device array (one per GPU; calls on one GPU must not overlap)."""
        assert drafts.is_cuda and drafts.dtype == torch.int32 and drafts.is_contiguous()
        assert tuple(drafts.shape) == (self.B, S, self.n)
        hd = mtpc_head()
        hd.B, hd.d, hd.n, hd.r, hd.v = self.B, self.d, self.n, self.r, self.v
        hd.dtype = BF16 if self.h.dtype == torch.bfloat16 else F32
        hd.h, hd.ld_h = self.h.data_ptr(), self.h.stride(0)
        hd.W = self.W.data_ptr()
        hd.Wsum = self.Wsum.data_ptr() if self.Wsum is not None else None
        hd.workspace, hd.workspace_bytes = None, 0
        hd.stream = torch.cuda.current_stream(self.h.device).cuda_stream
        hd.W_stage_major = self.W_stage_major.data_ptr() if self.W_stage_major is not None else None
        hd.W_stage_bytes = self.W_stage_bytes
        _check(lib().mtpc_sample_static(FAMILY[self.family], C.byref(hd), self._layers_ref(), S, seed, offset,
                                        drafts.data_ptr(),
                                        latents.data_ptr() if latents is not None and latents.numel() > 0 else None,
                                        prefix_logq.data_ptr() if prefix_logq is not None else None,
                                        self._phi_ptr(logphi)))

    def loss_backward(self, targets: torch.Tensor, coef: torch.Tensor, out: Optional[dict] = None,
                      recompute: bool = False) -> dict:
        """Loss of Sec. 4.1 and its gradients: targets [B,n] int32, coef [B,n] fp32.
        Returns {"loss" [B], "dh" [B,d], "dW" [n,r,v,d], "dWsum" [r,d] or None, "dlayers" or None,
        "dR" (layers computed from h) or None}, all fp32."""
        dev = self.h.device
        assert targets.is_cuda and targets.dtype == torch.int32 and targets.is_contiguous()
        assert coef.is_cuda and coef.dtype == torch.float32 and coef.is_contiguous()
        assert tuple(targets.shape) == (self.B, self.n) and tuple(coef.shape) == (self.B, self.n)
        f32 = dict(dtype=torch.float32, device=dev)
        if out is None:
            out = {"loss": torch.empty(self.B, **f32), "dh": torch.empty(self.B, self.d, **f32),
                   "dW": torch.empty(self.n, self.r, self.v, self.d, **f32),
                   "dWsum": None if self.family == "ff" else torch.empty(self.r, self.d, **f32),
                   "dlayers": None if self.layers is None else torch.empty_like(self.layers),
                   "dR": None if self.R is None else torch.empty(self.R.shape, **f32)}
        # the library picks its plan from the workspace size it is handed
        need = self.workspace_bytes(OP_BACKWARD, mode=1 if recompute else 0)
        hd = self._head(need)
        if recompute:
            hd.workspace_bytes = need
        args = [targets.data_ptr(), coef.data_ptr(), out["loss"].data_ptr(), out["dh"].data_ptr(),
                out["dW"].data_ptr()]
        if self.family != "ff":
            args.append(out["dWsum"].data_ptr())
        if self.family in ("hmm", "btree"):
            args.append(out["dlayers"].data_ptr() if out["dlayers"] is not None else None)
            args.append(out["dR"].data_ptr() if out.get("dR") is not None else None)
        _check(self._call("loss_backward", hd, *args))
        return out

    def greedy_draft(self, want_latents: bool = True, want_prefix: bool = False,
                     logphi: Optional[torch.Tensor] = None):
        """The argmax traversal: returns (drafts [B,n] int32, latents [B,n_lat] or None, prefix_logq [B,n] or None)."""
        dev = self.h.device
        drafts = torch.empty(self.B, self.n, dtype=torch.int32, device=dev)
        nl = n_latents(self.family, self.n)
        lat = torch.empty(self.B, nl, dtype=torch.int32, device=dev) if want_latents else None
        pl = torch.empty(self.B, self.n, dtype=torch.float32, device=dev) if want_prefix else None
        hd = self._head(self.workspace_bytes(OP_SAMPLE, S=1))
        _check(self._call("greedy_draft", hd, drafts.data_ptr(),
                          lat.data_ptr() if lat is not None and lat.numel() > 0 else None,
                          pl.data_ptr() if pl is not None else None, self._phi_ptr(logphi)))
        return drafts, lat, pl

    def _phi_ptr(self, logphi):
        if logphi is None:
            return None
        assert logphi.is_cuda and logphi.dtype == torch.float32 and logphi.is_contiguous()
        assert tuple(logphi.shape) == (self.B, self.n, self.r, self.v)
        return logphi.data_ptr()

    def window_scores(self, x: torch.Tensor, x2: Optional[torch.Tensor] = None, prefix: bool = False,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Scores of the windows x [B,T,n] and (optionally) x2 [B,T2,n], int32, in one unembedding pass:
        log-likelihoods [B,T+T2], or prefix marginals [B,T+T2,n] with prefix=True (x's windows first)."""
        def chk(t):
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
            assert t.dim() == 3 and t.shape[0] == self.B and t.shape[2] == self.n
            return t.shape[1]
        T = chk(x)
        T2 = chk(x2) if x2 is not None else 0
        shape = (self.B, T + T2, self.n) if prefix else (self.B, T + T2)
        if out is None:
            out = torch.empty(shape, dtype=torch.float32, device=self.h.device)
        else:
            assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == shape
        hd = self._head(self.workspace_bytes(OP_WINDOWS, S=T + T2))
        _check(self._call("window_scores", hd, x.data_ptr(), T, x2.data_ptr() if x2 is not None else None, T2,
                          SCORE_PREFIX if prefix else SCORE_JOINT, out.data_ptr()))
        return out

    def table_scores(self, logphi: torch.Tensor, x: torch.Tensor, prefix: bool = False,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Scores of windows x [B,T,n] (or [B,n]) int32 from the table logphi [B,n,r,v] a sample() call
        left: log-likelihoods [B,T], or prefix marginals [B,T,n] with prefix=True."""
        assert x.is_cuda and x.dtype == torch.int32 and x.is_contiguous()
        squeeze = x.dim() == 2
        xs = x.unsqueeze(1) if squeeze else x
        assert xs.dim() == 3 and xs.shape[0] == self.B and xs.shape[2] == self.n
        T = xs.shape[1]
        shape = (self.B, T, self.n) if prefix else (self.B, T)
        if out is None:
            out = torch.empty(shape, dtype=torch.float32, device=self.h.device)
        else:
            assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == self.B * T * (self.n if prefix else 1)
            out = out.view(shape)
        hd = self._head(self.workspace_bytes(OP_TABLE, S=T))
        _check(self._call("table_scores", hd, self._phi_ptr(logphi), xs.data_ptr(), T,
                          SCORE_PREFIX if prefix else SCORE_JOINT, out.data_ptr()))
        return out.squeeze(1) if squeeze else out

    def verify(self, drafts: torch.Tensor, p: torch.Tensor, prefix_logq: Optional[torch.Tensor] = None,
               logphi: Optional[torch.Tensor] = None, seed: int = 0, offset: int = 0, mode: str = "sampling"):
        """One verification per position: drafts [B,n] int32, p [B,n+1,v] fp32 verifier probabilities,
        prefix_logq [B,n] and logphi [B,n,r,v] from sample().  Returns (accepted [B], token [B]) int32."""
        dev = self.h.device
        assert drafts.is_cuda and drafts.dtype == torch.int32 and drafts.is_contiguous()
        assert tuple(drafts.shape) == (self.B, self.n)
        assert p.is_cuda and p.dtype == torch.float32 and p.is_contiguous()
        assert tuple(p.shape) == (self.B, self.n + 1, self.v)
        if prefix_logq is not None:
            assert prefix_logq.is_cuda and prefix_logq.dtype == torch.float32 and prefix_logq.is_contiguous()
            assert tuple(prefix_logq.shape) == (self.B, self.n)
        accepted = torch.empty(self.B, dtype=torch.int32, device=dev)
        token = torch.empty(self.B, dtype=torch.int32, device=dev)
        hd = self._head(self.workspace_bytes(OP_VERIFY))
        _check(self._call("verify", hd, self._phi_ptr(logphi), drafts.data_ptr(),
                          prefix_logq.data_ptr() if prefix_logq is not None else None, p.data_ptr(),
                          {"sampling": VERIFY_SAMPLING, "greedy": VERIFY_GREEDY}[mode], seed, offset,
                          accepted.data_ptr(), token.data_ptr()))
        return accepted, token


def philox_uniforms(B: int, S: int, slots: int, seed: int, offset: int = 0, device="cuda") -> torch.Tensor:
    out = torch.empty(B, S, slots, dtype=torch.float32, device=device)
    st = torch.cuda.current_stream(out.device).cuda_stream
    _check(lib().mtpc_philox_uniforms(B, S, slots, seed, offset, out.data_ptr(), st))
    return out


def profile_unembed(start_event: Optional[int], stop_event: Optional[int]) -> None:
    lib().mtpc_profile_unembed(start_event, stop_event)


def profile_circuit(start_event: Optional[int], stop_event: Optional[int]) -> None:
    lib().mtpc_profile_circuit(start_event, stop_event)
