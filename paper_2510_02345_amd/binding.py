"""ctypes binding of libcmoe.so.  Same names and argument order as include/cmoe.h.

Argument marshalling only: tensors are passed as raw device pointers
(`tensor.data_ptr()`), the stream as the current torch stream's handle.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(PKG, "libcmoe.so")
_lib = None

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4

EXPORTS = ("cmoe_create", "cmoe_destroy", "cmoe_workspace_bytes", "cmoe_route", "cmoe_permute", "cmoe_permute_static",
           "cmoe_ffn_forward", "cmoe_combine", "cmoe_forward", "cmoe_route_multi", "cmoe_workspace_bytes_multi",
           "cmoe_forward_multi", "cmoe_route_stats", "cmoe_compress_workspace_bytes", "cmoe_compress",
           "cmoe_quantize_int4", "cmoe_reconstruction_error", "cmoe_backward_workspace_bytes", "cmoe_backward",
           "cmoe_packed_bytes", "cmoe_pack_weights",
           "cmoe_last_hip_error", "cmoe_status_string",
           "cmoe_timing_enable", "cmoe_timing_read", "cmoe_timing_name", "cmoe_calibrate_mfma")


class CmoeError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status, self.hip = status, hip
        super().__init__(f"{where}: {status_string(status)} (status {status}, hipError {hip})")


class CompressConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("out_dim", "in_dim", "G", "K", "r", "q_group", "sketch", "n_iter",
                                         "use_gate")] + [("gate_gamma", C.c_float)]


class Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dx", "d_logits", "d_router_expert", "dw1_base", "dw2_base", "du1", "dv1",
                                          "du2", "dv2")]


class RouteOptions(C.Structure):
    _fields_ = [("top_g", C.c_int32), ("temperature", C.c_float), ("scale_by_cluster_prob", C.c_int32)]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "d_ff", "G", "K", "r", "top_k", "q_group", "activation")]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("router_cluster", "router_expert", "cluster_bias", "w1_base", "w2_base",
                                          "v1_q", "u1_q", "v2_q", "u2_q", "v1_s", "u1_s", "v2_s", "u2_s",
                                          "packed")]


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Loads libcmoe.so (built in-tree by paper_2510_02345_amd/build.py); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is not built: run `python -m paper_2510_02345_amd.build`")
    L = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.cmoe_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    L.cmoe_destroy.argtypes = [vp]
    L.cmoe_workspace_bytes.argtypes = [vp, i32]
    L.cmoe_workspace_bytes.restype = sz
    L.cmoe_route.argtypes = [vp, C.POINTER(Weights), vp, i32, vp, vp, vp, vp]
    L.cmoe_permute.argtypes = [vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.cmoe_permute_static.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.cmoe_ffn_forward.argtypes = [vp, C.POINTER(Weights), vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cmoe_combine.argtypes = [vp, C.POINTER(Weights), vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.cmoe_forward.argtypes = [vp, C.POINTER(Weights), vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cmoe_route_stats.argtypes = [vp, vp, i32, vp, vp, vp, C.c_float, C.c_float, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cmoe_route_multi.argtypes = [vp, C.POINTER(Weights), C.POINTER(RouteOptions), vp, i32, vp, vp, vp, vp]
    L.cmoe_workspace_bytes_multi.argtypes = [vp, i32, i32]
    L.cmoe_workspace_bytes_multi.restype = sz
    L.cmoe_forward_multi.argtypes = [vp, C.POINTER(Weights), C.POINTER(RouteOptions), vp, i32, vp, vp, vp, vp, vp, vp,
                                     vp, vp, sz, vp]
    L.cmoe_compress_workspace_bytes.argtypes = [C.POINTER(CompressConfig)]
    L.cmoe_compress_workspace_bytes.restype = sz
    L.cmoe_compress.argtypes = [C.POINTER(CompressConfig), vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cmoe_quantize_int4.argtypes = [vp, C.c_int64, i32, i32, vp, vp, vp]
    L.cmoe_reconstruction_error.argtypes = [C.POINTER(CompressConfig), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cmoe_packed_bytes.argtypes = [vp]
    L.cmoe_packed_bytes.restype = sz
    L.cmoe_pack_weights.argtypes = [vp, C.POINTER(Weights), vp, sz, vp]
    L.cmoe_backward_workspace_bytes.argtypes = [vp, i32]
    L.cmoe_backward_workspace_bytes.restype = sz
    L.cmoe_backward.argtypes = [vp, C.POINTER(Weights), vp, vp, i32, vp, vp, C.POINTER(Grads), vp, sz, vp]
    L.cmoe_last_hip_error.argtypes = [vp]
    L.cmoe_status_string.argtypes = [C.c_int]
    L.cmoe_status_string.restype = C.c_char_p
    L.cmoe_timing_enable.argtypes = [vp, C.c_int]
    L.cmoe_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32), i32]
    L.cmoe_timing_name.argtypes = [i32]
    L.cmoe_timing_name.restype = C.c_char_p
    L.cmoe_calibrate_mfma.argtypes = [i32, i32, i32, vp, vp, vp]
    for name in EXPORTS:
        if name not in ("cmoe_workspace_bytes", "cmoe_status_string", "cmoe_timing_name",
                        "cmoe_compress_workspace_bytes", "cmoe_workspace_bytes_multi",
                        "cmoe_backward_workspace_bytes", "cmoe_packed_bytes"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().cmoe_status_string(status).decode()


def _cur_stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _chk(status: int, where: str):
    if status != 0:
        raise CmoeError(status, where)


def compress(W, omega, G: int, K: int, r: int, q: int, n_iter: int = 2, use_gate: bool = False,
             gate_gamma: float = 0.05):
    """cmoe_compress on W [G*K][out][in] f16 (device) with the random test rows omega
    [sketch][in] f16.  Returns dict(base, u_q, u_s, v_q, v_s, report)."""
    import torch
    E, out_d, in_d = W.shape
    assert E == G * K and omega.shape[1] == in_d
    cfg = CompressConfig(out_d, in_d, G, K, r, q, omega.shape[0], n_iter, int(use_gate), float(gate_gamma))
    nbytes = lib().cmoe_compress_workspace_bytes(C.byref(cfg))
    if nbytes == 0:
        raise CmoeError(-2, "cmoe_compress_workspace_bytes")
    dev = W.device
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
    o = dict(base=torch.empty((G, out_d, in_d), dtype=torch.float16, device=dev),
             u_q=torch.empty((E, r, out_d // 2), dtype=torch.uint8, device=dev),
             u_s=torch.empty((E, r, out_d // q), dtype=torch.float16, device=dev),
             v_q=torch.empty((E, r, in_d // 2), dtype=torch.uint8, device=dev),
             v_s=torch.empty((E, r, in_d // q), dtype=torch.float16, device=dev),
             report=torch.empty((E, 4), dtype=torch.float32, device=dev))
    _chk(lib().cmoe_compress(C.byref(cfg), _ptr(W), _ptr(omega), _ptr(o["base"]), _ptr(o["u_q"]), _ptr(o["u_s"]),
                             _ptr(o["v_q"]), _ptr(o["v_s"]), _ptr(o["report"]), _ptr(ws), nbytes, _cur_stream()),
         "cmoe_compress")
    o["_workspace"] = ws      # kept alive until the caller synchronises
    return o


def quantize_int4(src, q: int):
    """cmoe_quantize_int4: src [rows][L] f32 (device) -> (codes uint8 [rows][L/2], scales f16 [rows][L/q])."""
    import torch
    rows, L = src.shape
    codes = torch.empty((rows, L // 2), dtype=torch.uint8, device=src.device)
    scales = torch.empty((rows, L // q), dtype=torch.float16, device=src.device)
    _chk(lib().cmoe_quantize_int4(_ptr(src), rows, L, q, _ptr(codes), _ptr(scales), _cur_stream()),
         "cmoe_quantize_int4")
    return codes, scales


def reconstruction_error(W, base, u_q, u_s, v_q, v_s, G: int, K: int, r: int, q: int):
    """cmoe_reconstruction_error: relative Frobenius error per expert of a stored form."""
    import torch
    E, out_d, in_d = W.shape
    cfg = CompressConfig(out_d, in_d, G, K, r, q, r, 0, 0, 0.0)
    nbytes = lib().cmoe_compress_workspace_bytes(C.byref(cfg))
    if nbytes == 0:
        raise CmoeError(-2, "cmoe_compress_workspace_bytes")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=W.device)
    err = torch.empty((E,), dtype=torch.float32, device=W.device)
    _chk(lib().cmoe_reconstruction_error(C.byref(cfg), _ptr(W), _ptr(base), _ptr(u_q), _ptr(u_s), _ptr(v_q),
                                         _ptr(v_s), _ptr(err), _ptr(ws), nbytes, _cur_stream()),
         "cmoe_reconstruction_error")
    torch.cuda.current_stream().synchronize()   # the workspace is freed on return
    return err


def calibrate_mfma(n_workgroups: int = 256, iters: int = 40000, device="cuda:0", zero_operands: bool = False):
    """cmoe_calibrate_mfma between two events: (TFLOP/s sustained by the matrix cores with every
    issue slot used and no memory traffic, shader clock in GHz during the loop)."""
    import torch
    ticks = torch.zeros((2,), dtype=torch.int64, device=device)
    sink = torch.empty((n_workgroups * 512,), dtype=torch.float32, device=device)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    _chk(lib().cmoe_calibrate_mfma(n_workgroups, max(iters // 20, 1), int(zero_operands), _ptr(ticks), _ptr(sink),
                                   _cur_stream()),
         "cmoe_calibrate_mfma")        # warm-up
    torch.cuda.synchronize()
    ticks.zero_()
    e0.record()
    _chk(lib().cmoe_calibrate_mfma(n_workgroups, iters, int(zero_operands), _ptr(ticks), _ptr(sink), _cur_stream()),
         "cmoe_calibrate_mfma")
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    t = ticks.cpu().tolist()
    flops = n_workgroups * 8.0 * iters * 32 * 16384
    return flops / (ms * 1e-3) / 1e12, (t[0] / t[1] * 0.1 if t[1] else 0.0)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Layer:
    """One layer: a cmoe handle, its device weights and a workspace for up to T_max tokens."""

    WEIGHT_NAMES = ("router_cluster", "router_expert", "cluster_bias", "w1_base", "w2_base",
                    "v1_q", "u1_q", "v2_q", "u2_q", "v1_s", "u1_s", "v2_s", "u2_s")

    def __init__(self, d, d_ff, G, K, r, top_k, q_group, weights: Dict[str, object], T_max: int, device="cuda:0",
                 pack: bool = True):
        """pack: make the one-time re-tiled copy of the bases and FP16 factor panels
        (cmoe_pack_weights) that every call then reads; pack=False keeps the canonical arrays only."""
        import torch
        self.torch = torch
        self.cfg = Config(d, d_ff, G, K, r, top_k, q_group, 0)
        self.device = torch.device(device)
        self._h = C.c_void_p()
        rc = lib().cmoe_create(C.byref(self.cfg), C.byref(self._h))
        if rc != OK:
            raise CmoeError(rc, "cmoe_create")
        self.w_t = {}
        for n in self.WEIGHT_NAMES:
            v = weights.get(n)
            if v is None:
                self.w_t[n] = None
            elif isinstance(v, torch.Tensor):
                self.w_t[n] = v.to(self.device).contiguous()
            else:
                self.w_t[n] = torch.from_numpy(v).to(self.device).contiguous()
        self.w = Weights(*[_ptr(self.w_t[n]) for n in self.WEIGHT_NAMES])
        self.T_max = T_max
        self.ws_bytes = lib().cmoe_workspace_bytes(self._h, T_max)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)
        assert self.ws.data_ptr() % 256 == 0
        self.packed = None
        if pack:
            self.pack()

    def pack(self):
        """(Re)build the packed copy of the bases from the layer's current w1_base / w2_base."""
        t = self.torch
        if self.packed is None:
            self.packed = t.empty(max(lib().cmoe_packed_bytes(self._h), 256), dtype=t.uint8, device=self.device)
        self.w.packed = None
        self._check(lib().cmoe_pack_weights(self._h, C.byref(self.w), _ptr(self.packed), self.packed.numel(),
                                            self._stream()), "cmoe_pack_weights")
        self.w.packed = _ptr(self.packed)

    def drop_canonical_bases(self):
        """Free w1_base / w2_base and pass NULL for them from now on: the packed buffer becomes the
        only resident copy of the bases.  Needs a packed copy; pack() is not possible afterwards."""
        if self.packed is None:
            raise ValueError("drop_canonical_bases needs the packed copy (pack=True)")
        self.torch.cuda.synchronize(self.device)
        self.w_t["w1_base"] = None
        self.w_t["w2_base"] = None
        self.w.w1_base = None
        self.w.w2_base = None

    def resident_weight_bytes(self):
        """Device bytes held for the layer's parameters (canonical tensors + packed buffer)."""
        n = sum(t.numel() * t.element_size() for t in self.w_t.values() if t is not None)
        return n + (self.packed.numel() if self.packed is not None else 0)

    def close(self):
        if self._h:
            lib().cmoe_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers ---------------------------------------------------------
    def _stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def _check(self, rc, where):
        if rc != OK:
            raise CmoeError(rc, where, lib().cmoe_last_hip_error(self._h))

    def _empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device=self.device)

    # -- the C ABI, one method per entry point ------------------------------
    def route(self, x):
        t = self.torch
        T, k = x.shape[0], self.cfg.top_k
        cid = self._empty((T,), t.int32)
        eidx = self._empty((T, k), t.int32)
        gate = self._empty((T, k), t.float32)
        self._check(lib().cmoe_route(self._h, C.byref(self.w), _ptr(x), T, _ptr(cid), _ptr(eidx), _ptr(gate),
                                     self._stream()), "cmoe_route")
        return cid, eidx, gate

    def permute(self, cluster_id):
        t = self.torch
        T = cluster_id.shape[0]
        perm = self._empty((T,), t.int32)
        inv = self._empty((T,), t.int32)
        offsets = self._empty((self.cfg.G + 1,), t.int32)
        self._check(lib().cmoe_permute(self._h, _ptr(cluster_id), T, _ptr(perm), _ptr(inv), _ptr(offsets),
                                       _ptr(self.ws), self.ws.numel(), self._stream()), "cmoe_permute")
        return perm, inv, offsets

    def permute_static(self, cluster_id, perm=None, inv=None, offsets=None):
        """cmoe_permute_static: no workspace argument, no allocation inside the call when the
        output tensors are passed in."""
        t = self.torch
        T = cluster_id.shape[0]
        perm = perm if perm is not None else self._empty((T,), t.int32)
        inv = inv if inv is not None else self._empty((T,), t.int32)
        offsets = offsets if offsets is not None else self._empty((self.cfg.G + 1,), t.int32)
        self._check(lib().cmoe_permute_static(self._h, _ptr(cluster_id), T, _ptr(perm), _ptr(inv), _ptr(offsets),
                                              self._stream()), "cmoe_permute_static")
        return perm, inv, offsets

    def ffn_forward(self, x, perm, offsets, expert_idx, gate):
        t = self.torch
        T = x.shape[0]
        yb = self._empty((T, self.cfg.d), t.float16)
        s = self._empty((T, self.cfg.top_k, self.cfg.r), t.float32)
        self._check(lib().cmoe_ffn_forward(self._h, C.byref(self.w), _ptr(x), T, _ptr(perm), _ptr(offsets),
                                           _ptr(expert_idx), _ptr(gate), _ptr(yb), _ptr(s), _ptr(self.ws),
                                           self.ws.numel(), self._stream()), "cmoe_ffn_forward")
        return yb, s

    def combine(self, yb, s, perm, inv_perm, offsets, expert_idx, gate):
        t = self.torch
        T = yb.shape[0]
        y = self._empty((T, self.cfg.d), t.float16)
        self._check(lib().cmoe_combine(self._h, C.byref(self.w), _ptr(yb), _ptr(s), _ptr(perm), _ptr(inv_perm),
                                       _ptr(offsets), _ptr(expert_idx), _ptr(gate), T, _ptr(y), _ptr(self.ws),
                                       self.ws.numel(), self._stream()), "cmoe_combine")
        return y

    def route_multi(self, x, top_g=1, temperature=1.0, scale_by_cluster_prob=False):
        """cmoe_route_multi: (cluster_id [T][top_g], expert_idx [T][top_g][k], gate [T][top_g][k])."""
        t = self.torch
        T, k = x.shape[0], self.cfg.top_k
        opt = RouteOptions(top_g, temperature, int(scale_by_cluster_prob))
        cid = self._empty((T, top_g), t.int32)
        eidx = self._empty((T, top_g, k), t.int32)
        gate = self._empty((T, top_g, k), t.float32)
        self._check(lib().cmoe_route_multi(self._h, C.byref(self.w), C.byref(opt), _ptr(x), T, _ptr(cid), _ptr(eidx),
                                           _ptr(gate), self._stream()), "cmoe_route_multi")
        return cid, eidx, gate

    def forward_multi(self, x, top_g=1, temperature=1.0, scale_by_cluster_prob=False, out=None):
        """cmoe_forward_multi; allocates its own workspace and outputs unless `out` (the dict an
        earlier call returned for the same T and top_g) is passed for reuse.  Returns a dict like forward(), with the
        routing outputs per (token, selected cluster) and perm / inv_perm over the virtual tokens."""
        t = self.torch
        T, k = x.shape[0], self.cfg.top_k
        opt = RouteOptions(top_g, temperature, int(scale_by_cluster_prob))
        nbytes = lib().cmoe_workspace_bytes_multi(self._h, T, top_g)
        if nbytes == 0:
            raise CmoeError(-1, "cmoe_workspace_bytes_multi")
        if out is not None:                      # buffers of an earlier call of the same shape
            o, ws = out, out["_workspace"]
            assert ws.numel() >= nbytes and o["y"].shape[0] == T and o["cluster_id"].shape[1] == top_g
        else:
            ws = self._empty((nbytes,), t.uint8)
            o = dict(y=self._empty((T, self.cfg.d), t.float16), cluster_id=self._empty((T, top_g), t.int32),
                     expert_idx=self._empty((T, top_g, k), t.int32), gate=self._empty((T, top_g, k), t.float32),
                     perm=self._empty((T * top_g,), t.int32), inv_perm=self._empty((T * top_g,), t.int32),
                     offsets=self._empty((self.cfg.G + 1,), t.int32))
        self._check(lib().cmoe_forward_multi(self._h, C.byref(self.w), C.byref(opt), _ptr(x), T, _ptr(o["y"]),
                                             _ptr(o["cluster_id"]), _ptr(o["expert_idx"]), _ptr(o["gate"]),
                                             _ptr(o["perm"]), _ptr(o["inv_perm"]), _ptr(o["offsets"]), _ptr(ws),
                                             nbytes, self._stream()), "cmoe_forward_multi")
        o["_workspace"] = ws
        return o

    def route_stats(self, x, perm, offsets, expert_idx, mu, cluster_act, cluster_idle, beta=0.05, lam=0.1):
        """Updates mu [E][d] f32, cluster_act [G] f32, cluster_idle [G] i32 in place; returns
        (expert_load [E] i32, cluster_load [G] i32, i_load [1] f32)."""
        t = self.torch
        T = x.shape[0]
        E = self.cfg.G * self.cfg.K
        load = self._empty((E,), t.int32)
        cload = self._empty((self.cfg.G,), t.int32)
        cv = self._empty((1,), t.float32)
        self._check(lib().cmoe_route_stats(self._h, _ptr(x), T, _ptr(perm), _ptr(offsets), _ptr(expert_idx),
                                           float(beta), float(lam), _ptr(mu), _ptr(cluster_act), _ptr(cluster_idle),
                                           _ptr(load), _ptr(cload), _ptr(cv), _ptr(self.ws), self.ws.numel(),
                                           self._stream()), "cmoe_route_stats")
        return load, cload, cv

    def backward(self, x, dy, expert_idx, gate):
        """Gradients of sum(dy * y) for the frozen selection (expert_idx, gate): dict of f32
        tensors dx, d_logits, d_router_expert, dw1_base, dw2_base, du1, dv1, du2, dv2.  The
        workspace (activations per token and per pair, transposed bases) is allocated on first
        use and kept."""
        t = self.torch
        c = self.cfg
        T = x.shape[0]
        E = c.G * c.K
        need = lib().cmoe_backward_workspace_bytes(self._h, T)
        if need == 0:
            raise CmoeError(-2, "cmoe_backward_workspace_bytes")
        if getattr(self, "bw_ws", None) is None or self.bw_ws.numel() < need:
            self.bw_ws = t.empty(need, dtype=t.uint8, device=self.device)
        f32 = t.float32
        out = dict(dx=self._empty((T, c.d), f32), d_logits=self._empty((T, c.top_k), f32),
                   d_router_expert=self._empty((E, c.d), f32), dw1_base=self._empty((c.G, c.d_ff, c.d), f32),
                   dw2_base=self._empty((c.G, c.d, c.d_ff), f32), du1=self._empty((E, c.r, c.d_ff), f32),
                   dv1=self._empty((E, c.r, c.d), f32), du2=self._empty((E, c.r, c.d), f32),
                   dv2=self._empty((E, c.r, c.d_ff), f32))
        g = Grads(**{n: _ptr(v) for n, v in out.items()})
        self._check(lib().cmoe_backward(self._h, C.byref(self.w), _ptr(x), _ptr(dy), T, _ptr(expert_idx), _ptr(gate),
                                        C.byref(g), _ptr(self.bw_ws), self.bw_ws.numel(), self._stream()),
                    "cmoe_backward")
        return out

    def forward_buffers(self, T):
        t = self.torch
        k = self.cfg.top_k
        return dict(y=self._empty((T, self.cfg.d), t.float16), cluster_id=self._empty((T,), t.int32),
                    expert_idx=self._empty((T, k), t.int32), gate=self._empty((T, k), t.float32),
                    perm=self._empty((T,), t.int32), inv_perm=self._empty((T,), t.int32),
                    offsets=self._empty((self.cfg.G + 1,), t.int32))

    def forward(self, x, out=None):
        T = x.shape[0]
        o = out if out is not None else self.forward_buffers(T)
        self._check(lib().cmoe_forward(self._h, C.byref(self.w), _ptr(x), T, _ptr(o["y"]), _ptr(o["cluster_id"]),
                                       _ptr(o["expert_idx"]), _ptr(o["gate"]), _ptr(o["perm"]), _ptr(o["inv_perm"]),
                                       _ptr(o["offsets"]), _ptr(self.ws), self.ws.numel(), self._stream()),
                    "cmoe_forward")
        return o

    # -- per-kernel timing (HIP events recorded by the library on the launch stream) ------
    def timing_enable(self, on: bool):
        self._check(lib().cmoe_timing_enable(self._h, int(on)), "cmoe_timing_enable")

    def timing_read(self):
        n = 16
        ms = (C.c_double * n)()
        cnt = (C.c_int32 * n)()
        used = lib().cmoe_timing_read(self._h, ms, cnt, n)
        if used < 0:
            raise CmoeError(used, "cmoe_timing_read", lib().cmoe_last_hip_error(self._h))
        return {lib().cmoe_timing_name(i).decode(): (ms[i], cnt[i]) for i in range(used)}
