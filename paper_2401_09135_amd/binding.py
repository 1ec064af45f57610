"""ctypes binding with the same names as the C ABI in include/als.h (argument marshalling
only).  torch supplies device buffers and streams."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

ALS_DTYPE_F32, ALS_DTYPE_BF16 = 0, 1
VEC = dict(theta=0, momentum=1, delta=2, worker_theta=3, worker_start=4, adam_m=5, adam_v=6, grad=7)

lib_path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libals.so")
if not os.path.exists(lib_path):
    raise ImportError(f"{lib_path} is missing: build it with `python paper_2401_09135_amd/build.py` "
                      "(there is no CPU fallback)")



def _load():
    # libals.so and torch must share ONE HIP runtime in the process (device pointers and
    # streams cross between them): load the runtime torch ships first, so that the
    # library's dependency on libamdhip64 resolves to it by soname.
    import torch
    rt = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(rt):
        C.CDLL(rt, mode=C.RTLD_GLOBAL)
    return C.CDLL(lib_path)


lib = _load()


class AlsError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("seq_len", C.c_int32),
                ("batch", C.c_int32), ("dtype", C.c_int32), ("n_workers", C.c_int32),
                ("dn_N", C.c_int32), ("max_local_steps", C.c_int32), ("flags", C.c_int32),
                ("head_dim", C.c_int32), ("norm_kind", C.c_int32),
                ("adam_beta1", C.c_double), ("adam_beta2", C.c_double), ("adam_eps", C.c_double),
                ("weight_decay", C.c_double), ("outer_lr", C.c_double), ("outer_beta", C.c_double),
                ("dn_c", C.c_double), ("norm_eps", C.c_double)]

    @classmethod
    def from_workload(cls, w: dict, flags: int = 0, max_local_steps: int | None = None) -> "Config":
        return cls(n_layers=w["L"], d_model=w["d"], n_heads=w["h"], d_ff=w["ff"], vocab=w["V"],
                   seq_len=w["S"], batch=w["B"], dtype=ALS_DTYPE_BF16 if w["dtype"] == "bf16" else ALS_DTYPE_F32,
                   n_workers=w["k"], dn_N=w["N"], max_local_steps=max_local_steps or w["H"], flags=flags,
                   head_dim=int(w.get("dh", 0)), norm_kind={"rms": 0, "layer": 1}[w.get("norm", "rms")],
                   adam_beta1=w["beta1"], adam_beta2=w["beta2"], adam_eps=w["adam_eps"],
                   weight_decay=w["wd"], outer_lr=w["outer_lr"], outer_beta=w["outer_beta"],
                   dn_c=w["dn_c"], norm_eps=w["norm_eps"])


class OuterRule(C.Structure):
    _fields_ = [("kind", C.c_int32), ("staleness_threshold", C.c_int32), ("poly_exponent", C.c_double),
                ("dc_lambda", C.c_double)]


RULE_DN, RULE_BUFFER = 0, 1
_P = C.c_void_p
lib.als_last_error.restype = C.c_char_p
lib.als_param_count.restype = C.c_int64
lib.als_param_count.argtypes = [C.POINTER(Config)]
lib.als_param_count_decayed.restype = C.c_int64
lib.als_param_count_decayed.argtypes = [C.POINTER(Config)]
lib.als_param_offsets.argtypes = [C.POINTER(Config), C.POINTER(C.c_int64), C.c_int]
lib.als_arena_bytes.restype = C.c_size_t
lib.als_arena_bytes.argtypes = [C.POINTER(Config)]
lib.als_init.argtypes = [C.POINTER(Config), _P, C.c_size_t, _P, C.POINTER(_P), C.c_int, C.POINTER(_P)]
lib.als_destroy.argtypes = [_P]
lib.als_worker_local_steps.argtypes = [_P, C.c_int, C.c_int, _P, _P, _P]
lib.als_outer_apply_dn.argtypes = [_P, _P, C.c_int, C.c_int]
lib.als_outer_apply_rule.argtypes = [_P, _P, C.c_int, C.c_int, C.POINTER(OuterRule)]
lib.als_worker_staleness.restype = C.c_int64
lib.als_worker_staleness.argtypes = [_P, C.c_int]
lib.als_dylu_schedule.argtypes = [_P, C.c_int, C.c_int, C.c_double, C.c_int, _P, _P, _P, _P]
lib.als_get_vector.argtypes = [_P, C.c_int, C.c_int, _P]
lib.als_set_vector.argtypes = [_P, C.c_int, C.c_int, _P]
lib.als_sync.argtypes = [_P, C.c_int]
lib.als_get_losses.argtypes = [_P, C.c_int, _P, C.c_int]
lib.als_server_t.restype = C.c_int64
lib.als_server_t.argtypes = [_P]
lib.als_worker_adam_steps.restype = C.c_int64
lib.als_worker_adam_steps.argtypes = [_P, C.c_int]
lib.als_worker_loss_grad.argtypes = [_P, C.c_int, _P, _P]
lib.als_k_dn_group.argtypes = [_P, _P, _P, C.POINTER(_P), C.POINTER(_P), C.POINTER(_P), C.c_int, C.c_int64,
                               C.c_int, C.c_int64, C.c_double, C.c_double, C.c_double, C.c_int, _P]
lib.als_k_adamw.argtypes = [_P, _P, _P, _P, _P, C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_double,
                            C.c_double, C.c_double, C.c_double, _P]
lib.als_k_gemm.argtypes = [_P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P,
                           C.c_size_t, _P]
lib.als_k_attention_fwd.argtypes = [_P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P]
lib.als_k_attention_bwd.argtypes = [_P, _P, _P, _P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P]


lib.als_prof_enable.argtypes = [C.c_int]
lib.als_prof_collect.argtypes = [C.c_int, _P, _P, _P, _P]
lib.als_prof_kernel_name.argtypes = [C.c_int, C.c_char_p, C.c_int]
lib.als_k_set_gemm_tile.argtypes = [C.c_int, C.c_int, C.c_int]


def prof_enable(on) -> None:
    """True / 1: time every MFMA GEMM launch; n > 1: every n-th; False / 0: off."""
    _check(lib.als_prof_enable(int(on)))


def set_gemm_tile(bm: int, bn: int, nbuf: int) -> None:
    """Tuning hook: force the MFMA GEMM tile (0, 0, 0 = automatic) wherever the shape allows it."""
    _check(lib.als_k_set_gemm_tile(bm, bn, nbuf))


def prof_collect(max_entries: int = 64):
    """[(kernel name, launches, total ms, total flops)] of the MFMA GEMM launches since enable."""
    ids = np.zeros(max_entries, np.int32)
    n_l = np.zeros(max_entries, np.int64)
    ms = np.zeros(max_entries, np.float64)
    fl = np.zeros(max_entries, np.float64)
    n = lib.als_prof_collect(max_entries, _np_ptr(ids), _np_ptr(n_l), _np_ptr(ms), _np_ptr(fl))
    if n < 0:
        _check(n)
    out = []
    for i in range(n):
        buf = C.create_string_buffer(160)
        _check(lib.als_prof_kernel_name(int(ids[i]), buf, 160))
        out.append((buf.value.decode(), int(n_l[i]), float(ms[i]), float(fl[i])))
    return out


def _check(rc: int) -> None:
    if rc != 0:
        raise AlsError(f"als error {rc}: {lib.als_last_error().decode()}")


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(_P)


def param_count(cfg: Config) -> int:
    return int(lib.als_param_count(C.byref(cfg)))


def param_count_decayed(cfg: Config) -> int:
    return int(lib.als_param_count_decayed(C.byref(cfg)))


def param_offsets(cfg: Config) -> np.ndarray:
    n = 6 * cfg.n_layers + 4
    out = (C.c_int64 * n)()
    rc = lib.als_param_offsets(C.byref(cfg), out, n)
    if rc < 0:
        _check(rc)
    return np.array(out[:rc], dtype=np.int64)


def dylu_schedule(speeds, H_max: int, tau_grace: float = 0.0, n_events: int = 0):
    """Returns (H[k] int32, ev_worker, ev_time, ev_group_end)."""
    v = np.ascontiguousarray(speeds, dtype=np.float64)
    k = int(v.size)
    H = np.zeros(max(k, 1), dtype=np.int32)
    ew = np.zeros(max(n_events, 1), dtype=np.int32)
    et = np.zeros(max(n_events, 1), dtype=np.float64)
    eg = np.zeros(max(n_events, 1), dtype=np.int32)
    _check(lib.als_dylu_schedule(_np_ptr(v), k, int(H_max), float(tau_grace), int(n_events), _np_ptr(H),
                                 _np_ptr(ew) if n_events else None, _np_ptr(et), _np_ptr(eg)))
    return H[:k], ew[:n_events], et[:n_events], eg[:n_events]


lib.als_lr_schedule.argtypes = [C.c_int64, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_double, _P]
lib.als_shard_sample.argtypes = [_P, _P, C.c_int, C.c_double, _P, _P]


def lr_schedule(t0: int, n: int, t_warmup: int, T: int, eta_max: float, eta_min: float) -> np.ndarray:
    out = np.zeros(max(n, 1), dtype=np.float32)
    _check(lib.als_lr_schedule(int(t0), int(n), int(t_warmup), int(T), float(eta_max), float(eta_min), _np_ptr(out)))
    return out[:n]


def shard_sample(sizes, learned, u: float):
    """Returns (probabilities[k], chosen shard)."""
    s = np.ascontiguousarray(sizes, dtype=np.float64)
    n = np.ascontiguousarray(learned, dtype=np.float64)
    if s.shape != n.shape:
        raise AlsError("sizes and learned must have the same length")
    p = np.zeros(max(s.size, 1), dtype=np.float64)
    pick = np.zeros(1, dtype=np.int32)
    _check(lib.als_shard_sample(_np_ptr(s), _np_ptr(n), int(s.size), float(u), _np_ptr(p), _np_ptr(pick)))
    return p[:s.size], int(pick[0])


def _stream_handle(stream) -> int:
    return 0 if stream is None else int(stream.cuda_stream)


class Context:
    """Owns the arena (a torch uint8 tensor) and the worker streams; wraps als_ctx."""

    def __init__(self, cfg: Config, theta0: np.ndarray, n_streams: int | None = None, device="cuda:0",
                 streams=None):
        """streams: optional list of torch streams to run the workers on (worker i uses stream
        i mod len(streams)); by default one new stream per worker."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.P = param_count(cfg)
        if self.P == 0:
            raise AlsError("invalid configuration: " + lib.als_last_error().decode())
        theta0 = np.ascontiguousarray(theta0, dtype=np.float32)
        if theta0.size != self.P:
            raise AlsError(f"theta0 has {theta0.size} elements, the configuration needs {self.P}")
        nbytes = int(lib.als_arena_bytes(C.byref(cfg)))
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        if streams is not None:
            self.streams, n_streams = list(streams), len(streams)
        else:
            n_streams = cfg.n_workers if n_streams is None else n_streams
            self.streams = [torch.cuda.Stream(device=self.device) for _ in range(n_streams)]
        handles = (_P * n_streams)(*[_stream_handle(s) for s in self.streams])
        torch.cuda.synchronize()
        self._ctx = _P()
        _check(lib.als_init(C.byref(cfg), base, nbytes, _np_ptr(theta0), handles, n_streams, C.byref(self._ctx)))
        self._keep = []

    def close(self):
        if getattr(self, "_ctx", None):
            lib.als_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def worker_local_steps(self, worker: int, tokens_dev, lr, want_losses: bool = False):
        """tokens_dev: torch int32 [n,B,S+1] on the device; lr: n floats."""
        n = int(tokens_dev.shape[0])
        assert tokens_dev.dtype == self.torch.int32 and tokens_dev.is_contiguous()
        lr = np.ascontiguousarray(np.broadcast_to(np.asarray(lr, dtype=np.float32), (n,)))
        out = np.zeros(n, dtype=np.float32) if want_losses else None
        self._keep.append(tokens_dev)
        _check(lib.als_worker_local_steps(self._ctx, worker, n, tokens_dev.data_ptr(), _np_ptr(lr),
                                          _np_ptr(out) if want_losses else None))
        return out

    def worker_loss_grad(self, worker: int, tokens_dev):
        out = np.zeros(1, dtype=np.float32)
        _check(lib.als_worker_loss_grad(self._ctx, worker, tokens_dev.data_ptr(), _np_ptr(out)))
        return float(out[0]), self.get_vector("grad", worker)

    def outer_apply_dn(self, workers, restart: bool = True):
        w = np.ascontiguousarray(workers, dtype=np.int32)
        _check(lib.als_outer_apply_dn(self._ctx, _np_ptr(w), int(w.size), 1 if restart else 0))

    def outer_apply_rule(self, workers, restart: bool = True, kind: int = RULE_DN, poly_exponent: float = 0.0,
                         staleness_threshold: int = -1, dc_lambda: float = 0.0):
        w = np.ascontiguousarray(workers, dtype=np.int32)
        rule = OuterRule(kind=kind, staleness_threshold=staleness_threshold, poly_exponent=poly_exponent,
                         dc_lambda=dc_lambda)
        _check(lib.als_outer_apply_rule(self._ctx, _np_ptr(w), int(w.size), 1 if restart else 0, C.byref(rule)))

    def staleness(self, worker: int) -> int:
        return int(lib.als_worker_staleness(self._ctx, worker))

    def get_vector(self, which: str, worker: int = 0) -> np.ndarray:
        out = np.empty(self.P, dtype=np.float32)
        _check(lib.als_get_vector(self._ctx, VEC[which], worker, _np_ptr(out)))
        return out

    def set_vector(self, which: str, worker: int, value: np.ndarray):
        v = np.ascontiguousarray(value, dtype=np.float32)
        assert v.size == self.P
        _check(lib.als_set_vector(self._ctx, VEC[which], worker, _np_ptr(v)))

    def sync(self, worker: int = -1):
        _check(lib.als_sync(self._ctx, worker))
        if worker < 0:
            self._keep.clear()

    def get_losses(self, worker: int, n: int) -> np.ndarray:
        out = np.zeros(n, dtype=np.float32)
        _check(lib.als_get_losses(self._ctx, worker, _np_ptr(out), n))
        return out

    @property
    def server_t(self) -> int:
        return int(lib.als_server_t(self._ctx))

    def adam_steps(self, worker: int) -> int:
        return int(lib.als_worker_adam_steps(self._ctx, worker))


# ---- stand-alone kernels on torch tensors ---------------------------------------------------
def _ptr_array(tensors):
    return (_P * len(tensors))(*[(t.data_ptr() if t is not None else None) for t in tensors])


def k_dn_group(theta, m, delta, theta_start, theta_worker, bf16_worker, N, t0, outer_lr, beta, c=0.0,
               restart=False, stream=None):
    G = len(theta_start)
    P = theta.numel()
    _check(lib.als_k_dn_group(theta.data_ptr(), m.data_ptr(), delta.data_ptr(), _ptr_array(theta_start),
                              _ptr_array(theta_worker), _ptr_array(bf16_worker) if bf16_worker else None,
                              G, P, int(N), int(t0), float(outer_lr), float(beta), float(c), int(bool(restart)),
                              _stream_handle(stream)))


def k_adamw(theta, grad, m, v, bf16_out, P_decay, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.1,
            stream=None):
    _check(lib.als_k_adamw(theta.data_ptr(), grad.data_ptr(), m.data_ptr(), v.data_ptr(),
                           bf16_out.data_ptr() if bf16_out is not None else None, theta.numel(),
                           int(P_decay), int(step), float(lr), float(beta1), float(beta2), float(eps),
                           float(wd), _stream_handle(stream)))


def _dt(t):
    import torch
    return ALS_DTYPE_BF16 if t.dtype == torch.bfloat16 else ALS_DTYPE_F32


def k_gemm(A, B, C_out, M, N, K, a_layout=0, b_layout=0, use_mfma=False, ws=None, stream=None):
    _check(lib.als_k_gemm(A.data_ptr(), B.data_ptr(), C_out.data_ptr(), M, N, K, a_layout, b_layout,
                          _dt(A), _dt(C_out), int(bool(use_mfma)), ws.data_ptr() if ws is not None else None,
                          ws.numel() * ws.element_size() if ws is not None else 0, _stream_handle(stream)))


STATIC_WS_BYTES = 64 << 20
lib.als_k_gemm_static_ws.argtypes = [_P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P]


def k_gemm_static_ws(A, B, C_out, M, N, K, a_layout=1, b_layout=0, stream=None):
    """als_k_gemm on the MFMA path with the split-K partials in the library's static device array."""
    _check(lib.als_k_gemm_static_ws(A.data_ptr(), B.data_ptr(), C_out.data_ptr(), M, N, K, a_layout, b_layout,
                                    _dt(C_out), _stream_handle(stream)))


lib.als_k_gemm_dw_grouped_ws_bytes.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
lib.als_k_gemm_dw_grouped_ws_bytes.restype = C.c_size_t
lib.als_k_gemm_dw_grouped.argtypes = [C.c_int, C.POINTER(_P), C.POINTER(_P), C.POINTER(_P), C.POINTER(C.c_int),
                                      C.POINTER(C.c_int), C.c_int, _P, C.c_size_t, _P]


def k_gemm_dw_grouped_ws_bytes(Ms, Ns) -> int:
    n = len(Ms)
    return int(lib.als_k_gemm_dw_grouped_ws_bytes(n, (C.c_int * n)(*Ms), (C.c_int * n)(*Ns)))


def k_gemm_dw_grouped(Xs, dYs, Cs, K, ws, stream=None):
    """als_k_gemm_dw_grouped: Cs[i] = Xs[i]^T dYs[i] for every i in one launch (Xs[i] [K, M_i], dYs[i]
    [K, N_i] bf16, Cs[i] [M_i, N_i] fp32); ws: uint8 device tensor of k_gemm_dw_grouped_ws_bytes."""
    n = len(Xs)
    Ms = [x.shape[1] for x in Xs]
    Ns = [y.shape[1] for y in dYs]
    _check(lib.als_k_gemm_dw_grouped(n, _ptr_array(Xs), _ptr_array(dYs), _ptr_array(Cs), (C.c_int * n)(*Ms),
                                     (C.c_int * n)(*Ns), int(K), ws.data_ptr(), ws.numel() * ws.element_size(),
                                     _stream_handle(stream)))


lib.als_k_gemm_ex.argtypes = [_P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                              _P, _P, _P, _P, C.c_size_t, _P]


def k_gemm_ex(A, B, C_out, M, N, K, a_layout=0, b_layout=0, use_mfma=False, epi=0, R=None, C2=None, U=None,
              ws=None, stream=None):
    p = lambda t: t.data_ptr() if t is not None else None
    _check(lib.als_k_gemm_ex(A.data_ptr(), B.data_ptr(), C_out.data_ptr(), M, N, K, a_layout, b_layout, _dt(A),
                             _dt(C_out), int(bool(use_mfma)), int(epi), p(R), p(C2), p(U), p(ws),
                             ws.numel() * ws.element_size() if ws is not None else 0, _stream_handle(stream)))


def k_attention_fwd(qkv, o, lse, B, S, h, dh, use_mfma=False, stream=None):
    _check(lib.als_k_attention_fwd(qkv.data_ptr(), o.data_ptr(), lse.data_ptr(), B, S, h, dh, _dt(qkv),
                                   int(bool(use_mfma)), _stream_handle(stream)))


def k_attention_bwd(qkv, o, d_o, lse, dscratch, dqkv, B, S, h, dh, use_mfma=False, stream=None):
    _check(lib.als_k_attention_bwd(qkv.data_ptr(), o.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
                                   dscratch.data_ptr(), dqkv.data_ptr(), B, S, h, dh, _dt(qkv),
                                   int(bool(use_mfma)), _stream_handle(stream)))
