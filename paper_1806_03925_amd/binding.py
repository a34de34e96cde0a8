"""ctypes binding of libgear.so: the same calls as include/gear.h, argument marshalling only.

PyTorch appears here for device memory (`tensor.data_ptr()`) and streams; every step of the
path runs inside the library's HIP kernels.  There is no fallback: if the library is missing
the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

GEAR_MAX_LAYERS = 8
GEAR_OK, GEAR_ERR_INVALID, GEAR_ERR_RANGE, GEAR_ERR_CAPACITY, GEAR_ERR_HIP = range(5)
GEAR_F32, GEAR_BF16 = 0, 1
DTYPE_CODE = {"f32": GEAR_F32, "bf16": GEAR_BF16}
TORCH_DTYPE = {GEAR_F32: torch.float32, GEAR_BF16: torch.bfloat16}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgear.so")

EXPORTS = (
    "gear_workspace_bytes", "gear_mlp_param_count", "gear_mlp_param_offset", "gear_workspace_region",
    "gear_fill_normal", "gear_init_tables", "gear_step", "gear_step_static", "gear_step_adam", "gear_refresh_dfv", "gear_expired_ids", "gear_stamp_dfv",
    "gear_refresh_dfv_n", "gear_stamp_dfv_n",
    "gear_dense_workspace_bytes", "gear_dense_infer", "gear_dense_backward", "gear_dense_backward_n", "gear_group_ids",
    "gear_gemm", "gear_profile_create", "gear_profile_destroy", "gear_profile_count", "gear_profile_span",
    "gear_debug_fail_launch", "gear_debug_helper_idle", "gear_status_string",
)


class gear_config(C.Structure):
    _fields_ = [("n_users", C.c_int64), ("n_urls", C.c_int64), ("n_images", C.c_int64),
                ("emb_dim", C.c_int32), ("dfv_dim", C.c_int32), ("n_layers", C.c_int32),
                ("layer_out", C.c_int32 * GEAR_MAX_LAYERS),
                ("emb_dtype", C.c_int32), ("dfv_dtype", C.c_int32), ("mlp_dtype", C.c_int32),
                ("max_batch", C.c_int32), ("max_nnz", C.c_int32),
                ("seed", C.c_uint64), ("emb_init_std", C.c_float)]


class gear_tables(C.Structure):
    _fields_ = [("user_emb", C.c_void_p), ("url_emb", C.c_void_p), ("mlp_params", C.c_void_p)]


class gear_batch(C.Structure):
    _fields_ = [("B", C.c_int32), ("nnz", C.c_int32), ("user_id", C.c_void_p), ("url_id", C.c_void_p),
                ("img_off", C.c_void_p), ("img_id", C.c_void_p), ("label", C.c_void_p)]


class gear_adam(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("t", C.c_int32),
                ("user_m", C.c_void_p), ("user_v", C.c_void_p), ("url_m", C.c_void_p), ("url_v", C.c_void_p),
                ("mlp_m", C.c_void_p), ("mlp_v", C.c_void_p)]


class gear_dense_config(C.Structure):
    _fields_ = [("n_images", C.c_int64), ("raw_dim", C.c_int32), ("dfv_dim", C.c_int32), ("dfv_dtype", C.c_int32),
                ("max_rows", C.c_int32)]


class gear_step_out(C.Structure):
    _fields_ = [("loss", C.c_void_p), ("n_ready", C.c_void_p), ("ready_ids", C.c_void_p),
                ("ready_grads", C.c_void_p), ("ready_cap", C.c_int32), ("status", C.c_void_p),
                ("dbg_img_unique", C.c_void_p), ("dbg_img_segoff", C.c_void_p),
                ("dbg_img_perm", C.c_void_p), ("dbg_n_img_unique", C.c_void_p), ("profile", C.c_void_p),
                ("one_stream", C.c_int32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1806_03925_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    cfgp = C.POINTER(gear_config)
    lib.gear_workspace_bytes.restype = C.c_size_t
    lib.gear_workspace_bytes.argtypes = [cfgp]
    lib.gear_mlp_param_count.restype = C.c_int64
    lib.gear_mlp_param_count.argtypes = [cfgp]
    lib.gear_mlp_param_offset.restype = C.c_int64
    lib.gear_mlp_param_offset.argtypes = [cfgp, C.c_int32, C.c_int32]
    lib.gear_workspace_region.restype = C.c_int
    lib.gear_workspace_region.argtypes = [cfgp, C.c_char_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.gear_fill_normal.restype = C.c_int
    lib.gear_fill_normal.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32,
                                     C.c_float, C.c_void_p]
    lib.gear_init_tables.restype = C.c_int
    lib.gear_init_tables.argtypes = [cfgp, C.POINTER(gear_tables), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gear_step.restype = C.c_int
    lib.gear_step.argtypes = [cfgp, C.POINTER(gear_batch), C.POINTER(gear_tables), C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_size_t,
                              C.POINTER(gear_step_out), C.c_void_p]
    lib.gear_step_static.restype = C.c_int
    lib.gear_step_static.argtypes = [cfgp, C.POINTER(gear_batch), C.POINTER(gear_tables), C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_float, C.POINTER(gear_step_out), C.c_void_p]
    lib.gear_step_adam.restype = C.c_int
    lib.gear_step_adam.argtypes = [cfgp, C.POINTER(gear_batch), C.POINTER(gear_tables), C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int32, C.c_float, C.POINTER(gear_adam), C.c_void_p, C.c_size_t,
                                   C.POINTER(gear_step_out), C.c_void_p]
    lib.gear_refresh_dfv.restype = C.c_int
    lib.gear_refresh_dfv.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.gear_expired_ids.restype = C.c_int
    lib.gear_expired_ids.argtypes = [cfgp, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gear_stamp_dfv.restype = C.c_int
    lib.gear_stamp_dfv.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    dcp = C.POINTER(gear_dense_config)
    lib.gear_dense_workspace_bytes.restype = C.c_size_t
    lib.gear_dense_workspace_bytes.argtypes = [dcp]
    lib.gear_dense_infer.restype = C.c_int
    lib.gear_dense_infer.argtypes = [dcp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p, C.c_void_p]
    lib.gear_dense_backward.restype = C.c_int
    lib.gear_dense_backward.argtypes = [dcp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_float,
                                        C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.gear_dense_backward_n.restype = C.c_int
    lib.gear_dense_backward_n.argtypes = [dcp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                          C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.gear_refresh_dfv_n.restype = C.c_int
    lib.gear_refresh_dfv_n.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                       C.c_void_p]
    lib.gear_stamp_dfv_n.restype = C.c_int
    lib.gear_stamp_dfv_n.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                     C.c_void_p]
    lib.gear_group_ids.restype = C.c_int
    lib.gear_group_ids.argtypes = [cfgp, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gear_gemm.restype = C.c_int
    lib.gear_gemm.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                              C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                              C.c_void_p]
    lib.gear_profile_create.restype = C.c_void_p
    lib.gear_profile_create.argtypes = []
    lib.gear_profile_destroy.restype = None
    lib.gear_profile_destroy.argtypes = [C.c_void_p]
    lib.gear_profile_count.restype = C.c_int32
    lib.gear_profile_count.argtypes = [C.c_void_p]
    lib.gear_profile_span.restype = C.c_int
    lib.gear_profile_span.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_float)]
    lib.gear_debug_fail_launch.restype = None
    lib.gear_debug_fail_launch.argtypes = [C.c_int32]
    lib.gear_debug_helper_idle.restype = C.c_int32
    lib.gear_debug_helper_idle.argtypes = []
    lib.gear_status_string.restype = C.c_char_p
    lib.gear_status_string.argtypes = [C.c_int]
    return lib


lib = _load()


class GearError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib.gear_status_string(code).decode()} (status {code})")


def _check(code: int, where: str) -> None:
    if code != GEAR_OK:
        raise GearError(code, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_config(n_users, n_urls, n_images, emb_dim, dfv_dim, layers: Sequence[int], emb_dtype="f32",
                dfv_dtype="f32", mlp_dtype="f32", max_batch=1, max_nnz=1, seed=0, emb_init_std=0.01) -> gear_config:
    cfg = gear_config()
    cfg.n_users, cfg.n_urls, cfg.n_images = int(n_users), int(n_urls), int(n_images)
    cfg.emb_dim, cfg.dfv_dim, cfg.n_layers = int(emb_dim), int(dfv_dim), len(layers)
    for i in range(GEAR_MAX_LAYERS):
        cfg.layer_out[i] = int(layers[i]) if i < len(layers) else 0
    cfg.emb_dtype, cfg.dfv_dtype, cfg.mlp_dtype = DTYPE_CODE[emb_dtype], DTYPE_CODE[dfv_dtype], DTYPE_CODE[mlp_dtype]
    cfg.max_batch, cfg.max_nnz = int(max_batch), int(max_nnz)
    cfg.seed, cfg.emb_init_std = int(seed), float(emb_init_std)
    return cfg


def gear_workspace_bytes(cfg: gear_config) -> int:
    return int(lib.gear_workspace_bytes(C.byref(cfg)))


def gear_mlp_param_count(cfg: gear_config) -> int:
    return int(lib.gear_mlp_param_count(C.byref(cfg)))


def gear_mlp_param_offset(cfg: gear_config, layer: int, which: int) -> int:
    return int(lib.gear_mlp_param_offset(C.byref(cfg), layer, which))


def gear_workspace_region(cfg: gear_config, name: str):
    off, size = C.c_size_t(), C.c_size_t()
    _check(lib.gear_workspace_region(C.byref(cfg), name.encode(), C.byref(off), C.byref(size)),
           "gear_workspace_region")
    return off.value, size.value


def gear_debug_fail_launch(nth: int) -> None:
    lib.gear_debug_fail_launch(int(nth))


def gear_debug_helper_idle() -> int:
    return int(lib.gear_debug_helper_idle())


def gear_fill_normal(dst: torch.Tensor, n_rows: int, dim: int, seed: int, stream_id: int, std: float) -> None:
    code = GEAR_BF16 if dst.dtype == torch.bfloat16 else GEAR_F32
    _check(lib.gear_fill_normal(dst.data_ptr(), code, n_rows, dim, seed, stream_id, std, _stream()),
           "gear_fill_normal")


@dataclass
class DeviceBatch:
    """A page-view batch resident in device memory (int32 ids / offsets, float32 labels)."""
    user_id: torch.Tensor
    url_id: torch.Tensor
    img_off: torch.Tensor
    img_id: torch.Tensor
    label: torch.Tensor

    @property
    def B(self) -> int:
        return int(self.user_id.numel())

    @property
    def nnz(self) -> int:
        return int(self.img_id.numel())

    @staticmethod
    def from_host(batch, device="cuda") -> "DeviceBatch":
        put = lambda a: torch.from_numpy(a).to(device)
        return DeviceBatch(put(batch.user_id), put(batch.url_id), put(batch.img_off), put(batch.img_id),
                           put(batch.label))

    def as_struct(self) -> gear_batch:
        return gear_batch(self.B, self.nnz, _ptr(self.user_id), _ptr(self.url_id), _ptr(self.img_off),
                          _ptr(self.img_id) if self.nnz else None, _ptr(self.label))


class GearState:
    """Caller-owned device arrays of one Fastgear/Slowgear pair, allocated through PyTorch."""

    def __init__(self, cfg: gear_config, device="cuda", ready_cap: Optional[int] = None, debug: bool = False):
        self.cfg = cfg
        dev = torch.device(device)
        et, dt = TORCH_DTYPE[cfg.emb_dtype], TORCH_DTYPE[cfg.dfv_dtype]
        self.user_emb = torch.empty((cfg.n_users, cfg.emb_dim), dtype=et, device=dev)
        self.url_emb = torch.empty((cfg.n_urls, cfg.emb_dim), dtype=et, device=dev)
        self.mlp_params = torch.empty(gear_mlp_param_count(cfg), dtype=torch.float32, device=dev)
        self.dfv_cache = torch.zeros((cfg.n_images, cfg.dfv_dim), dtype=dt, device=dev)
        self.grad_accum = torch.empty((cfg.n_images, cfg.dfv_dim), dtype=torch.float32, device=dev)
        self.counts = torch.empty(cfg.n_images, dtype=torch.int32, device=dev)
        self.workspace = torch.empty(gear_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
        self.ready_cap = cfg.max_nnz if ready_cap is None else int(ready_cap)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.n_ready = torch.zeros(1, dtype=torch.int32, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ready_ids = torch.empty(max(self.ready_cap, 1), dtype=torch.int32, device=dev)
        self.ready_grads = torch.empty((max(self.ready_cap, 1), cfg.dfv_dim), dtype=torch.float32, device=dev)
        self.profile = None          # a GearProfile to time every launch of the next steps
        self.one_stream = False      # True: the next steps launch every kernel on the current stream
        self.dbg = None
        if debug:
            n = cfg.max_nnz
            self.dbg = (torch.zeros(n, dtype=torch.int32, device=dev), torch.zeros(n + 1, dtype=torch.int32, device=dev),
                        torch.zeros(n, dtype=torch.int32, device=dev), torch.zeros(1, dtype=torch.int32, device=dev))

    def tables(self) -> gear_tables:
        return gear_tables(_ptr(self.user_emb), _ptr(self.url_emb), _ptr(self.mlp_params))

    def step_out(self) -> gear_step_out:
        d = self.dbg or (None, None, None, None)
        return gear_step_out(_ptr(self.loss), _ptr(self.n_ready), _ptr(self.ready_ids), _ptr(self.ready_grads),
                             self.ready_cap, _ptr(self.status), _ptr(d[0]), _ptr(d[1]), _ptr(d[2]), _ptr(d[3]),
                             self.profile.handle if self.profile is not None else None, 1 if self.one_stream else 0)

    def layer_params(self, layer: int):
        """Views of W_l [out x in] and b_l [out] inside mlp_params."""
        cfg = self.cfg
        fan_in = 2 * cfg.emb_dim + cfg.dfv_dim if layer == 0 else cfg.layer_out[layer - 1]
        out = cfg.layer_out[layer]
        wo, bo = gear_mlp_param_offset(cfg, layer, 0), gear_mlp_param_offset(cfg, layer, 1)
        return self.mlp_params[wo:wo + out * fan_in].view(out, fan_in), self.mlp_params[bo:bo + out]

    def region(self, name: str, B: int) -> torch.Tensor:
        """An intermediate of the last step, read out of the workspace (tests only)."""
        if name == "dx":
            return torch.cat([self.region("dx_emb", B), self.region("dx_dfv", B).float()], dim=1)
        off, size = gear_workspace_region(self.cfg, name)
        raw = self.workspace[off:off + size]
        F = 2 * self.cfg.emb_dim + self.cfg.dfv_dim
        d, D = self.cfg.emb_dim, self.cfg.dfv_dim
        if name == "x":
            return raw.view(TORCH_DTYPE[self.cfg.mlp_dtype])[:B * F].view(B, F)
        if name == "dx_emb":
            return raw.view(torch.float32)[:B * 2 * d].view(B, 2 * d)
        if name == "dx_dfv":
            return raw.view(TORCH_DTYPE[self.cfg.mlp_dtype])[:B * D].view(B, D)
        if name[0] == "h":
            H = self.cfg.layer_out[int(name[1:])]
            return raw.view(TORCH_DTYPE[self.cfg.mlp_dtype])[:B * H].view(B, H)
        return raw.view(torch.float32)[:B]


def gear_gemm(A: torch.Tensor, B: torch.Tensor, form: int, epilogue: int = 2, bias: Optional[torch.Tensor] = None,
              aux: Optional[torch.Tensor] = None, splits: int = 1) -> torch.Tensor:
    """form 0: A [M x K], B [N x K] -> A B^T (epilogue 0/1 in A's dtype, 2 in fp32);
    form 1: A [K x M], B [K x N] -> A^T B in fp32, contracted in `splits` ranges of K."""
    code = GEAR_BF16 if A.dtype == torch.bfloat16 else GEAR_F32
    dev = A.device
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    if form == 0:
        M, K = A.shape
        N = B.shape[0]
        out = torch.empty((M, N), dtype=torch.float32 if epilogue == 2 else A.dtype, device=dev)
        partial = None
    else:
        K, M = A.shape
        N = B.shape[1]
        out = torch.empty((M, N), dtype=torch.float32, device=dev)
        partial = torch.empty((splits, M, N), dtype=torch.float32, device=dev)
    _check(lib.gear_gemm(code, form, _ptr(A), _ptr(B), M, N, K, epilogue, _ptr(bias), _ptr(aux), _ptr(out), splits,
                         _ptr(partial), _ptr(status), _stream()), "gear_gemm")
    return out


class GearProfile:
    """HIP-event timing of every kernel launch of a step (gear_profile_* calls)."""

    def __init__(self):
        self.handle = lib.gear_profile_create()
        if not self.handle:
            raise GearError(GEAR_ERR_HIP, "gear_profile_create")

    def spans(self):
        """[(name, milliseconds)] of the last profiled step; the stream must have been synchronised."""
        out = []
        name, ms = C.c_char_p(), C.c_float()
        for i in range(lib.gear_profile_count(self.handle)):
            _check(lib.gear_profile_span(self.handle, i, C.byref(name), C.byref(ms)), "gear_profile_span")
            out.append((name.value.decode(), float(ms.value)))
        return out

    def close(self):
        if self.handle:
            lib.gear_profile_destroy(self.handle)
            self.handle = None


def gear_init_tables(state: GearState) -> None:
    t = state.tables()
    _check(lib.gear_init_tables(C.byref(state.cfg), C.byref(t), _ptr(state.grad_accum), _ptr(state.counts),
                                _stream()), "gear_init_tables")


def gear_step(state: GearState, batch: DeviceBatch, M: int, lr: float) -> None:
    """Enqueue one step on the current stream; outputs land in state.loss / n_ready / ready_* / status."""
    t, b, o = state.tables(), batch.as_struct(), state.step_out()
    _check(lib.gear_step(C.byref(state.cfg), C.byref(b), C.byref(t), _ptr(state.dfv_cache), _ptr(state.grad_accum),
                         _ptr(state.counts), M, lr, _ptr(state.workspace), state.workspace.numel(), C.byref(o),
                         _stream()), "gear_step")


def gear_step_static(state: GearState, batch: DeviceBatch, M: int, lr: float) -> None:
    """gear_step on the library's static scratch array instead of state.workspace (allocates nothing)."""
    t, b, o = state.tables(), batch.as_struct(), state.step_out()
    _check(lib.gear_step_static(C.byref(state.cfg), C.byref(b), C.byref(t), _ptr(state.dfv_cache),
                                _ptr(state.grad_accum), _ptr(state.counts), M, lr, C.byref(o), _stream()),
           "gear_step_static")


class AdamMoments:
    """Device memory for gear_step_adam: zeroed moment arrays and the step counter."""

    def __init__(self, state: GearState, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8):
        cfg, dev = state.cfg, state.grad_accum.device
        self.beta1, self.beta2, self.eps, self.t = beta1, beta2, eps, 0
        z = lambda *shape: torch.zeros(shape, dtype=torch.float32, device=dev)
        self.user_m, self.user_v = z(cfg.n_users, cfg.emb_dim), z(cfg.n_users, cfg.emb_dim)
        self.url_m, self.url_v = z(cfg.n_urls, cfg.emb_dim), z(cfg.n_urls, cfg.emb_dim)
        self.mlp_m, self.mlp_v = z(state.mlp_params.numel()), z(state.mlp_params.numel())

    def as_struct(self) -> gear_adam:
        return gear_adam(self.beta1, self.beta2, self.eps, self.t, _ptr(self.user_m), _ptr(self.user_v),
                         _ptr(self.url_m), _ptr(self.url_v), _ptr(self.mlp_m), _ptr(self.mlp_v))


def gear_step_adam(state: GearState, batch: DeviceBatch, M: int, lr: float, adam: AdamMoments) -> None:
    """gear_step with Adam; advances adam.t (the step number, from 1) before the call."""
    adam.t += 1
    t, b, o, a = state.tables(), batch.as_struct(), state.step_out(), adam.as_struct()
    _check(lib.gear_step_adam(C.byref(state.cfg), C.byref(b), C.byref(t), _ptr(state.dfv_cache),
                              _ptr(state.grad_accum), _ptr(state.counts), M, lr, C.byref(a), _ptr(state.workspace),
                              state.workspace.numel(), C.byref(o), _stream()), "gear_step_adam")


def gear_refresh_dfv(state: GearState, image_ids: Optional[torch.Tensor], new_dfv: torch.Tensor) -> None:
    n = new_dfv.shape[0]
    _check(lib.gear_refresh_dfv(C.byref(state.cfg), _ptr(state.dfv_cache), _ptr(image_ids), _ptr(new_dfv), n,
                                _ptr(state.status), _stream()), "gear_refresh_dfv")


def gear_refresh_dfv_n(state: GearState, image_ids: torch.Tensor, new_dfv: torch.Tensor, n_rows: torch.Tensor) -> None:
    """Rows r < n_rows[0] (a device word) of image_ids / new_dfv; the host does not read the count."""
    max_rows = min(int(image_ids.numel()), int(new_dfv.shape[0]))
    _check(lib.gear_refresh_dfv_n(C.byref(state.cfg), _ptr(state.dfv_cache), _ptr(image_ids), _ptr(new_dfv), _ptr(n_rows),
                                  max_rows, _ptr(state.status), _stream()), "gear_refresh_dfv_n")


def gear_stamp_dfv_n(state: GearState, dfv_stamp: torch.Tensor, image_ids: torch.Tensor, n_rows: torch.Tensor,
                     now: int) -> None:
    _check(lib.gear_stamp_dfv_n(C.byref(state.cfg), _ptr(dfv_stamp), _ptr(image_ids), _ptr(n_rows),
                                int(image_ids.numel()), int(now), _ptr(state.status), _stream()), "gear_stamp_dfv_n")


def gear_expired_ids(state: GearState, image_ids: torch.Tensor, dfv_stamp: torch.Tensor, now: int, expiry: int):
    """Returns (ids buffer [n], n_expired [1]), both on the device; the first n_expired ids are valid."""
    n = int(image_ids.numel())
    out = torch.empty(max(n, 1), dtype=torch.int32, device=dfv_stamp.device)
    n_out = torch.zeros(1, dtype=torch.int32, device=dfv_stamp.device)
    _check(lib.gear_expired_ids(C.byref(state.cfg), _ptr(image_ids) if n else None, n, _ptr(dfv_stamp), int(now),
                                int(expiry), _ptr(state.workspace), state.workspace.numel(), _ptr(out), _ptr(n_out),
                                _ptr(state.status), _stream()), "gear_expired_ids")
    return out, n_out


def gear_stamp_dfv(state: GearState, dfv_stamp: torch.Tensor, image_ids: Optional[torch.Tensor], now: int,
                   n: Optional[int] = None) -> None:
    count = int(image_ids.numel()) if n is None and image_ids is not None else int(n if n is not None else dfv_stamp.numel())
    _check(lib.gear_stamp_dfv(C.byref(state.cfg), _ptr(dfv_stamp), _ptr(image_ids), count, int(now), _ptr(state.status),
                              _stream()), "gear_stamp_dfv")


class DenseStandIn:
    """Device memory of the stand-in Dense Part (DFV[i] = Wd raw[i]) and the two calls on it."""

    def __init__(self, state: GearState, raw: torch.Tensor, wd: torch.Tensor, max_rows: int):
        cfg = state.cfg
        assert raw.dtype == torch.float32 and wd.dtype == torch.float32 and raw.is_contiguous() and wd.is_contiguous()
        assert raw.shape[0] == cfg.n_images and wd.shape == (cfg.dfv_dim, raw.shape[1])
        self.cfg = gear_dense_config(cfg.n_images, raw.shape[1], cfg.dfv_dim, cfg.dfv_dtype, max_rows)
        self.raw, self.wd, self.state = raw, wd, state
        nbytes = lib.gear_dense_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise GearError("gear_dense_workspace_bytes: invalid configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=raw.device)
        self.status = torch.zeros(1, dtype=torch.int32, device=raw.device)

    def infer(self, image_ids: Optional[torch.Tensor], n: Optional[int] = None) -> torch.Tensor:
        """Rows [n x dfv_dim] in the cache's type for the listed images (None: images 0..n-1)."""
        n = int(image_ids.numel()) if n is None else int(n)
        out = torch.empty((n, self.cfg.dfv_dim), dtype=self.state.dfv_cache.dtype, device=self.raw.device)
        _check(lib.gear_dense_infer(C.byref(self.cfg), _ptr(self.raw), _ptr(self.wd), _ptr(image_ids), n,
                                    _ptr(out) if n else _ptr(self.workspace), _ptr(self.workspace),
                                    self.workspace.numel(), _ptr(self.status), _stream()), "gear_dense_infer")
        return out

    def backward(self, ready_ids: torch.Tensor, ready_grads: torch.Tensor, n_ready: int, lr: float) -> None:
        _check(lib.gear_dense_backward(C.byref(self.cfg), _ptr(self.raw), _ptr(self.wd), _ptr(ready_ids),
                                       _ptr(ready_grads), int(n_ready), lr, _ptr(self.workspace),
                                       self.workspace.numel(), _ptr(self.status), _stream()), "gear_dense_backward")

    def backward_n(self, ready_ids: torch.Tensor, ready_grads: torch.Tensor, n_ready: torch.Tensor, lr: float) -> None:
        """The same with the number of emissions left on the device (a step's n_ready word)."""
        assert ready_ids.numel() >= self.cfg.max_rows and ready_grads.shape[0] >= self.cfg.max_rows
        _check(lib.gear_dense_backward_n(C.byref(self.cfg), _ptr(self.raw), _ptr(self.wd), _ptr(ready_ids),
                                         _ptr(ready_grads), _ptr(n_ready), lr, _ptr(self.workspace),
                                         self.workspace.numel(), _ptr(self.status), _stream()), "gear_dense_backward_n")


def gear_group_ids(state: GearState, keys: torch.Tensor, key_range: int):
    n = int(keys.numel())
    dev = keys.device
    unique = torch.zeros(max(n, 1), dtype=torch.int32, device=dev)
    segoff = torch.zeros(n + 1, dtype=torch.int32, device=dev)
    perm = torch.zeros(max(n, 1), dtype=torch.int32, device=dev)
    n_unique = torch.zeros(1, dtype=torch.int32, device=dev)
    _check(lib.gear_group_ids(C.byref(state.cfg), _ptr(keys) if n else None, n, key_range, _ptr(state.workspace),
                              state.workspace.numel(), _ptr(unique), _ptr(segoff), _ptr(perm), _ptr(n_unique),
                              _stream()), "gear_group_ids")
    return unique, segoff, perm, n_unique
