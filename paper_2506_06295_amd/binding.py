"""ctypes binding of libdllmc.so: argument marshalling only.

Every step of the cached denoising path runs inside the HIP library; torch is used
here for device memory and the stream handle.  Loading fails loudly when the library has
not been built (``python -c "import __graft_entry__ as g; g.build()"``): there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdllmc.so")

DLLMC_F32, DLLMC_BF16 = 0, 1
_DTYPES = {"f32": (DLLMC_F32, torch.float32), "bf16": (DLLMC_BF16, torch.bfloat16)}
_ERR = {-1: "EINVAL", -2: "ESTATE", -3: "EHIP", -4: "ENOMEM", -5: "ETOOBIG"}

EXPORTS = (
    "dllmc_workspace_bytes", "dllmc_create", "dllmc_num_selected", "dllmc_step",
    "dllmc_read_cache", "dllmc_read_scores", "dllmc_destroy", "dllmc_strerror",
    "dllmc_last_hip_error", "dllmc_op_select", "dllmc_op_vverify", "dllmc_op_linear",
    "dllmc_op_attention", "dllmc_profile_enable", "dllmc_profile_read", "dllmc_kernel_class_name",
    "dllmc_set_gemm_tuning", "dllmc_op_attention_scratch_bytes", "dllmc_plan_gemm_slices",
    "dllmc_gen_workspace_bytes", "dllmc_gen_create", "dllmc_gen_step", "dllmc_gen_read",
    "dllmc_gen_destroy", "dllmc_op_head_scratch_bytes", "dllmc_op_head", "dllmc_set_policy",
    "dllmc_set_layer_rho", "dllmc_layer_num_selected", "dllmc_probe_copy", "dllmc_probe_read", "dllmc_probe_mfma",
    "dllmc_op_linear_static", "dllmc_op_linear_static_max_elements",
    "dllmc_pool_bytes", "dllmc_workspace_bytes_paged", "dllmc_create_paged", "dllmc_set_page_table",
    "dllmc_pool_create", "dllmc_pool_available", "dllmc_pool_alloc", "dllmc_pool_free", "dllmc_pool_destroy",
)
NUM_KERNEL_CLASSES = 13


class dllmc_model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("batch", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float)]


class dllmc_layer_weights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g",
                                          "w_gate", "w_up", "w_down")]


class dllmc_paging(C.Structure):
    _fields_ = [("page_rows", C.c_int32), ("pool_pages", C.c_int32), ("page_table", C.POINTER(C.c_int32)),
                ("pool", C.c_void_p), ("pool_bytes", C.c_size_t)]


class dllmc_gen_config(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm_g", C.c_void_p), ("lm_head", C.c_void_p),
                ("vocab", C.c_int32), ("steps", C.c_int32), ("block_len", C.c_int32)]


class dllmc_kernel_stat(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("alg_bytes", C.c_double),
                ("flops", C.c_double)]


class DllmcError(RuntimeError):
    pass


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DllmcError(f"{LIB_PATH} is missing: build it first (__graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        L.dllmc_workspace_bytes.restype = C.c_size_t
        L.dllmc_workspace_bytes.argtypes = [C.POINTER(dllmc_model), C.c_int32, C.c_int32]
        L.dllmc_create.restype = C.c_int
        L.dllmc_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(dllmc_model),
                                   C.POINTER(dllmc_layer_weights), C.c_int32, C.c_int32, C.c_float,
                                   C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.dllmc_pool_bytes.restype = C.c_size_t
        L.dllmc_pool_bytes.argtypes = [C.POINTER(dllmc_model), C.c_int32, C.c_int32]
        L.dllmc_workspace_bytes_paged.restype = C.c_size_t
        L.dllmc_workspace_bytes_paged.argtypes = [C.POINTER(dllmc_model), C.c_int32, C.c_int32,
                                                  C.POINTER(dllmc_paging)]
        L.dllmc_create_paged.restype = C.c_int
        L.dllmc_create_paged.argtypes = [C.POINTER(C.c_void_p), C.POINTER(dllmc_model),
                                         C.POINTER(dllmc_layer_weights), C.c_int32, C.c_int32, C.c_float,
                                         C.c_int32, C.c_int32, C.POINTER(dllmc_paging), C.c_void_p,
                                         C.c_size_t, C.c_void_p]
        L.dllmc_set_page_table.restype = C.c_int
        L.dllmc_set_page_table.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.dllmc_pool_create.restype = C.c_int
        L.dllmc_pool_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32]
        L.dllmc_pool_available.restype = C.c_int32
        L.dllmc_pool_available.argtypes = [C.c_void_p]
        L.dllmc_pool_alloc.restype = C.c_int
        L.dllmc_pool_alloc.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
        L.dllmc_pool_free.restype = C.c_int
        L.dllmc_pool_free.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        L.dllmc_pool_destroy.restype = C.c_int
        L.dllmc_pool_destroy.argtypes = [C.c_void_p]
        L.dllmc_num_selected.restype = C.c_int32
        L.dllmc_num_selected.argtypes = [C.c_void_p]
        L.dllmc_step.restype = C.c_int
        L.dllmc_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_int32)]
        L.dllmc_read_cache.restype = C.c_int
        L.dllmc_read_cache.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.dllmc_read_scores.restype = C.c_int
        L.dllmc_read_scores.argtypes = [C.c_void_p, C.c_void_p]
        L.dllmc_destroy.restype = C.c_int
        L.dllmc_destroy.argtypes = [C.c_void_p]
        L.dllmc_strerror.restype = C.c_char_p
        L.dllmc_strerror.argtypes = [C.c_int]
        L.dllmc_last_hip_error.restype = C.c_int
        L.dllmc_op_select.restype = C.c_int
        L.dllmc_op_select.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p]
        L.dllmc_op_vverify.restype = C.c_int
        L.dllmc_op_vverify.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.dllmc_op_linear.restype = C.c_int
        L.dllmc_op_linear.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.dllmc_op_linear_static.restype = C.c_int
        L.dllmc_op_linear_static.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                             C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.dllmc_op_linear_static_max_elements.restype = C.c_size_t
        L.dllmc_op_linear_static_max_elements.argtypes = []
        L.dllmc_op_attention.restype = C.c_int
        L.dllmc_op_attention.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.dllmc_op_attention_scratch_bytes.restype = C.c_size_t
        L.dllmc_set_policy.restype = C.c_int
        L.dllmc_set_policy.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_uint32]
        L.dllmc_gen_workspace_bytes.restype = C.c_size_t
        L.dllmc_gen_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(dllmc_gen_config)]
        L.dllmc_gen_create.restype = C.c_int
        L.dllmc_gen_create.argtypes = [C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(dllmc_gen_config),
                                       C.c_void_p, C.c_size_t]
        L.dllmc_gen_step.restype = C.c_int
        L.dllmc_gen_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.dllmc_gen_read.restype = C.c_int
        L.dllmc_gen_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.dllmc_gen_destroy.restype = C.c_int
        L.dllmc_gen_destroy.argtypes = [C.c_void_p]
        L.dllmc_op_head_scratch_bytes.restype = C.c_size_t
        L.dllmc_op_head_scratch_bytes.argtypes = [C.c_int32] * 4
        L.dllmc_op_head.restype = C.c_int
        L.dllmc_op_head.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_float,
                                    C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p]
        L.dllmc_op_attention_scratch_bytes.argtypes = []
        L.dllmc_profile_enable.restype = C.c_int
        L.dllmc_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        L.dllmc_profile_read.restype = C.c_int
        L.dllmc_profile_read.argtypes = [C.c_void_p, C.POINTER(dllmc_kernel_stat), C.c_int32]
        L.dllmc_kernel_class_name.restype = C.c_char_p
        L.dllmc_kernel_class_name.argtypes = [C.c_int32]
        L.dllmc_plan_gemm_slices.restype = C.c_int32
        L.dllmc_plan_gemm_slices.argtypes = [C.c_int32] * 5 + [C.c_size_t]
        L.dllmc_set_gemm_tuning.restype = C.c_int
        L.dllmc_set_gemm_tuning.argtypes = [C.c_int32] * 7
        L.dllmc_set_layer_rho.restype = C.c_int
        L.dllmc_set_layer_rho.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int32]
        L.dllmc_layer_num_selected.restype = C.c_int32
        L.dllmc_layer_num_selected.argtypes = [C.c_void_p, C.c_int32]
        L.dllmc_probe_copy.restype = C.c_int
        L.dllmc_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.dllmc_probe_read.restype = C.c_int
        L.dllmc_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.dllmc_probe_mfma.restype = C.c_int
        L.dllmc_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        L = lib()
        msg = L.dllmc_strerror(rc).decode()
        extra = f" (hipError {L.dllmc_last_hip_error()})" if rc == -3 else ""
        raise DllmcError(f"{what}: {_ERR.get(rc, rc)} {msg}{extra}")


def _stream_handle() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class CachedDenoiser:
    """dllmc_create / dllmc_step / dllmc_destroy around torch-owned device memory."""

    def __init__(self, *, n_layers: int, d_model: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, d_ffn: int, batch: int, dtype: str,
                 weights: Sequence[Dict[str, torch.Tensor]], L_p: int, L_r: int, rho: float,
                 K_p: int, K_r: int, rms_eps: float = 1e-5, rope_theta: float = 10000.0,
                 paging: Optional[Dict] = None):
        """paging: None for the flat cache layout, else dict(page_rows, pool_pages, page_table
        [B][pages per sequence] of ints[, pool: uint8 device tensor shared between contexts])."""
        self._h = None
        L = lib()
        code, tdt = _DTYPES[dtype]
        self.torch_dtype = tdt
        self.B, self.L_p, self.L_r, self.n, self.d, self.T = batch, L_p, L_r, L_p + L_r, d_model, n_layers
        self.d_kv = n_kv_heads * head_dim
        self.model = dllmc_model(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, batch,
                                 code, rms_eps, rope_theta)
        if len(weights) != n_layers:
            raise DllmcError("one weight dict per layer expected")
        self._weights = weights  # keep the tensors alive: the library borrows the pointers
        arr = (dllmc_layer_weights * n_layers)()
        for l, w in enumerate(weights):
            for name, _ in dllmc_layer_weights._fields_:
                t = w[name]
                if not (t.is_cuda and t.is_contiguous() and t.dtype == tdt):
                    raise DllmcError(f"layer {l} {name}: need a contiguous {tdt} device tensor")
                setattr(arr[l], name, t.data_ptr())
        self.stream = _stream_handle()
        h = C.c_void_p()
        self.paging = None
        if paging is None:
            nbytes = L.dllmc_workspace_bytes(C.byref(self.model), L_p, L_r)
            if nbytes == 0:
                raise DllmcError("dllmc_workspace_bytes: invalid model description")
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            _check(L.dllmc_create(C.byref(h), C.byref(self.model), arr, L_p, L_r, rho, K_p, K_r,
                                  self.workspace.data_ptr(), nbytes, self.stream), "dllmc_create")
        else:
            table = self._table(paging["page_table"])
            pool = paging.get("pool")
            self._pool = pool   # keep a shared pool alive
            pg = dllmc_paging(int(paging["page_rows"]), int(paging["pool_pages"]), table,
                              None if pool is None else pool.data_ptr(),
                              0 if pool is None else pool.numel() * pool.element_size())
            nbytes = L.dllmc_workspace_bytes_paged(C.byref(self.model), L_p, L_r, C.byref(pg))
            if nbytes == 0:
                raise DllmcError("dllmc_workspace_bytes_paged: invalid model or paging description")
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            _check(L.dllmc_create_paged(C.byref(h), C.byref(self.model), arr, L_p, L_r, rho, K_p, K_r,
                                        C.byref(pg), self.workspace.data_ptr(), nbytes, self.stream),
                   "dllmc_create_paged")
            self.paging = dict(paging)
        self._h = h
        self.num_selected = L.dllmc_num_selected(h)
        self.sel_idx = torch.full((n_layers, batch, L_r), -1, dtype=torch.int32, device="cuda")

    @staticmethod
    def _table(page_table):
        flat = [int(p) for row in page_table for p in row]
        return (C.c_int32 * len(flat))(*flat)

    def set_page_table(self, page_table) -> None:
        """New page table for a paged context; the next step must be step 0."""
        _check(lib().dllmc_set_page_table(self._h, self._table(page_table)), "dllmc_set_page_table")

    def step(self, hidden_in: torch.Tensor, step_idx: int, hidden_out: Optional[torch.Tensor] = None):
        """Enqueue one denoising step; returns (hidden_out, n_sel).  self.sel_idx[:, :, :n_sel]
        holds the recomputed response rows per layer and sequence once the stream is synced."""
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        for t in (hidden_in, hidden_out):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype
                    and tuple(t.shape) == (self.B, self.n, self.d)):
                raise DllmcError("hidden states must be contiguous [B, n, d] device tensors of the model dtype")
        n_sel = C.c_int32(0)
        _check(lib().dllmc_step(self._h, hidden_in.data_ptr(), step_idx, hidden_out.data_ptr(),
                                self.sel_idx.data_ptr(), C.byref(n_sel)), "dllmc_step")
        return hidden_out, n_sel.value

    def set_policy(self, metric: str = "cosine", selection: str = "verify", v_update: str = "all",
                   seed: int = 0, source: str = "v") -> None:
        """Variants of the paper's ablations; see dllmc_set_policy."""
        _check(lib().dllmc_set_policy(self._h, {"v": 0, "k": 1}[source], {"cosine": 0, "l2": 1}[metric],
                                      {"verify": 0, "random": 1}[selection],
                                      {"all": 0, "selected": 1}[v_update], seed & 0xFFFFFFFF),
               "dllmc_set_policy")

    def set_layer_rho(self, rho_layers) -> None:
        """One update ratio per layer, or None for the single ratio given at creation."""
        if rho_layers is None:
            _check(lib().dllmc_set_layer_rho(self._h, None, 0), "dllmc_set_layer_rho")
            return
        arr = (C.c_float * len(rho_layers))(*[float(r) for r in rho_layers])
        _check(lib().dllmc_set_layer_rho(self._h, arr, len(rho_layers)), "dllmc_set_layer_rho")

    def layer_num_selected(self, layer: int) -> int:
        k = lib().dllmc_layer_num_selected(self._h, layer)
        if k < 0:
            raise DllmcError("dllmc_layer_num_selected: invalid argument")
        return k

    def read_cache(self, layer: int, which: int) -> torch.Tensor:
        width = self.d_kv if which < 2 else self.d
        out = torch.empty((self.B, self.n, width), dtype=self.torch_dtype, device="cuda")
        _check(lib().dllmc_read_cache(self._h, layer, which, out.data_ptr()), "dllmc_read_cache")
        return out

    def read_scores(self) -> torch.Tensor:
        out = torch.empty((self.T, self.B, self.L_r), dtype=torch.float32, device="cuda")
        _check(lib().dllmc_read_scores(self._h, out.data_ptr()), "dllmc_read_scores")
        return out

    def profile_enable(self, on: bool) -> None:
        _check(lib().dllmc_profile_enable(self._h, 1 if on else 0), "dllmc_profile_enable")

    def profile_read(self, reset: bool = True) -> Dict[str, Dict[str, float]]:
        arr = (dllmc_kernel_stat * NUM_KERNEL_CLASSES)()
        _check(lib().dllmc_profile_read(self._h, arr, 1 if reset else 0), "dllmc_profile_read")
        return {lib().dllmc_kernel_class_name(i).decode(): {
            "launches": int(arr[i].launches), "ms": arr[i].ms, "alg_bytes": arr[i].alg_bytes,
            "flops": arr[i].flops} for i in range(NUM_KERNEL_CLASSES)}

    def close(self) -> None:
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib().dllmc_destroy(h), "dllmc_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pool_bytes(model: dllmc_model, page_rows: int, pool_pages: int) -> int:
    return lib().dllmc_pool_bytes(C.byref(model), page_rows, pool_pages)


class PagePool:
    """dllmc_pool_*: host-side allocator of page ids."""

    def __init__(self, pool_pages: int):
        self._h = None
        h = C.c_void_p()
        _check(lib().dllmc_pool_create(C.byref(h), pool_pages), "dllmc_pool_create")
        self._h = h

    @property
    def available(self) -> int:
        return lib().dllmc_pool_available(self._h)

    def alloc(self, count: int) -> List[int]:
        ids = (C.c_int32 * max(count, 1))()
        _check(lib().dllmc_pool_alloc(self._h, count, ids), "dllmc_pool_alloc")
        return list(ids[:count])

    def free(self, ids: Sequence[int]) -> None:
        arr = (C.c_int32 * max(len(ids), 1))(*[int(i) for i in ids])
        _check(lib().dllmc_pool_free(self._h, arr, len(ids)), "dllmc_pool_free")

    def close(self) -> None:
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib().dllmc_pool_destroy(h), "dllmc_pool_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Generator:
    """dllmc_gen_* around a CachedDenoiser: the closed denoising loop, tokens stay on the device."""

    def __init__(self, den: CachedDenoiser, embed: torch.Tensor, final_norm_g: torch.Tensor,
                 lm_head: torch.Tensor, steps: int, block_len: int = 0):
        self._h = None
        self.den = den
        vocab = lm_head.shape[0]
        for name, t, shape in (("embed", embed, (vocab + 1, den.d)), ("final_norm_g", final_norm_g, (den.d,)),
                               ("lm_head", lm_head, (vocab, den.d))):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == den.torch_dtype and tuple(t.shape) == shape):
                raise DllmcError(f"{name}: need a contiguous {den.torch_dtype} device tensor of shape {shape}")
        self._keep = (embed, final_norm_g, lm_head)
        self.vocab, self.steps = vocab, steps
        self.cfg = dllmc_gen_config(embed.data_ptr(), final_norm_g.data_ptr(), lm_head.data_ptr(),
                                    vocab, steps, block_len)
        L = lib()
        nbytes = L.dllmc_gen_workspace_bytes(den._h, C.byref(self.cfg))
        if nbytes == 0:
            raise DllmcError("dllmc_gen_workspace_bytes: invalid configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        _check(L.dllmc_gen_create(C.byref(h), den._h, C.byref(self.cfg), self.workspace.data_ptr(), nbytes),
               "dllmc_gen_create")
        self._h = h

    def step(self, tokens: torch.Tensor, step_idx: int):
        """Enqueue one step of the loop on tokens [B, n] int32 (updated in place); returns
        (positions revealed per sequence, n_sel); den.sel_idx is filled as by den.step."""
        den = self.den
        if not (tokens.is_cuda and tokens.is_contiguous() and tokens.dtype == torch.int32
                and tuple(tokens.shape) == (den.B, den.n)):
            raise DllmcError("tokens must be a contiguous int32 [B, n] device tensor")
        n_rev, n_sel = C.c_int32(0), C.c_int32(0)
        _check(lib().dllmc_gen_step(self._h, tokens.data_ptr(), step_idx, den.sel_idx.data_ptr(),
                                    C.byref(n_sel), C.byref(n_rev)), "dllmc_gen_step")
        return n_rev.value, n_sel.value

    def read(self, hidden: bool = False):
        """(x0 [B, L_r] int32, conf [B, L_r] float32, chosen [B, L_r] int32[, hidden_out]) of the
        most recent step."""
        den = self.den
        x0 = torch.empty((den.B, den.L_r), dtype=torch.int32, device="cuda")
        conf = torch.empty((den.B, den.L_r), dtype=torch.float32, device="cuda")
        chosen = torch.empty((den.B, den.L_r), dtype=torch.int32, device="cuda")
        hout = torch.empty((den.B, den.n, den.d), dtype=den.torch_dtype, device="cuda") if hidden else None
        _check(lib().dllmc_gen_read(self._h, x0.data_ptr(), conf.data_ptr(), chosen.data_ptr(), _ptr(hout)),
               "dllmc_gen_read")
        return (x0, conf, chosen, hout) if hidden else (x0, conf, chosen)

    def close(self) -> None:
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib().dllmc_gen_destroy(h), "dllmc_gen_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def op_head(dtype: str, hidden: torch.Tensor, final_norm_g: torch.Tensor, lm_head: torch.Tensor,
            eps: float, rows: Optional[torch.Tensor] = None):
    """(x0 [M] int32, conf [M] float32) of the listed rows of hidden [*, d]."""
    d = hidden.shape[1]
    vocab = lm_head.shape[0]
    M = hidden.shape[0] if rows is None else rows.numel()
    code = _DTYPES[dtype][0]
    scratch = torch.empty(lib().dllmc_op_head_scratch_bytes(code, M, vocab, d), dtype=torch.uint8, device="cuda")
    x0 = torch.empty(M, dtype=torch.int32, device="cuda")
    conf = torch.empty(M, dtype=torch.float32, device="cuda")
    _check(lib().dllmc_op_head(code, hidden.data_ptr(), _ptr(rows), M, final_norm_g.data_ptr(), eps,
                               lm_head.data_ptr(), vocab, d, scratch.data_ptr(), x0.data_ptr(),
                               conf.data_ptr(), _stream_handle()), "dllmc_op_head")
    return x0, conf


def set_gemm_tuning(nw: int = -1, nw_dual: int = -1, force_s: int = -1, target_wg: int = -1,
                    tile_min_m: int = -1, fat_min_m: int = -1, tall_max_m: int = -1) -> None:
    _check(lib().dllmc_set_gemm_tuning(nw, nw_dual, force_s, target_wg, tile_min_m, fat_min_m,
                                       tall_max_m),
           "dllmc_set_gemm_tuning")


def op_select(scores: torch.Tensor, k: int) -> torch.Tensor:
    B, Lr = scores.shape
    out = torch.empty((B, max(k, 1)), dtype=torch.int32, device="cuda")
    _check(lib().dllmc_op_select(scores.data_ptr(), B, Lr, k, out.data_ptr(), _stream_handle()),
           "dllmc_op_select")
    return out[:, :k]


def op_vverify(dtype: str, h: torch.Tensor, wv: torch.Tensor, v_cache: torch.Tensor) -> torch.Tensor:
    """Scores [rows]; v_cache is overwritten with the new V rows."""
    rows, d = h.shape
    d_kv = wv.shape[0]
    scores = torch.empty(rows, dtype=torch.float32, device="cuda")
    scratch = torch.empty(rows * d_kv * 8, dtype=torch.float32, device="cuda")
    _check(lib().dllmc_op_vverify(_DTYPES[dtype][0], h.data_ptr(), wv.data_ptr(), v_cache.data_ptr(),
                                  scores.data_ptr(), rows, d, d_kv, scratch.data_ptr(),
                                  _stream_handle()), "dllmc_op_vverify")
    return scores


def op_linear(dtype: str, a: torch.Tensor, w: torch.Tensor, row_idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    K = a.shape[1]
    N = w.shape[0]
    M = a.shape[0] if row_idx is None else row_idx.numel()
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    scratch = torch.empty(M * N * 8, dtype=torch.float32, device="cuda")
    _check(lib().dllmc_op_linear(_DTYPES[dtype][0], a.data_ptr(), _ptr(row_idx), M, w.data_ptr(), N, K,
                                 out.data_ptr(), scratch.data_ptr(), _stream_handle()),
           "dllmc_op_linear")
    return out


def op_linear_static(dtype: str, a: torch.Tensor, w: torch.Tensor, out: torch.Tensor,
                     row_idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dllmc_op_linear_static into the caller's `out` (float32 [M, N]); allocates nothing."""
    M = a.shape[0] if row_idx is None else row_idx.numel()
    _check(lib().dllmc_op_linear_static(_DTYPES[dtype][0], a.data_ptr(), _ptr(row_idx), M, w.data_ptr(),
                                        w.shape[0], a.shape[1], out.data_ptr(), _stream_handle()),
           "dllmc_op_linear_static")
    return out


def op_attention(dtype: str, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                 H_q: int, H_kv: int, d_h: int, split_keys: bool = True) -> torch.Tensor:
    B, Mq, _ = q.shape
    n = k_cache.shape[1]
    out = torch.empty_like(q)
    scratch = None
    if split_keys:
        scratch = torch.empty(lib().dllmc_op_attention_scratch_bytes(), dtype=torch.uint8, device="cuda")
    _check(lib().dllmc_op_attention(_DTYPES[dtype][0], q.data_ptr(), B, Mq, k_cache.data_ptr(),
                                    v_cache.data_ptr(), n, H_q, H_kv, d_h, out.data_ptr(),
                                    _ptr(scratch), _stream_handle()), "dllmc_op_attention")
    return out


def probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """dst = src with the library's plain copy kernel (achievable-bandwidth probe)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise DllmcError("probe_copy: size mismatch")
    _check(lib().dllmc_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_handle()),
           "dllmc_probe_copy")


def probe_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    _check(lib().dllmc_probe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                  _stream_handle()), "dllmc_probe_read")


def probe_mfma(iters: int, sink: torch.Tensor, shape: int = 0) -> float:
    """Enqueues the MFMA loop (shape 0: 16x16x32, 1: 32x32x16); returns the flops of the launch."""
    f = C.c_double(0.0)
    _check(lib().dllmc_probe_mfma(iters, shape, sink.data_ptr(), C.byref(f), _stream_handle()),
           "dllmc_probe_mfma")
    return f.value
