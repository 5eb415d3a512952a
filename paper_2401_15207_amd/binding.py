"""ctypes binding of libhift.so.  Argument marshalling only: every step of the HiFT path runs in
the library's HIP kernels.  PyTorch is used to allocate device / pinned memory and streams."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch ships its own HIP runtime; it must be loaded first so that libhift.so binds to that
# same runtime (one runtime per process: streams and pointers are shared with torch).
import torch  # noqa: F401

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhift.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2401_15207_amd.build); "
                      "there is no fallback path")
lib = C.CDLL(LIB_PATH)

STRATEGY = {"bottom2up": 0, "top2down": 1, "random": 2}
OPT_KIND = {"adamw": 0, "adagrad": 1, "sgd": 2, "adafactor": 3}


class HiftError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"hift status {status}: {msg}")
        self.status = status


class Config(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_seq", C.c_int32), ("n_classes", C.c_int32),
                ("norm_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32),
                ("state_on_host", C.c_int32), ("master_on_host", C.c_int32), ("no_packed_copies", C.c_int32),
                ("tie_embeddings", C.c_int32), ("lora_rank", C.c_int32), ("lora_alpha", C.c_float), ("unfused", C.c_int32)]


class Memory(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("device_master", "device_forward", "device_packed", "device_grad", "device_state",
                 "device_activations", "device_workspace", "device_total", "pinned_total",
                 "para", "gra", "sta", "pgs", "residual", "total", "n_params", "peak_trainable")] + \
               [("k", C.c_int32), ("reserved", C.c_int32), ("zeta1", C.c_double), ("zeta_fpft", C.c_double),
                ("zeta_hift", C.c_double), ("zeta_hift_peak", C.c_double)]


class Opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("momentum", C.c_double)]


class Batch(C.Structure):
    _fields_ = [("tokens", C.c_void_p), ("labels", C.c_void_p), ("batch", C.c_int32), ("seq", C.c_int32)]


class TensorInfo(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("unit", C.c_int32), ("kind", C.c_int32), ("offset", C.c_int64),
                ("rows", C.c_int64), ("cols", C.c_int64)]


lib.hift_last_error.restype = C.c_char_p
_vp, _i32, _i64, _u64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
_P = C.POINTER
_SIGS = {
    "hift_group_count": [_i32, _i32, _P(_i32)],
    "hift_group_order": [_i32, C.c_int, _u64, _P(_i32)],
    "hift_tensor_count": [_P(Config), _P(_i32), _P(_i64)],
    "hift_tensor_at": [_P(Config), _i32, _P(TensorInfo)],
    "hift_query_bytes": [_P(Config), _P(Opt), _i32, _i32, _i32, _P(_sz), _P(_sz)],
    "hift_memory_report": [_P(Config), _P(Opt), _i32, _i32, _i32, _P(Memory)],
    "hift_read_factored_state": [_vp, _i32, _vp, _sz],
    "hift_lr_at_cycle": [_i32, C.c_double, _i64, _i64, _i64, _P(C.c_double)],
    "hift_set_lr_schedule": [_vp, _i32, C.c_double, _i64, _i64],
    "hift_train": [_vp, _P(Batch), _i32, _i64, _vp],
    "hift_checkpoint_bytes": [_vp, _P(_sz)],
    "hift_checkpoint_save": [_vp, _vp, _sz],
    "hift_checkpoint_load": [_vp, _vp, _sz],
    "hift_model_create": [_P(Config), _P(Opt), _i32, _i32, _i32, _vp, _vp, _sz, _vp, _sz, _vp, _vp, _vp, _P(_vp)],
    "hift_model_create_chunked": [_P(Config), _P(Opt), _i32, _i32, _i32, _vp, _vp, _sz, _P(_vp), _P(_sz), _i32, _vp, _vp, _vp,
                                  _P(_vp)],
    "hift_set_group_schedule": [_vp, C.c_int, _i32, _u64, _P(_i32)],
    "hift_schedule_group_at": [_vp, _i64, _P(_i32)],
    "hift_group_units": [_vp, _i32, _P(_i32), _P(_i32)],
    "hift_step": [_vp, _P(Batch), _i32, _P(C.c_float)],
    "hift_set_lr": [_vp, C.c_double],
    "hift_cycle_index": [_vp, _P(_i64), _P(_i64)],
    "hift_lora_param_count": [_P(Config), _P(_i64)],
    "hift_lora_write": [_vp, _vp, _sz],
    "hift_lora_read": [_vp, _i32, _vp, _sz],
    "hift_lora_step": [_vp, _P(Batch), _P(C.c_float)],
    "hift_read_params": [_vp, _i32, _i32, _i32, _vp, _sz],
    "hift_write_params": [_vp, _i32, _i32, _vp, _sz],
    "hift_write_params_device": [_vp, _i32, _i32, _vp, _sz],
    "hift_read_state": [_vp, _i32, _i32, _i32, _vp, _sz],
    "hift_transfer_stats": [_vp, _P(_u64), _P(_u64)],
    "hift_last_step_ms": [_vp, _P(C.c_float), _P(C.c_float)],
    "hift_set_state_copy_engine": [_vp, _i32, _i32],
    "hift_profile_enable": [_vp, _i32],
    "hift_profile_read": [_vp, _i32, _P(_i64), _P(C.c_double), _P(C.c_double)],
    "hift_profile_read_rowwise": [_vp, _i32, _P(C.c_char_p), _P(_i64), _P(C.c_double), _P(C.c_double)],
    "hift_kernel_gemm": [_i32, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp,
                         _i32, _i64, _i64, _i64, _vp],
    "hift_kernel_packed_bytes": [_i64, _i64, _P(_sz)],
    "hift_kernel_pack_b": [_i32, _i64, _i64, _vp, _i64, _vp, _vp],
    "hift_kernel_gemm_packed": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp],
    "hift_kernel_optimizer": [_P(Opt), _i64, _i32, _i64, _vp, _vp, _vp, _vp, _vp, _vp],
    "hift_kernel_norm_fwd": [_i32, _i32, _i64, _i32, C.c_float, _vp, _vp, _vp, _vp, _vp, _vp],
    "hift_kernel_packed_workspace_bytes": [_P(_sz)],
    "hift_kernel_gemm_packed_ws": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _sz, _vp],
    "hift_kernel_gemm_packed_static": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp],
    "hift_kernel_linear_fused": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _vp],
    "hift_kernel_gemm_packed_rowsq": [_i64, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _vp],
    "hift_kernel_row_sumsq": [_i64, _i32, _vp, _i32, _vp, _vp],
    "hift_kernel_linear_norm_fused": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _vp,
                                      C.c_float, _vp, _vp, _vp],
    "hift_kernel_linear_gelu": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp],
    "hift_kernel_attention_fwd": [_i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp],
    "hift_kernel_attention_bwd": [_i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "hift_kernel_cross_entropy": [_i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp],
}
for _n, _a in _SIGS.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = C.c_int
lib.hift_model_destroy.argtypes = [_vp]
lib.hift_model_destroy.restype = None


def _check(st):
    if st != 0:
        raise HiftError(st, lib.hift_last_error().decode())


def make_config(cfg: dict, state_on_host: int = 0) -> Config:
    return Config(cfg["arch"], cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["d_ffn"], cfg["vocab"],
                  cfg["max_seq"], cfg.get("n_classes", 0), cfg["norm_eps"], cfg.get("rope_base", 10000.0),
                  cfg["dtype"], cfg.get("state_on_host", state_on_host), cfg.get("master_on_host", 0),
                  cfg.get("no_packed_copies", 0), cfg.get("tie_embeddings", 0), cfg.get("lora_rank", 0),
                  cfg.get("lora_alpha", 0.0), cfg.get("unfused", 0))


def make_opt(opt: dict) -> Opt:
    return Opt(OPT_KIND[opt["kind"]], opt["lr"], opt.get("beta1", 0.9), opt.get("beta2", 0.999),
               opt.get("eps", 1e-8), opt.get("weight_decay", 0.0), opt.get("momentum", 0.0))


def group_count(n_units: int, m: int) -> int:
    k = _i32()
    _check(lib.hift_group_count(n_units, m, C.byref(k)))
    return k.value


def group_order(k: int, strategy: str, seed: int = 0):
    out = (_i32 * k)()
    _check(lib.hift_group_order(k, STRATEGY[strategy], seed & (2 ** 64 - 1), out))
    return list(out)


def tensor_list(cfg: dict):
    """[(name, shape, kind, unit, offset)] in canonical order, and the parameter count."""
    c = make_config(cfg)
    n, total = _i32(), _i64()
    _check(lib.hift_tensor_count(C.byref(c), C.byref(n), C.byref(total)))
    out = []
    for i in range(n.value):
        t = TensorInfo()
        _check(lib.hift_tensor_at(C.byref(c), i, C.byref(t)))
        shape = (t.rows, t.cols) if t.kind == 0 else (t.rows,)
        out.append((t.name.decode(), shape, t.kind, t.unit, t.offset))
    return out, total.value


LR_KIND = {"constant": 0, "linear": 1}


def lr_at_cycle(kind: str, base_lr: float, warmup_cycles: int, total_cycles: int, cycle: int) -> float:
    out = C.c_double()
    _check(lib.hift_lr_at_cycle(LR_KIND[kind], base_lr, warmup_cycles, total_cycles, cycle, C.byref(out)))
    return out.value


def memory_report(cfg: dict, opt: dict, m: int, max_batch: int, max_seq: int) -> dict:
    c, o, out = make_config(cfg), make_opt(opt), Memory()
    _check(lib.hift_memory_report(C.byref(c), C.byref(o), m, max_batch, max_seq, C.byref(out)))
    return {n: getattr(out, n) for n, _t in Memory._fields_ if n != "reserved"}


def query_bytes(cfg: dict, opt: dict, m: int, max_batch: int, max_seq: int):
    c, o = make_config(cfg), make_opt(opt)
    d, p = _sz(), _sz()
    _check(lib.hift_query_bytes(C.byref(c), C.byref(o), m, max_batch, max_seq, C.byref(d), C.byref(p)))
    return d.value, p.value


def _ptr(t):
    return None if t is None else t.data_ptr()


def kernel_gemm(dtype, a_kmajor, b_kmajor, out_f32, M, N, K, A, lda, B, ldb, Cm, ldc, bias=None, R=None,
                batch=1, sa=0, sb=0, sc=0, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_gemm(dtype, int(a_kmajor), int(b_kmajor), int(out_f32), M, N, K, _ptr(A), lda, _ptr(B),
                                ldb, _ptr(Cm), ldc, _ptr(bias), _ptr(R), batch, sa, sb, sc, st))


def kernel_packed_bytes(N, K) -> int:
    b = _sz()
    _check(lib.hift_kernel_packed_bytes(N, K, C.byref(b)))
    return b.value


def kernel_pack_b(b_kmajor, N, K, B, ldb, Bp, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_pack_b(int(b_kmajor), N, K, _ptr(B), ldb, _ptr(Bp), st))


def kernel_gemm_packed(out_f32, M, N, K, A, lda, Bp, Cm, ldc, bias=None, R=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_gemm_packed(int(out_f32), M, N, K, _ptr(A), lda, _ptr(Bp), _ptr(Cm), ldc, _ptr(bias),
                                       _ptr(R), st))


def kernel_optimizer(opt: dict, count, decay, t, master, grad, s1, s2, compute_copy=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    o = make_opt(opt)
    _check(lib.hift_kernel_optimizer(C.byref(o), count, int(decay), t, _ptr(master), _ptr(grad), _ptr(s1), _ptr(s2),
                                     _ptr(compute_copy), st))


def kernel_norm_fwd(dtype, rms, rows, d, eps, x, g, b, y, stats, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_norm_fwd(dtype, int(rms), rows, d, eps, _ptr(x), _ptr(g), _ptr(b), _ptr(y), _ptr(stats), st))


def kernel_packed_workspace_bytes():
    n = _sz()
    _check(lib.hift_kernel_packed_workspace_bytes(C.byref(n)))
    return n.value


def kernel_gemm_packed_ws(out_f32, M, N, K, A, lda, Bp, Cm, ldc, bias, R, workspace, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_gemm_packed_ws(out_f32, M, N, K, _ptr(A), lda, _ptr(Bp), _ptr(Cm), ldc, _ptr(bias), _ptr(R),
                                          _ptr(workspace), workspace.numel() * workspace.element_size(), st))


def kernel_gemm_packed_static(out_f32, M, N, K, A, lda, Bp, Cm, ldc, bias=None, R=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_gemm_packed_static(int(out_f32), M, N, K, _ptr(A), lda, _ptr(Bp), _ptr(Cm), ldc, _ptr(bias),
                                              _ptr(R), st))


EPILOGUE_SWIGLU, EPILOGUE_ROPE, EPILOGUE_SWIGLU_BWD = 1, 2, 3
UNFUSED_EPILOGUES, UNFUSED_ATTENTION, UNFUSED_NORM, UNSHARED_LAST_ROUND = 1, 2, 4, 8   # hift_config.unfused


def kernel_linear_fused(epilogue, M, N, K, A, lda, W, packed_scratch, C, aux, cos_sin, seq, rot_cols, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_linear_fused(epilogue, M, N, K, _ptr(A), lda, _ptr(W), _ptr(packed_scratch), _ptr(C), _ptr(aux),
                                        _ptr(cos_sin), seq, rot_cols, st))


def kernel_gemm_packed_rowsq(M, N, K, A, lda, Bp, Cm, ldc, R, rowsq, workspace=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_gemm_packed_rowsq(M, N, K, _ptr(A), lda, _ptr(Bp), _ptr(Cm), ldc, _ptr(R), _ptr(rowsq),
                                             _ptr(workspace), st))


def kernel_row_sumsq(rows, d, x, n, out, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_row_sumsq(rows, d, _ptr(x), n, _ptr(out), st))


def kernel_linear_norm_fused(epilogue, M, N, K, A, lda, W, gain, packed_scratch, Cm, aux, cos_sin, seq, rot_cols, rowsq,
                             norm_eps, stats, workspace=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_linear_norm_fused(epilogue, M, N, K, _ptr(A), lda, _ptr(W), _ptr(gain), _ptr(packed_scratch),
                                             _ptr(Cm), _ptr(aux), _ptr(cos_sin), seq, rot_cols, _ptr(rowsq), norm_eps,
                                             _ptr(stats), _ptr(workspace), st))


def kernel_linear_gelu(backward, M, N, K, A, lda, W, bias, packed_scratch, Cm, aux, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_linear_gelu(int(backward), M, N, K, _ptr(A), lda, _ptr(W), _ptr(bias), _ptr(packed_scratch),
                                       _ptr(Cm), _ptr(aux), st))


def kernel_attention_fwd(batch, heads, seq, head_dim, causal, qkv, prob, ctx, lse=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_attention_fwd(batch, heads, seq, head_dim, int(causal), _ptr(qkv), _ptr(prob), _ptr(ctx), _ptr(lse), st))


def kernel_attention_bwd(batch, heads, seq, head_dim, causal, qkv, ctx, lse, dctx, dsum, dqkv, cos_sin=None, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_attention_bwd(batch, heads, seq, head_dim, int(causal), _ptr(qkv), _ptr(ctx), _ptr(lse),
                                         _ptr(dctx), _ptr(dsum), _ptr(dqkv), _ptr(cos_sin), st))


def kernel_cross_entropy(dtype, rows, V, logits, labels, row_loss, loss_out, stream=None):
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib.hift_kernel_cross_entropy(dtype, rows, V, _ptr(logits), _ptr(labels), _ptr(row_loss), _ptr(loss_out), st))


def _hip_runtime():
    """The HIP runtime this process already uses (the one torch loaded)."""
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                return C.CDLL(line.split()[-1])
    raise RuntimeError("no HIP runtime is loaded")


PINNED_CHUNK_BYTES = 32 << 30   # default size of the blocks the pinned arena is allocated in


class _PinnedArena:
    """Page-locked host memory of exactly the size asked for.  torch's pinned allocator rounds a
    request up to a power of two, which for arenas of tens of GB can double the host memory used."""

    def __init__(self, nbytes: int):
        self.hip = _hip_runtime()
        self.hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
        self.hip.hipHostFree.argtypes = [C.c_void_p]
        p = C.c_void_p()
        err = self.hip.hipHostMalloc(C.byref(p), nbytes, 0)
        if err != 0 or not p.value:
            raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed (error {err})")
        self.ptr, self.nbytes = p.value, nbytes

    def data_ptr(self) -> int:
        return self.ptr

    def free(self):
        if getattr(self, "ptr", None):
            self.hip.hipHostFree(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class HiftModel:
    """Owns the arenas (torch tensors) and streams a hift_model lives in."""

    def __init__(self, cfg: dict, opt: dict, m: int, max_batch: int, max_seq: int, init_params=None,
                 state_on_host: int = 0, device: str = "cuda:0", master_on_host: int = 0, no_packed_copies: int = 0,
                 unfused: int = 0, pinned_chunk_bytes: int = PINNED_CHUNK_BYTES, lora_rank: int = 0,
                 lora_alpha: float = 0.0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("HiftModel needs a GPU: there is no CPU path")
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = dict(cfg, state_on_host=state_on_host, master_on_host=master_on_host,
                        no_packed_copies=no_packed_copies, unfused=unfused, lora_rank=lora_rank, lora_alpha=lora_alpha)
        self.c, self.o = make_config(self.cfg), make_opt(opt)
        self.opt_dict, self.m0, self.max_batch, self.max_seq = dict(opt), m, max_batch, max_seq
        dbytes, pbytes = query_bytes(self.cfg, opt, m, max_batch, max_seq)
        self.device_arena = torch.empty(dbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.device_arena.data_ptr()
        self._dev_ptr = (base + 255) & ~255
        # the pinned arena in chunks of at most pinned_chunk_bytes: hosts refuse very large page-locked blocks
        self.pinned_chunks = []
        left = pbytes
        while left > 0:
            n = min(left, max(16, pinned_chunk_bytes & ~15))
            self.pinned_chunks.append(_PinnedArena((n + 15) & ~15))
            left -= n
        self.compute_stream = torch.cuda.Stream(self.device)
        self.h2d_stream = torch.cuda.Stream(self.device)
        self.d2h_stream = torch.cuda.Stream(self.device)
        self.device_bytes, self.pinned_bytes = dbytes, pbytes
        init = None
        if init_params is not None:
            init = np.ascontiguousarray(init_params, dtype=np.float32)
        h = _vp()
        nch = len(self.pinned_chunks)
        ptrs = (_vp * max(nch, 1))(*[a.data_ptr() for a in self.pinned_chunks])
        sizes = (_sz * max(nch, 1))(*[a.nbytes for a in self.pinned_chunks])
        if nch == 1:
            _check(lib.hift_model_create(C.byref(self.c), C.byref(self.o), m, max_batch, max_seq,
                                         None if init is None else init.ctypes.data, self._dev_ptr, dbytes,
                                         ptrs[0], sizes[0], self.compute_stream.cuda_stream,
                                         self.h2d_stream.cuda_stream, self.d2h_stream.cuda_stream, C.byref(h)))
        else:
            _check(lib.hift_model_create_chunked(C.byref(self.c), C.byref(self.o), m, max_batch, max_seq,
                                                 None if init is None else init.ctypes.data, self._dev_ptr, dbytes,
                                                 ptrs, sizes, nch, self.compute_stream.cuda_stream,
                                                 self.h2d_stream.cuda_stream, self.d2h_stream.cuda_stream, C.byref(h)))
        self.h = h
        self.k = None
        self.tensors, self.n_params = tensor_list(self.cfg)
        self.n_units = cfg["n_layers"] + 2

    def close(self):
        if getattr(self, "h", None):
            lib.hift_model_destroy(self.h)      # waits for the streams
            self.h = None
        for a in getattr(self, "pinned_chunks", []):
            a.free()
        self.pinned_chunks = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_group_schedule(self, strategy: str, m: int, seed: int = 0) -> int:
        k = _i32()
        _check(lib.hift_set_group_schedule(self.h, STRATEGY[strategy], m, seed & (2 ** 64 - 1), C.byref(k)))
        self.k = k.value
        return self.k

    def schedule_group_at(self, t: int) -> int:
        g = _i32()
        _check(lib.hift_schedule_group_at(self.h, t, C.byref(g)))
        return g.value

    def group_units(self, gid: int):
        lo, hi = _i32(), _i32()
        _check(lib.hift_group_units(self.h, gid, C.byref(lo), C.byref(hi)))
        return lo.value, hi.value

    def step(self, tokens, labels, group_id: int, want_loss: bool = True):
        """tokens / labels: int32 torch tensors on the device ([B,S] and [B,S] or [B])."""
        assert tokens.dtype == self.torch.int32 and labels.dtype == self.torch.int32
        assert tokens.is_cuda and labels.is_cuda and tokens.is_contiguous() and labels.is_contiguous()
        b = Batch(tokens.data_ptr(), labels.data_ptr(), tokens.shape[0], tokens.shape[1])
        loss = C.c_float()
        # the batch may still be in the making on torch's current stream: the step starts after it, and the
        # caching allocator must not hand the buffers out again before the step has read them
        cur = self.torch.cuda.current_stream()
        self.compute_stream.wait_stream(cur)
        tokens.record_stream(self.compute_stream)
        labels.record_stream(self.compute_stream)
        _check(lib.hift_step(self.h, C.byref(b), group_id, C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def lora_param_count(self) -> int:
        n = _i64()
        _check(lib.hift_lora_param_count(C.byref(self.c), C.byref(n)))
        return n.value

    def lora_write(self, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        _check(lib.hift_lora_write(self.h, v.ctypes.data, v.size))

    def lora_read(self, which: int = 0) -> np.ndarray:
        out = np.empty(self.lora_param_count(), dtype=np.float32)
        _check(lib.hift_lora_read(self.h, which, out.ctypes.data, out.size))
        return out

    def lora_step(self, tokens, labels, want_loss: bool = True):
        assert tokens.dtype == self.torch.int32 and labels.dtype == self.torch.int32
        assert tokens.is_cuda and labels.is_cuda and tokens.is_contiguous() and labels.is_contiguous()
        b = Batch(tokens.data_ptr(), labels.data_ptr(), tokens.shape[0], tokens.shape[1])
        loss = C.c_float()
        self.compute_stream.wait_stream(self.torch.cuda.current_stream())
        tokens.record_stream(self.compute_stream)
        labels.record_stream(self.compute_stream)
        _check(lib.hift_lora_step(self.h, C.byref(b), C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def set_lr(self, lr: float):
        _check(lib.hift_set_lr(self.h, lr))

    def cycle_index(self):
        s, c = _i64(), _i64()
        _check(lib.hift_cycle_index(self.h, C.byref(s), C.byref(c)))
        return s.value, c.value

    def _unit_count(self, lo, hi):
        return sum(int(np.prod(shape)) for _n, shape, _k, u, _o in self.tensors if lo <= u < hi)

    def read_params(self, unit_lo: int = 0, unit_hi: int | None = None, which: int = 0) -> np.ndarray:
        unit_hi = self.n_units if unit_hi is None else unit_hi
        out = np.empty(self._unit_count(unit_lo, unit_hi), dtype=np.float32)
        _check(lib.hift_read_params(self.h, unit_lo, unit_hi, which, out.ctypes.data, out.size))
        return out

    def write_params(self, unit_lo: int, unit_hi: int, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        _check(lib.hift_write_params(self.h, unit_lo, unit_hi, v.ctypes.data, v.size))

    def write_params_device(self, unit_lo: int, unit_hi: int, values):
        """values: contiguous float32 torch tensor on the device, complete on the current stream."""
        assert values.is_cuda and values.dtype == self.torch.float32 and values.is_contiguous()
        self.torch.cuda.current_stream().synchronize()
        _check(lib.hift_write_params_device(self.h, unit_lo, unit_hi, values.data_ptr(), values.numel()))

    def read_state(self, unit_lo: int, unit_hi: int, slot: int) -> np.ndarray:
        out = np.empty(self._unit_count(unit_lo, unit_hi), dtype=np.float32)
        _check(lib.hift_read_state(self.h, unit_lo, unit_hi, slot, out.ctypes.data, out.size))
        return out

    def transfer_stats(self):
        a, b = _u64(), _u64()
        _check(lib.hift_transfer_stats(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def last_step_ms(self):
        a, b = C.c_float(), C.c_float()
        _check(lib.hift_last_step_ms(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def set_state_copy_engine(self, engine: int, blocks: int = 16):
        _check(lib.hift_set_state_copy_engine(self.h, engine, blocks))

    def profile_enable(self, on: bool):
        _check(lib.hift_profile_enable(self.h, int(on)))

    def set_lr_schedule(self, kind: str, base_lr: float, warmup_cycles: int, total_cycles: int):
        _check(lib.hift_set_lr_schedule(self.h, LR_KIND[kind], base_lr, warmup_cycles, total_cycles))

    def train(self, batches, n_steps: int, want_losses: bool = True):
        """batches: list of (tokens, labels) device tensors; returns the losses (or None)."""
        arr = (Batch * len(batches))()
        self.compute_stream.wait_stream(self.torch.cuda.current_stream())  # the batches may still be in the making
        for i, (tok, lab) in enumerate(batches):
            arr[i] = Batch(tok.data_ptr(), lab.data_ptr(), tok.shape[0], tok.shape[1])
            tok.record_stream(self.compute_stream)
            lab.record_stream(self.compute_stream)
        losses = np.empty(n_steps, dtype=np.float32) if want_losses else None
        _check(lib.hift_train(self.h, arr, len(batches), n_steps, None if losses is None else losses.ctypes.data))
        return losses

    def checkpoint_save(self) -> np.ndarray:
        n = _sz()
        _check(lib.hift_checkpoint_bytes(self.h, C.byref(n)))
        buf = np.empty(n.value, dtype=np.uint8)
        _check(lib.hift_checkpoint_save(self.h, buf.ctypes.data, buf.size))
        return buf

    def checkpoint_load(self, buf: np.ndarray):
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        _check(lib.hift_checkpoint_load(self.h, buf.ctypes.data, buf.size))

    def read_factored_state(self, tensor_index: int) -> np.ndarray:
        _name, shape, _kind, _unit, _off = self.tensors[tensor_index]
        n = int(shape[0] + shape[1]) if len(shape) >= 2 else int(shape[0])
        out = np.empty(n, dtype=np.float32)
        _check(lib.hift_read_factored_state(self.h, tensor_index, out.ctypes.data, out.size))
        return out

    def memory(self) -> dict:
        """hift_memory_report of this model's configuration."""
        return memory_report(self.cfg, self.opt_dict, self.m0, self.max_batch, self.max_seq)

    def profile_read(self, category: int):
        n, ms, w = _i64(), C.c_double(), C.c_double()
        _check(lib.hift_profile_read(self.h, category, C.byref(n), C.byref(ms), C.byref(w)))
        return n.value, ms.value, w.value

    def profile_read_rowwise(self):
        """{kind name: (launches, total ms, algorithmic bytes)} of the row-wise kernels since profile_enable."""
        out, kind = {}, 0
        while True:
            name, n, ms, w = C.c_char_p(), _i64(), C.c_double(), C.c_double()
            if lib.hift_profile_read_rowwise(self.h, kind, C.byref(name), C.byref(n), C.byref(ms), C.byref(w)) != 0:
                break                                   # past the last kind
            out[name.value.decode()] = (n.value, ms.value, w.value)
            kind += 1
        return out

    def synchronize(self):
        self.compute_stream.synchronize()
        self.h2d_stream.synchronize()
        self.d2h_stream.synchronize()
