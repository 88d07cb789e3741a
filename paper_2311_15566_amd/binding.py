"""ctypes binding of include/spotshard.h: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspotshard.so")

SS_OK, SS_EINVAL, SS_ENOMEM, SS_ESTATE, SS_EHIP, SS_EINTR = range(6)
_STATUS = {1: "SS_EINVAL", 2: "SS_ENOMEM", 3: "SS_ESTATE", 4: "SS_EHIP", 5: "SS_EINTR"}
_NORM = {"layernorm": 0, "rmsnorm": 1}
_ACT = {"gelu_tanh": 0, "relu": 1, "swiglu": 2}
_POS = {"learned": 0, "rope": 1}
_DTYPE = {"f32": 0, "bf16": 1, "f16": 2}


class SpotShardError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"{_STATUS.get(status, status)}: {text}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "ffn", "vocab", "max_pos",
                                         "norm", "act", "pos", "has_bias", "dtype", "kv_dtype")] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float)]


class Slice(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layer_lo", "layer_hi", "head_lo", "head_hi", "ffn_lo", "ffn_hi")]


_LAYER_FIELDS = ("ln1_g", "ln1_b", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo",
                 "ln2_g", "ln2_b", "w1", "b1", "wg", "wu", "w2", "b2")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class Weights(C.Structure):
    _fields_ = [("slice", Slice)] + [(n, C.c_void_p) for n in ("wte", "wpe", "lm_head", "lnf_g", "lnf_b")] + \
               [("layers", C.POINTER(LayerWeights))]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    # PyTorch first: its wheel brings a HIP runtime of its own and loads it into the global symbol scope.  The
    # library's HIP calls (its kernels' registration at load time included) must end up in that same runtime, or
    # the streams and device pointers PyTorch hands over belong to a runtime the library's calls do not reach
    # (seen as "no ROCm-capable device is detected" on the first copy).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.ss_last_error.restype = C.c_char_p
    L.ss_version.restype = C.c_char_p
    L.ss_shard_device_bytes.restype = sz
    L.ss_shard_device_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(Slice), i32, i32]
    L.ss_shard_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Slice), C.POINTER(Weights), i32, i32, vp, sz, vp,
                                  C.POINTER(vp)]
    L.ss_shard_destroy.argtypes = [vp]
    L.ss_shard_reset.argtypes = [vp, vp]
    L.ss_prefill.argtypes = [C.POINTER(vp), i32, vp, i32, i32, vp, vp, vp]
    L.ss_decode_step.argtypes = [C.POINTER(vp), i32, vp, i32, vp, vp, vp]
    L.ss_decode_step_static.argtypes = [C.POINTER(vp), i32, vp, i32, vp, vp, vp]
    L.ss_static_scratch_bytes.restype = sz
    L.ss_static_scratch_bytes.argtypes = []
    L.ss_stage_prefill.argtypes = [C.POINTER(vp), i32, vp, vp, i32, i32, vp, vp, vp, vp]
    L.ss_stage_decode_step.argtypes = [C.POINTER(vp), i32, vp, vp, i32, vp, vp, vp, vp]
    L.ss_committed_len.argtypes = [vp, C.POINTER(i32), vp]
    L.ss_kv_repack.argtypes = [vp, vp, C.POINTER(i32), i32, C.POINTER(C.c_uint64), vp]
    L.ss_kv_export_bytes.restype = sz
    L.ss_kv_export_bytes.argtypes = [vp]
    L.ss_kv_export.argtypes = [vp, vp, sz, vp]
    L.ss_kv_import.argtypes = [vp, vp, C.POINTER(i32), sz, vp]
    L.ss_debug_interrupt_after_layer.argtypes = [vp, i32]
    L.ss_set_graph_launch.argtypes = [vp, i32]
    L.ss_shard_geometry.argtypes = [vp, C.POINTER(i32)]
    L.ss_kernel_timing.argtypes = [vp, i32]
    L.ss_shard_create_from_resident.argtypes = [vp, vp, C.POINTER(vp), i32, i32, i32, vp, C.c_size_t, vp, C.POINTER(vp), C.POINTER(C.c_uint64)]
    L.ss_shard_model_context_bytes.argtypes = [vp]
    L.ss_shard_model_context_bytes.restype = C.c_size_t
    L.ss_debug_force_gemm_shape.argtypes = [i32, i32]
    L.ss_debug_force_prefill_block.argtypes = [i32, i32]
    L.ss_debug_matrix_core_probe.argtypes = [vp, C.c_uint64, i32, i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.ss_kernel_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), vp]
    return L


lib = _load()


def version() -> str:
    return lib.ss_version().decode()


def _check(status):
    if status != SS_OK:
        raise SpotShardError(status, lib.ss_last_error().decode())


def _desc(d: dict) -> ModelDesc:
    return ModelDesc(d["n_layers"], d["d_model"], d["n_heads"], d["head_dim"], d["ffn"], d["vocab"], d["max_pos"],
                     _NORM[d["norm"]], _ACT[d["act"]], _POS[d["pos"]], int(d["has_bias"]), _DTYPE[d["dtype"]],
                     _DTYPE[kv_dtype_of(d)], d["norm_eps"], d["rope_theta"])


def kv_dtype_of(d: dict) -> str:
    """Cache element type: the descriptor's "kv_dtype", default half for a bf16 model."""
    return d.get("kv_dtype") or ("f32" if d["dtype"] == "f32" else "f16")


def _slice(s: dict) -> Slice:
    return Slice(*(s[k] for k in ("layer_lo", "layer_hi", "head_lo", "head_hi", "ffn_lo", "ffn_hi")))


def _hptr(a):
    if a is None:
        return None
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("host tensors must be C-contiguous")
    return a.ctypes.data


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def device_bytes(desc: dict, slc: dict, max_batch: int, max_seq: int) -> int:
    d, s = _desc(desc), _slice(slc)
    return lib.ss_shard_device_bytes(C.byref(d), C.byref(s), max_batch, max_seq)


class Shard:
    """One position's model context + cache context on the current device."""

    def __init__(self, desc: dict, slc: dict, parent: dict, max_batch: int, max_seq: int, stream=None):
        import torch
        self.desc, self.slice = dict(desc), dict(slc)
        self.max_batch, self.max_seq = max_batch, max_seq
        d, s = _desc(desc), _slice(slc)
        nbytes = lib.ss_shard_device_bytes(C.byref(d), C.byref(s), max_batch, max_seq)
        if nbytes == 0:
            # let create produce the error text
            nbytes = 256
        self.mem = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")   # gaps between tensors stay zero
        layers = (LayerWeights * len(parent["layers"]))()
        for i, Lw in enumerate(parent["layers"]):
            for f in _LAYER_FIELDS:
                setattr(layers[i], f, _hptr(Lw.get(f)))
        w = Weights(_slice(parent["slice"]), _hptr(parent["wte"]), _hptr(parent["wpe"]), _hptr(parent["lm_head"]),
                    _hptr(parent["lnf_g"]), _hptr(parent["lnf_b"]), layers)
        h = C.c_void_p()
        self.handle = None
        _check(lib.ss_shard_create(C.byref(d), C.byref(s), C.byref(w), max_batch, max_seq,
                                   C.c_void_p(self.mem.data_ptr()), nbytes, _stream(stream), C.byref(h)))
        self.handle = h

    @classmethod
    def from_resident(cls, desc: dict, slc: dict, sources, max_batch: int, max_seq: int, stream=None, mem=None):
        """A shard whose model context is copied out of resident shards (device to device).
        mem: a zeroed uint8 CUDA tensor of at least device_bytes(...) to build it in, or None."""
        import torch
        self = cls.__new__(cls)
        self.desc, self.slice = dict(desc), dict(slc)
        self.max_batch, self.max_seq = max_batch, max_seq
        d, s = _desc(desc), _slice(slc)
        nbytes = lib.ss_shard_device_bytes(C.byref(d), C.byref(s), max_batch, max_seq) or 256
        self.mem = mem if mem is not None else torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        nbytes = self.mem.numel()
        arr = (C.c_void_p * len(sources))(*[x.handle for x in sources])
        h, moved = C.c_void_p(), C.c_uint64()
        self.handle = None
        _check(lib.ss_shard_create_from_resident(C.byref(d), C.byref(s), arr, len(sources), max_batch, max_seq,
                                                 C.c_void_p(self.mem.data_ptr()), nbytes, _stream(stream), C.byref(h),
                                                 C.byref(moved)))
        self.handle = h
        self.bytes_copied = moved.value
        return self

    def model_context(self):
        """The bytes of device memory that hold the model context (a view, uint8)."""
        return self.mem[:lib.ss_shard_model_context_bytes(self.handle)]

    def destroy(self):
        if self.handle is not None:
            lib.ss_shard_destroy(self.handle)
            self.handle = None
            self.mem = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reset(self, stream=None):
        _check(lib.ss_shard_reset(self.handle, _stream(stream)))

    def interrupt_after_layer(self, layer: int):
        _check(lib.ss_debug_interrupt_after_layer(self.handle, layer))

    def set_graph_launch(self, enabled: bool):
        _check(lib.ss_set_graph_launch(self.handle, int(enabled)))

    def kernel_timing(self, enabled: bool):
        _check(lib.ss_kernel_timing(self.handle, int(enabled)))

    def kernel_timing_read(self, stream=None):
        ms, cnt = (C.c_double * 8)(), (C.c_int64 * 8)()
        _check(lib.ss_kernel_timing_read(self.handle, ms, cnt, _stream(stream)))
        names = ("embed", "qkv_gemm", "decode_attn", "resid_gemm", "ffn_up_gemm", "lm_head", "commit")
        return {n: (ms[i], cnt[i]) for i, n in enumerate(names)}

    def geometry(self):
        out = (C.c_int32 * 6)()
        _check(lib.ss_shard_geometry(self.handle, out))
        return dict(zip(("layers", "heads", "ffn", "max_batch", "max_seq", "elem_bytes"), list(out)))


def _group(group):
    arr = (C.c_void_p * len(group))(*[g.handle for g in group])
    return arr, len(group)


def prefill(group, tokens, logits=None, next_tokens=None, stream=None):
    """tokens: device int32 [B, S_in]; logits: device float32 [B, V] or None; next_tokens: device int32 [B] or None."""
    arr, n = _group(group)
    B, S = tokens.shape
    _check(lib.ss_prefill(arr, n, _dptr(tokens), B, S, _dptr(logits), _dptr(next_tokens), _stream(stream)))


def decode_step(group, tokens_in, logits=None, next_tokens=None, stream=None):
    arr, n = _group(group)
    _check(lib.ss_decode_step(arr, n, _dptr(tokens_in), tokens_in.shape[0], _dptr(logits), _dptr(next_tokens),
                              _stream(stream)))


def decode_step_static(group, tokens_in, logits=None, next_tokens=None, stream=None):
    """ss_decode_step with the step's scratch in the library's static device array (allocates nothing)."""
    arr, n = _group(group)
    _check(lib.ss_decode_step_static(arr, n, _dptr(tokens_in), tokens_in.shape[0], _dptr(logits), _dptr(next_tokens),
                                     _stream(stream)))


def static_scratch_bytes() -> int:
    return int(lib.ss_static_scratch_bytes())


def stage_prefill(group, B, S, tokens=None, hidden_in=None, hidden_out=None, logits=None, next_tokens=None, stream=None):
    """A pipeline stage's initial phase: tokens (device int32 [B, S]) or hidden_in (device float32 [B*S, d]);
    hidden_out (device float32 [B*S, d]) or logits / next_tokens."""
    arr, n = _group(group)
    _check(lib.ss_stage_prefill(arr, n, _dptr(tokens), _dptr(hidden_in), B, S, _dptr(hidden_out), _dptr(logits),
                                _dptr(next_tokens), _stream(stream)))


def stage_decode_step(group, B, tokens_in=None, hidden_in=None, hidden_out=None, logits=None, next_tokens=None,
                      stream=None):
    """A pipeline stage's decode step: tokens_in (device int32 [B]) or hidden_in (device float32 [B, d]);
    hidden_out (device float32 [B, d]) or logits / next_tokens."""
    arr, n = _group(group)
    _check(lib.ss_stage_decode_step(arr, n, _dptr(tokens_in), _dptr(hidden_in), B, _dptr(hidden_out), _dptr(logits),
                                    _dptr(next_tokens), _stream(stream)))


def committed_len(shard, stream=None) -> np.ndarray:
    out = (C.c_int32 * shard.max_batch)()
    _check(lib.ss_committed_len(shard.handle, out, _stream(stream)))
    return np.array(list(out), dtype=np.int32)


def kv_repack(dst, src, batch_map, first_source=True, stream=None) -> int:
    bm = (C.c_int32 * dst.max_batch)(*[int(v) for v in batch_map])
    moved = C.c_uint64(0)
    _check(lib.ss_kv_repack(dst.handle, src.handle, bm, int(first_source), C.byref(moved), _stream(stream)))
    return moved.value


def force_gemm_shape(tiles_per_block: int = 0, k_slices: int = 0):
    """Test aid: force the decode GEMMs' launch shape for plans built from now on (0, 0 = library's choice)."""
    _check(lib.ss_debug_force_gemm_shape(int(tiles_per_block), int(k_slices)))


def force_prefill_block(rows_per_block: int = 0, tokens_per_block: int = 0):
    """Test aid: force the block of the initial phase's GEMMs, rows x tokens: 128 x 128, 128 x 256 or 256 x 256
    (0 x 0 = library's choice)."""
    _check(lib.ss_debug_force_prefill_block(int(rows_per_block), int(tokens_per_block)))


def matrix_core_probe(operands, lds_reads: bool, loads: bool, iters: int, stream=None):
    """Measurement aid: (TFLOP/s, cycles per 64 products, GHz) of the matrix cores on `operands` (a device tensor of 1 MiB or
    more), optionally with the LDS reads and direct-to-LDS loads of the initial phase's GEMM."""
    t, c, g = C.c_double(), C.c_double(), C.c_double()
    _check(lib.ss_debug_matrix_core_probe(operands.data_ptr(), operands.numel() * operands.element_size(), int(lds_reads), int(loads),
                                          int(iters), C.byref(t), C.byref(c), C.byref(g), _stream(stream)))
    return t.value, c.value, g.value


def device_kv_bytes(shard) -> int:
    """Bytes of the committed cache rows the shard holds (what ss_kv_export would write)."""
    return int(lib.ss_kv_export_bytes(shard.handle))


def kv_export(shard, stream=None) -> np.ndarray:
    n = lib.ss_kv_export_bytes(shard.handle)
    dt = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[kv_dtype_of(shard.desc)]   # bf16: raw bit patterns
    out = np.empty(n // np.dtype(dt).itemsize, dtype=dt)
    _check(lib.ss_kv_export(shard.handle, out.ctypes.data if n else None, n, _stream(stream)))
    return out


def kv_import(shard, flat: np.ndarray, lens, stream=None):
    flat = np.ascontiguousarray(flat)
    ln = (C.c_int32 * shard.max_batch)(*[int(v) for v in lens])
    _check(lib.ss_kv_import(shard.handle, flat.ctypes.data if flat.size else None, ln, flat.nbytes, _stream(stream)))
