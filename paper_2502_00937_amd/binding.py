"""ctypes binding for include/vitenc.h.  Function names mirror the C ABI one to one."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

VIT_OK, VIT_EINVAL, VIT_ENOMEM, VIT_ECAPACITY, VIT_EDEVICE = 0, -1, -2, -3, -4
VIT_DTYPE_FP32, VIT_DTYPE_BF16 = 0, 1
VIT_STATIC_SCRATCH_BYTES, VIT_STATIC_MAX_IMAGES = 128 << 20, 256
# order of include/vitenc.h's VIT_PROF_* enumerators
PROF_FAMILIES = ("patchify", "gemm_patch", "layernorm", "attention", "gemm_qkv", "gemm_out", "gemm_fc1", "gemm_fc2",
                 "gemm_proj")


class VitError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"vitenc status {status}: {message}")
        self.status = status


class vit_config_t(C.Structure):
    _fields_ = [
        ("image_size", C.c_int32), ("patch_size", C.c_int32), ("channels", C.c_int32),
        ("hidden", C.c_int32), ("heads", C.c_int32), ("mlp", C.c_int32),
        ("layers_local", C.c_int32), ("layers_global", C.c_int32),
        ("has_cls", C.c_int32), ("final_ln", C.c_int32), ("ln_eps", C.c_float),
        ("proj_layers", C.c_int32), ("proj_dims", C.c_int32 * 2), ("dtype", C.c_int32),
        ("token_merge", C.c_int32),
    ]


def lib_path() -> str:
    return os.path.join(_HERE, "libvitenc.so")


def load_library():
    """Load libvitenc.so; there is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2502_00937_amd.build`")
    lib = C.CDLL(path)
    lib.vit_last_error.restype = C.c_char_p
    lib.vit_weight_count.restype = C.c_size_t
    lib.vit_weight_count.argtypes = [C.POINTER(vit_config_t)]
    lib.vit_encoder_create.restype = C.c_int
    lib.vit_encoder_create.argtypes = [C.POINTER(vit_config_t), C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_void_p)]
    lib.vit_encoder_query.restype = C.c_int
    lib.vit_encoder_query.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                      C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.vit_encode_packed.restype = C.c_int
    lib.vit_encode_packed.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vit_encode_packed_graph.restype = C.c_int
    lib.vit_encode_packed_graph.argtypes = lib.vit_encode_packed.argtypes
    lib.vit_encode_packed_static.restype = C.c_int
    lib.vit_encode_packed_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_size_t, C.c_void_p, C.c_void_p]
    lib.vit_encoder_destroy.restype = None
    lib.vit_encoder_destroy.argtypes = [C.c_void_p]
    lib.vit_profile_enable.restype = C.c_int
    lib.vit_profile_enable.argtypes = [C.c_void_p, C.c_int]
    lib.vit_profile_tiles_enable.restype = C.c_int
    lib.vit_profile_tiles_enable.argtypes = [C.c_void_p, C.c_int]
    lib.vit_profile_tiles_read.restype = C.c_int
    lib.vit_profile_tiles_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                           C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.vit_handoff_create.restype = C.c_int
    lib.vit_handoff_create.argtypes = [C.c_int, C.POINTER(C.c_void_p)]
    lib.vit_handoff_destroy.restype = None
    lib.vit_handoff_destroy.argtypes = [C.c_void_p]
    lib.vit_handoff_expect.restype = C.c_int
    lib.vit_handoff_expect.argtypes = [C.c_void_p, C.c_int64, C.c_int32]
    lib.vit_handoff_publish.restype = C.c_int
    lib.vit_handoff_publish.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vit_handoff_complete.restype = C.c_int32
    lib.vit_handoff_complete.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_size_t)]
    lib.vit_handoff_pull.restype = C.c_int
    lib.vit_handoff_pull.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_size_t)]
    lib.vit_handoff_release.restype = C.c_int
    lib.vit_handoff_release.argtypes = [C.c_void_p, C.c_int64]
    lib.vit_preprocess_tiles.restype = C.c_int
    lib.vit_preprocess_tiles.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p, C.c_size_t,
                                         C.c_void_p]
    lib.vit_mfma_ceiling.restype = C.c_int
    lib.vit_mfma_ceiling.argtypes = [C.c_int, C.c_double, C.c_int32, C.POINTER(C.c_double)]
    lib.vit_profile_read.restype = C.c_int
    lib.vit_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _LIB = lib
    return lib


def _check(status: int):
    if status != VIT_OK:
        raise VitError(status, load_library().vit_last_error().decode())


def _to_struct(cfg: dict) -> vit_config_t:
    c = vit_config_t()
    for k in ("image_size", "patch_size", "channels", "hidden", "heads", "mlp", "layers_local", "layers_global",
              "has_cls", "final_ln", "proj_layers"):
        setattr(c, k, int(cfg[k]))
    c.ln_eps = float(cfg["ln_eps"])
    dims = list(cfg["proj_dims"]) + [0, 0]
    c.proj_dims[0], c.proj_dims[1] = int(dims[0]), int(dims[1])
    c.dtype = {"fp32": VIT_DTYPE_FP32, "bf16": VIT_DTYPE_BF16}[cfg["dtype"]]
    c.token_merge = int(cfg.get("token_merge", 1))
    return c


# ---- functions mirroring the C ABI ------------------------------------------------------
def vit_weight_count(cfg: dict) -> int:
    return int(load_library().vit_weight_count(C.byref(_to_struct(cfg))))


def vit_encoder_create(cfg: dict, weights: np.ndarray, device: int = 0) -> int:
    """weights: host fp32 array in the documented order.  Returns the opaque handle."""
    w = np.ascontiguousarray(weights, dtype=np.float32)
    handle = C.c_void_p()
    _check(load_library().vit_encoder_create(C.byref(_to_struct(cfg)), w.ctypes.data, w.size, device, C.byref(handle)))
    return handle.value


def vit_encoder_query(handle: int, n_tiles: int, n_images: int):
    """Returns (n_tokens, out_dim, out_bytes, workspace_bytes)."""
    n_tok, out_dim, out_b, ws_b = C.c_int64(), C.c_int32(), C.c_size_t(), C.c_size_t()
    _check(load_library().vit_encoder_query(handle, n_tiles, n_images, C.byref(n_tok), C.byref(out_dim),
                                            C.byref(out_b), C.byref(ws_b)))
    return n_tok.value, out_dim.value, out_b.value, ws_b.value


def vit_encode_packed(handle: int, pixels_ptr: int, images_per_request, tile_offsets, out_ptr: int,
                      out_capacity_bytes: int, workspace_ptr: int, workspace_bytes: int, stream: int = 0):
    """Raw call: device pointers as integers, host arrays as sequences.  Returns request_token_offsets."""
    ipr = np.ascontiguousarray(images_per_request, dtype=np.int32)
    to = np.ascontiguousarray(tile_offsets, dtype=np.int32)
    if (ipr >= 0).all() and to.size != int(ipr.sum()) + 1:  # the C side cannot see the array length
        raise VitError(VIT_EINVAL, "tile_offsets must have sum(images_per_request) + 1 entries")
    rto = np.zeros(ipr.size + 1, dtype=np.int64)
    _check(load_library().vit_encode_packed(handle, pixels_ptr, ipr.ctypes.data if ipr.size else None, ipr.size,
                                            to.ctypes.data, out_ptr, out_capacity_bytes, rto.ctypes.data,
                                            workspace_ptr, workspace_bytes, stream))
    return rto


def vit_encode_packed_graph(handle: int, pixels_ptr: int, images_per_request, tile_offsets, out_ptr: int,
                            out_capacity_bytes: int, workspace_ptr: int, workspace_bytes: int, stream: int = 0):
    """Raw call of the graph-replaying variant (same arguments as vit_encode_packed)."""
    ipr = np.ascontiguousarray(images_per_request, dtype=np.int32)
    to = np.ascontiguousarray(tile_offsets, dtype=np.int32)
    if (ipr >= 0).all() and to.size != int(ipr.sum()) + 1:
        raise VitError(VIT_EINVAL, "tile_offsets must have sum(images_per_request) + 1 entries")
    rto = np.zeros(ipr.size + 1, dtype=np.int64)
    _check(load_library().vit_encode_packed_graph(handle, pixels_ptr, ipr.ctypes.data if ipr.size else None, ipr.size,
                                                  to.ctypes.data, out_ptr, out_capacity_bytes, rto.ctypes.data,
                                                  workspace_ptr, workspace_bytes, stream))
    return rto


def vit_encode_packed_static(handle: int, pixels_ptr: int, images_per_request, tile_offsets, out_ptr: int,
                             out_capacity_bytes: int, stream: int = 0):
    """Raw call of the allocation-free variant (workspace = the library's static device array)."""
    ipr = np.ascontiguousarray(images_per_request, dtype=np.int32)
    to = np.ascontiguousarray(tile_offsets, dtype=np.int32)
    if (ipr >= 0).all() and to.size != int(ipr.sum()) + 1:
        raise VitError(VIT_EINVAL, "tile_offsets must have sum(images_per_request) + 1 entries")
    rto = np.zeros(ipr.size + 1, dtype=np.int64)
    _check(load_library().vit_encode_packed_static(handle, pixels_ptr, ipr.ctypes.data if ipr.size else None, ipr.size,
                                                   to.ctypes.data, out_ptr, out_capacity_bytes, rto.ctypes.data,
                                                   stream))
    return rto


def vit_preprocess_tiles(image_ptr: int, height: int, width: int, channels: int, tile_size: int, grid_rows: int,
                         grid_cols: int, thumbnail: bool, mean, std, out_ptr: int, out_capacity_bytes: int,
                         stream: int = 0) -> None:
    """Raw pointers in, nothing returned: resize + rescale + normalise + tile on the current device."""
    m = (C.c_float * channels)(*[float(v) for v in mean])
    sd = (C.c_float * channels)(*[float(v) for v in std])
    _check(load_library().vit_preprocess_tiles(C.c_void_p(image_ptr), height, width, channels, tile_size, grid_rows,
                                               grid_cols, 1 if thumbnail else 0, m, sd, C.c_void_p(out_ptr),
                                               out_capacity_bytes, C.c_void_p(stream)))


def preprocess_tiles(image, tile_size: int, grid_rows: int, grid_cols: int, thumbnail: bool, mean, std, out=None):
    """image: torch uint8 [H, W, C] on the GPU -> fp32 [n_tiles, C, S, S] (the encoder's `pixels`)."""
    import torch

    assert image.is_cuda and image.dtype == torch.uint8 and image.is_contiguous() and image.dim() == 3
    H, W, Cn = image.shape
    n_tiles = grid_rows * grid_cols + (1 if thumbnail else 0)
    if out is None:
        out = torch.empty((n_tiles, Cn, tile_size, tile_size), dtype=torch.float32, device=image.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    with torch.cuda.device(image.device):
        vit_preprocess_tiles(image.data_ptr(), H, W, Cn, tile_size, grid_rows, grid_cols, thumbnail, mean, std,
                             out.data_ptr(), out.numel() * 4, torch.cuda.current_stream().cuda_stream)
    return out


def vit_mfma_ceiling(device: int = 0, seconds: float = 0.1, random_operands: bool = True) -> float:
    """Sustained TFLOP/s of a register-only bf16 MFMA loop on `device` (measurement aid)."""
    out = C.c_double(0.0)
    _check(load_library().vit_mfma_ceiling(int(device), float(seconds), 1 if random_operands else 0, C.byref(out)))
    return out.value


def vit_encoder_destroy(handle: int) -> None:
    load_library().vit_encoder_destroy(handle)


class TokenHandoff:
    """Pull-style hand-off table (argument marshalling over the vit_handoff_* calls).  Pointers and
    streams are raw integers (torch: tensor.data_ptr(), torch.cuda.current_stream().cuda_stream)."""

    def __init__(self, device: int = 0):
        h = C.c_void_p()
        _check(load_library().vit_handoff_create(int(device), C.byref(h)))
        self._h = h

    def close(self):
        if self._h:
            load_library().vit_handoff_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def expect(self, request_id: int, n_images: int):
        _check(load_library().vit_handoff_expect(self._h, request_id, n_images))

    def publish(self, request_id: int, image_index: int, ptr: int, nbytes: int, stream: int = 0):
        _check(load_library().vit_handoff_publish(self._h, request_id, image_index, C.c_void_p(ptr), nbytes,
                                                  C.c_void_p(stream)))

    def complete(self, request_id: int):
        """(all images published?, bytes published so far)"""
        n = C.c_size_t(0)
        done = load_library().vit_handoff_complete(self._h, request_id, C.byref(n))
        return bool(done), int(n.value)

    def pull(self, request_id: int, dst_ptr: int, capacity: int, stream: int = 0) -> int:
        n = C.c_size_t(0)
        _check(load_library().vit_handoff_pull(self._h, request_id, C.c_void_p(dst_ptr), capacity, C.c_void_p(stream),
                                               C.byref(n)))
        return int(n.value)

    def release(self, request_id: int):
        _check(load_library().vit_handoff_release(self._h, request_id))


def check_pixels(cfg: dict, pixels_shape, tile_offsets) -> None:
    """The C ABI takes `pixels` as a bare pointer: the tile count it reads is tile_offsets[-1].  Refuse a tensor
    that does not hold exactly that many [C, S, S] tiles before the library reads past it."""
    to = np.asarray(tile_offsets)
    want = (int(cfg["channels"]), int(cfg["image_size"]), int(cfg["image_size"]))
    if len(pixels_shape) != 4 or tuple(int(v) for v in pixels_shape[1:]) != want:
        raise VitError(VIT_EINVAL, f"pixels must be [n_tiles, {want[0]}, {want[1]}, {want[2]}], got {tuple(pixels_shape)}")
    if to.size == 0 or int(to[-1]) != int(pixels_shape[0]):
        raise VitError(VIT_EINVAL, f"tile_offsets ends at {int(to[-1]) if to.size else None} but pixels holds "
                                   f"{int(pixels_shape[0])} tiles")


# ---- convenience wrapper: torch tensors for device memory and the stream ----------------
class VitEncoder:
    """Owns a handle; allocates output/workspace tensors with torch and passes raw pointers."""

    def __init__(self, cfg: dict, weights: np.ndarray, device: int = 0):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("VitEncoder needs a HIP device; there is no CPU path")
        self.cfg = dict(cfg)
        self.device = device
        self._torch = torch
        self._handle = vit_encoder_create(cfg, weights, device)
        self._ws = None

    def close(self):
        if self._handle:
            self._torch.cuda.synchronize(self.device)
            vit_encoder_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._handle

    def query(self, n_tiles: int, n_images: int):
        return vit_encoder_query(self._handle, n_tiles, n_images)

    def encode(self, pixels, images_per_request, tile_offsets, out=None, graph=False):
        """pixels: torch fp32 device tensor [n_tiles, C, S, S].  Returns (tokens, request_token_offsets).
        graph=True goes through vit_encode_packed_graph, which replays a recorded launch sequence from the third call
        with the same `pixels` and `out` tensors and batch shape on (pass `out`: a fresh one per call never repeats)."""
        torch = self._torch
        assert pixels.is_cuda and pixels.dtype == torch.float32 and pixels.is_contiguous()
        check_pixels(self.cfg, pixels.shape, tile_offsets)
        n_tiles = int(pixels.shape[0])
        n_images = int(np.asarray(tile_offsets).size - 1)
        n_tok, out_dim, out_bytes, ws_bytes = self.query(n_tiles, n_images)
        dt = torch.bfloat16 if self.cfg["dtype"] == "bf16" else torch.float32
        if out is None:
            out = torch.empty((n_tok, out_dim), dtype=dt, device=pixels.device)
        assert out.is_contiguous() and out.dtype == dt
        if self._ws is None or self._ws.numel() < ws_bytes:
            self._ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=pixels.device)
        stream = torch.cuda.current_stream(pixels.device).cuda_stream
        call = vit_encode_packed_graph if graph else vit_encode_packed
        rto = call(self._handle, pixels.data_ptr(), images_per_request, tile_offsets, out.data_ptr(),
                   out.numel() * out.element_size(), self._ws.data_ptr(), self._ws.numel(), stream)
        return out, rto

    def profile_enable(self, on: bool = True):
        _check(load_library().vit_profile_enable(self._handle, 1 if on else 0))

    def profile_read(self):
        """{family: (total ms, launches)}; "gemm" is the sum over the matrix-product families."""
        k = len(PROF_FAMILIES)
        ms = (C.c_double * k)()
        n = (C.c_int64 * k)()
        _check(load_library().vit_profile_read(self._handle, ms, n))
        prof = {PROF_FAMILIES[i]: (ms[i], n[i]) for i in range(k)}
        products = [v for f, v in prof.items() if f.startswith("gemm_")]
        prof["gemm"] = (sum(v[0] for v in products), sum(v[1] for v in products))
        return prof

    def profile_tiles_enable(self, on: bool = True):
        _check(load_library().vit_profile_tiles_enable(self._handle, 1 if on else 0))

    def profile_tiles_read(self):
        """{family: (k-loop us per tile, epilogue us per tile, shader clock MHz, tiles stamped)} of each family's
        last launch on the persistent matrix-product kernel."""
        k = len(PROF_FAMILIES)
        main, epi, mhz, n = (C.c_double * k)(), (C.c_double * k)(), (C.c_double * k)(), (C.c_int64 * k)()
        _check(load_library().vit_profile_tiles_read(self._handle, main, epi, mhz, n))
        return {PROF_FAMILIES[i]: (main[i], epi[i], mhz[i], n[i]) for i in range(k) if n[i] > 0}
