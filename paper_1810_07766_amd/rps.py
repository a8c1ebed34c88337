"""Thin ctypes binding of the HIP library's C ABI (include/rps.h).

Argument marshalling only: every step of the round runs in the library's HIP
kernels.  PyTorch supplies device memory and the stream, nothing else.  There is
no CPU fallback: if the shared library is missing, importing this module raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librps.so")

RPS_OK, RPS_EINVAL, RPS_ENOMEM, RPS_EHIP, RPS_EUNSUPPORTED, RPS_ETOOBIG = 0, -1, -2, -3, -4, -5
RPS_DTYPE_F32, RPS_DTYPE_BF16 = 0, 1
RPS_FLAG_SERVER_IDENTITY = 1
RPS_FLAG_LAYOUT_TILED = 2
RPS_TILE_BYTES = 128

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built: run `python -m paper_1810_07766_amd.build` (hipcc, gfx950). "
        "There is no fallback path.")
# The tensors this binding is handed are PyTorch's, and PyTorch ships its own copy of the HIP
# runtime: it has to be the one already in the process when the library is loaded, so that both
# talk to the same runtime (loaded the other way round, the library binds to the system copy, the
# process ends up with two runtimes, and the library's first HIP call reports no device).
import torch  # noqa: E402,F401
_lib = ctypes.CDLL(LIB_PATH)

_ctx_p = ctypes.c_void_p
_lib.rps_create.argtypes = [ctypes.POINTER(_ctx_p), ctypes.c_int32, ctypes.c_int64,
                            ctypes.POINTER(ctypes.c_int64), ctypes.c_double, ctypes.c_float,
                            ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p]
_lib.rps_create_external.argtypes = [ctypes.POINTER(_ctx_p), ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                     ctypes.POINTER(ctypes.c_int64), ctypes.c_double, ctypes.c_float,
                                     ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p]
_lib.rps_storage_elems.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32]
_lib.rps_storage_elems.restype = ctypes.c_int64
_lib.rps_destroy.argtypes = [_ctx_p]
_lib.rps_set_synthetic_grad.argtypes = [_ctx_p, ctypes.c_float, ctypes.c_float]
_lib.rps_set_gamma.argtypes = [_ctx_p, ctypes.c_float]
_lib.rps_set_row_pitch.argtypes = [_ctx_p, ctypes.c_int64]
_lib.rps_recommended_row_pitch.argtypes = [ctypes.c_int64, ctypes.c_int32]
_lib.rps_recommended_row_pitch.restype = ctypes.c_int64
_lib.rps_local_step.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
_lib.rps_lossy_average.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_uint64]
_lib.rps_round.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
_lib.rps_round_gradient_averaging.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
_lib.rps_get_masks.argtypes = [_ctx_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.rps_masks_host.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_uint64, ctypes.c_uint32,
                                ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.rps_set_mask_override.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.rps_consensus.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
_lib.rps_consensus_static.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32,
                                      ctypes.c_void_p, ctypes.c_void_p]
_lib.rps_estimate_mixing.argtypes = [_ctx_p, ctypes.c_uint64, ctypes.c_int64, ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_double)]
_lib.rps_convert_layout.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
_lib.rps_set_launch_tuning.argtypes = [_ctx_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
_lib.rps_noise_cells.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
_lib.rps_query_occupancy.argtypes = [_ctx_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
_lib.rps_set_profiling.argtypes = [_ctx_p, ctypes.c_int32]
_lib.rps_get_kernel_time.argtypes = [_ctx_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
_lib.rps_get_kernel_times.argtypes = [_ctx_p, ctypes.c_void_p, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
_lib.rps_last_hip_error.argtypes = [_ctx_p]
_lib.rps_strerror.argtypes = [ctypes.c_int]
_lib.rps_strerror.restype = ctypes.c_char_p
for _name in ("rps_create", "rps_create_external", "rps_destroy", "rps_set_synthetic_grad", "rps_set_gamma", "rps_set_row_pitch", "rps_local_step",
              "rps_lossy_average", "rps_round", "rps_round_gradient_averaging", "rps_get_masks", "rps_masks_host", "rps_set_mask_override",
              "rps_consensus", "rps_consensus_static", "rps_estimate_mixing", "rps_convert_layout", "rps_set_launch_tuning", "rps_query_occupancy", "rps_noise_cells", "rps_set_profiling", "rps_get_kernel_time", "rps_get_kernel_times", "rps_last_hip_error"):
    getattr(_lib, _name).restype = ctypes.c_int

EXPORTS = ("rps_create", "rps_create_external", "rps_storage_elems", "rps_destroy", "rps_set_synthetic_grad", "rps_set_gamma",
           "rps_set_row_pitch", "rps_recommended_row_pitch", "rps_local_step",
           "rps_lossy_average", "rps_round", "rps_round_gradient_averaging", "rps_get_masks", "rps_masks_host", "rps_set_mask_override",
           "rps_consensus", "rps_consensus_static", "rps_estimate_mixing", "rps_convert_layout", "rps_set_launch_tuning", "rps_query_occupancy", "rps_noise_cells", "rps_set_profiling", "rps_get_kernel_time", "rps_get_kernel_times",
           "rps_last_hip_error",
           "rps_strerror")


class RpsError(RuntimeError):
    def __init__(self, code, hip=0):
        self.code, self.hip = code, hip
        msg = _lib.rps_strerror(code).decode()
        super().__init__(f"rps error {code}: {msg}" + (f" (hipError_t {hip})" if hip else ""))


def _check(code, ctx=None):
    if code != RPS_OK:
        raise RpsError(code, _lib.rps_last_hip_error(ctx) if code == RPS_EHIP else 0)


def rps_strerror(code: int) -> str:
    return _lib.rps_strerror(code).decode()


def _ptr(t, ctx):
    """Device pointer of a torch tensor after checking it is what the ABI expects."""
    import torch
    if t is None:
        return None
    want = torch.float32 if ctx.dtype == RPS_DTYPE_F32 else torch.bfloat16
    if not (t.is_cuda and t.dtype == want):
        raise RpsError(RPS_EINVAL)
    if ctx.flags & RPS_FLAG_LAYOUT_TILED:      # [tiles, n, tile width], see rps.h
        T = RPS_TILE_BYTES // t.element_size()
        if not t.is_contiguous() or tuple(t.shape) != ((ctx.N + T - 1) // T, ctx.n, T):
            raise RpsError(RPS_EINVAL)
    else:                                      # [n, N] with the context's row pitch
        if tuple(t.shape) != (ctx.n, ctx.N) or (ctx.N > 1 and t.stride(1) != 1) or (ctx.n > 1 and t.stride(0) != ctx.pitch):
            raise RpsError(RPS_EINVAL)
    return ctypes.c_void_p(t.data_ptr())


class RpsContext:
    """Owns one rps_ctx handle.  Methods mirror the C entry points one to one."""

    def __init__(self, n, N, p, gamma, seed, dtype=RPS_DTYPE_F32, block_offsets=None, flags=0, stream=None,
                 external_servers=0):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        nb = external_servers if external_servers else n
        off = None
        if block_offsets is not None:
            vals = [int(v) for v in block_offsets]
            if len(vals) != nb + 1:
                raise RpsError(RPS_EINVAL)
            off = (ctypes.c_int64 * (nb + 1))(*vals)
        handle = _ctx_p()
        if external_servers:
            _check(_lib.rps_create_external(ctypes.byref(handle), n, external_servers, N, off, p, gamma, seed, dtype,
                                            ctypes.c_void_p(stream)))
        else:
            _check(_lib.rps_create(ctypes.byref(handle), n, N, off, p, gamma, seed, dtype, flags,
                                   ctypes.c_void_p(stream)))
        self._h = handle
        self.n, self.N, self.dtype, self.blocks, self.flags, self.pitch = n, N, dtype, nb, flags, N

    def destroy(self):
        if getattr(self, "_h", None) and _lib is not None:   # (_lib is None at interpreter shutdown)
            h, self._h = self._h, None
            _check(_lib.rps_destroy(h))

    __del__ = destroy

    def set_synthetic_grad(self, sigma, weight_decay=0.0):
        _check(_lib.rps_set_synthetic_grad(self._h, sigma, weight_decay), self._h)

    def set_gamma(self, gamma):
        _check(_lib.rps_set_gamma(self._h, gamma), self._h)

    def set_row_pitch(self, pitch):
        """Row-major: X and G are views [n, N] of arrays whose rows are `pitch` elements apart."""
        _check(_lib.rps_set_row_pitch(self._h, pitch), self._h)
        self.pitch = pitch

    def empty_state(self, fill=None):
        """New row-major state tensor [n, N] with the context's row pitch (a view of [n, pitch])."""
        import torch
        dt = torch.float32 if self.dtype == RPS_DTYPE_F32 else torch.bfloat16
        buf = torch.empty(self.n, self.pitch, device="cuda", dtype=dt) if fill is None else \
            torch.full((self.n, self.pitch), fill, device="cuda", dtype=dt)
        return buf[:, : self.N]

    def local_step(self, X, G, step):
        _check(_lib.rps_local_step(self._h, _ptr(X, self), _ptr(G, self), step), self._h)

    def lossy_average(self, X, step):
        _check(_lib.rps_lossy_average(self._h, _ptr(X, self), step), self._h)

    def round(self, X, G, step):
        _check(_lib.rps_round(self._h, _ptr(X, self), _ptr(G, self), step), self._h)

    def round_gradient_averaging(self, X, G, step):
        if G is None:
            raise RpsError(RPS_EINVAL)
        _check(_lib.rps_round_gradient_averaging(self._h, _ptr(X, self), _ptr(G, self), step), self._h)

    def get_masks(self, step):
        import numpy as np
        n, nb = self.n, self.blocks
        up = np.empty((n, nb), dtype=np.uint8)
        down = np.empty((n, nb), dtype=np.uint8)
        server = np.empty(nb, dtype=np.int32)
        _check(_lib.rps_get_masks(self._h, step, up.ctypes.data, down.ctypes.data, server.ctypes.data), self._h)
        return server, up, down

    def set_mask_override(self, server=None, up=None, down=None):
        import numpy as np
        if server is None and up is None and down is None:
            _check(_lib.rps_set_mask_override(self._h, None, None, None), self._h)
            return
        up = np.ascontiguousarray(up, dtype=np.uint8)
        down = np.ascontiguousarray(down, dtype=np.uint8)
        server = np.ascontiguousarray(server, dtype=np.int32)
        if up.shape != (self.n, self.blocks) or down.shape != (self.n, self.blocks) or server.shape != (self.blocks,):
            raise RpsError(RPS_EINVAL)
        _check(_lib.rps_set_mask_override(self._h, up.ctypes.data, down.ctypes.data, server.ctypes.data), self._h)

    def consensus(self, X):
        """(sum_i ||x_i - xbar||^2, ||xbar||^2) of the state."""
        d, m = ctypes.c_double(), ctypes.c_double()
        _check(_lib.rps_consensus(self._h, _ptr(X, self), ctypes.byref(d), ctypes.byref(m)), self._h)
        return d.value, m.value

    def estimate_mixing(self, first_step, rounds):
        """Monte-Carlo (alpha1, alpha2) of the mixing matrix over the generated outcomes of `rounds` steps."""
        a1, a2 = ctypes.c_double(), ctypes.c_double()
        _check(_lib.rps_estimate_mixing(self._h, first_step, rounds, ctypes.byref(a1), ctypes.byref(a2)), self._h)
        return a1.value, a2.value

    def to_tiled(self, X):
        """Row-major [n, N] tensor -> new tile-major tensor [tiles, n, T] (device copy by the library)."""
        import torch
        want = torch.float32 if self.dtype == RPS_DTYPE_F32 else torch.bfloat16
        if not (X.is_cuda and X.dtype == want and tuple(X.shape) == (self.n, self.N)
                and (self.N == 1 or X.stride(1) == 1) and (self.n == 1 or X.stride(0) == self.pitch)):
            raise RpsError(RPS_EINVAL)
        T = RPS_TILE_BYTES // X.element_size()
        out = torch.empty((self.N + T - 1) // T, self.n, T, device=X.device, dtype=X.dtype)
        _check(_lib.rps_convert_layout(self._h, out.data_ptr(), X.data_ptr(), 1), self._h)
        return out

    def from_tiled(self, Xt):
        """Tile-major tensor -> new row-major [n, N] tensor."""
        import torch
        want = torch.float32 if self.dtype == RPS_DTYPE_F32 else torch.bfloat16
        T = RPS_TILE_BYTES // Xt.element_size()
        if not (Xt.is_cuda and Xt.is_contiguous() and Xt.dtype == want
                and tuple(Xt.shape) == ((self.N + T - 1) // T, self.n, T)):
            raise RpsError(RPS_EINVAL)
        out = torch.empty(self.n, self.pitch, device=Xt.device, dtype=Xt.dtype)[:, : self.N]
        _check(_lib.rps_convert_layout(self._h, out.data_ptr(), Xt.data_ptr(), 0), self._h)
        return out

    def set_launch_tuning(self, rows_in_flight, waves_per_workgroup, max_waves_per_cu=0, tiles_per_wave=0):
        _check(_lib.rps_set_launch_tuning(self._h, rows_in_flight, waves_per_workgroup, max_waves_per_cu, tiles_per_wave),
               self._h)

    def query_occupancy(self, gradient_source):
        """Wavefronts of the round kernel per compute unit with this context's launch shape
        (gradient_source: 0 none, 1 buffer, 2 in-register)."""
        waves = ctypes.c_int32(0)
        _check(_lib.rps_query_occupancy(self._h, gradient_source, ctypes.byref(waves)), self._h)
        return waves.value

    def set_profiling(self, enable):
        _check(_lib.rps_set_profiling(self._h, 1 if enable else 0), self._h)

    def get_kernel_times(self, capacity=4096):
        """Per-launch kernel milliseconds (numpy array) since profiling was enabled / last read."""
        import numpy as np
        ms = np.zeros(capacity, dtype=np.float64)
        cnt = ctypes.c_int64()
        _check(_lib.rps_get_kernel_times(self._h, ms.ctypes.data, capacity, ctypes.byref(cnt)), self._h)
        return ms[: min(cnt.value, capacity)]

    def get_kernel_time(self):
        """(total kernel milliseconds, launches) since profiling was enabled / last read."""
        ms, cnt = ctypes.c_double(), ctypes.c_int64()
        _check(_lib.rps_get_kernel_time(self._h, ctypes.byref(ms), ctypes.byref(cnt)), self._h)
        return ms.value, cnt.value


# function-style aliases with the C names
def rps_create(n, N, block_offsets, p, gamma, seed, dtype=RPS_DTYPE_F32, flags=0, stream=None):
    return RpsContext(n, N, p, gamma, seed, dtype, block_offsets, flags, stream)


def rps_create_external(n, servers, N, block_offsets, p, gamma, seed, dtype=RPS_DTYPE_F32, stream=None):
    return RpsContext(n, N, p, gamma, seed, dtype, block_offsets, 0, stream, external_servers=servers)


def rps_storage_elems(n, N, dtype=RPS_DTYPE_F32, flags=0):
    return _lib.rps_storage_elems(n, N, dtype, flags)


def rps_destroy(ctx):
    ctx.destroy()


def rps_set_synthetic_grad(ctx, sigma, weight_decay=0.0):
    ctx.set_synthetic_grad(sigma, weight_decay)


def rps_set_gamma(ctx, gamma):
    ctx.set_gamma(gamma)


def rps_set_row_pitch(ctx, pitch):
    ctx.set_row_pitch(pitch)


def rps_recommended_row_pitch(N, dtype=RPS_DTYPE_F32):
    return _lib.rps_recommended_row_pitch(N, dtype)


def rps_local_step(ctx, X, G, step):
    ctx.local_step(X, G, step)


def rps_lossy_average(ctx, X, step):
    ctx.lossy_average(X, step)


def rps_round(ctx, X, G, step):
    ctx.round(X, G, step)


def rps_round_gradient_averaging(ctx, X, G, step):
    ctx.round_gradient_averaging(X, G, step)


def rps_get_masks(ctx, step):
    return ctx.get_masks(step)


def rps_masks_host(n, p, seed, step, flags=0, servers=0):
    """(server, up, down) of `step` from the library's host copy of the generator (no GPU)."""
    import numpy as np
    nb = servers if servers > 0 else n
    up = np.empty((max(n, 0), max(nb, 0)), dtype=np.uint8)
    down = np.empty_like(up)
    server = np.empty(max(nb, 0), dtype=np.int32)
    _check(_lib.rps_masks_host(n, servers, p, seed, flags, step, up.ctypes.data, down.ctypes.data, server.ctypes.data))
    return server, up, down


def rps_consensus(ctx, X):
    return ctx.consensus(X)


def rps_consensus_static(X, n, N, out, dtype=RPS_DTYPE_F32, flags=0, stream=None):
    """Allocation-free consensus statistics: X a device tensor holding the state, out a device
    tensor of 2 float64 that receives (distance, ||xbar||^2) in stream order."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    if not (out.is_cuda and out.is_contiguous() and out.dtype == torch.float64 and out.numel() == 2
            and X.is_cuda and X.is_contiguous()):
        raise RpsError(RPS_EINVAL)
    _check(_lib.rps_consensus_static(ctypes.c_void_p(X.data_ptr()), n, N, dtype, flags, ctypes.c_void_p(out.data_ptr()),
                                     ctypes.c_void_p(stream)))


def rps_noise_cells():
    """(radius[4096], cos_sin[4096, 2]) float32 as the library computes them on the host."""
    import numpy as np
    radius = np.empty(4096, dtype=np.float32)
    cos_sin = np.empty((4096, 2), dtype=np.float32)
    _check(_lib.rps_noise_cells(radius.ctypes.data, cos_sin.ctypes.data))
    return radius, cos_sin


def rps_estimate_mixing(ctx, first_step, rounds):
    return ctx.estimate_mixing(first_step, rounds)


def rps_convert_layout(ctx, X, to_tiled):
    return ctx.to_tiled(X) if to_tiled else ctx.from_tiled(X)


def rps_set_mask_override(ctx, server=None, up=None, down=None):
    ctx.set_mask_override(server, up, down)
