"""Thin ctypes binding of libpcr.so (include/pcr.h).  Argument marshalling only: every step of
the decode path runs in the library's HIP kernels.  PyTorch is used for device memory and the
current stream.  There is no CPU fallback: without the built library, or without a GPU for the
calls that need one, these functions raise."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpcr.so")

OK, E_ARG, E_FORMAT, E_TRUNCATED, E_UNSUPPORTED, E_RANGE, E_NOMEM, E_DEVICE = 0, -1, -2, -3, -4, -5, -6, -7
NUM_STAGES = 9
STAGE_NAMES = ("index_parse", "unstuff", "dc_first", "ac_first", "ac_refine", "refine_blocks", "refine_apply", "pixel", "sequential")

# every symbol include/pcr.h declares: name -> (restype, argtypes)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_vp = ctypes.c_void_p
SYMBOLS = {
    "pcr_open": (ctypes.c_int, [_vp, ctypes.c_size_t, ctypes.c_int, ctypes.POINTER(_vp)]),
    "pcr_open_device": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, ctypes.POINTER(_vp)]),
    "pcr_rebind_device": (ctypes.c_int, [_vp, _vp, ctypes.c_size_t, _vp]),
    "pcr_close": (None, [_vp]),
    "pcr_num_images": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int)]),
    "pcr_num_scan_groups": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int)]),
    "pcr_available_scan_groups": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int)]),
    "pcr_group_end_offset": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_image_info": (ctypes.c_int, [_vp, ctypes.c_int] + [ctypes.POINTER(ctypes.c_int)] * 3 + [ctypes.POINTER(ctypes.c_int32)]),
    "pcr_output_layout": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_index": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint32)]),
    "pcr_reassemble": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, _u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]),
    "pcr_coef_layout": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_decode_coefficients": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp]),
    "pcr_decode_batch": (ctypes.c_int, [_vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp, _vp]),
    "pcr_decode_batch_triangle": (ctypes.c_int, [_vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp, _vp]),
    "pcr_decode_batch_smooth": (ctypes.c_int, [_vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp, _vp]),
    "pcr_upgrade_batch": (ctypes.c_int, [_vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp, _vp]),
    "pcr_resident_scan_group": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int)]),
    "pcr_enable_stage_timing": (ctypes.c_int, [_vp, ctypes.c_int]),
    "pcr_set_lane_decoders": (ctypes.c_int, [_vp, ctypes.c_int]),
    "pcr_last_decoder_shapes": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "pcr_last_stage_ms": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_float)]),
    "pcr_probe_scalar_issue_rate": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]),
    "pcr_stage_ms_history": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32)]),
    "pcr_crop_resize_batch": (ctypes.c_int, [_vp, _vp, _vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float),
                                             ctypes.POINTER(ctypes.c_float), _vp, ctypes.c_size_t, _vp]),
    "pcr_decode_crop_batch": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float),
                                             ctypes.POINTER(ctypes.c_float), _vp, ctypes.c_size_t, _vp, _vp]),
    "pcr_msssim_batch": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "pcr_msssim_batch_static": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "pcr_scan_ends": (ctypes.c_int, [_vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]),
    "pcr_record_size": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_size_t), ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint64),
                                       ctypes.POINTER(ctypes.c_uint32)]),
    "pcr_record_write": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_size_t), _vp, ctypes.c_uint32, _vp, ctypes.c_size_t,
                                        ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_record_write_indexed": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_size_t), _vp, ctypes.c_uint32, ctypes.c_uint32, _vp,
                                                ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_transcode_progressive": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, ctypes.c_size_t, ctypes.c_uint32, _vp, ctypes.c_size_t,
                                                 ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_symbol_histograms": (ctypes.c_int, [_vp, ctypes.c_uint32, _vp, _vp]),
    "pcr_transcode_progressive_counted": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, ctypes.c_size_t, ctypes.c_uint32, _vp, _vp, ctypes.c_size_t,
                                                         ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_transcode_symbol_counts": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, ctypes.c_size_t, ctypes.c_uint32, _vp]),
    "pcr_select_scan_group": (ctypes.c_int, [_vp, ctypes.c_float, _vp, _vp, ctypes.c_size_t, _vp, ctypes.POINTER(ctypes.c_float),
                                             ctypes.POINTER(ctypes.c_int), _vp]),
    "pcr_prefix_length": (ctypes.c_int, [_vp, ctypes.c_size_t, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64)]),
    "pcr_loader_create": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(_vp)]),
    "pcr_loader_destroy": (None, [_vp]),
    "pcr_loader_staging": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_size_t)]),
    "pcr_loader_stream": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(_vp)]),
    "pcr_loader_set_rate": (ctypes.c_int, [_vp, ctypes.c_double, ctypes.c_double]),
    "pcr_loader_upload": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(_vp)]),
    "pcr_loader_read_file": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(_vp)]),
    "pcr_loader_decode": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, _vp, ctypes.c_size_t, _vp]),
    "pcr_loader_decode_crop": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, _vp, _vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float), _vp, ctypes.c_size_t, _vp]),
    "pcr_loader_wait": (ctypes.c_int, [_vp, ctypes.c_int]),
    "pcr_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}

_lib = None


class PcrError(RuntimeError):
    def __init__(self, code, what=""):
        msg = lib().pcr_strerror(code).decode() if _lib is not None else str(code)
        super().__init__("%s failed: %s (%d)" % (what or "pcr call", msg, code))
        self.code = code


def lib():
    """Load libpcr.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpcr.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(or paper_1911_00472_amd/build.py) first; there is no fallback path")
        try:
            import torch  # noqa: F401  (PyTorch brings its own copy of the HIP runtime; it must be the first one this process
        except ImportError:                  # loads, or its later initialisation finds no GPU: libpcr.so then binds to the same copy)
            pass
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            f = getattr(L, name)
            f.restype = res
            f.argtypes = args
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise PcrError(rc, what)


class Record:
    """One opened PCR record (pcr_open ... pcr_close)."""

    def __init__(self, data, device=0, stream=None, _borrowed_handle=None):
        self._h = _vp()
        self._keep = None
        self._owned = _borrowed_handle is None
        if _borrowed_handle is not None:                    # a loader slot's handle: the loader closes it
            self._h = _vp(_borrowed_handle)
        elif hasattr(data, "data_ptr"):                       # a CUDA uint8 tensor: bytes already on the device (borrowed)
            import torch
            assert data.is_cuda and data.dtype == torch.uint8 and data.is_contiguous()
            device = data.device.index
            s = torch.cuda.current_stream(device).cuda_stream if stream is None else stream
            _check(lib().pcr_open_device(data.data_ptr(), data.numel(), s, ctypes.byref(self._h)), "pcr_open_device")
            self._keep = data
        else:
            buf = np.frombuffer(data, np.uint8) if not isinstance(data, np.ndarray) else data
            _check(lib().pcr_open(buf.ctypes.data_as(_vp), buf.size, device, ctypes.byref(self._h)), "pcr_open")
        self.device = device
        self._refresh()

    def _refresh(self):
        v = ctypes.c_int()
        _check(lib().pcr_num_images(self._h, ctypes.byref(v)), "pcr_num_images"); self.n = v.value
        _check(lib().pcr_num_scan_groups(self._h, ctypes.byref(v)), "pcr_num_scan_groups"); self.G = v.value
        _check(lib().pcr_available_scan_groups(self._h, ctypes.byref(v)), "pcr_available_scan_groups"); self.k_avail = v.value

    def rebind_device(self, tensor, stream=None):
        """Bind this handle to another record (a CUDA uint8 tensor, borrowed), re-using its device buffers."""
        import torch
        assert tensor.is_cuda and tensor.dtype == torch.uint8 and tensor.is_contiguous() and tensor.device.index == self.device
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        self.n = self.G = self.k_avail = 0
        _check(lib().pcr_rebind_device(self._h, tensor.data_ptr(), tensor.numel(), s), "pcr_rebind_device")
        self._keep = tensor
        self._refresh()

    def close(self):
        if self._h:
            if self._owned:
                lib().pcr_close(self._h)
            self._h = _vp()
            self._keep = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def group_end_offset(self, k):
        v = ctypes.c_uint64()
        _check(lib().pcr_group_end_offset(self._h, k, ctypes.byref(v)), "pcr_group_end_offset")
        return v.value

    def image_info(self, i):
        w, h, c, lab = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int32()
        _check(lib().pcr_image_info(self._h, i, ctypes.byref(w), ctypes.byref(h), ctypes.byref(c), ctypes.byref(lab)), "pcr_image_info")
        return w.value, h.value, c.value, lab.value

    def output_layout(self):
        self._refresh()                                      # (a loader slot's handle may have been bound to another record)
        o = np.zeros(self.n + 1, np.uint64)
        _check(lib().pcr_output_layout(self._h, o.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))), "pcr_output_layout")
        return o

    def coef_layout(self):
        self._refresh()
        o = np.zeros(self.n + 1, np.uint64)
        _check(lib().pcr_coef_layout(self._h, o.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))), "pcr_coef_layout")
        return o

    def index(self):
        off = np.zeros((self.G, self.n), np.uint64)
        ln = np.zeros((self.G, self.n), np.uint32)
        _check(lib().pcr_index(self._h, off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                               ln.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))), "pcr_index")
        return off, ln

    def reassemble(self, i, k):
        L = ctypes.c_size_t()
        _check(lib().pcr_reassemble(self._h, i, k, None, 0, ctypes.byref(L)), "pcr_reassemble")
        out = np.empty(L.value, np.uint8)
        _check(lib().pcr_reassemble(self._h, i, k, out.ctypes.data_as(_u8p), out.size, ctypes.byref(L)), "pcr_reassemble")
        return out.tobytes()

    def decode_coefficients(self, k, out=None, stream=None):
        """int16 CUDA tensor of coef_layout()[n] elements (asynchronous on the stream)."""
        import torch
        if out is None:
            out = torch.empty(int(self.coef_layout()[-1]), dtype=torch.int16, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_decode_coefficients(self._h, k, out.data_ptr(), s), "pcr_decode_coefficients")
        return out

    def decode_batch(self, k, out=None, status=None, stream=None):
        """uint8 CUDA tensor of output_layout()[n] bytes, ragged NHWC (asynchronous on the stream)."""
        import torch
        if out is None:
            out = torch.empty(int(self.output_layout()[-1]), dtype=torch.uint8, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_decode_batch(self._h, k, out.data_ptr(), out.numel(), s, status.data_ptr() if status is not None else None),
               "pcr_decode_batch")
        return out

    def decode_batch_triangle(self, k, out=None, status=None, stream=None):
        """decode_batch with sub-sampled chroma interpolated by the triangle filter instead of replicated."""
        import torch
        if out is None:
            out = torch.empty(int(self.output_layout()[-1]), dtype=torch.uint8, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_decode_batch_triangle(self._h, k, out.data_ptr(), out.numel(), s, status.data_ptr() if status is not None else None),
               "pcr_decode_batch_triangle")
        return out

    def decode_batch_smooth(self, k, out=None, status=None, stream=None):
        """decode_batch with the five lowest AC coefficients of components that hold only their DC first scan predicted
        from the neighbouring DC coefficients."""
        import torch
        if out is None:
            out = torch.empty(int(self.output_layout()[-1]), dtype=torch.uint8, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_decode_batch_smooth(self._h, k, out.data_ptr(), out.numel(), s, status.data_ptr() if status is not None else None),
               "pcr_decode_batch_smooth")
        return out

    def symbol_histograms(self, restart_interval=0, out=None, stream=None):
        """uint32 CUDA tensor [n, 10, 2, 256]: per image, scan of the transcoder's script and table slot, how often each
        Huffman symbol occurs in the progressive file transcode_progressive would write (counted on the device)."""
        import torch
        if out is None:
            out = torch.empty((self.n, HIST_SCANS, 2, 256), dtype=torch.int32, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_symbol_histograms(self._h, restart_interval, out.data_ptr(), s), "pcr_symbol_histograms")
        return out

    def upgrade_batch(self, k, out=None, status=None, stream=None):
        """As decode_batch, but decodes only the scan groups above resident_scan_group() on top of the planes the
        previous decode_batch / upgrade_batch left on the device."""
        import torch
        if out is None:
            out = torch.empty(int(self.output_layout()[-1]), dtype=torch.uint8, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_upgrade_batch(self._h, k, out.data_ptr(), out.numel(), s, status.data_ptr() if status is not None else None),
               "pcr_upgrade_batch")
        return out

    def crop_resize_batch(self, pixels, crops, out_h, out_w, mean, inv_std, out=None, stream=None):
        """pixels: uint8 CUDA tensor in output_layout(); crops: int32 CUDA tensor [n, 5] (x0, y0, w, h, flip).
        Returns a float16 CUDA tensor [n, C, out_h, out_w] (asynchronous on the stream)."""
        import torch
        assert crops.is_cuda and crops.dtype == torch.int32 and crops.is_contiguous() and tuple(crops.shape) == (self.n, 5)
        C = self.image_info(0)[2]
        if out is None:
            out = torch.empty((self.n, C, out_h, out_w), dtype=torch.float16, device="cuda:%d" % self.device)
        m = (ctypes.c_float * 3)(*([float(v) for v in mean] + [0.0] * 3)[:3])
        sd = (ctypes.c_float * 3)(*([float(v) for v in inv_std] + [1.0] * 3)[:3])
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_crop_resize_batch(self._h, pixels.data_ptr(), crops.data_ptr(), out_h, out_w, m, sd, out.data_ptr(),
                                           out.numel() * 2, s), "pcr_crop_resize_batch")
        return out

    def msssim_batch(self, a, b, out=None, stream=None):
        """Multi-scale structural similarity of every image's pictures in two decoded batches (uint8 CUDA tensors
        in output_layout()).  Returns a float32 CUDA tensor [n] (asynchronous on the stream)."""
        import torch
        total = int(self.output_layout()[-1])
        for t in (a, b):
            assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous() and t.numel() >= total
        if out is None:
            out = torch.empty(self.n, dtype=torch.float32, device="cuda:%d" % self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_msssim_batch(self._h, a.data_ptr(), b.data_ptr(), out.data_ptr(), s), "pcr_msssim_batch")
        return out

    def msssim_batch_static(self, a, b, out, stream=None):
        """msssim_batch through the entry point that allocates nothing: `out` (float32 CUDA tensor [n]) is the
        caller's; PcrError(E_RANGE) when the record's tile sums exceed the library's fixed array."""
        import torch
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() >= self.n
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_msssim_batch_static(self._h, a.data_ptr(), b.data_ptr(), out.data_ptr(), s), "pcr_msssim_batch_static")
        return out

    def select_scan_group(self, min_mean_score, stream=None):
        """Lowest scan group whose mean MS-SSIM against the highest available group reaches min_mean_score.
        Returns (scan_group, {group: mean score} for the groups tried)."""
        import torch
        total = int(self.output_layout()[-1])
        dev = "cuda:%d" % self.device
        a = torch.empty(total, dtype=torch.uint8, device=dev)
        b = torch.empty(total, dtype=torch.uint8, device=dev)
        scores = torch.empty(self.n, dtype=torch.float32, device=dev)
        means = (ctypes.c_float * self.G)()
        k = ctypes.c_int(0)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_select_scan_group(self._h, float(min_mean_score), a.data_ptr(), b.data_ptr(), total, scores.data_ptr(), means,
                                           ctypes.byref(k), s), "pcr_select_scan_group")
        return int(k.value), {g + 1: float(means[g]) for g in range(self.G) if means[g] >= 0}

    def decode_crop_batch(self, k, crops, out_h, out_w, mean, inv_std, pixels=None, out=None, status=None, stream=None):
        """decode_batch(k) + crop_resize_batch in one call.  pixels=None: one fused kernel, the full-resolution pixels
        never reach memory; otherwise a uint8 CUDA working buffer of output_layout()[n] bytes that receives the parts of
        the pictures the boxes touch.  Returns the float16 tensor."""
        import torch
        assert crops.is_cuda and crops.dtype == torch.int32 and crops.is_contiguous() and tuple(crops.shape) == (self.n, 5)
        C = self.image_info(0)[2]
        if out is None:
            out = torch.empty((self.n, C, out_h, out_w), dtype=torch.float16, device="cuda:%d" % self.device)
        m = (ctypes.c_float * 3)(*([float(v) for v in mean] + [0.0] * 3)[:3])
        sd = (ctypes.c_float * 3)(*([float(v) for v in inv_std] + [1.0] * 3)[:3])
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().pcr_decode_crop_batch(self._h, k, crops.data_ptr(), pixels.data_ptr() if pixels is not None else None,
                                           pixels.numel() if pixels is not None else 0, out_h, out_w, m, sd,
                                           out.data_ptr(), out.numel() * 2, s, status.data_ptr() if status is not None else None),
               "pcr_decode_crop_batch")
        return out

    def resident_scan_group(self):
        v = ctypes.c_int(0)
        _check(lib().pcr_resident_scan_group(self._h, ctypes.byref(v)), "pcr_resident_scan_group")
        return int(v.value)

    def set_lane_decoders(self, mode):
        _check(lib().pcr_set_lane_decoders(self._h, int(mode)), "pcr_set_lane_decoders")

    def last_decoder_shapes(self):
        """(launches with one lane per unit, launches with one wavefront per unit) of the last decode call's AC scans."""
        a, b = ctypes.c_int(0), ctypes.c_int(0)
        _check(lib().pcr_last_decoder_shapes(self._h, ctypes.byref(a), ctypes.byref(b)), "pcr_last_decoder_shapes")
        return a.value, b.value

    def enable_stage_timing(self, on=True):
        _check(lib().pcr_enable_stage_timing(self._h, 1 if on else 0), "pcr_enable_stage_timing")

    def last_stage_ms(self):
        ms = (ctypes.c_float * NUM_STAGES)()
        _check(lib().pcr_last_stage_ms(self._h, ms), "pcr_last_stage_ms")
        return dict(zip(STAGE_NAMES, (float(x) for x in ms)))

    def stage_ms_history(self):
        """(calls, {stage: (summed ms, timed launches)}) over the calls since timing was switched on."""
        ms = (ctypes.c_double * NUM_STAGES)()
        launches = (ctypes.c_uint32 * NUM_STAGES)()
        calls = ctypes.c_uint32(0)
        _check(lib().pcr_stage_ms_history(self._h, ms, launches, ctypes.byref(calls)), "pcr_stage_ms_history")
        return int(calls.value), {n: (float(ms[i]), int(launches[i])) for i, n in enumerate(STAGE_NAMES)}


def probe_scalar_issue_rate(waves_per_cu, device=0):
    """10^9 dependent scalar-ALU instructions per second the device issues with that many wavefronts per CU."""
    v = ctypes.c_double(0)
    _check(lib().pcr_probe_scalar_issue_rate(device, waves_per_cu, ctypes.byref(v)), "pcr_probe_scalar_issue_rate")
    return float(v.value)


def prefix_length(first_bytes, k):
    """Bytes of a record to read for scan group k, from its first bytes (24 + 8 G always suffice).  Returns
    (True, length), or (False, number of first bytes needed to tell)."""
    buf = np.frombuffer(first_bytes, np.uint8) if not isinstance(first_bytes, np.ndarray) else first_bytes
    need = ctypes.c_uint64(0)
    rc = lib().pcr_prefix_length(buf.ctypes.data_as(_vp), buf.size, k, ctypes.byref(need))
    if rc == E_TRUNCATED:
        return False, int(need.value)
    _check(rc, "pcr_prefix_length")
    return True, int(need.value)


def scan_ends(jpeg):
    """End offset of every scan region of a JPEG file (the last equals len(jpeg))."""
    buf = np.frombuffer(jpeg, np.uint8)
    ends = (ctypes.c_uint64 * 64)()
    n = ctypes.c_int(0)
    _check(lib().pcr_scan_ends(buf.ctypes.data_as(_vp), buf.size, ends, 64, ctypes.byref(n)), "pcr_scan_ends")
    return [int(ends[i]) for i in range(n.value)]


def _file_table(files):
    bufs = [np.frombuffer(f, np.uint8) for f in files]
    ptrs = (_vp * len(bufs))(*[b.ctypes.data for b in bufs])
    sizes = (ctypes.c_size_t * len(bufs))(*[b.size for b in bufs])
    return bufs, ptrs, sizes


def record_write(files, labels=None):
    """One record (bytes) from JPEG files (bytes objects): pcr_record_size + pcr_record_write."""
    bufs, ptrs, sizes = _file_table(files)
    total, G = ctypes.c_uint64(0), ctypes.c_uint32(0)
    _check(lib().pcr_record_size(ptrs, sizes, len(bufs), ctypes.byref(total), ctypes.byref(G)), "pcr_record_size")
    out = np.empty(int(total.value), np.uint8)
    lab = None if labels is None else np.ascontiguousarray(labels, np.int32)
    assert lab is None or lab.size == len(bufs)
    written = ctypes.c_uint64(0)
    _check(lib().pcr_record_write(ptrs, sizes, lab.ctypes.data_as(_vp) if lab is not None else None, len(bufs), out.ctypes.data_as(_vp),
                                  out.size, ctypes.byref(written)), "pcr_record_write")
    assert written.value == out.size
    return out.tobytes()


def record_write_indexed(files, labels=None, entry_interval=128):
    """A version-2 record (bytes) from JPEG files: as record_write, plus entry points about every entry_interval MCUs
    of every scan (every entry_interval / 2 in AC refinement scans), which the decoder uses as it uses restart intervals
    (pcr_record_write_indexed)."""
    bufs, ptrs, sizes = _file_table(files)
    lab = None if labels is None else np.ascontiguousarray(labels, np.int32)
    assert lab is None or lab.size == len(bufs)
    total = sum(b.size for b in bufs)
    cap = total + total // 20 + 64 * 1024 + 64 * len(bufs) * 4
    written = ctypes.c_uint64(0)
    for _ in range(2):
        out = np.empty(cap, np.uint8)
        rc = lib().pcr_record_write_indexed(ptrs, sizes, lab.ctypes.data_as(_vp) if lab is not None else None, len(bufs), entry_interval,
                                            out.ctypes.data_as(_vp), out.size, ctypes.byref(written))
        if rc != E_RANGE or written.value <= cap:
            break
        cap = int(written.value)
    _check(rc, "pcr_record_write_indexed")
    return out[:int(written.value)].tobytes()


HIST_SCANS = 10
HIST_ENTRIES = HIST_SCANS * 2 * 256


def transcode_progressive(src_jpeg, coef, restart_interval=0, counts=None):
    """Progressive file (bytes) holding the quantised coefficients `coef` (int16 numpy array in the layout of
    coef_layout() for this one image) under the frame header and quantisation tables of src_jpeg.  counts: the image's
    symbol counts (uint32 [10, 2, 256], e.g. a row of Record.symbol_histograms()) to build the Huffman tables from."""
    src = np.frombuffer(src_jpeg, np.uint8)
    coef = np.ascontiguousarray(coef, np.int16)
    out = np.empty(src.size + src.size // 2 + 4096, np.uint8)
    written = ctypes.c_uint64(0)
    if counts is not None:
        counts = np.ascontiguousarray(counts, np.uint32)
        assert counts.size == HIST_ENTRIES

    def call(buf):
        if counts is None:
            return lib().pcr_transcode_progressive(src.ctypes.data_as(_vp), src.size, coef.ctypes.data_as(_vp), coef.size, restart_interval,
                                                   buf.ctypes.data_as(_vp), buf.size, ctypes.byref(written))
        return lib().pcr_transcode_progressive_counted(src.ctypes.data_as(_vp), src.size, coef.ctypes.data_as(_vp), coef.size, restart_interval,
                                                       counts.ctypes.data_as(_vp), buf.ctypes.data_as(_vp), buf.size, ctypes.byref(written))
    rc = call(out)
    if rc == E_RANGE and written.value > out.size:
        out = np.empty(int(written.value), np.uint8)
        rc = call(out)
    _check(rc, "pcr_transcode_progressive")
    return out[:int(written.value)].tobytes()


def transcode_symbol_counts(src_jpeg, coef, restart_interval=0):
    """uint32 [10, 2, 256]: the symbol counts transcode_progressive makes for itself on the host."""
    src = np.frombuffer(src_jpeg, np.uint8)
    coef = np.ascontiguousarray(coef, np.int16)
    counts = np.zeros(HIST_ENTRIES, np.uint32)
    _check(lib().pcr_transcode_symbol_counts(src.ctypes.data_as(_vp), src.size, coef.ctypes.data_as(_vp), coef.size, restart_interval,
                                             counts.ctypes.data_as(_vp)), "pcr_transcode_symbol_counts")
    return counts.reshape(HIST_SCANS, 2, 256)


def transcode_files(files, device=0, threads=None, restart_interval=0, device_counts=True):
    """The paper's encoding step for a list of JPEG files (baseline or progressive): their coefficients are decoded
    and the symbols of the new scans counted on the device, the progressive files written on the host.  Returns the
    progressive files; record_write() groups them."""
    rec = record_write(files)
    with pcr_open(rec, device) as r:
        lay = r.coef_layout()
        hist = r.symbol_histograms(restart_interval).cpu().numpy() if device_counts else None
        coef = r.decode_coefficients(r.G).cpu().numpy()
    from concurrent.futures import ThreadPoolExecutor                 # (the C call releases the interpreter lock)
    with ThreadPoolExecutor(threads or min(16, os.cpu_count() or 1)) as ex:
        return list(ex.map(lambda i: transcode_progressive(files[i], coef[int(lay[i]):int(lay[i + 1])], restart_interval,
                                                           None if hist is None else hist[i]), range(len(files))))


class Loader:
    """pcr_loader_*: `slots` re-used sets of pinned staging buffer, device buffer, stream and record handle."""

    def __init__(self, slots, slot_bytes, device=0):
        self._h = _vp()
        self.device, self.slots, self.slot_bytes = device, slots, slot_bytes
        _check(lib().pcr_loader_create(device, slots, slot_bytes, ctypes.byref(self._h)), "pcr_loader_create")

    def close(self):
        if self._h:
            lib().pcr_loader_destroy(self._h)
            self._h = _vp()

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def staging(self, slot):
        """The slot's pinned host buffer as a numpy uint8 array (a view, valid until close)."""
        p, cap = _vp(), ctypes.c_size_t(0)
        _check(lib().pcr_loader_staging(self._h, slot, ctypes.byref(p), ctypes.byref(cap)), "pcr_loader_staging")
        return np.ctypeslib.as_array(ctypes.cast(p, _u8p), shape=(cap.value,))

    def stream(self, slot):
        p = _vp()
        _check(lib().pcr_loader_stream(self._h, slot, ctypes.byref(p)), "pcr_loader_stream")
        return p.value or 0

    def set_rate(self, bytes_per_second, burst_bytes=0.0):
        _check(lib().pcr_loader_set_rate(self._h, float(bytes_per_second), float(burst_bytes)), "pcr_loader_set_rate")

    def upload(self, slot, nbytes):
        """Upload the first nbytes of the slot's staging buffer and bind the slot's handle; returns it as a Record
        (owned by the loader; valid until the slot's next upload)."""
        h = _vp()
        _check(lib().pcr_loader_upload(self._h, slot, nbytes, ctypes.byref(h)), "pcr_loader_upload")
        return Record(None, device=self.device, _borrowed_handle=h.value)

    def read_file(self, slot, path, k):
        """Read from the record file at `path` exactly the prefix scan group k needs into the slot's staging buffer,
        upload it and bind the slot's handle.  Returns (Record, bytes read)."""
        h = _vp()
        n = ctypes.c_size_t(0)
        _check(lib().pcr_loader_read_file(self._h, slot, os.fsencode(path), k, ctypes.byref(n), ctypes.byref(h)), "pcr_loader_read_file")
        return Record(None, device=self.device, _borrowed_handle=h.value), int(n.value)

    def decode(self, slot, k, out, status=None):
        _check(lib().pcr_loader_decode(self._h, slot, k, out.data_ptr(), out.numel(), status.data_ptr() if status is not None else None),
               "pcr_loader_decode")
        return out

    def decode_crop(self, slot, k, crops, out_h, out_w, mean, inv_std, pixels, out, status=None):
        """decode_crop_batch on the slot's handle and stream: pixels is the uint8 working buffer, out the float16 result."""
        m = (ctypes.c_float * 3)(*([float(v) for v in mean] + [0.0] * 3)[:3])
        sd = (ctypes.c_float * 3)(*([float(v) for v in inv_std] + [1.0] * 3)[:3])
        _check(lib().pcr_loader_decode_crop(self._h, slot, k, crops.data_ptr(), pixels.data_ptr() if pixels is not None else None,
                                            pixels.numel() if pixels is not None else 0, out_h, out_w, m, sd,
                                            out.data_ptr(), out.numel() * 2, status.data_ptr() if status is not None else None),
               "pcr_loader_decode_crop")
        return out

    def wait(self, slot):
        _check(lib().pcr_loader_wait(self._h, slot), "pcr_loader_wait")


def pcr_open(data, device=0):
    """Open a record from host bytes (copied to the device)."""
    return Record(data, device)


def pcr_open_device(tensor, stream=None):
    """Open a record whose bytes are a CUDA uint8 tensor (borrowed until close)."""
    return Record(tensor, stream=stream)
