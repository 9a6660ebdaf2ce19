"""ctypes binding of the C ABI in include/ad.h: argument marshalling only.

Every step of the decoding path runs inside the HIP library; PyTorch is used here for
device memory (weight blobs, workspace) and for the stream handle, nothing else.
There is no fallback: if the library is missing this module raises on import of `lib()`.
"""
from __future__ import annotations

import atexit
import ctypes as C
import os
import sys
import weakref

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libad_mi355x.so")

AD_OK, AD_EINVAL, AD_ESTATE, AD_ENOMEM, AD_EDEVICE = 0, -1, -2, -3, -4
AD_F32, AD_BF16 = 0, 1
AD_VERIFIER, AD_DRAFTER = 0, 1
AD_NEVER = -1

EXPORTS = [
    "ad_config_check", "ad_workspace_bytes", "ad_weights_count", "ad_weights_bytes", "ad_weights_entry",
    "ad_weights_pack",
    "ad_create", "ad_destroy", "ad_last_error", "ad_encode", "ad_verify", "ad_verify_static", "ad_draft_nat", "ad_output",
    "ad_decode_greedy", "ad_decode_iad", "ad_decode_gad", "ad_debug_logits", "ad_time_verify_forward",
    "ad_suffix_match", "ad_host_simulate", "ad_set_option", "ad_get_option", "ad_calibration_copy", "ad_set_gadpp", "ad_time_output_projection", "ad_calibration_mfma",
]
AD_OPT_GRAPHS = 3
AD_OPT_GRAPHS_CAPTURED = 4
AD_OPT_SPIN_WAIT = 5
AD_OPT_FUSE_CROSSQ = 6
AD_OPT_OVERLAP_ENCODERS = 7


class AdConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "enc_layers", "dec_layers", "d_model", "n_heads", "d_ffn", "vocab",
        "max_batch", "max_src", "max_len", "k_max", "bos", "pad", "eos", "mask",
        "dtype", "tie_output", "debug_logits")]


class AdStats(C.Structure):
    _fields_ = [("iterations", C.c_int64), ("rows_verified", C.c_int64), ("draft_rows", C.c_int64),
                ("tokens_out", C.c_int64), ("t_encode_us", C.c_double), ("t_draft_us", C.c_double),
                ("t_verify_us", C.c_double), ("t_host_us", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class AdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"ad error {code}: {msg}")
        self.code = code


_lib = None
_I32P = C.POINTER(C.c_int32)


def lib():
    """The loaded HIP library.  Raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2205_10350_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    L = C.CDLL(LIB_PATH)
    cfgp = C.POINTER(AdConfig)
    L.ad_config_check.argtypes = [cfgp]; L.ad_config_check.restype = C.c_int
    L.ad_workspace_bytes.argtypes = [cfgp, C.c_int]; L.ad_workspace_bytes.restype = C.c_size_t
    L.ad_weights_count.argtypes = [cfgp]; L.ad_weights_count.restype = C.c_int
    L.ad_weights_bytes.argtypes = [cfgp]; L.ad_weights_bytes.restype = C.c_size_t
    L.ad_weights_entry.argtypes = [cfgp, C.c_int, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t), _I32P, _I32P, _I32P]
    L.ad_weights_entry.restype = C.c_int
    L.ad_weights_pack.argtypes = [cfgp, C.c_int, C.POINTER(C.c_float), C.c_void_p]; L.ad_weights_pack.restype = C.c_int
    L.ad_create.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
    L.ad_create.restype = C.c_int
    L.ad_destroy.argtypes = [C.c_void_p]; L.ad_destroy.restype = C.c_int
    L.ad_last_error.argtypes = [C.c_void_p]; L.ad_last_error.restype = C.c_char_p
    L.ad_encode.argtypes = [C.c_void_p, C.c_int, _I32P, _I32P, C.c_int, _I32P]; L.ad_encode.restype = C.c_int
    L.ad_verify.argtypes = [C.c_void_p, _I32P, _I32P, _I32P, _I32P, _I32P]; L.ad_verify.restype = C.c_int
    L.ad_verify_static.argtypes = [C.c_void_p, _I32P, _I32P, _I32P, _I32P, _I32P]; L.ad_verify_static.restype = C.c_int
    L.ad_draft_nat.argtypes = [C.c_void_p, C.c_int, _I32P]; L.ad_draft_nat.restype = C.c_int
    L.ad_output.argtypes = [C.c_void_p, _I32P, _I32P]; L.ad_output.restype = C.c_int
    sp = C.POINTER(AdStats)
    L.ad_decode_greedy.argtypes = [C.c_void_p, _I32P, _I32P, C.c_int, _I32P, _I32P, _I32P, sp]
    L.ad_decode_greedy.restype = C.c_int
    L.ad_decode_iad.argtypes = [C.c_void_p, _I32P, _I32P, _I32P, _I32P, C.c_int, C.c_int, _I32P, _I32P, _I32P, sp]
    L.ad_decode_iad.restype = C.c_int
    L.ad_decode_gad.argtypes = [C.c_void_p, _I32P, _I32P, C.c_int, C.c_int, C.c_int, _I32P, _I32P, C.c_int, _I32P,
                                _I32P, _I32P, sp]
    L.ad_decode_gad.restype = C.c_int
    L.ad_debug_logits.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_int)]
    L.ad_debug_logits.restype = C.c_int
    L.ad_time_verify_forward.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                         C.POINTER(C.c_double)]
    L.ad_time_verify_forward.restype = C.c_int
    L.ad_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.ad_calibration_copy.restype = C.c_int
    L.ad_calibration_mfma.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
    L.ad_calibration_mfma.restype = C.c_int
    L.ad_set_option.argtypes = [C.c_void_p, C.c_int, C.c_int]; L.ad_set_option.restype = C.c_int
    L.ad_set_gadpp.argtypes = [C.c_void_p, C.c_int32, C.c_float]; L.ad_set_gadpp.restype = C.c_int
    L.ad_time_output_projection.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
    L.ad_time_output_projection.restype = C.c_int
    L.ad_get_option.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int)]; L.ad_get_option.restype = C.c_int
    L.ad_suffix_match.argtypes = [_I32P, C.c_int, _I32P, C.c_int, C.POINTER(C.c_int)]; L.ad_suffix_match.restype = C.c_int
    L.ad_host_simulate.argtypes = [C.c_int, _I32P, C.c_int, _I32P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                   _I32P, _I32P, _I32P, C.c_int, sp]
    L.ad_host_simulate.restype = C.c_int
    _lib = L
    return L


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(_I32P)


def _check(rc, ctx=None):
    if rc != AD_OK:
        raise AdError(rc, (lib().ad_last_error(ctx) or b"").decode())


def make_config(dims: dict, *, max_batch, max_src, max_len, k_max, dtype, special, tie_output=False,
                debug_logits=False) -> AdConfig:
    return AdConfig(dims["enc_layers"], dims["dec_layers"], dims["d_model"], dims["n_heads"], dims["d_ffn"],
                    dims["vocab"], max_batch, max_src, max_len, k_max, special["bos"], special["pad"],
                    special["eos"], special["mask"], AD_BF16 if dtype == "bf16" else AD_F32,
                    int(tie_output), int(debug_logits))


# ---- host-only calls -------------------------------------------------------------------------
def config_check(cfg: AdConfig) -> int:
    return lib().ad_config_check(C.byref(cfg))


def workspace_bytes(cfg: AdConfig, with_drafter: bool) -> int:
    return lib().ad_workspace_bytes(C.byref(cfg), int(with_drafter))


def weights_layout(cfg: AdConfig):
    """[(name, offset, rows, cols, elem_bytes)], total bytes."""
    L = lib()
    n = L.ad_weights_count(C.byref(cfg))
    out = []
    name = C.create_string_buffer(64)
    off = C.c_size_t(); r = C.c_int32(); c = C.c_int32(); eb = C.c_int32()
    for i in range(n):
        _check(L.ad_weights_entry(C.byref(cfg), i, name, 64, C.byref(off), C.byref(r), C.byref(c), C.byref(eb)))
        out.append((name.value.decode(), off.value, r.value, c.value, eb.value))
    return out, L.ad_weights_bytes(C.byref(cfg))


def suffix_match(o, x):
    o, x = _i32(o), _i32(x)
    i = C.c_int(-1)
    found = lib().ad_suffix_match(_p(o), len(o), _p(x), len(x), C.byref(i))
    return i.value if found else None


def host_simulate(mode, g, aux, *, k=1, k_max=64, max_out=64, eos=2, bos=0):
    g, aux = _i32(g), _i32(aux)
    out = np.zeros(max_out, dtype=np.int32)
    n = np.zeros(1, dtype=np.int32)
    acc = np.zeros(max_out + 1, dtype=np.int32)
    st = AdStats()
    _check(lib().ad_host_simulate(mode, _p(g), len(g), _p(aux), len(aux), k, k_max, max_out, eos, bos,
                                  _p(out), _p(n), _p(acc), len(acc), C.byref(st)))
    return out[:n[0]].tolist(), acc[:st.iterations].tolist(), st.as_dict()


# ---- device side ------------------------------------------------------------------------------
def pack_weights_host(cfg: AdConfig, params: dict) -> np.ndarray:
    """Lays a {name: fp32 ndarray} parameter set out as the library's flat blob (host bytes).
    The library does the rounding to bf16 and the tiling of GEMM matrices; with a tied output
    projection the "out.w" entry is filled from the embedding table."""
    L = lib()
    layout, total = weights_layout(cfg)
    blob = np.zeros(total, dtype=np.uint8)
    for i, (name, off, rows, cols, eb) in enumerate(layout):
        src = params["emb"] if (name == "out.w" and name not in params) else params[name]
        w = np.ascontiguousarray(src, dtype=np.float32).reshape(rows, cols)
        _check(L.ad_weights_pack(C.byref(cfg), i, w.ctypes.data_as(C.POINTER(C.c_float)), C.c_void_p(blob.ctypes.data)))
    return blob


def pack_weights(cfg: AdConfig, params: dict, device="cuda"):
    import torch
    return torch.from_numpy(pack_weights_host(cfg, params)).to(device)


def calibration_copy(dst, src, stream=None):
    """Plain device copy of known size (torch tensors on the GPU, equal byte sizes, a multiple of
    16): the launch that memory-traffic counters are calibrated against."""
    import torch
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    st = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().ad_calibration_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, C.c_void_p(st)))


def calibration_mfma(iters=4000, stream=None):
    """Measured dense bf16 MFMA rate of the chip in TFLOP/s (register operands, nothing else in the way)."""
    import torch
    scratch = torch.empty(512 * 1024, dtype=torch.uint8, device="cuda")
    st = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    t = C.c_double(0)
    _check(lib().ad_calibration_mfma(C.c_void_p(scratch.data_ptr()), scratch.numel(), iters, C.c_void_p(st), C.byref(t)))
    torch.cuda.synchronize()
    return t.value


# Contexts that are still open.  They are closed by an atexit hook, i.e. at the very start of the
# interpreter's shutdown, while the HIP runtime, torch and any profiler tool are still fully
# alive: ad_destroy synchronizes the stream and destroys graphs and events, which must not happen
# from a finalizer that runs after those libraries have begun to tear themselves down.
_live = weakref.WeakSet()


@atexit.register
def _close_all():
    for ctx in list(_live):
        try:
            ctx.close()
        except Exception:
            pass


class Context:
    """One ad_ctx with its device memory.  Methods mirror the C entry points.  Also a context
    manager: `with Context(...) as ctx:` closes it on the way out."""

    def __init__(self, cfg: AdConfig, verifier_params: dict, drafter_params: dict | None = None, device="cuda:0"):
        import torch
        self._torch = torch
        self.cfg = cfg
        self.L = lib()
        _check(self.L.ad_config_check(C.byref(cfg)))
        torch.cuda.set_device(device)
        self.w_ver = pack_weights(cfg, verifier_params, device)
        self.w_dr = pack_weights(cfg, drafter_params, device) if drafter_params is not None else None
        nbytes = workspace_bytes(cfg, drafter_params is not None)
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=device)
        # a stream of the context's own (default priority): the null stream cannot be captured
        # into graphs.  Everything queued so far (weights, workspace) is finished first.
        torch.cuda.synchronize()
        self.stream = torch.cuda.Stream(device=device)
        h = C.c_void_p()
        _check(self.L.ad_create(C.byref(cfg), C.c_void_p(self.w_ver.data_ptr()),
                                C.c_void_p(self.w_dr.data_ptr()) if self.w_dr is not None else None,
                                C.c_void_p(self.workspace.data_ptr()), nbytes,
                                C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self.h = h
        self.B = 0
        _live.add(self)

    def close(self):
        if getattr(self, "h", None):
            self.L.ad_destroy(self.h)
            self.h = None
        _live.discard(self)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False

    def __del__(self):
        # never from interpreter shutdown: by then the atexit hook has closed every context, and a
        # context it could not reach is left to the process's end rather than to a HIP call
        # made while the runtime is going away
        if sys.is_finalizing():
            return
        try:
            self.close()
        except Exception:
            pass

    # -- marshalling helpers
    def _pad_rows(self, rows, width, fill=0):
        a = np.full((len(rows), width), fill, dtype=np.int32)
        lens = np.zeros(len(rows), dtype=np.int32)
        for b, r in enumerate(rows):
            r = np.asarray(r, dtype=np.int32)
            a[b, :min(len(r), width)] = r[:width]
            lens[b] = len(r)          # an over-long row keeps its true length: the library rejects it
        return a, lens

    def encode(self, model, srcs, max_out=None):
        src, src_len = self._pad_rows(srcs, self.cfg.max_src)
        mo = None if max_out is None else _i32(max_out)
        _check(self.L.ad_encode(self.h, model, _p(src), _p(src_len), len(srcs), _p(mo)), self.h)
        if model == AD_VERIFIER:
            self.B = len(srcs)

    def verify(self, drafts, want_verified=False, static=False):
        """drafts: list of B token lists (empty = sit out).  Returns n_accept, next, [verified].
        static=True calls ad_verify_static, the variant that allocates nothing."""
        km = self.cfg.k_max
        d, k = self._pad_rows(drafts, km)
        n = np.zeros(self.B, dtype=np.int32); nx = np.zeros(self.B, dtype=np.int32)
        ver = np.zeros((self.B, km), dtype=np.int32) if want_verified else None
        fn = self.L.ad_verify_static if static else self.L.ad_verify
        _check(fn(self.h, _p(d), _p(k), _p(n), _p(nx), _p(ver)), self.h)
        return (n, nx, ver) if want_verified else (n, nx)

    def draft_nat(self, k):
        out = np.zeros((self.B, self.cfg.k_max), dtype=np.int32)
        _check(self.L.ad_draft_nat(self.h, k, _p(out)), self.h)
        return out[:, :k]

    def output(self):
        out = np.zeros((self.B, self.cfg.max_len), dtype=np.int32)
        n = np.zeros(self.B, dtype=np.int32)
        _check(self.L.ad_output(self.h, _p(out), _p(n)), self.h)
        return [out[b, :n[b]].tolist() for b in range(self.B)]

    def _result(self, out, n, st):
        return [out[b, :n[b]].tolist() for b in range(len(n))], st.as_dict()

    def decode_greedy(self, srcs, max_out=None):
        src, sl = self._pad_rows(srcs, self.cfg.max_src)
        B = len(srcs)
        out = np.zeros((B, self.cfg.max_len), dtype=np.int32); n = np.zeros(B, dtype=np.int32); st = AdStats()
        mo = None if max_out is None else _i32(max_out)
        _check(self.L.ad_decode_greedy(self.h, _p(src), _p(sl), B, _p(mo), _p(out), _p(n), C.byref(st)), self.h)
        self.B = B
        return self._result(out, n, st)

    def decode_iad(self, srcs, guides=None, max_out=None):
        src, sl = self._pad_rows(srcs, self.cfg.max_src)
        B = len(srcs)
        g = gl = None
        stride = 0
        if guides is not None:
            stride = max(1, max(len(x) for x in guides))
            g, gl = self._pad_rows(guides, stride)
        out = np.zeros((B, self.cfg.max_len), dtype=np.int32); n = np.zeros(B, dtype=np.int32); st = AdStats()
        mo = None if max_out is None else _i32(max_out)
        _check(self.L.ad_decode_iad(self.h, _p(src), _p(sl), _p(g), _p(gl), stride, B, _p(mo), _p(out), _p(n),
                                    C.byref(st)), self.h)
        self.B = B
        return self._result(out, n, st)

    def decode_gad(self, srcs, k, use_drafter=False, draft_override=None, max_out=None):
        src, sl = self._pad_rows(srcs, self.cfg.max_src)
        B = len(srcs)
        D = dl = None
        stride = 0
        if draft_override is not None:
            stride = max(1, max(len(x) for x in draft_override))
            D, dl = self._pad_rows(draft_override, stride)
        out = np.zeros((B, self.cfg.max_len), dtype=np.int32); n = np.zeros(B, dtype=np.int32); st = AdStats()
        mo = None if max_out is None else _i32(max_out)
        _check(self.L.ad_decode_gad(self.h, _p(src), _p(sl), B, k, int(use_drafter), _p(D), _p(dl), stride, _p(mo),
                                    _p(out), _p(n), C.byref(st)), self.h)
        self.B = B
        return self._result(out, n, st)

    def set_gadpp(self, beta, tau):
        _check(self.L.ad_set_gadpp(self.h, int(beta), float(tau)), self.h)

    def set_option(self, option, value):
        _check(self.L.ad_set_option(self.h, option, value), self.h)

    def get_option(self, option):
        v = C.c_int(0)
        _check(self.L.ad_get_option(self.h, option, C.byref(v)), self.h)
        return v.value

    def time_output_projection(self, n_copies, reps=50):
        """Mean microseconds per launch of the output-projection kernel over `n_copies` rotating
        copies of the verifier's output matrix (made here, device to device)."""
        torch = self._torch
        layout, _ = weights_layout(self.cfg)
        name, off, rows, cols, eb = next(e for e in layout if e[0] == "out.w")
        nbytes = rows * cols * eb
        stride = (nbytes + 255) // 256 * 256
        buf = torch.empty(n_copies * stride, dtype=torch.uint8, device=self.w_ver.device)
        for i in range(n_copies):
            buf[i * stride:i * stride + nbytes].copy_(self.w_ver[off:off + nbytes])
        torch.cuda.synchronize()
        us = C.c_double(0)
        _check(self.L.ad_time_output_projection(self.h, C.c_void_p(buf.data_ptr()), stride, n_copies, reps, C.byref(us)), self.h)
        del buf
        return us.value

    def debug_logits(self):
        cap = self.cfg.max_batch * self.cfg.k_max
        buf = np.zeros((cap, self.cfg.vocab), dtype=np.float32)
        rows = C.c_int(0)
        _check(self.L.ad_debug_logits(self.h, buf.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(rows)), self.h)
        return buf[:rows.value].copy()

    def time_verify_forward(self, reps=20, back_to_back=False):
        a, b, d = C.c_double(0), C.c_double(0), C.c_double(0)
        _check(self.L.ad_time_verify_forward(self.h, reps, C.byref(a), C.byref(b), C.byref(d)), self.h)
        return (a.value, b.value, d.value) if back_to_back else (a.value, b.value)
