"""Python binding of the MI355X swarm-interaction library (argument marshalling only).

Every step of an interaction runs in the HIP kernels behind the C ABI declared in
``include/swarm.h``; this module converts arguments, owns nothing but the handle and
raises if the library is missing -- there is no CPU fallback.  PyTorch is used for
device memory and streams only.
"""
import ctypes
import os

import numpy as np
import torch   # loads the HIP runtime that libswarm.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswarm.so")

OK, EINVAL, ENOMEM, EDEVICE, ESTATE, ERANGE = range(6)
COMM, LIVE, SNAP = 0, 1, 2
DEFERRED, INPLACE = 0, 1
CONSTANT, GEOMETRIC = 0, 1
SCALE_FIXED, SCALE_PAIR_LINF, SCALE_GLOBAL_LINF = 0, 1, 2
CODEC_FIXED, CODEC_PREFIX = 0, 1
MLP_FP32, MLP_BF16X3 = 0, 1
_STATUS = {1: "SWARM_EINVAL", 2: "SWARM_ENOMEM", 3: "SWARM_EDEVICE", 4: "SWARM_ESTATE", 5: "SWARM_ERANGE"}

EXPORTS = ["swarm_init", "swarm_destroy", "swarm_set_objective_diag", "swarm_set_objective_lsq",
           "swarm_set_objective_mlp", "swarm_set_mlp_arithmetic", "swarm_local_steps", "swarm_mark_pending", "swarm_sample_matching", "swarm_sample_stale", "swarm_sample_steps",
           "swarm_gossip_round", "swarm_round_fused", "swarm_interact", "swarm_run_sequential", "swarm_sample_pair", "swarm_quantize", "swarm_dequantize",
           "swarm_read_models", "swarm_write_models", "swarm_models_ptr", "swarm_read_codes",
           "swarm_state_bytes", "swarm_save_state", "swarm_load_state",
           "swarm_potential", "swarm_potential_static", "swarm_pair_linf", "swarm_scale", "swarm_prefix_stats", "swarm_counters", "swarm_timing_reset", "swarm_kernel_times",
           "swarm_stream_copy", "swarm_stream_mix", "swarm_last_error"]


class SwarmError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class _Config(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint32), ("d", ctypes.c_uint64), ("n_edges", ctypes.c_uint32),
                ("edges", ctypes.POINTER(ctypes.c_uint32)), ("bits", ctypes.c_uint32), ("eps", ctypes.c_float),
                ("H", ctypes.c_uint32), ("lr", ctypes.c_float), ("stale_max", ctypes.c_uint32),
                ("seed", ctypes.c_uint64), ("apply_mode", ctypes.c_uint32), ("steps_law", ctypes.c_uint32),
                ("scale_policy", ctypes.c_uint32), ("codec", ctypes.c_uint32)]


def load_library():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1910_12308_amd.build` "
                          "(hipcc, gfx950).  There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, f32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    P = ctypes.POINTER
    sig = {
        "swarm_init": [P(_Config), vp, vp, P(vp)],
        "swarm_destroy": [vp],
        "swarm_set_objective_diag": [vp, vp, vp, f32],
        "swarm_set_objective_lsq": [vp, vp, vp, u32, u32],
        "swarm_set_objective_mlp": [vp, u32, u32, u32, vp, vp, f32, u32],
        "swarm_set_mlp_arithmetic": [vp, u32],
        "swarm_local_steps": [vp, vp, u32],
        "swarm_mark_pending": [vp, vp, u32],
        "swarm_sample_matching": [vp, vp, P(u32)],
        "swarm_sample_stale": [vp, vp],
        "swarm_sample_steps": [vp, vp],
        "swarm_gossip_round": [vp, vp, u32, vp],
        "swarm_round_fused": [vp, vp, u32, vp],
        "swarm_interact": [vp, u32, u32],
        "swarm_run_sequential": [vp, u32, vp, P(u32)],
        "swarm_sample_pair": [vp, P(u32), P(u32)],
        "swarm_quantize": [vp, u64, f32, u32, u64, u32, u32, vp, vp],
        "swarm_dequantize": [vp, vp, u64, f32, u32, vp, vp],
        "swarm_read_models": [vp, u32, u32, u32, u64, u64, vp],
        "swarm_write_models": [vp, u32, u32, u32, u64, u64, vp],
        "swarm_models_ptr": [vp, u32, P(vp)],
        "swarm_state_bytes": [vp, P(u64)],
        "swarm_save_state": [vp, vp, u64],
        "swarm_load_state": [vp, vp, u64],
        "swarm_read_codes": [vp, u32, u32, u64, u64, vp],
        "swarm_potential": [vp, P(ctypes.c_double), vp],
        "swarm_potential_static": [vp, u32, u64, vp, vp, vp],
        "swarm_pair_linf": [vp, vp, u32, vp],
        "swarm_scale": [vp, vp, vp],
        "swarm_prefix_stats": [vp, vp, P(u64)],
        "swarm_counters": [vp, P(u64), P(u64), P(u64), P(u64)],
        "swarm_timing_reset": [vp],
        "swarm_stream_copy": [vp, vp, u64, vp],
        "swarm_stream_mix": [vp, vp, u64, u32, u32, vp],
        "swarm_kernel_times": [vp, P(ctypes.c_double), P(u32), P(ctypes.c_double), P(u32)],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = ctypes.c_int
    lib.swarm_last_error.argtypes = [vp]
    lib.swarm_last_error.restype = ctypes.c_char_p
    return lib


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return ctypes.c_void_p(t.data_ptr())


def _host_u32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint32).reshape(-1))


class _DeviceView:
    """Exposes a raw device address to torch through __cuda_array_interface__."""

    def __init__(self, ptr, shape, owner):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<f4", "data": (int(ptr), False),
                                         "version": 2, "strides": None}


class Swarm:
    """One simulated swarm: n node models of dimension d on one GPU."""

    def __init__(self, n, d, edges, bits, eps, H, lr, stale_max=0, seed=0, x0=None, stream=None,
                 apply_mode=DEFERRED, steps_law=CONSTANT, scale_policy=SCALE_FIXED, codec=CODEC_FIXED):
        self._h = ctypes.c_void_p()
        self._lib = lib()
        edges = _host_u32(edges)
        self.n, self.d, self.bits, self.stale_max = int(n), int(d), int(bits), int(stale_max)
        self.row_bytes = self.d * self.bits // 8 + (8 * ((self.d + 511) // 512) if codec == CODEC_PREFIX else 0)
        cfg = _Config(self.n, self.d, edges.size // 2, edges.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                      self.bits, float(eps), int(H), float(lr), self.stale_max, int(seed) & 0xFFFFFFFFFFFFFFFF,
                      int(apply_mode), int(steps_law), int(scale_policy), int(codec))
        self._keep = []          # borrowed objective tensors must outlive the handle
        rc = self._lib.swarm_init(ctypes.byref(cfg), _dev_ptr(x0, torch.float32), _stream_ptr(stream),
                                  ctypes.byref(self._h))
        if rc != OK:
            raise SwarmError(rc, self._lib.swarm_last_error(None).decode())

    def _check(self, rc):
        if rc != OK:
            raise SwarmError(rc, self._lib.swarm_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._lib.swarm_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- objectives ------------------------------------------------------------------
    def set_objective_diag(self, a, c, sigma):
        self._keep = [a, c]
        self._check(self._lib.swarm_set_objective_diag(self._h, _dev_ptr(a, torch.float32),
                                                       _dev_ptr(c, torch.float32), float(sigma)))

    def set_objective_lsq(self, A, b, m_rows, batch):
        self._keep = [A, b]
        self._check(self._lib.swarm_set_objective_lsq(self._h, _dev_ptr(A, torch.float32),
                                                      _dev_ptr(b, torch.float32), int(m_rows), int(batch)))

    def set_objective_mlp(self, n_in, n_hid, n_out, class_means, label_cdf, data_sigma, batch):
        self._keep = [class_means, label_cdf]
        self._check(self._lib.swarm_set_objective_mlp(self._h, int(n_in), int(n_hid), int(n_out),
                                                      _dev_ptr(class_means, torch.float32),
                                                      _dev_ptr(label_cdf, torch.float32), float(data_sigma),
                                                      int(batch)))

    def set_mlp_arithmetic(self, arithmetic):
        """MLP_FP32 (default) or MLP_BF16X3 (three bf16 products per term, float32 accumulation)."""
        self._check(self._lib.swarm_set_mlp_arithmetic(self._h, int(arithmetic)))

    # ---- the interaction -------------------------------------------------------------
    def local_steps(self, nodes=None):
        if nodes is None:
            self._check(self._lib.swarm_local_steps(self._h, None, 0))
        else:
            nodes = _host_u32(nodes)
            self._check(self._lib.swarm_local_steps(self._h, nodes.ctypes.data_as(ctypes.c_void_p), nodes.size))

    def mark_pending(self, nodes=None):
        if nodes is None:
            self._check(self._lib.swarm_mark_pending(self._h, None, 0))
        else:
            nodes = _host_u32(nodes)
            self._check(self._lib.swarm_mark_pending(self._h, nodes.ctypes.data_as(ctypes.c_void_p), nodes.size))

    def sample_matching(self):
        pairs = np.zeros(2 * (self.n // 2), dtype=np.uint32)
        count = ctypes.c_uint32()
        self._check(self._lib.swarm_sample_matching(self._h, pairs.ctypes.data_as(ctypes.c_void_p),
                                                    ctypes.byref(count)))
        return pairs[:2 * count.value].reshape(-1, 2).copy()

    def sample_stale(self):
        out = np.zeros(self.n, dtype=np.uint8)
        self._check(self._lib.swarm_sample_stale(self._h, out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def round_fused(self, pairs=None, stale=None):
        """Local steps + gossip round in one pass (diagonal objective only)."""
        self._round(self._lib.swarm_round_fused, pairs, stale)

    def sample_steps(self):
        out = np.zeros(self.n, dtype=np.uint8)
        self._check(self._lib.swarm_sample_steps(self._h, out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def gossip_round(self, pairs=None, stale=None):
        self._round(self._lib.swarm_gossip_round, pairs, stale)

    def _round(self, fn, pairs, stale):
        sp = None
        if stale is not None:
            stale = np.ascontiguousarray(np.asarray(stale, dtype=np.uint8))
            assert stale.size == self.n
            sp = stale.ctypes.data_as(ctypes.c_void_p)
        if pairs is None:
            self._check(fn(self._h, None, 0, sp))
        else:
            pairs = _host_u32(pairs)
            self._check(fn(self._h, pairs.ctypes.data_as(ctypes.c_void_p), pairs.size // 2, sp))

    def interact(self, i, j):
        self._check(self._lib.swarm_interact(self._h, int(i), int(j)))

    def run_sequential(self, count):
        """The next `count` steps of Algorithm 1 in batched launches; returns (pairs, number of launches)."""
        pairs = np.zeros((int(count), 2), dtype=np.uint32)
        launches = ctypes.c_uint32()
        self._check(self._lib.swarm_run_sequential(self._h, int(count), pairs.ctypes.data_as(ctypes.c_void_p),
                                                   ctypes.byref(launches)))
        return pairs, launches.value

    def sample_pair(self):
        i, j = ctypes.c_uint32(), ctypes.c_uint32()
        self._check(self._lib.swarm_sample_pair(self._h, ctypes.byref(i), ctypes.byref(j)))
        return i.value, j.value

    # ---- state access ----------------------------------------------------------------
    def read_models(self, which=COMM, node0=0, count=None, k0=0, length=None):
        count = self.n - node0 if count is None else count
        length = self.d - k0 if length is None else length
        out = np.empty((count, length), dtype=np.float32)
        self._check(self._lib.swarm_read_models(self._h, which, node0, count, k0, length,
                                                out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def write_models(self, which, values, node0=0, k0=0):
        values = np.ascontiguousarray(np.asarray(values, dtype=np.float32))
        assert values.ndim == 2
        self._check(self._lib.swarm_write_models(self._h, which, node0, values.shape[0], k0, values.shape[1],
                                                 values.ctypes.data_as(ctypes.c_void_p)))

    def models_view(self, which=COMM):
        """Zero-copy torch view (n x d float32) of a model matrix owned by the handle."""
        ptr = ctypes.c_void_p()
        self._check(self._lib.swarm_models_ptr(self._h, which, ctypes.byref(ptr)))
        return torch.as_tensor(_DeviceView(ptr.value, (self.n, self.d), self), device="cuda")

    def save_state(self):
        """The whole state of the run as a host byte array (exact resume with load_state)."""
        size = ctypes.c_uint64()
        self._check(self._lib.swarm_state_bytes(self._h, ctypes.byref(size)))
        image = np.empty(size.value, dtype=np.uint8)
        self._check(self._lib.swarm_save_state(self._h, image.ctypes.data_as(ctypes.c_void_p), image.size))
        return image

    def load_state(self, image):
        image = np.ascontiguousarray(image, dtype=np.uint8)
        self._check(self._lib.swarm_load_state(self._h, image.ctypes.data_as(ctypes.c_void_p), image.size))

    def read_codes(self, node, age=0, byte0=0, length=None):
        length = self.row_bytes - byte0 if length is None else length
        out = np.empty(length, dtype=np.uint8)
        self._check(self._lib.swarm_read_codes(self._h, age, node, byte0, length,
                                               out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def potential(self, mu=None):
        gamma = ctypes.c_double()
        self._check(self._lib.swarm_potential(self._h, ctypes.byref(gamma), _dev_ptr(mu, torch.float32)))
        return gamma.value

    def pair_linf(self, pairs):
        pairs = _host_u32(pairs)
        out = np.empty(pairs.size // 2, dtype=np.float32)
        self._check(self._lib.swarm_pair_linf(self._h, pairs.ctypes.data_as(ctypes.c_void_p), pairs.size // 2,
                                              out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def scale(self):
        """(scale of the next round, largest disagreement of the last round that had pairs)."""
        eps, far = ctypes.c_float(), ctypes.c_float()
        self._check(self._lib.swarm_scale(self._h, ctypes.byref(eps), ctypes.byref(far)))
        return eps.value, far.value

    def prefix_stats(self):
        """(tile reads that stopped after 4, 8, 16 bits per coordinate; tiles that no level confirmed)."""
        tiles, bad = (ctypes.c_uint64 * 3)(), ctypes.c_uint64()
        self._check(self._lib.swarm_prefix_stats(self._h, tiles, ctypes.byref(bad)))
        return list(tiles), bad.value

    def counters(self, raise_on_range=True):
        vals = [ctypes.c_uint64() for _ in range(4)]
        rc = self._lib.swarm_counters(self._h, *[ctypes.byref(v) for v in vals])
        if rc != OK and (rc != ERANGE or raise_on_range):
            self._check(rc)
        return dict(rounds=vals[0].value, interactions=vals[1].value, bits_communicated=vals[2].value,
                    decode_failures=vals[3].value, range_clamped=(rc == ERANGE))

    def timing_reset(self):
        self._check(self._lib.swarm_timing_reset(self._h))

    def kernel_times(self):
        """Summed device ms and recorded call counts since the last timing_reset()."""
        g, l = ctypes.c_double(), ctypes.c_double()
        ng, nl = ctypes.c_uint32(), ctypes.c_uint32()
        self._check(self._lib.swarm_kernel_times(self._h, ctypes.byref(g), ctypes.byref(ng),
                                                 ctypes.byref(l), ctypes.byref(nl)))
        return dict(gossip_ms=g.value, gossip_calls=ng.value, local_ms=l.value, local_calls=nl.value)


def quantize(x, eps, bits, seed, node, event, stream=None):
    """Enc: packed b-bit codes (uint8 tensor of d*bits/8 bytes) of the device vector x."""
    codes = torch.empty(x.numel() * bits // 8, dtype=torch.uint8, device=x.device)
    rc = lib().swarm_quantize(_dev_ptr(x, torch.float32), x.numel(), float(eps), int(bits),
                              int(seed) & 0xFFFFFFFFFFFFFFFF, int(node), int(event), _dev_ptr(codes),
                              _stream_ptr(stream))
    if rc != OK:
        raise SwarmError(rc, lib().swarm_last_error(None).decode())
    return codes


def dequantize(codes, key, eps, bits, stream=None):
    """Dec: eps * (member of each code's residue class nearest to key/eps)."""
    out = torch.empty_like(key)
    rc = lib().swarm_dequantize(_dev_ptr(codes, torch.uint8), _dev_ptr(key, torch.float32), key.numel(),
                                float(eps), int(bits), _dev_ptr(out), _stream_ptr(stream))
    if rc != OK:
        raise SwarmError(rc, lib().swarm_last_error(None).decode())
    return out


def potential_static(X, gamma_out, mu=None, stream=None):
    """Gamma of the n x d device matrix X into the 1-element float64 device tensor gamma_out (and the
    mean model into mu), through the entry point that allocates nothing.  Asynchronous."""
    assert X.dim() == 2 and gamma_out.dtype == torch.float64 and gamma_out.numel() == 1
    rc = lib().swarm_potential_static(_dev_ptr(X, torch.float32), X.shape[0], X.shape[1], _dev_ptr(gamma_out),
                                      _dev_ptr(mu, torch.float32), _stream_ptr(stream))
    if rc != OK:
        raise SwarmError(rc, lib().swarm_last_error(None).decode())


def stream_copy(dst, src, stream=None):
    """Plain streaming copy kernel between two device tensors of equal byte size."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    rc = lib().swarm_stream_copy(_dev_ptr(dst), _dev_ptr(src), nbytes, _stream_ptr(stream))
    if rc != OK:
        raise SwarmError(rc, lib().swarm_last_error(None).decode())


def stream_mix(dst, src, stream_bytes, n_read, n_write, stream=None):
    """n_read streams of stream_bytes (consecutive in src) summed into n_write streams (consecutive in dst)."""
    assert src.numel() * src.element_size() >= n_read * stream_bytes
    assert dst.numel() * dst.element_size() >= n_write * stream_bytes
    rc = lib().swarm_stream_mix(_dev_ptr(dst), _dev_ptr(src), int(stream_bytes), int(n_read), int(n_write),
                                _stream_ptr(stream))
    if rc != OK:
        raise SwarmError(rc, lib().swarm_last_error(None).decode())
