"""ctypes binding of include/einet.h.  Argument marshalling only."""
import ctypes as C
import math
import os

import numpy as np

from .build import LIB_PATH

BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL = 0, 1, 2, 3
STRUCTURE_RAT, STRUCTURE_PD = 0, 1
MASK_NONE, MASK_SHARED, MASK_PER_SAMPLE = 0, 1, 2
MAX_DELTAS = 8

EXPORTED_SYMBOLS = [
    "einet_create", "einet_destroy", "einet_last_error", "einet_sizes", "einet_structure", "einet_bind",
    "einet_refresh", "einet_init_params", "einet_logp", "einet_logp_static", "einet_em_accumulate", "einet_em_update", "einet_em_reset", "einet_em_epoch",
    "einet_mixture_logp", "einet_sample", "einet_profile_enable", "einet_profile_read", "einet_profile_launches",
    "einet_measure_peaks",
]


class EinetError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"libeinet error {code}: {message}")
        self.code = code


class _Spec(C.Structure):
    _fields_ = [("structure", C.c_int32), ("K", C.c_int32), ("channels", C.c_int32), ("leaf_family", C.c_int32),
                ("max_batch", C.c_int32), ("num_vars", C.c_int32), ("depth", C.c_int32), ("num_replica", C.c_int32),
                ("seed", C.c_uint64), ("height", C.c_int32), ("width", C.c_int32), ("num_deltas", C.c_int32),
                ("deltas", C.c_int32 * MAX_DELTAS), ("axes", C.c_int32), ("leaf_param", C.c_int32)]


class _View(C.Structure):
    _fields_ = [("num_vars", C.c_int32), ("num_regions", C.c_int32), ("num_partitions", C.c_int32),
                ("num_replica", C.c_int32), ("num_layers", C.c_int32), ("K", C.c_int32), ("channels", C.c_int32),
                ("num_suff_stats", C.c_int32),
                ("scope_ptr", C.POINTER(C.c_int32)), ("scope_var", C.POINTER(C.c_int32)),
                ("region_replica", C.POINTER(C.c_int32)), ("partition", C.POINTER(C.c_int32)),
                ("layer_ptr", C.POINTER(C.c_int32)), ("layer_partition", C.POINTER(C.c_int32)),
                ("w_offset", C.POINTER(C.c_int64)), ("v_offset", C.POINTER(C.c_int64)),
                ("phi_offset", C.c_int64), ("den_offset", C.c_int64), ("tot_offset", C.c_int64)]


_lib = None


def load_library():
    """Loads libeinet.so (built in-tree by build.build_library); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run __graft_entry__.build() first (no CPU fallback exists)")
    # torch ships its own HIP runtime; load it first so that the library resolves libamdhip64 to the same
    # copy and shares torch's device context, streams and allocations
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
    lib.einet_create.argtypes = [C.POINTER(_Spec), C.POINTER(vp)]
    lib.einet_destroy.argtypes = [vp]
    lib.einet_destroy.restype = None
    lib.einet_last_error.argtypes = [vp]
    lib.einet_last_error.restype = C.c_char_p
    lib.einet_sizes.argtypes = [vp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.einet_structure.argtypes = [vp, C.POINTER(_View)]
    lib.einet_bind.argtypes = [vp, vp, vp, vp, vp]
    lib.einet_refresh.argtypes = [vp, vp]
    lib.einet_init_params.argtypes = [vp, C.c_uint64, f32, f32, vp]
    lib.einet_logp.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.einet_logp_static.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.einet_em_accumulate.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.einet_em_update.argtypes = [vp, f32, f32, f32, f32, vp]
    lib.einet_em_reset.argtypes = [vp, vp]
    lib.einet_em_epoch.argtypes = [vp, vp, vp, i32, C.c_int64, i32, f32, f32, f32, f32, vp, vp]
    lib.einet_mixture_logp.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.einet_sample.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.einet_profile_enable.argtypes = [vp, i32]
    lib.einet_profile_read.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                       C.POINTER(C.c_int64)]
    lib.einet_profile_launches.argtypes = [vp, C.c_int64, C.POINTER(C.c_int64), C.POINTER(i32), C.POINTER(f32),
                                           C.POINTER(C.c_int64)]
    lib.einet_measure_peaks.argtypes = [vp, vp, C.c_int64, i32, C.POINTER(C.c_double), vp]
    _lib = lib
    return lib


def _make_spec(spec, K, channels, family, max_batch, seed, leaf_param=0):
    s = _Spec()
    s.K, s.channels, s.leaf_family, s.max_batch = K, channels, family, max_batch
    s.leaf_param = leaf_param
    if spec["kind"] == "rat":
        s.structure = STRUCTURE_RAT
        s.num_vars, s.depth, s.num_replica, s.seed = spec["D"], spec["depth"], spec["R"], seed
    elif spec["kind"] == "pd":
        s.structure = STRUCTURE_PD
        s.height, s.width = spec["H"], spec["W"]
        deltas = list(spec["deltas"])
        s.num_deltas = len(deltas)
        for i, d in enumerate(deltas[:MAX_DELTAS]):
            s.deltas[i] = d
        s.axes = spec.get("axes", 3)
    else:
        raise ValueError(spec["kind"])
    return s


class EiNet:
    """A model handle plus the torch tensors that back its device buffers."""

    def __init__(self, structure, K, channels, family, max_batch, seed=0, leaf_param=0):
        self._lib = load_library()
        self._h = C.c_void_p()
        spec = _make_spec(structure, K, channels, family, max_batch, seed, leaf_param)
        rc = self._lib.einet_create(C.byref(spec), C.byref(self._h))
        if rc != 0:
            raise EinetError(rc, self._lib.einet_last_error(None).decode())
        n_p, n_s, ws = C.c_size_t(), C.c_size_t(), C.c_size_t()
        self._check(self._lib.einet_sizes(self._h, C.byref(n_p), C.byref(n_s), C.byref(ws)))
        self.n_params, self.n_stats, self.workspace_bytes = n_p.value, n_s.value, ws.value
        self.K, self.channels, self.family, self.max_batch = K, channels, family, max_batch
        self.params = self.stats = self.workspace = None
        self._structure = None

    def _check(self, rc):
        if rc != 0:
            raise EinetError(rc, self._lib.einet_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._lib.einet_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------- structure (host only)
    def structure(self):
        if self._structure is not None:
            return self._structure
        v = _View()
        self._check(self._lib.einet_structure(self._h, C.byref(v)))

        def arr(ptr, n, dtype):
            return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype).copy() if n else np.zeros(0, dtype)

        scope_ptr = arr(v.scope_ptr, v.num_regions + 1, np.int64)
        layer_ptr = arr(v.layer_ptr, v.num_layers + 1, np.int64)
        self._structure = dict(
            num_vars=v.num_vars, num_regions=v.num_regions, num_partitions=v.num_partitions,
            num_replica=v.num_replica, num_layers=v.num_layers, K=v.K, channels=v.channels, T=v.num_suff_stats,
            scope_ptr=scope_ptr, scope_var=arr(v.scope_var, int(scope_ptr[-1]), np.int64),
            region_replica=arr(v.region_replica, v.num_regions, np.int64),
            partition=arr(v.partition, 3 * v.num_partitions, np.int64).reshape(-1, 3),
            layer_ptr=layer_ptr, layer_partition=arr(v.layer_partition, int(layer_ptr[-1]), np.int64),
            w_offset=arr(v.w_offset, v.num_partitions, np.int64), v_offset=arr(v.v_offset, v.num_regions, np.int64),
            phi_offset=v.phi_offset, den_offset=v.den_offset, tot_offset=v.tot_offset)
        return self._structure

    def weight_blocks(self):
        """(offset, rows, row_len) of every normalised weight block, for the seeded parameter generator."""
        st = self.structure()
        n_parts = np.bincount(st["partition"][:, 0], minlength=st["num_regions"])
        blocks = []
        for n in range(st["num_partitions"]):
            parent = st["partition"][n, 0]
            blocks.append((int(st["w_offset"][n]), 1 if parent == 0 else self.K, self.K * self.K))
        for s in range(st["num_regions"]):
            if st["v_offset"][s] >= 0:
                blocks.append((int(st["v_offset"][s]), 1 if s == 0 else self.K, int(n_parts[s])))
        return blocks

    # ------------------------------------------------------------- device side
    def bind(self, device="cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: libeinet has no CPU path")
        self._torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.params = torch.zeros(self.n_params, dtype=torch.float32, device=self.device)
        self.stats = torch.zeros(self.n_stats, dtype=torch.float32, device=self.device)
        self.workspace = torch.zeros(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        self._check(self._lib.einet_bind(self._h, self.params.data_ptr(), self.stats.data_ptr(),
                                         self.workspace.data_ptr(), self._stream()))
        return self

    def _stream(self):
        return C.c_void_p(self._torch.cuda.current_stream().cuda_stream)

    def set_params(self, flat):
        torch = self._torch
        t = torch.as_tensor(np.asarray(flat, dtype=np.float32)) if not torch.is_tensor(flat) else flat
        assert t.numel() == self.n_params
        self.params.copy_(t.to(self.device, non_blocking=False))
        self.refresh()

    def init_params(self, seed=0, leaf_lo=0.1, leaf_hi=0.9):
        """Random initial parameters (flat Dirichlet weight rows, uniform leaf parameters), on the device."""
        self._check(self._lib.einet_init_params(self._h, seed, leaf_lo, leaf_hi, self._stream()))

    def refresh(self):
        self._check(self._lib.einet_refresh(self._h, self._stream()))

    def _mask_args(self, mask, B):
        if mask is None:
            return None, MASK_NONE
        D = int(self.structure()["num_vars"])
        assert mask.dtype == self._torch.uint8 and mask.is_cuda and mask.is_contiguous()
        if mask.dim() == 1:
            assert tuple(mask.shape) == (D,), f"shared mask must have shape ({D},)"
            return C.c_void_p(mask.data_ptr()), MASK_SHARED
        assert tuple(mask.shape) == (B, D), f"per-sample mask must have shape ({B}, {D})"
        return C.c_void_p(mask.data_ptr()), MASK_PER_SAMPLE

    def _batch_of(self, x):
        """The C ABI sees pointers only: a tensor of another shape would be read out of bounds by the kernels."""
        torch = self._torch
        D = int(self.structure()["num_vars"])
        assert x.dtype == torch.float32 and x.is_cuda and x.is_contiguous() and x.dim() == 3
        assert tuple(x.shape[1:]) == (D, self.channels), f"x must have shape (B, {D}, {self.channels})"
        return x.shape[0]

    def _out_arg(self, t, n):
        torch = self._torch
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous() and t.numel() >= n
        return C.c_void_p(t.data_ptr())

    def logp(self, x, mask=None, out=None):
        """x: cuda float32 [B, D, channels]; mask: cuda uint8 [D] or [B, D] (1 = observed) or None."""
        torch = self._torch
        B = self._batch_of(x)
        if out is None:
            out = torch.empty(B, dtype=torch.float32, device=self.device)
        m, mode = self._mask_args(mask, B)
        self._check(self._lib.einet_logp(self._h, x.data_ptr(), m, mode, B, self._out_arg(out, B), self._stream()))
        return out

    def logp_static(self, x, out, mask=None):
        """As logp, with the activations in the library's fixed arena: the call allocates nothing (out is required)."""
        B = self._batch_of(x)
        m, mode = self._mask_args(mask, B)
        self._check(self._lib.einet_logp_static(self._h, x.data_ptr(), m, mode, B, self._out_arg(out, B), self._stream()))
        return out

    def em_accumulate(self, x, mask=None, logp=None):
        B = self._batch_of(x)
        m, mode = self._mask_args(mask, B)
        lp = None if logp is None else self._out_arg(logp, B)
        self._check(self._lib.einet_em_accumulate(self._h, x.data_ptr(), m, mode, B, lp, self._stream()))
        return logp

    def em_update(self, step=1.0, min_var=0.0, max_var=math.inf, w_floor=0.0):
        self._check(self._lib.einet_em_update(self._h, step, min_var, max_var, w_floor, self._stream()))

    def em_reset(self):
        self._check(self._lib.einet_em_reset(self._h, self._stream()))

    def em_epoch(self, x, mask=None, batch=None, step=0.5, min_var=0.0, max_var=math.inf, w_floor=0.0, logp=None):
        """x: cuda float32 [N, D, channels], visited in mini-batches of `batch` (default max_batch) samples."""
        N = self._batch_of(x)
        m, mode = self._mask_args(mask, N)
        lp = None if logp is None else self._out_arg(logp, N)
        self._check(self._lib.einet_em_epoch(self._h, x.data_ptr(), m, mode, N, self.max_batch if batch is None else batch,
                                             step, min_var, max_var, w_floor, lp, self._stream()))
        return logp

    def sample(self, B, u, noise=None, x=None, mask=None, out=None):
        """Top-down sampling.  u: cuda float32 [num_partitions + num_regions, B] uniforms; noise: cuda float32
        [B, D, channels] (standard normal for Gaussian leaves, uniform for Bernoulli leaves) or None for the
        leaf means; x, mask: evidence as in logp (mask 1 = observed), both None for unconditional samples."""
        torch = self._torch
        st = self.structure()
        D = int(st["num_vars"])
        assert u.dtype == torch.float32 and u.is_cuda and u.is_contiguous()
        assert tuple(u.shape) == (int(st["num_partitions"]) + int(st["num_regions"]), B)
        if noise is not None:
            assert noise.dtype == torch.float32 and noise.is_cuda and noise.is_contiguous()
            assert tuple(noise.shape) == (B, D, self.channels)
        if out is None:
            out = torch.empty(B, D, self.channels, dtype=torch.float32, device=self.device)
        assert (x is None) == (mask is None)
        xp = None
        if x is not None:
            assert x.dtype == torch.float32 and x.is_cuda and x.is_contiguous() and tuple(x.shape) == tuple(out.shape)
            xp = C.c_void_p(x.data_ptr())
        m, mode = self._mask_args(mask, B)
        self._check(self._lib.einet_sample(self._h, B, xp, m, mode, u.data_ptr(),
                                           None if noise is None else C.c_void_p(noise.data_ptr()), out.data_ptr(),
                                           self._stream()))
        return out

    def profile_enable(self, enable=True):
        self._check(self._lib.einet_profile_enable(self._h, 1 if enable else 0))

    def profile_read(self):
        """{kernel class: (total milliseconds, launches)} since the last read."""
        cap = 16
        n = C.c_int()
        names, ms, cnt = (C.c_char_p * cap)(), (C.c_double * cap)(), (C.c_int64 * cap)()
        self._check(self._lib.einet_profile_read(self._h, cap, C.byref(n), names, ms, cnt))
        self._class_names = [names[i].decode() for i in range(min(n.value, cap))]
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(min(n.value, cap))}

    def profile_launches(self):
        """[(kernel class, milliseconds, work tag)] of the launches the last profile_read summed, in order."""
        n = C.c_int64()
        self._check(self._lib.einet_profile_launches(self._h, 0, C.byref(n), None, None, None))
        cap = n.value
        cls, ms, work = (C.c_int32 * cap)(), (C.c_float * cap)(), (C.c_int64 * cap)()
        self._check(self._lib.einet_profile_launches(self._h, cap, C.byref(n), cls, ms, work))
        return [(self._class_names[cls[i]], ms[i], work[i]) for i in range(cap)]


def measure_peaks(n_bytes=1 << 30, reps=5):
    """Streaming-copy rate (GB/s, read + written) and register-resident fp32 MFMA rates (TFLOP/s) of cuda:0."""
    import torch
    lib = load_library()
    src = torch.ones(n_bytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    out = (C.c_double * 4)()
    rc = lib.einet_measure_peaks(src.data_ptr(), dst.data_ptr(), n_bytes, reps, out,
                                 C.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise EinetError(rc, lib.einet_last_error(None).decode())
    return {"copy_gbs": out[0], "mfma_f32_32x32x2_tflops": out[1], "mfma_f32_16x16x4_tflops": out[2],
            "mfma_f32_16x16x4_4waves_tflops": out[3]}


# The C names, for callers who prefer the flat interface.
def einet_create(structure, K, channels, family, max_batch, seed=0, leaf_param=0):
    return EiNet(structure, K, channels, family, max_batch, seed, leaf_param)


def einet_destroy(m):
    m.close()


def einet_last_error(m):
    return load_library().einet_last_error(m._h if m is not None else None).decode()


def einet_sizes(m):
    return m.n_params, m.n_stats, m.workspace_bytes


def einet_structure(m):
    return m.structure()


def einet_bind(m, device="cuda:0"):
    return m.bind(device)


def einet_init_params(m, seed=0, leaf_lo=0.1, leaf_hi=0.9):
    m.init_params(seed, leaf_lo, leaf_hi)


def einet_refresh(m):
    m.refresh()


def einet_logp(m, x, mask=None, out=None):
    return m.logp(x, mask, out)


def einet_logp_static(m, x, out, mask=None):
    return m.logp_static(x, out, mask)


def einet_em_accumulate(m, x, mask=None, logp=None):
    return m.em_accumulate(x, mask, logp)


def einet_em_update(m, step=1.0, min_var=0.0, max_var=math.inf, w_floor=0.0):
    m.em_update(step, min_var, max_var, w_floor)


def einet_em_reset(m):
    m.em_reset()


def einet_em_epoch(m, x, mask=None, batch=None, step=0.5, min_var=0.0, max_var=math.inf, w_floor=0.0, logp=None):
    return m.em_epoch(x, mask, batch, step, min_var, max_var, w_floor, logp)


def einet_sample(m, B, u, noise=None, x=None, mask=None, out=None):
    return m.sample(B, u, noise, x, mask, out)


def einet_mixture_logp(component_logp, log_coef, out=None):
    """component_logp: cuda float32 [n_components, B]; log_coef: cuda float32 [n_components]."""
    import torch
    lib = load_library()
    for t in (component_logp, log_coef):
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous()
    n, B = component_logp.shape
    assert log_coef.shape == (n,)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=component_logp.device)
    with torch.cuda.device(component_logp.device):
        rc = lib.einet_mixture_logp(component_logp.data_ptr(), log_coef.data_ptr(), n, B, out.data_ptr(),
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise EinetError(rc, lib.einet_last_error(None).decode())
    return out


def einet_profile_enable(m, enable=True):
    m.profile_enable(enable)


def einet_profile_read(m):
    return m.profile_read()
