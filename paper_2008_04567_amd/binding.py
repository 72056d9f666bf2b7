"""Thin ctypes binding of libwpk.so: argument marshalling only, same names as the C ABI.

Tensors are anything with ``data_ptr()`` (PyTorch-ROCm device tensors) or a raw integer
address; streams are ``torch.cuda.Stream`` objects, raw ``hipStream_t`` integers or ``None``.
Every step of the convolution runs in the library's HIP kernels.  There is no CPU fallback: if
the library has not been built, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# WPK_LIBRARY names another build of the library (same ABI) to load instead of the in-tree one
LIB_PATH = os.environ.get("WPK_LIBRARY") or os.path.join(_HERE, "libwpk.so")
N_GENES = 10
NCHW, X_NHWC, Y_NHWC, NHWC = 0, 1, 2, 3   # layout codes of ConvDesc.layout

(OK, E_BAD_DESC, E_NULL_PTR, E_UNSUPPORTED, E_HIP, E_NO_CONFIG, E_BAD_ARG, E_IO, E_VERIFY,
 E_TOO_LARGE) = (0, -1, -2, -3, -4, -5, -6, -7, -8, -9)
NOALLOC_SCRATCH_BYTES = 32 << 20

DESC_FIELDS = ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w",
               "dil_h", "dil_w", "dtype", "layout")
CONFIG_FIELDS = ("bm", "bn", "bk", "wm", "wn", "split_k", "xcd_remap", "persist", "stages", "reduce")


class ConvDesc(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in DESC_FIELDS]

    def __repr__(self):
        return "ConvDesc(%s)" % ", ".join("%s=%d" % (f, getattr(self, f)) for f in DESC_FIELDS[:13])


class ConvConfig(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in CONFIG_FIELDS]

    def astuple(self):
        return tuple(getattr(self, f) for f in CONFIG_FIELDS)

    def asdict(self):
        return {f: getattr(self, f) for f in CONFIG_FIELDS}

    def __repr__(self):
        return "ConvConfig(%s)" % ", ".join("%s=%d" % (f, getattr(self, f)) for f in CONFIG_FIELDS)


class TuneOptions(ctypes.Structure):
    _fields_ = [("population", ctypes.c_int32), ("elites", ctypes.c_int32),
                ("next_population", ctypes.c_int32), ("participants", ctypes.c_int32),
                ("max_generations", ctypes.c_int32), ("patience", ctypes.c_int32),
                ("mutation", ctypes.c_double), ("eps", ctypes.c_double),
                ("seed", ctypes.c_uint64), ("reps", ctypes.c_int32),
                ("min_group_us", ctypes.c_double), ("mode", ctypes.c_int32),
                ("verbose", ctypes.c_int32), ("refine", ctypes.c_int32),
                ("zero_ahead", ctypes.c_int32), ("epilogue", ctypes.c_int32)]


class TuneReport(ctypes.Structure):
    _fields_ = [("best", ConvConfig), ("best_us", ctypes.c_double), ("default_us", ctypes.c_double),
                ("evaluations", ctypes.c_int32), ("generations", ctypes.c_int32),
                ("rejected", ctypes.c_int32), ("seconds", ctypes.c_double),
                ("stage", ctypes.c_int32), ("search_us", ctypes.c_double)]

    STAGE_NAMES = ("search", "rule", "refine", "default")

    @property
    def stage_name(self):
        return self.STAGE_NAMES[self.stage] if 0 <= self.stage < 4 else "?"


GA_CONSTRAINT_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                    ctypes.c_void_p)
GA_FITNESS_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                 ctypes.c_void_p)


class WpkError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s: %s (%d)" % (where, status_string(status), status)
        if status == E_HIP:
            msg += " hipError=%d" % lib().wpk_last_hip_error()
        super().__init__(msg)


_lib = None


def lib():
    """The loaded library.  Raises if libwpk.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libwpk.so is missing: build it with "
                               "`python -m paper_2008_04567_amd.build` (no CPU fallback exists)")
        try:                      # share PyTorch's HIP runtime: load it before the library
            import torch          # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        P, I, V, D = ctypes.POINTER, ctypes.c_int, ctypes.c_void_p, ctypes.c_double
        i32p = P(ctypes.c_int32)
        sig = {
            "wpk_conv_out_shape": (I, [P(ConvDesc), i32p, i32p]),
            "wpk_conv_flops": (D, [P(ConvDesc)]),
            "wpk_status_string": (ctypes.c_char_p, [I]),
            "wpk_last_hip_error": (I, []),
            "wpk_config_gene_ranges": (I, [i32p, i32p]),
            "wpk_config_from_genes": (I, [i32p, P(ConvConfig)]),
            "wpk_config_to_genes": (I, [P(ConvConfig), i32p]),
            "wpk_config_legal": (I, [P(ConvDesc), P(ConvConfig)]),
            "wpk_config_id": (I, [P(ConvConfig)]),
            "wpk_config_from_id": (I, [I, P(ConvConfig)]),
            "wpk_config_default": (I, [P(ConvDesc), P(ConvConfig)]),
            "wpk_conv2d_fwd": (I, [P(ConvDesc), V, V, V, V]),
            "wpk_conv2d_fwd_config": (I, [P(ConvDesc), P(ConvConfig), V, V, V, V]),
            "wpk_conv2d_fwd_noalloc": (I, [P(ConvDesc), P(ConvConfig), V, V, V, V]),
            "wpk_conv2d_ref": (I, [P(ConvDesc), V, V, V, V]),
            "wpk_conv2d_fwd_fused": (I, [P(ConvDesc), V, V, V, V, ctypes.c_int32, V, V]),
            "wpk_conv2d_fwd_fused_config": (I, [P(ConvDesc), P(ConvConfig), V, V, V, V, ctypes.c_int32,
                                                V, V]),
            "wpk_tune_default_options": (None, [P(TuneOptions)]),
            "wpk_conv_tune": (I, [P(ConvDesc)]),
            "wpk_conv_tune_ex": (I, [P(ConvDesc), P(TuneOptions), I, P(TuneReport)]),
            "wpk_cache_lookup": (I, [P(ConvDesc), P(ConvConfig)]),
            "wpk_cache_lookup_time": (I, [P(ConvDesc), P(ConvConfig), P(D)]),
            "wpk_cache_store": (I, [P(ConvDesc), P(ConvConfig), D]),
            "wpk_cache_clear": (I, []),
            "wpk_cache_size": (I, []),
            "wpk_cache_save": (I, [ctypes.c_char_p]),
            "wpk_cache_load": (I, [ctypes.c_char_p]),
            "wpk_ga_search": (I, [ctypes.c_int32, i32p, i32p, GA_CONSTRAINT_FN, GA_FITNESS_FN, V,
                                  P(TuneOptions), i32p, P(D), i32p, i32p, P(D), i32p,
                                  ctypes.c_int32]),
            "wpk_conv_plan": (I, [P(ConvDesc), ctypes.c_int32, ctypes.c_int32, P(V)]),
            "wpk_conv_plan_graph": (I, [P(ConvDesc), ctypes.c_int32, i32p, i32p, i32p, i32p, ctypes.c_int32,
                                        ctypes.c_int32, P(V)]),
            "wpk_plan_tensor_layout": (I, [V, ctypes.c_int32]),
            "wpk_plan_layer_layout": (I, [V, ctypes.c_int32]),
            "wpk_choose_layouts": (I, [ctypes.c_int32, i32p, i32p, i32p, i32p, ctypes.c_int32, P(D), i32p, P(D)]),
            "wpk_plan_set_weights": (I, [V, ctypes.c_int32, V, V]),
            "wpk_plan_run": (I, [V, P(V), P(V), V]),
            "wpk_plan_run_layer": (I, [V, ctypes.c_int32, V, V, V]),
            "wpk_plan_set_epilogue": (I, [V, ctypes.c_int32, V, ctypes.c_int32, V]),
            "wpk_plan_run_layer_fused": (I, [V, ctypes.c_int32, V, V, V, V]),
            "wpk_plan_run_fused": (I, [V, P(V), P(V), P(V), V]),
            "wpk_plan_set_pipeline": (I, [V, ctypes.c_int32]),
            "wpk_plan_num_layers": (I, [V]),
            "wpk_plan_num_unique": (I, [V]),
            "wpk_plan_layer_config": (I, [V, ctypes.c_int32, P(ConvConfig)]),
            "wpk_plan_set_layer_config": (I, [V, ctypes.c_int32, P(ConvConfig)]),
            "wpk_plan_destroy": (None, [V]),
            "wpk_config_kernel_name": (ctypes.c_char_p, [P(ConvConfig)]),
            "wpk_device_info": (I, [ctypes.c_char_p, ctypes.c_int32, i32p]),
            "wpk_version": (ctypes.c_char_p, []),
            "wpk_measure_peaks": (I, [D, P(D), P(D), P(D), V]),
            "wpk_set_workspace_limit": (I, [ctypes.c_int64]),
            "wpk_config_workspace_bytes": (ctypes.c_int64, [P(ConvDesc), P(ConvConfig), ctypes.c_int32,
                                                            P(ctypes.c_int64), P(ctypes.c_int64)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        L._signatures = sig
        _lib = L
    return _lib


# ---- marshalling helpers ----------------------------------------------------------------------
def make_desc(layer=None, **kw):
    """ConvDesc from a mapping with the 13 shape keys (dtype/layout default to fp32/NCHW)."""
    src = dict(layer or {})
    src.update(kw)
    d = ConvDesc()
    for f in DESC_FIELDS[:13]:
        setattr(d, f, int(src[f]))
    d.dtype = int(src.get("dtype", 0))
    d.layout = int(src.get("layout", 0))
    return d


def make_config(bm, bn, bk, wm, wn, split_k=1, xcd_remap=1, persist=0, stages=2, reduce=0):
    return ConvConfig(bm, bn, bk, wm, wn, split_k, 1 if persist else xcd_remap, persist, stages, reduce)


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    return ctypes.c_void_p(int(t))


def _stream(s):
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return ctypes.c_void_p(s.cuda_stream)
    return ctypes.c_void_p(int(s))


def _check(status, where):
    if status < 0:
        raise WpkError(status, where)
    return status


# ---- the ABI, name by name ---------------------------------------------------------------------
def status_string(status):
    return lib().wpk_status_string(int(status)).decode()


def version():
    return lib().wpk_version().decode()


def conv_out_shape(desc):
    p, q = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().wpk_conv_out_shape(ctypes.byref(desc), ctypes.byref(p), ctypes.byref(q)),
           "wpk_conv_out_shape")
    return p.value, q.value


def conv_flops(desc):
    return lib().wpk_conv_flops(ctypes.byref(desc))


def config_gene_ranges():
    lo, hi = (ctypes.c_int32 * N_GENES)(), (ctypes.c_int32 * N_GENES)()
    _check(lib().wpk_config_gene_ranges(lo, hi), "wpk_config_gene_ranges")
    return list(lo), list(hi)


def config_from_genes(genes):
    g = (ctypes.c_int32 * N_GENES)(*genes)
    c = ConvConfig()
    _check(lib().wpk_config_from_genes(g, ctypes.byref(c)), "wpk_config_from_genes")
    return c


def config_to_genes(cfg):
    g = (ctypes.c_int32 * N_GENES)()
    _check(lib().wpk_config_to_genes(ctypes.byref(cfg), g), "wpk_config_to_genes")
    return list(g)


def config_legal(desc, cfg):
    return _check(lib().wpk_config_legal(ctypes.byref(desc), ctypes.byref(cfg)),
                  "wpk_config_legal") == 1


def config_id(cfg):
    return _check(lib().wpk_config_id(ctypes.byref(cfg)), "wpk_config_id")


def config_from_id(cid):
    c = ConvConfig()
    _check(lib().wpk_config_from_id(int(cid), ctypes.byref(c)), "wpk_config_from_id")
    return c


def config_default(desc):
    c = ConvConfig()
    _check(lib().wpk_config_default(ctypes.byref(desc), ctypes.byref(c)), "wpk_config_default")
    return c


def config_kernel_name(cfg):
    return lib().wpk_config_kernel_name(ctypes.byref(cfg)).decode()


def legal_configs(desc, split_k=None, xcd_remap=None, persist=None, stages=None, reduce=None):
    """Every legal configuration of a descriptor (enumeration of the gene space)."""
    import itertools
    lo, hi = config_gene_ranges()
    out = []
    for genes in itertools.product(*[range(l, h + 1) for l, h in zip(lo, hi)]):
        c = config_from_genes(genes)
        if split_k is not None and c.split_k not in split_k:
            continue
        if xcd_remap is not None and c.xcd_remap != xcd_remap:
            continue
        if persist is not None and c.persist not in persist:
            continue
        if stages is not None and c.stages not in stages:
            continue
        if reduce is not None and c.reduce not in reduce:
            continue
        if config_legal(desc, c):
            out.append(c)
    return out


def conv2d_fwd(desc, x, w, y, stream=None):
    _check(lib().wpk_conv2d_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(y), _stream(stream)),
           "wpk_conv2d_fwd")


def conv2d_fwd_config(desc, cfg, x, w, y, stream=None):
    _check(lib().wpk_conv2d_fwd_config(ctypes.byref(desc), ctypes.byref(cfg), _ptr(x), _ptr(w),
                                       _ptr(y), _stream(stream)), "wpk_conv2d_fwd_config")


def conv2d_fwd_noalloc(desc, x, w, y, cfg=None, stream=None):
    _check(lib().wpk_conv2d_fwd_noalloc(ctypes.byref(desc), ctypes.byref(cfg) if cfg is not None else None,
                                        _ptr(x), _ptr(w), _ptr(y), _stream(stream)),
           "wpk_conv2d_fwd_noalloc")


def conv2d_ref(desc, x, w, y, stream=None):
    _check(lib().wpk_conv2d_ref(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(y), _stream(stream)),
           "wpk_conv2d_ref")


def tune_default_options(**overrides):
    o = TuneOptions()
    lib().wpk_tune_default_options(ctypes.byref(o))
    for k, v in overrides.items():
        setattr(o, k, v)
    return o


def conv_tune(desc):
    return _check(lib().wpk_conv_tune(ctypes.byref(desc)), "wpk_conv_tune")


def conv_tune_ex(desc, options=None, force=False):
    """Returns (config id, TuneReport)."""
    rep = TuneReport()
    cid = _check(lib().wpk_conv_tune_ex(ctypes.byref(desc),
                                        ctypes.byref(options) if options is not None else None,
                                        1 if force else 0, ctypes.byref(rep)), "wpk_conv_tune_ex")
    return cid, rep


def cache_lookup(desc):
    c = ConvConfig()
    hit = _check(lib().wpk_cache_lookup(ctypes.byref(desc), ctypes.byref(c)), "wpk_cache_lookup")
    return c if hit == 1 else None


def cache_lookup_time(desc):
    """(config, stored runtime in microseconds) or None."""
    c, us = ConvConfig(), ctypes.c_double()
    hit = _check(lib().wpk_cache_lookup_time(ctypes.byref(desc), ctypes.byref(c), ctypes.byref(us)),
                 "wpk_cache_lookup_time")
    return (c, us.value) if hit == 1 else None


def choose_layouts(x_tensor, y_tensor, residual_tensor, tensor_layout, cost):
    """wpk_choose_layouts: cost is n_layers x 2 x 2 (nested lists); returns (layouts, total)."""
    n, nt = len(x_tensor), len(tensor_layout)
    i32 = lambda v: (ctypes.c_int32 * len(v))(*[int(e) for e in v])
    flat = [float(cost[i][lx][ly]) for i in range(n) for lx in range(2) for ly in range(2)]
    chosen, total = (ctypes.c_int32 * nt)(), ctypes.c_double()
    _check(lib().wpk_choose_layouts(n, i32(x_tensor), i32(y_tensor),
                                    i32(residual_tensor) if residual_tensor is not None else None,
                                    i32(tensor_layout), nt, (ctypes.c_double * len(flat))(*flat), chosen,
                                    ctypes.byref(total)), "wpk_choose_layouts")
    return list(chosen), total.value


def cache_store(desc, cfg, us=0.0):
    _check(lib().wpk_cache_store(ctypes.byref(desc), ctypes.byref(cfg), float(us)),
           "wpk_cache_store")


def cache_clear():
    _check(lib().wpk_cache_clear(), "wpk_cache_clear")


def cache_size():
    return lib().wpk_cache_size()


def cache_save(path):
    _check(lib().wpk_cache_save(os.fsencode(path)), "wpk_cache_save")


def cache_load(path):
    return _check(lib().wpk_cache_load(os.fsencode(path)), "wpk_cache_load")


def ga_search(lo, hi, constraint, fitness, options=None, history_capacity=0):
    """The search engine on its own.  ``constraint(genes) -> bool`` (or None) and
    ``fitness(genes) -> float`` are Python callables.  Returns a dict like the oracle's."""
    n = len(lo)
    opt = options if options is not None else tune_default_options()
    width = max(opt.population, opt.next_population if opt.next_population > 0 else opt.population)
    c_lo, c_hi = (ctypes.c_int32 * n)(*lo), (ctypes.c_int32 * n)(*hi)
    cons = GA_CONSTRAINT_FN((lambda g, m, u: 1 if constraint(tuple(g[i] for i in range(m))) else 0)
                            if constraint else (lambda g, m, u: 1))
    fit = GA_FITNESS_FN(lambda g, m, u: float(fitness(tuple(g[i] for i in range(m)))))
    best = (ctypes.c_int32 * n)()
    best_f, evals = ctypes.c_double(), ctypes.c_int32()
    cap = int(history_capacity)
    hp = (ctypes.c_int32 * max(1, cap * width * n))()
    hf = (ctypes.c_double * max(1, cap * width))()
    hs = (ctypes.c_int32 * max(1, cap))()
    gens = _check(lib().wpk_ga_search(n, c_lo, c_hi, cons, fit, None, ctypes.byref(opt), best,
                                      ctypes.byref(best_f), ctypes.byref(evals), hp, hf, hs, cap),
                  "wpk_ga_search")
    history = []
    for g in range(min(gens, cap)):
        size = hs[g]
        pop = [tuple(hp[(g * width + i) * n + j] for j in range(n)) for i in range(size)]
        fits = [hf[g * width + i] for i in range(size)]
        history.append((pop, fits))
    return {"best": tuple(best), "best_fitness": best_f.value, "evaluations": evals.value,
            "generations": gens, "history": history}


def conv2d_fwd_fused(desc, x, w, y, bias=None, residual=None, relu=False, cfg=None, stream=None):
    """y = act(conv(x, w) + bias[k] + residual); with ``cfg`` through that configuration."""
    if cfg is None:
        _check(lib().wpk_conv2d_fwd_fused(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias),
                                          _ptr(residual), 1 if relu else 0, _ptr(y), _stream(stream)),
               "wpk_conv2d_fwd_fused")
    else:
        _check(lib().wpk_conv2d_fwd_fused_config(ctypes.byref(desc), ctypes.byref(cfg), _ptr(x), _ptr(w),
                                                 _ptr(bias), _ptr(residual), 1 if relu else 0,
                                                 _ptr(y), _stream(stream)),
               "wpk_conv2d_fwd_fused_config")


class Plan:
    """Owner of a ``wpk_plan*``."""

    def __init__(self, descs, tune=False, graph=None):
        """``graph`` = (x_tensor, y_tensor, residual_tensor or None, tensor_layout): wpk_conv_plan_graph."""
        arr = (ConvDesc * len(descs))(*descs)
        h = ctypes.c_void_p()
        if graph is None:
            _check(lib().wpk_conv_plan(arr, len(descs), 1 if tune else 0, ctypes.byref(h)),
                   "wpk_conv_plan")
        else:
            xt, yt, rt, tl = graph
            i32 = lambda v: (ctypes.c_int32 * len(v))(*[int(e) for e in v])
            _check(lib().wpk_conv_plan_graph(arr, len(descs), i32(xt), i32(yt), i32(rt) if rt is not None else None,
                                             i32(tl), len(tl), 1 if tune else 0, ctypes.byref(h)),
                   "wpk_conv_plan_graph")
        self.handle = h
        self.n = len(descs)

    def tensor_layout(self, tensor):
        return _check(lib().wpk_plan_tensor_layout(self.handle, tensor), "wpk_plan_tensor_layout")

    def layer_layout(self, layer):
        return _check(lib().wpk_plan_layer_layout(self.handle, layer), "wpk_plan_layer_layout")

    def set_weights(self, layer, w, stream=None):
        _check(lib().wpk_plan_set_weights(self.handle, layer, _ptr(w), _stream(stream)),
               "wpk_plan_set_weights")

    def pointer_arrays(self, xs, ys):
        """Host arrays of device pointers for run(); build once, reuse."""
        xa = (ctypes.c_void_p * self.n)(*[t.data_ptr() if hasattr(t, "data_ptr") else int(t) for t in xs])
        ya = (ctypes.c_void_p * self.n)(*[t.data_ptr() if hasattr(t, "data_ptr") else int(t) for t in ys])
        return xa, ya

    def run(self, xa, ya, stream=None):
        _check(lib().wpk_plan_run(self.handle, xa, ya, _stream(stream)), "wpk_plan_run")

    def run_layer(self, layer, x, y, stream=None):
        _check(lib().wpk_plan_run_layer(self.handle, layer, _ptr(x), _ptr(y), _stream(stream)),
               "wpk_plan_run_layer")

    def set_epilogue(self, layer, bias=None, relu=False, stream=None):
        _check(lib().wpk_plan_set_epilogue(self.handle, layer, _ptr(bias), 1 if relu else 0,
                                           _stream(stream)), "wpk_plan_set_epilogue")

    def run_layer_fused(self, layer, x, residual, y, stream=None):
        _check(lib().wpk_plan_run_layer_fused(self.handle, layer, _ptr(x), _ptr(residual), _ptr(y),
                                              _stream(stream)), "wpk_plan_run_layer_fused")

    def residual_array(self, rs):
        """Host array of device pointers (None entries allowed) for run_fused()."""
        return (ctypes.c_void_p * self.n)(*[None if t is None else
                                            (t.data_ptr() if hasattr(t, "data_ptr") else int(t))
                                            for t in rs])

    def run_fused(self, xa, ra, ya, stream=None):
        _check(lib().wpk_plan_run_fused(self.handle, xa, ra, ya, _stream(stream)), "wpk_plan_run_fused")

    def set_pipeline(self, ways):
        _check(lib().wpk_plan_set_pipeline(self.handle, int(ways)), "wpk_plan_set_pipeline")

    def num_layers(self):
        return lib().wpk_plan_num_layers(self.handle)

    def num_unique(self):
        return lib().wpk_plan_num_unique(self.handle)

    def layer_config(self, layer):
        c = ConvConfig()
        _check(lib().wpk_plan_layer_config(self.handle, layer, ctypes.byref(c)),
               "wpk_plan_layer_config")
        return c

    def set_layer_config(self, layer, cfg):
        _check(lib().wpk_plan_set_layer_config(self.handle, layer, ctypes.byref(cfg)),
               "wpk_plan_set_layer_config")

    def destroy(self):
        if self.handle:
            lib().wpk_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def config_workspace(desc, cfg, compute_units=256):
    """(bytes, shared tiles, slots per shared tile) of the workspace a launch of cfg uses."""
    tiles, slots = ctypes.c_int64(), ctypes.c_int64()
    nbytes = lib().wpk_config_workspace_bytes(ctypes.byref(desc), ctypes.byref(cfg), compute_units,
                                              ctypes.byref(tiles), ctypes.byref(slots))
    if nbytes < 0:
        raise WpkError(int(nbytes), "wpk_config_workspace_bytes")
    return int(nbytes), tiles.value, slots.value


def set_workspace_limit(nbytes):
    _check(lib().wpk_set_workspace_limit(int(nbytes)), "wpk_set_workspace_limit")


def measure_peaks(sustain_ms=60.0, stream=None):
    """Measured ceilings of the device: (fp32 MFMA TFLOP/s right after a pause, sustained over the
    second half of sustain_ms, copy GB/s read + written)."""
    burst, sustained, copy = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib().wpk_measure_peaks(float(sustain_ms), ctypes.byref(burst), ctypes.byref(sustained),
                                   ctypes.byref(copy), _stream(stream)), "wpk_measure_peaks")
    return burst.value, sustained.value, copy.value


def device_info():
    buf = ctypes.create_string_buffer(256)
    cus = ctypes.c_int32()
    _check(lib().wpk_device_info(buf, 256, ctypes.byref(cus)), "wpk_device_info")
    return buf.value.decode(), cus.value
