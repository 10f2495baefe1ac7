"""ctypes binding of libdlf.so: argument marshalling only, same names as include/dlf.h.

Every step of the hot path runs inside the library's HIP kernels; PyTorch is used by callers
for device buffers and streams only.  There is no CPU fallback: if the library is missing or a
call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdlf.so")

OP = {"conv": 0, "dwconv": 1, "fc": 2, "maxpool": 3, "gavgpool": 4}
ACT = {"none": 0, "relu": 1, "relu6": 2}
TUNER_DP, TUNER_GREEDY, TUNER_MANUAL, TUNER_LAYERWISE, TUNER_MAXFUSE = 0, 1, 2, 3, 4
DLF_OK = 0
DLF_ERR_INVALID_ARG = 1
DLF_ERR_SHAPE = 2
DLF_ERR_UNSUPPORTED = 3
DLF_ERR_INFEASIBLE = 4
DLF_ERR_OOM = 5
DLF_ERR_HIP = 6
DLF_ERR_NO_WEIGHTS = 7


class DlfError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("libdlf status %d: %s" % (status, msg))
        self.status = status


class LayerDesc(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("cin", ctypes.c_int32), ("cout", ctypes.c_int32),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("pad", ctypes.c_int32), ("has_bias", ctypes.c_int32), ("act", ctypes.c_int32),
                ("input_from", ctypes.c_int32), ("residual_from", ctypes.c_int32),
                ("weight", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


class TunerOpts(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("budgets", ctypes.POINTER(ctypes.c_int32)),
                ("n_budgets", ctypes.c_int32), ("opcount_critical", ctypes.c_double),
                ("alpha", ctypes.c_double), ("beta", ctypes.c_double),
                ("mp_scale", ctypes.c_double), ("mp_offset", ctypes.c_double),
                ("manual_group_last", ctypes.POINTER(ctypes.c_int32)),
                ("manual_budget", ctypes.POINTER(ctypes.c_int32)),
                ("manual_n", ctypes.c_int32), ("max_lds_bytes", ctypes.c_int32),
                ("fixed_budget", ctypes.c_int32)]


_lib = None


def lib():
    """Loads libdlf.so (built in-tree by paper_2011_05630_amd.build); fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libdlf.so is not built: run `python -m paper_2011_05630_amd.build` "
                           "(or __graft_entry__.build()) first")
    # PyTorch (the caller's source of device buffers and streams) ships its own HIP runtime.  It
    # has to be in the process before libdlf.so is, so that the library binds to that same runtime:
    # two HIP runtimes in one process cannot both open the device.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, u64p, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64), \
        ctypes.POINTER(ctypes.c_int32)
    L.dlf_net_create.argtypes = [ctypes.POINTER(LayerDesc), i32, i32, i32, i32,
                                 ctypes.POINTER(vp)]
    L.dlf_net_create.restype = i32
    L.dlf_net_destroy.argtypes = [vp]
    L.dlf_net_destroy.restype = None
    L.dlf_net_num_layers.argtypes = [vp]
    L.dlf_net_num_layers.restype = i32
    L.dlf_net_layer_info.argtypes = [vp, i32, i32p, i32p, i32p, u64p]
    L.dlf_net_layer_info.restype = i32
    L.dlf_plan.argtypes = [vp, i32, ctypes.POINTER(TunerOpts), ctypes.POINTER(vp)]
    L.dlf_plan.restype = i32
    L.dlf_plan_destroy.argtypes = [vp]
    L.dlf_plan_destroy.restype = None
    L.dlf_plan_num_groups.argtypes = [vp]
    L.dlf_plan_num_groups.restype = i32
    L.dlf_plan_group.argtypes = [vp, i32, i32p, i32p, i32p, i32p, i32p, u64p]
    L.dlf_plan_group.restype = i32
    L.dlf_group_cost.argtypes = [vp, i32, i32, i32, i32, i32, u64p]
    L.dlf_group_cost.restype = i32
    L.dlf_plan_workspace_bytes.argtypes = [vp]
    L.dlf_plan_workspace_bytes.restype = ctypes.c_size_t
    L.dlf_plan_bind_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    L.dlf_plan_bind_workspace.restype = i32
    L.dlf_run.argtypes = [vp, vp, vp, vp]
    L.dlf_run.restype = i32
    L.dlf_run_noalloc.argtypes = [vp, vp, vp, vp]
    L.dlf_run_noalloc.restype = i32
    L.dlf_static_workspace_bytes.argtypes = []
    L.dlf_static_workspace_bytes.restype = ctypes.c_size_t
    L.dlf_run_group.argtypes = [vp, i32, vp, vp, vp, vp]
    L.dlf_run_group.restype = i32
    L.dlf_plan_layer_output.argtypes = [vp, i32]
    L.dlf_plan_layer_output.restype = vp
    L.dlf_status_string.argtypes = [i32]
    L.dlf_status_string.restype = ctypes.c_char_p
    L.dlf_last_error.argtypes = []
    L.dlf_last_error.restype = ctypes.c_char_p
    L.dlf_cost_model_version.argtypes = []
    L.dlf_cost_model_version.restype = i32
    L.dlf_debug_force_config.argtypes = [i32, i32, i32, i32, i32, i32, i32]
    L.dlf_debug_force_config.restype = None
    L.dlf_debug_force_ksplit.argtypes = [i32]
    L.dlf_debug_force_ksplit.restype = None
    L.dlf_debug_pointwise_mode.argtypes = [i32]
    L.dlf_debug_pointwise_mode.restype = None
    L.dlf_debug_depthwise_mode.argtypes = [i32]
    L.dlf_debug_depthwise_mode.restype = None
    L.dlf_debug_depthwise_tile.argtypes = [i32, i32]
    L.dlf_debug_depthwise_tile.restype = None
    L.dlf_debug_block3x3_mode.argtypes = [i32, i32, i32, i32]
    L.dlf_debug_block3x3_mode.restype = None
    L.dlf_plan_set_overlap.argtypes = [vp, i32]
    L.dlf_plan_set_overlap.restype = i32
    L.dlf_plan_group_stream.argtypes = [vp, i32]
    L.dlf_plan_group_stream.restype = i32
    L.dlf_plan_group_config.argtypes = [vp, i32, i32p, i32p, i32p, i32p, i32p, i32p]
    L.dlf_plan_group_config.restype = i32
    L.dlf_run_profiled.argtypes = [vp, vp, vp, vp, i32, ctypes.POINTER(ctypes.c_float)]
    L.dlf_run_profiled.restype = i32
    L.dlf_plan_refine.argtypes = [vp, vp, vp, vp, i32, i32, i32p]
    L.dlf_plan_refine.restype = i32
    L.dlf_plan_group_io.argtypes = [vp, i32, i32p, i32p]
    L.dlf_plan_group_io.restype = i32
    L.dlf_i8conv_create.argtypes = [i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, i32, ctypes.POINTER(vp)]
    L.dlf_i8conv_create.restype = i32
    L.dlf_i8conv_destroy.argtypes = [vp]
    L.dlf_i8conv_destroy.restype = None
    L.dlf_i8conv_info.argtypes = [vp, i32p, i32p, i32p, i32p, u64p]
    L.dlf_i8conv_info.restype = i32
    L.dlf_i8conv_run.argtypes = [vp, vp, vp, vp]
    L.dlf_i8conv_run.restype = i32
    _lib = L
    return L


def _check(status):
    if status != DLF_OK:
        raise DlfError(status, lib().dlf_last_error().decode())


def dlf_net_create(layers, in_h, in_w, in_c, weights=None, biases=None):
    """layers: list of dicts (synth.nets format); weights[i]: fp16 ndarray or None; biases[i]:
    fp32 ndarray or None.  weights=None builds a shape-only network.  Returns an opaque handle."""
    n = len(layers)
    descs = (LayerDesc * n)()
    keep = []
    for i, Ld in enumerate(layers):
        d = descs[i]
        d.op, d.cin, d.cout = OP[Ld["op"]], Ld["cin"], Ld["cout"]
        d.kh, d.kw, d.stride, d.pad = Ld["kh"], Ld["kw"], Ld["stride"], Ld["pad"]
        d.has_bias, d.act = Ld["has_bias"], ACT[Ld["act"]]
        d.input_from, d.residual_from = Ld["input_from"], Ld["residual_from"]
        d.weight, d.bias = None, None
        if weights is not None and weights[i] is not None:
            w = np.ascontiguousarray(weights[i], dtype=np.float16)
            keep.append(w)
            d.weight = w.ctypes.data
        if biases is not None and biases[i] is not None:
            b = np.ascontiguousarray(biases[i], dtype=np.float32)
            keep.append(b)
            d.bias = b.ctypes.data
    h = ctypes.c_void_p()
    _check(lib().dlf_net_create(descs, n, in_h, in_w, in_c, ctypes.byref(h)))
    return h


def dlf_net_destroy(net):
    lib().dlf_net_destroy(net)


def dlf_net_num_layers(net):
    return lib().dlf_net_num_layers(net)


def dlf_status_string(status):
    return lib().dlf_status_string(status).decode()


def dlf_last_error():
    return lib().dlf_last_error().decode()


def dlf_net_layer_info(net, i):
    h, w, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    ops = ctypes.c_uint64()
    _check(lib().dlf_net_layer_info(net, i, ctypes.byref(h), ctypes.byref(w), ctypes.byref(c),
                                    ctypes.byref(ops)))
    return h.value, w.value, c.value, ops.value


def dlf_plan(net, batch, mode=TUNER_DP, budgets=None, group_last=None, group_budget=None,
             opcount_critical=0.0, alpha=0.0, beta=0.0, mp_scale=0.0, mp_offset=0.0,
             max_lds_bytes=0, fixed_budget=0):
    o = TunerOpts()
    o.mode = mode
    keep = []
    if budgets is not None:
        arr = (ctypes.c_int32 * len(budgets))(*budgets)
        keep.append(arr)
        o.budgets, o.n_budgets = arr, len(budgets)
    if group_last is not None:
        gl = (ctypes.c_int32 * len(group_last))(*group_last)
        gb = (ctypes.c_int32 * len(group_last))(*group_budget)
        keep += [gl, gb]
        o.manual_group_last, o.manual_budget, o.manual_n = gl, gb, len(group_last)
    o.opcount_critical, o.alpha, o.beta = opcount_critical, alpha, beta
    o.mp_scale, o.mp_offset = mp_scale, mp_offset
    o.max_lds_bytes = max_lds_bytes
    o.fixed_budget = fixed_budget
    h = ctypes.c_void_p()
    _check(lib().dlf_plan(net, batch, ctypes.byref(o), ctypes.byref(h)))
    return h


def dlf_plan_destroy(plan):
    lib().dlf_plan_destroy(plan)


def dlf_plan_num_groups(plan):
    return lib().dlf_plan_num_groups(plan)


def dlf_plan_group(plan, g):
    """-> dict(first, last, budget, tile_h, tile_w, model_cost)."""
    v = [ctypes.c_int32() for _ in range(5)]
    cost = ctypes.c_uint64()
    _check(lib().dlf_plan_group(plan, g, *[ctypes.byref(x) for x in v], ctypes.byref(cost)))
    return dict(first=v[0].value, last=v[1].value, budget=v[2].value, tile_h=v[3].value,
                tile_w=v[4].value, model_cost=cost.value)


def dlf_plan_group_config(plan, g):
    """-> dict(kind, variant, nslices, slice_c, stream0, lds_bytes) of the kernel configuration."""
    v = [ctypes.c_int32() for _ in range(6)]
    _check(lib().dlf_plan_group_config(plan, g, *[ctypes.byref(x) for x in v]))
    return dict(kind=v[0].value, variant=v[1].value, nslices=v[2].value, slice_c=v[3].value,
                stream0=v[4].value, lds_bytes=v[5].value)


def dlf_plan_group_io(plan, g):
    """-> (in_layer, res_layer): producers of the group's input (-1 = net input) and residual
    operand (-2 = none)."""
    a, b = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().dlf_plan_group_io(plan, g, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def dlf_plan_groups(plan):
    return [dlf_plan_group(plan, g) for g in range(dlf_plan_num_groups(plan))]


def dlf_group_cost(net, batch, first, last, budget, max_lds_bytes=0):
    """Cost-model picoseconds, or None if the layers cannot run as one group."""
    c = ctypes.c_uint64()
    s = lib().dlf_group_cost(net, batch, first, last, budget, max_lds_bytes, ctypes.byref(c))
    if s == DLF_ERR_INFEASIBLE:
        return None
    _check(s)
    return c.value


def dlf_plan_workspace_bytes(plan):
    return lib().dlf_plan_workspace_bytes(plan)


def dlf_plan_bind_workspace(plan, dev_ptr, nbytes):
    _check(lib().dlf_plan_bind_workspace(plan, dev_ptr, nbytes))


def dlf_run(plan, in_ptr, out_ptr, stream=None):
    _check(lib().dlf_run(plan, in_ptr, out_ptr, stream))


def dlf_run_noalloc(plan, in_ptr, out_ptr, stream=None):
    _check(lib().dlf_run_noalloc(plan, in_ptr, out_ptr, stream))


def dlf_static_workspace_bytes():
    return int(lib().dlf_static_workspace_bytes())


def dlf_run_profiled(plan, in_ptr, out_ptr, stream, reps):
    """-> list of mean per-group durations in milliseconds (HIP events on `stream`)."""
    n = dlf_plan_num_groups(plan)
    ms = (ctypes.c_float * n)()
    _check(lib().dlf_run_profiled(plan, in_ptr, out_ptr, stream, reps, ms))
    return list(ms)


def dlf_plan_refine(plan, in_ptr, out_ptr, stream, top_k=6, reps=5):
    """Times the top_k modelled tilings (and pointwise forms) of every group on the GPU and keeps
    the fastest; -> number of groups whose configuration changed."""
    changed = ctypes.c_int32(0)
    _check(lib().dlf_plan_refine(plan, in_ptr, out_ptr, stream, top_k, reps, ctypes.byref(changed)))
    return changed.value


def dlf_run_group(plan, g, in_ptr, res_ptr, out_ptr, stream=None):
    _check(lib().dlf_run_group(plan, g, in_ptr, res_ptr, out_ptr, stream))


def dlf_plan_layer_output(plan, layer):
    return lib().dlf_plan_layer_output(plan, layer)


def dlf_i8conv_create(batch, h, w, cin, cout, ksize, relu, weight=None, scale=None, bias=None, budget=0, pool=False):
    """weight: numpy int8 [cout,ksize,ksize,cin] (None: shape-only layer), scale / bias: numpy fp32 [cout]."""
    out = ctypes.c_void_p()
    wp = sp = bp = None
    if weight is not None:
        weight = np.ascontiguousarray(weight, dtype=np.int8)
        scale = np.ascontiguousarray(scale, dtype=np.float32)
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if weight.shape != (cout, ksize, ksize, cin) or scale.shape != (cout,) or bias.shape != (cout,):
            raise ValueError("weight [cout,ksize,ksize,cin], scale [cout], bias [cout] expected")
        wp, sp, bp = weight.ctypes.data, scale.ctypes.data, bias.ctypes.data
    _check(lib().dlf_i8conv_create(batch, h, w, cin, cout, ksize, int(bool(relu)), int(bool(pool)), wp, sp, bp, budget,
                                   ctypes.byref(out)))
    return out


def dlf_i8conv_destroy(layer):
    lib().dlf_i8conv_destroy(layer)


def dlf_i8conv_info(layer):
    """-> dict(th, tw, shape, grid, op_count)."""
    th, tw, sh, gr = (ctypes.c_int32() for _ in range(4))
    ops = ctypes.c_uint64()
    _check(lib().dlf_i8conv_info(layer, ctypes.byref(th), ctypes.byref(tw), ctypes.byref(sh),
                                 ctypes.byref(gr), ctypes.byref(ops)))
    return dict(th=th.value, tw=tw.value, shape=sh.value, grid=gr.value, op_count=ops.value)


def dlf_i8conv_run(layer, in_ptr, out_ptr, stream=None):
    _check(lib().dlf_i8conv_run(layer, in_ptr, out_ptr, stream))


def dlf_cost_model_version():
    return lib().dlf_cost_model_version()


def dlf_debug_force_ksplit(ksplit=1):
    """Testing hook (after dlf_debug_force_config): K of the forced tiling split over `ksplit` waves."""
    lib().dlf_debug_force_ksplit(ksplit)


def dlf_debug_depthwise_mode(mode=0):
    """Testing hook: 0 = depthwise kernels chosen by modelled cost, 1 = wherever they apply, 2 = never,
    3 = wherever they apply, a depthwise + 1x1 pair always on the register kernel."""
    lib().dlf_debug_depthwise_mode(mode)


def dlf_debug_depthwise_tile(wx=0, rw=0):
    """Testing hook: wx > 0 fixes the tile of the depthwise + 1x1 tile kernel (wx waves side by side, rw
    rows per wave); 0 restores the automatic choice."""
    lib().dlf_debug_depthwise_tile(wx, rw)


def dlf_debug_pointwise_mode(mode=0):
    """Testing hook: 0 = pointwise kernel chosen by modelled cost, 1 = wherever it applies, 2 = never,
    3 / 4 / 5 = wherever it applies with 64x64 / 32x32 / split-K 64x64 work items, 6 / 7 = with
    128x128 / 64x256 workgroup blocks."""
    lib().dlf_debug_pointwise_mode(mode)


def dlf_plan_set_overlap(plan, on=True):
    """on: groups that do not depend on the group in front of them run beside it on a second stream;
    off (the default): every group on the caller's stream, in order."""
    _check(lib().dlf_plan_set_overlap(plan, 1 if on else 0))


def dlf_plan_group_stream(plan, g):
    """0 = group g runs on the caller's stream, 1 = on the plan's second stream."""
    return lib().dlf_plan_group_stream(plan, g)


def dlf_debug_block3x3_mode(mode=0, shape=-1, th=0, tw=0):
    """Testing hook: 0 = block 3x3 kernel chosen by modelled cost, 1 = wherever it applies, 2 = never;
    shape >= 0 also fixes its shape (0 / 1: 128 channels x 256 pixels, activations 32 / 64 input
    channels at a time; 2 / 3: 64 x 512 likewise) and pixel tile."""
    lib().dlf_debug_block3x3_mode(mode, shape, th, tw)


def dlf_debug_force_config(th=0, tw=0, variant=0, nslices=1, slice_c=0, stream0=0, kc=0):
    """Testing hook: th > 0 forces the tile/register-tile/slicing of every group planned
    afterwards (th = 0 restores automatic choice)."""
    lib().dlf_debug_force_config(th, tw, variant, nslices, slice_c, stream0, kc)
