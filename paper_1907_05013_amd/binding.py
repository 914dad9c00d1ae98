"""ctypes binding of libpooch.so: the same entry points as include/pooch.h, argument
marshalling only.  Every step of the training path runs inside the library's HIP kernels;
there is no Python or CPU fallback -- if the library is missing, loading fails loudly.

Two layers:
  * `lib()` returns the ctypes handle with argument / return types declared for every
    symbol of the header (SYMBOLS lists them);
  * `Context` wraps one pooch_ctx: builds the graph from a layer list, owns the torch
    tensors that back the arena / pinned buffer and the torch streams, converts numpy
    arrays to pointers and statuses to exceptions.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpooch.so")

OK, E_INVALID, E_STATE, E_BUDGET, E_HIP, E_NOPROFILE = 0, -1, -2, -3, -4, -5
KEEP, SWAP, RECOMPUTE = 0, 1, 2
MODE_INCORE, MODE_SWAPALL_NOSCHED, MODE_SWAPALL, MODE_SWAPOPT, MODE_POOCH, MODE_REFINE, MODE_SUPERNEURONS = range(7)
MODES = {"incore": 0, "swapall_nosched": 1, "swapall": 2, "swapopt": 3, "pooch": 4, "refine": 5, "superneurons": 6}


class Stats(C.Structure):
    _fields_ = [("step_ms", C.c_double), ("predicted_ms", C.c_double),
                ("swap_out_bytes", C.c_uint64), ("swap_in_bytes", C.c_uint64),
                ("peak_bytes", C.c_uint64), ("extent_bytes", C.c_uint64),
                ("resident_bytes", C.c_uint64), ("arena_bytes", C.c_uint64),
                ("n_keep", C.c_int32), ("n_swap", C.c_int32), ("n_recompute", C.c_int32),
                ("n_commands", C.c_int32), ("n_refwd", C.c_int32), ("reserved", C.c_int32),
                ("scratch_bytes", C.c_uint64)]


_ctx = C.c_void_p
_i32, _i64, _dbl, _sz = C.c_int32, C.c_int64, C.c_double, C.c_size_t
_pi, _pi64, _pd, _pf, _pu8 = C.POINTER(C.c_int), C.POINTER(_i64), C.POINTER(_dbl), C.POINTER(C.c_float), C.POINTER(C.c_uint8)
_pi32 = C.POINTER(_i32)

# name -> (restype, argtypes): every symbol include/pooch.h declares
SYMBOLS = {
    "pooch_create": (_i32, [C.c_void_p, _sz, C.c_void_p, _sz, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_ctx)]),
    "pooch_destroy": (None, [_ctx]),
    "pooch_last_error": (C.c_char_p, [_ctx]),
    "pooch_input": (_i32, [_ctx, _pi64, C.c_int]),
    "pooch_conv": (_i32, [_ctx, _i32, C.c_int, _pi, _pi, _pi, C.c_int]),
    "pooch_bn": (_i32, [_ctx, _i32, C.c_float]),
    "pooch_relu": (_i32, [_ctx, _i32]),
    "pooch_add": (_i32, [_ctx, _i32, _i32]),
    "pooch_maxpool": (_i32, [_ctx, _i32, _pi, _pi, _pi, C.c_int]),
    "pooch_gavgpool": (_i32, [_ctx, _i32]),
    "pooch_fc": (_i32, [_ctx, _i32, C.c_int]),
    "pooch_softmax_ce": (_i32, [_ctx, _i32]),
    "pooch_set_fusion": (_i32, [_ctx, C.c_int]),
    "pooch_node_fused": (_i32, [_ctx, _i32]),
    "pooch_set_relu_masks": (_i32, [_ctx, C.c_int]),
    "pooch_node_keeps_mask": (_i32, [_ctx, _i32]),
    "pooch_bn_stats_source": (_i32, [_ctx, _i32]),
    "pooch_refine_profile": (_i32, [_ctx, C.c_int, _pf]),
    "pooch_finalize": (_i32, [_ctx]),
    "pooch_num_params": (_i32, [_ctx]),
    "pooch_param_info": (_i32, [_ctx, _i32, _pi64, _pi32]),
    "pooch_set_param": (_i32, [_ctx, _i32, C.c_void_p]),
    "pooch_get_grad": (_i32, [_ctx, _i32, C.c_void_p]),
    "pooch_set_batch": (_i32, [_ctx, C.c_void_p, C.c_void_p]),
    "pooch_capture_tensor": (_i32, [_ctx, _i32, C.c_void_p]),
    "pooch_inject_failure": (_i32, [_ctx, _i64]),
    "pooch_get_bn_stats": (_i32, [_ctx, _i32, C.c_void_p, C.c_void_p]),
    "pooch_set_bn_decay": (_i32, [_ctx, C.c_float]),
    "pooch_get_bn_running": (_i32, [_ctx, _i32, C.c_void_p, C.c_void_p]),
    "pooch_set_bn_running": (_i32, [_ctx, _i32, C.c_void_p, C.c_void_p]),
    "pooch_num_nodes": (_i32, [_ctx]),
    "pooch_num_fmaps": (_i32, [_ctx]),
    "pooch_fmap_info": (_i32, [_ctx, _i32, C.POINTER(_sz), _pi32]),
    "pooch_resident_bytes": (_sz, [_ctx]),
    "pooch_profile": (_i32, [_ctx, C.c_int, C.c_int]),
    "pooch_profile_step": (_i32, [_ctx, C.c_int, _pf]),
    "pooch_finish_profile": (_i32, [_ctx]),
    "pooch_sgd_update": (_i32, [_ctx, C.c_float]),
    "pooch_get_param": (_i32, [_ctx, _i32, C.c_void_p]),
    "pooch_get_profile": (_i32, [_ctx, _pd, _pd, _pd, _pd, _pd]),
    "pooch_set_profile": (_i32, [_ctx, _pd, _pd, _pd, _pd, _pd]),
    "pooch_plan": (_i32, [_ctx, C.c_int, C.c_int, _pd]),
    "pooch_set_search_effort": (_i32, [_ctx, C.c_int]),
    "pooch_get_plan": (_i32, [_ctx, _pu8]),
    "pooch_set_plan": (_i32, [_ctx, _pu8, C.c_int]),
    "pooch_simulate": (_i32, [_ctx, _pu8, C.c_int, _pd, C.POINTER(_sz)]),
    "pooch_plan_evaluations": (_i64, [_ctx]),
    "pooch_get_overhead_sets": (_i32, [_ctx, _pu8, _pu8]),
    "pooch_get_commands": (_i32, [_ctx, _pi64, _i64, _pi64]),
    "pooch_step": (_i32, [_ctx, _pf]),
    "pooch_step_static_scratch": (_i32, [_ctx, _pf]),
    "pooch_get_stats": (_i32, [_ctx, C.POINTER(Stats)]),
    "pooch_step_timed": (_i32, [_ctx, _pf, _pd, _pd, _pd, _pd]),
    "pooch_node_kernel": (C.c_char_p, [_ctx, _i32, C.c_int]),
    "pooch_measure_link": (_i32, [_ctx, _sz, C.c_int, _pd, _pd]),
}

_lib = None


def lib():
    """the loaded library; raises if it has not been built (python -m paper_1907_05013_amd.build)"""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpooch.so is not built: run `python -m paper_1907_05013_amd.build` "
                               "(there is no fallback path)")
        # torch first: the library then binds to the HIP runtime torch has already loaded, so
        # the arena torch allocates and the kernels launched here live in one runtime
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


_hip = None


def _hip_rt():
    """the HIP runtime already in the process (torch's), for pinned host allocations that are
    returned to the system as soon as a context closes (torch caches its own pinned blocks) and for
    the context's three streams"""
    global _hip
    if _hip is None:
        import torch  # noqa: F401
        # the copy of the runtime that torch has mapped into this process, by its path: opening it by a
        # fixed soname could load a second runtime (or none) next to the one that owns the arena
        path = None
        with open("/proc/self/maps") as f:
            for line in f:
                name = line.rsplit(" ", 1)[-1].strip()
                if os.path.basename(name).startswith("libamdhip64.so"):
                    path = name
                    break
        if path is None:
            raise RuntimeError("no HIP runtime (libamdhip64) is mapped into this process: torch did not load one")
        h = C.CDLL(path)
        h.hipHostMalloc.restype = C.c_int
        h.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), _sz, C.c_uint]
        h.hipHostFree.restype = C.c_int
        h.hipHostFree.argtypes = [C.c_void_p]
        h.hipStreamCreateWithFlags.restype = C.c_int
        h.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        h.hipStreamDestroy.restype = C.c_int
        h.hipStreamDestroy.argtypes = [C.c_void_p]
        _hip = h
    return _hip


class PoochError(RuntimeError):
    def __init__(self, status, msg):
        RuntimeError.__init__(self, "pooch status %d: %s" % (status, msg))
        self.status = status


class BudgetError(PoochError):
    pass


def _ints(v):
    return (C.c_int * len(v))(*[int(x) for x in v])


def _dptr(a):
    return a.ctypes.data_as(_pd)


class Context:
    """One pooch_ctx.  `budget_bytes` is the size of the arena.  With device=None the context
    is planning-only (no GPU touched): graph, profile injection, planning, simulation."""

    def __init__(self, net, budget_bytes, pinned_bytes=0, device="cuda:0", fuse=True, masks=False):
        self.L = lib()
        self.fuse = bool(fuse)
        self.masks = bool(masks)
        self.net = net
        self.budget_bytes = int(budget_bytes)
        self._keep = []          # python objects whose memory the library borrows
        arena_ptr = pinned_ptr = None
        streams = [None, None, None]
        self.torch = None
        if device is not None:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("no GPU: a compute context needs one (use device=None for planning only)")
            self.torch = torch
            self.device = torch.device(device)
            # blocks that torch's caching allocator still holds from earlier contexts go back to the driver first, so that
            # an arena close to the device's capacity fits after smaller ones
            torch.cuda.empty_cache()
            self.arena = torch.empty(self.budget_bytes, dtype=torch.uint8, device=self.device)
            assert self.arena.data_ptr() % 256 == 0
            arena_ptr = self.arena.data_ptr()
            self._pinned_ptr = None
            if pinned_bytes > 0:
                ptr = C.c_void_p()
                err = _hip_rt().hipHostMalloc(C.byref(ptr), int(pinned_bytes), 0)
                if err != 0 or not ptr.value:
                    raise MemoryError("hipHostMalloc of %d bytes of pinned host memory failed (HIP error %d)" % (pinned_bytes, err))
                self._pinned_ptr = ptr
                pinned_ptr = ptr.value
            # Three streams of our own, created one after the other (default priority, non-blocking).  Streams handed out by
            # torch's pool were seen to share a hardware queue with one another after many contexts had come and gone in one
            # process: swap copies then sat in front of kernels (a 40 ms wait charged to a filter gradient, the step 30 % slower).
            self._hip_streams = []
            for _ in range(3):
                sp = C.c_void_p()
                err = _hip_rt().hipStreamCreateWithFlags(C.byref(sp), 1)      # hipStreamNonBlocking
                if err != 0 or not sp.value:
                    raise RuntimeError("hipStreamCreateWithFlags failed (HIP error %d)" % err)
                self._hip_streams.append(sp)
            streams = [sp.value for sp in self._hip_streams]
        h = _ctx()
        st = self.L.pooch_create(arena_ptr, self.budget_bytes, pinned_ptr, int(pinned_bytes) if pinned_ptr else 0,
                                 streams[0], streams[1], streams[2], C.byref(h))
        if st != OK:
            raise PoochError(st, "pooch_create failed")
        self.h = h
        self._build(net)

    # ---- plumbing
    def _chk(self, st):
        if st < 0:
            msg = self.L.pooch_last_error(self.h).decode()
            raise (BudgetError if st == E_BUDGET else PoochError)(st, msg)
        return st

    def close(self):
        if getattr(self, "h", None):
            if self.torch is not None:
                self.torch.cuda.synchronize()
            self.L.pooch_destroy(self.h)
            self.h = None
            if getattr(self, "_pinned_ptr", None) is not None:
                _hip_rt().hipHostFree(self._pinned_ptr)
                self._pinned_ptr = None
            for sp in getattr(self, "_hip_streams", []):
                _hip_rt().hipStreamDestroy(sp)
            self._hip_streams = []
            self.arena = None
            if self.torch is not None:
                self.torch.cuda.empty_cache()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _build(self, net):
        L, h = self.L, self.h
        self._chk(L.pooch_set_fusion(h, 1 if self.fuse else 0))
        self._chk(L.pooch_set_relu_masks(h, 1 if self.masks else 0))
        for i, layer in enumerate(net):
            op = layer["op"]
            if op == "input":
                dims = (_i64 * len(layer["shape"]))(*layer["shape"])
                r = L.pooch_input(h, dims, len(layer["shape"]))
            elif op == "conv":
                r = L.pooch_conv(h, layer["x"], layer["cout"], _ints(layer["k"]), _ints(layer["stride"]), _ints(layer["pad"]), len(layer["k"]))
            elif op == "bn":
                r = L.pooch_bn(h, layer["x"], layer["eps"])
            elif op == "relu":
                r = L.pooch_relu(h, layer["x"])
            elif op == "add":
                r = L.pooch_add(h, layer["a"], layer["b"])
            elif op == "maxpool":
                r = L.pooch_maxpool(h, layer["x"], _ints(layer["k"]), _ints(layer["stride"]), _ints(layer["pad"]), len(layer["k"]))
            elif op == "gavgpool":
                r = L.pooch_gavgpool(h, layer["x"])
            elif op == "fc":
                r = L.pooch_fc(h, layer["x"], layer["nout"])
            elif op == "softmax_ce":
                r = L.pooch_softmax_ce(h, layer["x"])
            else:
                raise ValueError(op)
            self._chk(r)
            assert r == i
        self._chk(L.pooch_finalize(h))
        self.n_nodes = L.pooch_num_nodes(h)
        self.n_fmaps = self._chk(L.pooch_num_fmaps(h))
        self.n_params = self._chk(L.pooch_num_params(h))

    def node_fused(self, node):
        """id of the relu this layer is executed in, or -1"""
        return self.L.pooch_node_fused(self.h, node)

    def node_keeps_mask(self, node):
        """True if this relu / add + relu keeps a one-bit mask for its backward instead of its output"""
        return self._chk(self.L.pooch_node_keeps_mask(self.h, node)) == 1

    def bn_stats_source(self, node):
        """id of the conv whose forward also produces this bn layer's batch statistics, or -1"""
        return self.L.pooch_bn_stats_source(self.h, node)

    # ---- parameters and data
    def param_info(self, i):
        numel, node = _i64(), _i32()
        self._chk(self.L.pooch_param_info(self.h, i, C.byref(numel), C.byref(node)))
        return numel.value, node.value

    def set_params(self, params):
        assert len(params) == self.n_params
        for i, p in enumerate(params):
            a = np.ascontiguousarray(p, np.float32)
            assert a.size == self.param_info(i)[0]
            self._chk(self.L.pooch_set_param(self.h, i, a.ctypes.data))

    def get_grads(self, shapes=None):
        out = []
        for i in range(self.n_params):
            g = np.empty(self.param_info(i)[0], np.float32)
            self._chk(self.L.pooch_get_grad(self.h, i, g.ctypes.data))
            out.append(g.reshape(shapes[i]) if shapes is not None else g)
        return out

    def get_params(self, shapes=None):
        out = []
        for i in range(self.n_params):
            p = np.empty(self.param_info(i)[0], np.float32)
            self._chk(self.L.pooch_get_param(self.h, i, p.ctypes.data))
            out.append(p.reshape(shapes[i]) if shapes is not None else p)
        return out

    def sgd_update(self, lr):
        self._chk(self.L.pooch_sgd_update(self.h, lr))

    def profile_step(self, timed=True):
        loss = C.c_float()
        self._chk(self.L.pooch_profile_step(self.h, 1 if timed else 0, C.byref(loss)))
        return loss.value

    def finish_profile(self):
        self._chk(self.L.pooch_finish_profile(self.h))

    def set_batch(self, x, labels):
        x = np.ascontiguousarray(x, np.float32)
        labels = np.ascontiguousarray(labels, np.int32)
        assert tuple(x.shape) == tuple(self.net[0]["shape"]) and labels.shape == (x.shape[0],)
        self._chk(self.L.pooch_set_batch(self.h, x.ctypes.data, labels.ctypes.data))

    def capture(self, node, array):
        """array: C-contiguous float32 of the layer's logical shape, or None to cancel"""
        if array is not None:
            assert array.dtype == np.float32 and array.flags.c_contiguous
            self._keep.append(array)
        self._chk(self.L.pooch_capture_tensor(self.h, node, array.ctypes.data if array is not None else None))

    def inject_failure(self, command_index):
        """test aid: the next replay fails with E_HIP at this command (negative: cancel)"""
        self._chk(self.L.pooch_inject_failure(self.h, int(command_index)))

    def bn_stats(self, node, channels):
        mean = np.empty(channels, np.float32)
        istd = np.empty(channels, np.float32)
        self._chk(self.L.pooch_get_bn_stats(self.h, node, mean.ctypes.data, istd.ctypes.data))
        return mean, istd

    def set_bn_decay(self, decay):
        self._chk(self.L.pooch_set_bn_decay(self.h, float(decay)))

    def get_bn_running(self, node, channels):
        mean = np.empty(channels, np.float32)
        var = np.empty(channels, np.float32)
        self._chk(self.L.pooch_get_bn_running(self.h, node, mean.ctypes.data, var.ctypes.data))
        return mean, var

    def set_bn_running(self, node, mean, var):
        mean = np.ascontiguousarray(mean, np.float32)
        var = np.ascontiguousarray(var, np.float32)
        self._chk(self.L.pooch_set_bn_running(self.h, node, mean.ctypes.data, var.ctypes.data))

    # ---- feature maps
    def fmaps(self):
        """[(bytes, producer node)]"""
        out = []
        for i in range(self.n_fmaps):
            b, p = _sz(), _i32()
            self._chk(self.L.pooch_fmap_info(self.h, i, C.byref(b), C.byref(p)))
            out.append((b.value, p.value))
        return out

    def resident_bytes(self):
        return self.L.pooch_resident_bytes(self.h)

    # ---- the three phases
    def profile(self, warmup=1, iters=3):
        self._chk(self.L.pooch_profile(self.h, warmup, iters))
        return self.get_profile()

    def refine_profile(self, iters=2):
        """re-time the layers under the installed plan (ordinary steps); returns the last loss"""
        loss = C.c_float()
        self._chk(self.L.pooch_refine_profile(self.h, iters, C.byref(loss)))
        return loss.value

    def get_profile(self):
        a = [np.empty(self.n_nodes) for _ in range(3)] + [np.empty(self.n_fmaps) for _ in range(2)]
        self._chk(self.L.pooch_get_profile(self.h, *[_dptr(v) for v in a]))
        return a

    def set_profile(self, t_fwd, t_bwd, t_refwd, t_out, t_in):
        a = [np.ascontiguousarray(v, np.float64) for v in (t_fwd, t_bwd, t_refwd, t_out, t_in)]
        assert [len(v) for v in a] == [self.n_nodes] * 3 + [self.n_fmaps] * 2
        self._chk(self.L.pooch_set_profile(self.h, *[_dptr(v) for v in a]))

    def plan(self, mode, max_bits=0, restarts=None):
        if restarts is not None:
            self._chk(self.L.pooch_set_search_effort(self.h, restarts))
        t = _dbl()
        self._chk(self.L.pooch_plan(self.h, MODES[mode] if isinstance(mode, str) else mode, max_bits, C.byref(t)))
        return self.get_plan(), t.value

    def get_plan(self):
        cls = np.empty(self.n_fmaps, np.uint8)
        self._chk(self.L.pooch_get_plan(self.h, cls.ctypes.data_as(_pu8)))
        return cls

    def set_plan(self, cls, sched=True):
        cls = np.ascontiguousarray(cls, np.uint8)
        assert cls.size == self.n_fmaps
        self._chk(self.L.pooch_set_plan(self.h, cls.ctypes.data_as(_pu8), 1 if sched else 0))

    def simulate(self, cls, sched=True, want_time=True):
        cls = np.ascontiguousarray(cls, np.uint8)
        assert cls.size == self.n_fmaps
        t, peak = _dbl(), _sz()
        self._chk(self.L.pooch_simulate(self.h, cls.ctypes.data_as(_pu8), 1 if sched else 0,
                                        C.byref(t) if want_time else None, C.byref(peak)))
        return (t.value if want_time else None), peak.value

    def plan_evaluations(self):
        return self.L.pooch_plan_evaluations(self.h)

    def overhead_sets(self):
        lo = np.empty(self.n_fmaps, np.uint8)
        li = np.empty(self.n_fmaps, np.uint8)
        self._chk(self.L.pooch_get_overhead_sets(self.h, lo.ctypes.data_as(_pu8), li.ctypes.data_as(_pu8)))
        return lo, li

    def commands(self):
        n = _i64()
        self._chk(self.L.pooch_get_commands(self.h, None, 0, C.byref(n)))
        rows = np.empty((n.value, 8), np.int64)
        self._chk(self.L.pooch_get_commands(self.h, rows.ctypes.data_as(_pi64), n.value, C.byref(n)))
        return rows

    def step(self):
        loss = C.c_float()
        self._chk(self.L.pooch_step(self.h, C.byref(loss)))
        return loss.value

    def step_static_scratch(self):
        """pooch_step with the kernels' scratch in the library's static device array (allocates nothing)"""
        loss = C.c_float()
        self._chk(self.L.pooch_step_static_scratch(self.h, C.byref(loss)))
        return loss.value

    def step_timed(self):
        loss = C.c_float()
        a = [np.empty(self.n_nodes) for _ in range(4)]
        self._chk(self.L.pooch_step_timed(self.h, C.byref(loss), *[_dptr(v) for v in a]))
        return loss.value, a[0], a[1], a[2], a[3]

    def node_kernel(self, node, part):
        return self.L.pooch_node_kernel(self.h, node, part).decode()

    def stats(self):
        s = Stats()
        self._chk(self.L.pooch_get_stats(self.h, C.byref(s)))
        return s

    def measure_link(self, nbytes, iters=5):
        a, b = _dbl(), _dbl()
        self._chk(self.L.pooch_measure_link(self.h, int(nbytes), iters, C.byref(a), C.byref(b)))
        return a.value, b.value
