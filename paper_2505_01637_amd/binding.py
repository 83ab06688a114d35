"""Thin ctypes binding of libmorello_mi355x.so (include/morello_mi355x.h).

Argument marshalling only: every step of the hot path runs in the library's
HIP kernels.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: importing works without a GPU, calling `solve` does not.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmorello_mi355x.so")

INF = (1 << 64) - 1
NONE = 0xFFFF
MAX_DIMS = 16
NOALLOC_MAX_QUERIES = 4096

OK, E_INVAL, E_NOMEM, E_HIP, E_RANGE, E_BUFSZ, E_OVERFLOW = 0, -1, -2, -3, -4, -5, -6

EXPORTS = ["mrl_target_create", "mrl_target_destroy", "mrl_geometry", "mrl_table_bytes", "mrl_solve", "mrl_solve_graph",
           "mrl_table_destroy", "mrl_query", "mrl_query_noalloc", "mrl_query_compressed", "mrl_rewrite_decode", "mrl_coord_of_spec",
           "mrl_emit_compressed", "mrl_schedule", "mrl_copy_dense", "mrl_last_error"]


class MorelloError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("mrl error %d: %s" % (code, msg))
        self.code = code


class _Microkernel(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("lanes", C.c_uint32), ("cost", C.c_uint64)]


class _TargetDesc(C.Structure):
    _fields_ = [("n_levels", C.c_uint32),
                ("capacity_bytes", C.c_uint64 * 4),
                ("load_coef", C.c_uint32 * 2 * 4 * 4),
                ("store_coef", C.c_uint32 * 2 * 4 * 4),
                ("convert_coef", C.c_uint32),
                ("zero_coef", C.c_uint32 * 4),
                ("loop_overhead", C.c_uint32),
                ("n_microkernels", C.c_uint32),
                ("mk", _Microkernel * 8),
                ("threads", C.c_uint32),
                ("sync_cost", C.c_uint32),
                ("level_weight", C.c_uint32 * 4),
                ("line_bytes", C.c_uint32),
                ("strip", C.c_uint32)]


class _LatticeDesc(C.Structure):
    _fields_ = [("kind", C.c_uint32),
                ("n_sizes", C.c_uint32 * 4),
                ("sizes", C.POINTER(C.c_uint32) * 4),
                ("layout_coord", C.c_uint8 * 5),
                ("dtype_coord", C.c_uint8 * 5),
                ("base_dtype_bytes", C.c_uint8 * 5)]


class Stats(C.Structure):
    _fields_ = [("n_specs", C.c_uint64), ("n_admissible", C.c_uint64), ("n_rewrites", C.c_uint64),
                ("n_levels_run", C.c_uint32), ("fill_ms", C.c_float), ("compress_ms", C.c_float),
                ("n_decision_boxes", C.c_uint64), ("n_cost_boxes", C.c_uint64),
                ("scratch_used", C.c_uint64), ("prefill_ms", C.c_float)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class _Coord(C.Structure):
    _fields_ = [("x", C.c_uint32 * MAX_DIMS)]


class _ScheduleNode(C.Structure):
    _fields_ = [("table", C.c_uint32), ("rewrite", C.c_uint16), ("n_children", C.c_uint16),
                ("cost", C.c_uint64), ("spec", _Coord)]


class Rewrite(C.Structure):
    _fields_ = [("cls", C.c_uint8), ("operand_or_dim", C.c_uint8), ("dst_level", C.c_uint8),
                ("transposed", C.c_uint8), ("convert", C.c_uint8),
                ("tile_size", C.c_uint32), ("mk_index", C.c_uint32)]


BOX_DTYPE = np.dtype([("lo", np.uint16, (MAX_DIMS,)), ("hi", np.uint16, (MAX_DIMS,)),
                      ("v0", np.uint64), ("v1", np.uint64)])

_lib = None


def lib():
    """Load the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run __graft_entry__.build() (hipcc, gfx950)" % LIB_PATH)
        # torch first: it brings its own HIP runtime, and the library must share that one.  Loaded the
        # other way round the process holds two runtimes and the library's finds no device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        _lib = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(_lib, name).restype = C.c_int32
        _lib.mrl_last_error.restype = C.c_char_p
        _lib.mrl_target_destroy.restype = None
        _lib.mrl_table_destroy.restype = None
    return _lib


def _check(rc):
    if rc != 0:
        raise MorelloError(rc, lib().mrl_last_error().decode())


def _target_desc(t):
    d = _TargetDesc()
    d.n_levels = t["n_levels"]
    for l in range(4):
        d.capacity_bytes[l] = t["capacity_bytes"][l]
        d.zero_coef[l] = t["zero_coef"][l]
        for k in range(4):
            for x in range(2):
                d.load_coef[l][k][x] = t["load_coef"][l][k][x]
                d.store_coef[l][k][x] = t["store_coef"][l][k][x]
    d.convert_coef = t["convert_coef"]
    d.loop_overhead = t["loop_overhead"]
    d.n_microkernels = len(t["microkernels"])
    for j, (kind, lanes, cost) in enumerate(t["microkernels"][:8]):
        d.mk[j].kind, d.mk[j].lanes, d.mk[j].cost = kind, lanes, cost
    d.threads = t.get("threads", 1)
    d.sync_cost = t.get("sync_cost", 0)
    for l in range(4):
        d.level_weight[l] = t.get("level_weight", [0, 0, 0, 0])[l]
    d.line_bytes = t.get("line_bytes", 0)
    d.strip = t.get("strip", 0)
    return d


def _lattice_desc(lat):
    d = _LatticeDesc()
    d.kind = lat["kind"]
    keep = []
    for a in range(4):
        arr = (C.c_uint32 * max(1, len(lat["sizes"][a])))(*lat["sizes"][a])
        keep.append(arr)
        d.n_sizes[a] = len(lat["sizes"][a])
        d.sizes[a] = C.cast(arr, C.POINTER(C.c_uint32))
    for i in range(5):
        d.layout_coord[i] = lat["layout_coord"][i]
        d.dtype_coord[i] = lat["dtype_coord"][i]
        d.base_dtype_bytes[i] = lat["base_dtype_bytes"][i]
    d._keep = keep
    return d


class Target:
    def __init__(self, desc):
        self._h = C.c_void_p()
        _check(lib().mrl_target_create(C.byref(_target_desc(desc)), C.byref(self._h)))

    def close(self):
        if self._h:
            lib().mrl_target_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def geometry(target, lattice, desc=None):
    """(extents, number of Specs); desc: the lattice's descriptor if the caller has built it."""
    nd, n = C.c_uint32(), C.c_uint64()
    ext = (C.c_uint32 * MAX_DIMS)()
    L = _lattice_desc(lattice) if desc is None else desc
    _check(lib().mrl_geometry(target._h, C.byref(L), C.byref(nd), ext, C.byref(n)))
    return list(ext[:nd.value]), n.value


def table_bytes(target, lattice):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().mrl_table_bytes(target._h, C.byref(_lattice_desc(lattice)), C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


class Table:
    """A solved table.  Holds the torch tensors that back it."""

    def __init__(self, handle, target, lattice, extents, tensors, stats, deps=()):
        self._h, self.target, self.lattice = handle, target, lattice
        self.extents, self._tensors, self.stats = extents, tensors, stats
        self._deps = tuple(deps)        # keeps the tables this one was solved against alive
        self.n_specs = int(np.prod(extents, dtype=np.uint64))

    def close(self):
        if self._h:
            lib().mrl_table_destroy(self._h)
            self._h = C.c_void_p()
            self._tensors = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def query(self, coords, compressed=False, noalloc=False):
        """(cost, rewrite id) of the Specs at `coords`; compressed=True answers from the two box
        lists alone (mrl_query_compressed) instead of the dense table; noalloc=True asks through
        mrl_query_noalloc (at most NOALLOC_MAX_QUERIES coordinates)."""
        coords = np.ascontiguousarray(coords, dtype=np.uint32).reshape(-1, len(self.extents))
        n = len(coords)
        buf = np.zeros((n, MAX_DIMS), dtype=np.uint32)
        buf[:, :coords.shape[1]] = coords
        cost = np.empty(n, dtype=np.uint64)
        rw = np.empty(n, dtype=np.uint16)
        fn = lib().mrl_query_compressed if compressed else lib().mrl_query_noalloc if noalloc else lib().mrl_query
        _check(fn(self._h, buf.ctypes.data_as(C.POINTER(_Coord)), C.c_size_t(n),
                  cost.ctypes.data_as(C.POINTER(C.c_uint64)), rw.ctypes.data_as(C.POINTER(C.c_uint16))))
        return cost, rw

    def schedule(self, coord):
        """Program of the Spec at `coord`: [(table, coord, rewrite id, cost, children)] in
        pre-order; table 0 = this table, 1 + i = the i-th table it was solved against, 3 + i = the
        i-th table that one's second dep was solved against."""
        goal = _Coord()
        for a, v in enumerate(coord):
            goal.x[a] = int(v)
        n = C.c_size_t()
        _check(lib().mrl_schedule(self._h, C.byref(goal), None, C.c_size_t(0), C.byref(n)))
        nodes = (_ScheduleNode * max(1, n.value))()
        _check(lib().mrl_schedule(self._h, C.byref(goal), nodes, C.c_size_t(n.value), C.byref(n)))
        dims = [len(t.extents) for t in self._schedule_tables()]
        return [(nd.table, tuple(nd.spec.x[:dims[nd.table]]), nd.rewrite, nd.cost, nd.n_children)
                for nd in nodes[:n.value]]

    def _schedule_tables(self):
        """Tables by the index a schedule node carries: this one, its deps, then the deps of its dep 1."""
        tabs = (self,) + tuple(self._deps)
        if len(self._deps) > 1:
            tabs += (None,) * (3 - len(tabs)) + tuple(self._deps[1]._deps)
        return tabs

    def program_text(self, coord):
        """The program of `coord` as indented text, one rewrite per line (the nesting of Section 2,
        Figure 1: a Move or a loop encloses the Spec it leaves, a microkernel is a leaf)."""
        tabs = self._schedule_tables()
        lines, open_children = [], []
        for t, x, rid, cost, k in self.schedule(coord):
            tab = tabs[t]
            sizes = tab.lattice["sizes"]
            r = tab.rewrite_decode(rid)
            if r.cls == 0:
                what = "microkernel %d" % r.mk_index
            elif r.cls == 1:
                what = "move operand %d to level %d%s%s" % (r.operand_or_dim, r.dst_level,
                                                           ", transposed" if r.transposed else "",
                                                           ", converted" if r.convert else "")
            elif r.cls == 2:
                d = r.operand_or_dim
                what = "loop over %s: %d steps of %d" % ("bmkn"[d], sizes[d][x[d]] // r.tile_size, r.tile_size)
            elif r.cls == 4:
                d = r.operand_or_dim
                what = "parallel loop over %s: %d steps of %d, serial-only body" % (
                    "bmkn"[d], sizes[d][x[d]] // r.tile_size, r.tile_size)
            else:
                what = "bufferize: the first stage into the intermediate, then the second out of it"
            lines.append("%stable %d  %s  %s  cost %d  %s" % ("  " * len(open_children), t,
                         "x".join(str(sizes[d][x[d]]) for d in range(4)), tuple(x[4:]), cost, what))
            if k:
                open_children.append(k)
            else:
                while open_children:
                    open_children[-1] -= 1
                    if open_children[-1]:
                        break
                    open_children.pop()
        return "\n".join(lines)

    def rewrite_decode(self, rid):
        r = Rewrite()
        _check(lib().mrl_rewrite_decode(self._h, C.c_uint16(rid), C.byref(r)))
        return r

    def coord_of_spec(self, shape, levels, layouts=None, dtypes=None):
        sh = (C.c_uint32 * 4)(*shape)
        lv = (C.c_uint8 * 5)(*(list(levels) + [0] * (5 - len(levels))))
        ly = (C.c_uint8 * 5)(*(list(layouts or []) + [0] * (5 - len(layouts or []))))
        dt = (C.c_uint8 * 5)(*(list(dtypes or []) + [0] * (5 - len(dtypes or []))))
        out = _Coord()
        _check(lib().mrl_coord_of_spec(self._h, sh, lv, ly, dt, C.byref(out)))
        return list(out.x[:len(self.extents)])

    def boxes(self, which):
        """which: 0 decisions, 1 costs.  numpy structured array (BOX_DTYPE), sorted by lo."""
        n = C.c_size_t()
        _check(lib().mrl_emit_compressed(self._h, C.c_uint32(which), None, C.c_size_t(0), C.byref(n)))
        out = np.zeros(n.value, dtype=BOX_DTYPE)
        _check(lib().mrl_emit_compressed(self._h, C.c_uint32(which), C.c_void_p(out.ctypes.data),
                                         C.c_size_t(n.value), C.byref(n)))
        return out

    def dense(self):
        cost = np.empty(self.n_specs, dtype=np.uint64)
        arg = np.empty(self.n_specs, dtype=np.uint16)
        _check(lib().mrl_copy_dense(self._h, cost.ctypes.data_as(C.POINTER(C.c_uint64)),
                                    arg.ctypes.data_as(C.POINTER(C.c_uint16))))
        return cost, arg


def solve(target, lattice, deps=(), scratch_bytes=None, stream=None, buffers=None):
    """Fill and compress one lattice on the current CUDA/HIP device.

    target: Target; lattice: dict (workloads.py); deps: solved Tables a fused
    lattice reads.  buffers: optional (cost, argmin, scratch) torch uint8
    tensors to reuse.  Device memory comes from torch; nothing else does.
    """
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("mrl solve needs a GPU: there is no CPU path")
    L = _lattice_desc(lattice)
    ext, n = geometry(target, lattice, desc=L)
    cb, ab = 8 * n, 2 * n
    if buffers is None:
        sb = table_bytes(target, lattice)[2] if scratch_bytes is None else scratch_bytes
        dev = torch.device("cuda", torch.cuda.current_device())
        buffers = (torch.empty(cb, dtype=torch.uint8, device=dev),
                   torch.empty(ab, dtype=torch.uint8, device=dev),
                   torch.empty(sb, dtype=torch.uint8, device=dev))
    d_cost, d_arg, d_scr = buffers
    assert d_cost.numel() >= cb and d_arg.numel() >= ab
    st = torch.cuda.current_stream() if stream is None else stream
    dep_arr = (C.c_void_p * max(1, len(deps)))(*[d._h for d in deps])
    h = C.c_void_p()
    stats = Stats()
    rc = lib().mrl_solve(target._h, C.byref(L), dep_arr if deps else None, C.c_uint32(len(deps)),
                         C.c_void_p(d_cost.data_ptr()), C.c_void_p(d_arg.data_ptr()),
                         C.c_void_p(d_scr.data_ptr()), C.c_size_t(d_scr.numel()),
                         C.c_void_p(st.cuda_stream), C.byref(h), C.byref(stats))
    _check(rc)
    return Table(h, target, lattice, ext, buffers, stats, deps)


_side_streams = {}


def _side_stream(dev, i):
    """The i-th extra stream of a device for the calling thread (default priority), created once."""
    import threading
    import torch
    pool = _side_streams.setdefault((dev, threading.get_ident()), [])
    while len(pool) <= i:
        pool.append(torch.cuda.Stream(device=dev))
    return pool[i]


class _Job(C.Structure):
    _fields_ = [("lattice", C.c_void_p), ("n_deps", C.c_uint32), ("deps", C.c_uint32 * 2),
                ("d_cost", C.c_void_p), ("d_argmin", C.c_void_p), ("d_scratch", C.c_void_p),
                ("scratch_bytes", C.c_size_t), ("hip_stream", C.c_void_p)]


def solve_lattices(target, lattices, scratch_bytes=None, buffers=None):
    """Solve [(label, lattice, dep labels)] with one call of mrl_solve_graph; returns {label: Table}.

    The library runs every lattice from a host thread of its own, on a stream of its own
    (default priority): lattices that do not depend on each other overlap on the device, and a
    lattice starts when the fill of those it reads is queued, while they are still being
    compressed.  buffers: optional {label: (cost, argmin, scratch)} torch uint8 tensors to reuse.
    """
    # dependency order (checked before any device work)
    order, seen, left = [], set(), list(lattices)
    while left:
        ok = [job for job in left if all(d in seen for d in job[2])]
        if not ok:
            raise ValueError("lattice dependencies form a cycle or name an unknown label")
        order += ok
        seen.update(job[0] for job in ok)
        left = [job for job in left if job[0] not in seen]
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("mrl solve needs a GPU: there is no CPU path")
    dev = torch.cuda.current_device()
    device = torch.device("cuda", dev)
    index = {job[0]: i for i, job in enumerate(order)}
    jobs = (_Job * len(order))()
    keep, held, exts = [], [], []
    for i, (label, lat, deps) in enumerate(order):
        L = _lattice_desc(lat)
        keep.append(L)
        ext, n = geometry(target, lat, desc=L)
        exts.append(ext)
        if buffers is None:
            sb = table_bytes(target, lat)[2] if scratch_bytes is None else scratch_bytes
            bufs = (torch.empty(8 * n, dtype=torch.uint8, device=device),
                    torch.empty(2 * n, dtype=torch.uint8, device=device),
                    torch.empty(sb, dtype=torch.uint8, device=device))
        else:
            bufs = buffers[label]
        assert bufs[0].numel() >= 8 * n and bufs[1].numel() >= 2 * n
        held.append(bufs)
        jobs[i].lattice = C.cast(C.pointer(L), C.c_void_p)
        jobs[i].n_deps = len(deps)
        for k, d in enumerate(deps):
            jobs[i].deps[k] = index[d]
        jobs[i].d_cost, jobs[i].d_argmin, jobs[i].d_scratch = (b.data_ptr() for b in bufs)
        jobs[i].scratch_bytes = bufs[2].numel()
        # the last lattice (on the calling thread) takes the current stream, the others side streams
        last = i == len(order) - 1
        jobs[i].hip_stream = torch.cuda.current_stream().cuda_stream if last else _side_stream(dev, i).cuda_stream
    handles = (C.c_void_p * len(order))()
    stats = (Stats * len(order))()
    torch.cuda.synchronize()            # the side streams start after everything queued so far
    _check(lib().mrl_solve_graph(target._h, jobs, C.c_uint32(len(order)), handles, stats))
    done = {}
    for i, (label, lat, deps) in enumerate(order):
        st = Stats.from_buffer_copy(stats[i])
        done[label] = Table(C.c_void_p(handles[i]), target, lat, exts[i], held[i], st, [done[d] for d in deps])
    return done


def solve_config(cfg, scratch_bytes=None):
    """Solve every lattice of a workloads.config() dict.  Returns (Target, {label: Table})."""
    target = Target(cfg["target"])
    return target, solve_lattices(target, cfg["lattices"], scratch_bytes=scratch_bytes)
