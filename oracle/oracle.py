"""ctypes wrapper around the C oracle (oracle/morello_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, the smoke check and the
benchmark's CPU-baseline leg.  It never imports the HIP package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "morello_oracle.c")
_LIB = os.path.join(_HERE, "libmorello_oracle.so")

INF = (1 << 64) - 1
NONE = 0xFFFF
MAXD = 16


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


class _Target(C.Structure):
    _fields_ = [("n_levels", C.c_uint32),
                ("capacity_bytes", C.c_uint64 * 4),
                ("load_coef", C.c_uint32 * 2 * 4 * 4),
                ("store_coef", C.c_uint32 * 2 * 4 * 4),
                ("convert_coef", C.c_uint32),
                ("zero_coef", C.c_uint32 * 4),
                ("loop_overhead", C.c_uint32),
                ("n_microkernels", C.c_uint32),
                ("mk_kind", C.c_uint32 * 8),
                ("mk_lanes", C.c_uint32 * 8),
                ("mk_cost", C.c_uint64 * 8),
                ("threads", C.c_uint32),
                ("sync_cost", C.c_uint32),
                ("level_weight", C.c_uint32 * 4),
                ("line_bytes", C.c_uint32),
                ("strip", C.c_uint32)]


class _Lattice(C.Structure):
    _fields_ = [("kind", C.c_uint32),
                ("n_sizes", C.c_uint32 * 4),
                ("sizes", C.POINTER(C.c_uint32) * 4),
                ("layout_coord", C.c_uint8 * 5),
                ("dtype_coord", C.c_uint8 * 5),
                ("base_dtype_bytes", C.c_uint8 * 5)]


class Box(C.Structure):
    _fields_ = [("lo", C.c_uint16 * MAXD), ("hi", C.c_uint16 * MAXD),
                ("v0", C.c_uint64), ("v1", C.c_uint64)]


BOX_DTYPE = np.dtype([("lo", np.uint16, (MAXD,)), ("hi", np.uint16, (MAXD,)),
                      ("v0", np.uint64), ("v1", np.uint64)])

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_solve.restype = C.c_int
        _lib.orc_geometry.restype = C.c_int
        _lib.orc_cost_values.restype = C.c_int
        _lib.orc_merge.restype = C.c_int64
        _lib.orc_decompress.restype = C.c_int
        _lib.orc_free.restype = None
    return _lib


def _target(t):
    s = _Target()
    s.n_levels = t["n_levels"]
    for l in range(4):
        s.capacity_bytes[l] = t["capacity_bytes"][l]
        s.zero_coef[l] = t["zero_coef"][l]
        for k in range(4):
            for x in range(2):
                s.load_coef[l][k][x] = t["load_coef"][l][k][x]
                s.store_coef[l][k][x] = t["store_coef"][l][k][x]
    s.convert_coef = t["convert_coef"]
    s.loop_overhead = t["loop_overhead"]
    s.n_microkernels = len(t["microkernels"])
    for j, (kind, lanes, cost) in enumerate(t["microkernels"]):
        s.mk_kind[j], s.mk_lanes[j], s.mk_cost[j] = kind, lanes, cost
    s.threads = t.get("threads", 1)
    s.sync_cost = t.get("sync_cost", 0)
    for l in range(4):
        s.level_weight[l] = t.get("level_weight", [0, 0, 0, 0])[l]
    s.line_bytes = t.get("line_bytes", 0)
    s.strip = t.get("strip", 0)
    return s


def _lattice(lat):
    s = _Lattice()
    keep = []
    s.kind = lat["kind"]
    for d in range(4):
        arr = (C.c_uint32 * len(lat["sizes"][d]))(*lat["sizes"][d])
        keep.append(arr)
        s.n_sizes[d] = len(lat["sizes"][d])
        s.sizes[d] = C.cast(arr, C.POINTER(C.c_uint32))
    for i in range(5):
        s.layout_coord[i] = lat["layout_coord"][i]
        s.dtype_coord[i] = lat["dtype_coord"][i]
        s.base_dtype_bytes[i] = lat["base_dtype_bytes"][i]
    s._keep = keep
    return s


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def layout_offset(layout, rows, cols, strip, i, j):
    """Buffer offset of element (i, j) of a rows x cols tensor (Section 2.4.2): layout 0 row-major,
    1 column-major, 2 packed in strips of `strip` columns, 3 packed with odd-even shuffled strips."""
    f = lib().orc_layout_offset
    f.restype = C.c_uint64
    f.argtypes = [C.c_uint32] + [C.c_uint64] * 5
    return int(f(layout, rows, cols, strip, i, j))


def geometry(target, lattice):
    """(extents, merge_order, ids) with ids = dict(move_base, tile_base, bufferize, maxs)."""
    T, L = _target(target), _lattice(lattice)
    nd = C.c_uint32()
    ext = (C.c_uint32 * MAXD)()
    mo = (C.c_uint32 * MAXD)()
    ids = (C.c_uint32 * 4)()
    rc = lib().orc_geometry(C.byref(T), C.byref(L), C.byref(nd), ext, mo, ids)
    if rc:
        raise ValueError("orc_geometry failed: %d" % rc)
    n = nd.value
    return list(ext[:n]), list(mo[:n]), {"move_base": ids[0], "tile_base": ids[1],
                                        "bufferize": ids[2], "maxs": ids[3]}


def solve(target, lattice, deps=None, goals=None):
    """Fill the table.  deps = ((latticeM, costM), (latticeE, costE)) for kind F,
    ((latticeM, costM),) for kind P (the serial-only table of the same lattice) and for
    kind 8 (the table of Move Specs).
    Returns dict(cost u64[N], argmin u16[N], n_admissible, n_rewrites, rc)."""
    T, L = _target(target), _lattice(lattice)
    ext, _, _ = geometry(target, lattice)
    n = int(np.prod(ext, dtype=np.uint64))
    cost = np.empty(n, dtype=np.uint64)
    arg = np.empty(n, dtype=np.uint16)
    na, nr = C.c_uint64(), C.c_uint64()
    LM = LE = None
    cM = cE = None
    if deps is not None:
        LM = _lattice(deps[0][0])
        cM = np.ascontiguousarray(deps[0][1], dtype=np.uint64)
        if len(deps) > 1:
            LE = _lattice(deps[1][0])
            cE = np.ascontiguousarray(deps[1][1], dtype=np.uint64)
    g = None if goals is None else np.ascontiguousarray(goals, dtype=np.uint64)
    rc = lib().orc_solve(
        C.byref(T), C.byref(L),
        C.byref(LM) if LM is not None else None, _p(cM, C.c_uint64) if cM is not None else None,
        C.byref(LE) if LE is not None else None, _p(cE, C.c_uint64) if cE is not None else None,
        _p(g, C.c_uint64) if g is not None else None, C.c_uint64(0 if g is None else len(g)),
        _p(cost, C.c_uint64), _p(arg, C.c_uint16), C.byref(na), C.byref(nr))
    if rc not in (0, -6):
        raise ValueError("orc_solve failed: %d" % rc)
    return {"cost": cost, "argmin": arg, "n_admissible": na.value, "n_rewrites": nr.value,
            "rc": rc, "extents": ext}


def cost_values(target, lattice, cost):
    T, L = _target(target), _lattice(lattice)
    cost = np.ascontiguousarray(cost, dtype=np.uint64)
    v0 = np.empty_like(cost)
    v1 = np.empty_like(cost)
    rc = lib().orc_cost_values(C.byref(T), C.byref(L), _p(cost, C.c_uint64),
                               _p(v0, C.c_uint64), _p(v1, C.c_uint64))
    if rc:
        raise ValueError("orc_cost_values failed: %d" % rc)
    return v0, v1


def merge(ext, merge_order, v0, v1, first_pass_by_lines=True):
    """Canonical box list (numpy structured array, BOX_DTYPE) of a dense table."""
    e = (C.c_uint32 * len(ext))(*ext)
    mo = (C.c_uint32 * len(merge_order))(*merge_order)
    v0 = np.ascontiguousarray(v0, dtype=np.uint64)
    v1 = np.ascontiguousarray(v1, dtype=np.uint64)
    out = C.POINTER(Box)()
    nb = lib().orc_merge(C.c_uint32(len(ext)), e, mo, C.c_uint32(len(merge_order)),
                         _p(v0, C.c_uint64), _p(v1, C.c_uint64),
                         C.c_int(1 if first_pass_by_lines else 0), C.byref(out))
    if nb < 0:
        raise MemoryError("orc_merge failed: %d" % nb)
    buf = C.string_at(out, nb * C.sizeof(Box))
    lib().orc_free(out)
    return np.frombuffer(buf, dtype=BOX_DTYPE).copy()


def decompress(ext, boxes):
    n = int(np.prod(ext, dtype=np.uint64))
    e = (C.c_uint32 * len(ext))(*ext)
    boxes = np.ascontiguousarray(boxes, dtype=BOX_DTYPE)
    v0 = np.zeros(n, dtype=np.uint64)
    v1 = np.zeros(n, dtype=np.uint64)
    cover = np.zeros(n, dtype=np.uint8)
    rc = lib().orc_decompress(C.c_uint32(len(ext)), e, C.cast(boxes.ctypes.data, C.POINTER(Box)),
                              C.c_uint64(len(boxes)), _p(v0, C.c_uint64), _p(v1, C.c_uint64),
                              _p(cover, C.c_uint8))
    if rc:
        raise ValueError("orc_decompress: box outside the lattice")
    return v0, v1, cover


def query_boxes(lattice, dec, cst, coords):
    """Point queries answered from the two box lists alone (Section 4.1: the table is kept as
    boxes and a lookup finds the box that holds the Spec's coordinate).

    By the definition of the lists: exactly one box of each list contains the coordinate.  The
    decision box gives the rewrite id; the cost box gives cost / volume as a reduced fraction
    v0/v1, so cost = v0 * volume / v1 with volume = b*m*k*n of the Spec's sizes ((INF, 0) stands
    for no implementation).  A linear scan over the boxes: slow, for tests only."""
    sizes = lattice["sizes"]
    cost, arg = [], []
    for x in np.asarray(coords, dtype=np.int64).reshape(len(coords), -1):
        nd = len(x)
        found = []
        for boxes in (dec, cst):
            inside = np.all((boxes["lo"][:, :nd] <= x) & (x <= boxes["hi"][:, :nd]), axis=1)
            hit = np.flatnonzero(inside)
            if len(hit) != 1:
                raise ValueError("coordinate %s lies in %d boxes" % (list(x), len(hit)))
            found.append(boxes[hit[0]])
        vol = 1
        for d in range(4):
            vol *= int(sizes[d][x[d]])
        v0, v1 = int(found[1]["v0"]), int(found[1]["v1"])
        if v1 == 0:
            cost.append(INF)
        else:
            if (v0 * vol) % v1:
                raise ValueError("cost fraction times volume is not an integer")
            cost.append(v0 * vol // v1)
        arg.append(int(found[0]["v0"]))
    return np.array(cost, dtype=np.uint64), np.array(arg, dtype=np.uint16)


def compress_table(target, lattice, cost, argmin):
    """Both box lists of a solved table: (decision_boxes, cost_boxes)."""
    ext, mo, _ = geometry(target, lattice)
    dec = merge(ext, mo, argmin.astype(np.uint64), np.zeros(len(argmin), dtype=np.uint64))
    v0, v1 = cost_values(target, lattice, cost)
    cst = merge(ext, mo, v0, v1)
    return dec, cst


def solve_config(cfg, goals=None):
    """Solve every lattice of a workloads.config() dict in order; returns {label: result}."""
    out = {}
    for label, lat, deps in cfg["lattices"]:
        d = None
        if deps:
            d = tuple((next(l for (lb, l, _) in cfg["lattices"] if lb == name), out[name]["cost"])
                      for name in deps)
        out[label] = solve(cfg["target"], lat, deps=d, goals=goals)
        out[label]["lattice"] = lat
    return out


# ---------------------------------------------------------------------------
# The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a stand-alone
# executable (sanitize_driver.c, which includes the oracle's source) reads a
# problem from a file and writes every result to another.

_DRIVER_SRC = os.path.join(_HERE, "sanitize_driver.c")


def build_sanitized(workdir):
    exe = os.path.join(workdir, "oracle_sanitized")
    subprocess.check_call(["gcc", "-O1", "-g", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe, _DRIVER_SRC])
    return exe


def run_sanitized(exe, cfg, workdir):
    """Solve and compress every lattice of `cfg` in the sanitized executable.  Returns
    {label: dict(rc, cost, argmin, n_admissible, n_rewrites, decision_boxes, cost_boxes)}."""
    labels = [label for label, _, _ in cfg["lattices"]]
    blob = bytearray(bytes(_target(cfg["target"])))
    blob += np.uint32(len(labels)).tobytes()
    for label, lat, deps in cfg["lattices"]:
        blob += np.uint32(lat["kind"]).tobytes()
        blob += np.array([len(s) for s in lat["sizes"]], dtype=np.uint32).tobytes()
        for s in lat["sizes"]:
            blob += np.array(s, dtype=np.uint32).tobytes()
        for key in ("layout_coord", "dtype_coord", "base_dtype_bytes"):
            blob += np.array(lat[key], dtype=np.uint8).tobytes()
        dep = [labels.index(d) for d in deps] + [-1, -1]
        blob += np.array(dep[:2], dtype=np.int32).tobytes()
    src, dst = os.path.join(workdir, "problem.bin"), os.path.join(workdir, "result.bin")
    with open(src, "wb") as f:
        f.write(bytes(blob))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    done = subprocess.run([exe, src, dst], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if done.returncode != 0:
        raise RuntimeError("sanitized oracle failed (status %d):\n%s" % (done.returncode, done.stdout[-4000:]))
    raw = open(dst, "rb").read()
    out, at = {}, 0

    def take(dtype, count):
        nonlocal at
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=at)
        at += a.nbytes
        return a

    for label in labels:
        rc = int(take(np.int32, 1)[0])
        n = int(take(np.uint64, 1)[0])
        r = {"rc": rc, "cost": take(np.uint64, n), "argmin": take(np.uint16, n)}
        r["n_admissible"], r["n_rewrites"] = (int(v) for v in take(np.uint64, 2))
        for key in ("decision_boxes", "cost_boxes"):
            nb = int(take(np.uint64, 1)[0])
            r[key] = take(BOX_DTYPE, nb)
        out[label] = r
    assert at == len(raw)
    return out
