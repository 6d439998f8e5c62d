"""Thin ctypes binding of the C ABI in include/gtree.h.

Argument marshalling only: device memory comes from PyTorch (int64 tensors used as
raw 64-bit words), every protocol step runs in the HIP library.  There is no CPU
fallback: if the library is missing, loading fails loudly.
"""
import ctypes as C
import os
import re

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgtree_hip.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "gtree.h")

GT_OK, GT_EINVAL, GT_ENOMEM, GT_ESTATE, GT_EHIP = 0, -1, -2, -3, -4
X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_L, X_SCORE, X_C_PAPER = range(9)


class GtError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, _strerror(code), code))


class _Plane2(C.Structure):
    _fields_ = [("own", C.c_void_p), ("next", C.c_void_p)]


class _Shares(C.Structure):
    _fields_ = [("party", _Plane2 * 3), ("n", C.c_size_t)]


class _Stats(C.Structure):
    _fields_ = [("rounds", C.c_uint64), ("wire_bytes", (C.c_uint64 * 3) * 3), ("wire_bits_dev", (C.c_uint64 * 3) * 3),
                ("scorer_bytes", C.c_uint64 * 2), ("kernel_ms", C.c_double)]


GT_FLAG_PROFILE = 1
GT_FLAG_LEVELWISE_INFER = 2
GT_FLAG_INFER_TILE = {16: 0x100, 32: 0x200, 64: 0x300}
KC_NAMES = ("share", "mult", "eqgrid", "count", "small", "local", "eqgrid_rows", "eqgrid_store", "infer", "partmm")


class _Prof(C.Structure):
    _fields_ = [("ms", C.c_double * 10), ("launches", C.c_uint64 * 10)]


class _Params(C.Structure):
    _fields_ = [("tau", C.c_uint32), ("K", C.c_uint32), ("seed", (C.c_uint64 * 4) * 5),
                ("flags", C.c_uint32), ("hip_stream", C.c_void_p)]


_lib = None


def declared_symbols():
    """Entry points declared in include/gtree.h."""
    text = open(HEADER_PATH).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gt_[a-z0-9_]+)\s*\(", text)))


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library %s is not built: run __graft_entry__.build() "
                           "(hipcc --offload-arch=gfx950); there is no CPU fallback" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, u32, sz, i = C.c_void_p, C.c_uint32, C.c_size_t, C.c_int
    S = C.POINTER(_Shares)
    sig = {
        "gt_ctx_create": (i, [C.POINTER(vp), C.POINTER(_Params)]),
        "gt_ctx_destroy": (i, [vp]),
        "gt_stats_get": (i, [vp, C.POINTER(_Stats)]),
        "gt_stats_reset": (i, [vp]),
        "gt_prof_get": (i, [vp, C.POINTER(_Prof)]),
        "gt_train_reset": (i, [vp, vp, S, S]),
        "gt_op_counter": (u32, [vp]),
        "gt_strerror": (C.c_char_p, [i]),
        "gt_share_a": (i, [vp, vp, sz, S]),
        "gt_reconstruct_a": (i, [vp, S, vp, sz]),
        "gt_mult": (i, [vp, S, S, sz, S]),
        "gt_eq_a": (i, [vp, S, vp, sz, S]),
        "gt_ge_a": (i, [vp, S, S, sz, S]),
        "gt_oaa": (i, [vp, S, sz, S, sz, S]),
        "gt_oaa_static": (i, [vp, S, sz, S, sz, S]),
        "gt_div": (i, [vp, S, S, sz, S]),
        "gt_train_create": (i, [vp, S, S, sz, u32, u32, C.POINTER(vp)]),
        "gt_train_level": (i, [vp, vp, u32]),
        "gt_train_set_heuristic": (i, [vp, i]),
        "gt_train_set_literal": (i, [vp, vp, i]),
        "gt_train_set_partition": (i, [vp, vp, i]),
        "gt_oaa_literal": (i, [vp, S, sz, S, sz, S]),
        "gt_train_finish": (i, [vp, vp, C.POINTER(vp)]),
        "gt_train_destroy": (i, [vp]),
        "gt_train_export_size": (sz, [vp, i]),
        "gt_train_export": (i, [vp, vp, i, S]),
        "gt_train_import": (i, [vp, vp, u32, S, S, S, S, S]),
        "gt_tree_import": (i, [vp, S, S, S, u32, C.POINTER(vp)]),
        "gt_tree_export": (i, [vp, vp, S, S]),
        "gt_tree_destroy": (i, [vp]),
        "gt_infer_batch": (i, [vp, vp, S, sz, u32, S]),
        "gt_forest_create": (i, [vp, C.POINTER(vp), sz, C.POINTER(vp)]),
        "gt_forest_destroy": (i, [vp]),
        "gt_infer_forest": (i, [vp, vp, S, sz, u32, S]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def _strerror(code):
    try:
        return load().gt_strerror(code).decode()
    except Exception:
        return "?"


def _chk(rc, what):
    if rc != GT_OK:
        raise GtError(rc, what)


class Shares:
    """Six device planes of one shared vector: t[p, 0] = party p's own component,
    t[p, 1] = its next component (torch int64 used as raw 64-bit words)."""

    def __init__(self, n, device="cuda:0", t=None):
        import torch
        self.n = int(n)
        self.t = t if t is not None else torch.zeros((3, 2, max(self.n, 1)), dtype=torch.int64, device=device)

    def c_struct(self):
        s = _Shares()
        stride = self.t.stride(1) * 8
        base = self.t.data_ptr()
        for p in range(3):
            s.party[p].own = base + (2 * p) * stride
            s.party[p].next = base + (2 * p + 1) * stride
        s.n = self.n
        return s

    def planes(self):
        """numpy uint64 array (3, 2, n)."""
        return self.t[:, :, :self.n].cpu().numpy().view(np.uint64)

    def components(self):
        """(3, n) components, after checking that the replicated copies agree."""
        pl = self.planes()
        for p in range(3):
            if not np.array_equal(pl[p, 1], pl[(p + 1) % 3, 0]):
                raise AssertionError("replicated copies of component %d differ" % ((p + 1) % 3))
        return np.ascontiguousarray(pl[:, 0, :])


def _ref(s):
    return None if s is None else C.byref(s.c_struct())


class GTree:
    """One protocol context (keys, operation counter, message buffers, stream)."""

    def __init__(self, seed, tau=16, K=2, device="cuda:0", stream=None, profile=False, flags=0):
        import torch
        self.L = load()
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        prm = _Params()
        prm.tau, prm.K, prm.flags = int(tau), int(K), (GT_FLAG_PROFILE if profile else 0) | int(flags)
        sd = np.asarray(seed, dtype=np.uint64).reshape(5, 4)
        for a in range(5):
            for b in range(4):
                prm.seed[a][b] = int(sd[a, b])
        self.stream = stream
        prm.hip_stream = None if stream is None else stream.cuda_stream
        self.tau, self.K = int(tau), int(K)
        h = C.c_void_p()
        _chk(self.L.gt_ctx_create(C.byref(h), C.byref(prm)), "gt_ctx_create")
        self.ctx = h
        self._train = None
        self._tshape = None

    def close(self):
        if getattr(self, "_train", None):
            self.L.gt_train_destroy(self._train)
            self._train = None
        if getattr(self, "ctx", None):
            self.L.gt_ctx_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers -----------------------------------------------------------
    def dev(self, arr):
        """numpy uint64 -> device int64 tensor holding the same words."""
        a = np.ascontiguousarray(np.asarray(arr, dtype=np.uint64).reshape(-1))
        return self.torch.from_numpy(a.view(np.int64)).to(self.device)

    def new(self, n):
        return Shares(n, self.device)

    def stats(self):
        st = _Stats()
        _chk(self.L.gt_stats_get(self.ctx, C.byref(st)), "gt_stats_get")
        wire = np.array([[st.wire_bytes[a][b] for b in range(3)] for a in range(3)], dtype=np.uint64)
        return int(st.rounds), wire, float(st.kernel_ms)

    def wire_bits_dev(self):
        """(3, 3) payload bits per directed pair, counted by the kernels at their message stores."""
        st = _Stats()
        _chk(self.L.gt_stats_get(self.ctx, C.byref(st)), "gt_stats_get")
        return np.array([[st.wire_bits_dev[a][b] for b in range(3)] for a in range(3)], dtype=np.uint64)

    def prof(self):
        """{class name: (milliseconds, launches)} since the last stats_reset (profile=True)."""
        pr = _Prof()
        _chk(self.L.gt_prof_get(self.ctx, C.byref(pr)), "gt_prof_get")
        return {KC_NAMES[k]: (float(pr.ms[k]), int(pr.launches[k])) for k in range(len(KC_NAMES))}

    def stats_reset(self):
        _chk(self.L.gt_stats_reset(self.ctx), "gt_stats_reset")

    def op_counter(self):
        return int(self.L.gt_op_counter(self.ctx))

    # -- sharing -----------------------------------------------------------
    def share_a(self, plain):
        """plain: device int64 tensor or numpy uint64 array."""
        t = plain if self.torch.is_tensor(plain) else self.dev(plain)
        t = t.contiguous().view(-1)
        out = self.new(t.numel())
        _chk(self.L.gt_share_a(self.ctx, t.data_ptr(), t.numel(), _ref(out)), "gt_share_a")
        return out

    def reconstruct_a(self, s):
        out = self.torch.zeros(max(s.n, 1), dtype=self.torch.int64, device=self.device)
        _chk(self.L.gt_reconstruct_a(self.ctx, _ref(s), out.data_ptr(), s.n), "gt_reconstruct_a")
        return out[:s.n]

    def rec(self, s):
        return self.reconstruct_a(s).cpu().numpy().view(np.uint64)

    # -- building blocks ---------------------------------------------------
    def mult(self, x, y):
        z = self.new(x.n)
        _chk(self.L.gt_mult(self.ctx, _ref(x), _ref(y), x.n, _ref(z)), "gt_mult")
        return z

    def eq_a(self, x, y_pub=None):
        z = self.new(x.n)
        y = None if y_pub is None else (y_pub if self.torch.is_tensor(y_pub) else self.dev(y_pub))
        _chk(self.L.gt_eq_a(self.ctx, _ref(x), None if y is None else y.data_ptr(), x.n, _ref(z)), "gt_eq_a")
        return z

    def ge_a(self, x, y):
        z = self.new(x.n)
        _chk(self.L.gt_ge_a(self.ctx, _ref(x), _ref(y), x.n, _ref(z)), "gt_ge_a")
        return z

    def oaa(self, W, u):
        z = self.new(u.n)
        _chk(self.L.gt_oaa(self.ctx, _ref(W), W.n, _ref(u), u.n, _ref(z)), "gt_oaa")
        return z

    def oaa_static(self, W, u, z=None):
        """gt_oaa without any allocation inside the library (the caller may pass z)."""
        z = self.new(u.n) if z is None else z
        _chk(self.L.gt_oaa_static(self.ctx, _ref(W), W.n, _ref(u), u.n, _ref(z)), "gt_oaa_static")
        return z

    def div(self, S, Q):
        q = self.new(S.n)
        _chk(self.L.gt_div(self.ctx, _ref(S), _ref(Q), S.n, _ref(q)), "gt_div")
        return q

    # -- training ----------------------------------------------------------
    def train_create(self, X, Y, N, d, H):
        if self._train:
            self.L.gt_train_destroy(self._train)
            self._train = None
        h = C.c_void_p()
        _chk(self.L.gt_train_create(self.ctx, _ref(X), _ref(Y), N, d, H, C.byref(h)), "gt_train_create")
        self._train, self._tshape = h, (N, d, H)

    def train_reset(self, X, Y):
        _chk(self.L.gt_train_reset(self.ctx, self._train, _ref(X), _ref(Y)), "gt_train_reset")

    def train_set_partition(self, by_products):
        _chk(self.L.gt_train_set_partition(self.ctx, self._train, int(bool(by_products))), "gt_train_set_partition")

    def train_set_literal(self, literal):
        _chk(self.L.gt_train_set_literal(self.ctx, self._train, int(bool(literal))), "gt_train_set_literal")

    def oaa_literal(self, W, u):
        z = self.new(u.n)
        _chk(self.L.gt_oaa_literal(self.ctx, _ref(W), W.n, _ref(u), u.n, _ref(z)), "gt_oaa_literal")
        return z

    def train_set_heuristic(self, by_reconstruction):
        _chk(self.L.gt_train_set_heuristic(self._train, int(bool(by_reconstruction))), "gt_train_set_heuristic")

    def scorer_bytes(self):
        st = _Stats()
        _chk(self.L.gt_stats_get(self.ctx, C.byref(st)), "gt_stats_get")
        return int(st.scorer_bytes[0]), int(st.scorer_bytes[1])

    def train_level(self, h):
        _chk(self.L.gt_train_level(self.ctx, self._train, h), "gt_train_level")

    def train_finish(self):
        h = C.c_void_p()
        _chk(self.L.gt_train_finish(self.ctx, self._train, C.byref(h)), "gt_train_finish")
        return Tree(self, h, self._tshape[2])

    def train_export(self, what):
        n = self.L.gt_train_export_size(self._train, what)
        out = self.new(n)
        _chk(self.L.gt_train_export(self.ctx, self._train, what, _ref(out)), "gt_train_export")
        return out

    def train_import(self, h, M, Tprev, Flevel, Cc, gamma):
        _chk(self.L.gt_train_import(self.ctx, self._train, h, _ref(M), _ref(Tprev), _ref(Flevel),
                                    _ref(Cc), _ref(gamma)), "gt_train_import")

    # -- inference ---------------------------------------------------------
    def tree_import(self, feat, thr, leaf, H):
        h = C.c_void_p()
        _chk(self.L.gt_tree_import(self.ctx, _ref(feat), _ref(thr), _ref(leaf), H, C.byref(h)), "gt_tree_import")
        return Tree(self, h, H)

    def infer_batch(self, tree, I, NI, d):
        R = self.new(NI)
        _chk(self.L.gt_infer_batch(self.ctx, tree.h, _ref(I), NI, d, _ref(R)), "gt_infer_batch")
        return R


    def forest_create(self, trees):
        arr = (C.c_void_p * len(trees))(*[t.h for t in trees])
        h = C.c_void_p()
        _chk(self.L.gt_forest_create(self.ctx, arr, len(trees), C.byref(h)), "gt_forest_create")
        return Forest(self, h, len(trees))

    def infer_forest(self, forest, I, NI, d):
        """Shares of the labels, tree after tree: R[t*NI + i]."""
        R = self.new(NI * forest.ntrees)
        _chk(self.L.gt_infer_forest(self.ctx, forest.h, _ref(I), NI, d, _ref(R)), "gt_infer_forest")
        return R


class Forest:
    def __init__(self, g, h, ntrees):
        self.g, self.h, self.ntrees = g, h, ntrees

    def close(self):
        if self.h:
            self.g.L.gt_forest_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Tree:
    def __init__(self, g, h, H):
        self.g, self.h, self.H = g, h, H

    def export(self):
        feat, leaf = self.g.new((1 << self.H) - 1), self.g.new(1 << self.H)
        _chk(self.g.L.gt_tree_export(self.g.ctx, self.h, _ref(feat), _ref(leaf)), "gt_tree_export")
        return feat, leaf

    def close(self):
        if self.h:
            self.g.L.gt_tree_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
