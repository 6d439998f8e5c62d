"""ctypes binding of the CPU oracle (test infrastructure, see gtree_oracle.h)."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgtree_oracle.so")

X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_L, X_SCORE, X_C_PAPER = range(9)


def build_oracle(force=False):
    """Compile gtree_oracle.c with gcc (OpenMP over independent elements)."""
    src = os.path.join(_HERE, "gtree_oracle.c")
    hdr = os.path.join(_HERE, "gtree_oracle.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
           "-o", _LIB_PATH, src]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None
_u64p = C.POINTER(C.c_uint64)
_u32p = C.POINTER(C.c_uint32)


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_u64p)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build_oracle()
    L = C.CDLL(_LIB_PATH)
    vp, u32, u64, sz, i = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t, C.c_int
    sig = {
        "orc_ctx_create": (vp, [_u64p, u32, u32]),
        "orc_ctx_destroy": (None, [vp]),
        "orc_stats": (None, [vp, _u64p, _u64p]),
        "orc_stats_bits": (None, [vp, _u64p]),
        "orc_stats_scorer": (None, [vp, _u64p]),
        "orc_train_set_heuristic": (None, [vp, i]),
        "orc_train_set_literal": (None, [vp, i]),
        "orc_train_set_partition": (None, [vp, i]),
        "orc_oaa_literal": (None, [vp, _u64p, sz, _u64p, sz, _u64p]),
        "orc_stats_reset": (None, [vp]),
        "orc_op_counter": (u32, [vp]),
        "orc_set_threads": (None, [i]),
        "orc_get_threads": (i, []),
        "orc_chacha_block": (None, [_u32p, u32, u32, u32, u32, i, _u32p]),
        "orc_chacha_quarter": (None, [_u32p]),
        "orc_prf_word": (u64, [vp, i, u32, u32, u64]),
        "orc_zero_sharing": (None, [vp, u32, u32, u64, i, _u64p]),
        "orc_dealer": (None, [vp, u32, u64, _u64p]),
        "orc_dabit_grid": (None, [vp, u32, u64, _u64p]),
        "orc_share_a": (None, [vp, _u64p, sz, _u64p]),
        "orc_reconstruct_a": (None, [_u64p, sz, _u64p]),
        "orc_reconstruct_b": (None, [_u64p, sz, _u64p]),
        "orc_mult": (None, [vp, _u64p, _u64p, sz, _u64p]),
        "orc_eq_b": (None, [vp, _u64p, _u64p, sz, _u64p]),
        "orc_eq_a": (None, [vp, _u64p, _u64p, sz, _u64p]),
        "orc_ge_a": (None, [vp, _u64p, _u64p, sz, _u64p]),
        "orc_oaa": (None, [vp, _u64p, sz, _u64p, sz, _u64p]),
        "orc_div": (None, [vp, _u64p, _u64p, sz, _u64p]),
        "orc_train_create": (vp, [vp, _u64p, _u64p, sz, u32, u32]),
        "orc_train_destroy": (None, [vp]),
        "orc_train_level": (i, [vp, vp, u32]),
        "orc_train_finish": (i, [vp, vp, _u64p, _u64p]),
        "orc_train_export_size": (sz, [vp, i]),
        "orc_train_export": (i, [vp, i, _u64p]),
        "orc_train_import": (i, [vp, u32, _u64p, _u64p, _u64p, _u64p, _u64p]),
        "orc_infer_batch": (i, [vp, _u64p, _u64p, _u64p, u32, _u64p, sz, u32, _u64p]),
        "orc_infer_rows": (i, [vp, _u64p, _u64p, _u64p, u32, _u64p, sz, u32, C.POINTER(C.c_size_t), sz, _u64p]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def chacha_block(key8, c12, c13, c14, c15, rounds):
    L = _load()
    key = np.asarray(key8, dtype=np.uint32)
    out = np.zeros(16, dtype=np.uint32)
    L.orc_chacha_block(key.ctypes.data_as(_u32p), c12, c13, c14, c15, rounds,
                       out.ctypes.data_as(_u32p))
    return out


def chacha_quarter(v4):
    L = _load()
    v = np.array(v4, dtype=np.uint32)
    L.orc_chacha_quarter(v.ctypes.data_as(_u32p))
    return v


def set_threads(n):
    _load().orc_set_threads(int(n))


def get_threads():
    return int(_load().orc_get_threads())


class Oracle:
    """One protocol context: keys, tau, K, operation counter, message counters."""

    def __init__(self, seed, tau=16, K=2):
        L = _load()
        self.L = L
        self.seed = np.ascontiguousarray(np.asarray(seed, dtype=np.uint64).reshape(5, 4))
        self.tau, self.K = int(tau), int(K)
        self.ctx = L.orc_ctx_create(_p(self.seed.reshape(-1)), self.tau, self.K)
        self._train = None

    def close(self):
        if self._train:
            self.L.orc_train_destroy(self._train)
            self._train = None
        if self.ctx:
            self.L.orc_ctx_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- bookkeeping -------------------------------------------------------
    def stats(self):
        r = C.c_uint64(0)
        w = np.zeros(9, dtype=np.uint64)
        self.L.orc_stats(self.ctx, C.byref(r), _p(w))
        return int(r.value), w.reshape(3, 3).copy()

    def wire_bits(self):
        """(3, 3) payload bits per directed pair."""
        w = np.zeros(9, dtype=np.uint64)
        self.L.orc_stats_bits(self.ctx, _p(w))
        return w.reshape(3, 3).copy()

    def scorer_bytes(self):
        w = np.zeros(2, dtype=np.uint64)
        self.L.orc_stats_scorer(self.ctx, _p(w))
        return int(w[0]), int(w[1])

    def stats_reset(self):
        self.L.orc_stats_reset(self.ctx)

    def op_counter(self):
        return int(self.L.orc_op_counter(self.ctx))

    # -- randomness --------------------------------------------------------
    def prf_word(self, key_index, op, stream, j):
        return int(self.L.orc_prf_word(self.ctx, key_index, op, stream, j))

    def zero_sharing(self, op, stream, e, boolean=False):
        a = np.zeros(3, dtype=np.uint64)
        self.L.orc_zero_sharing(self.ctx, op, stream, e, int(boolean), _p(a))
        return a

    def dealer(self, op, e):
        a = np.zeros(14, dtype=np.uint64)
        self.L.orc_dealer(self.ctx, op, e, _p(a))
        return dict(rA=a[0:3].copy(), rho=a[3:6].copy(), bB=a[6:9].copy(), bA=a[9:12].copy(),
                    r=int(a[12]), beta=int(a[13]))

    def dabit_grid(self, op, e):
        a = np.zeros(7, dtype=np.uint64)
        self.L.orc_dabit_grid(self.ctx, op, e, _p(a))
        return dict(bB=a[0:3].copy(), bA=a[3:6].copy(), beta=int(a[6]))

    # -- sharing -----------------------------------------------------------
    def share(self, plain):
        x = np.ascontiguousarray(np.asarray(plain, dtype=np.uint64).reshape(-1))
        out = np.zeros((3, x.size), dtype=np.uint64)
        self.L.orc_share_a(self.ctx, _p(x), x.size, _p(out.reshape(-1)))
        return out

    @staticmethod
    def rec(comp):
        comp = np.ascontiguousarray(comp, dtype=np.uint64)
        n = comp.shape[1]
        out = np.zeros(n, dtype=np.uint64)
        _load().orc_reconstruct_a(_p(comp.reshape(-1)), n, _p(out))
        return out

    @staticmethod
    def rec_b(comp):
        comp = np.ascontiguousarray(comp, dtype=np.uint64)
        n = comp.shape[1]
        out = np.zeros(n, dtype=np.uint64)
        _load().orc_reconstruct_b(_p(comp.reshape(-1)), n, _p(out))
        return out

    # -- building blocks ---------------------------------------------------
    def _c(self, a):
        a = np.ascontiguousarray(a, dtype=np.uint64)
        assert a.ndim == 2 and a.shape[0] == 3
        return a

    def mult(self, x, y):
        x, y = self._c(x), self._c(y)
        z = np.zeros_like(x)
        self.L.orc_mult(self.ctx, _p(x.reshape(-1)), _p(y.reshape(-1)), x.shape[1], _p(z.reshape(-1)))
        return z

    def eq_b(self, x, y_pub=None):
        x = self._c(x)
        y = None if y_pub is None else np.ascontiguousarray(y_pub, dtype=np.uint64)
        z = np.zeros_like(x)
        self.L.orc_eq_b(self.ctx, _p(x.reshape(-1)), _p(y), x.shape[1], _p(z.reshape(-1)))
        return z

    def eq_a(self, x, y_pub=None):
        x = self._c(x)
        y = None if y_pub is None else np.ascontiguousarray(y_pub, dtype=np.uint64)
        z = np.zeros_like(x)
        self.L.orc_eq_a(self.ctx, _p(x.reshape(-1)), _p(y), x.shape[1], _p(z.reshape(-1)))
        return z

    def ge_a(self, x, y):
        x, y = self._c(x), self._c(y)
        z = np.zeros_like(x)
        self.L.orc_ge_a(self.ctx, _p(x.reshape(-1)), _p(y.reshape(-1)), x.shape[1], _p(z.reshape(-1)))
        return z

    def oaa(self, W, u):
        W, u = self._c(W), self._c(u)
        z = np.zeros_like(u)
        self.L.orc_oaa(self.ctx, _p(W.reshape(-1)), W.shape[1], _p(u.reshape(-1)), u.shape[1],
                       _p(z.reshape(-1)))
        return z

    def oaa_literal(self, W, u):
        W, u = self._c(W), self._c(u)
        z = np.zeros_like(u)
        self.L.orc_oaa_literal(self.ctx, _p(W.reshape(-1)), W.shape[1], _p(u.reshape(-1)), u.shape[1],
                               _p(z.reshape(-1)))
        return z

    def div(self, S, Q):
        S, Q = self._c(S), self._c(Q)
        z = np.zeros_like(S)
        self.L.orc_div(self.ctx, _p(S.reshape(-1)), _p(Q.reshape(-1)), S.shape[1], _p(z.reshape(-1)))
        return z

    # -- training ----------------------------------------------------------
    def train_create(self, X, Y, N, d, H):
        """X: (3, N*d) components of the row-major N x d matrix; Y: (3, N*K)."""
        X, Y = self._c(X), self._c(Y)
        assert X.shape[1] == N * d and Y.shape[1] == N * self.K
        if self._train:
            self.L.orc_train_destroy(self._train)
        self._train = self.L.orc_train_create(self.ctx, _p(X.reshape(-1)), _p(Y.reshape(-1)), N, d, H)
        self._tshape = (N, d, H)

    def train_set_partition(self, by_products):
        self.L.orc_train_set_partition(self._train, int(bool(by_products)))

    def train_set_literal(self, literal):
        self.L.orc_train_set_literal(self._train, int(bool(literal)))

    def train_set_heuristic(self, by_reconstruction):
        self.L.orc_train_set_heuristic(self._train, int(bool(by_reconstruction)))

    def train_level(self, h):
        rc = self.L.orc_train_level(self.ctx, self._train, h)
        if rc:
            raise RuntimeError("orc_train_level(%d) -> %d" % (h, rc))

    def train_finish(self):
        N, d, H = self._tshape
        feat = np.zeros((3, (1 << H) - 1), dtype=np.uint64)
        leaf = np.zeros((3, 1 << H), dtype=np.uint64)
        rc = self.L.orc_train_finish(self.ctx, self._train, _p(feat.reshape(-1)), _p(leaf.reshape(-1)))
        if rc:
            raise RuntimeError("orc_train_finish -> %d" % rc)
        return feat, leaf

    def train_export(self, what):
        n = self.L.orc_train_export_size(self._train, what)
        out = np.zeros((3, n), dtype=np.uint64)
        rc = self.L.orc_train_export(self._train, what, _p(out.reshape(-1)))
        if rc:
            raise RuntimeError("orc_train_export(%d) -> %d" % (what, rc))
        return out

    def train_import(self, h, M, Tprev, Flevel, Cc, gamma):
        args = [self._c(a).reshape(-1) if a is not None else None for a in (M, Tprev, Flevel, Cc, gamma)]
        rc = self.L.orc_train_import(self._train, h, *[_p(a) for a in args])
        if rc:
            raise RuntimeError("orc_train_import -> %d" % rc)

    # -- inference ---------------------------------------------------------
    def infer(self, feat, thr, leaf, H, I, NI, d):
        feat, leaf, I = self._c(feat), self._c(leaf), self._c(I)
        thr = None if thr is None else self._c(thr)
        R = np.zeros((3, NI), dtype=np.uint64)
        rc = self.L.orc_infer_batch(self.ctx, _p(feat.reshape(-1)),
                                    None if thr is None else _p(thr.reshape(-1)),
                                    _p(leaf.reshape(-1)), H, _p(I.reshape(-1)), NI, d,
                                    _p(R.reshape(-1)))
        if rc:
            raise RuntimeError("orc_infer_batch -> %d" % rc)
        return R

    def infer_rows(self, feat, thr, leaf, H, I_rows, NI, d, rows):
        """I_rows: (3, len(rows)*d) components of the listed rows of a batch of NI instances."""
        feat, leaf, I_rows = self._c(feat), self._c(leaf), self._c(I_rows)
        thr = None if thr is None else self._c(thr)
        rows = np.ascontiguousarray(rows, dtype=np.uintp)
        R = np.zeros((3, rows.size), dtype=np.uint64)
        rc = self.L.orc_infer_rows(self.ctx, _p(feat.reshape(-1)), None if thr is None else _p(thr.reshape(-1)),
                                   _p(leaf.reshape(-1)), H, _p(I_rows.reshape(-1)), NI, d,
                                   rows.ctypes.data_as(C.POINTER(C.c_size_t)), rows.size, _p(R.reshape(-1)))
        if rc:
            raise RuntimeError("orc_infer_rows -> %d" % rc)
        return R
