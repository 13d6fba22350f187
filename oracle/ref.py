"""ctypes/numpy front end of the CPU oracle (oracle/combo_ref.cpp).

Test infrastructure only: used by tests/, the smoke check and the CPU-baseline leg of
the benchmark.  It marshals numpy arrays to the C functions and does no arithmetic of
the method itself.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def lib(path=None):
    """The oracle's shared object, loaded once.  `path` (first call only) names another
    build of it: the mutation tests pass a deliberately wrong copy to show that the pins
    catch it.  Nothing but an explicit argument can replace the oracle."""
    global _LIB
    if _LIB is not None and path is not None:
        raise RuntimeError("the oracle is already loaded; a different build must be named on the first call")
    if _LIB is None:
        if path is None:
            path = _build.LIB
            if not os.path.exists(path):
                _build.build()
        L = ctypes.CDLL(path)
        L.combo_ref_segment_bounds.argtypes = [ctypes.c_int64, ctypes.c_int32, _i64p, _i64p]
        L.combo_ref_segment_bounds.restype = ctypes.c_int
        L.combo_ref_mix64.argtypes = [ctypes.c_uint64]
        L.combo_ref_mix64.restype = ctypes.c_uint64
        L.combo_ref_hash.argtypes = [ctypes.c_uint64] * 5
        L.combo_ref_hash.restype = ctypes.c_uint64
        L.combo_ref_reduce.argtypes = [ctypes.c_uint64, ctypes.c_uint32]
        L.combo_ref_reduce.restype = ctypes.c_uint32
        L.combo_ref_make_peer_table.argtypes = [_i32p, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint64]
        L.combo_ref_make_peer_table.restype = ctypes.c_int
        L.combo_ref_make_peer_table_pooled.argtypes = L.combo_ref_make_peer_table.argtypes
        L.combo_ref_make_peer_table_pooled.restype = ctypes.c_int
        L.combo_ref_peer_in_degree.argtypes = [_i32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.c_int32]
        L.combo_ref_peer_in_degree.restype = ctypes.c_int
        _u8p = ctypes.POINTER(ctypes.c_uint8)
        L.combo_ref_make_peer_table_dynamic.argtypes = [_i32p, _u8p, ctypes.c_int32, ctypes.c_int32,
                                                        ctypes.c_int32, ctypes.c_uint64,
                                                        ctypes.c_uint64]
        L.combo_ref_make_peer_table_dynamic.restype = ctypes.c_int
        L.combo_ref_gossip_round_dynamic.argtypes = [_f32p, _f32p, ctypes.c_int64, _i32p, _f32p, _u8p,
                                                     ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                                     ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
        L.combo_ref_gossip_round_dynamic.restype = ctypes.c_int
        L.combo_ref_aggregation_divergence.argtypes = [_f64p, _f32p, ctypes.c_int64, _f32p,
                                                       ctypes.c_int32, ctypes.c_int64]
        L.combo_ref_aggregation_divergence.restype = ctypes.c_int
        common = [ctypes.c_int64, _i32p, _f32p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                  ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
        L.combo_ref_gossip_round.argtypes = [_f32p, _f32p] + common
        L.combo_ref_gossip_round.restype = ctypes.c_int
        L.combo_ref_gossip_round_f64.argtypes = [_f64p, _f32p] + common
        L.combo_ref_gossip_round_f64.restype = ctypes.c_int
        L.combo_ref_local_sgd_then_gossip.argtypes = [_f32p, _f32p, _f32p, ctypes.c_float] + common
        L.combo_ref_local_sgd_then_gossip.restype = ctypes.c_int
        L.combo_ref_local_sgd_steps_then_gossip.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int32,
                                                            ctypes.c_float] + common
        L.combo_ref_local_sgd_steps_then_gossip.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(t)


def _check2d(a, dtype, name):
    if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.ndim == 2
            and a.strides[1] == a.itemsize and a.strides[0] % a.itemsize == 0):
        raise ValueError(f"{name}: need a row-major 2-D {dtype} array (row pitch allowed)")
    return a.strides[0] // a.itemsize


def _out_like(X, ld):
    """float32 output with X's shape and row pitch."""
    N, ncols = X.shape
    return np.empty((N, ld), np.float32)[:, :ncols]


def segment_bounds(P, S):
    lo = np.empty(S, np.int64)
    hi = np.empty(S, np.int64)
    rc = lib().combo_ref_segment_bounds(P, S, _p(lo, _i64p), _p(hi, _i64p))
    if rc:
        raise ValueError("combo_ref_segment_bounds rejected the arguments")
    return lo, hi


def mix64(z):
    return int(lib().combo_ref_mix64(z & 0xFFFFFFFFFFFFFFFF))


def peer_hash(seed, rnd, w, s, j):
    return int(lib().combo_ref_hash(seed, rnd, w, s, j))


def reduce(h, m):
    return int(lib().combo_ref_reduce(h, m))


def make_peer_table(N, S, R, seed, rnd):
    peers = np.empty((N, S, R), np.int32)
    rc = lib().combo_ref_make_peer_table(_p(peers, _i32p), N, S, R, seed, rnd)
    if rc:
        raise ValueError("combo_ref_make_peer_table rejected the arguments")
    return peers


def make_peer_table_pooled(N, S, R, seed, rnd):
    peers = np.empty((N, S, R), np.int32)
    rc = lib().combo_ref_make_peer_table_pooled(_p(peers, _i32p), N, S, R, seed, rnd)
    if rc:
        raise ValueError("combo_ref_make_peer_table_pooled rejected the arguments")
    return peers


def peer_in_degree(peers, N, S, R):
    peers = _peers_arg(peers, N, S, R)
    deg = np.empty(N, np.int32)
    rc = lib().combo_ref_peer_in_degree(_p(deg, _i32p), _p(peers, _i32p), N, S, R)
    if rc:
        raise ValueError("combo_ref_peer_in_degree rejected the arguments")
    return deg


def aggregation_divergence(X, d=None):
    """Squared L2 distance of every worker's row from the (weighted) mean of all rows."""
    N, P = X.shape
    ld = _check2d(X, np.float32, "X")
    dist2 = np.empty(N, np.float64)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_aggregation_divergence(_p(dist2, _f64p), _p(X, _f32p), ld, dp, N, P)
    if rc:
        raise ValueError("combo_ref_aggregation_divergence rejected the arguments")
    return dist2


def _status_arg(status, N):
    status = np.ascontiguousarray(status, dtype=np.uint8)
    if status.shape != (N,):
        raise ValueError("status must have shape (N,)")
    return status


def make_peer_table_dynamic(status, N, S, R, seed, rnd):
    status = _status_arg(status, N)
    peers = np.empty((N, S, R), np.int32)
    rc = lib().combo_ref_make_peer_table_dynamic(_p(peers, _i32p),
                                                 _p(status, ctypes.POINTER(ctypes.c_uint8)),
                                                 N, S, R, seed, rnd)
    if rc:
        raise ValueError("combo_ref_make_peer_table_dynamic rejected the arguments")
    return peers


def gossip_round_dynamic(X, peers, status, P, S, R, d=None, col0=0):
    N, ncols = X.shape
    ld = _check2d(X, np.float32, "X")
    Y = _out_like(X, ld)
    if _check2d(Y, np.float32, "Y") != ld:
        raise ValueError("internal: pitch mismatch")
    peers = _peers_arg(peers, N, S, R)
    status = _status_arg(status, N)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_gossip_round_dynamic(_p(Y, _f32p), _p(X, _f32p), ld, _p(peers, _i32p), dp,
                                              _p(status, ctypes.POINTER(ctypes.c_uint8)),
                                              N, P, S, R, col0, ncols)
    if rc:
        raise ValueError("combo_ref_gossip_round_dynamic rejected the arguments")
    return Y


def _peers_arg(peers, N, S, R):
    peers = np.ascontiguousarray(peers, dtype=np.int32)
    if peers.size != N * S * R:
        raise ValueError("peer table has the wrong size")
    return peers


def _d_arg(d, N):
    if d is None:
        return None, None
    d = np.ascontiguousarray(d, dtype=np.float32)
    if d.shape != (N,):
        raise ValueError("dataset sizes must have shape (N,)")
    return d, _p(d, _f32p)


def gossip_round(X, peers, P, S, R, d=None, col0=0, out=None):
    """fp32 round on a column window.  X: (N, ncols) float32 view (row pitch allowed)."""
    N, ncols = X.shape
    ld = _check2d(X, np.float32, "X")
    Y = _out_like(X, ld) if out is None else out
    ldy = _check2d(Y, np.float32, "Y")
    if ldy != ld or Y.shape != X.shape:
        raise ValueError("Y must have X's shape and pitch")
    peers = _peers_arg(peers, N, S, R)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_gossip_round(_p(Y, _f32p), _p(X, _f32p), ld, _p(peers, _i32p), dp,
                                      N, P, S, R, col0, ncols)
    if rc:
        raise ValueError("combo_ref_gossip_round rejected the arguments")
    return Y


def gossip_round_f64(X, peers, P, S, R, d=None, col0=0):
    N, ncols = X.shape
    ld = _check2d(X, np.float32, "X")
    Yfull = np.empty((N, ld), np.float64)
    peers = _peers_arg(peers, N, S, R)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_gossip_round_f64(_p(Yfull, _f64p), _p(X, _f32p), ld, _p(peers, _i32p),
                                          dp, N, P, S, R, col0, ncols)
    if rc:
        raise ValueError("combo_ref_gossip_round_f64 rejected the arguments")
    return Yfull[:, :ncols]


def local_sgd_then_gossip(X, G, lr, peers, P, S, R, d=None, col0=0):
    """Steps X in place (X <- X - lr*G), then returns the round on the stepped X."""
    N, ncols = X.shape
    ld = _check2d(X, np.float32, "X")
    ldg = _check2d(G, np.float32, "G")
    if ldg != ld or G.shape != X.shape:
        raise ValueError("G must have X's shape and pitch")
    Y = _out_like(X, ld)
    if _check2d(Y, np.float32, "Y") != ld:
        raise ValueError("internal: pitch mismatch")
    peers = _peers_arg(peers, N, S, R)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_local_sgd_then_gossip(_p(Y, _f32p), _p(X, _f32p), _p(G, _f32p),
                                               ctypes.c_float(lr), ld, _p(peers, _i32p), dp,
                                               N, P, S, R, col0, ncols)
    if rc:
        raise ValueError("combo_ref_local_sgd_then_gossip rejected the arguments")
    return Y


def local_sgd_steps_then_gossip(X, G, lr, peers, P, S, R, d=None, col0=0):
    """G: (tau, N, ncols) float32, C-contiguous with X's pitch.  Steps X in place tau
    times, then returns the round on the stepped X."""
    N, ncols = X.shape
    ld = _check2d(X, np.float32, "X")
    if G.shape[0] > 0 and not (G.dtype == np.float32 and G.ndim == 3 and G.shape[1:] == X.shape
                               and G.strides == (N * ld * 4, ld * 4, 4)):
        raise ValueError("G must be (tau, N, ncols) float32 with X's pitch and slice stride N*ld")
    Y = _out_like(X, ld)
    peers = _peers_arg(peers, N, S, R)
    dk, dp = _d_arg(d, N)
    rc = lib().combo_ref_local_sgd_steps_then_gossip(_p(Y, _f32p), _p(X, _f32p), _p(G, _f32p),
                                                     G.shape[0], ctypes.c_float(lr), ld,
                                                     _p(peers, _i32p), dp, N, P, S, R, col0, ncols)
    if rc:
        raise ValueError("combo_ref_local_sgd_steps_then_gossip rejected the arguments")
    return Y
