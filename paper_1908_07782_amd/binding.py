"""ctypes binding of libcombo.so - argument marshalling only."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcombo.so")

TUNE_TILE_COLS = 0
TUNE_XCD_SWIZZLE = 1
TUNE_FUSED_MODE = 2
TUNE_KERNEL = 3
TUNE_SLAB_COLS = 4
TUNE_SLAB_ORDER = 5
TUNE_SLAB_THREADS = 6
TUNE_SLAB_LDS_FLOOR = 7

EXPORTS = ("combo_bandwidth_probe", "combo_round_relayout", "combo_aggregation_divergence_noalloc", "combo_round_hashed", "combo_round_kernel_kind", "combo_aggregation_divergence_tiled", "combo_tiled_cols", "combo_tiled_elems", "combo_pack_tiled", "combo_unpack_tiled",
           "combo_segment_gossip_round_tiled", "combo_local_sgd_steps_then_gossip_tiled",
           "combo_local_sgd_steps_then_gossip", "combo_aggregation_divergence", "combo_aggregation_divergence_workspace",
           "combo_make_peer_table_dynamic", "combo_segment_gossip_round_dynamic",
           "combo_make_peer_table", "combo_make_peer_table_pooled", "combo_peer_in_degree", "combo_segment_gossip_round", "combo_local_sgd_then_gossip",
           "combo_tune", "combo_get_tune", "combo_strerror")

_LIB = None


class ComboError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


def lib():
    """Load libcombo.so (built by paper_1908_07782_amd/build.py).  Fails loudly."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            # nothing built yet: compile the HIP library now; there is no other code path
            try:
                from . import build as _build
                _build.build()
            except Exception as e:  # noqa: BLE001
                raise ImportError(f"{LIB_PATH} is missing and could not be built ({e}); run "
                                  "`python -m paper_1908_07782_amd.build` - there is no fallback "
                                  "path") from e
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64,
                                  ctypes.c_float)
        L.combo_make_peer_table.argtypes = [vp, i32, i32, i32, u64, u64, vp]
        L.combo_make_peer_table.restype = ctypes.c_int
        L.combo_make_peer_table_pooled.argtypes = [vp, i32, i32, i32, u64, u64, vp]
        L.combo_make_peer_table_pooled.restype = ctypes.c_int
        L.combo_peer_in_degree.argtypes = [vp, vp, i32, i32, i32, vp]
        L.combo_peer_in_degree.restype = ctypes.c_int
        L.combo_make_peer_table_dynamic.argtypes = [vp, vp, i32, i32, i32, u64, u64, vp]
        L.combo_make_peer_table_dynamic.restype = ctypes.c_int
        L.combo_segment_gossip_round_dynamic.argtypes = [vp, vp, i64, vp, vp, vp, i32, i64, i32, i32, vp]
        L.combo_segment_gossip_round_dynamic.restype = ctypes.c_int
        L.combo_aggregation_divergence_workspace.argtypes = [i32, i64]
        L.combo_aggregation_divergence_workspace.restype = ctypes.c_int64
        L.combo_aggregation_divergence.argtypes = [vp, vp, i64, vp, i32, i64, vp, i64, vp]
        L.combo_aggregation_divergence.restype = ctypes.c_int
        L.combo_segment_gossip_round.argtypes = [vp, vp, i64, vp, vp, i32, i64, i32, i32, vp]
        L.combo_segment_gossip_round.restype = ctypes.c_int
        L.combo_local_sgd_then_gossip.argtypes = [vp, vp, vp, f32, i64, vp, vp, i32, i64, i32, i32, vp]
        L.combo_local_sgd_then_gossip.restype = ctypes.c_int
        L.combo_local_sgd_steps_then_gossip.argtypes = [vp, vp, vp, i32, f32, i64, vp, vp, i32, i64,
                                                        i32, i32, vp]
        L.combo_local_sgd_steps_then_gossip.restype = ctypes.c_int
        L.combo_tiled_cols.argtypes = [i32, i32]
        L.combo_tiled_cols.restype = ctypes.c_int32
        L.combo_tiled_elems.argtypes = [i32, i64, i32]
        L.combo_tiled_elems.restype = ctypes.c_int64
        L.combo_pack_tiled.argtypes = [vp, vp, i64, i32, i64, i32, vp]
        L.combo_pack_tiled.restype = ctypes.c_int
        L.combo_unpack_tiled.argtypes = [vp, i64, vp, i32, i64, i32, vp]
        L.combo_unpack_tiled.restype = ctypes.c_int
        L.combo_segment_gossip_round_tiled.argtypes = [vp, vp, i32, vp, vp, vp, i32, i64, i32, i32, vp]
        L.combo_segment_gossip_round_tiled.restype = ctypes.c_int
        L.combo_local_sgd_steps_then_gossip_tiled.argtypes = [vp, vp, vp, i32, f32, i32, vp, vp, i32,
                                                              i64, i32, i32, vp]
        L.combo_local_sgd_steps_then_gossip_tiled.restype = ctypes.c_int
        L.combo_aggregation_divergence_tiled.argtypes = [vp, vp, i32, vp, i32, i64, vp, i64, vp]
        L.combo_aggregation_divergence_tiled.restype = ctypes.c_int
        L.combo_aggregation_divergence_noalloc.argtypes = [vp, vp, i64, i32, vp, i32, i64, vp]
        L.combo_aggregation_divergence_noalloc.restype = ctypes.c_int
        L.combo_round_relayout.argtypes = [vp, i64, i32, vp, i64, i32, vp, i32, f32, vp, vp, vp, i32, i64,
                                           i32, i32, vp]
        L.combo_round_relayout.restype = ctypes.c_int
        L.combo_bandwidth_probe.argtypes = [ctypes.c_int, vp, vp, i32, i64, i64, i32, i32, vp]
        L.combo_bandwidth_probe.restype = ctypes.c_int
        L.combo_round_hashed.argtypes = [vp, vp, vp, i32, f32, i64, i32, vp, i32, i64, i32, i32, u64, u64, vp]
        L.combo_round_hashed.restype = ctypes.c_int
        L.combo_round_kernel_kind.argtypes = [i32, i32]
        L.combo_round_kernel_kind.restype = ctypes.c_int
        L.combo_tune.argtypes = [ctypes.c_int, ctypes.c_int]
        L.combo_tune.restype = ctypes.c_int
        L.combo_get_tune.argtypes = [ctypes.c_int]
        L.combo_get_tune.restype = ctypes.c_int
        L.combo_strerror.argtypes = [ctypes.c_int]
        L.combo_strerror.restype = ctypes.c_char_p
        _LIB = L
    return _LIB


def strerror(status):
    return lib().combo_strerror(int(status)).decode()


def tune(key, value):
    rc = lib().combo_tune(int(key), int(value))
    if rc:
        raise ComboError(rc, "combo_tune")


def round_kernel_kind(N, R):
    """1 if the row-major entry points use the LDS-slab kernel for this shape, 0 for the
    row-tile kernel."""
    return lib().combo_round_kernel_kind(int(N), int(R))


def get_tune(key):
    return lib().combo_get_tune(int(key))


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, dtype, name, optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if not (t.is_cuda and t.dtype == dtype):
        raise ValueError(f"{name}: need a {dtype} tensor in device memory")
    return ctypes.c_void_p(t.data_ptr())


def _matrix(t, name):
    if not (t.dim() == 2 and t.stride(1) == 1):
        raise ValueError(f"{name}: need a 2-D tensor whose rows are contiguous (row pitch allowed)")
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _check_round_inputs(peers, dataset_sizes, status, N, S, R, device):
    """Host-side size checks of the small device inputs of a round: a short or strided
    table, dataset-size or status array would be an out-of-bounds device read."""
    if R > 0 and (peers is None or not peers.is_cuda or peers.dtype != torch.int32
                  or not peers.is_contiguous() or peers.numel() < N * S * R):
        raise ValueError("peers: need a contiguous int32 device tensor with N*S*R entries")
    if dataset_sizes is not None and (not dataset_sizes.is_cuda or dataset_sizes.dtype != torch.float32
                                      or not dataset_sizes.is_contiguous() or dataset_sizes.numel() < N):
        raise ValueError("dataset_sizes: need a contiguous float32 device tensor with N entries")
    if status is not None and (not status.is_cuda or status.dtype != torch.uint8
                               or not status.is_contiguous() or status.numel() < N):
        raise ValueError("status: need a contiguous uint8 device tensor with N entries")
    for name, t in (("peers", peers if R > 0 else None), ("dataset_sizes", dataset_sizes), ("status", status)):
        if t is not None and t.device != device:
            raise ValueError(f"{name}: lives on {t.device}, the parameters on {device}")


def make_peer_table(peers, N, S, R, seed, rnd, stream=None):
    """combo_make_peer_table: fills the int32 device tensor `peers` (N*S*R entries)."""
    if R > 0 and (peers is None or peers.numel() < N * S * R or not peers.is_contiguous()):
        raise ValueError("peers: need a contiguous int32 device tensor with N*S*R entries")
    rc = lib().combo_make_peer_table(_dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
                                     N, S, R, ctypes.c_uint64(seed), ctypes.c_uint64(rnd),
                                     _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_make_peer_table")
    return peers


def make_peer_table_pooled(peers, N, S, R, seed, rnd, stream=None):
    """combo_make_peer_table_pooled: one pool per worker for all of its S*R requests."""
    if R > 0 and (peers is None or peers.numel() < N * S * R or not peers.is_contiguous()):
        raise ValueError("peers: need a contiguous int32 device tensor with N*S*R entries")
    rc = lib().combo_make_peer_table_pooled(_dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
                                            N, S, R, ctypes.c_uint64(seed), ctypes.c_uint64(rnd),
                                            _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_make_peer_table_pooled")
    return peers


def peer_in_degree(degree, peers, N, S, R, stream=None):
    """combo_peer_in_degree: degree (int32[N], device) <- serve load of the table."""
    if degree.numel() < N or not degree.is_contiguous():
        raise ValueError("degree: need a contiguous int32 device tensor with N entries")
    _check_round_inputs(peers, None, None, N, S, R, degree.device)
    rc = lib().combo_peer_in_degree(_dev_ptr(degree, torch.int32, "degree"),
                                    _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
                                    N, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_peer_in_degree")
    return degree


def make_peer_table_dynamic(peers, status, N, S, R, seed, rnd, stream=None):
    """combo_make_peer_table_dynamic: status is a uint8 device tensor of N entries."""
    if R > 0 and (peers is None or peers.numel() < N * S * R or not peers.is_contiguous()):
        raise ValueError("peers: need a contiguous int32 device tensor with N*S*R entries")
    if status is None:
        raise ValueError("status is required")
    _check_round_inputs(peers, None, status, N, S, R, status.device)
    rc = lib().combo_make_peer_table_dynamic(_dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
                                             _dev_ptr(status, torch.uint8, "status"), N, S, R,
                                             ctypes.c_uint64(seed), ctypes.c_uint64(rnd),
                                             _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_make_peer_table_dynamic")
    return peers


def segment_gossip_round_dynamic(dst, src, peers, status, P, S, R, dataset_sizes=None, stream=None):
    """combo_segment_gossip_round_dynamic on (N, ld)-strided float32 device tensors."""
    N = src.shape[0]
    ld = _matrix(src, "src")
    if _matrix(dst, "dst") != ld or dst.shape[0] != N:
        raise ValueError("dst must have src's row count and pitch")
    if status is None:
        raise ValueError("status is required")
    _check_round_inputs(peers, dataset_sizes, status, N, S, R, src.device)
    rc = lib().combo_segment_gossip_round_dynamic(
        _dev_ptr(dst, torch.float32, "dst"), _dev_ptr(src, torch.float32, "src"), ld,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        _dev_ptr(status, torch.uint8, "status"), N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_segment_gossip_round_dynamic")
    return dst


def aggregation_divergence_workspace(N, P):
    n = lib().combo_aggregation_divergence_workspace(N, P)
    if n < 0:
        raise ComboError(int(n), "combo_aggregation_divergence_workspace")
    return int(n)


def aggregation_divergence(dist2, x, P, workspace, dataset_sizes=None, stream=None):
    """combo_aggregation_divergence: dist2 (float64[N], device) <- squared distance of
    every row of x[:, :P] from the (weighted) mean row.  workspace: any device tensor of
    at least aggregation_divergence_workspace(N, P) bytes."""
    N = x.shape[0]
    ld = _matrix(x, "x")
    if dist2.numel() < N or not dist2.is_contiguous():
        raise ValueError("dist2: need a contiguous float64 device tensor with N entries")
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous device tensor")
    _check_round_inputs(None, dataset_sizes, None, N, 1, 0, x.device)
    rc = lib().combo_aggregation_divergence(
        _dev_ptr(dist2, torch.float64, "dist2"), _dev_ptr(x, torch.float32, "x"), ld,
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True), N, P,
        ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
        _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_aggregation_divergence")
    return dist2


def segment_gossip_round(dst, src, peers, P, S, R, dataset_sizes=None, stream=None):
    """combo_segment_gossip_round on (N, ld)-strided float32 device tensors dst, src."""
    N = src.shape[0]
    ld = _matrix(src, "src")
    if _matrix(dst, "dst") != ld or dst.shape[0] != N:
        raise ValueError("dst must have src's row count and pitch")
    _check_round_inputs(peers, dataset_sizes, None, N, S, R, src.device)
    rc = lib().combo_segment_gossip_round(
        _dev_ptr(dst, torch.float32, "dst"), _dev_ptr(src, torch.float32, "src"), ld,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_segment_gossip_round")
    return dst


def local_sgd_then_gossip(dst, src, grad, lr, peers, P, S, R, dataset_sizes=None, stream=None):
    """combo_local_sgd_then_gossip: src is stepped in place, dst receives the round."""
    N = src.shape[0]
    ld = _matrix(src, "src")
    if _matrix(dst, "dst") != ld or _matrix(grad, "grad") != ld or dst.shape[0] != N \
            or grad.shape[0] != N:
        raise ValueError("dst and grad must have src's row count and pitch")
    _check_round_inputs(peers, dataset_sizes, None, N, S, R, src.device)
    rc = lib().combo_local_sgd_then_gossip(
        _dev_ptr(dst, torch.float32, "dst"), _dev_ptr(src, torch.float32, "src"),
        _dev_ptr(grad, torch.float32, "grad"), ctypes.c_float(lr), ld,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_local_sgd_then_gossip")
    return dst


def local_sgd_steps_then_gossip(dst, src, grads, lr, peers, P, S, R, dataset_sizes=None, stream=None):
    """combo_local_sgd_steps_then_gossip: grads is a (tau, N, ld)-strided float32 device
    tensor (slice stride N*ld); tau = grads.shape[0]."""
    N = src.shape[0]
    ld = _matrix(src, "src")
    if _matrix(dst, "dst") != ld or dst.shape[0] != N:
        raise ValueError("dst must have src's row count and pitch")
    tau = grads.shape[0]
    if tau > 0 and not (grads.dim() == 3 and grads.shape[1] == N and grads.stride(2) == 1
                        and (N == 1 or grads.stride(1) == ld)
                        and (tau == 1 or grads.stride(0) == N * ld)):
        raise ValueError("grads: need (tau, N, .) float32 with src's pitch and slice stride N*ld")
    _check_round_inputs(peers, dataset_sizes, None, N, S, R, src.device)
    rc = lib().combo_local_sgd_steps_then_gossip(
        _dev_ptr(dst, torch.float32, "dst"), _dev_ptr(src, torch.float32, "src"),
        _dev_ptr(grads, torch.float32, "grads") if tau > 0 else None, tau, ctypes.c_float(lr), ld,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_local_sgd_steps_then_gossip")
    return dst


# ---- tiled arena layout [T][N][Wt] ----------------------------------------------------
def tiled_cols(N, R):
    w = lib().combo_tiled_cols(N, R)
    if w < 0:
        raise ComboError(int(w), "combo_tiled_cols")
    return int(w)


def tiled_elems(N, P, tile_cols):
    n = lib().combo_tiled_elems(N, P, tile_cols)
    if n < 0:
        raise ComboError(int(n), "combo_tiled_elems")
    return int(n)


def _flat(t, n, name):
    if not (t.is_contiguous() and t.numel() >= n):
        raise ValueError(f"{name}: need a contiguous float32 device tensor of at least {n} elements")
    return _dev_ptr(t, torch.float32, name)


def pack_tiled(tiled, rows, N, P, tile_cols, stream=None):
    """combo_pack_tiled: rows is an (N, ld)-strided matrix, tiled a flat buffer."""
    ld = _matrix(rows, "rows")
    rc = lib().combo_pack_tiled(_flat(tiled, tiled_elems(N, P, tile_cols), "tiled"),
                                _dev_ptr(rows, torch.float32, "rows"), ld, N, P, tile_cols,
                                _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_pack_tiled")
    return tiled


def unpack_tiled(rows, tiled, N, P, tile_cols, stream=None):
    ld = _matrix(rows, "rows")
    rc = lib().combo_unpack_tiled(_dev_ptr(rows, torch.float32, "rows"), ld,
                                  _flat(tiled, tiled_elems(N, P, tile_cols), "tiled"), N, P, tile_cols,
                                  _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_unpack_tiled")
    return rows


def segment_gossip_round_tiled(dst, src, tile_cols, peers, N, P, S, R, dataset_sizes=None,
                               status=None, stream=None):
    n = tiled_elems(N, P, tile_cols)
    _check_round_inputs(peers, dataset_sizes, status, N, S, R, src.device)
    rc = lib().combo_segment_gossip_round_tiled(
        _flat(dst, n, "dst"), _flat(src, n, "src"), tile_cols,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        _dev_ptr(status, torch.uint8, "status", optional=True), N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_segment_gossip_round_tiled")
    return dst


def local_sgd_steps_then_gossip_tiled(dst, src, grads, tau, lr, tile_cols, peers, N, P, S, R,
                                      dataset_sizes=None, stream=None):
    n = tiled_elems(N, P, tile_cols)
    _check_round_inputs(peers, dataset_sizes, None, N, S, R, src.device)
    rc = lib().combo_local_sgd_steps_then_gossip_tiled(
        _flat(dst, n, "dst"), _flat(src, n, "src"),
        _flat(grads, n * tau, "grads") if tau > 0 else None, tau, ctypes.c_float(lr), tile_cols,
        _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
        N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_local_sgd_steps_then_gossip_tiled")
    return dst


def aggregation_divergence_tiled(dist2, x, tile_cols, N, P, workspace, dataset_sizes=None, stream=None):
    """combo_aggregation_divergence_tiled: x is a flat tiled buffer [T][N][tile_cols]."""
    if dist2.numel() < N or not dist2.is_contiguous():
        raise ValueError("dist2: need a contiguous float64 device tensor with N entries")
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous device tensor")
    _check_round_inputs(None, dataset_sizes, None, N, 1, 0, x.device)
    rc = lib().combo_aggregation_divergence_tiled(
        _dev_ptr(dist2, torch.float64, "dist2"), _flat(x, tiled_elems(N, P, tile_cols), "x"), tile_cols,
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True), N, P,
        ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
        _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_aggregation_divergence_tiled")
    return dist2


def aggregation_divergence_noalloc(dist2, x, N, P, tile_cols=0, dataset_sizes=None, stream=None):
    """combo_aggregation_divergence_noalloc: the divergence monitor without a workspace
    argument.  tile_cols == 0: x is an (N, ld)-strided matrix; else a flat tiled buffer."""
    if dist2.numel() < N or not dist2.is_contiguous():
        raise ValueError("dist2: need a contiguous float64 device tensor with N entries")
    _check_round_inputs(None, dataset_sizes, None, N, 1, 0, x.device)
    if tile_cols:
        ld, px = 0, _flat(x, tiled_elems(N, P, tile_cols), "x")
    else:
        if x.shape[0] != N:
            raise ValueError("x: need N rows")
        ld, px = _matrix(x, "x"), _dev_ptr(x, torch.float32, "x")
    rc = lib().combo_aggregation_divergence_noalloc(
        _dev_ptr(dist2, torch.float64, "dist2"), px, ld, tile_cols,
        _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True), N, P,
        _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_aggregation_divergence_noalloc")
    return dist2


def round_relayout(dst, dst_tile_cols, src, src_tile_cols, peers, N, P, S, R, *, grads=None, lr=0.0,
                   dataset_sizes=None, status=None, stream=None):
    """combo_round_relayout: a round from one layout into another.  A side with tile_cols == 0
    is an (N, ld)-strided matrix, else a flat tiled buffer; grads (tau, ...) has src's layout."""
    tau = 0 if grads is None else int(grads.shape[0])
    _check_round_inputs(peers, dataset_sizes, status, N, S, R, dst.device)

    def side(t, tile, name):
        if tile:
            return _flat(t, tiled_elems(N, P, tile), name), 0
        if t.shape[0] != N:
            raise ValueError(f"{name}: need N rows")
        return _dev_ptr(t, torch.float32, name), _matrix(t, name)

    pd, dst_ld = side(dst, dst_tile_cols, "dst")
    ps, src_ld = side(src, src_tile_cols, "src")
    pg = None
    if tau:
        if src_tile_cols:
            pg = _flat(grads.reshape(-1), tiled_elems(N, P, src_tile_cols) * tau, "grads")
        else:
            if not (grads.dim() == 3 and grads.shape[1] == N and grads.stride(2) == 1
                    and (N == 1 or grads.stride(1) == src_ld) and (tau == 1 or grads.stride(0) == N * src_ld)):
                raise ValueError("grads: need (tau, N, .) float32 with src's pitch and slice stride N*ld")
            pg = _dev_ptr(grads, torch.float32, "grads")
    rc = lib().combo_round_relayout(pd, dst_ld, dst_tile_cols, ps, src_ld, src_tile_cols, pg, tau,
                                    ctypes.c_float(lr),
                                    _dev_ptr(peers, torch.int32, "peers", optional=(R == 0)),
                                    _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
                                    _dev_ptr(status, torch.uint8, "status", optional=True),
                                    N, P, S, R, _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_round_relayout")
    return dst


PROBE_COPY, PROBE_READ, PROBE_WRITE, PROBE_ROW_CHUNKS, PROBE_TILES, PROBE_MULTI_READ, PROBE_LDS_READ = range(7)


def bandwidth_probe(kind, dst, src, P, cols=0, param=None, stream=None):
    """combo_bandwidth_probe on (N, ld) float32 device matrices (src may be None for the
    write-only probe).  param defaults to 4 words in flight for the flat passes and to
    strip i -> workgroup i for the strip copies."""
    if param is None:
        param = 0 if kind in (PROBE_ROW_CHUNKS, PROBE_TILES) else 4
    N = dst.shape[0]
    ld = _matrix(dst, "dst")
    if src is not None and (src.shape[0] != N or _matrix(src, "src") != ld):
        raise ValueError("src must have dst's row count and pitch")
    rc = lib().combo_bandwidth_probe(int(kind), _dev_ptr(dst, torch.float32, "dst"),
                                     _dev_ptr(src, torch.float32, "src", optional=True), N, ld, P,
                                     int(cols), int(param), _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_bandwidth_probe")
    return dst


def round_hashed(dst, src, N, P, S, R, seed, rnd, *, grads=None, lr=0.0, tile_cols=0,
                 dataset_sizes=None, stream=None):
    """combo_round_hashed: peer selection + optional local steps + aggregation in one
    launch.  Row-major: dst/src are (N, ld)-strided, grads (tau, N, ld); tiled: flat buffers."""
    tau = 0 if grads is None else int(grads.shape[0])
    _check_round_inputs(None, dataset_sizes, None, N, S, 0, src.device)
    if tile_cols:
        n = tiled_elems(N, P, tile_cols)
        ld = tile_cols
        pd, ps = _flat(dst, n, "dst"), _flat(src, n, "src")
        pg = _flat(grads.reshape(-1), n * tau, "grads") if tau else None
    else:
        ld = _matrix(src, "src")
        if _matrix(dst, "dst") != ld or dst.shape[0] != N or src.shape[0] != N:
            raise ValueError("dst must have src's row count and pitch")
        pd, ps = _dev_ptr(dst, torch.float32, "dst"), _dev_ptr(src, torch.float32, "src")
        pg = _dev_ptr(grads, torch.float32, "grads") if tau else None
    rc = lib().combo_round_hashed(pd, ps, pg, tau, ctypes.c_float(lr), ld, tile_cols,
                                  _dev_ptr(dataset_sizes, torch.float32, "dataset_sizes", optional=True),
                                  N, P, S, R, ctypes.c_uint64(seed), ctypes.c_uint64(rnd),
                                  _stream_ptr(stream))
    if rc:
        raise ComboError(rc, "combo_round_hashed")
    return dst
