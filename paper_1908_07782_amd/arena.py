"""A double-buffered parameter arena for N simulated workers, driven through the C ABI.

Convenience only: it owns the two parameter buffers, the peer table and the round
counter (torch tensors), and every step is two library calls (peer table, then the
round) enqueued on the current stream - nothing here computes on its own.  The front
buffer always holds the pre-round state and the back buffer receives the aggregate
(Sec. 4.1 of the segmented-gossip paper: pulled segments are the providers' state from
before the aggregation), then the two are swapped.
"""
import torch

from . import binding as _b
from . import workloads as _w


class GossipArena:
    def __init__(self, N, P, S, R, *, layout="tiled", seed=0, dataset_sizes=None, selection="segment",
                 device="cuda"):
        if layout not in ("tiled", "rows"):
            raise ValueError("layout must be 'tiled' or 'rows'")
        if selection not in ("segment", "pooled"):
            raise ValueError("selection must be 'segment' (R distinct peers per segment) or 'pooled'")
        self.N, self.P, self.S, self.R = int(N), int(P), int(S), int(R)
        self.layout, self.seed, self.selection = layout, int(seed), selection
        self.round = 0
        self.device = torch.device(device)
        self.ld = _w.row_pitch(self.P)
        if layout == "tiled":
            self.tile_cols = _b.tiled_cols(self.N, self.R)
            n = _b.tiled_elems(self.N, self.P, self.tile_cols)
            self._buf = torch.zeros((2, n), dtype=torch.float32, device=self.device)
        else:
            self.tile_cols = 0
            self._buf = torch.zeros((2, self.N, self.ld), dtype=torch.float32, device=self.device)
        self._cur = 0
        self.peers = torch.zeros(max(self.N * self.S * self.R, 1), dtype=torch.int32, device=self.device)
        self.dataset_sizes = None
        if dataset_sizes is not None:
            self.dataset_sizes = torch.as_tensor(dataset_sizes, dtype=torch.float32).to(self.device).contiguous()
            if self.dataset_sizes.shape != (self.N,):
                raise ValueError("dataset_sizes must have N entries")
        self._ws = None

    # ---- buffers ---------------------------------------------------------------------
    @property
    def front(self):
        """The current parameters in the arena's own layout."""
        return self._buf[self._cur]

    @property
    def back(self):
        return self._buf[1 - self._cur]

    def like_front(self, tau=1):
        """A zeroed gradient buffer of tau slices in the arena's layout."""
        shape = (tau,) + tuple(self.front.shape)
        return torch.zeros(shape, dtype=torch.float32, device=self.device)

    def load(self, rows):
        """Set the parameters from an (N, >=P) row-major float32 device tensor."""
        rows = rows.to(self.device)
        if rows.shape[0] != self.N or rows.shape[1] < self.P:
            raise ValueError("rows must be (N, >= P)")
        if self.layout == "tiled":
            _b.pack_tiled(self.front, rows, self.N, self.P, self.tile_cols)
        else:
            self.front[:, :self.P].copy_(rows[:, :self.P])
        return self

    def export(self, out=None):
        """The current parameters as an (N, P) row-major tensor."""
        if self.layout == "rows":
            res = self.front[:, :self.P]
            return res.clone() if out is None else out.copy_(res)
        if out is None:
            out = torch.empty((self.N, self.ld), dtype=torch.float32, device=self.device)
        _b.unpack_tiled(out, self.front, self.N, self.P, self.tile_cols)
        return out[:, :self.P]

    def pack_like_front(self, dst, rows):
        """Convert an (N, >=P) row-major tensor (e.g. gradients) into the arena's layout."""
        if self.layout == "tiled":
            _b.pack_tiled(dst, rows, self.N, self.P, self.tile_cols)
        else:
            dst[:, :self.P].copy_(rows[:, :self.P])
        return dst

    # ---- one synchronisation round ---------------------------------------------------
    def _make_table(self, status):
        N, S, R = self.N, self.S, self.R
        if status is not None:
            _b.make_peer_table_dynamic(self.peers, status, N, S, R, self.seed, self.round)
        elif self.selection == "pooled":
            _b.make_peer_table_pooled(self.peers, N, S, R, self.seed, self.round)
        else:
            _b.make_peer_table(self.peers, N, S, R, self.seed, self.round)
        return self.peers if R > 0 else None

    def step_in(self, rows, grads=None, lr=0.0, status=None):
        """A round whose front buffer is the caller's row-major (N, ld) tensor `rows` (and
        row-major gradients (tau, N, ld)): the result lands in the arena's own layout, so a
        tiled arena is entered without a separate conversion pass."""
        peers = self._make_table(status)
        _b.round_relayout(self.back, self.tile_cols, rows, 0, peers, self.N, self.P, self.S, self.R,
                          grads=grads, lr=lr, dataset_sizes=self.dataset_sizes, status=status)
        self._cur = 1 - self._cur
        self.round += 1
        return self

    def step_out(self, out_rows, grads=None, lr=0.0, status=None):
        """A round from the arena's front buffer into the caller's row-major (N, ld) tensor
        `out_rows` (gradients in the arena's layout).  The arena's own buffers are unchanged."""
        peers = self._make_table(status)
        _b.round_relayout(out_rows, 0, self.front, self.tile_cols, peers, self.N, self.P, self.S, self.R,
                          grads=grads, lr=lr, dataset_sizes=self.dataset_sizes, status=status)
        self.round += 1
        return out_rows

    def step(self, grads=None, lr=0.0, status=None):
        """Peer table of the current round, then the aggregation (after the tau local SGD
        steps with `grads`, shape (tau,) + front.shape, if given), then swap.  `status`
        (uint8[N]: 0 offline, 1 active, 2 newcomer) selects the dynamic-worker semantics."""
        N, P, S, R = self.N, self.P, self.S, self.R
        if status is not None and grads is not None:
            raise ValueError("dynamic workers and fused local steps cannot be combined")
        peers = self._make_table(status)
        d = self.dataset_sizes
        if self.layout == "tiled":
            if grads is not None:
                _b.local_sgd_steps_then_gossip_tiled(self.back, self.front, grads.reshape(-1),
                                                     grads.shape[0], lr, self.tile_cols, peers, N, P, S, R,
                                                     dataset_sizes=d)
            else:
                _b.segment_gossip_round_tiled(self.back, self.front, self.tile_cols, peers, N, P, S, R,
                                              dataset_sizes=d, status=status)
        else:
            if grads is not None:
                _b.local_sgd_steps_then_gossip(self.back, self.front, grads, lr, peers, P, S, R,
                                               dataset_sizes=d)
            elif status is not None:
                _b.segment_gossip_round_dynamic(self.back, self.front, peers, status, P, S, R,
                                                dataset_sizes=d)
            else:
                _b.segment_gossip_round(self.back, self.front, peers, P, S, R, dataset_sizes=d)
        self._cur = 1 - self._cur
        self.round += 1
        return self

    # ---- monitoring ------------------------------------------------------------------
    def divergence(self):
        """Squared L2 distance of every worker from the (weighted) mean of all workers
        (Sec. 4.3, Definition 2), float64[N] on the device."""
        if self._ws is None:
            self._ws = torch.empty(_b.aggregation_divergence_workspace(self.N, self.P) // 8,
                                   dtype=torch.float64, device=self.device)
        out = torch.empty(self.N, dtype=torch.float64, device=self.device)
        if self.layout == "tiled":
            _b.aggregation_divergence_tiled(out, self.front, self.tile_cols, self.N, self.P, self._ws,
                                            dataset_sizes=self.dataset_sizes)
        else:
            _b.aggregation_divergence(out, self.front, self.P, self._ws, dataset_sizes=self.dataset_sizes)
        return out

    def serve_load(self):
        """How many requests of the last table each worker serves (int32[N])."""
        deg = torch.empty(self.N, dtype=torch.int32, device=self.device)
        _b.peer_in_degree(deg, self.peers, self.N, self.S, self.R)
        return deg
