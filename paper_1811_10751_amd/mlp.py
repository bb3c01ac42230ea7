"""Coded MLP training loop: a sequence of C-ABI calls (no arithmetic in Python).

One iteration follows Sec. VII / IX of arXiv 1811.10751: for every layer the coded forward
step O1 and the element-wise C1; the last-layer error; then for every layer, from the last
to the first, the coded backward step O2, the coded update O3 and the element-wise C2.
"""
from __future__ import annotations

from . import binding as B


class CodedMLP:
    def __init__(self, sizes, batch, m, n, d1, d2, P, worker_dtype=B.GPD_F32, subst=B.GPD_SUB_AUTO,
                 rho_detect=0.0, stream=None):
        self.sizes, self.batch = tuple(sizes), batch
        self.layers = [B.gpd_layer_create(sizes[l + 1], sizes[l], batch, m, n, d1, d2, P,
                                          worker_dtype=worker_dtype, subst=subst,
                                          rho_detect=rho_detect, stream=stream)
                       for l in range(len(sizes) - 1)]
        self.Wts = [None] * len(self.layers)
        self.stream = stream
        self._ckpt = None
        self.repaired = []
        self.restored = False
        # device tensors of the last iteration, for inspection: acts[l] = input of layer l (acts[0]
        # = X, acts[L] = network output), deltas[l] = error Delta of layer l
        self.acts = []
        self.deltas = []
        self._act_bufs = None
        self.fused = None              # None: not tried yet; False: the network is outside the fused path

    def encode_weights(self, Ws):
        """Ws: list of float32 CUDA tensors (N_out x N_in).  Done once before training."""
        self.Wts = [B.gpd_layer_encode_weights(L, W) for L, W in zip(self.layers, Ws)]

    def decode_weights(self):
        return [B.gpd_layer_decode_weights(L, Wt) for L, Wt in zip(self.layers, self.Wts)]

    def checkpoint(self):
        """Keeps a copy of the coded weights (Sec. VII, error model 2: the network is checkpointed
        at regular intervals; here in device memory)."""
        self._ckpt = [wt.clone() for wt in self.Wts]

    def restore(self):
        """Puts the last checkpoint back (after a decoding failure or a failed verification)."""
        if self._ckpt is None:
            raise RuntimeError("no checkpoint taken")
        for wt, c in zip(self.Wts, self._ckpt):
            wt.copy_(c)

    def _regenerate(self, l, rep):
        """Regeneration (Sec. VII): the coded weights of the nodes a node-level decode has just
        found erroneous are recomputed from the other nodes.  Returns the nodes repaired."""
        bad = [p for p in range(self.layers[l].P) if rep.node_err_count[p] > 0]
        if bad and rep.status == B.GPD_OK:
            B.gpd_layer_regenerate(self.layers[l], self.Wts[l], bad)
        return bad

    def step(self, X, Y, eta, decay=0.0, correct_errors=False, want_report=False, regenerate=False,
             restore_on_failure=False):
        """One training iteration on the mini-batch X (N_0 x batch), labels Y (N_L x batch).
        Returns (network output, per-layer list of (forward report, backward report)).
        regenerate (with correct_errors = GPD_CORRECT_NODES): nodes located as erroneous get
        their coded weights regenerated right after the decode that found them.
        restore_on_failure: a decode that reports errors it cannot locate (GPD_E_DECODE_FAIL)
        stops the iteration at once and puts the last checkpoint back; the call then returns
        (None, reports so far) with self.restored set."""
        regenerate = regenerate and int(correct_errors) == B.GPD_CORRECT_NODES
        want_report = want_report or regenerate or restore_on_failure
        if not (correct_errors or want_report) and self.fused is not False:
            # small batches, nothing to correct or report: the whole iteration through gpd_mlp_step
            # (one launch for the master's work between two coded products; same arithmetic)
            if self._act_bufs is None:
                import torch
                self._act_bufs = [torch.empty((L.N_out, L.batch), dtype=torch.float32, device=X.device)
                                  for L in self.layers]
            self.fused = B.gpd_mlp_step(self.layers, self.Wts, X, Y, eta, decay, self._act_bufs)
            if self.fused:
                self.acts = [X] + self._act_bufs
                self.deltas = [L.workspace_delta(X.device) for L in self.layers]
                self.repaired, self.restored = [], False
                return self._act_bufs[-1], [[None, None] for _ in self.layers]
        acts = [X]
        reps = []
        self.repaired = []
        self.restored = False

        def failed(rep):
            if restore_on_failure and rep is not None and rep.status == B.GPD_E_DECODE_FAIL:
                self.restore()
                self.restored = True
                return True
            return False

        for l, (L, Wt) in enumerate(zip(self.layers, self.Wts)):
            # (the logistic function, step C1, is applied by the decode itself)
            act, rf = B.gpd_coded_layer_step(L, B.GPD_STEP_FORWARD, Wt, acts[-1],
                                             correct_errors=correct_errors, want_report=want_report,
                                             fuse_sigmoid=True)
            reps.append([rf, None])
            if failed(rf):
                return None, reps
            if regenerate:
                self.repaired += [(l, "forward", p) for p in self._regenerate(l, rf)]
            acts.append(act)
        delta = B.gpd_l2_delta(Y, acts[-1], 2.0 / self.batch, stream=self.stream)
        self.acts = acts
        self.deltas = [None] * len(self.layers)
        for l in range(len(self.layers) - 1, -1, -1):
            self.deltas[l] = delta
            C, rb = B.gpd_coded_layer_step(self.layers[l], B.GPD_STEP_BACKWARD_UPDATE, self.Wts[l],
                                           acts[l], Dlt=delta, eta=eta, decay=decay,
                                           correct_errors=correct_errors, want_report=want_report,
                                           skip_output=(l == 0), fuse_sigmoid=True)
            reps[l][1] = rb
            if failed(rb):
                return None, reps
            if regenerate and l > 0:
                self.repaired += [(l, "backward", p) for p in self._regenerate(l, rb)]
            if l > 0:
                delta = C                 # already C o Y (1 - Y), step C2, Y = acts[l]
        return acts[-1], reps


class CodedAutoencoder:
    """Sparse autoencoder with one hidden layer (Sec. X): N0 -> N1 -> N0, both weight matrices
    kept encoded; the loss is the reconstruction error plus beta * sum_i KL(rho || rho_hat_i)."""

    def __init__(self, N0, N1, batch, m, n, P, d1=1, d2=1, worker_dtype=B.GPD_F32, stream=None):
        self.N0, self.N1, self.batch, self.stream = N0, N1, batch, stream
        self.l1 = B.gpd_layer_create(N1, N0, batch, m, n, d1, d2, P, worker_dtype=worker_dtype, stream=stream)
        self.l2 = B.gpd_layer_create(N0, N1, batch, m, n, d1, d2, P, worker_dtype=worker_dtype, stream=stream)
        self.Wt1 = self.Wt2 = None

    def encode_weights(self, W1, W2):
        self.Wt1 = B.gpd_layer_encode_weights(self.l1, W1)
        self.Wt2 = B.gpd_layer_encode_weights(self.l2, W2)

    def decode_weights(self):
        return B.gpd_layer_decode_weights(self.l1, self.Wt1), B.gpd_layer_decode_weights(self.l2, self.Wt2)

    def step(self, X, eta, rho, beta, decay=0.0):
        """One iteration on the mini-batch X (N0 x batch); returns the reconstruction."""
        S1, _ = B.gpd_coded_layer_step(self.l1, B.GPD_STEP_FORWARD, self.Wt1, X)
        Y1 = B.gpd_sigmoid_fwd(S1, stream=self.stream)
        S2, _ = B.gpd_coded_layer_step(self.l2, B.GPD_STEP_FORWARD, self.Wt2, Y1)
        Y2 = B.gpd_sigmoid_fwd(S2, stream=self.stream)
        d2 = B.gpd_l2_delta(X, Y2, 2.0 / self.batch, stream=self.stream)
        C2, _ = B.gpd_coded_layer_step(self.l2, B.GPD_STEP_BACKWARD_UPDATE, self.Wt2, Y1, Dlt=d2, eta=eta,
                                       decay=decay)
        rho_hat = B.gpd_row_mean(Y1, stream=self.stream)
        d1 = B.gpd_sigmoid_bwd_sparse(C2, Y1, rho_hat, rho, beta / self.batch, stream=self.stream)
        B.gpd_coded_layer_step(self.l1, B.GPD_STEP_BACKWARD_UPDATE, self.Wt1, X, Dlt=d1, eta=eta, decay=decay,
                               skip_output=True)
        return Y2
