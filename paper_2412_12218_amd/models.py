"""Layer chaining of the two benchmark models (Section VI: 2-layer GCN with hidden size 16,
4-layer AGNN with hidden size 32): HotPath is the forward pass the benchmark times, TrainPath
the forward + backward pass of the same two models, PlannedGraph the per-graph adaptation that the
paper's outlook (Section VII) names: statistics of the graph decide how it is prepared.

Every step is a call into libftc through `binding`; this module only owns the device
buffers between the calls (allocated once in __init__, so a forward pass allocates nothing).
"""
import torch

from . import binding as B


class PlannedGraph:
    """Per-graph adaptive preparation (Section VII: fit the use of the hardware to the input graph).

    One pass over the graph's statistics (ftc_degree_stats, the window build's summary) goes to the host,
    ftc_plan_graph turns it into choices, and this class carries them out: relabel the nodes by degree
    class, or try the community ordering (label propagation) and keep it only if the windows then share
    more columns (sum_uniq drops), or leave the graph as it is.  `g` and `win` are the graph and window
    index to run the layers on; features enter with enter(X) and results leave with leave(Y), so the
    caller keeps the original numbering (permutation in, permutation out).  All device work is libftc's;
    the host only compares the few numbers the plan is made of."""

    def __init__(self, g, D, dtype, lp_rounds=10, side=None):
        self.g_given = g
        self.g, self.perm, self.inv, self.applied = g, None, None, "none"
        ws = B._workspace(B.lib().ftc_reorder_workspace_bytes(g.n, g.nnz), g.row_ptr.device)
        self.win = B.ftc_build_windows_concurrent(g, side)
        stats = B.ftc_degree_stats(g)
        self.sum_uniq_given = int(self.win.summary[0].item())          # the one host read the plan needs
        self.plan = B.ftc_plan_graph(g.n, g.nnz, int(stats[0].item()), self.sum_uniq_given, D, dtype)
        self.sum_uniq = self.sum_uniq_given
        order = self.plan["reorder"]
        if order == B.FTC_ORDER_DEGREE_CLASSES:
            perm, inv = B.ftc_degree_order(g, B.FTC_ORDER_DEGREE_CLASSES, ws=ws)
            self._relabel(perm, inv, ws, side, "degree classes", keep_if_fewer_columns=False)
        elif order == B.FTC_ORDER_COMMUNITIES:
            labels = B.ftc_label_propagation(g, lp_rounds, ws=ws)
            perm, inv, _ = B.ftc_order_by_key(labels, ws=ws)
            self._relabel(perm, inv, ws, side, "communities", keep_if_fewer_columns=True)

    def _relabel(self, perm, inv, ws, side, name, keep_if_fewer_columns):
        g2, flag = B.ftc_permute_graph(self.g_given, perm, inv, ws=ws)
        win2 = B.ftc_build_windows_concurrent(g2, side)
        su2 = int(win2.summary[0].item())
        assert int(flag.item()) == 0
        # a trial ordering is kept only if it makes the rows of a window share at least 2 % more columns
        if keep_if_fewer_columns and su2 > 0.98 * self.sum_uniq_given:
            self.trial = {"ordering": name, "sum_uniq": su2, "kept": False}
            return
        self.g, self.win, self.perm, self.inv, self.applied, self.sum_uniq = g2, win2, perm, inv, name, su2

    def enter(self, X, out=None):
        """Rows of X (original numbering) in the numbering of self.g."""
        return X if self.perm is None else B.ftc_permute_rows(X, self.perm, out=out)

    def leave(self, Y, out=None):
        """Rows of Y (numbering of self.g) back in the original numbering."""
        return Y if self.inv is None else B.ftc_permute_rows(Y, self.inv, out=out)


class HotPath:
    """window build + GCN normalisation + 2-layer GCN + 4-layer AGNN on one graph."""

    def __init__(self, g, d_feat=128, gcn_hidden=16, agnn_hidden=32, n_out=8, agnn_layers=4,
                 act_dtype=torch.float16, path=B.FTC_PATH_AUTO, concurrent_build=True):
        dev = g.row_ptr.device
        L = B.lib()
        self.g, self.path, self.agnn_layers = g, path, agnn_layers
        self.win = B.Windows(g)
        # the independent kernels of the window build overlap on three side streams owned here
        self.side = B.SideStreams() if concurrent_build else None
        n, nnz = g.n, g.nnz
        f32 = dict(dtype=torch.float32, device=dev)
        act = dict(dtype=act_dtype, device=dev)
        self.ws_win = B._workspace(L.ftc_build_windows_workspace_bytes(n, nnz, 16, 8), dev)
        self.dinv = torch.empty(n, **f32)    # the GCN layers take the factored normalisation: no per-edge values
        self.gcn_h = torch.empty((n, gcn_hidden), **act)
        self.gcn_out = torch.empty((n, n_out), **f32)
        ws_gcn = max(L.ftc_gcn_layer_workspace_bytes(n, nnz, d_feat, gcn_hidden),
                     L.ftc_gcn_layer_workspace_bytes(n, nnz, gcn_hidden, n_out))
        self.agnn_h = [torch.empty((n, agnn_hidden), **act) for _ in range(2)]
        self.agnn_out = torch.empty((n, n_out), **f32)
        ws_agnn = L.ftc_agnn_layer_workspace_bytes(n, nnz, agnn_hidden)
        self.ws = B._workspace(max(ws_gcn, ws_agnn), dev)

    def build(self):
        g, w = self.g, self.win
        B.ftc_build_windows_concurrent(g, self.side, out=w, ws=self.ws_win)
        B._check(B.lib().ftc_gcn_norm(B.C.byref(g.c), B.C.byref(w.c), None, B._ptr(self.dinv),
                                      B._stream()))

    def gcn(self, X, W1, W2):
        B.ftc_gcn_layer(self.g, self.win, None, X, W1, relu=True, out=self.gcn_h, path=self.path,
                        ws=self.ws, dinv=self.dinv)
        B.ftc_gcn_layer(self.g, self.win, None, self.gcn_h, W2, relu=False, out=self.gcn_out,
                        path=self.path, ws=self.ws, dinv=self.dinv)
        return self.gcn_out

    def agnn(self, X, W_in, W_out, betas):
        a, b = self.agnn_h
        B.ftc_update_gemm(X, W_in, out=a, relu=True)
        for layer in range(self.agnn_layers):
            B.ftc_agnn_layer(self.g, self.win, a, beta=betas[layer], out=b, path=self.path, ws=self.ws)
            a, b = b, a
        B.ftc_update_gemm(a, W_out, out=self.agnn_out)
        return self.agnn_out

    def step(self, X, W1, W2, W_in, W_out, betas):
        self.build()
        self.gcn(X, W1, W2)
        self.agnn(X, W_in, W_out, betas)

    def capture(self, X, W1, W2, W_in, W_out, betas):
        """The step as a HIP graph: every call of the library only enqueues kernels (and the window build's
        fork / join events) on the stream it is given and allocates nothing, so the whole step can be
        captured once and replayed with one launch; the results land in the same buffers as step()'s.
        The library keeps no state, so nothing has to run eagerly first."""
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(X, W1, W2, W_in, W_out, betas)
        return graph


class TrainPath:
    """Forward + backward of the two models on one graph with a symmetric pattern (the paper
    names training in Sections II and V and gives no formulas: the gradients are the derivatives
    of the forward definitions).  The GCN normalisation is the factored one, whose transposed
    operator is the operator itself; the AGNN backward needs the transposed index, built once here."""

    def __init__(self, g, win, dinv, d_feat=128, gcn_hidden=16, agnn_hidden=32, n_out=8, agnn_layers=4,
                 act_dtype=torch.float16, path=B.FTC_PATH_AUTO, fused=True):
        dev = g.row_ptr.device
        L = B.lib()
        self.g, self.win, self.dinv, self.path, self.agnn_layers = g, win, dinv, path, agnn_layers
        n, nnz = g.n, g.nnz
        self.T, flag = B.ftc_transpose_index(g, win)
        self.pattern_flag = flag           # handed to the single-pass backward, which refuses a non-symmetric pattern
        if int(flag.item()) != 0:
            raise ValueError("TrainPath needs a symmetric sparsity pattern with ascending, duplicate-free rows")
        f32 = dict(dtype=torch.float32, device=dev)
        act = dict(dtype=act_dtype, device=dev)
        self.gcn_h = torch.empty((n, gcn_hidden), **act)
        self.gcn_out = torch.empty((n, n_out), **f32)
        self.agnn_h = [None] + [torch.empty((n, agnn_hidden), **act) for _ in range(agnn_layers)]
        # single-pass forward / backward pair when the shape allows it: per-row softmax denominators are
        # kept instead of the per-entry probabilities, and no transposed index is read
        self.fused = bool(fused and win is not None and L.ftc_agnn_layer_backward_fused_workspace_bytes(n, nnz, agnn_hidden) > 0
                          and (agnn_hidden * self.agnn_h_itemsize(act_dtype)) % 16 == 0)
        self.agnn_z = [torch.empty(n, **f32) for _ in range(agnn_layers)] if self.fused else []
        # 16-bit activations: every layer also keeps its unrounded output for the backward pass
        self.keep_f32 = self.fused and act_dtype != torch.float32
        self.agnn_y32 = [torch.empty((n, (agnn_hidden + 3) // 4 * 4), **f32) for _ in range(agnn_layers)] \
            if self.keep_f32 else []
        self.agnn_p = [torch.empty(nnz, **f32) for _ in range(agnn_layers)] if not self.fused else []
        self.d_agnn_h = [torch.empty((n, agnn_hidden), **act) for _ in range(2)]
        self.agnn_h0 = torch.empty((n, agnn_hidden), **act)     # output of the in-projection
        self.d_agnn_h0 = torch.empty((n, agnn_hidden), **f32)   # gradient entering the in-projection
        self.agnn_out = torch.empty((n, n_out), **f32)
        self.dbeta = torch.empty(agnn_layers, **f32)
        self.ws = B._workspace(max(
            L.ftc_gcn_layer_workspace_bytes(n, nnz, d_feat, gcn_hidden),
            L.ftc_gcn_layer_workspace_bytes(n, nnz, gcn_hidden, n_out),
            L.ftc_gcn_layer_backward_workspace_bytes(n, nnz, d_feat, gcn_hidden),
            L.ftc_gcn_layer_backward_workspace_bytes(n, nnz, gcn_hidden, n_out),
            L.ftc_agnn_layer_workspace_bytes(n, nnz, agnn_hidden),
            L.ftc_agnn_layer_backward_workspace_bytes(n, nnz, agnn_hidden),
            L.ftc_agnn_layer_backward_fused_workspace_bytes(n, nnz, agnn_hidden),
            L.ftc_update_gemm_backward_workspace_bytes(n, d_feat, agnn_hidden),
            L.ftc_update_gemm_backward_workspace_bytes(n, agnn_hidden, n_out)), dev)

    @staticmethod
    def agnn_h_itemsize(dtype):
        return torch.empty(0, dtype=dtype).element_size()

    def gcn_forward(self, X, W1, W2):
        B.ftc_gcn_layer(self.g, self.win, None, X, W1, relu=True, out=self.gcn_h, path=self.path, ws=self.ws,
                        dinv=self.dinv)
        B.ftc_gcn_layer(self.g, self.win, None, self.gcn_h, W2, relu=False, out=self.gcn_out, path=self.path,
                        ws=self.ws, dinv=self.dinv)
        return self.gcn_out

    def gcn_backward(self, X, W1, W2, d_out):
        """d_out = dL/d(gcn_out), fp32.  Returns (dW1, dW2); the input features get no gradient."""
        d_h, dW2 = B.ftc_gcn_layer_backward(self.g, self.win, None, self.gcn_h, W2, d_out, dinv=self.dinv,
                                            path=self.path, ws=self.ws)
        _, dW1 = B.ftc_gcn_layer_backward(self.g, self.win, None, X, W1, d_h, Y=self.gcn_h, dinv=self.dinv,
                                          want_dX=False, path=self.path, ws=self.ws)
        return dW1, dW2

    def agnn_forward(self, H0, betas):
        """Propagation layers only; every layer keeps what its backward pass needs: the softmax
        denominators (and its unrounded output when the activations are 16-bit) on the single-pass route,
        the attention probabilities on the edge-array route."""
        self.agnn_h[0] = H0
        for l in range(self.agnn_layers):
            keep = dict(row_z=self.agnn_z[l]) if self.fused else dict(edge_p=self.agnn_p[l])
            if self.keep_f32:
                keep["out_f32"] = self.agnn_y32[l]
            B.ftc_agnn_layer(self.g, self.win, self.agnn_h[l], beta=betas[l], out=self.agnn_h[l + 1],
                             path=self.path, ws=self.ws, **keep)
        return self.agnn_h[self.agnn_layers]

    def agnn_backward(self, betas, d_out, first_in_f32=False):
        """d_out = dL/d(last layer's output), in the activation type.  Returns (dL/dH0, dbeta[layers]);
        dL/dH0 in fp32 when first_in_f32 (what the backward of the in-projection takes)."""
        d = d_out
        for l in reversed(range(self.agnn_layers)):
            nxt = self.d_agnn_h0 if (l == 0 and first_in_f32) else self.d_agnn_h[l & 1]
            if self.fused:
                y = self.agnn_y32[l][:, :self.agnn_h[l].shape[1]] if self.keep_f32 else self.agnn_h[l + 1]
                B.ftc_agnn_layer_backward_fused(self.g, self.win, self.agnn_h[l], self.agnn_z[l], y, d,
                                                beta=betas[l], dH=nxt, dbeta=self.dbeta[l:l + 1], ws=self.ws,
                                                pattern_flag=self.pattern_flag)
            else:
                B.ftc_agnn_layer_backward(self.g, self.win, self.T, self.agnn_h[l], self.agnn_p[l], d, beta=betas[l],
                                          dH=nxt, dbeta=self.dbeta[l:l + 1], path=self.path, ws=self.ws)
            d = nxt
        return d, self.dbeta

    def agnn_model_forward(self, X, W_in, W_out, betas):
        """The whole AGNN model of the benchmark: ReLU in-projection, propagation layers, out-projection."""
        B.ftc_update_gemm(X, W_in, out=self.agnn_h0, relu=True)
        h = self.agnn_forward(self.agnn_h0, betas)
        B.ftc_update_gemm(h, W_out, out=self.agnn_out)
        return self.agnn_out

    def agnn_model_backward(self, X, W_in, W_out, betas, d_out):
        """d_out = dL/d(agnn_out), fp32.  Returns (dW_in, dW_out, dbeta[layers])."""
        h_last = self.agnn_h[self.agnn_layers]
        d_h, dW_out = B.ftc_update_gemm_backward(h_last, W_out, d_out, dX=self.d_agnn_h[self.agnn_layers & 1], ws=self.ws)
        d_h0, dbeta = self.agnn_backward(betas, d_h, first_in_f32=True)
        _, dW_in = B.ftc_update_gemm_backward(X, W_in, d_h0, Z=self.agnn_h0, want_dX=False, ws=self.ws)
        return dW_in, dW_out, dbeta
