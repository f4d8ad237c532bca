"""One pass of the hot path on one GPU: buffers and the order of library calls, nothing else.

Per step (Alg. 3 of the paper, with the W workers simulated on the one device):
    worker sketches   S^w = S(g^w)                cs_sketch_accumulate_bundle  (T[w/8][j][b][w%8])
    aggregate         S_t = (1/W) sum_w S^w       cs_bundle_merge
                      (fold_workers: both at once, S_t += (1/W) S(g^w), cs_sketch_accumulate_sum)
    momentum, error   S_u = rho S_u + S_t ; S_v += S_u      cs_sketch_momentum   (stateful only)
    query all         est = estimate(S_v or S_t)  cs_sketch_estimate
    choose largest    idx = top-k |est|           cs_heavy_hitters_topk
    second round      x = (1/W) sum_w g^w[idx]    cs_gather_exact
    feedback          S_v -= S(est[idx]) ; S_u -= S(estimate(S_u, idx))   cs_sketch_feedback (stateful)
Every arithmetic step runs inside libcsketch.so; this class only owns tensors.
"""
from __future__ import annotations

import torch

from . import binding as B


class HotPath:
    def __init__(self, d: int, W: int, r: int, c: int, k: int, seed: int,
                 rho: float | None = None, device="cuda:0", P: int = 1, fold_workers: bool = False):
        """P > 1: the sketch is queried for the top P*k coordinates, the workers for their exact
        values, and the k largest exact sums are kept (Alg. 3 as the paper trains with it).
        fold_workers: the workers, which share this GPU, are summed as they are sketched
        (cs_sketch_accumulate_sum straight into S_t): no worker tables, no merge."""
        self.d, self.W, self.r, self.c, self.k = d, W, r, c, k
        self.P = P
        self.fold_workers = fold_workers
        self.kq = min(P * k, d)          # coordinates asked of the sketch
        self.rho = rho
        self.device = torch.device(device)
        self.params = B.cs_params_init(r, c, seed, d)
        f32 = dict(dtype=torch.float32, device=self.device)
        # the W workers' sketches as one bundle: T[w // 8][j][b][w % 8] = S^w[j][b]
        self.T = torch.zeros(B.cs_bundle_floats(self.params, 1 if fold_workers else W), **f32)
        self.S_t = torch.zeros(r, c, **f32)
        self.S_u = torch.zeros(r, c, **f32) if rho is not None else None
        self.S_v = torch.zeros(r, c, **f32) if rho is not None else None
        self.est = torch.empty(d, **f32)
        self.cand = torch.empty(self.kq, dtype=torch.int64, device=self.device)
        self.est_at_cand = torch.empty(self.kq, **f32)
        self.x_cand = torch.empty(self.kq, **f32)
        # with P = 1 the candidates are the selection
        self.idx = self.cand if P == 1 else torch.empty(k, dtype=torch.int64, device=self.device)
        self.est_at_idx = self.est_at_cand
        self.x = self.x_cand if P == 1 else torch.empty(k, **f32)
        self.delta = torch.empty(k, **f32)
        self.uhat = torch.empty(k, **f32)
        self.topk_ws = torch.empty(B.cs_topk_workspace_bytes(d, self.kq), dtype=torch.uint8,
                                   device=self.device)
        # counts of the estimates by magnitude bin: filled by the estimate, read by the selection
        self.hist = torch.zeros(B.CS_TOPK_HIST_BINS, dtype=torch.int64, device=self.device)
        n_est = B.cs_estimate_workspace_bytes(self.params, d)
        self.est_ws = (torch.empty(n_est, dtype=torch.uint8, device=self.device)
                       if n_est else None)

    # individual stages (bench.py times them separately) ---------------------------------
    def worker_table(self, w: int):
        """Worker w's own sketch (a strided view of the bundle)."""
        g = B.CS_BUNDLE_GROUP
        return self.T.view(-1, self.r, self.c, g)[w // g, :, :, w % g]

    def accumulate(self, g_w):
        if self.fold_workers:
            B.cs_sketch_zero(self.params, self.S_t)
            B.cs_sketch_accumulate_sum(self.params, self.S_t, g_w, scale=1.0 / self.W)
            return
        B.cs_bundle_zero(self.params, self.T, self.W)
        B.cs_sketch_accumulate_bundle(self.params, self.T, g_w)

    def merge(self):
        if self.fold_workers:
            return                       # S_t is complete already
        B.cs_bundle_merge(self.params, self.S_t, self.T, self.W, alpha=1.0 / self.W, beta=0.0)

    def momentum(self):
        if self.rho is not None:
            B.cs_sketch_momentum(self.params, self.S_u, self.S_v, self.S_t, self.rho)

    def query_table(self):
        return self.S_v if self.rho is not None else self.S_t

    def estimate(self):
        B.cs_sketch_estimate(self.params, self.query_table(), self.est, 0, self.est_ws, self.hist)

    def topk(self):
        B.cs_heavy_hitters_topk(self.est, self.kq, self.cand, self.est_at_cand, self.topk_ws, self.hist)

    def gather(self, g_w):
        B.cs_gather_exact(g_w, self.cand, self.x_cand, alpha=1.0 / self.W)
        if self.P > 1:
            B.cs_select_exact_topk(self.cand, self.x_cand, self.k, self.idx, self.x, self.topk_ws)

    def feedback(self):
        if self.rho is not None:
            B.cs_sketch_feedback(self.params, self.S_v, self.idx, self.delta)
            B.cs_sketch_feedback(self.params, self.S_u, self.idx, self.uhat)

    def step(self, g_w):
        """g_w: list of W fp32[d] device tensors.  Returns (idx, x): chosen coordinates
        (ascending) and their exact mean over workers."""
        self.accumulate(g_w)
        self.merge()
        self.momentum()
        self.estimate()
        self.topk()
        self.gather(g_w)
        self.feedback()
        return self.idx, self.x


class ReproduciblePath(HotPath):
    """The same step with sums that do not depend on the order of the additions, for debugging
    and for checkpoints that must resume bit for bit: the workers' vectors and the feedback go
    through the 64-bit fixed-point update (every contribution rounded once to a multiple of
    2^-frac_bits, integer sums), everything else is elementwise or integer already.  Two runs on
    equal inputs give equal bits; about one atomic request per coordinate and row, so far
    slower than HotPath.

        worker sketches   acc += fixed(g^w) for every w            cs_fixed_accumulate
        aggregate         S_t = float(acc) / W                     cs_fixed_to_float
        feedback          val = estimate(S, idx); S += float(fixed(-val at idx))
                          cs_sketch_estimate_sparse, cs_fixed_accumulate_sparse, cs_sketch_axpby
    `dropped` counts the coordinates that were left out (not finite, or too large for the
    chosen frac_bits) since the object was made."""

    def __init__(self, d, W, r, c, k, seed, rho=None, device="cuda:0", frac_bits: int = 40):
        super().__init__(d, 1, r, c, k, seed, rho=rho, device=device)     # no bundle of W tables
        self.W = W
        self.frac_bits = frac_bits
        self.acc = torch.zeros(r, c, dtype=torch.int64, device=self.device)
        self.dropped = torch.zeros(1, dtype=torch.int64, device=self.device)
        self.S_fb = torch.empty(r, c, dtype=torch.float32, device=self.device)

    def accumulate(self, g_w):
        self.acc.zero_()
        for g in g_w:
            B.cs_fixed_accumulate(self.params, self.acc, g, self.frac_bits, dropped=self.dropped)

    def merge(self):
        B.cs_fixed_to_float(self.params, self.acc, self.frac_bits, self.S_t, alpha=1.0 / self.W)

    def _feedback(self, S, val):
        B.cs_sketch_estimate_sparse(self.params, S, self.idx, val)
        self.acc.zero_()
        B.cs_fixed_accumulate_sparse(self.params, self.acc, self.idx, val, self.frac_bits,
                                     scale=-1.0, dropped=self.dropped)
        B.cs_fixed_to_float(self.params, self.acc, self.frac_bits, self.S_fb)
        B.cs_sketch_axpby(self.params, S, 1.0, self.S_fb, 1.0)

    def feedback(self):
        if self.rho is not None:
            self._feedback(self.S_v, self.delta)
            self._feedback(self.S_u, self.uhat)


class DenseStatePath(HotPath):
    """Alg. 3 as printed: momentum u^w and error accumulation v^w are dense vectors on every
    worker (2 W d floats), the sketch is taken of v^w, the second round returns exact sums of
    v^w, and u^w, v^w are zeroed on the coordinates of the update.  Costs one more streaming
    pass over the state (20 bytes per coordinate and worker) than the sketch-space form.

        momentum, error   u^w = rho u^w + g^w ; v^w += u^w          cs_dense_momentum
        worker sketches   S^w = S(v^w)                              cs_sketch_accumulate_bundle
        aggregate, query, choose                                    as in HotPath (stateless)
        second round      x = (1/W) sum_w v^w[idx]                  cs_gather_exact
        masking           u^w[idx] = v^w[idx] = 0                   cs_dense_mask
    """

    def __init__(self, d, W, r, c, k, seed, rho, device="cuda:0", P: int = 1):
        super().__init__(d, W, r, c, k, seed, rho=None, device=device, P=P)
        self.m = rho
        f32 = dict(dtype=torch.float32, device=self.device)
        self.u_w = [torch.zeros(d, **f32) for _ in range(W)]
        self.v_w = [torch.zeros(d, **f32) for _ in range(W)]

    def dense_momentum(self, g_w):
        B.cs_dense_momentum(self.u_w, self.v_w, g_w, self.m)

    def mask(self):
        B.cs_dense_mask(self.u_w, self.v_w, self.idx)

    def step(self, g_w):
        self.dense_momentum(g_w)
        self.accumulate(self.v_w)
        self.merge()
        self.estimate()
        self.topk()
        self.gather(self.v_w)
        self.mask()
        return self.idx, self.x


class GraphedStep:
    """One step of a HotPath (or DenseStatePath) captured once as a HIP graph and replayed.

    Every stage of a step is a fixed sequence of kernel launches on the caller's stream with
    fixed device pointers -- no allocation, no host synchronisation, no memset node -- so the
    whole step can be recorded and replayed with one submission.  That matters when a step is
    dozens of launches of a few microseconds each (small vectors); for d = 10^8 the kernels
    dominate and the graph changes nothing.  The gradients live in static buffers `g_w` that the
    caller overwrites before each replay; results appear in the HotPath's own tensors."""

    def __init__(self, path: HotPath, g_w):
        self.path = path
        self.g_w = g_w
        # one warm-up step outside the capture, on a side stream (a captured launch does not
        # execute, the warm-up does: the state it advanced is put back afterwards)
        saved = [t.clone() for t in self._state()]
        side = torch.cuda.Stream(device=path.device)
        side.wait_stream(torch.cuda.current_stream(path.device))
        with torch.cuda.stream(side):
            path.step(g_w)
        torch.cuda.current_stream(path.device).wait_stream(side)
        torch.cuda.synchronize(path.device)
        for t, s in zip(self._state(), saved):
            t.copy_(s)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            path.step(g_w)

    def _state(self):
        p = self.path
        out = [t for t in (p.S_u, p.S_v) if t is not None]
        out += list(getattr(p, "u_w", [])) + list(getattr(p, "v_w", []))
        return out

    def replay(self):
        self.graph.replay()
        return self.path.idx, self.path.x
