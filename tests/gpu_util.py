"""Helpers of the GPU parity tests: marshal a workloads.Trace into the library."""
import numpy as np

import paper_2508_13231_amd as K
import workloads as W


class Gpu:
    """A library context with one uploaded trace; device tensors via torch."""

    def __init__(self, tr, device=0, score_kernel=None):
        import torch
        self.torch = torch
        self.tr = tr
        self.dev = torch.device("cuda", device)
        self.ctx = K.kvp_create(device)
        self.problem = K.make_problem(tr.L, tr.N, tr.P, tr.K, tr.plane_bytes, tr.page_bytes, tr.token_bytes,
                                      tr.bw_hbm, tr.bw_link, tr.bw_dram, tr.cap_pages)
        K.kvp_trace_upload(self.ctx, self.problem, W.pack_bits(tr.access), W.pack_bits(tr.alive),
                           W.pack_bits(tr.persist), W.pack_bits(tr.written))
        if score_kernel is not None:
            K.kvp_set_score_kernel(self.ctx, score_kernel)
        self.unit = K.kvp_plane_unit(self.ctx)
        self.shape_words = (tr.L, tr.N, tr.n_words)

    def close(self):
        if self.ctx is not None:
            K.kvp_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def to_dev(self, a, dtype=None):
        t = self.torch.from_numpy(np.ascontiguousarray(a))
        return t.to(self.dev)

    def words(self, X):
        """bool [S][L][N][P] -> device int32 tensor of packed words."""
        w = W.pack_bits(X).view(np.int32)
        return self.to_dev(w)

    def score(self, X, counters=True):
        """X: bool [S][L][N][P].  Returns numpy (cost, excess, counters, occ)."""
        torch = self.torch
        tr = self.tr
        S = X.shape[0]
        d_x = self.words(X)
        d_cost = torch.empty(S, dtype=torch.float64, device=self.dev)
        d_ex = torch.empty(S, dtype=torch.int32, device=self.dev)
        d_cnt = torch.empty((S, tr.L, tr.N, 4), dtype=torch.int32, device=self.dev) if counters else None
        d_occ = torch.empty((S, tr.N), dtype=torch.int32, device=self.dev) if counters else None
        K.kvp_score(self.ctx, d_x, S, d_cost, d_ex, d_cnt, d_occ)
        torch.cuda.synchronize()
        out = [d_cost.cpu().numpy(), d_ex.cpu().numpy().view(np.uint32)]
        out += [d_cnt.cpu().numpy().view(np.uint32), d_occ.cpu().numpy().view(np.uint32)] if counters else [None, None]
        return out

    def baseline(self, kind):
        """Schedule of kvp_baseline as bool [L][N][P]."""
        torch = self.torch
        tr = self.tr
        d = torch.full((tr.L, tr.N, tr.n_words), -1, dtype=torch.int32, device=self.dev)
        K.kvp_baseline(self.ctx, kind, d)
        torch.cuda.synchronize()
        return self.unpack(d.cpu().numpy().view(np.uint32))

    def kernel_used(self):
        return K.kvp_score_kernel_used(self.ctx)

    def delta(self, X, moves, give_counters):
        torch = self.torch
        tr = self.tr
        S = X.shape[0]
        d_x = self.words(X)
        d_mv = self.to_dev(W.moves_to_records(moves).view(np.int32))
        d_delta = torch.empty(S, dtype=torch.float64, device=self.dev)
        d_ver = torch.empty(S, dtype=torch.int32, device=self.dev)
        d_cnt = d_occ = None
        if give_counters:
            d_cost = torch.empty(S, dtype=torch.float64, device=self.dev)
            d_ex = torch.empty(S, dtype=torch.int32, device=self.dev)
            d_cnt = torch.empty((S, tr.L, tr.N, 4), dtype=torch.int32, device=self.dev)
            d_occ = torch.empty((S, tr.N), dtype=torch.int32, device=self.dev)
            K.kvp_score(self.ctx, d_x, S, d_cost, d_ex, d_cnt, d_occ)
        K.kvp_delta_score(self.ctx, d_x, S, d_mv, d_cnt, d_occ, d_delta, d_ver)
        torch.cuda.synchronize()
        return d_delta.cpu().numpy(), d_ver.cpu().numpy()

    def unpack(self, words):
        return W.unpack_bits(words, self.tr.P)


def expected_counters(sc, tr, unit):
    """Oracle step bytes -> the library's counter units [L][N][4]."""
    sb = sc.step_bytes.astype(np.uint64)
    c = np.zeros((tr.L, tr.N, 4), dtype=np.uint64)
    c[..., 0] = sb[..., 0] // unit
    assert (sb[..., 0] % unit == 0).all()
    c[..., 1] = sb[..., 2] // max(tr.token_bytes, 1)
    c[..., 2] = sb[..., 4] // tr.page_bytes
    c[..., 3] = sb[..., 5] // tr.page_bytes
    return c
