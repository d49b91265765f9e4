"""Shared machinery of the GPU parity tests: runs the HIP path (through the C ABI binding) and
the CPU oracle side by side on the same seeded inputs.

Comparison rules (stated once here, used by every test):
  * integers that do not depend on floating point (accepted lengths under an imposed
    schedule, appended tokens given the proposals, counters) must be bit-identical;
  * logits: |gpu - oracle| <= TOL[dtype]  (1e-4 in fp32 mode, 2e-2 in bf16 mode) at every width the paper uses
    (d <= 1024).  bf16 models wider than that: 2e-2 * sqrt(d / 1024) (tol_of): the error is the rounding of the GEMM
    inputs to bf16, a sum over d terms of independent roundings, and grows like sqrt(d) as the logits themselves do
    with weights of fixed variance;
  * an argmax entry is right iff oracle_logit[gpu_choice] >= max(oracle_logit) - 2*TOL:
    where the oracle's top-1/top-2 margin is at least 2*TOL this forces equality, inside
    the margin either token is a correct answer at that precision;
  * because near-ties may legitimately differ, multi-step runs are teacher-forced: after
    each step the GPU's proposals are overwritten with the oracle's, so both sides keep
    decoding the same sequence and every step is checked on its own.
"""
from __future__ import annotations

import numpy as np

import workloads as wl
from oracle import CombinedModel, scorers

TOL = {"f32": 1e-4, "bf16": 2e-2}


def tol_of(cfg):
    if cfg.dtype == "bf16" and cfg.d_model > 1024:
        return TOL["bf16"] * (cfg.d_model / 1024.0) ** 0.5
    return TOL[cfg.dtype]


def oracle_model(cfg, weights):
    return CombinedModel(weights, cfg.n_enc, cfg.n_dec, cfg.n_heads, cfg.k, cfg.ln_eps, cfg.local_q, cfg.local_m)


def gpu_context(cfg, weights, max_batch=None):
    from paper_1811_03115_amd import binding
    ctx = binding.Context(binding.config_from_workload(cfg, max_batch=max_batch))
    ctx.bpd_load_weights(weights)
    if cfg.local_q:
        ctx.bpd_set_local_attention(cfg.local_q, cfg.local_m)
    return ctx


def check_argmax(choice, z, tol, what=""):
    """choice: int array [...]; z: oracle logits [..., V]."""
    choice = np.asarray(choice)
    zc = np.take_along_axis(z, choice[..., None].astype(np.int64), axis=-1)[..., 0]
    zmax = z.max(axis=-1)
    bad = zc < zmax - 2 * tol
    assert not bad.any(), f"{what}: {int(bad.sum())} argmax entries outside tolerance; worst gap {float((zmax - zc).max())}"
    exact = choice == z.argmax(axis=-1)
    return float(exact.mean())


class LockStep:
    """Teacher-forced side-by-side decoding of one batch."""

    def __init__(self, cfg, weights, ctx, src, src_len, max_len, k=None, sample=None):
        self.cfg, self.ctx = cfg, ctx
        self.k = cfg.k if k is None else k
        self.B = src.shape[0]
        self.tol = tol_of(cfg)
        self.model = oracle_model(cfg, weights)
        self.sample = list(range(self.B)) if sample is None else list(sample)
        self.max_len = np.asarray(max_len)
        self.fns = {b: scorers(self.model, src[b, :src_len[b]]) for b in self.sample}
        self.prefix = {b: [] for b in self.sample}
        self.done = {b: False for b in self.sample}
        ctx.bpd_encode(src, src_len, max_len)
        # first invocation: proposals from the empty prefix
        P, A, j, fin = ctx.bpd_get_state()
        assert (j == 0).all() and (fin == 0).all()
        self.P = {}
        self.match = []
        for b in self.sample:
            z0 = self.fns[b][0]([])                                   # [k_max, V]
            self.match.append(check_argmax(P[b], z0, self.tol, f"first proposals b={b}"))
            self.P[b] = z0.argmax(-1).astype(np.int32)
        self._force(P)

    def _force(self, P_gpu):
        P = P_gpu.copy()
        for b in self.sample:
            P[b, :len(self.P[b])] = self.P[b]
        self.ctx.bpd_set_proposals(P)
        self.P_all = P

    def step(self, imposed=None, check_logits=True, two_phase=False, top_n=1):
        """One step on both sides; returns the accepted lengths.

        two_phase: the step runs with bpd_set_two_phase(True).  Where that mode is active (bf16, more than 16 block
        rows, k > 1) the table holds head 1 of every row and row k-hat only: those entries are checked against the
        oracle's logits and all the others must read -1.
        top_n > 1: top-n verification (Section 5.1) with bpd_set_top_n(top_n).  Proposal P_{i+1} has to be accepted
        where the oracle's p_1 logit of it at row i is at least 2*tol above the n-th best, and must not be where it is
        more than 2*tol below; between the two either decision is correct at this precision.
        """
        k, ctx, cfg = self.k, self.ctx, self.cfg
        zs = {}
        for b in self.sample:
            if not self.done[b]:
                zs[b] = self.fns[b][1](self.prefix[b], list(self.P[b][:k]))[:, :k]      # [k, k, V]
        if check_logits:
            lg = ctx.bpd_debug_step_logits(k).cpu().numpy()
            for b, z in zs.items():
                err = np.abs(lg[b] - z).max()
                assert err <= self.tol, f"logits b={b}: max abs err {err} > {self.tol}"
                self.max_logit_err = max(getattr(self, "max_logit_err", 0.0), float(err))
        import torch
        acc_t = torch.zeros(self.B, dtype=torch.int32, device="cuda")
        ctx.bpd_set_two_phase(two_phase)
        ctx.bpd_set_top_n(top_n)
        try:
            ctx.bpd_step(k, imposed, acc_t)
        finally:
            ctx.bpd_set_two_phase(False)
            ctx.bpd_set_top_n(1)
        acc = acc_t.cpu().numpy()
        P_gpu, A_gpu, j_gpu, fin_gpu = ctx.bpd_get_state()
        out_ids, out_len = ctx.bpd_get_output()
        partial_table = two_phase and cfg.dtype == "bf16" and self.B * k > 16 and k > 1
        for b in self.sample:
            if self.done[b]:
                assert acc[b] == 0 and fin_gpu[b] == 1
                continue
            z = zs[b]
            P = [int(t) for t in self.P[b][:k]]
            j = len(self.prefix[b])
            room = int(self.max_len[b]) - j

            def cut(kv):
                if cfg.eos_id >= 0 and cfg.eos_id in P[:kv]:
                    kv = P.index(cfg.eos_id) + 1
                return min(kv, room)

            # head 1 of every row is always there: it is what verification reads
            self.match.append(check_argmax(A_gpu[b, :k, 0], z[:, 0], self.tol, f"A column 1 b={b}"))
            if imposed is not None:
                lo = hi = int(np.clip(imposed[b], 1, k))
            elif top_n > 1:
                nth = np.sort(z[:, 0], axis=-1)[:, -top_n]                       # n-th best logit of p_1 per row
                zp = np.array([z[i - 1, 0, P[i]] for i in range(1, k)])         # p_1's logit of proposal i+1 at row i
                must = zp >= nth[:k - 1] + 2 * self.tol
                may = zp >= nth[:k - 1] - 2 * self.tol
                lo = 1 + (int(np.argmin(must)) if not must.all() else k - 1)
                hi = 1 + (int(np.argmin(may)) if not may.all() else k - 1)
            else:
                # exact verification against the GPU's own head-1 choices where those are
                # within tolerance, so that the integer decision is compared like with like
                lo = 1
                while lo < k and P[lo] == int(A_gpu[b, lo - 1, 0]):
                    lo += 1
                hi = lo
            assert cut(lo) <= acc[b] <= cut(hi), f"accepted length b={b}: gpu {acc[b]}, oracle {cut(lo)}..{cut(hi)}"
            k_hat = int(acc[b])
            assert k_hat >= 1
            if partial_table:
                self.match.append(check_argmax(A_gpu[b, k_hat - 1, :k], z[k_hat - 1], self.tol, f"A row k-hat b={b}"))
                rest = np.ones((k, k), bool)
                rest[:, 0] = False
                rest[k_hat - 1, :] = False
                assert (A_gpu[b, :k, :k][rest] == -1).all(), f"two-phase table b={b}: entries outside column 1 / row k-hat"
            else:
                self.match.append(check_argmax(A_gpu[b, :k, :k], z, self.tol, f"A table b={b}"))
            A = z.argmax(-1)
            eos = cfg.eos_id >= 0 and cfg.eos_id in P[:k_hat]
            self.prefix[b].extend(P[:k_hat])
            assert j_gpu[b] == len(self.prefix[b]) == out_len[b]
            assert out_ids[b, :out_len[b]].tolist() == self.prefix[b]
            assert (out_ids[b, out_len[b]:] == cfg.pad_id).all()
            self.done[b] = bool(eos or len(self.prefix[b]) >= self.max_len[b])
            assert bool(fin_gpu[b]) == self.done[b]
            # next proposals: row k-hat of the table on both sides
            assert P_gpu[b, :k].tolist() == A_gpu[b, k_hat - 1, :k].tolist()
            self.P[b] = A[k_hat - 1].astype(np.int32)
        self._force(P_gpu)
        return acc
