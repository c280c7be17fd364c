"""Sequencing of the library calls for a multi-step run (no arithmetic here).

State of the method on the device: alpha (fp32[B]), r (fp64[B]), the last update
norm (fp64[B]) and the clip counts (uint64[n]).  `start` seeds the recurrence
with the norm of the exact first step (Algorithm 1, init line); each `step_*`
runs one IntSGD step on the current stream and chains the next alpha without
touching the host.
"""
import torch

from . import binding as B


class Stepper:
    def __init__(self, desc: B.Desc, *, eta, beta=0.9, eps=1e-8, device="cuda"):
        self.desc = desc
        self.eta, self.beta, self.eps = float(eta), float(beta), float(eps)
        nb = desc.num_blocks
        self.alpha = torch.zeros(nb, dtype=torch.float32, device=device)
        self.r = torch.zeros(nb, dtype=torch.float64, device=device)
        self.norm_sq = torch.zeros(nb, dtype=torch.float64, device=device)
        self.sat_count = torch.zeros(desc.n, dtype=torch.int64, device=device)  # uint64 bits
        self.workspace = B.new_workspace(desc, device)
        B.intsgd_prepare(desc)

    def start(self, first_normsq, r0=None):
        """r_0 = 0 (or r0) and ||x^1 - x^0||^2 given: computes alpha_1."""
        self.norm_sq.copy_(torch.as_tensor(first_normsq, dtype=torch.float64))
        if r0 is None:
            self.r.zero_()
        else:
            self.r.copy_(torch.as_tensor(r0, dtype=torch.float64))
        self.next_alpha()

    def next_alpha(self, stream=None, eta=None):
        """a8 on the device state; eta = the stepsize of the step that will USE the new alpha."""
        B.intsgd_next_alpha(self.desc, self.norm_sq, self.r, self.beta, self.eps,
                            self.eta if eta is None else eta, self.alpha, stream)

    def step_fused(self, grads, x, k, stream=None, chain_alpha=True, eta_next=None):
        """The whole step a1-a8 in one call (chain_alpha=False: stop after a7).
        grads: list of n device tensors; x updated in place.  Under a stepsize schedule set
        self.eta to eta_k before the call and pass eta_next = eta_{k+1}."""
        self.desc.step = k
        if chain_alpha:
            B.intsgd_step_fused_next_alpha(self.desc, grads, self.alpha, self.eta, x, self.r,
                                           self.beta, self.eps, self.norm_sq, self.sat_count,
                                           self.workspace, stream, eta_next=eta_next)
        else:
            B.intsgd_step_fused(self.desc, grads, self.alpha, self.eta, x, self.norm_sq,
                                self.sat_count, self.workspace, stream)

    def step_two_pass(self, grads, x, k, sum_buf, stream=None, chain_alpha=True, eta_next=None):
        """F1 (compress + aggregate) then F2 (decode + update + norm) then a8."""
        self.desc.step = k
        B.intsgd_compress_sum(self.desc, grads, self.alpha, sum_buf, self.sat_count,
                              self.workspace, stream)
        B.intsgd_decode_update_norm(self.desc, sum_buf, self.alpha, self.eta, x, self.norm_sq,
                                    self.workspace, stream)
        if chain_alpha:
            self.next_alpha(stream, eta_next)

    def step_unfused(self, grads, x, k, q_bufs, sum_buf, x_old, stream=None, chain_alpha=True,
                     eta_next=None):
        """a1-a3, a4, a5-a6, a7, a8 as five separate calls (x_old: scratch copy of x)."""
        self.desc.step = k
        B.intsgd_compress(self.desc, grads, self.alpha, q_bufs, self.sat_count, self.workspace,
                          stream)
        B.intsgd_int_sum(self.desc, q_bufs, sum_buf, stream)
        if stream is None:
            x_old.copy_(x)
        else:       # the copy must be ordered with the library calls: same stream
            with torch.cuda.stream(torch.cuda.ExternalStream(int(stream))):
                x_old.copy_(x)
        B.intsgd_decode_update(self.desc, sum_buf, self.alpha, self.eta, x, None, stream)
        B.intsgd_update_norm(self.desc, x, x_old, self.norm_sq, self.workspace, stream)
        if chain_alpha:
            self.next_alpha(stream, eta_next)

    def step_momentum(self, grads, x, m, k, mu, weight_decay, stream=None, chain_alpha=True,
                      eta_next=None):
        """The whole step with the momentum / weight-decay update (m: device fp32[d] state)."""
        self.desc.step = k
        B.intsgd_step_momentum(self.desc, grads, self.alpha, self.eta, mu, weight_decay, x, m,
                               self.r if chain_alpha else None, self.beta, self.eps, self.norm_sq,
                               self.sat_count, self.workspace, stream, eta_next=eta_next)
