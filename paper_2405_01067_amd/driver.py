"""Algorithm 1 on one GPU: the phases of AB training for a stack of L linear layers and G emulated
groups, issued through the C ABI of the library.

This module holds control flow, the step schedule and pointer marshalling only; every tensor
operation of the method runs in the library's kernels:

    abDecomposition of every W with the cut-off rule          ab_factorize_batched
    group training (the A groups train A, the B groups B,     lr_linear_fwd_grouped, lr_linear_bwd_grouped (the
      the other factor frozen), learning-rate rebound           frozen factor's gradient skipped), ab_adamw_step
                                                                over the trained factors of all groups
                                                                and layers in one launch, ab_lr_rebound_scale
    A <- allReduce(A / worldSize), B likewise, W <- A B       ab_merge_batched over all layers (mean of the
                                                                G copies; W_out is the product of the means)

What belongs to the model and not to the method is supplied by the caller: the batches, the loss
gradient at the output of the last layer, and the full-rank data-parallel steps of the warm-up
and rebound phases (a callback that receives the dense weights, the step number inside the phase
and the learning-rate factor of the rebound).  The layers form a chain without activations:
the output of layer l is the input of layer l + 1.

Groups are emulated as G copies of the factors in one GPU's memory (at most eight per call of the
grouped entry points); a step issues, per layer, one grouped forward and one grouped backward for
all groups (lr_linear_fwd_grouped, lr_linear_bwd_grouped) and one optimiser launch for everything.
"""
from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence

from . import binding as abt


@dataclass(frozen=True)
class Schedule:
    """Step counts of the phases (Section "Hyperparameter considerations": warm-up 20 % of the
    training steps, numABSteps 3.33 %, full-rank rebound 0.25 numABSteps, learning-rate rebound
    0.5 numABSteps), rounded to whole steps, at least one each."""
    total_steps: int
    warmup_steps: int
    ab_steps: int
    rebound_steps: int
    lr_rebound_steps: int


def schedule(total_steps: int) -> Schedule:
    if total_steps < 1:
        raise abt.AbtError("total_steps must be positive")
    # integer arithmetic: 20 % = 1/5, 3.33 % = 1/30, rounded half up
    warm = max(1, (2 * total_steps + 5) // 10)
    ab = max(1, (2 * total_steps + 30) // 60)
    reb = max(1, (ab + 2) // 4)
    lr_reb = max(1, (ab + 1) // 2)
    return Schedule(total_steps, warm, ab, reb, lr_reb)


def group_target(group: int, groups: int) -> str:
    """Algorithm 1: the first half of the workers trains A, the second half B."""
    return "A" if group < (groups + 1) // 2 else "B"


class ABDriver:
    """Walks Algorithm 1 for `weights` (fp32 GPU matrices W_l [m_l, n_l] with n_{l+1} = m_l).

    batch(group, step) -> X [M, n_0] in the compute dtype; loss_grad(Y, group, step) -> dY [M, m_last]
    in the compute dtype; full_rank_step(weights, phase, i, lr_scale) trains the dense weights in place
    (phase is "warmup" or "rebound", i counts from 0 inside the phase).  `step` counts the steps of
    the whole run from 0.
    """

    def __init__(self, weights: Sequence, groups: int, tau: float, lr: float,
                 batch: Callable, loss_grad: Callable, full_rank_step: Optional[Callable] = None,
                 dtype=None, k_cap: Optional[int] = None, beta1: float = 0.9, beta2: float = 0.999,
                 eps: float = 1e-8, weight_decay: float = 0.01):
        torch = abt._torch()
        if not 1 <= groups <= abt.MAX_GROUPS:
            raise abt.AbtError(f"between 1 and {abt.MAX_GROUPS} groups")
        self.torch = torch
        self.W = list(weights)
        for l, w in enumerate(self.W):
            abt._dev_tensor(w, f"W[{l}]")
            if w.dtype != torch.float32 or w.dim() != 2:
                raise abt.AbtError("weights must be fp32 matrices")
            if l and w.shape[1] != self.W[l - 1].shape[0]:
                raise abt.AbtError("layer l + 1 must take the output of layer l")
        self.G = groups
        self.tau, self.lr = float(tau), float(lr)
        self.hyper = dict(beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay)
        self.batch, self.loss_grad, self.full_rank_step = batch, loss_grad, full_rank_step
        self.on_synchronize: Optional[Callable] = None   # called with the driver after every synchronisation
        self.dtype = dtype or torch.float32
        if self.dtype not in (torch.float32, torch.bfloat16):
            raise abt.AbtError("compute dtype must be float32 or bfloat16")
        self.k_cap = k_cap
        self.step = 0                  # steps of the whole run done so far
        self.ranks: List[int] = []     # selected by the cut-off rule at the last decomposition
        self.log: List[tuple] = []     # (phase, first step, steps) in the order walked

    # ------------------------------------------------------------------ phases
    def full_rank_phase(self, phase: str, steps: int, lr_rebound_steps: int):
        """Traditional full-rank data-parallel training: the caller's callback, `steps` times, under
        the learning-rate rebound that follows a change of the parameters' shape."""
        for i in range(steps):
            if self.full_rank_step is not None:
                self.full_rank_step(self.W, phase, i, abt.lr_rebound_scale(i, lr_rebound_steps))
            self.step += 1
        self.log.append((phase, self.step - steps, steps))

    def decompose(self):
        """A, B <- abDecomposition(W) for every layer with the cut-off rule (Eq. 3), then one copy of
        the factors per group.  The layer and merge kernels take ranks in steps of 32: the factors
        keep the zero columns / rows that the decomposition leaves beyond the selected rank up to the
        next multiple of 32 (they stay zero under training: their gradients and their weight decay
        vanish, and the products A B do not see them)."""
        torch = self.torch
        caps = []
        for w in self.W:
            cap = min(w.shape) if self.k_cap is None else min(self.k_cap, min(w.shape))
            if self.dtype == torch.bfloat16:
                cap = min(384, cap)
            cap = cap // 32 * 32
            if cap < 32:
                raise abt.AbtError("ranks come in steps of 32: min(m, n) and k_cap must be 32 or more")
            caps.append(cap)
        outs = abt.ab_factorize_batched([dict(W=w, tau=self.tau, k_cap=c) for w, c in zip(self.W, caps)])
        self.ranks = [int(o["k"].item()) for o in outs]
        self.A, self.B, self.widths = [], [], []
        for o, k, cap in zip(outs, self.ranks, caps):
            kk = min(cap, (k + 31) // 32 * 32)
            self.widths.append(kk)
            a0, b0 = o["A"][:, :kk].contiguous(), o["B"][:kk, :].contiguous()
            self.A.append([a0.clone() for _ in range(self.G)])
            self.B.append([b0.clone() for _ in range(self.G)])
        self.log.append(("decompose", self.step, 0))
        return self.ranks

    def group_phase(self, steps: int, lr_rebound_steps: int):
        """Independent subgroup training: every group runs forward and backward through the chain of
        factored layers on its own batch and trains its target factor; the other factor is frozen."""
        torch = self.torch
        L, G = len(self.W), self.G
        low = self.dtype != torch.float32
        # optimiser state of the trained factors starts afresh: the parameters have changed shape
        trained = [[(self.A if group_target(g, G) == "A" else self.B)[l][g] for l in range(L)] for g in range(G)]
        grads = [[torch.empty_like(t) for t in row] for row in trained]
        mom = [[torch.zeros_like(t) for t in row] for row in trained]
        var = [[torch.zeros_like(t) for t in row] for row in trained]
        # the layer kernels read the factors in the compute dtype; fp32 masters stay in self.A / self.B
        if low:
            Ac = [[torch.empty_like(a, dtype=self.dtype) for a in row] for row in self.A]
            Bc = [[torch.empty_like(b, dtype=self.dtype) for b in row] for row in self.B]
            self._round_copies([x for row in self.A + self.B for x in row], [x for row in Ac + Bc for x in row])
        else:
            Ac, Bc = self.A, self.B
        table = []
        for g in range(G):
            for l in range(L):
                entry = dict(param=trained[g][l], grad=grads[g][l], exp_avg=mom[g][l], exp_avg_sq=var[g][l])
                if low:
                    entry["param_bf16"] = (Ac if group_target(g, G) == "A" else Bc)[l][g]
                table.append(entry)
        plan = abt.AdamwPlan(table)
        targets = [group_target(g, G) for g in range(G)]
        for i in range(steps):
            # forward of every layer for all groups in one grouped call, then the backward likewise
            acts = [[self.batch(g, self.step) for g in range(G)]]
            Ts = []
            for l in range(L):
                outs = abt.lr_linear_fwd_grouped([dict(X=acts[l][g], A=Ac[l][g], B=Bc[l][g]) for g in range(G)])
                acts.append([y for y, _ in outs])
                Ts.append([t for _, t in outs])
            dY = [self.loss_grad(acts[L][g], g, self.step) for g in range(G)]
            for l in reversed(range(L)):
                outs = abt.lr_linear_bwd_grouped(
                    [dict(dY=dY[g], X=acts[l][g], T=Ts[l][g], A=Ac[l][g], B=Bc[l][g], dX=(l > 0),
                          dA=grads[g][l] if targets[g] == "A" else None,
                          dB=grads[g][l] if targets[g] == "B" else None) for g in range(G)])
                dY = [o[0] for o in outs]
            # one optimiser launch for the trained factors of all groups and layers
            abt.ab_adamw_step(plan, step=i + 1, lr=self.lr, lr_scale=abt.lr_rebound_scale(i, lr_rebound_steps),
                              **self.hyper)
            self.step += 1
        self.log.append(("group", self.step - steps, steps))

    def _round_copies(self, masters, copies):
        """copies <- masters rounded to the compute dtype, by the optimiser kernel itself: a step of
        size zero on zero gradients and zero moments leaves the parameter as it is and writes its
        rounded copy."""
        torch = self.torch
        n = max(x.numel() for x in masters)
        zero = [torch.zeros(n, dtype=torch.float32, device=masters[0].device) for _ in range(3)]
        table = [dict(param=p, grad=zero[0][:p.numel()], exp_avg=zero[1][:p.numel()], exp_avg_sq=zero[2][:p.numel()],
                      param_bf16=c) for p, c in zip(masters, copies)]
        # the moments are shared by all entries and stay zero: (1 - beta) * 0 + beta * 0
        abt.ab_adamw_step(table, step=1, lr=0.0, lr_scale=0.0, **self.hyper)

    def synchronize(self):
        """A <- allReduce(A / worldSize), B <- allReduce(B / worldSize), W <- A B for every layer, in
        one batched call; the same call re-factorises the merged weight with the cut-off rule and its
        ranks are recorded (merged_ranks)."""
        layers = [dict(A_copies=self.A[l], B_copies=self.B[l], tau=self.tau, W_out=self.W[l])
                  for l in range(len(self.W))]
        outs = abt.ab_merge_batched(layers)
        self.merged_ranks = [int(o["k"].item()) for o in outs]
        self.merged = outs
        self.A = self.B = None          # the network is full rank again
        self.log.append(("synchronize", self.step, 0))
        if self.on_synchronize is not None:
            self.on_synchronize(self)
        return self.merged_ranks

    # ------------------------------------------------------------------ the whole procedure
    def run(self, total_steps: int) -> Schedule:
        s = schedule(total_steps)
        self.full_rank_phase("warmup", min(s.warmup_steps, total_steps), 0)
        while self.step < total_steps:
            self.decompose()
            self.group_phase(min(s.ab_steps, total_steps - self.step), s.lr_rebound_steps)
            self.synchronize()
            left = total_steps - self.step
            if left > 0:
                self.full_rank_phase("rebound", min(s.rebound_steps, left), s.lr_rebound_steps)
        return s
