"""Sequencing of the library calls for one workload: the loop of Algorithm 1 as
seen from one GPU, where the K workers are K device-resident accumulators.

This module allocates device memory through PyTorch, uploads host-generated
inputs, and issues abs_accumulate / abs_sync_update / abs_swap_buffers in the
order of Algorithm 1.  It computes nothing itself.
"""
import numpy as np
import torch

import abs_workloads as wl

from . import ABS_BF16, ABS_F32, Context, Layout, TensorSet


def _upload(a):
    """numpy -> device tensor; uint16 bf16 bit patterns travel as int16."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


class DeviceRun:
    """Device state and call sequence for one workload.

    overlap=True : accumulation and sync-update on different streams;
    overlap=False: both on one stream, in program order;
    acc_streams=n: the K workers' accumulations spread over n streams;
    lam          : coefficient of the delayed gradient compensation (None: off);
    lam_from_momentum: take x_t - x_{t-1} from the momentum instead of a stored x_{t-1};
    adam         : (beta1, beta2, eps) switches the update rule to Adam;
    lars         : trust coefficient eta switches it to LARS (one layer per tensor);
    batched=True : a worker's m_k gradients of a step go in one abs_accumulate_batch
                   call (same bits, the accumulator is read and written once);
    step_fold=f  : Step 2 of all K workers goes in ONE abs_ctx_accumulate_step call per
                   iteration, a launch folding at most f gradients per worker (f = 1: one
                   launch per round of gradients, the traffic of single calls; f = 8: the
                   batched traffic, normally one launch).
    """

    def __init__(self, w, x0, pool, schedule, overlap=True, P=None, acc_streams=1, lam=None, batched=False,
                 adam=None, lars=None, lam_from_momentum=False, step_fold=None):
        self.w = w
        self.P = int(w.P if P is None else P)
        self.K = w.K
        self.m = np.asarray(schedule)
        self.gdt = ABS_BF16 if w.grad_dtype == "bf16" else ABS_F32
        self.ragged = w.tensor_sizes is not None
        self.lam = None if lam is None else float(lam)   # delayed gradient compensation coefficient
        self.dcm = self.lam is not None and bool(lam_from_momentum)      # no x_{t-1} buffer then
        self.batched = bool(batched)                     # one accumulate launch per worker and step
        self.step_fold = None if step_fold is None else int(step_fold)   # one accumulate call per step
        self.adam = None if adam is None else tuple(float(t) for t in adam)   # (beta1, beta2, eps)
        self.adam_step = 0                               # applied Adam updates so far
        self.lars = None if lars is None else float(lars)   # LARS trust coefficient eta (ragged layouts)
        self._streams = [torch.cuda.Stream(device=torch.device("cuda:0")) for _ in range(9)]
        self.ctx = None
        if not self.ragged:
            self.x = _upload(np.ascontiguousarray(x0, dtype=np.float32))
            self.v = torch.zeros_like(self.x)
            self.acc = [[torch.empty_like(self.x) for _ in range(self.K)] for _ in range(2)]
            # stale garbage on purpose: accumulation must overwrite, never rely on zeros
            for gen in self.acc:
                for a in gen:
                    a.fill_(float("nan"))
            self.pool = [_upload(g) for g in pool]
            self.pool_ptr = [g.data_ptr() for g in self.pool]
            self.xp = self.x.clone() if (self.lam is not None and not self.dcm) else None   # x_{t-1}; starts equal to x_0
            if self.adam is not None:
                self.xp = torch.zeros_like(self.x)                        # second moment
            torch.cuda.synchronize()
            self.x_arg, self.v_arg = self.x.data_ptr(), self.v.data_ptr()
            self.xp_arg = self.xp.data_ptr() if self.xp is not None else None
        else:
            sizes = list(w.tensor_sizes)
            off = wl.tensor_offsets(sizes)
            self.layout = Layout(sizes)

            def split(a):
                # one separate allocation per tensor, as a framework would hold them
                return [_upload(np.ascontiguousarray(a[off[t]:off[t + 1]])) for t in range(len(sizes))]

            self.x_t = split(np.ascontiguousarray(x0, dtype=np.float32))
            self.v_t = [torch.zeros_like(t) for t in self.x_t]
            self.acc_t = [[[torch.full_like(t, float("nan")) for t in self.x_t]
                           for _ in range(self.K)] for _ in range(2)]
            self.pool_t = [split(g) for g in pool]
            torch.cuda.synchronize()
            self.x_set = TensorSet(self.layout, self.x_t)
            self.v_set = TensorSet(self.layout, self.v_t)
            self.acc_sets = [[TensorSet(self.layout, self.acc_t[g][k]) for k in range(self.K)]
                             for g in range(2)]
            self.pool_sets = [TensorSet(self.layout, p, dtype=self.gdt) for p in self.pool_t]
            self.x_arg, self.v_arg = self.x_set, self.v_set
            self.xp_arg = None
            if (self.lam is not None and not self.dcm) or self.adam is not None:
                self.xp_t = [t.clone() if self.adam is None else torch.zeros_like(t) for t in self.x_t]
                torch.cuda.synchronize()
                self.xp_arg = TensorSet(self.layout, self.xp_t)
        if self.lars is not None:
            if not self.ragged:
                raise ValueError("LARS works per tensor: the workload needs a ragged layout")
            self.gbar_t = [torch.zeros_like(t) for t in self.x_t]        # workspace for the averaged gradient
            torch.cuda.synchronize()
            self.gbar_set = TensorSet(self.layout, self.gbar_t)
        self.configure_streams(overlap, acc_streams)
        self.lr, self.mu, self.wd = float(w.lr), float(w.mu), float(w.wd)
        self.applied = []
        self.count_history = []

    def configure_streams(self, overlap, acc_streams=1):
        """(Re)build the double-buffer context over the same device buffers with
        another stream plan.  Counts restart at zero (as at creation), so the
        next step applies nothing; parameters and momentum carry on."""
        torch.cuda.synchronize()
        if self.ctx is not None:
            self.ctx.close()
        acc_streams = max(1, min(int(acc_streams), 8))
        self.s_acc = self._streams[0]
        self.s_upd = self._streams[8] if overlap else self.s_acc
        self.acc_streams = self._streams[:acc_streams]
        self.stream_plan = {"overlap": bool(overlap), "acc_streams": acc_streams}
        if not self.ragged:
            self.ctx = Context(self.acc[0], self.acc[1], self.s_acc, self.s_upd, P=self.P)
        else:
            self.ctx = Context(self.acc_sets[0], self.acc_sets[1], self.s_acc, self.s_upd,
                               layout=self.layout)
        if acc_streams > 1:
            self.ctx.abs_set_accumulate_streams(self.acc_streams)

    def grad_arg(self, r):
        return self.pool_sets[r] if self.ragged else self.pool_ptr[r]

    def plan_step(self, t, pool_size=None):
        """[(worker, gradient argument)] for step t, in issue order."""
        R = len(self.pool_sets if self.ragged else self.pool) if pool_size is None else pool_size
        calls = []
        for k in range(self.K):
            for j in range(int(self.m[t, k])):
                calls.append((k, self.grad_arg(wl.pool_index(self.w, t, k, j, R))))
        return calls

    def sync_update(self):
        """Step 1 + update on the delayed generation (compensated when lam is set,
        Adam when adam is set: v is then the first moment, xp the second)."""
        if self.lars is not None:
            return self.ctx.abs_sync_update_lars(self.x_arg, self.v_arg, self.gbar_set, self.lr, self.mu,
                                                 self.wd, self.lars)
        if self.adam is not None:
            b1, b2, eps = self.adam
            ok = self.ctx.abs_sync_update_adam(self.x_arg, self.v_arg, self.xp_arg, self.lr, b1, b2, eps,
                                               self.wd, self.adam_step + 1)
            if ok:
                self.adam_step += 1
            return ok
        if self.lam is None:
            return self.ctx.abs_sync_update(self.x_arg, self.v_arg, self.lr, self.mu, self.wd)
        if self.dcm:
            return self.ctx.abs_sync_update_dcm(self.x_arg, self.v_arg, self.lr, self.mu, self.wd, self.lam)
        return self.ctx.abs_sync_update_dc(self.x_arg, self.xp_arg, self.v_arg, self.lr, self.mu, self.wd,
                                           self.lam)

    def accumulate(self, calls):
        """Step 2 of all workers for one iteration, issued the way this run was set up.
        Returns the number of kernel launches it took."""
        ctx, n, gdt = self.ctx, self.w.n, self.gdt
        if self.step_fold is not None:
            # plan_step lists the calls worker by worker, which is the order the step call takes
            m = [0] * self.K
            for k, _ in calls:
                m[k] += 1
            ctx.abs_accumulate_step([g for _, g in calls], m, [n] * len(calls), fold=self.step_fold,
                                    grad_dtype=gdt)
            return -(-max(m) // self.step_fold) * -(-self.K // 16)
        if not self.batched:
            for k, g in calls:
                ctx.abs_accumulate(k, g, n, grad_dtype=gdt)
            return len(calls)
        per_worker = {}
        for k, g in calls:
            per_worker.setdefault(k, []).append(g)
        for k, gs in per_worker.items():
            ctx.abs_accumulate_batch(k, gs, [n] * len(gs), grad_dtype=gdt)
        return sum(-(-len(gs) // 8) for gs in per_worker.values())

    def step(self, t, calls=None):
        """One iteration of Algorithm 1: Step 1 + update on the delayed generation,
        Step 2 (accumulation) on the current one, then the swap."""
        applied = self.sync_update()
        self.accumulate(self.plan_step(t) if calls is None else calls)
        self.ctx.abs_swap_buffers()
        return applied

    def run(self, steps, record_counts=True):
        for t in range(steps):
            self.applied.append(self.step(t))
            if record_counts:
                self.count_history.append(self.ctx.counts(1))   # just-finished generation
        torch.cuda.synchronize()

    def read_state(self):
        torch.cuda.synchronize()
        if not self.ragged:
            return self.x.cpu().numpy(), self.v.cpu().numpy()
        return (np.concatenate([t.cpu().numpy() for t in self.x_t]),
                np.concatenate([t.cpu().numpy() for t in self.v_t]))

    def read_second_state(self):
        """The rule's second state vector: x_{t-1} (compensation) or Adam's second moment."""
        torch.cuda.synchronize()
        if not self.ragged:
            return self.xp.cpu().numpy()
        return np.concatenate([t.cpu().numpy() for t in self.xp_t])

    def read_state_at(self, idx):
        """x and v at flat element indices idx (ragged: indices into the concatenation)."""
        torch.cuda.synchronize()
        if not self.ragged:
            i = torch.from_numpy(np.asarray(idx)).cuda()
            return self.x[i].cpu().numpy(), self.v[i].cpu().numpy()
        off = wl.tensor_offsets(self.w.tensor_sizes)
        idx = np.asarray(idx)
        tens = np.searchsorted(off, idx, side="right") - 1
        xs = np.empty(idx.size, dtype=np.float32)
        vs = np.empty(idx.size, dtype=np.float32)
        for t in np.unique(tens):
            sel = np.nonzero(tens == t)[0]
            loc = torch.from_numpy(idx[sel] - off[t]).cuda()
            xs[sel] = self.x_t[t][loc].cpu().numpy()
            vs[sel] = self.v_t[t][loc].cpu().numpy()
        return xs, vs

    def close(self):
        self.ctx.close()
