"""A torch.optim-shaped front end of the C library, for callers that hold ``torch.nn.Parameter``s.

Bookkeeping only (which matrix, which seed, which step): every arithmetic step runs in the HIP
kernels behind ``flora.py``.  Two ways to drive it:

* grouped: ``opt.step()`` after ``backward()`` -- one grouped launch per entry point for the
  whole parameter set;
* layer by layer: ``opt.attach()`` registers a post-accumulate-grad hook on every parameter, so
  a weight is updated the moment its gradient exists and the gradient is freed at once (the
  layer-wise updating the paper combines Flora with in its appendix on memory profiling).

Schedules follow the paper's two algorithms:
  ``tau`` micro-batches per update (Algorithm 1: one projection per accumulation cycle, the
  accumulator is decompressed with 1/tau and reset); ``beta`` > 0 turns the state into a
  compressed momentum (Algorithm 2: EMA line, projection resampled every ``kappa`` updates with
  the state moved to the new projection).  With both, every micro-batch is compressed straight
  into the momentum, b = (1 - beta) / tau, which by linearity is Algorithm 2 on the mean
  gradient of the cycle.

``state_dict()`` / ``load_state_dict()`` carry the compressed states together with the seeds and
counters that stand for the projections (the paper's point that only the seed is kept), so a resumed
run continues bit for bit.

Only 2-D parameters, fp32 or bf16, are accepted (the paper projects the attention and feed-forward
weight matrices).  Gradients may be fp32 or bf16 at every rank; at ranks 64/128/256 bf16 gradients take
the fastest kernel (``param.grad_dtype = torch.bfloat16`` makes autograd produce them).
"""
from __future__ import annotations

from typing import Iterable, Optional

from . import flora


class Flora:
    def __init__(self, params: Iterable, r: int, lr: Optional[float] = 1e-3, *, tau: int = 1, beta: float = 0.0,
                 kappa: int = 1000, rule: str = "sgd", seed: int = 0, eps1: float = 1e-30, eps2: float = 1e-3,
                 clip_d: float = 1.0, scale_parameter: Optional[bool] = None):
        """rule: "sgd", "adafactor" (factored second moment) or "unfactored".
        lr=None with an Adafactor rule selects the published relative step size and parameter
        scaling; a number is a fixed learning rate (parameter scaling then only if asked for)."""
        import torch
        self._torch = torch
        self.params = list(params)
        if not self.params:
            raise ValueError("no parameters")
        if rule not in ("sgd", "adafactor", "unfactored"):
            raise ValueError("rule must be sgd, adafactor or unfactored")
        if rule == "sgd" and lr is None:
            raise ValueError("the sgd rule needs a learning rate")
        if tau < 1 or kappa < 1 or not (0.0 <= beta < 1.0):
            raise ValueError("tau >= 1, kappa >= 1, 0 <= beta < 1")
        for p in self.params:
            if p.dim() != 2 or p.dtype not in (torch.float32, torch.bfloat16) or not p.is_cuda or not p.is_contiguous():
                raise ValueError("parameters must be contiguous 2-D fp32 or bf16 CUDA tensors")
        if len({p.dtype for p in self.params}) != 1:
            raise ValueError("all parameters must have one dtype")
        self.wdt = flora.F32 if self.params[0].dtype == torch.float32 else flora.BF16
        self.r, self.lr, self.tau, self.beta, self.kappa, self.rule = r, lr, tau, beta, kappa, rule
        self.global_seed = seed
        self.eps1, self.eps2, self.clip_d = eps1, eps2, clip_d
        self.scale_parameter = (lr is None) if scale_parameter is None else bool(scale_parameter)
        self.shapes = [(p.shape[0], p.shape[1]) for p in self.params]
        count = len(self.params)
        dev = self.params[0].device
        self.state = [torch.zeros((n, r), device=dev, dtype=torch.float32) for n, _ in self.shapes]
        self.row_stat = self.col_stat = self.second = self.sumsq = None
        if rule == "adafactor":
            self.row_stat = [torch.zeros(n, device=dev) for n, _ in self.shapes]
            self.col_stat = [torch.zeros(m, device=dev) for _, m in self.shapes]
        if rule == "unfactored":
            self.second = [torch.zeros((n, m), device=dev) for n, m in self.shapes]
        if rule != "sgd":
            self._sumsq_buf = torch.zeros((count, 4), device=dev)
            self.sumsq = [self._sumsq_buf[i] for i in range(count)]
        # per-matrix counters: micro-batches seen in the current cycle, updates done, resamples
        self.micro = [0] * count
        self.updates = [0] * count
        self.epoch = [0] * count
        self.seed = [flora.derive_seed(seed, l, 0) for l in range(count)]
        self._handles = []
        self._sumsq_ready = False
        # what one optimizer step moves through the update passes, for calls that cover only part of it
        per = self.params[0].element_size() + (4 if rule == "unfactored" else 0)
        self.step_weight_mib = sum(n * m for n, m in self.shapes) * per / 2.0 ** 20

    # ------------------------------------------------------------------ descriptors
    def _descriptors(self, idx):
        ps = [self.params[l] for l in idx]

        def pick(xs):
            return [xs[l] for l in idx]

        return flora.matrices([self.shapes[l] for l in idx], grads=[p.grad for p in ps], weights=ps,
                              states=pick(self.state),
                              row_stats=pick(self.row_stat) if self.row_stat else None,
                              col_stats=pick(self.col_stat) if self.col_stat else None,
                              second_moments=pick(self.second) if self.second else None,
                              weight_sumsqs=pick(self.sumsq) if self.sumsq else None,
                              seeds=[self.seed[l] for l in idx], seeds_next=[self.seed[l] for l in idx])

    def _grad_dtype(self, idx):
        torch = self._torch
        dts = {self.params[l].grad.dtype for l in idx}
        if len(dts) != 1:
            raise ValueError("all gradients of one call must have one dtype")
        dt = dts.pop()
        if dt == torch.float32:
            return flora.F32
        if dt == torch.bfloat16:
            return flora.BF16
        raise ValueError("gradients must be fp32 or bf16")

    def _update_struct(self, t: int, last_of_cycle_alpha: float, zero_after: bool):
        if self.rule == "sgd":
            return flora.sgd_update(self.lr, last_of_cycle_alpha, zero_state_after=zero_after,
                                    step_weight_mib=self.step_weight_mib)
        rho, beta2 = flora.adafactor_schedule(t)
        lr = rho if self.lr is None else self.lr
        mk = flora.factored_update if self.rule == "adafactor" else flora.unfactored_update
        return mk(lr, last_of_cycle_alpha, beta2, self.eps1, self.clip_d, zero_state_after=zero_after,
                  scale_parameter=self.scale_parameter, eps2=self.eps2, step_weight_mib=self.step_weight_mib)

    # ------------------------------------------------------------------ one call for a set of matrices
    def _run(self, idx, stream=None):
        """Consumes the gradients of matrices `idx` (all at the same point of their schedules)."""
        if stream is None:
            stream = self._torch.cuda.current_stream()
        l0 = idx[0]
        micro, t = self.micro[l0], self.updates[l0]
        if any(self.micro[l] != micro or self.updates[l] != t for l in idx):
            raise RuntimeError("matrices of one call must be at the same step")
        if any(self.params[l].grad is None for l in idx):
            raise RuntimeError("a parameter has no gradient")
        if self.sumsq is not None and self.scale_parameter and not self._sumsq_ready:
            flora.weight_sumsq(self._descriptors(list(range(len(self.params)))), self.wdt, stream)
            self._sumsq_ready = True
        gdt = self._grad_dtype(idx)
        momentum = self.beta > 0.0
        first, last = micro == 0, micro == self.tau - 1
        transfer = False
        if momentum and first and t % self.kappa == 0:
            # resample (Algorithm 2): at t = 0 the state is all zero and the new seed is simply used
            for l in idx:
                self.epoch[l] += 1
            new = [flora.derive_seed(self.global_seed, l, self.epoch[l]) for l in idx]
            transfer = t > 0
        mats = self._descriptors(idx)
        if momentum and first and t % self.kappa == 0:
            f = flora.fields(mats)
            f["seed_next"][:] = new
            if not transfer:
                f["seed"][:] = new
            for l, s in zip(idx, new):
                self.seed[l] = s
        if momentum:
            a = self.beta if first else 1.0
            b = (1.0 - self.beta) / self.tau
        else:
            # Algorithm 1: the accumulator starts each cycle at zero, so the cycle's first
            # micro-batch overwrites it
            a, b = (0.0 if first else 1.0), 1.0
        if last:
            upd = self._update_struct(t + 1, 1.0 if momentum else 1.0 / self.tau, zero_after=False)
            flora.fused_step(mats, self.r, gdt, self.wdt, a, b, transfer, upd, stream)
        else:
            if transfer:
                flora.momentum_transfer(mats, self.r, stream)
                flora.fields(mats)["seed"][:] = [self.seed[l] for l in idx]
            flora.compress(mats, self.r, gdt, a, b, stream)
        for l in idx:
            self.micro[l] = 0 if last else micro + 1
            if last:
                self.updates[l] += 1
                if not momentum:
                    # Algorithm 1: a new projection for the next accumulation cycle
                    self.epoch[l] += 1
                    self.seed[l] = flora.derive_seed(self.global_seed, l, self.epoch[l])

    # ------------------------------------------------------------------ public
    def step(self, stream=None):
        """Grouped: consumes every parameter's gradient (one micro-batch)."""
        self._run(list(range(len(self.params))), stream)

    def zero_grad(self, set_to_none: bool = True):
        for p in self.params:
            if set_to_none:
                p.grad = None
            elif p.grad is not None:
                p.grad.zero_()

    def attach(self):
        """Layer by layer: each parameter is stepped from a hook as soon as its gradient has been
        accumulated, and the gradient is released."""
        if self._handles:
            return
        for l, p in enumerate(self.params):
            def hook(param, l=l):
                self._run([l])
                param.grad = None
            self._handles.append(p.register_post_accumulate_grad_hook(hook))

    def detach(self):
        for h in self._handles:
            h.remove()
        self._handles = []

    # ------------------------------------------------------------------ checkpoints
    def state_dict(self):
        """Everything a resumed run needs: the compressed states, the second-moment statistics and,
        because the projections are never stored, the seeds and counters that define them."""
        def clone(xs):
            return None if xs is None else [x.detach().clone() for x in xs]
        return {
            "config": {"r": self.r, "tau": self.tau, "beta": self.beta, "kappa": self.kappa, "rule": self.rule,
                       "seed": self.global_seed, "shapes": [tuple(s) for s in self.shapes]},
            "state": clone(self.state), "row_stat": clone(self.row_stat), "col_stat": clone(self.col_stat),
            "second": clone(self.second),
            "sumsq": None if self.sumsq is None else self._sumsq_buf.detach().clone(),
            "micro": list(self.micro), "updates": list(self.updates), "epoch": list(self.epoch),
            "matrix_seed": [int(x) for x in self.seed], "sumsq_ready": self._sumsq_ready,
        }

    def load_state_dict(self, sd):
        cfg = sd["config"]
        mine = {"r": self.r, "tau": self.tau, "beta": self.beta, "kappa": self.kappa, "rule": self.rule,
                "seed": self.global_seed, "shapes": [tuple(s) for s in self.shapes]}
        if {k: (list(map(tuple, v)) if k == "shapes" else v) for k, v in cfg.items()} != mine:
            raise ValueError("checkpoint was written by an optimizer with a different configuration")

        def put(dst, src):
            if (dst is None) != (src is None):
                raise ValueError("checkpoint does not match the update rule")
            if dst is not None:
                for d, x in zip(dst, src):
                    d.copy_(x)
        put(self.state, sd["state"])
        put(self.row_stat, sd["row_stat"])
        put(self.col_stat, sd["col_stat"])
        put(self.second, sd["second"])
        if self.sumsq is not None:
            self._sumsq_buf.copy_(sd["sumsq"])
        self.micro, self.updates, self.epoch = list(sd["micro"]), list(sd["updates"]), list(sd["epoch"])
        self.seed = [int(x) for x in sd["matrix_seed"]]
        self._sumsq_ready = bool(sd["sumsq_ready"])
