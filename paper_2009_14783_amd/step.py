"""One worker's training step driven through the C ABI (buffer ownership and call order only).

`Worker` owns the device buffers (torch tensors: fp32 master weights, Adam moments, the flat
fp32 gradient buffer G, the low-precision weight copy, activation arena, workspace) and issues
the hs_* calls in the order of the paper's step: forward, loss with its weight, backward,
delayed-update accumulation, normalisation by the global sample count, Adam.  No arithmetic of
the method happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as hs


class Worker:
    def __init__(self, model: dict, compute: str, theta0: np.ndarray, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.compute = hs.HS_BF16 if compute == "bf16" else hs.HS_FP32
        self.cfg = hs.make_cfg(model["n_layers"], model["hidden"], model["n_heads"], model["ffn"], model["vocab"],
                               model["max_pos"], model.get("ln_eps", 1e-12), self.compute)
        self.ctx = hs.hs_ctx_create(self.cfg)
        self.P = hs.hs_param_count(self.cfg)
        assert theta0.dtype == np.float32 and theta0.size == self.P
        self.H = model["hidden"]
        self.act_dtype = torch.bfloat16 if self.compute == hs.HS_BF16 else torch.float32
        dev = self.device
        self.w = torch.from_numpy(theta0.copy()).to(dev)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.G = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.g = None                       # separate per-micro-batch gradient (unfused accumulation only)
        if self.compute == hs.HS_BF16:
            self.w_lowp = torch.empty(self.P, dtype=torch.bfloat16, device=dev)
            hs.hs_cast_params(self.w, self.w_lowp, self.P, hs.HS_BF16)
        else:
            self.w_lowp = None
        self.t = 0
        self._drop_on = False
        self._acts = self._ws = self._hidden = self._dhidden = None
        self._acts_bytes = self._ws_bytes = 0
        self.loss_buf = torch.zeros(64, dtype=torch.float32, device=dev)
        self.loss_out = torch.zeros(2, dtype=torch.float32, device=dev)     # the reported loss of a step

    def close(self):
        if self.ctx is not None:
            hs.hs_ctx_destroy(self.ctx)
            self.ctx = None

    # weights the forward/backward kernels read
    @property
    def w_compute(self):
        return self.w_lowp if self.compute == hs.HS_BF16 else self.w

    def _reserve(self, B, L, M):
        ab = hs.hs_acts_bytes(self.cfg, B, L, M)
        wb = hs.hs_workspace_bytes(self.cfg, B, L, M)
        if ab > self._acts_bytes:
            self._acts = torch.empty(ab, dtype=torch.uint8, device=self.device)
            self._acts_bytes = ab
        if wb > self._ws_bytes:
            self._ws = torch.empty(wb, dtype=torch.uint8, device=self.device)
            self._ws_bytes = wb
        n = B * L * self.H
        if self._hidden is None or self._hidden.numel() < n:
            self._hidden = torch.empty(n, dtype=self.act_dtype, device=self.device)
            self._dhidden = torch.empty(n, dtype=self.act_dtype, device=self.device)

    def upload(self, mb: dict) -> dict:
        """Host micro-batch (numpy) -> device tensors; done before the timed region."""
        dev = self.device
        out = dict(B=int(mb["ids"].shape[0]), L=int(mb["ids"].shape[1]), M=int(mb["mlm_pos"].size),
                   lens_host=np.ascontiguousarray(mb["lens"], dtype=np.int32),
                   ids=torch.from_numpy(np.ascontiguousarray(mb["ids"], dtype=np.int32)).to(dev),
                   lens=torch.from_numpy(np.ascontiguousarray(mb["lens"], dtype=np.int32)).to(dev),
                   mlm_pos=torch.from_numpy(np.ascontiguousarray(mb["mlm_pos"], dtype=np.int32)).to(dev),
                   mlm_label=torch.from_numpy(np.ascontiguousarray(mb["mlm_label"], dtype=np.int32)).to(dev),
                   n_seq=int(mb["ids"].shape[0]), drop=mb.get("drop"))
        self._reserve(out["B"], out["L"], out["M"])
        return out

    def forward_backward(self, d: dict, g: torch.Tensor, accumulate: int, loss_slot: int):
        """hs_encoder_fwd -> hs_mlm_loss -> hs_encoder_bwd for one uploaded micro-batch."""
        B, L, M = d["B"], d["L"], d["M"]
        self._reserve(B, L, M)
        drop = d.get("drop")           # dict(p, seed, stream) or None: the state both calls below must see
        if drop is not None or self._drop_on:
            hs.hs_set_dropout(self.ctx, drop["p"] if drop else 0.0, drop["seed"] if drop else 0, drop["stream"] if drop else 0)
            self._drop_on = drop is not None
        w = self.w_compute
        hs.hs_encoder_fwd(self.ctx, w, d["ids"], d["lens"], d["lens_host"], B, L, self._acts, self._hidden, self._ws,
                          self._ws_bytes)
        loss_ptr = self.loss_buf.data_ptr() + 4 * loss_slot
        hs.hs_mlm_loss(self.ctx, w, self._hidden, d["mlm_pos"], d["mlm_label"], M, B, L, loss_ptr, self._dhidden, g,
                       accumulate, self._ws, self._ws_bytes)
        hs.hs_encoder_bwd(self.ctx, w, self._acts, d["ids"], d["lens"], B, L, self._dhidden, g, accumulate, self._ws,
                          self._ws_bytes)

    def accumulate_micro_batches(self, batches: list, fused: bool = True, arm_last=None) -> int:
        """Runs every micro-batch and leaves the SUM of their gradients in G.  Entries that are
        None or carry dummy=True are workers/passes without data: they go through
        hs_grad_accum_normalize(ignore=1) and change nothing.  Returns the sample count.
        arm_last: a callable invoked right before the last real micro-batch of a fused run (used to arm
        the optimizer update that its backward pass then carries out)."""
        n_total, first = 0, True
        assert len(batches) <= self.loss_buf.numel()
        hs.hs_fill_zero(self.loss_buf, 4 * self.loss_buf.numel())
        real = [i for i, d in enumerate(batches) if d is not None and not d.get("dummy", False)]
        for i, d in enumerate(batches):
            if d is None or d.get("dummy", False):
                hs.hs_grad_accum_normalize(self.G, None, self.P, 1, 0.0)
                continue
            if fused:
                if first and d["M"] == 0:
                    hs.hs_fill_zero(self.G, 4 * self.P)
                    first = False
                if arm_last is not None and i == real[-1]:
                    arm_last()
                self.forward_backward(d, self.G, 0 if first else 1, i)
            else:
                if self.g is None:
                    self.g = torch.zeros(self.P, dtype=torch.float32, device=self.device)
                if first:
                    hs.hs_fill_zero(self.G, 4 * self.P)
                if d["M"] == 0:
                    hs.hs_fill_zero(self.g, 4 * self.P)
                self.forward_backward(d, self.g, 0, i)
                hs.hs_grad_accum_normalize(self.G, self.g, self.P, 0, 0.0)
            first = False
            n_total += d["n_seq"]
        if first:
            hs.hs_fill_zero(self.G, 4 * self.P)
        return n_total

    def train_step(self, batches: list, adam: dict, denom=None, fused: bool = True, update_in_backward: bool = True):
        """The whole hot path for one optimizer step.  Returns the sample count D; the loss sums
        stay on the device in loss_buf (read with reported_loss after synchronising).
        update_in_backward (fused accumulation only): normalisation and Adam are armed for the last
        micro-batch's backward pass, which applies them per parameter group as soon as that group's
        gradient is final (same arithmetic, same bits as the two separate calls)."""
        real = [d for d in batches if d is not None and not d.get("dummy", False)]
        D = sum(d["n_seq"] for d in real) if denom is None else denom
        wd = adam.get("weight_decay", 0.0)
        if fused and update_in_backward and real and D > 0:
            arm = lambda: hs.hs_arm_update(self.ctx, self.w, self.m, self.v, self.G, self.w_lowp, float(D), adam["lr"], adam["beta1"],
                                           adam["beta2"], adam["eps"], wd, self.t + 1)
            self.accumulate_micro_batches(batches, True, arm_last=arm)
            self.t += 1
            return D
        n_total = self.accumulate_micro_batches(batches, fused)
        D = n_total if denom is None else denom
        hs.hs_grad_accum_normalize(self.G, None, self.P, 0, float(D))
        self.t += 1
        hs.hs_adam_step(self.w, self.m, self.v, self.G, self.w_lowp, self.P, adam["lr"], adam["beta1"], adam["beta2"],
                        adam["eps"], wd, self.t)
        return D

    def reported_loss(self, D) -> float:
        """The weighted average of the step's loss sums (hs_weighted_loss); synchronises."""
        hs.hs_weighted_loss(self.loss_buf, self.loss_buf.numel(), float(D), self.loss_out)
        return float(self.loss_out[0].item())

    # ---- multi-step loop: schedule and checkpoints (call order only, like the rest of this class) ----
    def train(self, n_steps: int, micro_batches_of, adam: dict, schedule: dict) -> list:
        """n_steps updates; update number t = completed updates + 1 takes its micro-batches (host dicts)
        from micro_batches_of(t) and its learning rate from hs_lr_linear(t, **schedule).  Returns the
        reported loss of every update."""
        losses = []
        for _ in range(n_steps):
            t = self.t + 1
            lr = hs.hs_lr_linear(t, schedule["max_lr"], schedule["warmup"], schedule["total"])
            batches = [None if (mb is None or mb.get("dummy", False)) else self.upload(mb) for mb in micro_batches_of(t)]
            D = self.train_step(batches, dict(adam, lr=lr))
            losses.append(self.reported_loss(D))
        return losses

    def save_checkpoint(self, path: str, adam: dict, schedule: dict, seed: int, epoch: int = 0):
        """Everything needed to continue exactly: parameters, Adam moments, completed updates, the
        scheduler's numbers, the optimizer's hyper-parameters and the seed."""
        h = hs.hs_ckpt_header()
        h.cfg = self.cfg
        h.n_params, h.epoch, h.step, h.seed = self.P, epoch, self.t, seed
        h.max_lr, h.warmup, h.total = schedule["max_lr"], schedule["warmup"], schedule["total"]
        h.beta1, h.beta2, h.eps, h.weight_decay = adam["beta1"], adam["beta2"], adam["eps"], adam.get("weight_decay", 0.0)
        torch.cuda.synchronize(self.device)
        hs.hs_checkpoint_write(path, h, self.w.cpu().numpy(), self.m.cpu().numpy(), self.v.cpu().numpy())

    def load_checkpoint(self, path: str):
        """Restores a state written by save_checkpoint; returns (adam, schedule, seed, epoch)."""
        head = hs.hs_checkpoint_read_header(path)
        for f, _ in hs.hs_model_cfg._fields_:
            if f != "compute" and getattr(head.cfg, f) != getattr(self.cfg, f):
                raise ValueError(f"checkpoint is for another model ({f})")
        w, m, v = (np.empty(self.P, dtype=np.float32) for _ in range(3))
        head = hs.hs_checkpoint_read(path, w, m, v)
        self.w.copy_(torch.from_numpy(w)); self.m.copy_(torch.from_numpy(m)); self.v.copy_(torch.from_numpy(v))
        if self.w_lowp is not None:
            hs.hs_cast_params(self.w, self.w_lowp, self.P, hs.HS_BF16)
        self.t = int(head.step)
        adam = dict(beta1=head.beta1, beta2=head.beta2, eps=head.eps, weight_decay=head.weight_decay)
        schedule = dict(max_lr=head.max_lr, warmup=int(head.warmup), total=int(head.total))
        return adam, schedule, int(head.seed), int(head.epoch)


class PairWorker:
    """The translation workload's step (section "Transformer Translation Model") through the C ABI: hs_s2s_fwd ->
    hs_s2s_loss -> hs_s2s_bwd per micro-batch with the gradients summed in G, then normalisation by the global weight
    (the number of real target tokens unless the caller says otherwise) and Adam.  Buffer ownership and call order only."""

    def __init__(self, model: dict, compute: str, theta0: np.ndarray, label_smoothing: float = 0.1, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.compute = hs.HS_BF16 if compute == "bf16" else hs.HS_FP32
        self.cfg = hs.make_s2s_cfg(model["n_enc"], model["n_dec"], model["hidden"], model["n_heads"], model["ffn"], model["vocab"],
                                   model["max_pos"], model.get("ln_eps", 1e-5), self.compute)
        self.ctx = hs.hs_s2s_ctx_create(self.cfg)
        self.P = hs.hs_s2s_param_count(self.cfg)
        assert theta0.dtype == np.float32 and theta0.size == self.P
        self.H = model["hidden"]
        self.eps_ls = label_smoothing
        self.act_dtype = torch.bfloat16 if self.compute == hs.HS_BF16 else torch.float32
        dev = self.device
        self.w = torch.from_numpy(theta0.copy()).to(dev)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.G = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.w_lowp = None
        if self.compute == hs.HS_BF16:
            self.w_lowp = torch.empty(self.P, dtype=torch.bfloat16, device=dev)
            hs.hs_cast_params(self.w, self.w_lowp, self.P, hs.HS_BF16)
        self.t = 0
        self._drop_on = False
        self._acts = self._ws = self._out = self._dout = None
        self._acts_bytes = self._ws_bytes = 0
        self.loss_buf = torch.zeros(128, dtype=torch.float32, device=dev)      # slot i: loss sum, slot 64 + i: nll sum
        self.loss_out = torch.zeros(2, dtype=torch.float32, device=dev)

    def close(self):
        if self.ctx is not None:
            hs.hs_ctx_destroy(self.ctx)
            self.ctx = None

    @property
    def w_compute(self):
        return self.w_lowp if self.compute == hs.HS_BF16 else self.w

    def _reserve(self, B, Ls, Lt):
        ab, wb = hs.hs_s2s_acts_bytes(self.cfg, B, Ls, Lt), hs.hs_s2s_workspace_bytes(self.cfg, B, Ls, Lt)
        if ab > self._acts_bytes:
            self._acts, self._acts_bytes = torch.empty(ab, dtype=torch.uint8, device=self.device), ab
        if wb > self._ws_bytes:
            self._ws, self._ws_bytes = torch.empty(wb, dtype=torch.uint8, device=self.device), wb
        n = B * Lt * self.H
        if self._out is None or self._out.numel() < n:
            self._out = torch.empty(n, dtype=self.act_dtype, device=self.device)
            self._dout = torch.empty(n, dtype=self.act_dtype, device=self.device)

    def upload(self, mb: dict) -> dict:
        dev = self.device
        t = lambda k: torch.from_numpy(np.ascontiguousarray(mb[k], dtype=np.int32)).to(dev)
        out = dict(B=int(mb["src"].shape[0]), Ls=int(mb["src"].shape[1]), Lt=int(mb["tgt_in"].shape[1]), src=t("src"), src_lens=t("src_lens"),
                   tgt_in=t("tgt_in"), tgt_out=t("tgt_out"), tgt_lens=t("tgt_lens"),
                   tgt_lens_host=np.ascontiguousarray(mb["tgt_lens"], dtype=np.int32), n_seq=int(mb["src"].shape[0]),
                   n_tok=int(np.asarray(mb["tgt_lens"]).sum()), drop=mb.get("drop"))
        self._reserve(out["B"], out["Ls"], out["Lt"])
        return out

    def forward_backward(self, d: dict, g: torch.Tensor, accumulate: int, slot: int):
        B, Ls, Lt = d["B"], d["Ls"], d["Lt"]
        self._reserve(B, Ls, Lt)
        drop = d.get("drop")
        if drop is not None or self._drop_on:
            hs.hs_set_dropout(self.ctx, drop["p"] if drop else 0.0, drop["seed"] if drop else 0, drop["stream"] if drop else 0)
            self._drop_on = drop is not None
        w = self.w_compute
        hs.hs_s2s_fwd(self.ctx, w, d["src"], d["src_lens"], d["tgt_in"], d["tgt_lens"], B, Ls, Lt, self._acts, self._out)
        base = self.loss_buf.data_ptr()
        hs.hs_s2s_loss(self.ctx, w, self._out, d["tgt_out"], d["tgt_lens"], d.get("tgt_lens_host"), B, Lt, self.eps_ls, base + 4 * slot,
                       base + 4 * (64 + slot),
                       self._dout, g, accumulate, self._ws, self._ws_bytes)
        hs.hs_s2s_bwd(self.ctx, w, self._acts, d["src"], d["src_lens"], d["tgt_in"], d["tgt_lens"], B, Ls, Lt, self._dout, g, accumulate,
                      self._ws, self._ws_bytes)

    def train_step(self, batches: list, adam: dict, denom=None, update_in_backward: bool = False):
        """One optimizer step over the uploaded micro-batches (None = a pass without data).  Returns the weight D used
        (the number of real target tokens by default).  update_in_backward: normalisation and Adam are armed for the last
        micro-batch's backward pass, which applies them layer by layer as soon as a layer's gradient is final (same
        arithmetic, same bits as the two separate calls).  Off by default: at this model's sizes the update's memory
        traffic beside the small GEMMs of the backward pass costs more than it hides (6.58 against 6.49 ms per step)."""
        assert len(batches) <= 64
        hs.hs_fill_zero(self.loss_buf, 4 * self.loss_buf.numel())
        real = [i for i, d in enumerate(batches) if d is not None]
        D = float(denom if denom is not None else max(sum(batches[i]["n_tok"] for i in real), 1))
        self.t += 1
        first = True
        for i, d in enumerate(batches):
            if d is None:
                hs.hs_grad_accum_normalize(self.G, None, self.P, 1, 0.0)
                continue
            if update_in_backward and i == real[-1]:
                hs.hs_arm_update(self.ctx, self.w, self.m, self.v, self.G, self.w_lowp, D, adam["lr"], adam["beta1"], adam["beta2"],
                                 adam["eps"], adam.get("weight_decay", 0.0), self.t)
            self.forward_backward(d, self.G, 0 if first else 1, i)
            first = False
        if first:
            hs.hs_fill_zero(self.G, 4 * self.P)
        if first or not update_in_backward:
            hs.hs_grad_accum_normalize(self.G, None, self.P, 0, D)
            hs.hs_adam_step(self.w, self.m, self.v, self.G, self.w_lowp, self.P, adam["lr"], adam["beta1"], adam["beta2"], adam["eps"],
                            adam.get("weight_decay", 0.0), self.t)
        return D

    def reported_loss(self, D):
        """(smoothed loss, negative log-likelihood), both per unit of weight; synchronises."""
        hs.hs_weighted_loss(self.loss_buf, 64, float(D), self.loss_out)
        hs.hs_weighted_loss(self.loss_buf.data_ptr() + 256, 64, float(D), self.loss_out.data_ptr() + 4)
        out = self.loss_out.cpu().numpy().astype(np.float64)
        return float(out[0]), float(out[1])
