"""Flat device buffers of one model's optimizer state and the three calls of one training step.

Memory per parameter (Sec. 2.2, Eq. 8 of the paper): FP8 gradient 1 B, FP8 first moment 1 B, FP16
second moment 2 B, FP16 master weight 2 B -- 6 B -- plus the 1 B (E4M3) or 2 B (bf16) weight copy
handed back to the model.  The bf16 gradient source belongs to the caller.
"""
from __future__ import annotations

import torch

from . import binding as B
from .placement import RegionAllocator, StripedArena


class OptimizerState:
    def __init__(self, tensors, total_elems: int, cfg: B.AutoscaleCfg, device: int = 0,
                 grad_fmt: int = B.E5M2, wcopy: int = B.WCOPY_E4M3, spread: bool = False,
                 grad_buffer: bool = False, master_fmt: int = B.STATE_F16, v_fmt: int = B.STATE_F16,
                 share_with: "OptimizerState" = None, arena_order=None, second_m: bool = False,
                 wcopy_over_grad: bool = False, n_grad_buffers: int = 1):
        """`share_with`: another state over the same flat buffers.  Parameter groups (say, no weight decay on
        biases and LayerNorm weights) are one state each, over disjoint tensor lists of the same buffers; each
        has its own context and metadata and is stepped with its own hyper-parameters.
        `second_m`: a second first-moment buffer (1 B/param more), so that `step(..., pair_m=True)` can run the Adam
        step without its read-only pass (fp8lm_adam_step_fp8_m2); `m` always names the buffer that holds the moment.
        `n_grad_buffers`: with grad_buffer, how many bf16 gradient sources to allocate (`grads`; `grad` is the first).
        `wcopy_over_grad`: the E4M3 weight copy is written over the FP8 gradient (`wq` is `g8`): after a step the buffer
        holds the weights, after a quantisation the gradient; 1 B/param less, the same bytes, the same speed."""
        dev = torch.device(f"cuda:{device}")
        self.tensors = list(tensors)
        self.total = int(total_elems)
        self.cfg = cfg
        self.grad_fmt = grad_fmt
        self.wcopy_kind = wcopy
        self.master_fmt, self.v_fmt = master_fmt, v_fmt
        state_dtype = {B.STATE_F16: torch.float16, B.STATE_BF16: torch.bfloat16, B.STATE_E4M3: torch.uint8,
                       B.STATE_F32: torch.float32}
        self.ctx = B.Context(self.tensors, device)
        n = max(self.total, 16)
        qdt = torch.uint8 if wcopy == B.WCOPY_E4M3 else torch.bfloat16
        # (name, elements, type, bytes per element that the update pass moves through the buffer), in the order of
        # allocation.  With `spread` the buffers are placed so that no HBM region carries more than about three fifths
        # of that traffic (see placement.py: typically v and the copy in one region, w, m and the FP8 gradient in
        # another; the gradient sources, which the cast reads while it writes the FP8 gradient, beside v); otherwise
        # they are carved out of one allocation.
        esz = lambda dt: torch.empty((), dtype=dt).element_size()
        grad_names = (["grad"] + [f"grad_{i}" for i in range(1, n_grad_buffers)]) if grad_buffer else []
        plan = [("v", n, state_dtype[v_fmt], 2.0 * esz(state_dtype[v_fmt]))] \
            + ([] if wcopy_over_grad else [("wq", n, qdt, 1.0 * esz(qdt))]) \
            + [(g, n, torch.bfloat16, 0.0) for g in grad_names] \
            + [("w", n, state_dtype[master_fmt], 2.0 * esz(state_dtype[master_fmt])),
               ("m", n, torch.uint8, 1.0 if second_m else 2.0)] + ([("m_other", n, torch.uint8, 1.0)] if second_m else []) \
            + [("g8", n, torch.uint8, 2.0 if wcopy_over_grad else 1.0)]
        if wcopy_over_grad:
            assert wcopy == B.WCOPY_E4M3 and not second_m and share_with is None, \
                "only an E4M3 copy fits the gradient's buffer; the step with a pair of moments reads the gradient twice"
        self.placement = {}
        if share_with is not None:
            o = share_with
            assert (o.grad_fmt, o.wcopy_kind, o.master_fmt, o.v_fmt) == (grad_fmt, wcopy, master_fmt, v_fmt)
            assert o.g8.numel() >= n
            bufs = dict(g8=o.g8, m=o.m, v=o.v, w=o.w, wq=o.wq)
            assert not second_m, "parameter groups share one first-moment buffer"
            if o.grad is not None:
                bufs["grad"] = o.grad
            self.spread = o.spread
        elif spread:
            # everything but the FP8 gradient region by region, by measurement; the FP8 gradient, the one buffer the
            # cast writes, in pieces that alternate between regions (if that fails it is placed like the others)
            g8_weight = next(w for name, _, _, w in plan if name == "g8")
            alloc = RegionAllocator(self.ctx, device)
            bufs = alloc.allocate([entry for entry in plan if entry[0] != "g8"], even_weight=g8_weight)
            self.spread = alloc.spread
            self.placement = dict(alloc.log, where=alloc.where)
            striped = None
            if self.spread:
                try:
                    striped = StripedArena(self.ctx, n, device)
                    bufs["g8"] = striped.tensor(0, n)
                    self.placement["g8_striped"] = striped.log
                except RuntimeError as e:
                    self.placement["g8_striped"] = {"gave_up": str(e).splitlines()[0][:120]}
            if "g8" not in bufs:
                bufs["g8"] = torch.zeros(n, dtype=torch.uint8, device=dev)
        else:
            # one allocation, the buffers carved out of it one after the other (what a caller of the C ABI with an
            # arena of its own would do): where they lie relative to each other is then the same in every process
            # Default order: v, copy, gradient sources, w, FP8 gradient, m.  Where the pieces of such an allocation
            # lie among the HBM regions is up to the driver (see placement.py); `spread` is the way to decide it.
            items = [(name, k, dt) for name, k, dt, _ in plan]
            order = (list(arena_order) + grad_names[1:]) if arena_order else \
                [nm for nm in ["v", "wq"] + grad_names + ["w", "g8", "m", "m_other"] if any(nm == it[0] for it in items)]
            assert sorted(order) == sorted(name for name, _, _ in items), order
            items.sort(key=lambda it: order.index(it[0]))
            align = (2 << 20) if n >= (2 << 20) else 256
            offs, end = [], 0
            for _, k, dt in items:
                offs.append(end)
                end += (k * torch.empty((), dtype=dt).element_size() + align - 1) // align * align
            self.arena = torch.zeros(end, dtype=torch.uint8, device=dev)
            bufs = {name: self.arena[o:o + k * torch.empty((), dtype=dt).element_size()].view(dt)
                    for (name, k, dt), o in zip(items, offs)}
            self.spread = False
            self.placement = {"arena_bytes": end, "order": [name for name, _, _ in items]}
        self.g8, self.m, self.v, self.w = bufs["g8"], bufs["m"], bufs["v"], bufs["w"]
        self.wq = self.g8 if wcopy_over_grad else bufs["wq"]
        self.grad = bufs.get("grad")       # bf16 gradient source, only if asked for
        self.grads = [bufs[g] for g in grad_names]
        self.m_other = bufs.get("m_other")  # the other buffer of the first-moment pair, only if asked for
        self.g_meta = self.ctx.new_meta(cfg)
        self.m_meta = self.ctx.new_meta(cfg)
        self.v_meta = self.ctx.new_meta(cfg)
        self.w_meta = self.ctx.new_meta(cfg)
        self.q_meta = self.ctx.new_meta(cfg)

    @property
    def state_bytes_per_param(self) -> int:
        """Eq. 8's four buffers: FP8 gradient, first moment, second moment, master weight."""
        return self.g8.element_size() + self.m.element_size() + self.v.element_size() + self.w.element_size()

    def init_master(self, w_bf16: torch.Tensor) -> None:
        self.ctx.init_master(w_bf16, self.w, self.w_meta, self.master_fmt)

    def quantize_grad(self, grad_bf16: torch.Tensor) -> None:
        self.ctx.amax_scale(grad_bf16, self.grad_fmt, self.g_meta, self.cfg)
        self.ctx.cast_fp8(grad_bf16, self.g8, self.grad_fmt, self.g_meta, self.cfg)

    def quantize_grad_delayed(self, grad_bf16: torch.Tensor) -> None:
        """Single pass: scale from the amax history, cast, and record this step's amax."""
        self.ctx.cast_fp8_delayed(grad_bf16, self.g8, self.grad_fmt, self.g_meta, self.cfg)

    def adam(self, hp: B.AdamHparams) -> None:
        self.ctx.adam_step_fp8(self.g8, self.grad_fmt, self.g_meta, self.m, self.m_meta, self.v, self.v_meta,
                               self.w, self.w_meta, self.wq, self.q_meta, hp)

    def step(self, grad: torch.Tensor, hp: B.AdamHparams, delayed: bool = False, speculative: bool = False,
             pair_m: bool = False) -> None:
        """One pass of the whole hot path: amax + scale, FP8 cast, FP8 Adam, from a bf16, fp16 or fp32
        gradient buffer.  With `delayed` the
        gradient is quantised in a single pass with the scale of the preceding steps.  With
        hp.m_scale_mode == MSCALE_FROM_CAST the cast also does the Adam step's first pass.  With `speculative` the
        just-in-time quantisation goes through quantize_fp8 (same results; tensors whose scale does not change are
        read once).  With `pair_m` (state created with second_m) the Adam step goes through adam_step_fp8_m2 (same
        results; no read-only pass; the first moment moves to the other buffer of the pair)."""
        fused = hp.m_scale_mode == B.MSCALE_FROM_CAST
        if pair_m:
            assert self.m_other is not None and not fused and not delayed
            if speculative:
                self.ctx.quantize_fp8(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg)
            else:
                self.quantize_grad(grad)
            self.ctx.adam_step_fp8_m2(self.g8, self.grad_fmt, self.g_meta, self.m, self.m_other, self.m_meta, self.v,
                                      self.v_meta, self.w, self.w_meta, self.wq, self.q_meta, hp)
            self.m, self.m_other = self.m_other, self.m
            return
        if speculative:
            assert not delayed
            if fused:
                self.ctx.quantize_fp8_for_adam(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg, self.m, self.m_meta,
                                               hp.beta1)
            else:
                self.ctx.quantize_fp8(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg)
            self.adam(hp)
            return
        if not delayed:
            self.ctx.amax_scale(grad, self.grad_fmt, self.g_meta, self.cfg)
        if fused:
            self.ctx.cast_fp8_for_adam(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg, self.m, self.m_meta,
                                       hp.beta1, delayed=delayed)
        elif delayed:
            self.ctx.cast_fp8_delayed(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg)
        else:
            self.ctx.cast_fp8(grad, self.g8, self.grad_fmt, self.g_meta, self.cfg)
        self.adam(hp)
