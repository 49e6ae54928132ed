"""Device-side plumbing for running a workload through liblpk: arenas in HBM,
descriptor lists, and the order of the library calls of one training step.

No arithmetic of the method happens here -- PyTorch only allocates device
memory, copies inputs in and results out, and provides the stream.

HBM layout: one flat arena per role (theta, comp, int16 grad, fp32 source),
every tensor starting on a 256-byte boundary inside it so all of them take the
16-byte vector path; per-tensor int32 fraclen arrays, a uint64 vmax array and
a uint32 status word stay on the device, so consecutive steps chain on one
stream without a host round trip.
"""
import numpy as np
import torch

from . import binding as lpk

ALIGN = 256


def _offsets(sizes, elem_bytes):
    offs, pos = [], 0
    for n, eb in zip(sizes, elem_bytes):
        offs.append(pos)
        pos += (n * eb + ALIGN - 1) // ALIGN * ALIGN
    return offs, max(pos, ALIGN)


class DeviceState:
    def __init__(self, cfg, device="cuda:0", kahan=True, n_src=1, comp_bits=None, mom_bits=None, fl_mom0=16,
                 sec_bits=None, fl_sec0=40, grad_bits=16):
        """cfg: workloads.Config.  n_src: how many fp32 source arenas stay resident (gradient cycle).
        comp_bits: per-tensor width of comp when it differs from theta's.  mom_bits: per-tensor width of a
        velocity tensor (momentum update; ADAM's first moment); its fraclen starts at fl_mom0 and is re-selected
        every step.  sec_bits: per-tensor width of ADAM's second moment, fraclen from fl_sec0, re-selected too.
        grad_bits: width of the quantized gradients (16, or 8 for the all-8-bit mode)."""
        self.cfg, self.device, self.kahan = cfg, torch.device(device), kahan
        nt = cfg.n_tensors
        tb = [b // 8 for b in cfg.bits]
        cbits = list(comp_bits) if comp_bits is not None else list(cfg.bits)
        cb = [b // 8 for b in cbits]
        self.comp_bits = cbits
        dt = {1: torch.int8, 2: torch.int16}
        dev = self.device

        self.off_theta, tot_t = _offsets(cfg.sizes, tb)
        self.off_comp, tot_c = _offsets(cfg.sizes, cb)
        self.grad_bits = grad_bits
        self.off_grad, tot_g = _offsets(cfg.sizes, [grad_bits // 8] * nt)
        self.off_src, tot_s = _offsets(cfg.sizes, [4] * nt)
        self.arena_theta = torch.zeros(tot_t, dtype=torch.uint8, device=dev)
        self.arena_comp = torch.zeros(tot_c, dtype=torch.uint8, device=dev) if kahan else None
        self.arena_grad = torch.zeros(tot_g, dtype=torch.uint8, device=dev)
        self.arena_src = [torch.zeros(tot_s, dtype=torch.uint8, device=dev) for _ in range(n_src)]
        self.src_bytes = tot_s
        self.mom_bits = list(mom_bits) if mom_bits is not None else None
        if self.mom_bits:
            mb = [b // 8 for b in self.mom_bits]
            self.off_mom, tot_m = _offsets(cfg.sizes, mb)
            self.arena_mom = torch.zeros(tot_m, dtype=torch.uint8, device=dev)

        self.sec_bits = list(sec_bits) if sec_bits is not None else None
        if self.sec_bits:
            sb = [b // 8 for b in self.sec_bits]
            self.off_sec, tot_u = _offsets(cfg.sizes, sb)
            self.arena_sec = torch.zeros(tot_u, dtype=torch.uint8, device=dev)

        def view(arena, off, n, eb, dtype):
            return arena[off:off + n * eb].view(dtype)

        self.theta = [view(self.arena_theta, o, n, e, dt[e]) for o, n, e in zip(self.off_theta, cfg.sizes, tb)]
        self.comp = ([view(self.arena_comp, o, n, e, dt[e]) for o, n, e in zip(self.off_comp, cfg.sizes, cb)]
                     if kahan else [None] * nt)
        self.grad = [view(self.arena_grad, o, n, grad_bits // 8, dt[grad_bits // 8]) for o, n in zip(self.off_grad, cfg.sizes)]
        self.src = [[view(a, o, n, 4, torch.float32) for o, n in zip(self.off_src, cfg.sizes)] for a in self.arena_src]

        self.mom = ([view(self.arena_mom, o, n, e, dt[e]) for o, n, e in zip(self.off_mom, cfg.sizes, mb)]
                    if self.mom_bits else [None] * nt)
        self.sec = ([view(self.arena_sec, o, n, e, dt[e]) for o, n, e in zip(self.off_sec, cfg.sizes, sb)]
                    if self.sec_bits else [None] * nt)
        self.lists = []
        for k in range(n_src):
            descs = [lpk.make_desc(self.theta[t], self.comp[t], self.grad[t], self.src[k][t], momentum=self.mom[t],
                                   second=self.sec[t]) for t in range(nt)]
            self.lists.append(lpk.TensorList(descs))

        i32 = dict(dtype=torch.int32, device=dev)
        self.fl_theta = torch.tensor([b - 1 for b in cfg.bits], **i32)   # grid theta is on now
        self.fl_next = self.fl_theta.clone()                               # grid the next step moves it to
        self.fl_spare = self.fl_theta.clone()
        self.fl_grad = torch.full((nt,), grad_bits - 1, **i32)
        self.fl_mom = torch.full((nt,), fl_mom0, **i32)                    # grid the velocity is on now
        self.fl_mom_next = self.fl_mom.clone()
        self.fl_mom_spare = self.fl_mom.clone()
        self.fl_sec = torch.full((nt,), fl_sec0, **i32)                    # grid the second moment is on now
        self.fl_sec_next = self.fl_sec.clone()
        self.fl_sec_spare = self.fl_sec.clone()
        self.umax = torch.zeros(nt, dtype=torch.int64, device=dev)         # uint64 payload
        self.mmax = torch.zeros(nt, dtype=torch.int64, device=dev)         # uint64 payload
        self.vmax = torch.zeros(nt, dtype=torch.int64, device=dev)         # uint64 payload
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)        # uint32 payload
        self._host_src = None

    # ---- host <-> device copies --------------------------------------------------------------------
    def host_src(self):
        """Pinned host staging buffer with the layout of a source arena."""
        if self._host_src is None:
            self._host_src = torch.zeros(self.src_bytes, dtype=torch.uint8, pin_memory=True)
        return self._host_src

    def host_src_views(self):
        h = self.host_src().numpy()
        return [h[o:o + 4 * n].view(np.float32) for o, n in zip(self.off_src, self.cfg.sizes)]

    def upload_src(self, k=0):
        self.arena_src[k].copy_(self.host_src(), non_blocking=False)

    def download(self):
        """(theta list, comp list, fl_theta, fl_grad, vmax, status) as numpy / ints, after a sync."""
        torch.cuda.synchronize(self.device)
        th = [t.cpu().numpy() for t in self.theta]
        co = [c.cpu().numpy() if c is not None else None for c in self.comp]
        vm = self.vmax.cpu().numpy().view(np.uint64)
        return th, co, self.fl_theta.cpu().numpy(), self.fl_grad.cpu().numpy(), vm, int(self.status.cpu().numpy().view(np.uint32)[0])

    # ---- the calls of the path ----------------------------------------------------------------------
    def init_theta(self, k=0):
        """theta0 (already in source arena k) -> fraclen from its max-abs -> DFX theta; comp starts at 0."""
        L = self.lists[k]
        lpk.lpk_select_fraclen(L, lpk.LPK_F32, lpk.LPK_SEL_THETA, None, None, self.fl_theta, self.fl_theta, self.status)
        lpk.lpk_quantize_tensor(L, lpk.LPK_SEL_THETA, self.fl_theta, self.status)
        self.fl_next.copy_(self.fl_theta)
        if self.arena_comp is not None:
            self.arena_comp.zero_()

    def quantize_grads(self, k=0):
        """fp32 gradients in source arena k -> per-tensor fraclen -> int16 gradients."""
        L = self.lists[k]
        lpk.lpk_select_fraclen(L, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, self.fl_grad, self.fl_grad, self.status)
        lpk.lpk_quantize_tensor(L, lpk.LPK_SEL_GRAD, self.fl_grad, self.status)

    def quantize_grads_onepass(self, k=0):
        """The same result as quantize_grads with one read of the fp32 gradients where last step's fraclens still
        hold (lpk_select_quantize: fl_grad is guess and result)."""
        lpk.lpk_select_quantize(self.lists[k], lpk.LPK_SEL_GRAD, self.fl_grad, self.fl_grad, self.status)

    def select_grads(self, k=0):
        """fp32 gradients in source arena k -> per-tensor fraclen only (for the steps that quantize in registers)."""
        lpk.lpk_select_fraclen(self.lists[k], lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, self.fl_grad, self.fl_grad, self.status)

    def update(self, lr_q16, wd_q16=0, k=0, want_vmax=True):
        """The fused lazy update; theta moves from grid fl_theta to fl_next."""
        lpk.lpk_kahan_sgd_step(self.lists[k], self.fl_theta, self.fl_next, self.fl_grad, lr_q16, wd_q16,
                               self.vmax if want_vmax else None, self.status)
        if self.cfg.reselect:
            # fraclen for the step after this one, from this step's vmax (one-step lag); rotate the three arrays
            lpk.lpk_select_fraclen(self.lists[k], lpk.LPK_VMAX_U64, lpk.LPK_SEL_THETA, self.vmax, self.fl_theta,
                                   self.fl_next, self.fl_spare, self.status)
            self.fl_theta, self.fl_next, self.fl_spare = self.fl_next, self.fl_spare, self.fl_theta

    def update_momentum(self, lr_q16, mu_q16, wd_q16=0, k=0, fused=False):
        """Momentum update with the lazy update inside; the velocity moves from grid fl_mom to fl_mom_next, and
        the grid after that is re-selected from this step's mmax (one-step lag), like theta's in `update`.
        fused: read the fp32 gradients directly instead of the int16 ones."""
        L = self.lists[k]
        call = lpk.lpk_momentum_sgd_step_f32grad if fused else lpk.lpk_momentum_sgd_step
        call(L, self.fl_theta, self.fl_next, self.fl_mom, self.fl_mom_next, self.fl_grad,
                                  lr_q16, mu_q16, wd_q16, self.vmax, self.mmax, self.status)
        if self.cfg.reselect:
            lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_THETA, self.vmax, self.fl_theta,
                                   self.fl_next, self.fl_spare, self.status)
            self.fl_theta, self.fl_next, self.fl_spare = self.fl_next, self.fl_spare, self.fl_theta
        lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_MOMENTUM, self.mmax, self.fl_mom_next,
                               self.fl_mom_next, self.fl_mom_spare, self.status)
        self.fl_mom, self.fl_mom_next, self.fl_mom_spare = self.fl_mom_next, self.fl_mom_spare, self.fl_mom

    def update_adam(self, hyper, k=0, fused=False):
        """ADAM with the lazy update inside; both moments move to the grids chosen one step earlier, and the grids
        after those are re-selected from this step's mmax / umax (one-step lag), like theta's in `update`.
        fused: read the fp32 gradients directly instead of the int16 ones."""
        L = self.lists[k]
        call = lpk.lpk_adam_step_f32grad if fused else lpk.lpk_adam_step
        call(L, self.fl_theta, self.fl_next, self.fl_mom, self.fl_mom_next, self.fl_sec, self.fl_sec_next,
                          self.fl_grad, hyper, self.vmax, self.mmax, self.umax, self.status)
        if self.cfg.reselect:
            lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_THETA, self.vmax, self.fl_theta,
                                   self.fl_next, self.fl_spare, self.status)
            self.fl_theta, self.fl_next, self.fl_spare = self.fl_next, self.fl_spare, self.fl_theta
        lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_MOMENTUM, self.mmax, self.fl_mom_next,
                               self.fl_mom_next, self.fl_mom_spare, self.status)
        self.fl_mom, self.fl_mom_next, self.fl_mom_spare = self.fl_mom_next, self.fl_mom_spare, self.fl_mom
        lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_SECOND, self.umax, self.fl_sec_next,
                               self.fl_sec_next, self.fl_sec_spare, self.status)
        self.fl_sec, self.fl_sec_next, self.fl_sec_spare = self.fl_sec_next, self.fl_sec_spare, self.fl_sec

    def step_fused(self, step_idx, k=0):
        """The whole path with quantization fused into the update: max-abs fraclen selection, then one pass that
        reads the fp32 gradients directly (the int16 gradient arena is not touched)."""
        L = self.lists[k]
        lpk.lpk_select_fraclen(L, lpk.LPK_F32, lpk.LPK_SEL_GRAD, None, None, self.fl_grad, self.fl_grad, self.status)
        lpk.lpk_kahan_sgd_step_f32grad(L, self.fl_theta, self.fl_next, self.fl_grad, self.cfg.lr_q16(step_idx),
                                       self.cfg.wd_q16, self.vmax, self.status)
        if self.cfg.reselect:
            lpk.lpk_select_fraclen(L, lpk.LPK_VMAX_U64, lpk.LPK_SEL_THETA, self.vmax, self.fl_theta,
                                   self.fl_next, self.fl_spare, self.status)
            self.fl_theta, self.fl_next, self.fl_spare = self.fl_next, self.fl_spare, self.fl_theta

    def step(self, step_idx, k=0, mu_q16=None, onepass=False):
        """One pass of the whole hot path over gradients already resident in source arena k."""
        if onepass:
            self.quantize_grads_onepass(k)
        else:
            self.quantize_grads(k)
        if mu_q16 is None:
            self.update(self.cfg.lr_q16(step_idx), self.cfg.wd_q16, k)
        else:
            self.update_momentum(self.cfg.lr_q16(step_idx), mu_q16, self.cfg.wd_q16, k)

    def capture_step(self, step_idx, k=0, fused=False, onepass=False):
        """Record one whole step over source arena k (max-abs selection, quantization, update; or, fused, max-abs
        selection and the update fed from the fp32 gradients; or, onepass, lpk_select_quantize and the update) into a HIP graph and
        return it (a torch.cuda.CUDAGraph; `.replay()` enqueues the step).  The library calls only enqueue kernels --
        no allocation, no synchronization, no memset node -- so they can be captured as they are.  The learning
        rate is a kernel argument and is frozen into the graph; workloads that rotate their fraclen arrays between
        steps (fraclen re-selection) cannot be replayed from one recording."""
        assert not self.cfg.reselect, "fraclen re-selection swaps device arrays between steps"
        step = self.step_fused if fused else (lambda s, kk: self.step(s, kk, onepass=onepass))
        step(step_idx, k)                           # warm-up outside the capture (first-use initialisation)
        torch.cuda.synchronize(self.device)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(step_idx, k)
        return graph

    def close(self):
        for L in self.lists:
            L.destroy()
        self.lists = []
