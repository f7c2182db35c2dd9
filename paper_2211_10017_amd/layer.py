"""MoEExpertLayer: owns the device buffers of one expert FFN layer and chains the five C-ABI
calls (Sec. 3.3: gate -> permute -> grouped GEMM pair -> un-permute/scale).  It allocates
every buffer once; forward() only marshals pointers, so it can run in a tight loop."""
from __future__ import annotations

import torch

from . import binding as B


class MoEExpertLayer:
    def __init__(self, T, d, F, E, k, bits, group_size=0, act_dtype=torch.float16, renormalize=True,
                 y_dtype=None, out_dtype=torch.float32, device="cuda:0", fuse_routing=True, activation="relu"):
        # what a whole layer call takes (the gate's limits are the narrowest of the entry points')
        if not (1 <= k <= 2 and k <= E <= B.LAYER_MAX_EXPERTS):
            raise B.MoeError("a layer call takes k = 1 or 2 experts per token and k <= E <= %d experts (k=%d E=%d)"
                             % (B.LAYER_MAX_EXPERTS, k, E))
        if T < 0 or d <= 0 or F <= 0 or d % 64 or F % 64:
            raise B.MoeError("a layer call takes T >= 0 and d, F positive multiples of 64 (T=%d d=%d F=%d)" % (T, d, F))
        self.T, self.d, self.F, self.E, self.k = T, d, F, E, k
        self.bits, self.group_size, self.renormalize = bits, group_size, renormalize
        self.act_dtype, self.out_dtype = act_dtype, out_dtype
        self.activation = B.ACTIVATIONS[activation]
        # y_perm is kept in fp32 for bf16 activations: an 8-bit significand on y would cost
        # more than the layer's whole error budget
        self.y_dtype = y_dtype or (torch.float32 if act_dtype == torch.bfloat16 else act_dtype)
        dev = self.device = torch.device(device)
        R = self.R = T * k
        g1 = d if group_size in (0, d) else group_size
        g2 = F if group_size in (0, F) else group_size
        self.bytes1 = d * F * bits // 8
        self.w1_packed = torch.empty(E * self.bytes1, dtype=torch.uint8, device=dev)
        self.w2_packed = torch.empty(E * self.bytes1, dtype=torch.uint8, device=dev)
        self.s1 = torch.empty((E, d // g1, F), dtype=torch.float16, device=dev)
        self.s2 = torch.empty((E, F // g2, d), dtype=torch.float16, device=dev)
        self.wg = torch.empty((d, E), dtype=act_dtype, device=dev)
        self.gate_bias = None
        self.b1 = self.b2 = None
        # per-call buffers
        self.expert_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.expert_scale = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.x_perm = torch.empty((R, d), dtype=act_dtype, device=dev)
        self.perm_src = torch.empty(R, dtype=torch.int32, device=dev)
        self.inv_perm = torch.empty(R, dtype=torch.int32, device=dev)
        self.expert_offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
        self.y_perm = torch.empty((R, d), dtype=self.y_dtype, device=dev)
        self.out = torch.empty((T, d), dtype=out_dtype, device=dev)
        self.ws_permute = torch.empty(B.moe_permute_workspace_bytes(T, k, E), dtype=torch.uint8, device=dev)
        self.ws_ffn = torch.empty(B.moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, act_dtype),
                                  dtype=torch.uint8, device=dev)
        self._plans = {}
        self._bare = {}
        # large batches: the row gather (and for k = 1 the un-permute and gate scale) run inside
        # the GEMMs instead of as copies of their own
        self.routed = bool(fuse_routing) and B.moe_grouped_ffn_wq_routed_supported(R, E, T, d, F, bits, group_size, act_dtype)
        # decode-sized batches: the permutation is rebuilt inside fc1 (no permute launch, no x_perm copy)
        self.gated = B.moe_grouped_ffn_wq_gated_supported(T, k, E, d, F, bits, group_size, act_dtype) if fuse_routing else 0

    # -- offline: quantise one expert matrix from its fp32 master (which = 1 | 2) ------------
    def load_expert(self, which: int, e: int, w_fp32, q_canon_out=None):
        packed = self.w1_packed if which == 1 else self.w2_packed
        scales = self.s1 if which == 1 else self.s2
        B.moe_quantize_experts_into(w_fp32.unsqueeze(0), self.bits, self.group_size, q_canon_out,
                                    scales[e:e + 1], packed[e * self.bytes1:(e + 1) * self.bytes1])

    def share_weights_from(self, other: "MoEExpertLayer"):
        for name in ("w1_packed", "w2_packed", "s1", "s2"):
            setattr(self, name, getattr(other, name))

    # -- per call ---------------------------------------------------------------------------
    # The steps one by one (bench.py times them separately); each runs its entry of the same plan
    # forward() replays, so the fused and un-fused variants cannot drift apart.
    def _step(self, name, x, finished=None):
        for fn, args, what in self._plan(x, finished):
            if what.startswith(name):
                rc = fn(*args)
                if rc != 0:
                    B._check(rc, what)

    def gate(self, x, finished=None):
        self._step("moe_gate_topk", x, finished)
        return self.expert_idx, self.expert_scale

    def permute(self, x, finished=None):
        self._step("moe_permute", x, finished)

    def ffn(self, x, finished=None):
        self._step("moe_grouped_ffn_wq", x, finished)

    def ffn_streaming_kernel_only(self, x, finished=None):
        """The decode path's streaming kernel without its slice reduction (the gated call with a NULL output), for
        timing that kernel alone.  Raises MoeError where the FFN call does not take the decode kernel."""
        fn, args, what = [c for c in self._plan(x, finished) if c[2].startswith("moe_grouped_ffn_wq")][0]
        if what != "moe_grouped_ffn_wq_gated":
            raise B.MoeError("ffn_streaming_kernel_only: this layer does not run the gated FFN call")
        bare = self._bare.get(id(args))
        if bare is None:
            if len(self._bare) > 256:
                self._bare.clear()
            bare = self._bare[id(args)] = (args, args[:18] + (None,) + args[19:])      # (keeps args alive: id stays unique)
        rc = fn(*bare[1])
        if rc != 0:
            B._check(rc, what)

    def combine(self, x, finished=None):
        self._step("moe_combine", x, finished)       # nothing to do when fc2 stored the output itself
        return self.out

    def forward(self, x, finished=None):
        """The four per-call entry points back to back.  The argument lists are marshalled once per
        (input tensor, weight buffers, stream) and then replayed: in a decode-sized layer the
        kernels are shorter than the time Python needs to rebuild them.
        finished: uint8 [T] on the device, nonzero for rows pruned from the batch (their output
        rows are zero and their experts' weights are not read on their account)."""
        for fn, args, name in self._plan(x, finished):
            rc = fn(*args)
            if rc != 0:
                B._check(rc, name)
        return self.out

    def _plan(self, x, finished):
        opt = lambda t: 0 if t is None else t.data_ptr()  # noqa: E731
        key = (x.data_ptr(), opt(finished), self.w1_packed.data_ptr(), self.w2_packed.data_ptr(), self.s1.data_ptr(),
               self.s2.data_ptr(), self.wg.data_ptr(), opt(self.gate_bias), opt(self.b1), opt(self.b2),
               torch.cuda.current_stream().cuda_stream)
        calls = self._plans.get(key)
        if calls is None:
            calls = self._plans[key] = self._marshal(x, finished, key[-1])
            if len(self._plans) > 256:
                self._plans.pop(next(iter(self._plans)))
        return calls

    def _marshal(self, x, finished, stream):
        import ctypes
        lib = B.load()
        vp = ctypes.c_void_p
        p = lambda t: None if t is None else vp(t.data_ptr())  # noqa: E731
        if x.dtype != self.act_dtype or tuple(x.shape) != (self.T, self.d) or not x.is_contiguous() or not x.is_cuda:
            raise B.MoeError("x must be a contiguous [T, d] CUDA tensor in the layer's activation dtype")
        if finished is not None and (finished.dtype != torch.uint8 or finished.numel() != self.T
                                     or not finished.is_contiguous() or not finished.is_cuda):
            raise B.MoeError("finished must be a contiguous uint8 [T] CUDA tensor")
        active = vp(self.expert_offsets.data_ptr() + 4 * self.E)
        dt, ydt, odt = B._DT[self.act_dtype], B._DT[self.y_dtype], B._DT[self.out_dtype]
        st = vp(stream)
        gate = (lib.moe_gate_topk, (p(x), dt, p(self.wg), p(self.gate_bias), p(finished), self.T, self.d, self.E, self.k,
                                    int(self.renormalize), p(self.expert_idx), p(self.expert_scale), st), "moe_gate_topk")
        combine = (lib.moe_combine, (p(self.y_perm), ydt, p(self.inv_perm), p(self.expert_scale), active, self.T, self.k,
                                     self.d, p(self.out), odt, st), "moe_combine")
        if self.gated:
            # level 2 with an fp32 layer output: fc2 adds the scaled rows straight into out (no combine launch)
            fused = self.gated == 2 and self.out_dtype == torch.float32
            ffn = (lib.moe_grouped_ffn_wq_gated,
                   (p(x), dt, p(self.expert_idx), p(self.expert_scale) if fused else None, self.T, self.k, self.E, self.d,
                    self.F, self.bits, self.group_size, self.activation, p(self.w1_packed), p(self.s1), p(self.b1),
                    p(self.w2_packed), p(self.s2), p(self.b2), p(self.out) if fused else p(self.y_perm),
                    odt if fused else ydt, p(self.perm_src), p(self.inv_perm), p(self.expert_offsets), p(self.ws_ffn),
                    self.ws_ffn.numel(), st), "moe_grouped_ffn_wq_gated")
            return [gate, ffn] if fused else [gate, ffn, combine]
        if self.routed:
            # index only (no x_perm copy); fc1 gathers, and fc2 scatters when there is one expert per
            # token and no pruned row (a pruned token's output row would stay unwritten)
            scatter = self.k == 1 and finished is None
            permute = (lib.moe_permute, (p(self.expert_idx), None, dt, self.T, self.k, self.E, self.d, None,
                                         p(self.perm_src), p(self.inv_perm), p(self.expert_offsets), p(self.ws_permute),
                                         self.ws_permute.numel(), st), "moe_permute")
            ffn = (lib.moe_grouped_ffn_wq_routed,
                   (p(x), dt, p(self.perm_src), self.k, p(self.expert_scale) if scatter else None, p(self.expert_offsets),
                    self.R, self.E, self.T, self.d, self.F, self.bits, self.group_size, self.activation, p(self.w1_packed), p(self.s1),
                    p(self.b1), p(self.w2_packed), p(self.s2), p(self.b2), p(self.out) if scatter else p(self.y_perm),
                    odt if scatter else ydt, p(self.ws_ffn), self.ws_ffn.numel(), st), "moe_grouped_ffn_wq_routed")
            return [gate, permute, ffn] if scatter else [gate, permute, ffn, combine]
        permute = (lib.moe_permute, (p(self.expert_idx), p(x), dt, self.T, self.k, self.E, self.d, p(self.x_perm),
                                     p(self.perm_src), p(self.inv_perm), p(self.expert_offsets), p(self.ws_permute),
                                     self.ws_permute.numel(), st), "moe_permute")
        ffn = (lib.moe_grouped_ffn_wq, (p(self.x_perm), dt, p(self.expert_offsets), self.R, self.E, self.T, self.d,
                                        self.F, self.bits, self.group_size, self.activation, p(self.w1_packed), p(self.s1), p(self.b1),
                                        p(self.w2_packed), p(self.s2), p(self.b2), p(self.y_perm), ydt,
                                        p(self.ws_ffn), self.ws_ffn.numel(), st), "moe_grouped_ffn_wq")
        return [gate, permute, ffn, combine]
