"""MoEExpertLayer: owns the device buffers of one expert FFN layer and chains the five C-ABI
calls (Sec. 3.3: gate -> permute -> grouped GEMM pair -> un-permute/scale).  It allocates
every buffer once; forward() only marshals pointers, so it can run in a tight loop."""
from __future__ import annotations

import torch

from . import binding as B


class MoEExpertLayer:
    def __init__(self, T, d, F, E, k, bits, group_size=0, act_dtype=torch.float16, renormalize=True,
                 y_dtype=None, out_dtype=torch.float32, device="cuda:0"):
        self.T, self.d, self.F, self.E, self.k = T, d, F, E, k
        self.bits, self.group_size, self.renormalize = bits, group_size, renormalize
        self.act_dtype, self.out_dtype = act_dtype, out_dtype
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
    def gate(self, x, finished=None):
        return B.moe_gate_topk(x, self.wg, self.gate_bias, self.k, self.renormalize,
                               out=(self.expert_idx, self.expert_scale), finished=finished)

    def permute(self, x):
        return B.moe_permute(self.expert_idx, x, self.E,
                             out=(self.x_perm, self.perm_src, self.inv_perm, self.expert_offsets),
                             workspace=self.ws_permute)

    def ffn(self):
        return B.moe_grouped_ffn_wq(self.x_perm, self.expert_offsets, self.E, self.d, self.F, self.bits,
                                    self.group_size, self.w1_packed, self.s1, self.w2_packed, self.s2,
                                    self.b1, self.b2, y_perm=self.y_perm, workspace=self.ws_ffn,
                                    max_rows_per_expert=self.T)

    def combine(self):
        return B.moe_combine(self.y_perm, self.inv_perm, self.expert_scale, self.T, self.k, out=self.out,
                             active_rows=self.expert_offsets[self.E:])

    def forward(self, x, finished=None):
        """The four per-call entry points back to back.  The argument lists are marshalled once per
        (input tensor, weight buffers, stream) and then replayed: in a decode-sized layer the
        kernels are shorter than the time Python needs to rebuild them.
        finished: uint8 [T] on the device, nonzero for rows pruned from the batch (their output
        rows are zero and their experts' weights are not read on their account)."""
        opt = lambda t: 0 if t is None else t.data_ptr()  # noqa: E731
        key = (x.data_ptr(), opt(finished), self.w1_packed.data_ptr(), self.w2_packed.data_ptr(), self.s1.data_ptr(),
               self.s2.data_ptr(), self.wg.data_ptr(), opt(self.gate_bias), opt(self.b1), opt(self.b2),
               torch.cuda.current_stream().cuda_stream)
        calls = self._plans.get(key)
        if calls is None:
            calls = self._plans[key] = self._marshal(x, finished, key[-1])
            if len(self._plans) > 256:
                self._plans.pop(next(iter(self._plans)))
        for fn, args, name in calls:
            rc = fn(*args)
            if rc != 0:
                B._check(rc, name)
        return self.out

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
        return [
            (lib.moe_gate_topk, (p(x), dt, p(self.wg), p(self.gate_bias), p(finished), self.T, self.d, self.E, self.k,
                                 int(self.renormalize), p(self.expert_idx), p(self.expert_scale), st), "moe_gate_topk"),
            (lib.moe_permute, (p(self.expert_idx), p(x), dt, self.T, self.k, self.E, self.d, p(self.x_perm),
                               p(self.perm_src), p(self.inv_perm), p(self.expert_offsets), p(self.ws_permute),
                               self.ws_permute.numel(), st), "moe_permute"),
            (lib.moe_grouped_ffn_wq, (p(self.x_perm), dt, p(self.expert_offsets), self.R, self.E, self.T, self.d,
                                      self.F, self.bits, self.group_size, p(self.w1_packed), p(self.s1), p(self.b1),
                                      p(self.w2_packed), p(self.s2), p(self.b2), p(self.y_perm), ydt,
                                      p(self.ws_ffn), self.ws_ffn.numel(), st), "moe_grouped_ffn_wq"),
            (lib.moe_combine, (p(self.y_perm), ydt, p(self.inv_perm), p(self.expert_scale), active, self.T, self.k, self.d,
                               p(self.out), odt, st), "moe_combine"),
        ]
