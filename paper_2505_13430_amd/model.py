"""Device-memory plumbing around the C ABI: uploads a tensor table, owns the
scale arena and the workspace, and forwards to the binding.  No arithmetic of
the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as qb
from . import synth


class DeviceModel:
    """A model bound to device tensors.  `tensors` follow qzo_model_create's
    order: bf16 tensors for the fixed parts, uint8 [N, K/2] for packed int4."""

    def __init__(self, shape: dict, tensors, scale_arena: torch.Tensor):
        self.shape = dict(shape)
        self.tensors = tensors
        self.scales = scale_arena
        self.handle = qb.qzo_model_create(shape, tensors, scale_arena)
        self._ws = None
        self._ws_key = None
        self.result = torch.zeros(8, dtype=torch.int32, device=scale_arena.device)
        self.loss = torch.zeros(2, dtype=torch.float32, device=scale_arena.device)
        self.dense_master = None

    @classmethod
    def from_host(cls, shape: dict, host_tensors, host_scales, device="cuda:0"):
        """host_tensors: numpy fp32 arrays holding bf16-exact values, or uint8
        packed weights; host_scales: fp32 array of bf16-exact scales."""
        dev = []
        for a in host_tensors:
            t = torch.from_numpy(np.ascontiguousarray(a))
            dev.append(t.to(device) if t.dtype in (torch.uint8, torch.int32) else t.to(device).to(torch.bfloat16))
        arena = torch.from_numpy(np.ascontiguousarray(host_scales, dtype=np.float32)).to(device).to(
            torch.float16 if shape.get("scale_fp16") else torch.bfloat16)
        return cls(shape, dev, arena)

    @classmethod
    def from_host_codebook(cls, shape: dict, table, device="cuda:0"):
        """Codebook variant.  table: (name, kind, array) with kind 'bf16' (fp32 holding bf16
        values), 'codes' (uint16 [N,K/8]), 'codebook' (fp32 holding fp16 values, [65536,8]) or
        'chscale' (fp32 holding fp16 values, [N]); channel scales form the fp16 arena."""
        dev, scales = [], []
        for _, kind, a in table:
            a = np.ascontiguousarray(a)
            if kind == "chscale":
                scales.append(a.reshape(-1))
            elif kind == "codes":
                dev.append(torch.from_numpy(a.view(np.int16)).to(device))
            elif kind == "codebook":
                dev.append(torch.from_numpy(a).to(device).to(torch.float16))
            else:
                dev.append(torch.from_numpy(a).to(device).to(torch.bfloat16))
        arena = torch.from_numpy(np.concatenate(scales).astype(np.float32)).to(device).to(torch.float16)
        return cls(dict(shape, quant=1), dev, arena)

    @classmethod
    def synthetic(cls, shape: dict, seed: int, device="cuda:0", asym=False, nf4=False):
        """Random-init model built on the device: weights ~ N(0, 0.02) drawn by
        torch, quantized by the library's RTN kernel (Eq. 3), tensor by tensor.
        asym: the zero-point variant (quant = 2) as the 4-bit checkpoints of Sec. 4.1 hold it: the
        library's asymmetric RTN kernel gives every group a zero-point and an fp16 scale (each
        output row's weights are shifted by up to 0.03 so that the zero-points spread)."""
        if asym:
            shape = dict(shape, quant=2, scale_fp16=1)
        if nf4:
            # NormalFloat-4: uniform random level indices, block-64 scales ~ U(0.03, 0.09) (the absmax
            # of 64 weights ~ N(0, 0.02)): the shapes, sizes and work of such a checkpoint
            shape = dict(shape, quant=3, group=64)
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        d, V = shape["d_model"], shape["vocab"]
        llama = shape["arch"] == "llama"
        n_scales = qb.qzo_model_scale_count(shape)
        arena = torch.empty(n_scales, dtype=torch.float16 if asym else torch.bfloat16, device=device)
        off = 0

        def fixed(*sz, mean=0.0, std=0.02):
            return (torch.randn(*sz, generator=gen, device=device) * std + mean).to(torch.bfloat16)

        def quant(N, K):
            nonlocal off
            if nf4:
                n = N * (K // 64)
                arena[off:off + n] = (torch.rand(n, generator=gen, device=device) * 0.06 + 0.03).to(torch.bfloat16)
                off += n
                return [torch.randint(0, 256, (N, K // 2), generator=gen, device=device, dtype=torch.uint8)]
            w = torch.randn(N, K, generator=gen, device=device) * 0.02
            q = torch.empty(N, K // 2, dtype=torch.uint8, device=device)
            n = N * (K // 128)
            if asym:
                w += 0.03 * torch.sin(torch.arange(N, device=device, dtype=torch.float32))[:, None]
                zp = torch.empty(N, K // 128, dtype=torch.uint8, device=device)
                qb.qzo_rtn_quantize_asym(w, q, zp, arena[off:off + n].view(N, K // 128))
                off += n
                return [q, zp]
            qb.qzo_rtn_quantize(w, q, arena[off:off + n].view(N, K // 128))
            off += n
            return [q]

        tensors = [fixed(V, d)]
        if not llama:
            tensors.append(fixed(shape["max_seq"], d))
        lin = synth.quantized_linears(shape)
        for _ in range(shape["n_layers"]):
            if llama:
                tensors += ([fixed(d, mean=1.0, std=0.1)] + quant(*lin[0][1:]) + quant(*lin[1][1:]) +
                            [fixed(d, mean=1.0, std=0.1)] + quant(*lin[2][1:]) + quant(*lin[3][1:]))
            else:
                tensors += ([fixed(d, mean=1.0, std=0.1), fixed(d)] + quant(*lin[0][1:]) +
                            [fixed(lin[0][1])] + quant(*lin[1][1:]) + [fixed(d)] +
                            [fixed(d, mean=1.0, std=0.1), fixed(d)] + quant(*lin[2][1:]) +
                            [fixed(lin[2][1])] + quant(*lin[3][1:]) + [fixed(d)])
        tensors.append(fixed(d, mean=1.0, std=0.1))
        if not llama:
            tensors.append(fixed(d))
        tensors.append(fixed(V, d))
        torch.cuda.synchronize()
        assert off == n_scales
        return cls(shape, tensors, arena)

    @classmethod
    def synthetic_codebook(cls, shape: dict, seed: int, device="cuda:0"):
        """Random-init codebook-variant model built on the device: uniform 16-bit codes,
        one fp16 [65536, 8] codebook ~ N(0, 0.02) per linear, fp16 channel scales ~ U(0.5, 1.5)."""
        assert shape["arch"] == "llama"
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        d, V = shape["d_model"], shape["vocab"]
        cfg = dict(shape, quant=1)
        arena = (torch.rand(qb.qzo_model_scale_count(cfg), generator=gen, device=device) + 0.5).to(torch.float16)

        def fixed(*sz, mean=0.0, std=0.02):
            return (torch.randn(*sz, generator=gen, device=device) * std + mean).to(torch.bfloat16)

        def lin(N, K):
            codes = torch.randint(-32768, 32768, (N, K // 8), generator=gen, device=device, dtype=torch.int16)
            cb = (torch.randn(65536, 8, generator=gen, device=device) * 0.02).to(torch.float16)
            return [codes, cb]

        tensors = [fixed(V, d)]
        ql = synth.quantized_linears(shape)
        for _ in range(shape["n_layers"]):
            tensors += [fixed(d, mean=1.0, std=0.1)] + lin(*ql[0][1:]) + lin(*ql[1][1:])
            tensors += [fixed(d, mean=1.0, std=0.1)] + lin(*ql[2][1:]) + lin(*ql[3][1:])
        tensors += [fixed(d, mean=1.0, std=0.1), fixed(V, d)]
        torch.cuda.synchronize()
        return cls(cfg, tensors, arena)

    def workspace(self, batch, seq):
        if self._ws_key != (batch, seq):
            n = qb.qzo_workspace_bytes(self.handle, batch, seq)
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.scales.device)
            self._ws_key = (batch, seq)
        return self._ws

    def forward_loss(self, tokens, seed, eps, sign, stream=None) -> torch.Tensor:
        ws = self.workspace(*tokens.shape)
        out = self.loss[0:1] if sign > 0 else self.loss[1:2]
        qb.qzo_forward_loss(self.handle, tokens, seed, eps, sign, ws, out, stream)
        return out

    def step(self, tokens, seed, eps, eta, clip, stream=None) -> torch.Tensor:
        ws = self.workspace(*tokens.shape)
        qb.qzo_step(self.handle, tokens, seed, eps, eta, clip, ws, self.result, stream)
        return self.result

    def enable_joint(self):
        """Joint mode: an fp32 master of every 16-bit tensor (table order), copied from the tensors;
        from here on the library rewrites those tensors from the master."""
        parts = [t.reshape(-1) for t in self.tensors if t.dtype in (torch.bfloat16, torch.float16)]
        self.dense_master = torch.cat(parts).to(torch.float32)       # a copy: dtype conversion only
        assert self.dense_master.numel() == qb.qzo_model_dense_count(self.shape)
        self.joint_table = torch.empty(qb.qzo_model_joint_table_bytes(self.shape), dtype=torch.uint8,
                                       device=self.scales.device)
        qb.qzo_model_enable_joint(self.handle, self.dense_master, self.joint_table)
        self._ws = None                                              # the workspace layout may differ
        self._ws_key = None
        return self.dense_master

    def step_joint(self, tokens, seed, eps, eta, eta_dense, clip, stream=None) -> torch.Tensor:
        ws = self.workspace(*tokens.shape)
        qb.qzo_step_joint(self.handle, tokens, seed, eps, eta, eta_dense, clip, ws, self.result, stream)
        return self.result

    def set_int4_path(self, mode: int):
        """0: by token count, 1: always the fused kernel, 2: always expand-then-multiply."""
        qb.qzo_model_set_int4_path(self.handle, mode)
        self._ws = None                                              # the workspace layout depends on it
        self._ws_key = None

    def apply_update(self, seed, eta, d_clipped, stream=None):
        qb.qzo_model_apply_update(self.handle, seed, eta, d_clipped, stream)

    def close(self):
        if self.handle is not None:
            qb.qzo_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
