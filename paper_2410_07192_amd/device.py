"""Device-memory plumbing for the tests and the benchmark: PyTorch allocates HBM / pinned host
buffers and hands raw pointers to the library.  No computation happens here."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as pf


def to_device(a: np.ndarray) -> torch.Tensor:
    """NumPy array -> contiguous device tensor with the same bytes (uint16 travels as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor, dtype=None) -> np.ndarray:
    a = t.detach().cpu().numpy()
    if dtype is not None:
        a = a.view(dtype)
    return a


def storage_tensor(a: np.ndarray, md) -> torch.Tensor:
    """float32 values -> device tensor in the model's storage dtype."""
    return to_device(pf.to_storage(a, md))


def read_storage(t: torch.Tensor, md) -> np.ndarray:
    """Device tensor in the model's storage dtype -> float32 NumPy array."""
    if md.dtype == pf.PF_DTYPE_BF16:
        return pf.bf16_bits_to_f32(to_host(t, np.uint16))
    return to_host(t).astype(np.float32, copy=False)


def empty_storage(shape, md) -> torch.Tensor:
    dt = torch.int16 if md.dtype == pf.PF_DTYPE_BF16 else torch.float32
    return torch.empty(shape, dtype=dt, device="cuda")


class DeviceModel:
    """A model's parameters in the library's layout plus an execution context for one configuration."""

    def __init__(self, shape, params, g=1, streamed=False, n_slots=0, batch=None, training=False, adam=None):
        self.shape = shape
        self.md = pf.model_desc(shape, batch)
        self.cfg = pf.pf_exec_config(g, int(streamed), n_slots, int(training))
        md = self.md
        size, _ = pf.pf_layer_blob_layout(md)
        self.blobs = []
        for P in params["layers"]:
            if streamed:
                t = torch.empty(size, dtype=torch.uint8, pin_memory=True)
                pf.pack_layer_blob(md, P, out=t.numpy())
            else:
                t = torch.from_numpy(pf.pack_layer_blob(md, P)).cuda()
            self.blobs.append(t)
        self.tok = storage_tensor(params["tok_emb"], md) if shape.vocab > 0 else None
        self.pos = storage_tensor(params["pos_emb"], md) if shape.vocab > 0 else None
        self.lnf_g = storage_tensor(params["lnf_g"], md) if "lnf_g" in params else None
        self.lnf_b = storage_tensor(params["lnf_b"], md) if "lnf_b" in params else None
        self.arena_bytes = pf.pf_ctx_arena_bytes(md, self.cfg)
        self.arena = torch.empty(self.arena_bytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.ctx = pf.Context(md, self.cfg, [b.data_ptr() for b in self.blobs],
                              self.tok.data_ptr() if self.tok is not None else None,
                              self.pos.data_ptr() if self.pos is not None else None,
                              self.lnf_g.data_ptr() if self.lnf_g is not None else None,
                              self.lnf_b.data_ptr() if self.lnf_b is not None else None, base, self.arena_bytes,
                              adam)
        self.chain = pf.pf_build_chain(md, self.cfg) if not (training and shape.vocab == 0) else None
        self._io = None

    def set_io(self, inputs: torch.Tensor, n_in: int, outputs: torch.Tensor | None, n_out: int):
        self._io = (inputs, outputs)
        self.ctx.pf_ctx_set_io(inputs.data_ptr(), n_in, outputs.data_ptr() if outputs is not None else None, n_out)

    def chunk(self, begin, end):
        return pf.pf_chunk(0, 0, begin, end, 0, 0)

    def close(self):
        self.ctx.destroy()


def random_layer_blob(md, seed, pinned=False):
    """A layer blob drawn on the device (N(0, 0.02^2) everywhere, LayerNorm scales 1 + N): for the
    large benchmark workloads, where drawing and transposing on the host would take minutes.  Same
    distribution as synth.make_layer_params, different stream of random numbers."""
    size, off = pf.pf_layer_blob_layout(md)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    if md.dtype == pf.PF_DTYPE_BF16:
        n = size // 2
        vals = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        step = 1 << 26
        for a in range(0, n, step):
            b = min(n, a + step)
            vals[a:b] = (torch.randn(b - a, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        for i in (0, 6):
            vals[off[i] // 2: off[i] // 2 + md.d_model] += 1.0
        raw = vals.view(torch.uint8)
    else:
        n = size // 4
        vals = torch.randn(n, device="cuda", generator=gen) * 0.02
        for i in (0, 6):
            vals[off[i] // 4: off[i] // 4 + md.d_model] += 1.0
        raw = vals.view(torch.uint8)
    if pinned:
        host = torch.empty(size, dtype=torch.uint8, pin_memory=True)
        host.copy_(raw)
        return host
    return raw


class RawModel:
    """Like DeviceModel but from ready-made blobs and embedding tensors (device plumbing only)."""

    def __init__(self, shape, blobs, tok, pos, lnf_g, lnf_b, g=1, streamed=False, n_slots=0, training=False, adam=None):
        self.shape = shape
        self.md = pf.model_desc(shape)
        self.cfg = pf.pf_exec_config(g, int(streamed), n_slots, int(training))
        self.blobs, self.tok, self.pos, self.lnf_g, self.lnf_b = blobs, tok, pos, lnf_g, lnf_b
        self.arena_bytes = pf.pf_ctx_arena_bytes(self.md, self.cfg)
        self.arena = torch.empty(self.arena_bytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) // 256 * 256
        ptr = lambda t: t.data_ptr() if t is not None else None
        self.ctx = pf.Context(self.md, self.cfg, [b.data_ptr() for b in blobs], ptr(tok), ptr(pos), ptr(lnf_g),
                              ptr(lnf_b), base, self.arena_bytes, adam)
        self.chain = pf.pf_build_chain(self.md, self.cfg) if not (training and shape.vocab == 0) else None

    def set_io(self, inputs, n_in, outputs, n_out):
        self._io = (inputs, outputs)
        self.ctx.pf_ctx_set_io(inputs.data_ptr(), n_in, outputs.data_ptr() if outputs is not None else None, n_out)

    def close(self):
        self.ctx.destroy()
        self.arena = None
