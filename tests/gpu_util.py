"""Test-side glue for the HIP path: numpy <-> device tensors and calls through the C-ABI binding.

Holds no arithmetic of the method: it moves seeded inputs to the device, calls libdsk, and brings
results back as numpy arrays."""
import numpy as np
import torch

from paper_2411_02820_amd import binding as B
from paper_2411_02820_amd import synth


def torch_dtype(shape):
    return torch.float32 if shape.dtype == "f32" else torch.bfloat16


def to_dev(a, shape, pinned=False):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch_dtype(shape))
    if pinned:
        p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        p.copy_(t)
        return p
    return t.cuda()


def to_np(t):
    return t.detach().float().cpu().numpy()


class GpuModel:
    def __init__(self, shape: synth.ModelShape, max_tokens: int, max_kv_rows: int = None):
        self.shape = shape
        self.handle = B.dsk_model_create(B.config_from_shape(shape), max_tokens,
                                         max_tokens if max_kv_rows is None else max_kv_rows)

    def close(self):
        if self.handle:
            B.dsk_model_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def load_from_generator(self, seed, layers=None, scale=None):
        """Uploads host-generated tensors (the same arrays the oracle gets)."""
        moe = self.shape.n_experts > 0
        for l in (range(self.shape.n_layers) if layers is None else layers):
            for kind in ((synth.G1, synth.WQ, synth.WK, synth.WV, synth.WO, synth.G2, synth.WR) if moe else range(9)):
                w = synth.layer_tensor(self.shape, seed, l, kind)
                if scale is not None and kind not in (synth.G1, synth.G2):
                    w = w * np.float32(scale)
                B.dsk_model_set_tensor(self.handle, l, kind, to_dev(w, self.shape))
            for e in range(self.shape.n_experts):
                for kind in (synth.WG, synth.WU, synth.WD):
                    w = synth.expert_tensor(self.shape, seed, l, e, kind)
                    if scale is not None:
                        w = w * np.float32(scale)
                    B.dsk_model_set_tensor(self.handle, l, B.DSK_EXPERT(e, kind), to_dev(w, self.shape))
        torch.cuda.synchronize()

    def init_random(self, seed, std=synth.WEIGHT_STD):
        B.dsk_model_init_random(self.handle, seed, std)
        torch.cuda.synchronize()

    def get_tensor(self, layer, kind, expert=None):
        out = torch.empty(self.shape.tensor_shape(kind), dtype=torch_dtype(self.shape), device="cuda")
        B.dsk_model_get_tensor(self.handle, layer, kind if expert is None else B.DSK_EXPERT(expert, kind), out)
        torch.cuda.synchronize()
        return out

    def new_cache(self, n_rows, fill=None):
        s = self.shape
        t = torch.empty((s.n_layers, 2, n_rows, s.n_kv_heads, s.head_dim), dtype=torch_dtype(s), device="cuda")
        if fill is not None:
            t.fill_(fill)
        return t

    def partial(self, hidden_in, lo, hi, kv_reused, lens, kv_out=None, n_rows=None, positions=None,
                want_hidden=True, flags=0, stream=None):
        """hidden_in / kv_reused: device or pinned tensors (or None for kv_reused).  Returns (kv_out, hidden_out)."""
        cu = synth.cu_seqlens(lens)
        T = int(cu[-1])
        pos = synth.packed_positions(lens) if positions is None else positions
        batch = B.Batch(cu, pos)
        if kv_out is None:
            kv_out = self.new_cache(T if n_rows is None else n_rows, fill=float("nan"))
        hidden_out = torch.empty((T, self.shape.hidden), dtype=torch_dtype(self.shape), device="cuda") if want_hidden else None
        B.dsk_partial_prefill(self.handle, hidden_in, lo, hi, None if kv_reused is None else B.kv_desc(kv_reused),
                              B.kv_desc(kv_out), batch.desc, hidden_out, flags, stream)
        self._keep = (batch, hidden_in, kv_reused)
        return kv_out, hidden_out

    def partial_groups(self, groups, kv_reused, lens, kv_out=None, flags=0, stream=None):
        """groups: list of (lo, hi, hidden_in tensor).  Returns (kv_out, [hidden_out per group])."""
        cu = synth.cu_seqlens(lens)
        T = int(cu[-1])
        batch = B.Batch(cu, synth.packed_positions(lens))
        if kv_out is None:
            kv_out = self.new_cache(T, fill=float("nan"))
        outs = [torch.empty((T, self.shape.hidden), dtype=torch_dtype(self.shape), device="cuda") for _ in groups]
        B.dsk_partial_prefill_groups(self.handle, [(lo, hi, h, o) for (lo, hi, h), o in zip(groups, outs)],
                                     None if kv_reused is None else B.kv_desc(kv_reused), B.kv_desc(kv_out),
                                     batch.desc, flags, stream)
        self._keep = (batch, groups, kv_reused)
        return kv_out, outs

    def suffix(self, suffix_hidden_in, kv, lens, slens, suffix_row0=None, stream=None):
        cu, cus = synth.cu_seqlens(lens), synth.cu_seqlens(slens)
        spos = synth.packed_positions(slens, start=lens)
        pb, sb = B.Batch(cu), B.Batch(cus, spos)
        row0 = int(cu[-1]) if suffix_row0 is None else suffix_row0
        out = torch.empty((int(cus[-1]), self.shape.hidden), dtype=torch_dtype(self.shape), device="cuda")
        B.dsk_suffix_prefill(self.handle, suffix_hidden_in, B.kv_desc(kv), pb.desc, sb.desc, row0, out, stream)
        self._keep2 = (pb, sb, suffix_hidden_in)
        return out
