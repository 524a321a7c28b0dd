"""Device-memory owners for the flexco library: weights, KV pool, finetune state, batches.

PyTorch is used for allocation, host<->device copies and layout staging of INPUTS only
(packing [out, in] weight blocks, scattering seeded prefix rows into pages).  Nothing of
the layer's computation happens here.
"""
import ctypes as C

import numpy as np
import torch

from . import binding as B

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
DTYPE_CODE = {"f32": B.FLEXCO_F32, "bf16": B.FLEXCO_BF16}


def c_cfg(cfg):
    mask = sum(1 << B.TARGET_NAMES.index(t) for t in cfg.lora_targets)
    return B.LayerCfg(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, DTYPE_CODE[cfg.dtype],
                      cfg.page_size, cfg.lora_rank if mask else 0, mask, cfg.rms_eps, cfg.rope_theta, cfg.lora_scale)


def _dev(a, dtype, device):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dtype).contiguous()


class ParamArena:
    """One flat parameter buffer and one flat gradient buffer for the bypass matrices of many layers, so that an
    optimizer step over all of them is a single flexco_adam_step call (and zeroing the gradients a single fill).
    Pieces are handed out 16-byte aligned (the library's alignment rule for every matrix)."""

    def __init__(self, n_elems, dtype, device="cuda"):
        self.param = torch.zeros(n_elems, dtype=dtype, device=device)
        self.grad = torch.zeros(n_elems, dtype=torch.float32, device=device)
        self.used = 0

    @staticmethod
    def padded(n):
        return (n + 7) // 8 * 8            # 8 bf16 elements = 16 bytes; keeps the fp32 pieces aligned as well

    def take(self, shape):
        n = int(np.prod(shape))
        o = self.used
        assert o + n <= self.param.numel(), "parameter arena is full"
        self.used = o + self.padded(n)
        return self.param[o:o + n].view(*shape), self.grad[o:o + n].view(*shape)


def lora_param_elems(cfg):
    """elements (padded per matrix) one adapter of this configuration takes in a ParamArena"""
    n = 0
    for t in cfg.lora_targets:
        i_, o_ = B.target_dims_py(cfg, t)
        n += ParamArena.padded(cfg.lora_rank * i_) + ParamArena.padded(o_ * cfg.lora_rank)
    return n


class DeviceLora:
    """One LoRA adapter and its gradient buffers on the GPU.  lora: {target: (A [in, r], B [r, out])} in the
    paper's orientation (stored transposed: A [r, in], B [out, r]).  arena: a ParamArena the matrices and their
    gradients are carved from instead of tensors of their own."""

    def __init__(self, cfg, lora, device="cuda", arena=None):
        dt = TORCH_DTYPE[cfg.dtype]
        self.c = B.Lora()
        self.A, self.Bm, self.dA, self.dB = {}, {}, {}, {}
        for t in cfg.lora_targets:
            i = B.TARGET_NAMES.index(t)
            A, Bm = lora[t]
            if arena is None:
                self.A[t] = _dev(np.ascontiguousarray(A.T), dt, device)      # [r, in]
                self.Bm[t] = _dev(np.ascontiguousarray(Bm.T), dt, device)    # [out, r]
                self.dA[t] = torch.zeros(self.A[t].shape, dtype=torch.float32, device=device)
                self.dB[t] = torch.zeros(self.Bm[t].shape, dtype=torch.float32, device=device)
            else:
                self.A[t], self.dA[t] = arena.take(A.T.shape)
                self.Bm[t], self.dB[t] = arena.take(Bm.T.shape)
                self.A[t].copy_(_dev(np.ascontiguousarray(A.T), dt, device))
                self.Bm[t].copy_(_dev(np.ascontiguousarray(Bm.T), dt, device))
            self.c.A[i], self.c.B[i] = self.A[t].data_ptr(), self.Bm[t].data_ptr()
            self.c.dA[i], self.c.dB[i] = self.dA[t].data_ptr(), self.dB[t].data_ptr()


class DeviceIa3:
    """One (IA)^3 adapter and its gradient buffers on the GPU.  ia3: {"k", "v": [nkv d], "ff": [F]}."""

    def __init__(self, cfg, ia3, device="cuda"):
        dt = TORCH_DTYPE[cfg.dtype]
        self.l = {n: _dev(ia3[n], dt, device) for n in ("k", "v", "ff")}
        self.dl = {n: torch.zeros(self.l[n].shape, dtype=torch.float32, device=device) for n in ("k", "v", "ff")}
        self.c = B.Ia3(self.l["k"].data_ptr(), self.l["v"].data_ptr(), self.l["ff"].data_ptr(),
                       self.dl["k"].data_ptr(), self.dl["v"].data_ptr(), self.dl["ff"].data_ptr())

    def zero_grads(self):
        for t in self.dl.values():
            t.zero_()


class DeviceLayer:
    """Frozen weights (+ one LoRA adapter and its gradient buffers) of one layer on the GPU.
    W: {wq, wk, wv, wo, wg, wu, wd [out, in], g1, g2, optional bq, bk, bv};
    lora: {target: (A [in, r], B [r, out])} in the paper's orientation (stored transposed)."""

    def __init__(self, cfg, W, lora=None, device="cuda", arena=None):
        self.cfg = cfg
        self.c = c_cfg(cfg)
        dt = TORCH_DTYPE[cfg.dtype]
        self.dtype = dt
        self.t = {
            "wqkv": _dev(np.concatenate([W["wq"], W["wk"], W["wv"]], axis=0), dt, device),
            "wo": _dev(W["wo"], dt, device),
            "wgu": _dev(np.concatenate([W["wg"], W["wu"]], axis=0), dt, device),
            "wd": _dev(W["wd"], dt, device),
            "g1": _dev(W["g1"], dt, device), "g2": _dev(W["g2"], dt, device),
        }
        if "bq" in W:
            self.t["bqkv"] = _dev(np.concatenate([W["bq"], W["bk"], W["bv"]]), dt, device)
        self.w = B.BaseWeights(self.t["wqkv"].data_ptr(), self.t["bqkv"].data_ptr() if "bqkv" in self.t else None,
                               self.t["wo"].data_ptr(), self.t["wgu"].data_ptr(), self.t["wd"].data_ptr(),
                               self.t["g1"].data_ptr(), self.t["g2"].data_ptr())
        self.lora = None
        self.A, self.Bm, self.dA, self.dB = {}, {}, {}, {}
        if lora and cfg.lora_targets:
            dl = DeviceLora(cfg, lora, device, arena)
            self.lora, self.A, self.Bm, self.dA, self.dB = dl.c, dl.A, dl.Bm, dl.dA, dl.dB

    def zero_grads(self):
        for t in self.dA:
            self.dA[t].zero_()
            self.dB[t].zero_()

    def grads_numpy(self):
        """{target: (dA [in, r], dB [r, out])} in the paper's orientation, float64"""
        return {t: (self.dA[t].double().cpu().numpy().T.copy(), self.dB[t].double().cpu().numpy().T.copy())
                for t in self.dA}


class DevicePool:
    """Paged KV cache of one layer: K [P, nkv, ps, d], V [P, nkv, d, ps]."""

    def __init__(self, cfg, num_pages, device="cuda"):
        self.cfg, self.num_pages = cfg, num_pages
        dt = TORCH_DTYPE[cfg.dtype]
        self.k = torch.zeros((num_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim), dtype=dt, device=device)
        self.v = torch.zeros((num_pages, cfg.n_kv_heads, cfg.head_dim, cfg.page_size), dtype=dt, device=device)
        self.c = B.KVPool(self.k.data_ptr(), self.v.data_ptr(), num_pages, cfg.page_size)

    def fill_random(self, seed):
        """N(0, 1) in every slot of every page (device generator): stands in for cached prefixes
        whose values no check reads."""
        g = torch.Generator(device=self.k.device)
        g.manual_seed(seed)
        for t in (self.k, self.v):
            flat = t.view(-1)
            step = 1 << 28
            for o in range(0, flat.numel(), step):
                n = min(step, flat.numel() - o)
                flat[o:o + n] = torch.randn(n, generator=g, device=t.device, dtype=torch.float32).to(t.dtype)

    def _idx(self, pages, n, start=0):
        p = torch.arange(start, start + n, device=self.k.device)
        pg = torch.as_tensor(np.asarray(pages, dtype=np.int64), device=self.k.device)[p // self.cfg.page_size]
        return pg, p % self.cfg.page_size

    def write_rows(self, pages, k_rows, v_rows, start=0):
        """Stage logical rows [n, nkv*d] (numpy or tensor) at positions start.. of a sequence."""
        cfg = self.cfg
        n = k_rows.shape[0]
        if n == 0:
            return
        pg, off = self._idx(pages, n, start)
        tk = torch.as_tensor(k_rows).to(device=self.k.device, dtype=self.k.dtype).view(n, cfg.n_kv_heads, cfg.head_dim)
        tv = torch.as_tensor(v_rows).to(device=self.k.device, dtype=self.k.dtype).view(n, cfg.n_kv_heads, cfg.head_dim)
        self.k[pg, :, off, :] = tk
        self.v[pg, :, :, off] = tv

    def read_rows(self, pages, n, start=0):
        pg, off = self._idx(pages, n, start)
        k = self.k[pg, :, off, :].reshape(n, -1).double().cpu().numpy()
        v = self.v[pg, :, :, off].reshape(n, -1).double().cpu().numpy()
        return k, v


class DeviceFtState:
    def __init__(self, cfg, L, device="cuda", keep_u=True, ia3=False):
        dt = TORCH_DTYPE[cfg.dtype]
        z = lambda w, d=dt: torch.zeros((L, w), dtype=d, device=device)
        self.L = L
        self.q_cache, self.attn = z(cfg.q_dim), z(cfg.q_dim)
        self.x, self.x2 = z(cfg.hidden), z(cfg.hidden)
        self.gate, self.up = z(cfg.ffn), z(cfg.ffn)
        self.lse = z(cfg.n_q_heads, torch.float32)
        self.dk_accum, self.dv_accum = z(cfg.kv_dim, torch.float32), z(cfg.kv_dim, torch.float32)
        self.c = B.FtState(L, self.q_cache.data_ptr(), self.x.data_ptr(), self.x2.data_ptr(), self.gate.data_ptr(),
                           self.up.data_ptr(), self.attn.data_ptr(), self.lse.data_ptr(), self.dk_accum.data_ptr(),
                           self.dv_accum.data_ptr())
        # rank-r products x_t A_t^T of the forward pass, kept for the backward pass
        self.u = {}
        if keep_u and cfg.lora_targets:
            for t in cfg.lora_targets:
                self.u[t] = z(cfg.lora_rank, torch.float32)
                self.c.saved_u[B.TARGET_NAMES.index(t)] = self.u[t].data_ptr()

        # unscaled key / value rows: the other operand of the (IA)^3 products
        if ia3:
            self.k0, self.v0 = z(cfg.kv_dim), z(cfg.kv_dim)
            self.c.saved_k0, self.c.saved_v0 = self.k0.data_ptr(), self.v0.data_ptr()

    def zero_accum(self):
        self.dk_accum.zero_()
        self.dv_accum.zero_()


class DeviceBatch:
    """Index maps of a mixed batch: built on the host by the library, uploaded in one copy."""

    def __init__(self, cfg, requests, seq_pages, num_pages, kv_split_pages=0, device="cuda"):
        self.desc, self._keep = B.make_batch_desc([r.kind for r in requests], [r.start_pos for r in requests],
                                                  [r.n_new for r in requests], [r.adapter for r in requests],
                                                  [seq_pages[r.seq_id] for r in requests])
        self.host_maps, self.blob = B.flexco_build_maps(self.desc, cfg.page_size, num_pages, cfg.n_q_heads,
                                                        cfg.n_kv_heads, kv_split_pages)
        self.dev_blob = None
        self.maps = None
        if device is not None:
            self.dev_blob = torch.from_numpy(self.blob).to(device)
            self.maps = B.flexco_maps_rebase(self.host_maps, self.blob, self.dev_blob)

    def numpy(self):
        return B.maps_to_numpy(self.host_maps, self.blob)


class Workspace:
    def __init__(self, cfg_c, T_max, n_parts_max, win_max=0, kv_max=0, device="cuda"):
        self.bytes = B.flexco_workspace_bytes(cfg_c, T_max, n_parts_max, win_max, kv_max)
        self.buf = torch.empty(max(self.bytes, 256), dtype=torch.uint8, device=device)

    @property
    def ptr(self):
        return self.buf.data_ptr()
