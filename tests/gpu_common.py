"""Runs the same seeded mixed batch through the CPU oracle and through the HIP library
(via the C ABI) and hands both results to the parity tests.  Holds no arithmetic of the
method: the oracle side calls oracle/, the GPU side calls paper_2402_18789_amd."""
import numpy as np
import torch

from oracle import layer as OL
from oracle.maps import build_maps
from workload import gen
from workload.configs import KIND_FINETUNE
import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH

TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(a, b):
    """max |a - b| / max |b|  (b = oracle)"""
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = float(np.max(np.abs(b)))
    return float(np.max(np.abs(a - b))) / (den if den > 0 else 1.0)


def to_np(t):
    return t.detach().double().cpu().numpy()


class Case:
    """One layer, one pool, at most one finetune sequence; both sides in lock step."""

    def __init__(self, cfg, batch, seed=0, layer=0, kv_split_pages=0, pool_dtype=np.float64, weights=None, lora=None,
                 keep_u=True, adapters=None, gpu_page_shift=0, storage_oracle=False):
        """gpu_page_shift: the device side keeps every sequence in the physical pages `oracle page id + shift`
        of a pool that many pages larger (the oracle's results do not depend on which pages hold a
        sequence), so that a case can sit astride the 2^31-element / 4 GiB offsets of a large pool.
        storage_oracle: for a bf16 configuration, run the oracle a second time with every stored tensor rounded
        to bf16 (its own pool and state; results in last_y_s, last_dx_s, grads_s, s_ft), so that a test can tell
        error of the storage type from error of the kernels' arithmetic.
        adapters: optional list of LoRA weight sets indexed by adapter id (several adapters served in one
        batch); `lora` (default: adapter 0's seeded weights) is then adapters[ft adapter], the one trained."""
        self.cfg, self.seed, self.layer_id = cfg, seed, layer
        self.W = weights if weights is not None else gen.layer_weights(cfg, seed, layer)
        self.lora = lora if lora is not None else gen.lora_weights(cfg, seed, layer)
        self.batch = batch
        self.split = kv_split_pages
        self.shift = int(gpu_page_shift)
        # oracle state
        self.o_pool = OL.KVPool(batch.num_pages, cfg.page_size, cfg.kv_dim, dtype=pool_dtype)
        self.o_ft = {}
        self.storage = "bf16" if (storage_oracle and cfg.dtype == "bf16") else None
        self.s_pool = OL.KVPool(batch.num_pages, cfg.page_size, cfg.kv_dim, dtype=pool_dtype) if self.storage else None
        self.s_ft, self.grads_s, self.last_y_s, self.last_dx_s = {}, {}, None, None
        # device state
        self.dev = HH.DeviceLayer(cfg, self.W, self.lora)
        self.adapters_o, self.adapters_d, self._keep = None, None, []
        if adapters is not None:
            self.adapters_o, self.adapters_d = adapters, []
            for lo in adapters:
                if lo is self.lora:
                    self.adapters_d.append(self.dev.lora)        # the trained adapter: gradients land in self.dev
                else:
                    dl = HH.DeviceLora(cfg, lo)
                    self._keep.append(dl)
                    self.adapters_d.append(dl.c)
        self.d_pool = HH.DevicePool(cfg, batch.num_pages + self.shift)
        self.d_ft = {}
        for r in batch.requests:
            if r.kind == KIND_FINETUNE:
                L = batch.seq_capacity[r.seq_id]
                self.o_ft[r.seq_id] = OL.FtState(cfg, L)
                if self.storage:
                    self.s_ft[r.seq_id] = OL.FtState(cfg, L)
                self.d_ft[r.seq_id] = HH.DeviceFtState(cfg, L, keep_u=keep_u)
        self.fill_prefixes(batch)

    def dpages(self, pages):
        """device-side page ids of an oracle-side page list"""
        return (np.asarray(pages, dtype=np.int64) + self.shift).astype(np.int32)

    def fill_prefixes(self, batch):
        """Seeded K/V rows for every position already cached when the batch starts."""
        for r in batch.requests:
            if r.start_pos == 0:
                continue
            k, v = gen.kv_prefix(self.cfg, self.seed, self.layer_id, r.seq_id, r.start_pos)
            pages = batch.seq_pages[r.seq_id]
            slots = self.o_pool.slots(pages, r.start_pos)
            self.o_pool.k[slots], self.o_pool.v[slots] = k, v
            if self.storage:
                self.s_pool.k[slots], self.s_pool.v[slots] = k, v
            self.d_pool.write_rows(self.dpages(pages), k, v)

    def forward(self, batch, x, oracle=True, return_all=False):
        """-> (y_gpu, y_oracle or None, device batch)"""
        cfg = self.cfg
        db = HH.DeviceBatch(cfg, batch.requests, {sid: self.dpages(p) for sid, p in batch.seq_pages.items()},
                            batch.num_pages + self.shift, self.split)
        ws = HH.Workspace(self.dev.c, db.host_maps.T, db.host_maps.n_parts)
        dt = HH.TORCH_DTYPE[cfg.dtype]
        x_d = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda", dt)
        y_d = torch.empty_like(x_d)
        ft_seq = [r.seq_id for r in batch.requests if r.kind == KIND_FINETUNE]
        ft_c = self.d_ft[ft_seq[0]].c if ft_seq else None
        if self.adapters_d is not None:
            B.flexco_layer_forward_multi(self.dev.c, self.dev.w, self.adapters_d, db.maps, x_d, y_d, self.d_pool.c, ft_c,
                                         ws.ptr, ws.bytes)
        else:
            B.flexco_layer_forward(self.dev.c, self.dev.w, self.dev.lora, db.maps, x_d, y_d, self.d_pool.c, ft_c,
                                   ws.ptr, ws.bytes)
        torch.cuda.synchronize()
        y_o = None
        if oracle:
            om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
            y_o = OL.layer_forward_mixed(cfg, self.W, self.adapters_o if self.adapters_o is not None else self.lora, om, x,
                                         self.o_pool, self.o_ft, return_all=return_all)
            if self.storage:
                self.last_y_s = OL.layer_forward_mixed(cfg, self.W, self.adapters_o if self.adapters_o is not None else
                                                       self.lora, om, x, self.s_pool, self.s_ft, storage=self.storage)
        return to_np(y_d), y_o, db

    def backward_window(self, seq_id, win_start, win_len, dY, grads_o, need_dx=True):
        """One token-window backward step on both sides -> (dX_gpu, dX_oracle)"""
        cfg = self.cfg
        pages = self.batch.seq_pages[seq_id]
        l = win_start + win_len
        st_d, st_o = self.d_ft[seq_id], self.o_ft[seq_id]
        ws = HH.Workspace(self.dev.c, 0, 0, win_len, l)
        dt = HH.TORCH_DTYPE[cfg.dtype]
        dY_d = torch.from_numpy(np.ascontiguousarray(dY, dtype=np.float32)).to("cuda", dt)
        dX_d = torch.empty_like(dY_d) if need_dx else None
        pages_d = torch.from_numpy(self.dpages(pages)).to("cuda")
        B.flexco_lora_bwd(self.dev.c, self.dev.w, self.dev.lora, self.d_pool.c, pages_d, len(pages), st_d.c,
                          win_start, win_len, dY_d, dX_d, ws.ptr, ws.bytes)
        torch.cuda.synchronize()
        slots = self.o_pool.slots(pages, l)
        K, V = self.o_pool.k[slots].astype(np.float64), self.o_pool.v[slots].astype(np.float64)
        dX_o = OL.layer_backward_window(cfg, self.W, self.lora, st_o, K, V, win_start, win_len, dY, grads_o, need_dx)
        if self.storage:
            Ks, Vs = self.s_pool.k[slots].astype(np.float64), self.s_pool.v[slots].astype(np.float64)
            self.last_dx_s = OL.layer_backward_window(cfg, self.W, self.lora, self.s_ft[seq_id], Ks, Vs, win_start, win_len,
                                                      dY, self.grads_s, need_dx, storage=self.storage)
        return (to_np(dX_d) if need_dx else None), dX_o


def elem_err(a, b, rtol):
    """Elementwise view of the same comparison: the largest |a - b| / (atol + rtol |b|) over the elements, with
    atol = 1e-3 max|b| - at most 1 means every element is within rtol of its own reference value, up to a floor
    of a thousandth of the tensor's largest one."""
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    atol = 1e-3 * float(np.max(np.abs(b))) if b.size else 0.0
    den = atol + rtol * np.abs(b)
    den = np.where(den > 0, den, 1.0)
    return float(np.max(np.abs(a - b) / den)) if b.size else 0.0


def assert_close(name, got, ref, tol, report=None):
    e = rel_err(got, ref)
    if report is not None:
        report.append((name, e))
    assert e <= tol, "%s: max relative error %.3e > %.1e" % (name, e, tol)
    return e


STORAGE_SLACK = 1.5


def assert_close_storage(name, got, ref, ref_storage, tol, report=None, slack=STORAGE_SLACK):
    """The bar is `tol` against the plain oracle.  A bf16 tensor may miss it only as far as the storage type itself
    does: `ref_storage` is the oracle's result with EXACT (fp64) arithmetic and every stored tensor rounded to
    bf16 where the device rounds.  Its distance from the plain oracle is what no implementation with this storage
    type can be expected to beat on this tensor; a device result beyond `tol` must be no further from the plain
    oracle than `slack` times that distance (both are maxima over a tensor of rounding effects of the same
    law, hence a factor and not equality; observed factors: 0.7 .. 1.46).
    (A bound of the device result against `ref_storage` itself cannot be tight: two correct implementations
    that differ only in the last bits of their accumulations round a fraction of the stored elements to
    different neighbours, and differ from each other by up to 8e-3 on the cases that need this rule.)
    -> (error vs plain, error of the storage oracle vs plain or None)"""
    e = rel_err(got, ref)
    es = rel_err(ref_storage, ref) if ref_storage is not None else None
    if report is not None:
        report.append((name, e) if es is None else (name, e, es))
    if e <= tol:
        return e, es
    assert es is not None, "%s: max relative error %.3e > %.1e" % (name, e, tol)
    assert e <= slack * es, "%s: max relative error %.3e > %.1e, and > %.2f x %.3e (what bf16 storage with exact " \
                            "arithmetic costs here)" % (name, e, tol, slack, es)
    return e, es
