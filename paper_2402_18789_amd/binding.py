"""ctypes binding of libflexco.so: the same names as include/flexco.h, argument marshalling only.

Every step of the layer runs inside the library's HIP kernels; PyTorch tensors are used
here only as owners of device memory (data_ptr) and for the current stream handle.
There is no fallback: if the shared library is missing, importing fails loudly.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  loaded first: the library shares torch's HIP runtime (libamdhip64.so)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FLEXCO_LIB_PATH", os.path.join(_HERE, "libflexco.so"))
# FLEXCO_HOST_ONLY=1: the library at FLEXCO_LIB_PATH is a build of the host sources alone (index maps, scheduler,
# graph pruning; see build.py --host-sanitized): only the symbols it has are bound, calling a device entry point fails
HOST_ONLY = os.environ.get("FLEXCO_HOST_ONLY") == "1"

FLEXCO_OK, FLEXCO_EINVAL, FLEXCO_ESHAPE, FLEXCO_EWORKSPACE, FLEXCO_EPAGE, FLEXCO_EUNSUPPORTED, FLEXCO_EHIP = \
    0, -1, -2, -3, -4, -5, -6
FLEXCO_F32, FLEXCO_BF16 = 0, 1
FLEXCO_DECODE, FLEXCO_PREFILL, FLEXCO_FINETUNE = 0, 1, 2
FLEXCO_REQ_WAITING, FLEXCO_REQ_RUNNING, FLEXCO_REQ_FINISHED = 0, 1, 2
TARGET_NAMES = ("q", "k", "v", "o", "gate", "up", "down")
N_TARGETS = 7
ABI_VERSION = 8


class FlexcoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("flexco error %d: %s" % (code, msg))
        self.code = code


class LayerCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "dtype",
                                         "page_size", "lora_rank", "lora_targets")] + \
               [(n, C.c_float) for n in ("rms_eps", "rope_theta", "lora_scale")]


class BaseWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wqkv", "bqkv", "wo", "wgu", "wd", "g1", "g2")]


class Lora(C.Structure):
    _fields_ = [("A", C.c_void_p * N_TARGETS), ("B", C.c_void_p * N_TARGETS),
                ("dA", C.c_void_p * N_TARGETS), ("dB", C.c_void_p * N_TARGETS)]


class BatchDesc(C.Structure):
    _fields_ = [("n_req", C.c_int32)] + [(n, C.POINTER(C.c_int32)) for n in
                                         ("kind", "start_pos", "n_new", "adapter", "req_page_off", "req_pages")]


_MAP_SCALARS = ("T", "n_req", "n_ft", "n_seg", "max_pages", "page_size", "n_tiles", "n_items", "n_parts",
                "tile_tokens", "kv_split_pages", "ft_req", "ft_tok0", "ft_pos0", "n_lora", "max_kv_len", "blob_ints", "n_adapters", "ft_adapter",
                "num_pages", "n_single", "stream_pages", "chunk_tile_pages")
_MAP_ARRAYS = ("tok_req", "tok_pos", "slot", "req_tok_off", "req_kv_len", "req_kind", "block_table", "ft_tok",
               "seg_off", "seg_adapter", "lora_tok", "tile_req", "tile_tok0", "tile_ntok", "tile_nsplit",
               "tile_part0", "item_tile", "item_split", "tok_tile", "tok_lora", "tok_adapter", "item_ntiles")
MAX_ADAPTERS = 8


class Maps(C.Structure):
    _fields_ = [(n, C.c_int32) for n in _MAP_SCALARS] + [("adapter_tok_off", C.c_int32 * (MAX_ADAPTERS + 1))] + \
               [(n, C.c_void_p) for n in _MAP_ARRAYS]


class KVPool(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("num_pages", C.c_int32), ("page_size", C.c_int32)]


class FtState(C.Structure):
    _fields_ = [("seq_len", C.c_int32)] + [(n, C.c_void_p) for n in
                                           ("q_cache", "saved_x", "saved_x2", "saved_gate", "saved_up", "saved_attn",
                                            "lse", "dk_accum", "dv_accum")] + [("saved_u", C.c_void_p * 7)] + \
               [("saved_k0", C.c_void_p), ("saved_v0", C.c_void_p)]


class Adapter(C.Structure):
    _fields_ = [("bottleneck", C.c_int32), ("w_down", C.c_void_p), ("w_up", C.c_void_p), ("dw_down", C.c_void_p),
                ("dw_up", C.c_void_p)]


class Ia3(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("l_k", "l_v", "l_ff", "dl_k", "dl_v", "dl_ff")]


class Graph(C.Structure):
    _fields_ = [("n_ops", C.c_int32), ("n_tensors", C.c_int32)] + [(n, C.c_void_p) for n in
                ("op_kind", "op_cheap", "op_in_off", "op_in", "op_out", "tensor_class", "need_grad")]


OP_KINDS = {"source": 0, "matmul": 1, "add": 2, "rmsnorm": 3, "rope": 4, "attention": 5, "swiglu": 6, "mul": 7, "relu": 8}
TENSOR_ACTIVATION, TENSOR_FROZEN, TENSOR_TRAINABLE = 0, 1, 2
KEEP_NONE, KEEP_STORE, KEEP_REMAT, KEEP_BITMASK = 0, 1, 2, 3


class ModelLayer(C.Structure):
    _fields_ = [("w", BaseWeights), ("lora", C.c_void_p), ("pool", KVPool), ("ft", C.c_void_p)]


class LmHead(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("g_final", C.c_void_p), ("w_lm", C.c_void_p)]


class LatencyModel(C.Structure):
    _fields_ = [("n_c", C.c_int32), ("n_s", C.c_int32), ("c_grid", C.c_void_p), ("s_grid", C.c_void_p),
                ("ms", C.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libflexco.so is not built: run `python paper_2402_18789_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.flexco_last_error.restype = C.c_char_p
    lib.flexco_abi_version.restype = C.c_int32
    if lib.flexco_abi_version() != ABI_VERSION:
        raise ImportError("libflexco.so has ABI version %d, binding expects %d" % (lib.flexco_abi_version(), ABI_VERSION))
    P = C.POINTER
    i32, vp, sz, f32 = C.c_int32, C.c_void_p, C.c_size_t, C.c_float
    sigs = {
        "flexco_maps_blob_ints": [P(BatchDesc), i32, i32, i32, i32, P(sz)],
        "flexco_build_maps": [P(BatchDesc), i32, i32, i32, i32, i32, vp, sz, P(Maps)],
        "flexco_maps_rebase": [P(Maps), vp, vp, P(Maps)],
        "flexco_workspace_bytes": [P(LayerCfg), i32, i32, i32, i32, P(sz)],
        "flexco_layer_forward": [P(LayerCfg), P(BaseWeights), P(Lora), P(Maps), vp, vp, P(KVPool), P(FtState), vp, sz, vp],
        "flexco_layer_forward_multi": [P(LayerCfg), P(BaseWeights), P(Lora), i32, P(Maps), vp, vp, P(KVPool), P(FtState), vp,
                                       sz, vp],
        "flexco_layer_forward_ia3": [P(LayerCfg), P(BaseWeights), P(Ia3), P(Maps), vp, vp, P(KVPool), P(FtState), vp, sz, vp],
        "flexco_ia3_bwd": [P(LayerCfg), P(BaseWeights), P(Ia3), P(KVPool), vp, i32, P(FtState), i32, i32, vp, vp, vp, sz, vp],
        "flexco_adapter_workspace_bytes": [i32, i32, i32, i32, i32, P(sz)],
        "flexco_adapter_fwd": [i32, i32, P(Adapter), P(Maps), vp, vp, i32, vp, sz, vp],
        "flexco_adapter_bwd": [i32, i32, P(Adapter), vp, i32, i32, i32, vp, vp, sz, vp],
        "flexco_attention_mixed": [P(LayerCfg), P(Maps), vp, P(KVPool), vp, vp, vp, sz, vp],
        "flexco_lora_fwd": [vp, vp, i32, i32, i32, i32, f32, i32, P(vp), P(vp), i32, P(i32), P(i32), i32, vp, vp],
        "flexco_lora_fwd_static": [vp, vp, i32, i32, i32, i32, f32, i32, P(vp), P(vp), i32, P(i32), P(i32), i32, vp],
        "flexco_lora_bwd": [P(LayerCfg), P(BaseWeights), P(Lora), P(KVPool), vp, i32, P(FtState), i32, i32, vp, vp, vp, sz, vp],
        "flexco_attention_window_bwd": [P(LayerCfg), P(KVPool), vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "flexco_gemm": [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
        "flexco_gemm_plan": [i32, i32, i32, i32, C.c_int64, P(i32)],
        "flexco_prune_graph": [P(Graph), vp],
        "flexco_kernel_timer_start": [i32, i32],
        "flexco_kernel_timer_stop": [i32, P(C.c_double), P(C.c_int64)],
        "flexco_model_forward": [P(LayerCfg), P(ModelLayer), i32, P(Maps), vp, vp, vp, vp, sz, vp],
        "flexco_model_backward": [P(LayerCfg), P(ModelLayer), i32, vp, i32, i32, i32, vp, vp, i32, P(vp), vp, sz, vp],
        "flexco_relu_bitmask_fwd": [vp, vp, vp, i32, i32, i32, vp],
        "flexco_relu_bitmask_bwd": [vp, vp, vp, i32, i32, i32, vp],
        "flexco_bf16_fallbacks": [P(C.c_int64), i32],
        "flexco_attention_chunk_path": [i32],
        "flexco_kernel_timer_sample": [i32, i32],
        "flexco_kernel_timer_read": [i32, P(C.c_double), C.c_int64, P(C.c_int64)],
        "flexco_probe_mfma_lds": [i32, i32, i32, vp, sz, vp, P(C.c_double), vp],
        "flexco_probe_mfma": [i32, i32, vp, P(C.c_double), vp],
        "flexco_probe_read": [vp, sz, i32, vp, P(C.c_double), vp],
        "flexco_latency_estimate": [P(LatencyModel), i32, i32, P(C.c_double)],
        "flexco_sched_window": [P(LatencyModel), i32, C.c_double, i32, i32, P(i32)],
        "flexco_sched_inference": [i32, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, i32, P(i32), P(i32)],
        "flexco_sched_advance": [i32, vp, vp, vp, i32, vp, vp, vp, vp, vp],
        "flexco_lm_loss_workspace_bytes": [P(LmHead), i32, P(sz)],
        "flexco_lm_loss": [P(LmHead), vp, vp, i32, f32, vp, vp, vp, sz, vp],
        "flexco_adam_step": [vp, vp, vp, vp, vp, sz, i32, f32, f32, f32, f32, i32, vp],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name, None)
        if fn is None:
            if HOST_ONLY:          # a build of the host sources alone has no device entry points
                continue
            raise ImportError("libflexco.so lacks the symbol %s" % name)
        fn.argtypes = args
        fn.restype = C.c_int32
    return lib


_lib = _load()
EXPORTS = ("flexco_last_error", "flexco_abi_version", "flexco_maps_blob_ints", "flexco_build_maps",
           "flexco_maps_rebase", "flexco_workspace_bytes", "flexco_layer_forward", "flexco_layer_forward_multi", "flexco_attention_mixed",
           "flexco_lora_fwd", "flexco_lora_fwd_static", "flexco_lora_bwd", "flexco_attention_window_bwd", "flexco_gemm", "flexco_gemm_plan",
           "flexco_kernel_timer_start", "flexco_kernel_timer_stop", "flexco_kernel_timer_sample", "flexco_kernel_timer_read", "flexco_probe_mfma", "flexco_probe_mfma_lds", "flexco_probe_read",
           "flexco_latency_estimate", "flexco_sched_window", "flexco_sched_inference", "flexco_sched_advance",
           "flexco_lm_loss_workspace_bytes", "flexco_lm_loss", "flexco_adam_step", "flexco_prune_graph",
           "flexco_layer_forward_ia3", "flexco_ia3_bwd", "flexco_adapter_workspace_bytes", "flexco_adapter_fwd",
           "flexco_adapter_bwd", "flexco_model_forward", "flexco_model_backward",
           "flexco_relu_bitmask_fwd", "flexco_relu_bitmask_bwd", "flexco_bf16_fallbacks", "flexco_attention_chunk_path")
KERNEL_IDS = {"gemm_fwd": 0, "gemm_bwd": 1, "attn_fwd": 2, "attn_merge": 3, "attn_bwd": 4, "elemwise": 5, "lora": 6,
              "generic": 7}


def _check(rc):
    if rc != FLEXCO_OK:
        raise FlexcoError(rc, _lib.flexco_last_error().decode())


def _ptr(t):
    """device/host address of a torch tensor, numpy array, int or None"""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def flexco_last_error():
    return _lib.flexco_last_error().decode()


def flexco_abi_version():
    return _lib.flexco_abi_version()


def make_batch_desc(kind, start_pos, n_new, adapter, req_pages_lists):
    """Returns (BatchDesc, keepalive arrays)."""
    kind, start_pos, n_new, adapter = _i32(kind), _i32(start_pos), _i32(n_new), _i32(adapter)
    off = _i32(np.concatenate([[0], np.cumsum([len(p) for p in req_pages_lists])]))
    pages = _i32(np.concatenate([np.asarray(p, dtype=np.int32).reshape(-1) for p in req_pages_lists])
                 if len(req_pages_lists) else np.zeros(0))
    if pages.size == 0:
        pages = np.zeros(1, dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    d = BatchDesc(len(kind), ip(kind), ip(start_pos), ip(n_new), ip(adapter), ip(off), ip(pages))
    return d, (kind, start_pos, n_new, adapter, off, pages)


def flexco_maps_blob_ints(desc, page_size, n_q_heads, n_kv_heads, kv_split_pages=0):
    out = C.c_size_t(0)
    _check(_lib.flexco_maps_blob_ints(C.byref(desc), page_size, n_q_heads, n_kv_heads, kv_split_pages, C.byref(out)))
    return out.value


def flexco_build_maps(desc, page_size, num_pages, n_q_heads, n_kv_heads, kv_split_pages=0, blob=None):
    """Returns (Maps with host pointers, blob: np.int32 array that owns the arrays)."""
    if blob is None:
        blob = np.zeros(flexco_maps_blob_ints(desc, page_size, n_q_heads, n_kv_heads, kv_split_pages), dtype=np.int32)
    m = Maps()
    _check(_lib.flexco_build_maps(C.byref(desc), page_size, num_pages, n_q_heads, n_kv_heads, kv_split_pages,
                                  blob.ctypes.data, blob.size, C.byref(m)))
    return m, blob


def maps_to_numpy(m, blob):
    """Host view of every array of host-side maps (for the bit-exact parity tests)."""
    base = blob.ctypes.data
    cpt = None
    lens = {"tok_req": m.T, "tok_pos": m.T, "slot": m.T, "req_tok_off": m.n_req + 1, "req_kv_len": m.n_req,
            "req_kind": m.n_req, "block_table": m.n_req * m.max_pages, "ft_tok": m.n_ft, "seg_off": m.n_seg + 1,
            "seg_adapter": m.n_seg, "lora_tok": m.n_lora, "tile_req": m.n_tiles, "tile_tok0": m.n_tiles,
            "tile_ntok": m.n_tiles, "tile_nsplit": m.n_tiles, "tile_part0": m.n_tiles, "item_tile": m.n_items,
            "item_split": m.n_items, "tok_tile": m.T, "tok_lora": m.T, "tok_adapter": m.T, "item_ntiles": m.n_items}
    out = {n: getattr(m, n) for n in _MAP_SCALARS}
    out["adapter_tok_off"] = np.array(list(m.adapter_tok_off), dtype=np.int32)
    for n, ln in lens.items():
        off = (getattr(m, n) - base) // 4
        out[n] = blob[off:off + ln].copy()
    out["block_table"] = out["block_table"].reshape(m.n_req, m.max_pages)
    return out


def flexco_maps_rebase(host_maps, host_blob, other_blob):
    out = Maps()
    _check(_lib.flexco_maps_rebase(C.byref(host_maps), _ptr(host_blob), _ptr(other_blob), C.byref(out)))
    return out


def flexco_workspace_bytes(cfg, T_max, n_parts_max, win_max, kv_max):
    out = C.c_size_t(0)
    _check(_lib.flexco_workspace_bytes(C.byref(cfg), T_max, n_parts_max, win_max, kv_max, C.byref(out)))
    return out.value


def _opt(struct):
    return C.byref(struct) if struct is not None else None


def flexco_layer_forward_multi(cfg, w, adapters, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream=None):
    """adapters: sequence of Lora structs, indexed by adapter id"""
    arr = (Lora * len(adapters))(*adapters)
    _check(_lib.flexco_layer_forward_multi(C.byref(cfg), C.byref(w), arr, len(adapters), C.byref(maps), _ptr(x_in),
                                           _ptr(x_out), C.byref(pool), _opt(ft), _ptr(ws), ws_bytes, _stream(stream)))


def flexco_layer_forward(cfg, w, lora, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream=None):
    _check(_lib.flexco_layer_forward(C.byref(cfg), C.byref(w), _opt(lora), C.byref(maps), _ptr(x_in), _ptr(x_out),
                                     C.byref(pool), _opt(ft), _ptr(ws), ws_bytes, _stream(stream)))


def flexco_layer_forward_ia3(cfg, w, ia3, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream=None):
    _check(_lib.flexco_layer_forward_ia3(C.byref(cfg), C.byref(w), _opt(ia3), C.byref(maps), _ptr(x_in), _ptr(x_out),
                                         C.byref(pool), _opt(ft), _ptr(ws), ws_bytes, _stream(stream)))


def flexco_ia3_bwd(cfg, w, ia3, pool, seq_pages, n_seq_pages, ft, win_start, win_len, dY, dX, ws, ws_bytes, stream=None):
    _check(_lib.flexco_ia3_bwd(C.byref(cfg), C.byref(w), _opt(ia3), C.byref(pool), _ptr(seq_pages), n_seq_pages,
                               C.byref(ft), win_start, win_len, _ptr(dY), _ptr(dX), _ptr(ws), ws_bytes, _stream(stream)))


def flexco_adapter_workspace_bytes(dtype, hidden, bottleneck, T_max, win_max):
    out = C.c_size_t(0)
    _check(_lib.flexco_adapter_workspace_bytes(dtype, hidden, bottleneck, T_max, win_max, C.byref(out)))
    return out.value


def flexco_adapter_fwd(dtype, hidden, ad, maps, y, saved_in, seq_len, ws, ws_bytes, stream=None):
    _check(_lib.flexco_adapter_fwd(dtype, hidden, C.byref(ad), C.byref(maps), _ptr(y), _ptr(saved_in), seq_len, _ptr(ws),
                                   ws_bytes, _stream(stream)))


def flexco_adapter_bwd(dtype, hidden, ad, saved_in, seq_len, win_start, win_len, dY, ws, ws_bytes, stream=None):
    _check(_lib.flexco_adapter_bwd(dtype, hidden, C.byref(ad), _ptr(saved_in), seq_len, win_start, win_len, _ptr(dY),
                                   _ptr(ws), ws_bytes, _stream(stream)))


def flexco_attention_mixed(cfg, maps, q, pool, out, lse, ws, ws_bytes, stream=None):
    _check(_lib.flexco_attention_mixed(C.byref(cfg), C.byref(maps), _ptr(q), C.byref(pool), _ptr(out), _ptr(lse),
                                       _ptr(ws), ws_bytes, _stream(stream)))


def flexco_lora_fwd(x, y, T, in_features, out_features, rank, scale, dtype, A_list, B_list, seg_off, seg_adapter,
                    u_ws, stream=None):
    n = len(A_list)
    Aarr = (C.c_void_p * n)(*[_ptr(a) for a in A_list])
    Barr = (C.c_void_p * n)(*[_ptr(b) for b in B_list])
    so, sa = _i32(seg_off), _i32(seg_adapter)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    _check(_lib.flexco_lora_fwd(_ptr(x), _ptr(y), T, in_features, out_features, rank, scale, dtype, Aarr, Barr, n,
                                ip(so), ip(sa), len(sa), _ptr(u_ws), _stream(stream)))


def flexco_lora_fwd_static(x, y, T, in_features, out_features, rank, scale, dtype, A_list, B_list, seg_off, seg_adapter,
                           stream=None):
    n = len(A_list)
    Aarr = (C.c_void_p * n)(*[_ptr(a) for a in A_list])
    Barr = (C.c_void_p * n)(*[_ptr(b) for b in B_list])
    so, sa = _i32(seg_off), _i32(seg_adapter)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    _check(_lib.flexco_lora_fwd_static(_ptr(x), _ptr(y), T, in_features, out_features, rank, scale, dtype, Aarr, Barr,
                                       n, ip(so), ip(sa), len(sa), _stream(stream)))


def flexco_lora_bwd(cfg, w, lora, pool, seq_pages, n_seq_pages, ft, win_start, win_len, dY, dX, ws, ws_bytes,
                    stream=None):
    _check(_lib.flexco_lora_bwd(C.byref(cfg), C.byref(w), _opt(lora), C.byref(pool), _ptr(seq_pages), n_seq_pages,
                                C.byref(ft), win_start, win_len, _ptr(dY), _ptr(dX), _ptr(ws), ws_bytes,
                                _stream(stream)))


def flexco_attention_window_bwd(cfg, pool, seq_pages, n_seq_pages, win_start, win_len, q, out, lse, dout, dq,
                                dk_accum, dv_accum, ws, ws_bytes, stream=None):
    _check(_lib.flexco_attention_window_bwd(C.byref(cfg), C.byref(pool), _ptr(seq_pages), n_seq_pages, win_start,
                                            win_len, _ptr(q), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                            _ptr(dk_accum), _ptr(dv_accum), _ptr(ws), ws_bytes, _stream(stream)))


def flexco_gemm(A, W, Cout, bias, residual, M, N, K, trans_w, dtype, stream=None):
    _check(_lib.flexco_gemm(_ptr(A), _ptr(W), _ptr(Cout), _ptr(bias), _ptr(residual), M, N, K, int(trans_w), dtype,
                            _stream(stream)))


def flexco_gemm_plan(M, N, K, trans_w, part_elems=0):
    """-> list of (tile rows, tile columns, output columns, K splits, ring stages), one per launch"""
    out = (C.c_int32 * 11)()
    _check(_lib.flexco_gemm_plan(M, N, K, int(trans_w), int(part_elems), out))
    return [tuple(out[1 + 5 * i:6 + 5 * i]) for i in range(out[0])]


def flexco_probe_mfma(blocks, iters, sink, stream=None):
    """-> flops enqueued"""
    fl = C.c_double(0.0)
    _check(_lib.flexco_probe_mfma(blocks, iters, _ptr(sink), C.byref(fl), _stream(stream)))
    return fl.value


def flexco_probe_mfma_lds(blocks, iters, tile, sink, src=None, src_bytes=0, stream=None):
    """-> flops enqueued"""
    fl = C.c_double(0.0)
    _check(_lib.flexco_probe_mfma_lds(blocks, iters, tile, _ptr(src), src_bytes, _ptr(sink), C.byref(fl), _stream(stream)))
    return fl.value


def flexco_probe_read(src, nbytes, blocks, sink, stream=None):
    """-> bytes the kernel reads"""
    nb = C.c_double(0.0)
    _check(_lib.flexco_probe_read(_ptr(src), nbytes, blocks, _ptr(sink), C.byref(nb), _stream(stream)))
    return nb.value


def flexco_lm_loss_workspace_bytes(head, n_max):
    out = C.c_size_t(0)
    _check(_lib.flexco_lm_loss_workspace_bytes(C.byref(head), n_max, C.byref(out)))
    return out.value


def flexco_lm_loss(head, x, targets, n, scale, loss_accum, dX, ws, ws_bytes, stream=None):
    _check(_lib.flexco_lm_loss(C.byref(head), _ptr(x), _ptr(targets), n, scale, _ptr(loss_accum), _ptr(dX), _ptr(ws),
                               ws_bytes, _stream(stream)))


def flexco_adam_step(param, master, grad, m, v, n, dtype, lr, beta1, beta2, eps, step, stream=None):
    _check(_lib.flexco_adam_step(_ptr(param), _ptr(master), _ptr(grad), _ptr(m), _ptr(v), n, dtype, lr, beta1, beta2, eps,
                                 step, _stream(stream)))


class HostLatencyModel:
    """Owns the host arrays of a flexco_latency_model."""

    def __init__(self, c_grid, s_grid, ms):
        self.c_grid, self.s_grid = _i32(c_grid), _i32(s_grid)
        self.ms = np.ascontiguousarray(ms, dtype=np.float32)
        assert self.ms.shape == (self.c_grid.size, self.s_grid.size)
        self.c = LatencyModel(self.c_grid.size, self.s_grid.size, self.c_grid.ctypes.data, self.s_grid.ctypes.data,
                              self.ms.ctypes.data)


def flexco_latency_estimate(model, c, s):
    out = C.c_double(0.0)
    _check(_lib.flexco_latency_estimate(C.byref(model.c), c, s, C.byref(out)))
    return out.value


def flexco_sched_window(model, c, slo_ms, s_avail, quantum):
    out = C.c_int32(0)
    _check(_lib.flexco_sched_window(C.byref(model.c), c, slo_ms, s_avail, quantum, C.byref(out)))
    return out.value


def flexco_sched_inference(prompt_len, prefilled, gen_len, generated, state, max_batch, token_budget, chunk):
    """The five arrays are np.int32 (state is updated in place).  -> (entries [n, 4] = request, kind,
    start_pos, n_new; c)"""
    n = int(state.size)
    cap = max(1, n)
    out = np.zeros((4, cap), dtype=np.int32)
    n_out, c = C.c_int32(0), C.c_int32(0)
    _check(_lib.flexco_sched_inference(n, prompt_len.ctypes.data, prefilled.ctypes.data, gen_len.ctypes.data,
                                       generated.ctypes.data, state.ctypes.data, max_batch, token_budget, chunk,
                                       out[0].ctypes.data, out[1].ctypes.data, out[2].ctypes.data, out[3].ctypes.data,
                                       cap, C.byref(n_out), C.byref(c)))
    return out[:, :n_out.value].T.copy(), c.value


def flexco_sched_advance(entries, prompt_len, prefilled, gen_len, generated, state):
    e = np.ascontiguousarray(entries.T, dtype=np.int32) if len(entries) else np.zeros((4, 0), dtype=np.int32)
    _check(_lib.flexco_sched_advance(e.shape[1], e[0].ctypes.data, e[1].ctypes.data, e[3].ctypes.data, int(state.size),
                                     prompt_len.ctypes.data, prefilled.ctypes.data, gen_len.ctypes.data,
                                     generated.ctypes.data, state.ctypes.data))


def flexco_prune_graph(op_kind, op_cheap, op_inputs, op_out, tensor_class, need_grad):
    """op_inputs: one list of tensor ids per operator.  -> int32 array [n_tensors] of KEEP_* values"""
    n_ops, n_t = len(op_kind), len(tensor_class)
    off = np.zeros(n_ops + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(i) for i in op_inputs])
    flat = _i32([t for i in op_inputs for t in i] or [0])
    arrs = [_i32(op_kind), _i32(op_cheap), off, flat, _i32(op_out), _i32(tensor_class), _i32(need_grad)]
    g = Graph(n_ops, n_t, *[a.ctypes.data for a in arrs])
    keep = np.full(n_t, -1, dtype=np.int32)
    _check(_lib.flexco_prune_graph(C.byref(g), keep.ctypes.data))
    return keep


def flexco_kernel_timer_start(kernel_id, max_launches):
    _check(_lib.flexco_kernel_timer_start(kernel_id, max_launches))


def flexco_kernel_timer_sample(kernel_id, stride):
    _check(_lib.flexco_kernel_timer_sample(kernel_id, stride))


def flexco_relu_bitmask_fwd(x, y, mask, n, width, dtype, stream=None):
    _check(_lib.flexco_relu_bitmask_fwd(_ptr(x), _ptr(y), _ptr(mask), n, width, dtype, _stream(stream)))


def flexco_relu_bitmask_bwd(dy, mask, dx, n, width, dtype, stream=None):
    _check(_lib.flexco_relu_bitmask_bwd(_ptr(dy), _ptr(mask), _ptr(dx), n, width, dtype, _stream(stream)))


def flexco_bf16_fallbacks(reset=False):
    """-> {kernel class: bf16 launches that ran on the type-generic kernels}"""
    buf = (C.c_int64 * len(KERNEL_IDS))()
    _check(_lib.flexco_bf16_fallbacks(buf, int(bool(reset))))
    return {name: int(buf[i]) for name, i in KERNEL_IDS.items()}


def flexco_attention_chunk_path(mode):
    _check(_lib.flexco_attention_chunk_path(int(mode)))


def target_dims_py(cfg, t):
    """(in_features, out_features) of LoRA target t for a workload LayerCfg (marshalling helper: buffer sizes)"""
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    return {"q": (cfg.hidden, qd), "k": (cfg.hidden, kd), "v": (cfg.hidden, kd), "o": (qd, cfg.hidden),
            "gate": (cfg.hidden, cfg.ffn), "up": (cfg.hidden, cfg.ffn), "down": (cfg.ffn, cfg.hidden)}[t]


def make_model_layers(layers):
    """layers: list of (BaseWeights, Lora or None, KVPool, FtState or None) -> (ctypes array, keep-alive list)"""
    arr = (ModelLayer * len(layers))()
    keep = []
    for i, (w, lora, pool, ft) in enumerate(layers):
        arr[i].w = w
        arr[i].lora = C.cast(C.pointer(lora), C.c_void_p) if lora is not None else None
        arr[i].pool = pool
        arr[i].ft = C.cast(C.pointer(ft), C.c_void_p) if ft is not None else None
        keep.append((w, lora, pool, ft))
    return arr, keep


def flexco_model_forward(cfg, layers_arr, n_layers, maps, x_in, x_out, x_tmp, ws, ws_bytes, stream=None):
    _check(_lib.flexco_model_forward(C.byref(cfg), layers_arr, n_layers, C.byref(maps), _ptr(x_in), _ptr(x_out), _ptr(x_tmp),
                                     _ptr(ws), ws_bytes, _stream(stream)))


def flexco_model_backward(cfg, layers_arr, n_layers, seq_pages, n_seq_pages, win_start, win_len, dY, d_tmp, need_dx0, ws,
                          ws_bytes, stream=None):
    """-> device address of the buffer (dY or d_tmp) holding the bottom layer's input gradient, or None"""
    out = C.c_void_p(0)
    _check(_lib.flexco_model_backward(C.byref(cfg), layers_arr, n_layers, _ptr(seq_pages), n_seq_pages, win_start, win_len,
                                      _ptr(dY), _ptr(d_tmp), int(bool(need_dx0)), C.byref(out), _ptr(ws), ws_bytes,
                                      _stream(stream)))
    return out.value


def flexco_kernel_timer_read(kernel_id, capacity=4096):
    """-> list of the durations (ms) of the event pairs recorded so far, in issue order"""
    buf = (C.c_double * capacity)()
    n = C.c_int64(0)
    _check(_lib.flexco_kernel_timer_read(kernel_id, buf, capacity, C.byref(n)))
    return [buf[i] for i in range(min(n.value, capacity))]


def flexco_kernel_timer_stop(kernel_id):
    """-> (total milliseconds, timed launches)"""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(_lib.flexco_kernel_timer_stop(kernel_id, C.byref(ms), C.byref(n)))
    return ms.value, n.value
