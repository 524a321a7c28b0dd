"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the
header declares, builds index maps bit-identical to the oracle's, and rejects bad input
before launching anything."""
import ctypes as C
import os
import re
from types import SimpleNamespace as NS

import numpy as np
import pytest

import paper_2402_18789_amd.binding as B
from oracle.maps import build_maps, check_attention_cover
from workload import gen, CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COMMON = ("tok_req", "tok_pos", "slot", "req_tok_off", "req_kv_len", "req_kind", "block_table", "ft_tok", "seg_off",
          "seg_adapter", "tok_adapter")


# tests that call entry points of the device sources; not part of a build of the host sources alone
full_library = pytest.mark.skipif(B.HOST_ONLY, reason="needs the whole library, this is a host-only build")


@full_library
def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "flexco.h")).read()
    declared = set(re.findall(r"\b(flexco_[a-z_0-9]+)\s*\(", header))
    assert {"flexco_layer_forward", "flexco_attention_mixed", "flexco_lora_fwd", "flexco_lora_bwd"} <= declared
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
    assert B.flexco_abi_version() == B.ABI_VERSION


def c_maps(batch, nq, nkv, split=0):
    desc, keep = B.make_batch_desc([r.kind for r in batch.requests], [r.start_pos for r in batch.requests],
                                   [r.n_new for r in batch.requests], [r.adapter for r in batch.requests],
                                   [batch.seq_pages[r.seq_id] for r in batch.requests])
    m, blob = B.flexco_build_maps(desc, batch.page_size, batch.num_pages, nq, nkv, split)
    return B.maps_to_numpy(m, blob)


def work_items(cm, page_size):
    items = []
    for it in range(cm["n_items"]):
        tile, split, ntl = cm["item_tile"][it], cm["item_split"][it], cm["item_ntiles"][it]
        last = tile + ntl - 1
        t0, t1 = cm["tile_tok0"][tile], cm["tile_tok0"][last] + cm["tile_ntok"][last]
        k0 = split * cm["kv_split_pages"] * page_size
        items.append((t0, t1, k0, k0 + cm["kv_split_pages"] * page_size))
    return items


@pytest.mark.parametrize("name,nq,nkv,split", [("c1", 4, 4, 2), ("c1", 4, 4, 0), ("c2", 32, 8, 0), ("c2", 40, 8, 8),
                                               ("scaled", 8, 2, 4)])
def test_maps_bit_exact_vs_oracle(name, nq, nkv, split):
    batch = {"c1": gen.batch_c1(0), "c2": gen.batch_c2(0),
             "scaled": gen.batch_scaled(3, 9, 5, 300, [(0, 37, 37), (64, 50, 130)], [(96, 33, 129)])}[name]
    om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
    cm = c_maps(batch, nq, nkv, split)
    for k in ("T", "n_req", "n_ft", "n_seg", "max_pages"):
        assert cm[k] == om[k], k
    for k in COMMON:
        assert cm[k].dtype == np.int32 and np.array_equal(cm[k], om[k]), k
    # tokens with an adapter, grouped by adapter id; the offsets of the groups are host scalars
    groups = [np.nonzero(om["tok_adapter"] == a)[0] for a in range(8)]
    assert np.array_equal(cm["lora_tok"], np.concatenate(groups))
    assert cm["adapter_tok_off"].tolist() == np.concatenate([[0], np.cumsum([len(g) for g in groups])]).tolist()
    assert cm["n_adapters"] == int(om["tok_adapter"].max()) + 1
    assert np.array_equal(cm["lora_tok"][cm["tok_lora"][om["tok_adapter"] >= 0]], np.nonzero(om["tok_adapter"] >= 0)[0])
    # the work list covers every (token, visible position) exactly once
    assert check_attention_cover(om, work_items(cm, batch.page_size))
    # tiles partition the tokens of each request; partial rows are numbered densely
    assert np.array_equal(np.repeat(np.arange(cm["n_tiles"]), cm["tile_ntok"]), cm["tok_tile"])
    assert cm["n_parts"] == cm["tile_nsplit"].sum()
    # an item = a run of 1..4 tiles of one request x one split of the run's last tile; the runs partition the tiles
    runs = sorted(set(zip(cm["item_tile"].tolist(), cm["item_ntiles"].tolist())))
    assert [t for t, n in runs] == np.concatenate([[0], np.cumsum([n for t, n in runs])[:-1]]).tolist()
    assert sum(n for t, n in runs) == cm["n_tiles"] and all(1 <= n <= 4 for t, n in runs)
    for t, n in runs:
        assert len(set(cm["tile_req"][t:t + n].tolist())) == 1
    assert cm["n_items"] == sum(cm["tile_nsplit"][t + n - 1] for t, n in runs)
    assert np.array_equal(cm["tile_part0"], np.concatenate([[0], np.cumsum(cm["tile_nsplit"])[:-1]]))
    assert cm["tile_tokens"] == max(1, 16 // (nq // nkv))


def test_default_key_split_follows_the_batch_size():
    """128 pages per split (256 when no request sees more pages than that, or when the decode stream's pages outweigh the
    other requests' pages x column tiles) when that already gives the chip enough work items; fewer pages per split for
    batches of few requests (down to 8), so that a decode-only iteration of 16 requests is not 128
    wavefronts walking 1000 keys each.  Any split leaves the cover intact."""
    assert c_maps(gen.batch_c2(0), 32, 8)["kv_split_pages"] == 256     # contexts of at most 4096 keys = 256 pages
    c3 = c_maps(gen.batch_c3(0), 32, 8)                                # contexts of up to 8192 keys, a decode-heavy batch
    assert c3["kv_split_pages"] == 256 and c3["stream_pages"] > c3["chunk_tile_pages"]
    c4 = c_maps(gen.batch_c4(0), 40, 8)                                # contexts of up to 8192 keys, a 1024-row window on 3072
    assert c4["kv_split_pages"] == 128 and c4["stream_pages"] < c4["chunk_tile_pages"]
    for share, want in ((0.25, 128), (0.75, 256), (0.9, 256)):
        assert c_maps(gen.batch_c4(0, share), 40, 8)["kv_split_pages"] == want
    for n_dec, want in ((16, 8), (64, 16), (100, 32), (200, 256)):
        ctx = gen.rng(0, "split", n_dec).integers(256, 1025, size=n_dec)
        batch = gen.mixed_batch(16, 0, decode_ctx=ctx)
        cm = c_maps(batch, 32, 8)
        assert cm["kv_split_pages"] == want, (n_dec, cm["kv_split_pages"])
        assert cm["n_items"] * 8 >= 1024 or want == 8
        om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
        assert check_attention_cover(om, work_items(cm, batch.page_size))
    assert c_maps(gen.mixed_batch(16, 0, decode_ctx=(300,)), 32, 8, split=64)["kv_split_pages"] == 64   # an explicit value is kept


def count_single(cm):
    """Work items of one tile that holds one token, counted from the work list itself."""
    return sum(1 for it in range(cm["n_items"])
               if cm["item_ntiles"][it] == 1 and cm["tile_ntok"][cm["item_tile"][it]] == 1)


def work_sums(cm, page_size):
    """(pages read by the one-token items, sum over the other items of pages x tiles), from the work list itself."""
    stream = chunk = 0
    for it in range(cm["n_items"]):
        t0, ntl, sp = cm["item_tile"][it], cm["item_ntiles"][it], cm["item_split"][it]
        last = t0 + ntl - 1
        vis = cm["tok_pos"][cm["tile_tok0"][last] + cm["tile_ntok"][last] - 1] // page_size + 1
        pages = min((sp + 1) * cm["kv_split_pages"], vis) - sp * cm["kv_split_pages"]
        if ntl == 1 and cm["tile_ntok"][t0] == 1:
            stream += pages
        else:
            chunk += pages * ntl
    return stream, chunk


def test_work_sums_that_pick_the_attention_kernels():
    """stream_pages / chunk_tile_pages weigh the decode stream against the chunks' products (the default choice of
    flexco_attention_chunk_path): equal to the sums over the work list; the benchmark batch is stream-heavy, the
    14B-shaped batch with a 1024-row window on a 3072-row prefix chunk-heavy."""
    c2 = c_maps(gen.batch_c2(0), 32, 8)
    assert (c2["stream_pages"], c2["chunk_tile_pages"]) == work_sums(c2, 16)
    assert c2["chunk_tile_pages"] < c2["stream_pages"]
    c4 = c_maps(gen.batch_c4(0), 40, 8)
    assert (c4["stream_pages"], c4["chunk_tile_pages"]) == work_sums(c4, 16)
    assert c4["chunk_tile_pages"] > c4["stream_pages"]
    none = c_maps(gen.mixed_batch(16, 0, prefill=[(0, 100, 100)]), 32, 8)
    assert none["stream_pages"] == work_sums(none, 16)[0] and none["chunk_tile_pages"] == work_sums(none, 16)[1] > 0


def test_n_single_counts_the_one_token_work_items():
    """n_single is what decides which attention kernel takes the chunk items: zero exactly when no work item is a
    lone token.  A decode request gives one such item per key split; a chunk whose length leaves one token in its
    last tile gives them too; a chunk of whole tiles gives none."""
    c2 = c_maps(gen.batch_c2(0), 32, 8)
    assert c2["n_single"] == count_single(c2) >= 256                   # 256 decode requests
    tile = c2["tile_tokens"]                                           # 4 tokens per tile at 32 / 8 heads
    whole = c_maps(gen.mixed_batch(16, 0, prefill=[(0, 25 * tile, 25 * tile)], finetune=[(64, 7 * tile, 64 + 7 * tile)]), 32, 8)
    assert whole["n_single"] == 0 == count_single(whole)
    ragged = c_maps(gen.mixed_batch(16, 0, prefill=[(0, 25 * tile + 1, 25 * tile + 1)]), 32, 8, split=2)
    assert ragged["n_single"] == count_single(ragged)
    one = c_maps(gen.mixed_batch(16, 0, decode_ctx=(300,)), 32, 8, split=4)
    assert one["n_single"] == count_single(one) == -(-301 // (4 * 16))  # one item per key split of its 301 visible keys


@pytest.mark.parametrize("seed", range(30))
def test_random_batches_bit_exact_vs_oracle(seed):
    """Seeded random request mixes (counts, contexts, chunk lengths, adapters, head grouping, key split): the integer
    maps equal the oracle's bit for bit and the attention work list covers every (token, visible key) once."""
    g = gen.rng(seed, "random_maps")
    nq, nkv = [(4, 4), (8, 2), (10, 2), (8, 1), (32, 8), (40, 8), (16, 16)][seed % 7]
    ctx = g.integers(1, 700, size=int(g.integers(0, 40)))
    prefill = []
    for _ in range(int(g.integers(0, 4))):
        total = int(g.integers(2, 900))
        start = int(g.integers(0, total - 1))
        prefill.append((start, int(g.integers(1, total - start + 1)), total))
    finetune = []
    if g.integers(0, 2) or (len(ctx) == 0 and not prefill):
        total = int(g.integers(1, 600))
        start = int(g.integers(0, total))
        finetune.append((start, int(g.integers(1, total - start + 1)), total))
    batch = gen.mixed_batch(16, seed, decode_ctx=ctx, prefill=prefill, finetune=finetune)
    batch = gen.with_adapters(batch, [int(a) for a in g.integers(-1, 4, size=5)])
    split = int(g.choice([0, 0, 2, 6, 16, 64]))
    om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
    cm = c_maps(batch, nq, nkv, split)
    for k in ("T", "n_req", "n_ft", "n_seg", "max_pages"):
        assert cm[k] == om[k], k
    assert cm["n_single"] == count_single(cm)
    assert (cm["stream_pages"], cm["chunk_tile_pages"]) == work_sums(cm, batch.page_size)
    for k in COMMON:
        assert np.array_equal(cm[k], om[k]), k
    assert check_attention_cover(om, work_items(cm, batch.page_size))
    assert cm["n_parts"] == cm["tile_nsplit"].sum() and cm["n_items"] == len(cm["item_tile"])
    if split:
        assert cm["kv_split_pages"] == split


def test_work_list_is_deterministic():
    a, b = c_maps(gen.batch_c2(0), 32, 8), c_maps(gen.batch_c2(0), 32, 8)
    for k in a:
        assert np.array_equal(a[k], b[k])


def R(kind, seq, start, n, adapter=-1):
    return NS(kind=kind, seq_id=seq, start_pos=start, n_new=n, adapter=adapter)


@pytest.mark.parametrize("reqs,pages,code", [
    ([R(0, 0, 8, 1)], {0: [1, 2]}, B.FLEXCO_EPAGE),                       # kv_len 9 needs 3 pages of 4
    ([R(0, 0, 0, 1)], {0: [4]}, B.FLEXCO_EPAGE),                          # page id out of range
    ([R(0, 0, 0, 1)], {0: [-1]}, B.FLEXCO_EPAGE),
    ([R(0, 0, 0, 1), R(0, 1, 0, 1)], {0: [1], 1: [1]}, B.FLEXCO_EPAGE),   # duplicate slot
    ([R(1, 0, 0, 3), R(1, 0, 2, 2)], {0: [1, 2]}, B.FLEXCO_EPAGE),
    ([R(0, 0, 0, 0)], {0: [1]}, B.FLEXCO_EINVAL),
    ([R(3, 0, 0, 1)], {0: [1]}, B.FLEXCO_EINVAL),
    ([R(0, 0, -1, 1)], {0: [1]}, B.FLEXCO_EINVAL),
    ([R(2, 0, 0, 1, 0), R(2, 1, 0, 1, 0)], {0: [1], 1: [2]}, B.FLEXCO_EUNSUPPORTED),
])
def test_invalid_batches_are_rejected(reqs, pages, code):
    desc, keep = B.make_batch_desc([r.kind for r in reqs], [r.start_pos for r in reqs], [r.n_new for r in reqs],
                                   [r.adapter for r in reqs], [pages[r.seq_id] for r in reqs])
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_build_maps(desc, 4, 4, 4, 2, 0, blob=np.zeros(4096, dtype=np.int32))
    assert e.value.code == code and len(str(e.value)) > 20


def test_blob_too_small_and_bad_heads():
    b = gen.batch_c1(0)
    desc, keep = B.make_batch_desc([r.kind for r in b.requests], [r.start_pos for r in b.requests],
                                   [r.n_new for r in b.requests], [r.adapter for r in b.requests],
                                   [b.seq_pages[r.seq_id] for r in b.requests])
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_build_maps(desc, 16, b.num_pages, 4, 4, 0, blob=np.zeros(8, dtype=np.int32))
    assert e.value.code == B.FLEXCO_EWORKSPACE
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_build_maps(desc, 16, b.num_pages, 4, 3, 0)
    assert e.value.code == B.FLEXCO_ESHAPE
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_build_maps(desc, 16, b.num_pages, 4, 4, 3)          # odd split
    assert e.value.code == B.FLEXCO_EINVAL


def _cfg(**kw):
    from paper_2402_18789_amd.host import c_cfg
    return c_cfg(CONFIGS["c1_tiny_f32"].with_(**kw))


@full_library
def test_workspace_bytes_and_cfg_validation():
    c = _cfg()
    small = B.flexco_workspace_bytes(c, 68, 20, 32, 64)
    big = B.flexco_workspace_bytes(c, 136, 40, 64, 64)
    assert 0 < small < big
    for bad in (dict(head_dim=63), dict(n_kv_heads=3), dict(lora_rank=65), dict(hidden=0), dict(head_dim=512)):
        with pytest.raises(B.FlexcoError):
            B.flexco_workspace_bytes(_cfg(**bad), 8, 8, 8, 8)


@full_library
def test_workspace_covers_every_smaller_batch():
    """A workspace sized for T_max tokens must do for any batch of fewer tokens, including the small batches whose
    projections ask for split-K scratch (bf16, at most 256 tokens): the size never shrinks as T_max grows."""
    from workload import CONFIGS
    from paper_2402_18789_amd.host import c_cfg
    c = c_cfg(CONFIGS["c2_llama8b_layer"])
    sizes = [B.flexco_workspace_bytes(c, T, max(1, T // 4), 0, 0) for T in (1, 16, 255, 256, 257, 300, 512, 1024)]
    assert all(a <= b for a, b in zip(sizes, sizes[1:])), sizes


@full_library
def test_entry_points_validate_before_launch():
    """NULL / misaligned arguments fail on the host: no device is needed (or present) here."""
    c = _cfg()
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_gemm(0, 0, 0, None, None, 4, 4, 4, 0, B.FLEXCO_F32, stream=0)
    assert e.value.code == B.FLEXCO_EINVAL
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_gemm(16, 32, 48, None, None, 4, 0, 4, 0, B.FLEXCO_F32, stream=0)
    assert e.value.code == B.FLEXCO_EINVAL
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_gemm(16, 32, 50, None, None, 4, 4, 4, 0, B.FLEXCO_F32, stream=0)     # misaligned C
    assert e.value.code == B.FLEXCO_EINVAL
    w = B.BaseWeights()
    m = B.Maps()
    pool = B.KVPool(16, 16, 4, 16)
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_layer_forward(c, w, None, m, 16, 32, pool, None, 64, 1 << 20, stream=0)
    assert e.value.code == B.FLEXCO_EINVAL and "NULL" in str(e.value)
    # segmented LoRA: segments must tile [0, T)
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_lora_fwd(16, 32, 8, 16, 16, 4, 1.0, B.FLEXCO_F32, [48], [64], [0, 5], [0], 80, stream=0)
    assert e.value.code == B.FLEXCO_ESHAPE
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_lora_fwd(16, 32, 8, 16, 16, 4, 1.0, B.FLEXCO_F32, [48], [64], [0, 8], [1], 80, stream=0)
    assert e.value.code == B.FLEXCO_EINVAL


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message and prints no result line."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
