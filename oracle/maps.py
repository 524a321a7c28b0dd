"""Index maps of a mixed token batch (oracle side; test infrastructure).

The hybrid token scheduler (Sec. 6.2) hands the runtime, per iteration, a list of
inference requests (decode tokens, prefill chunks) plus a window of finetuning
tokens; the runtime runs them as ONE token batch (Sec. 6.2, fused forward) against
a paged KV cache (Sec. 7, memory management).  The paper does not spell out the
index arrays, so the conventions are fixed here:

  * tokens are laid out request by request, in the order the requests are given
  * token i of a request sits at absolute position start_pos + i of its sequence
  * after the iteration the sequence holds kv_len = start_pos + n_new positions
  * position p of a sequence lives in slot  pages[p // page_size] * page_size + p % page_size
  * block_table row r = the first ceil(kv_len_r / page_size) pages of the request's
    sequence, padded with -1 up to the longest row of the batch (at least 1 column)
  * ft_tok = ascending indices of the tokens whose request is a finetune window
  * LoRA segments = maximal runs of consecutive tokens with equal adapter id; tok_adapter = the
    adapter id of each token's request (-1: base model only)

All outputs are int32.  Invalid descriptions raise ValueError.
"""
import numpy as np

KIND_FINETUNE = 2


def build_maps(requests, seq_pages, page_size, num_pages=None):
    """requests: iterable of records with fields kind, seq_id, start_pos, n_new,
    adapter.  seq_pages: {seq_id: sequence of physical page ids}."""
    requests = list(requests)
    n_req = len(requests)
    if page_size <= 0:
        raise ValueError("page_size must be positive")
    tok_req, tok_pos, slot, tok_adapter = [], [], [], []
    req_tok_off = [0]
    req_kv_len, req_kind, req_seq = [], [], []
    rows = []
    for r, rq in enumerate(requests):
        if rq.n_new <= 0 or rq.start_pos < 0:
            raise ValueError(f"request {r}: n_new must be > 0 and start_pos >= 0")
        if rq.kind not in (0, 1, 2):
            raise ValueError(f"request {r}: unknown kind {rq.kind}")
        if rq.seq_id not in seq_pages:
            raise ValueError(f"request {r}: sequence {rq.seq_id} has no page list")
        pages = [int(p) for p in seq_pages[rq.seq_id]]
        kv_len = rq.start_pos + rq.n_new
        need = -(-kv_len // page_size)
        if need > len(pages):
            raise ValueError(f"request {r}: kv_len {kv_len} exceeds its {len(pages)} pages")
        for p in pages[:need]:
            if p < 0 or (num_pages is not None and p >= num_pages):
                raise ValueError(f"request {r}: page id {p} out of range")
        for i in range(rq.n_new):
            p = rq.start_pos + i
            tok_req.append(r)
            tok_pos.append(p)
            slot.append(pages[p // page_size] * page_size + p % page_size)
            tok_adapter.append(rq.adapter)
        req_tok_off.append(len(tok_req))
        req_kv_len.append(kv_len)
        req_kind.append(rq.kind)
        req_seq.append(rq.seq_id)
        rows.append(pages[:need])
    if len(set(slot)) != len(slot):
        raise ValueError("two tokens of the batch map to the same cache slot")
    max_pages = max([len(r) for r in rows] + [1])
    block_table = -np.ones((n_req, max_pages), dtype=np.int32)
    for r, row in enumerate(rows):
        block_table[r, :len(row)] = row
    T = len(tok_req)
    ft_tok = [t for t in range(T) if requests[tok_req[t]].kind == KIND_FINETUNE]
    seg_off, seg_adapter = [0], []
    for t in range(T):
        if t == 0 or tok_adapter[t] != tok_adapter[t - 1]:
            if t != 0:
                seg_off.append(t)
            seg_adapter.append(tok_adapter[t])
    if T:
        seg_off.append(T)
    i32 = lambda a: np.asarray(a, dtype=np.int32)
    return {
        "T": T, "n_req": n_req, "n_ft": len(ft_tok), "n_seg": len(seg_adapter),
        "max_pages": max_pages, "page_size": page_size,
        "tok_req": i32(tok_req), "tok_pos": i32(tok_pos), "slot": i32(slot),
        "req_tok_off": i32(req_tok_off), "req_kv_len": i32(req_kv_len),
        "req_kind": i32(req_kind), "req_seq": i32(req_seq),
        "block_table": block_table, "ft_tok": i32(ft_tok),
        "seg_off": i32(seg_off), "seg_adapter": i32(seg_adapter), "tok_adapter": i32(tok_adapter),
    }


def check_attention_cover(maps, work_items):
    """An attention work list is implementation-defined; what must hold is that the
    items cover every (token, kv position <= own position) pair exactly once.
    work_items: iterable of (tok_begin, tok_end, kv_begin, kv_end) over ONE request's
    tokens each, meaning tokens [tok_begin, tok_end) attend to cached positions
    [kv_begin, kv_end) clipped by the causal rule.  Returns True/raises."""
    T = maps["T"]
    covered = [dict() for _ in range(T)]
    for (t0, t1, k0, k1) in work_items:
        if not (0 <= t0 < t1 <= T):
            raise ValueError("token range out of bounds")
        r = int(maps["tok_req"][t0])
        if int(maps["tok_req"][t1 - 1]) != r:
            raise ValueError("work item spans two requests")
        for t in range(t0, t1):
            hi = min(k1, int(maps["tok_pos"][t]) + 1)
            for p in range(k0, hi):
                if p in covered[t]:
                    raise ValueError(f"(token {t}, position {p}) covered twice")
                covered[t][p] = 1
    for t in range(T):
        if len(covered[t]) != int(maps["tok_pos"][t]) + 1:
            raise ValueError(f"token {t}: {len(covered[t])} of {int(maps['tok_pos'][t]) + 1} positions covered")
    return True
