"""Hybrid token scheduler (oracle side; test infrastructure).

Sec. 6.2 (Hybrid Token Scheduler) describes two stages per iteration:

  1. the inference requests of the iteration are chosen by iteration-level scheduling: a fixed
     maximum number of running requests, a finished request is replaced by a waiting one as
     soon as there is one; long prompts are cut into chunks (chunked prefill);
  2. as many finetuning tokens as possible are appended: the window size is
     s = argmax f(c, s) <= SLO, with c the number of inference tokens just scheduled and f a
     latency estimate obtained by profiling offline.

The paper fixes neither the form of f nor tie-breaking details; the conventions here:

  * f is a table of profiled latencies over a grid of (c, s) pairs, interpolated bilinearly;
    outside the grid the nearest grid segment is extended linearly (its t or u leaves [0, 1]);
  * candidate window sizes are the multiples of a quantum up to the tokens available, and the
    available count itself; the largest candidate whose estimate meets the SLO wins, 0 if none;
  * requests are served in arrival (index) order: admission while fewer than max_batch run,
    then one decode token for every running request past its prompt, then prefill chunks of
    at most `chunk` tokens for running requests still in their prompt while the iteration's
    token budget lasts;
  * the iteration lists decode entries first, then prefill entries, each in index order.

Everything is plain Python on floats (IEEE double) and ints, one arithmetic operation at a time
in the order written, so that an implementation in C with the same order is bit-identical.
"""

WAITING, RUNNING, FINISHED = 0, 1, 2
KIND_DECODE, KIND_PREFILL = 0, 1


def _segment(grid, x):
    """Index i of the grid segment [grid[i], grid[i + 1]] used for x: the one that contains x,
    the first one below the grid, the last one above it."""
    n = len(grid)
    if n < 2:
        raise ValueError("a grid needs at least two points")
    i = 0
    while i + 2 < n and x >= grid[i + 1]:
        i += 1
    return i


def latency_estimate(c_grid, s_grid, ms, c, s):
    """f(c, s) in the unit of the table.  ms[i][j] is the profiled latency at (c_grid[i],
    s_grid[j]); grids ascend strictly."""
    i = _segment(c_grid, c)
    j = _segment(s_grid, s)
    t = (float(c) - float(c_grid[i])) / (float(c_grid[i + 1]) - float(c_grid[i]))
    u = (float(s) - float(s_grid[j])) / (float(s_grid[j + 1]) - float(s_grid[j]))
    f0 = float(ms[i][j]) + t * (float(ms[i + 1][j]) - float(ms[i][j]))            # along c at s_grid[j]
    f1 = float(ms[i][j + 1]) + t * (float(ms[i + 1][j + 1]) - float(ms[i][j + 1]))  # along c at s_grid[j + 1]
    return f0 + u * (f1 - f0)


def pick_window(c_grid, s_grid, ms, c, slo, s_avail, quantum):
    """s = argmax { f(c, s) <= slo } over the candidates 0, quantum, 2 quantum, ... <= s_avail and
    s_avail itself; 0 when no candidate meets the SLO (Sec. 6.2)."""
    if quantum <= 0 or s_avail < 0:
        raise ValueError("quantum must be positive and s_avail non-negative")
    candidates = list(range(0, s_avail + 1, quantum))
    if candidates[-1] != s_avail:
        candidates.append(s_avail)
    best = 0
    for s in candidates:                      # brute force: no monotonicity assumed
        if latency_estimate(c_grid, s_grid, ms, c, s) <= slo and s > best:
            best = s
    return best


def schedule_inference(prompt_len, prefilled, gen_len, generated, state, max_batch, token_budget, chunk):
    """One iteration of stage 1.  The lists describe the requests in arrival order; `state` is
    updated in place (admissions).  Returns the iteration's entries
    [(request index, kind, start_pos, n_new)], decode entries first."""
    n = len(state)
    if not (len(prompt_len) == len(prefilled) == len(gen_len) == len(generated) == n):
        raise ValueError("request arrays differ in length")
    if max_batch <= 0 or token_budget <= 0 or chunk <= 0:
        raise ValueError("max_batch, token_budget and chunk must be positive")
    running = sum(1 for st in state if st == RUNNING)
    for r in range(n):                        # admission in arrival order
        if running >= max_batch:
            break
        if state[r] == WAITING:
            state[r] = RUNNING
            running += 1
    entries = []
    budget = token_budget
    for r in range(n):                        # one token for every request that is generating
        if state[r] == RUNNING and prefilled[r] == prompt_len[r] and generated[r] < gen_len[r] and budget > 0:
            entries.append((r, KIND_DECODE, prompt_len[r] + generated[r], 1))
            budget -= 1
    for r in range(n):                        # prompt chunks while the budget lasts
        if state[r] == RUNNING and prefilled[r] < prompt_len[r] and budget > 0:
            take = min(prompt_len[r] - prefilled[r], chunk, budget)
            entries.append((r, KIND_PREFILL, prefilled[r], take))
            budget -= take
    return entries


def apply_iteration(entries, prompt_len, prefilled, gen_len, generated, state):
    """Advances the requests by what an iteration processed; a request whose prompt has just been
    completed starts generating in the next iteration; a request with all its tokens generated
    (or with nothing to generate, once its prompt is done) is finished."""
    for (r, kind, start, n_new) in entries:
        if kind == KIND_DECODE:
            generated[r] += 1
        else:
            prefilled[r] += n_new
        if prefilled[r] == prompt_len[r] and generated[r] >= gen_len[r]:
            state[r] = FINISHED
