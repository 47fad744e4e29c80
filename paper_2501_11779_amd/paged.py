"""Harness helper: move a generated token-major cache into a SlotPool (data plumbing only)."""
import torch

from . import workloads as W


def pages_needed(lengths, page_rows, extra_rows=1):
    return int(sum(-(-(int(n) + extra_rows) // page_rows) for n in lengths))


def into_pool(pool, inp, extra_rows=1, poison=True):
    """Reserve pages for every sequence of `inp` (rows cached + extra_rows), optionally fill what
    is mapped with NaN, and copy the cached rows in.  Returns a copy of `inp` whose cache entries
    are the pool's base addresses, strides and capacity."""
    w = inp["workload"]
    assert inp["layout"] == "token_major"
    dt = W.TORCH_DTYPE[w.dtype]
    slots, L = inp["slots"], inp["lengths"]
    status = pool.reserve(slots, L + extra_rows)
    if status != 0:
        raise RuntimeError(f"slot pool reserve failed with status {status}")
    for b in range(w.batch):
        s, n = int(slots[b]), int(L[b])
        mapped = pool.mapped_rows(s)
        for which, cache in (("k", inp["k_cache"]), ("v", inp["v_cache"])):
            view = pool.rows_view(which, s, mapped, dt)
            if poison:
                view.fill_(float("nan"))
            if pool.layout == "head_blocked":        # [page][row in page][H_kv][d]
                pr, full = pool.page_rows, n // pool.page_rows
                view[:full] = cache[s, :full * pr].reshape(full, pr, *cache.shape[2:])
                if n > full * pr:
                    view[full, :n - full * pr] = cache[s, full * pr:n]
            else:
                view[:n] = cache[s, :n]
    torch.cuda.synchronize()
    paged = dict(inp)
    paged["k_cache"], paged["v_cache"] = pool.k_ptr, pool.v_ptr
    paged["strides"], paged["capacity"], paged["n_slots"] = pool.strides, pool.capacity, pool.n_slots
    paged["block"] = pool.block
    return paged
