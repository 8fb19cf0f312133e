#!/usr/bin/env python3
"""Benchmark of the Twilight decode hot path on one MI355X.

A step = one decode step of one attention layer over one batch: append the
new token's K/V (INT4 quantise, page bounds), select pages, top-p prune,
sparse attention.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused:
this build is single-GPU by design.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")

# Paper context (another machine: one A100, FP16 KV, LongBench-derived prompts) - not a target.
PAPER_CONTEXT = {"quest_twi_vs_fa2_attention_speedup": 15.8, "quest_twi_vs_quest": 1.4,
                 "hardware": "1x NVIDIA A100", "source": "Section 5.2"}


def build_state(cfg_idx, scale, seed, batch, layers, bits=4, p=None, full_selector=False, offload=False,
                separate_append=False, kv_heads=None, separate_prune=False):
    """`layers` independent copies of the layer's cache (same contents, different memory).  Successive steps
    rotate over them, as the layers of a model do, so that a step finds its pools in HBM and not in the
    256 MB memory-side cache left warm by the previous step over the very same addresses."""
    import torch
    import paper_2502_02770_amd as T
    from workloads import synth
    t0 = time.time()
    w = synth.config(cfg_idx, scale=scale, seed=seed, batch=batch, kv_heads=kv_heads)
    if p is not None:
        w.p = float(p)
    if full_selector:
        w.full_selector = True          # no page selector: every token is a candidate of the pruner
    gen_s = time.time() - t0
    dev = "cuda:0"
    t0 = time.time()
    k = w.k.to(dev)
    v = w.v.to(dev) if w.v.numel() else None
    torch.cuda.synchronize()
    h2d_s = time.time() - t0
    start = torch.zeros(w.batch, dtype=torch.int32, device=dev)
    offs = torch.tensor(w.seq_offsets[:-1], dtype=torch.int32, device=dev)
    max_sel = None if w.full_selector else min(int(max(-(-int(b) // 16) for b in w.budget)), w.page_table.shape[1])
    caches, steps = [], []
    append_bulk = None
    for _ in range(layers):
        cache = T.PagedKV(w.num_q_heads, w.num_kv_heads, w.page_table, w.seq_lens, w.num_pool_pages, dev,
                          need_v=w.v.numel() > 0, quant_bits=bits, offload_kv=offload)
        # prefill: every token but the last of each sequence; the step appends the last one
        # (stage 4 as a bulk build; the second copy's launch is timed)
        timed = len(caches) == (1 if layers > 1 else 0) and not offload
        if timed:
            T.twilight_prof_enable(1)
        cache.append(k, v, start, cache.seq_lens - 1, offs, int(w.seq_lens.max()) - 1)
        if timed:
            torch.cuda.synchronize()
            rec = [ms for name, ms in T.twilight_prof_collect() if name == "kquant_append"]
            T.twilight_prof_enable(0)
            tokens = int((w.seq_lens - 1).sum())
            nb = tokens * w.num_kv_heads * ((512 if v is not None else 256) + (512 if v is not None else 256) + 16 * bits + 16) + 512 * w.num_kv_heads * sum((int(n) + 14) // 16 for n in w.seq_lens)
            if rec:
                append_bulk = {"us": rec[0] * 1e3, "tokens": tokens, "bytes": nb, "GBps": nb / (rec[0] * 1e-3) / 1e9,
                               "frac_of_peak": nb / (rec[0] * 1e-3) / 1e9 / HBM_PEAK_GBS}
        caches.append(cache)
        steps.append(T.DecodeStep(cache, max_sel=max_sel, with_kept_idx=False, with_lse=False))
    torch.cuda.synchronize()
    last = torch.tensor([w.seq_offsets[b + 1] - 1 for b in range(w.batch)], dtype=torch.int64, device=dev)
    k_last = k[last].contiguous()
    v_last = v[last].contiguous() if v is not None else None
    del k, v
    torch.cuda.empty_cache()
    q = w.q.to(dev)
    budget = w.budget.to(dev)
    one = torch.ones(w.batch, dtype=torch.int32, device=dev)
    pos = (caches[0].seq_lens - 1).contiguous()
    rows = torch.arange(w.batch, dtype=torch.int32, device=dev)
    turn = [0]
    fused_append = not separate_append

    def step():
        i = turn[0] % layers
        turn[0] += 1
        cache, st = caches[i], steps[i]
        if fused_append and not st.full and not separate_prune:
            # stages 4 + 1 + 2 in one call: the bounds (new token appended on the way), then selection, scoring, top-p
            # and the union in one launch per head where the lists are short enough (else the separate launches)
            st.select_prune(k_last, v_last, pos, q, budget, w.p)
            if v_last is not None:
                st.attend(q)
            return
        if fused_append and not st.full:
            st.append_select(k_last, v_last, pos, q, budget)       # stages 4 + 1 in one launch
        else:
            cache.append(k_last, v_last, pos, one, rows, 1)
            if not st.full:
                st.select(q, budget)
        st.prune(q, w.p)
        if v_last is not None:
            st.attend(q)

    def dense():
        i = turn[0] % layers
        turn[0] += 1
        steps[i].dense(q)

    return w, caches[0], steps[0], q, step, dense, dict(gen_s=gen_s, h2d_s=h2d_s, append_bulk=append_bulk)


def algorithmic_bytes(w, cache, st, bits=4):
    """Bytes each kernel must move per launch (per-unit figures x units, data-dependent ones read back)."""
    import torch
    Hq, Hkv = w.num_q_heads, w.num_kv_heads
    pages = sum((int(n) + 15) // 16 for n in w.seq_lens)
    tokens = int(w.seq_lens.sum())
    out = {}
    out["kquant_append"] = w.batch * Hkv * (2 * 256 + 2 * 256 + 80) + w.batch * Hkv * 2 * 512
    out["page_score"] = pages * Hkv * 512 + pages * Hq * 4
    if st.full:
        cand = tokens * Hkv            # group-shared loads
        out["int4_score"] = cand * (16 * bits + 16) + tokens * Hq * 4
        ncand = tokens * Hq
    else:
        ncand = int(st.sel_count.sum().item()) * 16
        out["int4_score"] = ncand * (16 * bits + 16) + ncand * 4
    out["page_select"] = pages * Hq * 4
    if not st.full:
        # the one-launch forms of twilight_select_prune: the codes and (scale, zero) of every candidate, the lists;
        # with the selection inside, the bounds of every page as well; no score rows through memory
        out["score_topp"] = ncand * (16 * bits + 16) + ncand // 16 * 4
        out["select_score_topp"] = out["score_topp"] + pages * Hq * 4
    # register-resident top-p reads each score once; the long-row path reads the row twice
    # (one histogram pass, one pass that writes the kept bitmap) - its launches are summed per step
    out["topp"] = ncand * 4 * (2 if st.full or ncand / (w.batch * Hq) > 8192 else 1)
    out["union"] = tokens * Hq // 8 + int(st.union_count.sum().item()) * 4      # long-row path: kept bitmaps in, index lists out
    U = int(st.union_count.sum().item())
    out["sparse_decode"] = U * (512 + 4)
    out["combine"] = 0
    out["dense_decode"] = tokens * Hkv * 512
    stats = dict(candidates_per_head=ncand / (w.batch * Hq), kept_per_head=float(st.kept_count.float().mean().item()),
                 union_per_group=U / (w.batch * Hkv), union_max=int(st.union_count.max().item()))
    return out, stats


def cpu_baseline(w, max_seconds=25.0):
    """The oracle, as it stands, on sequences of the same workload until ~max_seconds are used.  BLAS / OpenMP
    pools are held to one thread for this leg, so that the stated core count is what ran."""
    from oracle import twilight_oracle as O
    from workloads import synth
    from threadpoolctl import threadpool_info, threadpool_limits
    t0 = time.time()
    done = 0
    with threadpool_limits(limits=1):
        threads = max([int(x.get("num_threads", 1)) for x in threadpool_info()] + [1])
        for b in range(w.batch):
            O.twilight_decode(synth.bits(w.q[b]), synth.bits(w.seq_k(b)),
                              synth.bits(w.seq_v(b)) if w.v.numel() else synth.bits(w.seq_k(b)),
                              int(w.budget[b]), w.p, full_selector=w.full_selector)
            done += 1
            if time.time() - t0 > max_seconds:
                break
    dt = time.time() - t0
    tok = sum(int(w.seq_lens[b]) for b in range(done))
    per_layer_us = dt / tok * int(w.seq_lens.sum()) * 1e6     # scaled to the whole batch by tokens
    return {"value": per_layer_us, "unit": "\u00b5s/layer", "cores": threads, "kind": "oracle",
            "sample": "%d of %d sequences (%d tokens), all stages incl. quantising the whole cache, %.1f s; "
                      "scaled to the batch by token count; numpy with its thread pools limited to %d thread"
                      % (done, w.batch, tok, dt, threads)}


def percentiles(t):
    """p10 / p50 / p90 / max / mean of a tensor of counts."""
    import torch
    x = t.flatten().float().cpu()
    qs = torch.quantile(x, torch.tensor([0.1, 0.5, 0.9]))
    return {"p10": float(qs[0]), "p50": float(qs[1]), "p90": float(qs[2]), "max": float(x.max()), "mean": float(x.mean())}


def decode_balance(T, cache, union_count, union_stride):
    """How evenly the flattened attention work list spreads over the persistent grid: the kernel's own rule
    (shortest chunk of {c0, 2 c0, 4 c0} that leaves a workgroup at most `ipw` items; workgroup w takes items
    w, w + grid, ...) applied to the list lengths read back from the device."""
    grid, c0, ipw = T.twilight_decode_plan(cache.kv, T.TW_WS_DECODE, False)
    cnt = [min(int(c), union_stride) for c in union_count.cpu().tolist()]
    chunk = c0
    for c in (c0, 2 * c0):
        if sum(-(-n // c) for n in cnt) > ipw * grid and 2 * c <= 512:
            chunk = 2 * c
        else:
            break
    items = []
    for n in cnt:
        items += [min(chunk, n - t0) for t0 in range(0, n, chunk)]
    g = max(1, min(grid, len(items)))
    rows = [sum(items[w::g]) for w in range(g)]
    per = [len(items[w::g]) for w in range(g)]
    mean_rows = sum(rows) / g
    return {"grid_workgroups": g, "chunk": chunk, "items": len(items),
            "rows_per_workgroup_max_over_mean": (max(rows) / mean_rows) if mean_rows else None,
            "items_per_workgroup_max_over_mean": max(per) / (sum(per) / g) if per else None}


def kernel_pass(T, step, steps):
    """Steps with a HIP event pair on every kernel -> {kernel: [ms, ...]} (the first pass only creates the events)."""
    import torch
    T.twilight_prof_enable(1)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    T.twilight_prof_collect(cap=1)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    recs = T.twilight_prof_collect(cap=65536)
    T.twilight_prof_enable(0)
    kern = {}
    for name, ms in recs:
        kern.setdefault(name, []).append(ms)
    return kern


def plain_steps(step, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def dense_us_of(T, dense, reps):
    import torch
    T.twilight_prof_enable(1)
    for _ in range(reps):
        dense()
    torch.cuda.synchronize()
    d = [ms for name, ms in T.twilight_prof_collect() if name == "sparse_decode"]
    T.twilight_prof_enable(0)
    return sum(d[1:]) / max(1, len(d) - 1) * 1e3


def other_config(T, idx, steps, warmup, layers, batch=None):
    """One more benchmark configuration, measured the short way: per-kernel events, the same steps without
    events, dense attention through the same kernel; the roofline fraction of its dominant kernel."""
    import torch
    t0 = time.time()
    w, cache, st, q, step, dense, setup = build_state(idx, 1.0, 0, batch, layers)
    for _ in range(warmup):
        step()
    kern = kernel_pass(T, step, steps)
    kavg = {k: sum(v) / len(v) for k, v in kern.items()}
    kcalls = {k: len(v) / steps for k, v in kern.items()}
    us_plain = plain_steps(step, steps) * 1e3
    nbytes, stats = algorithmic_bytes(w, cache, st)
    dom = max(kavg, key=lambda k: kavg[k] * kcalls[k])
    ach = nbytes[dom] / (kavg[dom] * kcalls[dom] * 1e-3) / 1e9
    d_us = dense_us_of(T, dense, max(3, steps // 10)) if w.v.numel() else None
    res = {"workload": describe(w, 1.0) + ("" if batch is None else " - the C2 shape at a serving-size batch, not one of the five configurations"),
           "config_index": idx, "steps": steps, "layers_rotated": layers,
           "us_per_layer_events_off": us_plain, "dense_decode_us": d_us,
           "below_dense": (us_plain < d_us) if d_us else None,
           "dominant_kernel": dom, "dominant_kernel_us": kavg[dom] * kcalls[dom] * 1e3,
           "dominant_kernel_algorithmic_bytes": nbytes[dom], "dominant_kernel_GBps": ach, "frac": ach / HBM_PEAK_GBS,
           "per_kernel_us": {k: kavg[k] * kcalls[k] * 1e3 for k in kavg},
           "per_kernel_frac_of_peak": {k: nbytes[k] / (kavg[k] * kcalls[k] * 1e-3) / 1e9 / HBM_PEAK_GBS
                                       for k in ("page_score", "int4_score", "score_topp", "select_score_topp", "sparse_decode")
                                       if k in kavg and nbytes.get(k)},
           "dense_decode_frac_of_peak": (nbytes["dense_decode"] / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS) if d_us else None,
           "workload_stats": stats,
           "decode_work_list": decode_balance(T, cache, st.union_count, st.union_stride) if w.v.numel() and not st.full else None,
           "kquant_append_bulk": setup.get("append_bulk"),
           "seconds": None}
    del w, cache, st, q, step, dense
    torch.cuda.empty_cache()
    res["seconds"] = time.time() - t0
    return res


def describe(w, scale):
    return ("%s: batch %d, %d q / %d kv heads, head_dim 128, context %s, page 16, budget %s, p=%g%s"
            % (w.name, w.batch, w.num_q_heads, w.num_kv_heads,
               int(w.seq_lens[0]) if len(set(w.seq_lens.tolist())) == 1 else "ragged",
               ("all tokens" if w.full_selector else int(w.budget[0])) if len(set(w.budget.tolist())) == 1 else "n/8", w.p,
               "" if scale == 1.0 else " (scale %g)" % scale))


def profile_figures(dom):
    """What profiles/ holds for the dominant kernel of the headline configuration: the kernel-trace duration and the
    HBM traffic per dispatch from the counter runs.  Read from the committed summaries at run time; None when the
    summaries do not list a kernel of that stage."""
    from paper_2502_02770_amd.rocprof_summary import read_trace_table, read_traffic_table
    stem = {"page_score": "page_score_kernel", "int4_score": "int4_score", "sparse_decode": "sparse_decode_kernel",
            "topp": "topp_head_kernel", "score_topp": "topp_head_kernel", "select_score_topp": "topp_head_kernel",
            "page_select": "page_select", "combine": "combine_kernel",
            "kquant_append": "kquant_append_kernel"}.get(dom, dom)
    tr_file, tf_file = "c2_decode_step_kernel_trace.md", "c2_decode_step_hbm_traffic.md"
    tr = {k: v for k, v in read_trace_table(os.path.join(PROFILES, tr_file)).items() if k.startswith(stem)}
    tf = {k: v for k, v in read_traffic_table(os.path.join(PROFILES, tf_file)).items() if k[0].startswith(stem)}
    out = {"traffic": None, "traffic_source": None, "rocprofv3_kernel_us": None, "rocprofv3_source": None}
    if tr:
        name = max(tr, key=lambda k: tr[k]["calls"])
        out["rocprofv3_kernel_us"] = tr[name]["avg_ns"] / 1e3
        out["rocprofv3_kernel_median_us"] = tr[name]["median_ns"] / 1e3
        out["rocprofv3_source"] = "profiles/%s: `%s`, %d calls" % (tr_file, name, tr[name]["calls"])
        tf = {k: v for k, v in tf.items() if k[0] == name} or tf
    if tf:
        key = max(tf, key=lambda k: tf[k])
        out["traffic"] = tf[key]
        out["traffic_source"] = "profiles/%s: `%s` (FETCH_SIZE and WRITE_SIZE scaled by the copy-kernel calibration stated there)" % (tf_file, key[0])
    return out


def attention_variants(T, w, cache, st, q):
    """The ways of sharing work inside a GQA group (Appendix B.2): every head over the group's union (built, used
    by the step), every head over its own kept set, and every head padded to the longest list; and the pruner behind
    a token-level selector against the page-list form."""
    import torch
    sv = T.DecodeStep(cache, max_sel=st.max_sel, with_kept_idx=True, with_lse=False)
    sv.select(q, w.budget.to("cuda:0"))
    sv.prune(q, w.p)
    res = {}
    for name, fn in (("group_union", sv.attend), ("per_head", sv.attend_per_head)):
        for _ in range(3):
            fn(q)
        T.twilight_prof_enable(1)
        for _ in range(20):
            fn(q)
        torch.cuda.synchronize()
        r = T.twilight_prof_collect()
        T.twilight_prof_enable(0)
        res[name + "_us"] = sum(ms for k, ms in r) / 20 * 1e3            # decode + combine
    res["group_union_rows"] = int(sv.union_count.sum().item())
    res["per_head_rows"] = int(sv.kept_count.sum().item())
    # "padded" (Appendix B.2, Figure 11): every head's list padded to the longest kept list of the batch with
    # further candidates of its own, i.e. the uniform per-head budget a kernel without variable lengths needs.
    # The lists are put together with torch ops here (set-up only); the attention is the per-head entry point.
    dev = q.device
    L = int(sv.kept_count.max().item())
    slots = sv.max_sel * 16
    cand = (sv.sel_pages.long().unsqueeze(-1) * 16 + torch.arange(16, device=dev)).reshape(w.batch, w.num_q_heads, slots)
    sl = torch.arange(slots, device=dev)
    ok = (sl[None, None, :] < sv.sel_count.long().unsqueeze(-1) * 16) & (cand < cache.seq_lens.long()[:, None, None])
    is_kept = torch.zeros(w.batch, w.num_q_heads, cache.max_pages * 16 + 1, dtype=torch.bool, device=dev)
    kidx = sv.kept_idx.long().clone()
    kidx[torch.arange(kidx.shape[-1], device=dev)[None, None, :] >= sv.kept_count.long().unsqueeze(-1)] = cache.max_pages * 16
    is_kept.scatter_(2, kidx, True)
    prio = torch.gather(is_kept[..., :-1], 2, cand.clamp(0, cache.max_pages * 16 - 1)).int() * 2 + 1
    prio[~ok] = 0
    order = torch.argsort(prio, dim=2, descending=True, stable=True)[..., :L]
    lists = torch.gather(cand, 2, order)
    lcount = torch.minimum(ok.sum(2), torch.tensor(L, device=dev)).int()
    lists[torch.arange(L, device=dev)[None, None, :] >= lcount.long().unsqueeze(-1)] = 1 << 30
    lists = torch.sort(lists, dim=2).values.int().contiguous()
    del is_kept, kidx, prio, order, cand, ok
    ws_p = torch.empty(T.twilight_workspace_bytes(T.TW_WS_DECODE_PER_HEAD, cache.kv, 0, L), dtype=torch.uint8, device=dev)

    def padded(qq):
        T.twilight_sparse_decode_per_head(cache.kv, qq, lcount, lists, L, sv.out, None, ws_p)
    for _ in range(3):
        padded(q)
    T.twilight_prof_enable(1)
    for _ in range(20):
        padded(q)
    torch.cuda.synchronize()
    r = T.twilight_prof_collect()
    T.twilight_prof_enable(0)
    res["padded_us"] = sum(ms for k, ms in r) / 20 * 1e3
    # the pruner behind a token-level selector (twilight_topp_prune_tokens): the same candidates handed over as
    # token lists (gathered 80-byte pieces instead of whole 1280-byte pages), against the page-list form
    if slots <= 8192 and cache.max_pages * 16 <= 196608:
        tl = (sv.sel_pages.long().unsqueeze(-1) * 16 + torch.arange(16, device=dev)).reshape(w.batch, w.num_q_heads, slots).int().contiguous()
        tc = (sv.sel_count * 16).int().contiguous()
        ws_t = torch.empty(T.twilight_workspace_bytes(T.TW_WS_PRUNE_TOKENS, cache.kv, slots), dtype=torch.uint8, device=dev)

        def prune_tokens(qq):
            T.twilight_topp_prune_tokens(cache.kv, qq, tl, tc, slots, w.p, sv.kept_count, None, 0, sv.union_count,
                                         sv.union_idx, sv.union_stride, sv.status, ws_t)

        def prune_pages(qq):
            T.twilight_topp_prune(cache.kv, qq, sv.sel_pages, sv.sel_count, sv.max_sel, w.p, sv.kept_count, None, 0,
                                  sv.union_count, sv.union_idx, sv.union_stride, sv.status, sv.ws_prune)
        for name, fn in (("pruner_page_lists_us", prune_pages), ("pruner_token_lists_us", prune_tokens)):
            for _ in range(3):
                fn(q)
            T.twilight_prof_enable(1)
            for _ in range(20):
                fn(q)
            torch.cuda.synchronize()
            r = T.twilight_prof_collect()
            T.twilight_prof_enable(0)
            res[name] = sum(ms for k, ms in r) / 20 * 1e3
    res["padded_rows"] = int(lcount.sum().item())
    res["padded_list_length"] = L
    del sv
    return res


def channel_sparse_selector(T, w, cache, st, q, r=16):
    """The other token selector in front of the same pruner (Section 4.1): a channel-sparse one (r of 128 channels
    of the INT4 copy, twilight_ds_select_tokens) with the page selector's budget, then the pruner on its token lists
    and attention; per-kernel times with HIP events and the attention mass the result captures."""
    import torch
    from workloads import synth
    dev = q.device
    max_cand = st.max_sel * 16
    if max_cand > 8192 or cache.max_pages * 16 > 196608:
        return None
    _, masks = synth.calibrated_channels(w, r)
    masks = masks.to(dev)
    budget = w.budget.to(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    cand = torch.zeros(w.batch, w.num_q_heads, max_cand, **i32)
    cnt = torch.zeros(w.batch, w.num_q_heads, **i32)
    ws_ds = torch.empty(T.twilight_workspace_bytes(T.TW_WS_DS_SELECT, cache.kv, max_cand), dtype=torch.uint8, device=dev)
    ws_t = torch.empty(T.twilight_workspace_bytes(T.TW_WS_PRUNE_TOKENS, cache.kv, max_cand), dtype=torch.uint8, device=dev)
    sv = T.DecodeStep(cache, max_sel=st.max_sel, with_kept_idx=False, with_lse=True)

    def step():
        T.twilight_ds_select_tokens(cache.kv, q, masks, budget, cand, cnt, max_cand, ws_ds)
        T.twilight_topp_prune_tokens(cache.kv, q, cand, cnt, max_cand, w.p, sv.kept_count, None, 0, sv.union_count,
                                     sv.union_idx, sv.union_stride, sv.status, ws_t)
        sv.attend(q)
    for _ in range(3):
        step()
    kern = kernel_pass(T, step, 20)
    us = {k: sum(v) / 20 * 1e3 for k, v in kern.items()}
    lse_d = torch.zeros(w.batch, w.num_q_heads, dtype=torch.float32, device=dev)
    sv.dense(q, out=torch.empty_like(sv.out), lse=lse_d)
    step()
    torch.cuda.synchronize()
    m = torch.exp(sv.lse - lse_d).cpu()
    tokens = int(w.seq_lens.sum())
    return {"channels": r, "per_kernel_us": us, "step_us_sum_of_kernels": sum(us.values()),
            "int4_bytes_read": tokens * w.num_kv_heads * 80, "kept_per_head": float(sv.kept_count.float().mean()),
            "union_per_group": float(sv.union_count.float().mean()),
            "attention_mass_captured": {"mean": float(m.mean()), "min": float(m.min())}}


def mass_within_candidates(T, w, cache, st, q):
    """Per query head, the softmax mass of its kept set within its candidate set: as the pruner estimates it (INT4
    scores; top-p keeps this at or above p) and exactly (bf16 logits: log-sum-exp over the kept list minus that over
    the candidate list, both through the head-wise attention entry point).  Reporting only: torch ops on the side."""
    import torch
    dev = q.device
    sv = T.DecodeStep(cache, max_sel=st.max_sel, with_kept_idx=True, with_lse=True)
    sv.select(q, w.budget.to(dev))
    sv.prune(q, w.p)
    slots = sv.max_sel * 16
    b_, Hq = w.batch, w.num_q_heads
    scores = torch.empty(b_, Hq, slots, dtype=torch.float32, device=dev)
    T.twilight_int4_score(cache.kv, q, sv.sel_pages, sv.sel_count, sv.max_sel, scores, None)
    cand = (sv.sel_pages.long().unsqueeze(-1) * 16 + torch.arange(16, device=dev)).reshape(b_, Hq, slots)
    ok = (torch.arange(slots, device=dev)[None, None, :] < sv.sel_count.long().unsqueeze(-1) * 16) & (cand < cache.seq_lens.long()[:, None, None])
    kept = torch.zeros(b_, Hq, cache.max_pages * 16 + 1, dtype=torch.bool, device=dev)
    kidx = sv.kept_idx.long().clone()
    kidx[torch.arange(kidx.shape[-1], device=dev)[None, None, :] >= sv.kept_count.long().unsqueeze(-1)] = cache.max_pages * 16
    kept.scatter_(2, kidx, True)
    is_kept = torch.gather(kept[..., :-1], 2, cand.clamp(0, cache.max_pages * 16 - 1)) & ok
    sc = scores.double().masked_fill(~ok, float("-inf"))
    est = (torch.logsumexp(sc.masked_fill(~is_kept, float("-inf")), 2) - torch.logsumexp(sc, 2)).exp()
    # exact: head-wise attention over the kept lists, then over the candidate lists (ascending token positions)
    lse_k = torch.zeros(b_, Hq, dtype=torch.float32, device=dev)
    lse_c = torch.zeros_like(lse_k)
    ws = torch.empty(T.twilight_workspace_bytes(T.TW_WS_DECODE_PER_HEAD, cache.kv, 0, slots), dtype=torch.uint8, device=dev)
    T.twilight_sparse_decode_per_head(cache.kv, q, sv.kept_count, sv.kept_idx, sv.kept_stride, sv.out, lse_k, ws)
    lists = cand.masked_fill(~ok, 1 << 30).sort(dim=2).values.int().contiguous()
    T.twilight_sparse_decode_per_head(cache.kv, q, ok.sum(2).int().contiguous(), lists, slots, sv.out, lse_c, ws)
    torch.cuda.synchronize()
    exact = (lse_k - lse_c).double().exp()

    def summ(x):
        x = x.flatten().cpu()
        return {"mean": float(x.mean()), "min": float(x.min()), "p10": float(x.kthvalue(max(1, x.numel() // 10)).values)}
    return {"p": w.p, "estimated": summ(est), "exact": summ(exact)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=800)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="benchmark configuration 0..4 = C1..C5 (default 1 = C2)")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--kv-heads", type=int, default=None,
                    help="KV heads of the C2 shape (default 8; 32 = multi-head attention, one query head per KV head)")
    ap.add_argument("--layers", type=int, default=4,
                    help="independent copies of the cache that successive steps rotate over (1 = same memory every step)")
    ap.add_argument("--bits", type=int, default=4, choices=[2, 4, 8],
                    help="width of the quantised K copy the pruner scores from (4 = the method; 2 and 8: its bit-width study)")
    ap.add_argument("--p", type=float, default=None, help="override the config's top-p threshold (C3 is swept over p)")
    ap.add_argument("--full-selector", action="store_true",
                    help="skip the page selector: the pruner sees every token (the paper's pruner on top of full attention)")
    ap.add_argument("--offload", action="store_true",
                    help="bf16 K/V pools in pinned host memory (the paper's offloading scenario); attention is then bound by the host link")
    ap.add_argument("--separate-append", action="store_true",
                    help="append the step's token with twilight_kquant_append instead of twilight_append_select")
    ap.add_argument("--separate-prune", action="store_true",
                    help="twilight_append_select + twilight_topp_prune instead of twilight_select_prune (selection, scoring and top-p as launches of their own)")
    ap.add_argument("--graph", action="store_true", help="also time the steps replayed from HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="the timed steps and nothing beside them (no dense baseline, variants or other configs): for profiler runs")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short measurements of C1, C3 and C5")
    ap.add_argument("--breakdown", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run plain 256 MiB device copies (known traffic, for scaling rocprofv3 --pmc counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the decode hot path shards by (sequence, KV head) "
                 "with no exchange; no multi-GPU path is built). Use --gpus 1.")
    import torch
    import paper_2502_02770_amd as T
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    t_start = time.time()

    w, cache, st, q, step, dense, setup = build_state(a.config, a.scale, a.seed, a.batch, max(1, a.layers), a.bits, a.p, a.full_selector, a.offload, a.separate_append, a.kv_heads,
                                                      a.separate_prune)
    if a.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)          # elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # untimed pass with HIP events around every kernel: the per-kernel table, and which kernel
    # dominates the step (largest average duration x launches per step)
    kern = kernel_pass(T, step, a.steps)
    kavg_all = {k: sum(v) / len(v) for k, v in kern.items()}
    kcalls = {k: len(v) / a.steps for k, v in kern.items()}
    dom = max(kavg_all, key=lambda k: kavg_all[k] * kcalls[k])

    # attention mass that the attended sets capture (per query head: exp(lse over its group's union - lse over
    # all tokens), both from twilight_sparse_decode), and - the part the pruner answers for - the mass of each head's
    # kept set WITHIN its candidates: estimated (softmax of the INT4 scores, what top-p thresholds) and exact
    # (log-sum-exp of the bf16 logits over the kept list against that over the candidate list)
    captured = within = None
    if w.v.numel() and not a.step_only:
        lse_s = torch.zeros(w.batch, w.num_q_heads, dtype=torch.float32, device="cuda:0")
        lse_d = torch.zeros_like(lse_s)
        T.twilight_sparse_decode(cache.kv, q, st.union_count, st.union_idx, st.union_stride, st.out, lse_s, st.ws_decode)
        st.dense(q, lse=lse_d)
        torch.cuda.synchronize()
        m = torch.exp(lse_s - lse_d).cpu()
        captured = {"mean": float(m.mean()), "min": float(m.min()), "p10": float(m.flatten().kthvalue(max(1, m.numel() // 10)).values)}
        if not st.full and st.max_sel * 16 <= 16384:
            within = mass_within_candidates(T, w, cache, st, q)

    # ---- timed region: K steps; HIP events (on the launch stream) around the dominant kernel only,
    # so the event pairs do not stretch the step the way bracketing every launch does
    # (and only at every 101st of its launches in the default 800 steps: a launch that carries events delays the
    # stream by some 40 us; an odd period because every 128th step - some periodic work of the runtime - runs this
    # kernel 6 us slower, and a period that divides 128 would sample those steps far too often)
    T.twilight_prof_select(dom, every=101 if a.steps >= 512 else (41 if a.steps >= 256 else (19 if a.steps >= 128 else 3)))
    # (mode 3: the launch ahead of it carries events too - a timed kernel behind an untimed one reads 1.5 us long,
    #  its start stamp being taken before the predecessor has drained)
    T.twilight_prof_enable(3)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    recs = T.twilight_prof_collect(cap=65536)
    T.twilight_prof_enable(0)
    ms_per_step = (t1 - t0) * 1e3 / a.steps
    dom_ms = [ms for name, ms in recs if name == dom]
    dom_avg = sum(dom_ms) / len(dom_ms)

    # the same steps replayed from HIP graphs (one per cache copy): launch gaps removed
    ms_graph = None
    if a.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graphs = []
        with torch.cuda.stream(side):
            for _ in range(max(1, a.layers)):
                step()                               # the copy this graph will cover, once eagerly
            side.synchronize()
            for _ in range(max(1, a.layers)):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step()
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(a.warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(a.steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / a.steps

    # same K steps without the event pairs (launch-to-launch pipelining undisturbed)
    ms_plain = plain_steps(step, a.steps)

    kavg = dict(kavg_all)
    nbytes, stats = algorithmic_bytes(w, cache, st, a.bits)
    hist = {"kept_per_head": percentiles(st.kept_count), "union_per_group": percentiles(st.union_count)}
    if not st.full:
        hist["candidates_per_head"] = percentiles(st.sel_count * 16)
    balance = decode_balance(T, cache, st.union_count, st.union_stride) if w.v.numel() else None

    # dense decode attention through the same kernel, for the "below dense" comparison
    dense_us = None
    if w.v.numel() and not a.step_only:
        dense_us = dense_us_of(T, dense, max(3, a.steps // 10))

    # a kernel id launched several times per step (the long-row top-p) is priced per step:
    # all its launches' time against the bytes the stage moves per step
    dom_calls = kcalls[dom]
    variants = None
    if w.v.numel() and not st.full and not a.step_only:
        variants = attention_variants(T, w, cache, st, q)
        variants["channel_sparse_selector"] = channel_sparse_selector(T, w, cache, st, q)

    ach = nbytes[dom] / (dom_avg * dom_calls * 1e-3) / 1e9
    default_cfg = (a.config == 1 and a.scale == 1.0 and a.batch is None and a.seed == 0 and a.bits == 4 and a.p is None and a.kv_heads is None
                   and not a.full_selector and not a.offload and not a.separate_prune and not a.separate_append)
    prof = profile_figures(dom) if default_cfg else {"traffic": None, "traffic_source": None, "rocprofv3_kernel_us": None, "rocprofv3_source": None}
    roofline = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS,
                "traffic": prof["traffic"],
                "algorithmic_bytes": nbytes[dom], "avg_kernel_us": dom_avg * 1e3, "launches_per_step": dom_calls,
                "launches_timed": len(dom_ms),
                "note": "achieved / frac / avg_kernel_us are measured live in this run; traffic and rocprofv3_* are read from "
                        "the committed profiler summaries named beside them (another run of the same command), not measured here"}
    roofline.update({k: v for k, v in prof.items() if k != "traffic"})
    per_kernel = {k: {"us": kavg[k] * 1e3, "calls_per_step": kcalls[k], "bytes": nbytes.get(k),
                      "GBps": (nbytes.get(k, 0) / (kavg[k] * kcalls[k] * 1e-3) / 1e9) if kavg[k] > 0 else None,
                      "frac_of_peak": (nbytes.get(k, 0) / (kavg[k] * kcalls[k] * 1e-3) / 1e9 / HBM_PEAK_GBS) if kavg[k] > 0 else None}
                  for k in kavg}
    if setup.get("append_bulk"):
        per_kernel["kquant_append_bulk"] = setup["append_bulk"]
    if a.breakdown:
        sys.stderr.write("timed launches of %s (us): %s\n" % (dom, " ".join("%.2f" % (x * 1e3) for x in dom_ms)))
        for k, v in per_kernel.items():
            if "calls_per_step" in v:
                sys.stderr.write("%-16s %9.2f us x %-4.3g %12s B  %8.1f GB/s\n" % (k, v["us"], v["calls_per_step"], v["bytes"], v["GBps"] or 0))
        sys.stderr.write("sum of kernels %.2f us; step %.2f us (events on the dominant kernel) / %.2f us (events off); dense %s us\n"
                         % (sum(v["us"] * v["calls_per_step"] for v in per_kernel.values() if "calls_per_step" in v), ms_per_step * 1e3,
                            ms_plain * 1e3, dense_us))

    # the other benchmark configurations, the short way (default run only; each frees its memory before the next)
    others = None
    if default_cfg and not a.step_only and not a.no_other_configs:
        del cache, st, step, dense
        torch.cuda.empty_cache()
        others = []
        for idx, k in ((0, 200), (2, 200), (3, 20), (4, 100)):
            others.append(other_config(T, idx, k, 10 if idx != 3 else 3, max(1, a.layers) if idx not in (3, 4) else 2))
        # the headline shape at four times the batch: a launch then moves 277 MB of bounds and the fixed cost per
        # launch no longer sets the fraction of peak
        others.append(other_config(T, 1, 100, 10, 2, batch=32))

    cpu = None if a.no_cpu_baseline else cpu_baseline(w)
    line = {
        "metric": "sparse decode-attention \u00b5s/layer and achieved HBM GB/s vs peak (1 MI355X)",
        "value": ms_per_step * 1e3, "unit": "\u00b5s/layer", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 KV, int%d K estimate, fp32 accumulate" % a.bits, "data": "synthetic",
        "config": {"workload": describe(w, a.scale),
                   "config_index": a.config, "seed": a.seed, "layers_rotated": max(1, a.layers),
                   "kv_offloaded_to_host": bool(a.offload),
                   "append": "separate launch" if (a.separate_append or w.full_selector) else "inside page_score",
                   "selector_and_pruner": "separate calls" if (a.separate_prune or a.separate_append or w.full_selector) else "twilight_select_prune"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "us_per_layer_events_off": ms_plain * 1e3,
        "us_per_layer_graph_replay": None if ms_graph is None else ms_graph * 1e3,
        "dense_decode_us": dense_us,
        "dense_decode_GBps": (nbytes["dense_decode"] / (dense_us * 1e-6) / 1e9) if dense_us else None,
        "below_dense": (ms_plain * 1e3 < dense_us) if dense_us else None,
        "per_kernel": per_kernel,
        "workload_stats": stats,
        "histograms": hist,
        "decode_work_list": balance,
        "estimator_bits": a.bits,
        "attention_mass_captured": captured,
        "mass_of_kept_sets_within_candidates": within,
        "gqa_attention_variants": variants,
        "configs": others,
        "paper_context": PAPER_CONTEXT,
        "setup_seconds": {k: v for k, v in setup.items() if k != "append_bulk"},
        "wall_seconds": time.time() - t_start,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
