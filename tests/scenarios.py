"""Full-size runs of configurations 4 and 5 through the C ABI, with every host decision mirrored in the
allocator oracle and sampled attention outputs compared with the attention oracle.  Used by the GPU tests
(checks everywhere, fewer steps) and by ``bench.py`` (full step counts, timing, sparser checks).

Configuration 4: 28-layer decode step, batch 128, log-normal lengths; per step ``odma_advance`` -> the seeded
overflows go through ``odma_migrate_batch`` -> 28 x fused ``odma_decode_step`` with ``ODMA_REUSE_PLAN`` from the
second layer on.  Configuration 5: drift run on one layer, up to 256 slots, arrivals sliding from log-normal to a
Pareto tail clipped at 65 536, recalibration of the boundaries every 100 steps.

Data: layers the oracle looks at are drawn with the numpy generators shared with the oracle; the other layers
(configuration 4) and all of configuration 5 are drawn on the GPU with a seeded torch generator, and the rows the
oracle checks are copied to the host as its inputs.
"""
from __future__ import annotations

import math
import time
from typing import Dict, Iterable, Optional, Sequence

import numpy as np
import torch

import workloads as wl
from oracle import allocator as al
from oracle import attention as oa
from paper_2512_09427_amd import binding as B

DEV = "cuda:0"
ABS_TOL, REL_TOL = 2e-3, 1e-2                      # the stated tolerance
TIGHT_BF16 = (2e-5, 2e-4 + 2.0 ** -8)              # engineering bound, bf16 output


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _dev_bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def _check(got: np.ndarray, ref: np.ndarray, what: str, tight=TIGHT_BF16) -> float:
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got.astype(np.float64) - ref)
    for a, r, name in ((ABS_TOL, REL_TOL, "stated"), (*tight, "tight")):
        bad = err > a + r * np.abs(ref)
        if bad.any():
            idx = np.unravel_index(np.argmax(err - (a + r * np.abs(ref))), err.shape)
            raise AssertionError(f"{what} ({name} tolerance): {int(bad.sum())} of {bad.size} elements off; worst at {idx}: "
                                 f"got {got[idx]!r} ref {ref[idx]!r}")
    scale = np.abs(ref).max()
    return float(err.max() / scale) if scale > 0 else 0.0


def _make_pool(n_layers, w_or_geom, max_requests, window=10000):
    g = w_or_geom
    elems = n_layers * 4 * (g["main"] + g["safety"]) * 128
    k_pool = torch.zeros(elems, dtype=torch.bfloat16, device=DEV)
    v_pool = torch.zeros(elems, dtype=torch.bfloat16, device=DEV)
    args = dict(n_layers=n_layers, n_q_heads=28, n_kv_heads=4, head_dim=128, kv_dtype=B.BF16, out_dtype=B.BF16,
                main_tokens=g["main"], safety_tokens=g["safety"], large_cap=g["large_cap"], boundaries=g["boundaries"],
                max_requests=max_requests, window=window)
    cfg0, _ = B.make_config(**args)
    ws = torch.empty(B.odma_workspace_bytes(cfg0), dtype=torch.uint8, device=DEV)
    cfg, keep = B.make_config(**args, k_pool=k_pool, v_pool=v_pool, workspace=ws)
    return B.Pool(cfg, keep), (k_pool, v_pool, ws)


# ---------------------------------------------------------------------------------------------------------
# configuration 4
# ---------------------------------------------------------------------------------------------------------

def run_config4(*, steps: int = 64, n_layers: int = 28, check_layers: Sequence[int] = (0, 27),
                check_steps: Optional[Iterable[int]] = None, log=print) -> Dict:
    """Returns timings and counts; raises AssertionError on any mismatch with the oracles.

    ``check_steps``: steps whose outputs on ``check_layers`` go to the attention oracle (None: every step); the
    steps in which a request migrates are always checked.  Allocator decisions are compared at every step."""
    w = wl.qwen_b128_step(n_layers=n_layers, steps=steps)
    n, L = w.n_requests, n_layers
    check_layers = tuple(sorted(set(l for l in check_layers if l < L)))
    pool, keep = _make_pool(L, dict(main=w.main_tokens, safety=w.safety_tokens, large_cap=w.large_cap,
                                    boundaries=w.boundaries), n)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries, max_requests=n)
    ids = np.arange(n, dtype=np.int32)
    lens = w.lengths.copy()
    pred = (lens + steps).copy()
    # overflowing requests: slab = bucket of len0, start at cap - k so that the append of step k + 1 overflows
    caps0 = np.array([min(b for b in w.boundaries if b >= x) for x in lens])
    for r, kk in zip(w.extra["overflow_req"], np.minimum(w.extra["overflow_after"], steps - 2)):
        pred[r] = caps0[r]
        lens[r] = caps0[r] - kk
    rc, bk, off, cap, st = pool.odma_assign(ids, pred)
    assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(sim.assign(ids, pred.tolist())), "assign"
    total = lens + steps
    scale = float(w.data_scale)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(w.data_seed)

    # fill: the layers the oracle looks at from the shared numpy generators, the others on the GPU
    counts = torch.from_numpy(lens.astype(np.int32)).to(DEV)
    start = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)).to(DEV)
    zeros = torch.zeros(n, dtype=torch.int32, device=DEV)
    off_dev = torch.from_numpy(off.astype(np.int64)).to(DEV)
    kv_host = {}
    t0 = time.perf_counter()
    for l in range(L):
        if l in check_layers:
            kv_host[l] = [wl.request_kv(w, l, r, n_tokens=int(total[r])) for r in range(n)]
            k_rows = _dev_bf16(np.concatenate([k[:lens[r]] for r, (k, _) in enumerate(kv_host[l])]))
            v_rows = _dev_bf16(np.concatenate([v[:lens[r]] for r, (_, v) in enumerate(kv_host[l])]))
        else:
            k_rows = (torch.randn(int(lens.sum()), 4, 128, generator=gen, device=DEV) * scale).to(torch.bfloat16)
            v_rows = (torch.randn(int(lens.sum()), 4, 128, generator=gen, device=DEV) * scale).to(torch.bfloat16)
        pool.odma_append_kv(l, n, off_dev, zeros, counts, start, int(lens.max()), None, 0, k_rows, v_rows)
        torch.cuda.synchronize()
        del k_rows, v_rows
    pool.odma_advance(ids, lens.astype(np.int32))
    sim.advance(ids, lens.tolist())
    log(f"config 4: {n} requests, {int(lens.sum())} tokens, {L} layers filled in {time.perf_counter() - t0:.1f} s")

    # per-layer inputs of a step: queries and the new token's rows.  Checked layers get fresh seeded values every step.
    q_all = (torch.randn(L, n, 28, 128, generator=gen, device=DEV) * scale).to(torch.bfloat16)
    kn_all = (torch.randn(L, n, 4, 128, generator=gen, device=DEV) * scale).to(torch.bfloat16)
    vn_all = (torch.randn(L, n, 4, 128, generator=gen, device=DEV) * scale).to(torch.bfloat16)
    out = torch.zeros(L, n, 28, 128, dtype=torch.bfloat16, device=DEV)
    att = torch.zeros(n, dtype=torch.int32, device=DEV)
    check_steps = set(range(steps)) if check_steps is None else set(check_steps)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    step_ms, step_bytes, mig = [], [], []
    worst, checked, migrated = 0.0, 0, 0
    for s in range(steps):
        rc, ov, _ = pool.odma_advance(ids)
        sov, _ = sim.advance(ids)
        assert ov.tolist() == sov, f"advance, step {s}"
        movers = np.nonzero(ov)[0].astype(np.int32)
        if len(movers):
            e0, e1 = ev(), ev()
            e0.record()
            rc, noff, ncap, mst = pool.odma_migrate_batch(movers)
            e1.record()
            want = [sim.migrate(int(r)) for r in movers]
            assert rc == 0 and mst.tolist() == [0] * len(movers), f"migrate, step {s}"
            assert [(0, int(o), int(c)) for o, c in zip(noff, ncap)] == [t[:3] for t in want], f"migrate, step {s}"
            off[movers] = noff
            off_dev.copy_(torch.from_numpy(off.astype(np.int64)))
            assert pool.odma_advance(movers)[1].tolist() == sim.advance(movers)[0] == [0] * len(movers)
            torch.cuda.synchronize()
            tok = int(sum((int(lens[r]) + 15) // 16 * 16 for r in movers))
            mig.append(dict(step=s, requests=len(movers), tokens=tok, ms=e0.elapsed_time(e1),
                            bytes=2 * tok * w.kv_bytes_per_token * L))
            migrated += len(movers)
        q_np = {}
        for l in check_layers:                               # seeded values of this step for the layers the oracle sees
            q_np[l] = wl.queries(w, l, step=s)
            q_all[l].copy_(_dev_bf16(q_np[l]))
            kn_all[l].copy_(_dev_bf16(np.stack([kv_host[l][r][0][lens[r]] for r in range(n)])))
            vn_all[l].copy_(_dev_bf16(np.stack([kv_host[l][r][1][lens[r]] for r in range(n)])))
        att.copy_(torch.from_numpy((lens + 1).astype(np.int32)))
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for l in range(L):
            pool.odma_decode_step(l, n, q_all[l], kn_all[l], vn_all[l], off_dev, att, None, 0, out[l],
                                  B.REUSE_PLAN if l else 0)
        e1.record()
        torch.cuda.synchronize()
        step_ms.append(e0.elapsed_time(e1))
        step_bytes.append(int((lens + 1).sum()) * w.kv_bytes_per_token * L)
        lens += 1
        if s in check_steps or len(movers):
            for l in check_layers:
                got = wl.bf16_bits_to_f32(_bits(out[l]))
                ref = np.stack([oa.attend_one(q_np[l][r], kv_host[l][r][0][:lens[r]], kv_host[l][r][1][:lens[r]],
                                              1.0 / math.sqrt(128), np.float64) for r in range(n)])
                worst = max(worst, _check(got, ref, f"config 4 step {s} layer {l}"))
            checked += 1
        assert pool.odma_pool_lookup(ids)[1].tolist() == lens.tolist(), f"lengths, step {s}"
    assert migrated == len(w.extra["overflow_req"]) == sim.n_migrations, (migrated, sim.n_migrations)
    assert pool.odma_pool_snapshot()[0] == [tuple(r) for r in sim.snapshot()], "final pool state"
    # a migrated request reads back bit for bit from its Large-Bucket slab, appended rows included
    l = check_layers[-1]
    for r in w.extra["overflow_req"][:2]:
        k = torch.zeros(int(lens[r]), 4, 128, dtype=torch.bfloat16, device=DEV)
        v = torch.zeros_like(k)
        pool.odma_gather_kv(l, int(off[r]), int(lens[r]), None, k, v)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_bits(k), kv_host[l][r][0][:lens[r]])
        np.testing.assert_array_equal(_bits(v), kv_host[l][r][1][:lens[r]])
    ms = np.array(step_ms)
    by = np.array(step_bytes, dtype=np.float64)
    res = dict(requests=n, layers=L, steps=steps, kv_tokens_first_step=int(by[0] // (w.kv_bytes_per_token * L)),
               ms_per_step_median=float(np.median(ms)), ms_per_step_min=float(ms.min()), ms_per_step_max=float(ms.max()),
               kv_GBps=float(np.median(by / (ms * 1e-3) / 1e9)), decode_tokens_per_s=float(n / (np.median(ms) * 1e-3)),
               kernel_us_per_layer=float(np.median(ms) * 1e3 / L), bytes_per_launch=int(np.median(by) / L),
               migrations=migrated, migration_copies=mig, oracle_checked_steps=checked, check_layers=list(check_layers),
               max_err_over_max_ref=worst)
    pool.close()
    del keep
    torch.cuda.empty_cache()
    return res


# ---------------------------------------------------------------------------------------------------------
# configuration 5
# ---------------------------------------------------------------------------------------------------------

def run_config5(*, steps: int = 1000, slots: int = 256, clip: int = 65536, window: int = 2048, recal_every: int = 100,
                main_tokens: int = 1 << 20, safety_slabs: int = 4, check_every: int = 50, check_requests: int = 6,
                seed: int = 5, log=print) -> Dict:
    """Drift run on one layer.  Every allocator call is mirrored in the oracle and compared; every ``check_every``
    steps (and in every step with a migration) the longest and a few random live requests go to the attention oracle."""
    bounds0 = (512, 1024, 2048, 4096)
    pool, keep = _make_pool(1, dict(main=main_tokens, safety=safety_slabs * clip, large_cap=clip, boundaries=bounds0),
                            slots, window=window)
    sim = al.PoolSim(main_tokens, safety_slabs * clip, clip, boundaries=bounds0, max_requests=slots, window=window)
    arrivals = wl.drift_arrivals(seed=seed, n_steps=steps, clip=clip)
    next(arrivals)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1000 + seed)
    rng = np.random.default_rng(2000 + seed)
    data_scale = 1.0 / math.sqrt(128.0)
    live: Dict[int, dict] = {}                  # slot -> total, have, k, v (device rows of the whole request)
    done, traj = [], [dict(step=0, boundaries=list(bounds0))]
    counts = dict(admitted=0, rejected_after_assign=0, nomem=0, routed=0, migrations=0, stopped=0, completed=0, checks=0, checked_requests=0)
    kernel_ms, kv_bytes, batch_sum, worst = 0.0, 0, 0, 0.0
    ev = lambda: torch.cuda.Event(enable_timing=True)
    pending = []                                 # (start event, end event, bytes) of decode launches not yet read
    t_wall = time.perf_counter()
    for step in range(steps):
        migrated_now = False
        # ---- admission into free slots; the prompts of everybody admitted this step are appended in one call
        new_slots = []
        for s in range(slots):
            if s in live:
                continue
            a = arrivals.send(step)
            u = np.array([a.uncertainty], np.float32)
            rc, bk, off, cap, st = pool.odma_assign([s], [a.pred_len], u)
            assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(
                map(list, sim.assign([s], [a.pred_len], [u[0]]))), f"assign, step {step}"
            if st[0] != 0:
                counts["nomem"] += int(st[0] == B.NOMEM)
                continue
            counts["routed"] += int(bk[0] == len(bounds0))
            rc, ov, _ = pool.odma_advance([s], [a.prefilled])
            assert ov.tolist() == sim.advance([s], [a.prefilled])[0], f"prompt advance, step {step}"
            if ov[0]:                            # the prompt alone overflows an under-predicted bucket
                got, want = pool.odma_migrate(s), sim.migrate(s)
                assert got == want[:3], f"prompt migrate, step {step}"
                if got[0] != 0:                  # no Large-Bucket slab is free: the request cannot be admitted now
                    assert pool.odma_release([s])[1].tolist() == sim.release([s]), f"release, step {step}"
                    counts["rejected_after_assign"] += 1
                    continue
                assert pool.odma_advance([s], [a.prefilled])[1].tolist() == sim.advance([s], [a.prefilled])[0] == [0]
                counts["migrations"] += 1
            counts["admitted"] += 1
            k = torch.randn(a.total_len, 4, 128, generator=gen, device=DEV).to(torch.bfloat16)          # sharp keys
            v = (torch.randn(a.total_len, 4, 128, generator=gen, device=DEV) * data_scale).to(torch.bfloat16)
            live[s] = dict(total=a.total_len, have=a.prefilled, k=k, v=v)
            new_slots.append(s)
        if new_slots:
            o, _, _ = pool.odma_pool_lookup(new_slots)
            pre = np.array([live[s]["have"] for s in new_slots], dtype=np.int32)
            pool.odma_append_kv(0, len(new_slots), torch.from_numpy(o).to(DEV),
                                torch.zeros(len(new_slots), dtype=torch.int32, device=DEV), torch.from_numpy(pre).to(DEV),
                                torch.from_numpy(np.concatenate([[0], np.cumsum(pre)[:-1]]).astype(np.int64)).to(DEV),
                                int(pre.max()), None, 0,
                                torch.cat([live[s]["k"][:live[s]["have"]] for s in new_slots]),
                                torch.cat([live[s]["v"][:live[s]["have"]] for s in new_slots]))
        ids = sorted(live)
        # ---- bookkeeping of this step's token; what overflows migrates (or stops at L_max)
        rc, ov, _ = pool.odma_advance(ids)
        assert ov.tolist() == sim.advance(ids)[0], f"advance, step {step}"
        stopped = []
        for s, o in zip(ids, ov):
            if not o:
                continue
            got, want = pool.odma_migrate(s), sim.migrate(s)
            assert got == want[:3], f"migrate, step {step}"
            if got[0] == 0:
                counts["migrations"] += 1
                migrated_now = True
                assert pool.odma_advance([s])[1].tolist() == sim.advance([s])[0] == [0]
            else:
                stopped.append(s)
        ids = [s for s in ids if s not in stopped]
        if ids:
            off, ln, _ = pool.odma_pool_lookup(ids)
            assert ln.tolist() == [live[s]["have"] + 1 for s in ids], f"lengths, step {step}"
            k_new = torch.stack([live[s]["k"][live[s]["have"]] for s in ids])
            v_new = torch.stack([live[s]["v"][live[s]["have"]] for s in ids])
            q = torch.randn(len(ids), 28, 128, generator=gen, device=DEV).to(torch.bfloat16)
            out = torch.zeros(len(ids), 28, 128, dtype=torch.bfloat16, device=DEV)
            off_d, ln_d = torch.from_numpy(off).to(DEV), torch.from_numpy(ln).to(DEV)
            e0, e1 = ev(), ev()
            e0.record()
            pool.odma_decode_step(0, len(ids), q, k_new, v_new, off_d, ln_d, None, 0, out, 0)
            e1.record()
            pending.append((e0, e1, int(ln.sum()) * 2048))
            batch_sum += len(ids)
            for s in ids:
                live[s]["have"] += 1
            if step % check_every == 0 or migrated_now or step == steps - 1:
                order = sorted(range(len(ids)), key=lambda i: -ln[i])
                pick = order[:2] + [int(i) for i in rng.choice(len(ids), min(check_requests, len(ids)), replace=False)]
                got_all, q_bits = wl.bf16_bits_to_f32(_bits(out)), _bits(q)
                for i in dict.fromkeys(pick):
                    s = ids[i]
                    kb, vb = _bits(live[s]["k"][:live[s]["have"]]), _bits(live[s]["v"][:live[s]["have"]])
                    ref = oa.attend_one(q_bits[i], kb, vb, 1.0 / math.sqrt(128), np.float64)
                    worst = max(worst, _check(got_all[i], ref,
                                              f"config 5 step {step} slot {s} ({live[s]['have']} tokens)"))
                    counts["checked_requests"] += 1
                counts["checks"] += 1
        if len(pending) >= 64 or step == steps - 1:
            torch.cuda.synchronize()
            for e0, e1, nb in pending:
                kernel_ms += e0.elapsed_time(e1)
                kv_bytes += nb
            pending = []
        # ---- completions
        fin = [s for s in sorted(live) if live[s]["have"] >= live[s]["total"] or s in stopped]
        if fin:
            done += [live[s]["have"] for s in fin]
            counts["stopped"] += len(stopped)
            counts["completed"] += len(fin)
            assert pool.odma_release(fin)[1].tolist() == sim.release(fin), f"release, step {step}"
            for s in fin:
                del live[s]
        if step % recal_every == recal_every - 1:
            b_new = pool.odma_recalibrate(done)
            assert b_new == tuple(sim.recalibrate(done)), f"recalibrate, step {step}"
            traj.append(dict(step=step + 1, boundaries=list(b_new)))
            done = []
    st = pool.odma_pool_stats()
    assert st["migrations"] == sim.n_migrations == counts["migrations"], (st["migrations"], sim.n_migrations, counts)
    assert st["done_actual"] == sim.done_actual and st["done_reserved"] == sim.done_reserved
    assert st["done_reserved_both"] == sim.done_reserved_both and st["nomem"] == sim.n_nomem
    assert pool.odma_pool_snapshot()[0] == [tuple(r) for r in sim.snapshot()], "final pool state"
    live_tok, live_cap = st["live_tokens"], st["live_reserved"]
    res = dict(steps=steps, slots=slots, clip=clip, window=window, recalibrate_every_steps=recal_every,
               sustained_kv_GBps=kv_bytes / (kernel_ms * 1e-3) / 1e9, decode_kernel_ms_total=kernel_ms,
               kv_bytes_total=int(kv_bytes), mean_batch=batch_sum / steps,
               utilization_completed=st["done_actual"] / max(1, st["done_reserved"]),
               utilization_counting_left_slabs=st["done_actual"] / max(1, st["done_reserved_both"]),
               utilization_live_at_end=live_tok / max(1, live_cap),
               completed=counts["completed"], admitted=counts["admitted"], rejected_after_assign=counts["rejected_after_assign"], routed_to_large_bucket=counts["routed"],
               migrations=counts["migrations"], nomem=int(st["nomem"]), stopped_at_l_max=counts["stopped"],
               recalibrations=int(st["recalibrations"]), boundary_trajectory=traj,
               oracle_checked_steps=counts["checks"], oracle_checked_requests=counts["checked_requests"],
               max_err_over_max_ref=worst, wall_s=time.perf_counter() - t_wall)
    log(f"config 5: {res['completed']} completed, {res['migrations']} migrations, {res['nomem']} NOMEM, utilization "
        f"{res['utilization_completed']:.3f}, {res['sustained_kv_GBps']:.0f} GB/s over the decode launches, "
        f"boundaries {traj[-1]['boundaries']}, {res['wall_s']:.0f} s")
    pool.close()
    del keep
    torch.cuda.empty_cache()
    return res
