#!/usr/bin/env python3
"""Adaptive allocation loop under load, and the static worst-case baseline beside it (host only).

Runs the library's allocator (no GPU, no device memory) on a saturated queue of synthetic requests
whose length distribution drifts from a log-normal to a heavy-tailed Pareto, with the constants the
paper gives for its adaptive loop (Section III-C: B = 4 buckets, window 10 000 completions, refresh
every 1 000; Section III-B: gamma 0.2, tau 0.8), and reports what a memory budget admits:

  odma        boundaries recalibrated by the pool's background thread (Sections III-C, III-E)
  odma-fixed  the same pool with its initial boundaries never moved
  static      every request reserves the maximum length L_max (the baseline of Section V)

Per policy: requests resident at once and tokens generated per step under the same token budget,
the paper's utilization (sum of realized lengths / sum of reserved capacities over completed
requests), migrations, admissions that had to wait, and the boundary trajectory.

    python adaptive_loop.py --requests 100000
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

INITIAL_BOUNDARIES = (512, 1024, 2048, 4096)


def run_policy(B, wl, policy: str, n_requests: int, budget_tokens: int, l_max: int, max_live: int, seed: int,
               window: int, refresh: int, safety_slabs: int, room: int,
               gamma: float, tau: float, device: bool = False):
    if policy == "static":
        bounds, main, safety = (l_max,), budget_tokens, 0
    else:
        bounds = INITIAL_BOUNDARIES
        safety = safety_slabs * l_max
        main = budget_tokens - safety
    args = dict(n_layers=1, n_q_heads=28, n_kv_heads=4, head_dim=128, kv_dtype=B.BF16, out_dtype=B.BF16,
                main_tokens=main, safety_tokens=safety, large_cap=l_max, boundaries=bounds,
                max_requests=max_live, window=window, gamma=gamma, tau=tau)
    dev = None
    if device:
        # one layer of real K/V pools on the GPU: prefill rows are appended on admission, every step runs the
        # fused append + attention over the resident batch, migrations copy slabs (all synthetic values)
        import torch
        dev = DeviceSide(torch, B, args, budget_tokens, max_live)
        cfg, keep = B.make_config(**args, k_pool=dev.k_pool, v_pool=dev.v_pool, workspace=dev.ws)
    else:
        cfg, keep = B.make_config(**args)
    pool = B.Pool(cfg, keep)
    adaptive = policy == "odma"
    if adaptive:
        pool.odma_recalibrator_start(refresh)
    gen = wl.drift_arrivals(seed=seed, n_steps=1000, clip=l_max)
    next(gen)
    free_ids = list(range(max_live - 1, -1, -1))
    total_len = np.zeros(max_live, np.int64)
    cur_len = np.zeros(max_live, np.int64)
    live = np.zeros(max_live, bool)
    arrived = completed = steps = waits = 0
    conc_sum = util_sum = 0.0
    parked = []
    trajectory = [(0, bounds)]
    last_epoch = 0
    t0 = time.perf_counter()
    def try_admit(a) -> bool:
        """Reserve, prefill; False (pool unchanged) when memory for it is not there right now."""
        rid = free_ids[-1]
        if policy == "static":
            st = pool.odma_assign([rid], [l_max])[4][0]
        else:
            st = pool.odma_assign([rid], [a.pred_len], np.array([a.uncertainty], np.float32))[4][0]
            if st == B.OVERFLOW:                    # inflated estimate beyond L_max: reserve L_max itself
                st = pool.odma_assign([rid], [l_max])[4][0]
        if st == B.NOMEM:
            return False
        if st != 0:
            raise RuntimeError(f"assign failed with status {st}")
        if pool.odma_advance([rid], [a.prefilled])[1][0]:   # the prompt alone overflows an under-predicted bucket
            if pool.odma_migrate(rid)[0] != 0:
                pool.odma_release([rid])
                return False
            pool.odma_advance([rid], [a.prefilled])
        free_ids.pop()
        total_len[rid], cur_len[rid], live[rid] = a.total_len, a.prefilled, True
        admitted_now.append(rid)
        return True

    while completed < n_requests:
        # Admission.  Requests that found no memory wait in a side room (at most `room` of them, oldest
        # first) so that one request waiting for a Large-Bucket slab does not hold up the short ones.
        admitted_now = []
        still = []
        for a in parked:
            if free_ids and try_admit(a):
                continue
            still.append(a)
        parked = still
        while free_ids and arrived < n_requests and len(parked) < room:
            a = gen.send(1000.0 * arrived / n_requests)
            arrived += 1
            if not try_admit(a):
                parked.append(a)
                waits += 1
        if dev is not None and admitted_now:
            dev.prefill(pool, np.array(admitted_now, np.int32), cur_len)
        ids = np.nonzero(live)[0].astype(np.int32)
        if len(ids) == 0:
            raise RuntimeError("nothing admitted: the budget cannot hold a single request")
        # one decode step: every resident request appends one token
        ov = pool.odma_advance(ids)[1]
        stalled = []
        for rid in ids[ov != 0]:
            if pool.odma_migrate(int(rid))[0] == 0:
                pool.odma_advance([int(rid)])
            else:
                stalled.append(int(rid))            # safety pool full: the request waits a step
        cur_len[ids] += 1
        cur_len[stalled] -= 1
        if dev is not None:
            dev.decode(pool, np.setdiff1d(ids, np.array(stalled, np.int32)).astype(np.int32), cur_len)
        steps += 1
        st = pool.odma_pool_stats()
        conc_sum += len(ids)
        util_sum += st["live_tokens"] / max(1, st["live_reserved"])
        fin = ids[cur_len[ids] >= total_len[ids]]
        if len(fin):
            pool.odma_release(fin)
            if adaptive:
                pool.odma_report_completions(total_len[fin])
            live[fin] = False
            free_ids.extend(int(x) for x in fin)
            completed += len(fin)
        if adaptive and st["boundary_epoch"] != last_epoch:
            last_epoch = st["boundary_epoch"]
            trajectory.append((int(last_epoch), pool.odma_pool_snapshot()[1]))
    if adaptive:
        pool.odma_recalibrator_stop()
    st = pool.odma_pool_stats()
    res = {
        "policy": policy, "requests": int(completed), "steps": steps,
        "mean_resident_requests": round(conc_sum / steps, 1),
        "tokens_per_step": round(conc_sum / steps, 1),      # one token per resident request per step
        "utilization_completed": round(st["done_actual"] / max(1, st["done_reserved"]), 4),
        "utilization_completed_counting_left_slabs": round(st["done_actual"] / max(1, st["done_reserved_both"]), 4),
        "utilization_per_step_mean": round(util_sum / steps, 4),
        "migrations": int(st["migrations"]), "admissions_that_waited": int(waits),
        "recalibrations": int(st["recalibrations"]), "final_boundaries": list(pool.odma_pool_snapshot()[1]),
        "wall_s": round(time.perf_counter() - t0, 1),
    }
    if dev is not None:
        res.update(dev.summary())
    if adaptive:
        keep_every = max(1, len(trajectory) // 12)
        res["boundary_trajectory"] = [{"epoch": e, "boundaries": list(b)} for e, b in trajectory[::keep_every]]
    pool.close()
    return res


class DeviceSide:
    """GPU half of the loop: one layer of K/V pools, bulk prefill, the fused decode step, timing by stream events."""

    HQ, HKV, D = 28, 4, 128

    def __init__(self, torch, B, args, pool_tokens, max_live):
        self.torch, self.B = torch, B
        d = "cuda:0"
        elems = self.HKV * pool_tokens * self.D
        self.k_pool = torch.zeros(elems, dtype=torch.bfloat16, device=d)
        self.v_pool = torch.zeros(elems, dtype=torch.bfloat16, device=d)
        cfg0, _ = B.make_config(**args)
        self.ws = torch.empty(B.odma_workspace_bytes(cfg0), dtype=torch.uint8, device=d)
        g = torch.Generator(device=d)
        g.manual_seed(1234)
        rnd = lambda *shape: (torch.randn(*shape, device=d, generator=g) * 0.088).to(torch.bfloat16)
        self.rows_k, self.rows_v = rnd(1 << 16, self.HKV, self.D), rnd(1 << 16, self.HKV, self.D)   # prompt rows, reused
        self.q, self.k_new, self.v_new = rnd(max_live, self.HQ, self.D), rnd(max_live, self.HKV, self.D), rnd(max_live, self.HKV, self.D)
        self.out = torch.zeros(max_live, self.HQ, self.D, dtype=torch.bfloat16, device=d)
        self.events, self.ms, self.bytes, self.batch_sum, self.steps = [], 0.0, 0, 0, 0
        self.rnd = rnd
        self.pq = self.pout = None                       # prompt queries / outputs, grown on demand
        self.p_events, self.p_ms, self.p_pairs, self.p_tokens = [], 0.0, 0, 0

    def _up(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")

    def prefill(self, pool, rids, cur_len):
        off, _, _ = pool.odma_pool_lookup(rids)
        n_new = cur_len[rids].astype(np.int32)
        if n_new.max() > self.rows_k.shape[0]:
            raise RuntimeError("prompt longer than the synthetic row buffer")
        start = np.zeros(len(rids), np.int64)            # every prompt reads the buffer from its beginning
        off_d, n_d = self._up(off), self._up(n_new)
        pool.odma_append_kv(0, len(rids), off_d, self._up(np.zeros(len(rids), np.int32)), n_d,
                            self._up(start), int(n_new.max()), None, 0, self.rows_k, self.rows_v)
        # causal attention of the prompts over the slabs just filled (one layer), timed by stream events
        total = int(n_new.sum())
        if self.pq is None or self.pq.shape[0] < total:
            self.pq = self.rnd(max(total, 1 << 15), self.HQ, self.D)
            self.pout = self.torch.zeros_like(self.pq)
        q_start = np.concatenate([[0], np.cumsum(n_new)[:-1]]).astype(np.int64)
        e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
        e0.record()
        pool.odma_prefill_attention(0, len(rids), self.pq, total, self._up(q_start), n_d, off_d, n_d, None, 0, self.pout)
        e1.record()
        self.p_events.append((e0, e1))
        self.p_pairs += int((n_new.astype(np.int64) * (n_new.astype(np.int64) + 1) // 2).sum())
        self.p_tokens += total

    def decode(self, pool, ids, cur_len):
        if len(ids) == 0:
            return
        torch = self.torch
        off, _, _ = pool.odma_pool_lookup(ids)
        lens = cur_len[ids].astype(np.int32)             # lengths after this step's append
        n = len(ids)
        off_d, len_d = self._up(off), self._up(lens)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        pool.odma_decode_step(0, n, self.q[:n], self.k_new[:n], self.v_new[:n], off_d, len_d, None, 0, self.out[:n], 0)
        e1.record()
        self.events.append((e0, e1))
        self.bytes += int(lens.sum()) * 2048
        self.batch_sum += n
        self.steps += 1
        if len(self.events) >= 64:
            self._drain()

    def _drain(self):
        self.torch.cuda.synchronize()
        self.ms += sum(a.elapsed_time(b) for a, b in self.events)
        self.p_ms += sum(a.elapsed_time(b) for a, b in self.p_events)
        self.events, self.p_events = [], []

    def summary(self):
        self._drain()
        return {"device": {"layers": 1, "decode_ms_total": round(self.ms, 2), "kv_bytes_total": self.bytes,
                           "sustained_kv_GBps": round(self.bytes / (self.ms * 1e-3) / 1e9, 1),
                           "mean_batch": round(self.batch_sum / max(1, self.steps), 1),
                           "mean_step_us": round(1e3 * self.ms / max(1, self.steps), 1),
                           "prefill_ms_total": round(self.p_ms, 2), "prompt_tokens": self.p_tokens,
                           "prefill_TFLOPs": round(4 * self.D * self.HQ * self.p_pairs / max(self.p_ms, 1e-9) / 1e9, 1),
                           "note": "decode: plan + fused append/attention + reduction of one layer per step; prefill: append + "
                                   "causal attention of every admitted prompt; stream events"}}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--requests", type=int, default=100000)
    ap.add_argument("--budget-tokens", type=int, default=4 << 20,
                    help="KV slots per layer the pool may use (4 Mi tokens of a 28-layer bf16 GQA-4x128 model = 240 GB)")
    ap.add_argument("--l-max", type=int, default=16384, help="longest request served; capacity of a Large-Bucket slab")
    ap.add_argument("--max-live", type=int, default=8192, help="request slots of the serving loop")
    ap.add_argument("--window", type=int, default=10000)
    ap.add_argument("--refresh", type=int, default=1000)
    ap.add_argument("--safety-slabs", type=int, default=32, help="Large-Bucket slabs of L_max tokens (ODMA policies)")
    ap.add_argument("--waiting-room", type=int, default=64,
                    help="requests that may wait for memory while later arrivals are still admitted")
    ap.add_argument("--gamma", type=float, default=0.2, help="uncertainty inflation (Section III-B)")
    ap.add_argument("--tau", type=float, default=0.8, help="uncertainty above which a request goes to the Large Bucket")
    ap.add_argument("--seed", type=int, default=5)
    ap.add_argument("--policies", default="odma,odma-fixed,static")
    ap.add_argument("--device", action="store_true",
                    help="also run the data path on the GPU (one layer): prefill appends, fused decode step per step, "
                         "migration copies; reports the sustained KV GB/s of the decode launches")
    args = ap.parse_args()
    import workloads as wl
    from paper_2512_09427_amd import binding as B       # the library itself; no oracle, no fallback
    out = []
    for policy in args.policies.split(","):
        r = run_policy(B, wl, policy, args.requests, args.budget_tokens, args.l_max, args.max_live, args.seed,
                       args.window, args.refresh, args.safety_slabs, args.waiting_room, args.gamma, args.tau, args.device)
        print(f"{policy:11s} resident {r['mean_resident_requests']:8.1f}  utilization {r['utilization_completed']:.3f}  "
              f"migrations {r['migrations']:6d}  waited {r['admissions_that_waited']:6d}  steps {r['steps']:7d}  "
              f"final b = {r['final_boundaries']}  ({r['wall_s']} s)", file=sys.stderr, flush=True)
        out.append(r)
    base = next((r for r in out if r["policy"] == "static"), None)
    summary = {"budget_tokens": args.budget_tokens, "l_max": args.l_max, "window": args.window, "refresh": args.refresh,
               "gamma": args.gamma, "tau": args.tau, "safety_slabs": args.safety_slabs,
               "data": "synthetic drift (log-normal median 256 -> Pareto 1.2), predictor error exp(0.1 z)",
               "policies": out}
    if base:
        for r in out:
            r["resident_vs_static"] = round(r["mean_resident_requests"] / base["mean_resident_requests"], 2)
    print(json.dumps(summary))


if __name__ == "__main__":
    main()
