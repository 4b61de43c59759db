"""Where a launch of the copy kernel spends its time, from the kernel's own log (FT_LOG).

    python -m paper_2411_01830_amd.timeline --workload feature [--class 2] [--steps 3]

One step of the workload is replayed with FT_LOG; for every launch of the chosen link class the
per-ticket record (begin, end, workgroup) and the per-workgroup record (entry, exit) give: how long
after the first workgroup's entry each workgroup entered and began its first tile, what a tile takes
(first, middle, last of a workgroup), the gap between a workgroup's tiles, and the tail - workgroup
time left idle between a workgroup's exit and the launch's last exit. Workgroups whose tiles are slow
(median tile more than 1.25 x the launch's median) are listed apart; where the workload also carries
host-link traffic the log's compute-unit identifiers say which workgroups of the chosen class ran on a
unit that a host-link workgroup occupied at the same time, and what their tiles took. Prints markdown.
The log costs a wait and a barrier per tile, so the launch it describes is a few per cent slower than
the one bench.py times.
"""
import argparse
import sys

import numpy as np


def launch_summary(log, wg, t_in, t_out, payload):
    tb, te = log["t_begin_ns"].astype(np.int64), log["t_end_ns"].astype(np.int64)
    t_in, t_out = t_in.astype(np.int64), t_out.astype(np.int64)
    t0 = int(t_in.min())
    span = int(t_out.max()) - t0
    nwg = len(t_in)
    first_begin = np.full(nwg, -1, np.int64)
    dur_first, dur_mid, dur_last, gaps = [], [], [], []
    med_tile = np.zeros(nwg)
    tiles_of = np.zeros(nwg, np.int64)
    for g in range(nwg):
        mine = np.flatnonzero(wg == g)
        if len(mine) == 0:
            continue
        order = mine[np.argsort(tb[mine])]
        b, e = tb[order], te[order]
        first_begin[g] = b[0]
        d = e - b
        dur_first.append(d[0])
        dur_last.append(d[-1])
        dur_mid.extend(d[1:-1].tolist())
        gaps.extend((b[1:] - e[:-1]).tolist())
        med_tile[g] = np.median(d)
        tiles_of[g] = len(mine)
    have = first_begin >= 0
    med_all = float(np.median(te - tb))
    slow = have & (med_tile > 1.25 * med_all)
    idle_tail = float(np.sum(t_out.max() - t_out)) / nwg        # workgroup time idle before the launch's last exit
    q = lambda a, p: float(np.percentile(np.asarray(a, dtype=np.float64), p)) if len(a) else float("nan")
    out = {
        "payload_MB": payload / 1e6, "tickets": len(tb), "workgroups": nwg, "span_us": span / 1e3,
        "traffic_TBps": 2 * payload / span / 1e3 if span else float("nan"),
        "entry_skew_us": (q(t_in - t0, 50) / 1e3, q(t_in - t0, 100) / 1e3),
        "entry_to_first_tile_us": (q((first_begin - t_in)[have], 50) / 1e3, q((first_begin - t_in)[have], 100) / 1e3),
        "tile_first_us": q(dur_first, 50) / 1e3, "tile_mid_us": q(dur_mid, 50) / 1e3, "tile_last_us": q(dur_last, 50) / 1e3,
        "tile_mid_p90_us": q(dur_mid, 90) / 1e3, "gap_us": q(gaps, 50) / 1e3,
        "median_exit_to_last_exit_us": (int(t_out.max()) - q(t_out, 50)) / 1e3,
        "idle_tail_us_per_wg": idle_tail / 1e3,
        "idle_head_us_per_wg": float(np.sum((first_begin - t0)[have])) / nwg / 1e3,
        "slow_wgs": int(slow.sum()),
        "slow_tile_us": q(med_tile[slow], 50) / 1e3 if slow.any() else float("nan"),
        "fast_tile_us": q(med_tile[have & ~slow], 50) / 1e3,
        "tiles_per_fast_wg": q(tiles_of[have & ~slow], 50), "tiles_per_slow_wg": q(tiles_of[slow], 50) if slow.any() else float("nan"),
        "last_exit_is_slow_wg": bool(slow[int(np.argmax(t_out))]),
    }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="feature", choices=["tiny", "traffic", "feature", "contended", "large_mixed"])
    ap.add_argument("--class", dest="cls", type=int, default=2)
    ap.add_argument("--steps", type=int, default=3, help="steps replayed; the last one is reported")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        sys.exit(2)
    from paper_2411_01830_amd import binding as ft
    from paper_2411_01830_amd.replay import Replay
    rp = Replay(args.workload, args.workload == "large_mixed")
    rows = []

    raw = []       # (name, per-ticket log, workgroup of each ticket, entry, exit, unit) of the chosen class
    others = []    # (entry, exit, unit) of every workgroup of the other classes' launches, same clock

    def collect(name, pool, job, st):
        for c in range(3):
            if st.cls[c].payload_bytes == 0:
                continue
            if c != args.cls:
                _, t_in, t_out = ft.job_log_workgroups(pool, job, c, 0)
                others.append((t_in.astype(np.int64), t_out.astype(np.int64), ft.job_log_units(pool, job, c)))
                continue
            log = ft.job_log(pool, job, c)
            wg, t_in, t_out = ft.job_log_workgroups(pool, job, c, len(log["bytes"]))
            raw.append((name, log, wg, t_in, t_out, ft.job_log_units(pool, job, c)))
            rows.append((name, launch_summary(log, wg, t_in, t_out, st.cls[c].payload_bytes), st.cls[c].device_ms))
    for i in range(args.steps):
        rows.clear()
        raw.clear()
        others.clear()
        rp.step(ft.FT_LOG, collect)
    rp.close()
    print(f"# Timeline of the class-{args.cls} launches of `{args.workload}` (one step, FT_LOG)\n")
    print("| launch | MB | tickets | wgs | span us | event us | TB/s r+w | entry skew med/max | entry->1st tile med/max | "
          "tile first/mid/last (p90 mid) us | gap us | idle head us/wg | idle tail us/wg | slow wgs | tile fast/slow us | "
          "tiles per wg fast/slow | last exit slow? |")
    print("|" + "---|" * 17)
    tot = {"bytes": 0.0, "span": 0.0, "head": 0.0, "tail": 0.0}
    for name, s, ms in rows:
        print(f"| {name} | {s['payload_MB']:.1f} | {s['tickets']} | {s['workgroups']} | {s['span_us']:.1f} | {ms * 1e3:.1f} | "
              f"{s['traffic_TBps']:.2f} | {s['entry_skew_us'][0]:.2f} / {s['entry_skew_us'][1]:.2f} | "
              f"{s['entry_to_first_tile_us'][0]:.2f} / {s['entry_to_first_tile_us'][1]:.2f} | "
              f"{s['tile_first_us']:.2f} / {s['tile_mid_us']:.2f} / {s['tile_last_us']:.2f} ({s['tile_mid_p90_us']:.2f}) | "
              f"{s['gap_us']:.2f} | {s['idle_head_us_per_wg']:.2f} | {s['idle_tail_us_per_wg']:.2f} | {s['slow_wgs']} | "
              f"{s['fast_tile_us']:.2f} / {s['slow_tile_us']:.2f} | {s['tiles_per_fast_wg']:.0f} / {s['tiles_per_slow_wg']:.0f} | "
              f"{'yes' if s['last_exit_is_slow_wg'] else 'no'} |")
        tot["bytes"] += s["payload_MB"]
        tot["span"] += s["span_us"]
        tot["head"] += s["idle_head_us_per_wg"]
        tot["tail"] += s["idle_tail_us_per_wg"]
    if rows and others:
        # which workgroups shared a compute unit with a workgroup of another class's kernel while they ran
        o_in = np.concatenate([o[0] for o in others])
        o_out = np.concatenate([o[1] for o in others])
        o_unit = np.concatenate([o[2] for o in others])
        n_all = n_shared = 0
        tile_shared, tile_alone, units_seen = [], [], set()
        for name, log, wg, t_in, t_out, unit in raw:
            tb, te = log["t_begin_ns"].astype(np.int64), log["t_end_ns"].astype(np.int64)
            units_seen.update(int(u) for u in unit)
            for g in range(len(unit)):
                mine = wg == g
                if not mine.any():
                    continue
                m = (o_unit == unit[g]) & (o_in < int(t_out[g])) & (o_out > int(t_in[g]))
                n_all += 1
                d = float(np.median(te[mine] - tb[mine])) / 1e3
                if m.any():
                    n_shared += 1
                    tile_shared.append(d)
                else:
                    tile_alone.append(d)
        print(f"\nCompute units (identifiers from the log): {len(units_seen)} distinct units under the class-{args.cls} workgroups, "
              f"{len(set(int(u) for u in o_unit))} under the other classes' workgroups. Of {n_all} class-{args.cls} workgroups, {n_shared} "
              f"ran on a unit that a workgroup of another class occupied at the same time"
              + (f": their median tile {np.median(tile_shared):.2f} us, the others' {np.median(tile_alone):.2f} us." if tile_shared and tile_alone else "."))
    if rows:
        print(f"\nAll launches: {tot['bytes']:.1f} MB in {tot['span']:.1f} us of kernel span = "
              f"{2 * tot['bytes'] / tot['span']:.2f} TB/s read+write; workgroup time idle at the head "
              f"{tot['head']:.1f} us ({100 * tot['head'] / tot['span']:.1f} % of the span), at the tail "
              f"{tot['tail']:.1f} us ({100 * tot['tail'] / tot['span']:.1f} %).")


if __name__ == "__main__":
    main()
