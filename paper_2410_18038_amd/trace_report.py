"""Where and when the work of one fused launch ran, from the library's own records.

Input: the per-workgroup trace (``pod_attn_plan_set_trace``) and the event log
(``pod_attn_plan_set_event_log``) of one ``pod_attn_forward`` call in the fused mode.
Output: the numbers that show co-location (paper Section 4.1: both operations resident
on every multiprocessor; Section 5.1: the two overlap in time): how many hardware units
hold one workgroup that started in each operation, and for how much of the time a unit
spends on prefill items one of its wavefronts is also streaming a decode unit.
Plain numpy over the records; no attention arithmetic lives here.
"""
from __future__ import annotations

import numpy as np

TICKS_PER_US = 100.0          # the device's constant-rate clock runs at 100 MHz


def _union_length(begins: np.ndarray, ends: np.ndarray) -> float:
    """Total length of the union of the intervals [begin, end)."""
    if len(begins) == 0:
        return 0.0
    order = np.argsort(begins)
    b, e = begins[order].astype(np.int64), ends[order].astype(np.int64)
    reach = np.maximum.accumulate(e)
    # an interval opens a new run when it begins after everything before it has ended
    new_run = np.concatenate([[True], b[1:] > reach[:-1]])
    run_begin = b[new_run]
    run_end = reach[np.concatenate([np.nonzero(new_run)[0][1:] - 1, [len(b) - 1]])]
    return float((run_end - run_begin).sum())


def _overlap_length(pb, pe, db, de) -> float:
    """Length of (union of prefill intervals) intersected with (union of decode intervals)."""
    both = _union_length(np.concatenate([pb, db]), np.concatenate([pe, de]))
    return _union_length(pb, pe) + _union_length(db, de) - both


def colocation(trace: np.ndarray, events: np.ndarray, n_prefill_items: int, n_decode_units: int) -> dict:
    """Summary of one fused launch.  `trace`: one record per workgroup; `events`: one per item/unit."""
    units = np.unique(trace["cu"])
    per_unit = {int(u): trace[trace["cu"] == u] for u in units}
    both_first = sum(1 for t in per_unit.values()
                     if (t["first_role"] == 0).any() and (t["first_role"] == 1).any())
    exactly_pair = sum(1 for t in per_unit.values()
                       if len(t) == 2 and sorted(t["first_role"].tolist()) == [0, 1])
    t0 = int(trace["t_begin"].min())
    ev_p, ev_d = events[events["kind"] == 0], events[events["kind"] == 1]
    items_once = sorted(ev_p["item"].tolist()) == list(range(n_prefill_items))
    units_once = sorted(ev_d["item"].tolist()) == list(range(n_decode_units))
    overlapped_units, prefill_ticks, overlap_ticks = 0, 0.0, 0.0
    for u in units:
        p, d = ev_p[ev_p["cu"] == u], ev_d[ev_d["cu"] == u]
        pl = _union_length(p["t_begin"], p["t_end"])
        ov = _overlap_length(p["t_begin"], p["t_end"], d["t_begin"], d["t_end"]) if len(p) and len(d) else 0.0
        prefill_ticks += pl
        overlap_ticks += ov
        overlapped_units += 1 if ov > 0 else 0
    xcd_of = lambda cu: int(cu) >> 6
    per_xcd_items = np.bincount([xcd_of(c) for c in ev_p["cu"]], minlength=8).tolist()
    per_xcd_dunits = np.bincount([xcd_of(c) for c in ev_d["cu"]], minlength=8).tolist()
    first_p = trace[trace["first_role"] == 0]
    first_d = trace[trace["first_role"] == 1]

    def span_us(rec, a, b):
        return float(np.median((rec[b].astype(np.int64) - rec[a].astype(np.int64)))) / TICKS_PER_US if len(rec) else 0.0

    return {
        "workgroups": int(len(trace)),
        "hardware_units": int(len(units)),
        "units_with_both_first_roles": int(both_first),
        "units_with_exactly_one_of_each": int(exactly_pair),
        "prefill_items_logged_once": bool(items_once),
        "decode_units_logged_once": bool(units_once),
        "units_where_roles_overlap_in_time": int(overlapped_units),
        "share_of_prefill_time_with_decode_on_same_unit": overlap_ticks / prefill_ticks if prefill_ticks else 0.0,
        "launch_us": (int(trace["t_end"].max()) - t0) / TICKS_PER_US,
        "last_arrival_us": (int(trace["t_begin"].max()) - t0) / TICKS_PER_US,
        "median_first_phase_us": {"prefill_first": span_us(first_p, "t_begin", "t_switch"),
                                  "decode_first": span_us(first_d, "t_begin", "t_switch")},
        "prefill_items_per_xcd": per_xcd_items,
        "decode_units_per_xcd": per_xcd_dunits,
        "prefill_end_us": (int(ev_p["t_end"].max()) - t0) / TICKS_PER_US if len(ev_p) else 0.0,
        "decode_end_us": (int(ev_d["t_end"].max()) - t0) / TICKS_PER_US if len(ev_d) else 0.0,
    }


def as_text(name: str, rep: dict) -> str:
    lines = [f"co-location of one fused launch: {name}"]
    for k, v in rep.items():
        if isinstance(v, float):
            v = f"{v:.3f}"
        lines.append(f"  {k:48s} {v}")
    return "\n".join(lines)
