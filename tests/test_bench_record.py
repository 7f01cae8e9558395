"""The benchmark's result line must stay small: a harness that keeps only the tail of stdout
has to hold all of it, with `roofline` and `cpu_baseline` inside."""
import json

import bench
import synth


def _record(k, with_search=True):
    c = synth.CONFIGS[k]
    tile = None if c["op"] == "reduce_sum" else dict(bm=256, bn=256, bk=16, wm=128, wn=64, vec=4, raster=1, sched=4,
                                                   split_k=1, split_tail=0)
    cpu = {"value": 0.11, "unit": "TFLOP/s", "cores": 16, "kind": "oracle", "seconds": 1.25,
           "sample": "rows 0..4095 of C (4096 x 4096 x 4096 triple loop)"}
    search = {"evaluations": 351, "default_ms": 0.97, "best_ms": 0.955, "speedup_vs_default": 1.0157,
              "evaluations_to_within_1pct": 1} if with_search else None
    return bench.result_record(k, c, (4096, 4096, 4096), 20, 5, 0.0195, 0.9702, tile, 1, True, False, cpu, search)


def test_result_line_is_short_and_complete_for_every_workload():
    for k in synth.CONFIGS:
        out = _record(k)
        line = json.dumps(out)
        assert len(line) < 4000, (k, len(line))
        assert "tuner_log" not in out and "best_so_far_ms" not in out.get("search", {})
        for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                    "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
            assert key in out, key
        for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_source", "hbm_gbs", "kernel_ms_avg"):
            assert key in out["roofline"], key
        assert "workload" in out["config"] and "model" not in out["config"]


def test_headline_record_figures():
    out = _record(3)
    assert out["metric"] == bench.METRIC and out["dtype"] == "f32" and out["vs_baseline"] is None
    r = out["roofline"]
    assert r["bound"] == "mfma" and r["peak"] == 157.3 and r["unit"] == "TFLOP/s"
    # 2 * 4096^3 flop in 0.9702 ms
    assert abs(r["achieved"] - 2 * 4096 ** 3 / 0.9702e-3 / 1e12) < 1e-9
    assert abs(r["frac"] - r["achieved"] / 157.3) < 1e-12
    assert abs(out["value"] - 2 * 4096 ** 3 / (0.0195 / 20) / 1e12) < 1e-9
    # the stored traffic figure is only reported with its source and the rate it implies
    assert (r["traffic"] is None) == (r["traffic_source"] is None) == (r["hbm_gbs"] is None)
    if r["traffic"] is not None:
        assert abs(r["hbm_gbs"] - r["traffic"] / 0.9702e-3 / 1e9) < 1e-6


def test_reduce_record_is_priced_against_hbm():
    out = _record(7, with_search=False)
    assert out["roofline"]["bound"] == "hbm" and out["roofline"]["peak"] == 8000.0 and out["unit"] == "GB/s"
    assert "search" not in out


def test_traffic_table_covers_every_workload_and_names_existing_summaries():
    """Each workload has at least one measured-traffic entry, taken from a summary that is in
    the tree; an entry is only reported while the kernel sources hash to what it was taken with."""
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    assert sorted(bench.TRAFFIC) == list(range(1, 12))
    for k, entries in bench.TRAFFIC.items():
        assert entries
        for e in entries:
            assert e["bytes"] > 0 and len(e["kernel_hash"]) == 16
            assert os.path.isfile(os.path.join(root, e["source"])), e["source"]
