"""The module that turns rocprofv3 output into the summaries under profiles/, on a small
synthetic trace: the timed launches are the last `steps` dispatches of the convolution kernel,
warm-up launches stay out of every figure, counters are scaled by the calibration copy."""
import json

from paper_1705_10591_amd import profile_summary


def _bench_line(tmp_path, steps):
    line = {"steps": steps, "warmup": 2, "value": 1000.0, "unit": "GFLOP/s",
            "config": {"workload": "S9: dconv_single_channel {N: 1}"},
            "roofline": {"kernel": "dconv_single_channel", "kernel_ms": 0.0101, "bound": "hbm", "achieved": 4000.0,
                         "unit": "GB/s", "peak": 8000.0, "frac": 0.5}}
    p = tmp_path / "bench.out"
    p.write_text("some stderr-like noise\n" + json.dumps(line) + "\n")
    return str(p)


def test_trace_summary_uses_the_timed_launches_only(tmp_path, capsys):
    d = tmp_path / "trace" / "vm"
    d.mkdir(parents=True)
    rows = ['"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"']
    t = 1000
    durs = [50000, 30000, 20000] + [10000, 10200, 9800, 10100]        # three slow warm-up launches, four timed
    for i, dur in enumerate(durs):
        rows.append(f'"KERNEL_DISPATCH","void dconv::single_tiled_kernel<5>(dconv::SingleParams)",{t},{t + dur}')
        t += dur + 500
    rows.append(f'"KERNEL_DISPATCH","__amd_rocclr_copyBuffer",{t},{t + 3000}')
    (d / "1_kernel_trace.csv").write_text("\n".join(rows) + "\n")
    profile_summary.trace(str(tmp_path / "trace"), _bench_line(tmp_path, 4))
    out = capsys.readouterr().out
    assert "timed launches (the last 4 dispatches): median 10.05 us | min 9.80 us | max 10.20 us" in out
    assert "warm-up launches before them (not part of any figure): 3 dispatches" in out
    assert "--only S9 --steps 4" in out
    # 4000 GB/s over 10.1 us by events -> 4019.9 GB/s over the 10.05 us median
    assert "achieved 4019.9 GB/s = 0.5025 of the published peak" in out


def test_traffic_summary_scales_by_the_calibration_copy(tmp_path, capsys):
    for kind, counter, conv, copy in (("fetch", "FETCH_SIZE", 1000.0, 524288.0), ("write", "WRITE_SIZE", 8000.0, 1048576.0)):
        d = tmp_path / kind / "vm"
        d.mkdir(parents=True)
        rows = ['"Kernel_Name","Counter_Name","Counter_Value"']
        rows += [f'"void dconv::single_tiled_kernel<5>(dconv::SingleParams)","{counter}",{conv}'] * 3
        rows += [f'"__amd_rocclr_copyBuffer","{counter}",{copy}', f'"__amd_rocclr_copyBuffer","{counter}",5.0']
        (d / "1_counter_collection.csv").write_text("\n".join(rows) + "\n")
    profile_summary.traffic(str(tmp_path / "fetch"), str(tmp_path / "write"), _bench_line(tmp_path, 4))
    out = capsys.readouterr().out
    assert "scale factors (known / read): FETCH_SIZE 2.0000, WRITE_SIZE 1.0000" in out
    assert "fetched_bytes_per_launch: 2048000" in out          # 1000 KiB x 2.0
    assert "written_bytes_per_launch: 8192000" in out
    assert "traffic_bytes_per_launch: 10240000" in out
