"""Host logic of the profile summariser: per-dispatch aggregation of rocprofv3 counter CSVs and the HBM-traffic line that
bench.py reads back."""
import io
import json
import os
import sys
from contextlib import redirect_stdout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_1906_06440_amd import profile_summary as ps  # noqa: E402
import bench  # noqa: E402

HEAD = "Dispatch_Id,Kernel_Name,Grid_Size,Counter_Name,Counter_Value\n"


def _csv(tmp_path, name, rows):
    p = tmp_path / name
    p.write_text(HEAD + "".join("%d,%s,%d,%s,%g\n" % r for r in rows))
    return str(p)


def test_per_dispatch_sums_instances_and_means_over_dispatches(tmp_path):
    # dispatch 1: two hardware instances of the counter (summed); dispatch 2: one
    path = _csv(tmp_path, "c.csv", [(1, "brg::k(int)", 256, "FETCH_SIZE", 10), (1, "brg::k(int)", 256, "FETCH_SIZE", 30),
                                    (2, "brg::k(int)", 256, "FETCH_SIZE", 20), (3, "other", 64, "FETCH_SIZE", 7)])
    agg = ps._per_dispatch(path)
    assert agg[("brg::k(int)", "256")]["FETCH_SIZE"] == [40.0, 20.0]
    assert ps._kernel_mean(path, "FETCH_SIZE", "brg::k") == 30.0


def test_traffic_line_scales_by_the_copy_and_is_read_back_by_bench(tmp_path):
    # the copy moves 262144 KiB each way; FETCH_SIZE reads half of that for it (scale 2), WRITE_SIZE all of it (scale 1)
    f = _csv(tmp_path, "f.csv", [(1, "brg::conv_tile_f32<3>", 1, "FETCH_SIZE", 1000)])
    w = _csv(tmp_path, "w.csv", [(1, "brg::conv_tile_f32<3>", 1, "WRITE_SIZE", 500)])
    cf = _csv(tmp_path, "cf.csv", [(1, "__amd_rocclr_copyBuffer", 1, "FETCH_SIZE", 131072)])
    cw = _csv(tmp_path, "cw.csv", [(1, "__amd_rocclr_copyBuffer", 1, "WRITE_SIZE", 262144)])

    class A:
        fetch, write, copy_fetch, copy_write = f, w, cf, cw
        kernels, sources = "conv_tile_f32:2", "brg_conv_tile.hpp"
    out = io.StringIO()
    with redirect_stdout(out):
        ps.traffic(A)
    line = out.getvalue().strip()
    assert line.startswith("TRAFFIC ")
    t = json.loads(line[len("TRAFFIC "):])
    assert t["bytes_per_step"] == int(2 * (1000 * 2.0 + 500 * 1.0) * 1024)
    assert t["sources_sha"] == bench.kernel_sources_sha(["brg_conv_tile.hpp"])
    # bench.py accepts the line while the kernel source is unchanged and refuses it (null, with the reason) otherwise
    name = bench.TRAFFIC_PROFILE["cfg2"]
    (tmp_path / name).write_text("header\n" + line + "\n")
    assert bench.measured_traffic("cfg2", str(tmp_path)) == (t["bytes_per_step"], "profiles/" + name)
    stale = dict(t, sources_sha="0" * 16)
    (tmp_path / name).write_text("TRAFFIC " + json.dumps(stale) + "\n")
    got, why = bench.measured_traffic("cfg2", str(tmp_path))
    assert got is None and "other kernel sources" in why
    (tmp_path / name).write_text("no such line\n")
    assert bench.measured_traffic("cfg2", str(tmp_path))[0] is None
    assert bench.measured_traffic("cfg4")[0] is None


def test_committed_traffic_profiles_parse():
    for wk in ("cfg2", "cfg3"):
        val, src = bench.measured_traffic(wk)
        assert (val is None) or (val > 0 and src.startswith("profiles/"))
