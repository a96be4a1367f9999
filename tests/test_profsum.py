"""The profiler summariser on made-up counter files: scaling of FETCH_SIZE / WRITE_SIZE by the first device copy of the
run, the derived figures, and the traffic table that bench.py accepts only for the kernel source it was measured on.
CPU only."""
import argparse
import json
import os

from paper_2507_21433_amd import profsum

HEADER = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name",'
          '"Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name",'
          '"Counter_Value","Start_Timestamp","End_Timestamp"\n')
TILE = "void rc::match_tile_kernel<false, 256, 256, 0, true>(rc::(anonymous namespace)::MatchParams)"
COPY = "__amd_rocclr_copyBuffer"


def row(dispatch, kernel, counter, value, start, end):
    return f'{dispatch},{dispatch},"Agent 1",1,7,7,65536,1,"{kernel}",256,0,0,8,0,32,"{counter}",{value},{start},{end}\n'


def write_pass(root, name, rows, bench=None):
    d = os.path.join(root, f"pmc_w4_{name}", "host")
    os.makedirs(d)
    with open(os.path.join(d, "1_counter_collection.csv"), "w") as f:
        f.write(HEADER + "".join(rows))
    if bench:
        with open(os.path.join(root, f"pmc_w4_{name}.json"), "w") as f:
            f.write(json.dumps(bench) + "\n")


def test_summarise_scales_by_the_first_copy_and_keys_the_table_by_the_kernel_source(tmp_path):
    raw, out = str(tmp_path / "raw"), str(tmp_path / "out")
    bench = {"config": {"workload": "cfg4_made_up"},
             "roofline": {"algorithmic_flop": 32768.0 * 1000, "algorithmic_bytes": 1 << 31, "tflops": 1.0, "mfma_frac": 0.1,
                          "gb_per_s": 2.0, "hbm_frac": 0.2, "flop_per_byte": 3.0, "ridge_flop_per_byte": 312.5}}
    # pass A: 8 XCDs x 1000 cycles in 1000 ns -> 1 GHz; 1000 MFMAs x 32 busy cycles on 1024 SIMDs x 1000 cycles
    write_pass(raw, "A", [row(5, TILE, "GRBM_GUI_ACTIVE", 8000, 0, 1000), row(5, TILE, "SQ_VALU_MFMA_BUSY_CYCLES", 32000, 0, 1000),
                          row(5, TILE, "SQ_WAVE_CYCLES", 100, 0, 1000), row(5, TILE, "SQ_WAIT_INST_ANY", 25, 0, 1000)], bench)
    # passes D and E: the first copy of the run (dispatch 2) is the 1 GiB yardstick, a later, larger copy must not be taken
    write_pass(raw, "D", [row(2, COPY, "FETCH_SIZE", 524288, 0, 10), row(9, COPY, "FETCH_SIZE", 999999, 20, 30),
                          row(5, TILE, "FETCH_SIZE", 1048576, 40, 50), row(6, TILE, "FETCH_SIZE", 3145728, 60, 70)], bench)
    write_pass(raw, "E", [row(2, COPY, "WRITE_SIZE", 1048576, 0, 10), row(5, TILE, "WRITE_SIZE", 1024, 40, 50)], bench)
    assert profsum.summarise(argparse.Namespace(workload=4, dir=raw, out=out)) == 0
    table = json.load(open(os.path.join(out, "hbm_traffic.json")))
    assert table["kernel_source_sha256"] == profsum.kernel_source_hash()
    t = table["workloads"]["cfg4_made_up"]
    assert t["fetch_bytes"] == 2 * (1 << 20) * 2048          # mean of the two launches x 2048 bytes per count
    assert t["write_bytes"] == 1024 * 1024                   # 1024 bytes per count
    assert t["hbm_bytes_per_launch"] == t["fetch_bytes"] + t["write_bytes"]
    text = open(os.path.join(out, "match_tile_kernel_cfg4_made_up.md")).read()
    assert "**1.000 GHz**" in text and "**3.1 %**" in text and "25.0 % of wave cycles" in text
    assert "rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv" in text

    # bench.py takes the table only while the kernel source is the one it was measured on
    import bench
    old = bench.TRAFFIC_TABLE
    try:
        bench.TRAFFIC_TABLE = os.path.join(out, "hbm_traffic.json")
        got, note = bench.load_traffic()
        assert note is None and got == {"cfg4_made_up": t["hbm_bytes_per_launch"]}
        table["kernel_source_sha256"] = "0" * 64
        json.dump(table, open(bench.TRAFFIC_TABLE, "w"))
        got, note = bench.load_traffic()
        assert got == {} and "another version" in note
    finally:
        bench.TRAFFIC_TABLE = old


def test_the_tracked_table_matches_the_kernel_source():
    # the table under profiles/ has to be re-measured whenever the kernel source changes: a stale one makes
    # bench.py report traffic: null
    path = os.path.join(profsum.ROOT, "profiles", "hbm_traffic.json")
    table = json.load(open(path))
    assert table["kernel_source_sha256"] == profsum.kernel_source_hash(), "re-run the FETCH_SIZE / WRITE_SIZE passes"
    assert {"cfg2_qwq32b_step", "cfg3_clustered", "cfg4_high_concurrency", "cfg5_small_model"} <= set(table["workloads"])
