"""bench.py reports HBM traffic figures that come from profiler runs, not from the run itself: this test keeps the
constants in bench.py equal to the committed profile summary they were read from, and checks the summary's own
arithmetic (counter average x 1024 x calibration scale = bytes)."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILE = os.path.join(ROOT, "profiles", "bench_llama8b_5agents_hbm_traffic.md")
KERNELS_OF_CALL = {"align_kv": ("align_kernel",), "anchor_weights": ("dist_partial_kernel", "finalize_kernel"),
                   "suffix_attn": ("attn_mfma_kernel",)}


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)      # only defines functions and constants: nothing runs without main()
    return mod


def parse_profile():
    text = open(PROFILE).read()
    scale_f = float(re.search(r"FETCH_SIZE reads [0-9.]+ per launch -> scale x([0-9]+\.[0-9]+)", text).group(1))
    scale_w = float(re.search(r"WRITE_SIZE reads [0-9.]+ per launch -> scale x([0-9]+\.[0-9]+)", text).group(1))
    rows = {}
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 8 and cells[0] in sum(KERNELS_OF_CALL.values(), ()):
            rows[cells[0]] = dict(fetch_avg=float(cells[2]), read=int(cells[3]), write_avg=float(cells[4]),
                                  written=int(cells[5]), total=int(cells[6]))
    return scale_f, scale_w, rows


def test_profile_table_is_consistent():
    scale_f, scale_w, rows = parse_profile()
    assert set(rows) == set(sum(KERNELS_OF_CALL.values(), ()))
    for name, r in rows.items():
        # the averages are printed to one decimal: 0.05 KiB x scale of slack
        assert abs(r["read"] - r["fetch_avg"] * 1024 * scale_f) <= 0.05 * 1024 * scale_f + 1, name
        assert abs(r["written"] - r["write_avg"] * 1024 * scale_w) <= 0.05 * 1024 * scale_w + 1, name
        assert r["total"] == r["read"] + r["written"], name


def test_bench_traffic_constants_equal_the_profile():
    bench = load_bench()
    _, _, rows = parse_profile()
    for call, kernels in KERNELS_OF_CALL.items():
        read = sum(rows[k]["read"] for k in kernels)
        written = sum(rows[k]["written"] for k in kernels)
        assert bench.HBM_TRAFFIC_READ_WRITTEN[call] == (read, written), call
        assert bench.HBM_TRAFFIC_BYTES[call] == read + written, call


def test_streaming_kernels_move_their_algorithmic_bytes():
    """The align and distance kernels' measured traffic is within 1 % of the algorithmic bytes bench.py divides by."""
    bench = load_bench()
    from paper_2510_12872_amd import workloads
    one = workloads.scaled(workloads.LLAMA8B_5AGENTS, n_agents=1)
    assert abs(bench.HBM_TRAFFIC_BYTES["align_kv"] / one.align_bytes() - 1) < 0.01
    assert 0 <= bench.HBM_TRAFFIC_BYTES["anchor_weights"] / one.distance_bytes() - 1 < 0.02   # + partial sums


def test_mfma_busy_fraction_equals_the_profile():
    bench = load_bench()
    text = open(os.path.join(ROOT, "profiles", "suffix_attn_llama8b_5agents_mfma_counters.md")).read()
    m = re.search(r"= ([0-9.]+) %: the matrix", text)
    assert m and abs(float(m.group(1)) / 100 - bench.SUFFIX_ATTN_MFMA_BUSY_FRAC) < 5e-4
