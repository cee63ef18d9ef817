"""The seeded input generators: determinism, numpy/torch agreement, and the
property that makes mis-routing visible (blocks differ when any index differs)."""
import numpy as np
import torch

import iso_inputs as gen


def test_numpy_and_torch_generators_agree_bitwise():
    for kind, m in (("u32", 32), ("u32", 7), ("f32", 64), ("u32", 4096), ("u8", 48), ("u8", 5), ("u8", 4096)):
        a = gen.alltoall_send(3, 50, 5, m, kind)
        b = gen.alltoall_send_torch(3, 50, 5, m, kind, rank_chunk=16).numpy()
        assert a.dtype == np.uint8 and a.shape == (50, 5, m)
        assert np.array_equal(a, b)
        g = gen.allgather_send(3, 50, m, kind)
        assert np.array_equal(g, gen.allgather_send_torch(3, 50, m, kind).numpy())
    ranks = np.array([[5, 9], [0, 49]])
    slots = np.array([[1, 2]])
    a = gen.block_bytes(8, ranks, slots, 48)
    b = gen.block_bytes_torch(8, torch.from_numpy(ranks), torch.from_numpy(slots), 48).numpy()
    assert a.shape == (2, 2, 48) and np.array_equal(a, b)


def test_rows_are_a_pure_function_of_their_indices():
    full = gen.alltoall_send(9, 40, 6, 32)
    part = gen.alltoall_send(9, 40, 6, 32, rank_lo=10, rank_hi=17)
    assert np.array_equal(full[10:17], part)
    assert not np.array_equal(full, gen.alltoall_send(10, 40, 6, 32))


def test_every_block_and_every_word_is_distinct_enough():
    a = gen.alltoall_send(1, 64, 8, 32).reshape(64 * 8, 32)
    assert len({row.tobytes() for row in a}) == 64 * 8
    w = a.view(np.uint32)
    # first word alone already separates all (rank, slot) pairs (bijective stages)
    assert len(set(w[:, 0].tolist())) == 64 * 8
    # words inside a block are pairwise distinct
    big = gen.alltoall_send(1, 2, 2, 4096).reshape(4, 4096).view(np.uint32)
    for row in big:
        assert len(set(row.tolist())) == row.size


def test_f32_blocks_are_finite_and_in_range():
    f = gen.alltoall_send(2, 16, 3, 1024, "f32").view(np.float32)
    assert np.isfinite(f).all() and f.min() >= -1.0 and f.max() < 1.0
    assert abs(float(f.mean())) < 0.05


def test_config_table_matches_the_named_workloads():
    c = gen.CONFIGS
    assert [x.p for x in c] == [64, 32768, 65536, 262144, 32768]
    assert [x.s for x in c] == [8, 26, 12, 26, 40]
    assert [x.m for x in c] == [32, 256, 1024, 128, 4096]
    assert c[3].m_sweep == (16, 64, 128)
    c5 = c[4]
    assert len(set(c5.offsets)) == 40 and all(any(v) for v in c5.offsets)
    assert all(-3 <= x <= 3 for v in c5.offsets for x in v)
    assert gen.random_distinct(5, -3, 3, 40, 1606_07676) == list(c5.offsets)
    assert gen.get_config("2") is c[1] and gen.get_config(c[2].name) is c[2]


def test_bench_refuses_more_than_one_gpu():
    """The benchmark runs on one GPU only and must say so instead of starting ranks."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert out.returncode != 0 and out.stdout == ""
    assert "ONE GPU" in out.stderr


def test_u8_blocks_are_one_draw_per_byte():
    """Config 5's content: every byte its own mixer value (low 8 bits), so all 256 byte values
    occur about equally often and bytes of one block are not the bytes of consecutive words."""
    b = gen.alltoall_send(4, 8, 3, 4096, "u8")
    assert b.dtype == np.uint8 and b.shape == (8, 3, 4096)
    w = gen.block_words(4, np.arange(8)[:, None], np.arange(3)[None, :], 4096, "u8")
    assert np.array_equal(b, (w & 0xFF).astype(np.uint8))
    counts = np.bincount(b.reshape(-1), minlength=256)
    assert counts.min() > 0.7 * b.size / 256 and counts.max() < 1.3 * b.size / 256
    assert gen.get_config(5).kind == "u8"


def test_recorded_traffic_summaries_cover_the_benchmark_workloads():
    """bench.py counts roofline.traffic in child runs under rocprofv3 and, where that is switched off
    or fails, reports the value of the committed rocprofv3 summary of the same workload.  Every
    workload of the default run has one, its figures are consistent, and every summary states the
    command that made it."""
    import glob
    import os
    import re
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    for tag in ("c5_m4096", "c2_m256", "c3_m1024", "c4_m128"):
        t, source = bench.recorded_traffic(tag)
        assert isinstance(t, int) and t > 0 and source.startswith("recorded: profiles/"), tag
    files = sorted(glob.glob(os.path.join(root, "profiles", "*.txt")))
    assert len(files) >= 20
    for path in files:
        text = open(path).read()
        assert "rocprofv3 --" in text and "python3 bench.py" in text, path
        assert "_work" not in text, path
        if path.endswith("_hbm_traffic.txt"):
            t = int(re.search(r"^traffic_bytes_per_launch = (\d+)", text, re.M).group(1))
            a = int(re.search(r"^algorithmic_bytes_per_launch = (\d+)", text, re.M).group(1))
            assert 0.5 < t / a < 3.0, path
    # the benchmark workloads move what the schedule asks for and nothing more
    for tag in ("c5_m4096", "c2_m256", "c3_m1024", "c4_m128"):
        (path,) = glob.glob(os.path.join(root, "profiles", f"*{tag}_hbm_traffic.txt"))
        text = open(path).read()
        a = int(re.search(r"^algorithmic_bytes_per_launch = (\d+)", text, re.M).group(1))
        assert abs(bench.recorded_traffic(tag)[0] / a - 1.0) < 0.01, tag


def test_counter_summary_scales_by_the_plain_copy(tmp_path):
    """The per-launch traffic that bench.py derives from a rocprofv3 counter file: kernels of the
    step averaged, the plain copy's reading taken as 1 GiB, other counters and kernels ignored."""
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    rows = ["Kernel_Name,Counter_Name,Counter_Value",
            '"void iso::copy_kernel(uint4*)",FETCH_SIZE,524288.0',           # reads 2 x what it counts
            '"void iso::copy_kernel(uint4*)",FETCH_SIZE,524288.0',
            '"void iso::shift_round_kernel<a, b>(iso::ShiftArgs)",FETCH_SIZE,1000.0',
            '"void iso::shift_round_kernel<a, b>(iso::ShiftArgs)",FETCH_SIZE,3000.0',
            '"void iso::shift_round_kernel<a, b>(iso::ShiftArgs)",WRITE_SIZE,77.0',
            '"void at::native::fill_kernel()",FETCH_SIZE,999999.0']
    path = tmp_path / "x_counter_collection.csv"
    path.write_text("\n".join(rows) + "\n")
    kib, scale = bench.scaled_counter_average(str(path), "FETCH_SIZE")
    assert scale == 2.0 and kib == 4000.0
    assert bench.scaled_counter_average(str(path), "WRITE_SIZE") is None          # no copy to scale by
