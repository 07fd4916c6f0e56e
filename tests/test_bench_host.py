"""Host logic of bench.py that needs no GPU: the algorithmic byte counts that the roofline
figures divide by, the parsing of the committed counter summaries, and the one-GPU contract."""
import os
import subprocess
import sys

import pytest

import bench
from paper_2205_12268_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# Bytes per call worked out by hand from the workload shapes (fp32 maps, 4-byte positions, kept
# coefficients as 8-bit codes): transform = B*C_in*N*4 read + B*N*4 of norms;
# inverse = B*C_out*k*4 + B*k*4 + B*C_out*N*4; contraction = B*C_in*k + weights + B*C_out*k*4.
HAND = {
    2: dict(N=131072, k=32768,
            haar_fwd=134_217_728 + 524_288,
            scatter_ihaar=33_554_432 + 131_072 + 134_217_728,
            pointwise=8_388_608 + 2 * 65_536 + 33_554_432),
    3: dict(N=524_288, k=65_536,
            haar_fwd=536_870_912 + 8_388_608,
            scatter_ihaar=268_435_456 + 1_048_576 + 2_147_483_648,
            pointwise=16_777_216 + 2 * 16_384 + 268_435_456),
    4: dict(N=122_880, k=7_680,
            haar_fwd=503_316_480 + 3_932_160,
            scatter_ihaar=31_457_280 + 245_760 + 503_316_480,
            pointwise=7_864_320 + 16_384 + 31_457_280),
}


@pytest.mark.parametrize("n", sorted(HAND))
def test_algorithmic_bytes_match_hand_counts(n):
    cfg = synth.config(n)
    want = HAND[n]
    assert (cfg.N, cfg.k) == (want["N"], want["k"])
    got = bench.algorithmic_bytes(cfg)
    for stage in ("haar_fwd", "scatter_ihaar", "pointwise"):
        assert got[stage] == want[stage], stage
    # the keep pass reads the input again and writes the kept coefficients once, as codes
    assert got["gather"] == cfg.B * cfg.C_in * (4 * cfg.N + cfg.k) + 4 * cfg.B * cfg.k
    # kept coefficients that travel as fp32 (a fixed index list with the layer's own alpha)
    f32 = bench.algorithmic_bytes(cfg, 4, 4)
    assert f32["gather"] - got["gather"] == 3 * cfg.B * cfg.C_in * cfg.k == f32["pointwise"] - got["pointwise"]
    assert got["norm_select"] == 4 * cfg.B * (cfg.N + cfg.k)


def test_bf16_maps_halve_only_the_feature_map_terms():
    cfg = synth.config(2)
    f32, bf16 = bench.algorithmic_bytes(cfg, 4), bench.algorithmic_bytes(cfg, 2)
    maps_in, maps_out = cfg.B * cfg.C_in * cfg.N, cfg.B * cfg.C_out * cfg.N
    assert f32["haar_fwd"] - bf16["haar_fwd"] == 2 * maps_in
    assert f32["gather"] - bf16["gather"] == 2 * maps_in
    assert f32["scatter_ihaar"] - bf16["scatter_ihaar"] == 2 * maps_out
    assert f32["pointwise"] == bf16["pointwise"] and f32["norm_select"] == bf16["norm_select"]


def test_committed_counter_summaries_parse():
    """Every workload the bench reports a roofline for has a counter summary whose line for
    the dominant kernel parses, and the traffic it gives is at least the bytes the kernel
    must move (a summary below that would point at a broken calibration factor)."""
    prof = os.path.join(ROOT, "profiles")
    for n in (2, 3, 4):
        cfg = synth.config(n)
        traffic = bench.read_traffic(prof, cfg.name, "scatter_ihaar_kernel")
        assert traffic is not None, cfg.name
        need = bench.algorithmic_bytes(cfg)["scatter_ihaar"]
        assert 0.97 * need <= traffic <= 1.5 * need, (cfg.name, traffic, need)
    assert bench.read_traffic(prof, "no_such_workload", "scatter_ihaar_kernel") is None
    assert bench.read_traffic(prof, synth.config(2).name, "no_such_kernel") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""     # no JSON line that could be taken for a measurement


def test_copy_calibration_ignores_the_small_copies(tmp_path):
    """The counter summary scales FETCH_SIZE / WRITE_SIZE by what they read for the probe's
    copies of known size; small copies through the same runtime kernel must not enter it."""
    from paper_2205_12268_amd import profsum

    def write(path, counter, copies, kernel_value):
        rows = ["Kernel_Name,Counter_Name,Counter_Value"]
        rows += [f"__amd_rocclr_copyBuffer,{counter},{v}" for v in copies]
        rows += [f"some_kernel(float*),{counter},{kernel_value}"] * 2
        path.write_text("\n".join(rows) + "\n")

    f, w = tmp_path / "f.csv", tmp_path / "w.csv"
    write(f, "FETCH_SIZE", [13.0, 1.5, 512.0, 512.0, 512.0], 100.0)    # reads half the bytes
    write(w, "WRITE_SIZE", [16.0, 0.5, 1024.0, 1024.0, 1024.0], 300.0)
    text = profsum.traffic(str(f), str(w), 1024.0 * 1024.0)
    assert "scale 2.0000" in text and "scale 1.0000" in text
    line = next(ln for ln in text.splitlines() if ln.startswith("some_kernel"))
    assert [float(t) for t in line.split()[1:]] == [204800.0, 307200.0, 512000.0]


def test_block_byte_counts_of_both_routes():
    """Algorithmic bytes of the block (bench.py --config 6): with the middle tensors formed the
    expand layer's inverse writes, and the project layer's two passes read, the expanded tensor;
    chained, the inverse is gone and the two passes read the expand layer's compressed output
    and rank map instead."""
    cfg = synth.block_config(1, 4)
    B, C, Cm, N, k = cfg.B, cfg.C, cfg.C_mid, cfg.N, cfg.k
    assert (B, C, Cm, N, k) == (8, 256, 1024, 65536, 16384)
    formed = bench.block_algorithmic_bytes(cfg, 4, chained=False)
    chained = bench.block_algorithmic_bytes(cfg, 4, chained=True)
    assert formed["l0_scatter_ihaar"] == 4 * B * Cm * k + 4 * B * k + 4 * B * Cm * N
    assert formed["l1_haar_fwd"] == 4 * B * Cm * N + 4 * B * N
    assert chained["l0_scatter_ihaar"] == 0
    src = 4 * B * Cm * k + 4 * B * N
    assert chained["l1_haar_fwd"] == src + 4 * B * N
    assert chained["l1_gather"] == src + 4 * B * k + B * Cm * k          # int8 codes out
    # what the two routes share: the expand layer's passes, both contractions, the last inverse
    for name in ("l0_haar_fwd", "l0_gather", "l0_pointwise", "l1_pointwise", "l1_scatter_ihaar"):
        assert formed[name] == chained[name], name
    assert formed["l1_scatter_ihaar"] == 4 * B * C * k + 4 * B * k + 2 * 4 * B * C * N  # + the skip
    assert sum(chained.values()) < 0.62 * sum(formed.values())


def test_timing_table_rows_are_the_papers():
    """The 24 rows of the paper's table "Inference timing results": image sides, channel counts
    and keep ratios as printed; every row builds a valid block descriptor."""
    assert len(bench.PAPER_TABLE) == 24
    assert {r[0] for r in bench.PAPER_TABLE} == {96, 128, 256, 512}
    assert {r[4] for r in bench.PAPER_TABLE} == {(1, 8), (1, 4), (1, 2)}
    assert sum(1 for r in bench.PAPER_TABLE if r[4] == (1, 2)) == 9
    for side, c, e, B, (num, den), paper in bench.PAPER_TABLE:
        cfg = bench.block_from_shape(synth, f"{side},{c},{e},{B}", num, den)
        assert cfg.N == side * side and cfg.C_mid == c * e and 1.0 < paper < 2.5
        assert cfg.layer(1).C_in == cfg.C_mid and cfg.layer(0).C_out == cfg.C_mid
    rect = bench.block_from_shape(synth, "64x128,16,2,3", 1, 8)
    assert (rect.H, rect.W, rect.C, rect.expansion, rect.B) == (64, 128, 16, 2, 3)
    assert rect.w_dtype == synth.W_BF16 and synth.block_config(1, 4).name == "block_256x256_c256_e4_b8_keep1of4"
    w8 = bench.block_from_shape(synth, "256,256,4,8", 1, 4, "i8")       # --weights i8
    assert w8.w_dtype == synth.W_I8 and w8.layer(1).w_dtype == synth.W_I8 and w8.name.endswith("_w8")
