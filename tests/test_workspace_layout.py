"""Host-side bounds check of the workspace layout and of the kernels' index arithmetic.

A small host program (tests/host_probe/layout_probe.hip) is compiled against the driver's own
header and prints the regions `make_layout` lays out and the largest index each kernel-side
formula reaches; this test asserts that every such index stays inside its region and that the
32-bit byte offsets of the buffer instructions do not wrap, at the benchmark configurations'
geometry for the tile shapes the library uses there, and for the bf16 fused tile (one channel per
lane, two segments, 12 steps, four waves: 32 channels x 96 steps) whose counter-collection pass
once did not finish: its indexing is in bounds (1.34 GB of records in five slots for config 5), so
whatever stopped that pass is not an out-of-range record or a wrapped offset."""
import json
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2510_21450_amd")


@pytest.fixture(scope="module")
def probe(tmp_path_factory):
    if not os.path.exists(os.path.join(PKG, "libpararnn.so")):
        from paper_2510_21450_amd import build
        build.build()
    exe = tmp_path_factory.mktemp("probe") / "layout_probe"
    cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", f"-I{os.path.join(ROOT, 'include')}", os.path.join(ROOT, "tests", "host_probe", "layout_probe.hip"),
           f"-L{PKG}", "-lpararnn", f"-Wl,-rpath,{PKG}", "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]

    def run(G, S, PR, dtype, B, L, H, backward, tile, slots=1):
        out = subprocess.run([str(exe)] + [str(x) for x in (G, S, PR, dtype, B, L, H, int(backward), *tile, slots)],
                             capture_output=True, text=True, check=True).stdout
        return json.loads(out)
    return run


GRU, LSTM = (3, 1, 6), (4, 2, 8)
CASES = [
    # cell, dtype (0 fp32, 1 bf16), B, L, H, backward, tile, record slots
    ("C5 fused block, default tile", GRU, 1, 4, 65536, 4096, False, (1, 1, 12, 8), 5),
    ("C5 fused block, two-segment tile (not built)", GRU, 1, 4, 65536, 4096, False, (1, 2, 12, 4), 5),
    ("C5 fused block, two-segment tile, 8 slots", GRU, 1, 4, 65536, 4096, False, (1, 2, 12, 4), 8),
    ("C5 per-iteration", GRU, 1, 4, 65536, 4096, False, (2, 2, 8, 8), 1),
    ("C5 backward", GRU, 1, 4, 65536, 4096, True, (1, 1, 8, 8), 1),
    ("4 x C5 fused block", GRU, 1, 8, 131072, 4096, False, (1, 1, 12, 8), 5),
    ("C2 fused block", GRU, 0, 16, 4096, 1024, False, (1, 1, 12, 8), 5),
    ("C2 backward", GRU, 0, 16, 4096, 1024, True, (1, 2, 8, 16), 1),
    ("C3 fused block", LSTM, 0, 8, 2048, 2048, False, (1, 1, 16, 4), 5),
    ("C3 backward", LSTM, 0, 8, 2048, 2048, True, (1, 1, 16, 8), 1),
    ("small H, eight segments", GRU, 0, 3, 1000, 8, False, (1, 8, 4, 2), 5),
    ("widest H allowed", LSTM, 0, 1, 64, 1 << 22, False, (1, 2, 16, 4), 1),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_every_index_stays_inside_its_region(probe, case):
    _, (G, S, PR), dtype, B, L, H, backward, tile, slots = case
    r = probe(G, S, PR, dtype, B, L, H, backward, tile, slots)
    assert r["tiles_exact"] == 1 and r["n_tiles"] > 0                  # the tile count fits an int
    assert r["T"] == tile[1] * tile[2] * tile[3] and r["n_lt"] == -(-L // r["T"])
    assert r["off_rec"] % 256 == 0 and r["off_rec"] >= 128
    # record words (8 bytes each), all slots, end before the next region starts
    rec_end = r["off_rec"] + (r["rec_max"] + 1) * 8
    assert rec_end <= r["off_bnd"] <= r["total"], r
    if not backward:
        assert r["off_bnd"] + (r["bnd_max"] + 1) * 4 <= r["off_iter"] <= r["total"], r
        if dtype == 1:
            assert r["off_iter"] + (r["iter_max"] + 1) * 4 <= r["total"], r
    else:
        assert r["off_part"] + (r["part_max"] + 1) * 4 <= r["total"], r
    # byte offsets inside a wave's window are 32-bit
    assert r["off32_u"] < 2 ** 32 and r["off32_h"] < 2 ** 32, r


def test_two_segment_bf16_tile_at_config_5_geometry(probe):
    """The numbers of the shape that was withdrawn: 512 groups x 683 tiles, 32-column records."""
    r = probe(3, 1, 6, 1, 4, 65536, 4096, False, (1, 2, 12, 4), 5)
    assert (r["n_groups"], r["n_lt"], r["CW"], r["T"]) == (512, 683, 32, 96)
    assert r["n_rec"] == 512 * 683 * 3 * 32 and r["n_rec"] * 5 * 8 == 1342832640
