"""Host-side logic that needs no GPU: the index arithmetic the kernels rely on."""
import numpy as np


def _magic(d):
    return 0 if d <= 1 else (1 << 32) // d + 1


def _udiv_magic(u, d, m):
    """The kernels' division by a precomputed reciprocal, emulated with exact integers: high word of the
    32 x 32 product, then one multiply-and-compare."""
    if m == 0:
        return u
    q = (u * m) >> 32
    q &= 0xFFFFFFFF
    return q - 1 if ((q * d) & 0xFFFFFFFF) > u else q


def test_reciprocal_division_is_exact_over_the_admitted_range():
    """Sub-tile ids are below 2^30 / 16 and divisors (sub-tiles per image, per row) are arbitrary: the corrected
    form must be exact where the bare high-word estimate is not (power-of-two grids with many streams)."""
    rng = np.random.default_rng(5)
    bad_plain = 0
    for d in [2, 3, 4, 7, 16, 49, 64, 196, 4096, 16384, 65536, 12345, 99991, (1 << 20) + 3]:
        m = _magic(d)
        us = {0, 1, d - 1, d, d + 1, (1 << 26) - 1, (1 << 26), (1 << 30) - 1}
        us |= {k * d - 1 for k in (2, 1000, (1 << 26) // d) if k * d - 1 > 0}
        us |= {k * d for k in (2, 1000, (1 << 26) // d)}
        us |= set(int(v) for v in rng.integers(0, 1 << 30, size=2000))
        for u in us:
            assert _udiv_magic(u, d, m) == u // d, (u, d)
            bad_plain += ((u * m) >> 32) != u // d
    assert bad_plain > 0  # the uncorrected estimate does fail in this range: the correction is needed
    # the advisor's cases: last sub-tile of stream >= 16 at 32 streams of 128 x 128 sub-tiles
    d = 16384
    u = 17 * d - 1
    assert ((u * _magic(d)) >> 32) != u // d and _udiv_magic(u, d, _magic(d)) == u // d


def test_position_kernel_unit_shapes_terminate_and_fit(tmp_path):
    """The work-unit choice of the position-gather kernel (pure host code): compiled alone and run over the
    benchmark shapes and a sweep; it must end, and what it picks must respect the kernel's limits (staged units
    and output positions per thread, LDS budget) and cover every output row and stream."""
    import os
    import re
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "pos_shape_test"
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(root, "include"), "-I",
                    os.path.join(root, "paper_1802_09723_amd", "csrc"), os.path.join(root, "tests", "host", "pos_shape_test.cpp"),
                    "-o", str(exe)], check=True)
    cases = [(1, 32, 32, 16, 16, 3, 1, 1, 1, 1), (512, 13, 13, 384, 384, 3, 1, 1, 1, 1), (512, 27, 27, 96, 256, 5, 2, 2, 1, 1),
             (257, 256, 256, 16, 4, 3, 1, 1, 1, 1), (3, 100, 100, 32, 8, 1, 0, 1, 1, 1)]
    for n in (1, 2, 64):
        for hw, c in ((56, 64), (28, 128), (14, 256), (7, 512)):
            cases.append((n, hw, hw, c, c, 3, 1, 1, 2, 2))
    rng = np.random.default_rng(9)
    for _ in range(60):
        k = int(rng.choice([1, 3, 5, 7]))
        hw = int(rng.integers(k, 80))
        grp = int(rng.choice([1, 2]))
        cases.append((int(rng.integers(1, 600)), hw, int(rng.integers(k, 80)), 16 * grp * int(rng.integers(1, 9)),
                      4 * grp * int(rng.integers(1, 70)), k, int(rng.integers(0, k)), grp, int(rng.choice([1, 2])), int(rng.choice([1, 2]))))
    eligible = 0
    for cse in cases:
        out = subprocess.run([str(exe)] + [str(v) for v in cse], check=True, capture_output=True, text=True, timeout=10).stdout
        if out.strip() == "no":
            continue
        eligible += 1
        f = {k: int(v) for k, v in re.findall(r"(\w+)=(\d+)", out)}
        n, h, w, ci, co, k, pad, grp, es, terms = cse
        ho, wo = h + 2 * pad - k + 1, w + 2 * pad - k + 1
        assert f["npos"] * 2 <= 256 * 10 and f["G"] * f["R"] * wo <= 512 * 2, (cse, f)
        assert f["lds"] <= 160 * 1024 - 1024, (cse, f)
        assert f["nbands"] * f["R"] >= ho and f["nsg"] * f["G"] >= n, (cse, f)
        assert f["units"] == f["nsg"] * f["nbands"] * grp * f["ncg"], (cse, f)
        assert f["RB"] == f["R"] + k - 1 and f["WP"] == w + pad and f["npos"] == f["G"] * f["RB"] * f["WP"] + pad
    assert eligible >= 20


def test_binary_band_geometry_terminates_fits_and_covers(tmp_path):
    """The band choice of the binary delta kernel (pure host code), compiled alone and run over the configuration
    shapes and a sweep: it must end; the bands cover every output row; a band's window, flags, list and filter words
    fit the LDS budget; and where the single-launch step is allowed every input position lies in the window of the band
    that owns its row (else a change would be missed or counted twice)."""
    import os
    import re
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "bin_shape_test"
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(root, "include"), "-I",
                    os.path.join(root, "paper_1802_09723_amd", "csrc"), os.path.join(root, "tests", "host", "bin_shape_test.cpp"),
                    "-o", str(exe)], check=True)
    cases = [(1, 28, 28, 256, 256, 3, 1, 1, 1), (64, 28, 28, 256, 256, 3, 1, 1, 1), (1, 14, 14, 512, 512, 3, 1, 1, 1),
             (64, 14, 14, 512, 512, 3, 1, 1, 1), (1, 6, 300, 256, 16, 3, 1, 1, 1), (3, 30, 26, 128, 48, 3, 1, 1, 1),
             (1, 40, 40, 64, 32, 3, 1, 1, 1), (70000, 8, 8, 32, 8, 3, 1, 1, 1), (2, 11, 9, 128, 32, 3, 2, 1, 2),
             (1, 9, 9, 32, 8, 1, 2, 0, 1), (5, 200, 200, 32, 8, 5, 1, 2, 1)]
    rng = np.random.default_rng(17)
    for _ in range(80):
        k = int(rng.choice([1, 3, 5, 7]))
        grp = int(rng.choice([1, 2]))
        cases.append((int(rng.integers(1, 300)), int(rng.integers(k, 90)), int(rng.integers(k, 90)), 32 * grp * int(rng.integers(1, 9)),
                      grp * int(rng.integers(1, 130)), k, int(rng.choice([1, 2, 3])), int(rng.integers(0, k)), grp))
    banded = fused = 0
    for cse in cases:
        out = subprocess.run([str(exe)] + [str(v) for v in cse], check=True, capture_output=True, text=True, timeout=10).stdout
        if out.strip() == "no":
            continue
        f = {k: int(v) for k, v in re.findall(r"(\w+)=(\d+)", out)}
        n, h, w, ci, co, k, stride, pad, grp = cse
        assert f["ho"] == (h + 2 * pad - k) // stride + 1 and f["wo"] == (w + 2 * pad - k) // stride + 1
        if f["R"] == 0:
            continue
        banded += 1
        R, nb = f["R"], f["nbands"]
        assert nb * R >= f["ho"] and (nb - 1) * R < f["ho"], (cse, f)           # every output row in exactly one band
        assert n * nb <= 65535 and R * f["wo"] <= 65535, (cse, f)               # grid and 16-bit list entries
        assert f["lds"] <= (79 * 1024 if f["wlds"] else 64 * 1024 - 64), (cse, f)
        assert f["bth"] == (R - 1) * stride + k and f["btw"] == (f["wo"] - 1) * stride + k, (cse, f)
        if f["fused"]:
            fused += 1
            assert f["vec4"] == 1
            # band b stages input rows [b R stride - pad, b R stride - pad + bth) and all columns [-pad, -pad + btw);
            # it owns rows [b R stride, (b + 1) R stride), the last band up to h
            assert -pad + f["btw"] >= w, (cse, f)
            for b in range(nb):
                lo = b * R * stride
                hi = h if b == nb - 1 else (b + 1) * R * stride
                assert lo >= b * R * stride - pad and hi <= b * R * stride - pad + f["bth"], (cse, f, b)
    assert banded >= 40 and fused >= 10
