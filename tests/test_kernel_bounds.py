"""Bounds check of every kernel's addressing on the CPU (no GPU involved).

Each kernel family is compiled as plain C++ against tests/emul/hip/hip_runtime.h, a
stand-in for the HIP runtime that runs a launch as nested loops over workgroups and
threads, and linked with AddressSanitizer.  The driver (tests/emul/bounds_check.cpp)
allocates the operands with exactly the sizes the C-ABI documents and calls the same
launchers the library calls, so an index that leaves an operand, the workspace or an
LDS array aborts here instead of faulting a GPU.  Values are not checked (barriers and
cross-lane operations have no meaning in this emulation); parity is the GPU tests' job.
Two families are value checks all the same: MCOVER and M2COVER run the reduce kernels of the
matrix-core moment paths over accumulators that all hold 1 and count, per unique entry, how many
tile positions the tile table (or task list) and the kept-position rules map to it: exactly one.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMUL = os.path.join(ROOT, "tests", "emul")
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")

CASES = {
    # mttkrp: n R  (n <= 96 with R <= 32: the row kernel; multiples of 16: pair items; others: repacked first)
    "MTTKRP": [(1, 1), (5, 4), (16, 16), (17, 3), (32, 5), (48, 80), (64, 16), (100, 20), (160, 20),
               (208, 7), (256, 64), (512, 64)],
    # batax: n  (one-pass kernel to 16384, two-pass beyond; n % 4 != 0 takes the guarded loads)
    "BATAX": [(1,), (5,), (64,), (100,), (1000,), (1023,), (4096,), (8192,), (9001,), (12288,), (16384,), (16390,)],
    # ttm: rows nl R  (split-K shapes, the general MFMA path with and without ragged sizes, the plain path for R > 256)
    # (more than 16384 rows: the streaming split-K kernel)
    "TTM": [(8632, 512, 64), (16590, 128, 48), (1090, 256, 16), (208, 512, 32), (1, 64, 16), (777, 48, 32),
            (50, 7, 5), (33, 16, 256), (16385, 512, 64), (40001, 64, 16), (33000, 256, 48), (100, 500, 50),
            (10, 1, 1), (300, 130, 250), (40, 33, 300),
            # at most three row tiles per CU: the one-shot kernel (all NS, several CT, ragged last tile)
            (1089, 64, 64), (2088, 128, 48), (8290, 256, 32), (244, 64, 16), (11828, 512, 64), (12288, 512, 64),
            (4097, 128, 16), (12289, 512, 64)],
    # moment3: N n accumulate  (n = 64 is the MFMA path, others the plain path)
    # (n <= 40 and 64 < n <= 256: the tile path; 40 < n <= 64: the MFMA path; larger n: the plain path)
    "MOMENT3": [(5000, 64, 0), (4097, 64, 1), (63, 64, 0), (100000, 64, 0), (1000, 20, 0), (3, 5, 1),
                (700, 70, 0), (100, 1, 0), (3000, 13, 1), (257, 40, 0), (500, 48, 0), (130, 129, 0), (70, 200, 0),
                (33, 256, 0), (20, 300, 0), (50, 66, 1), (40, 100, 0)],
    # moment2: N n accumulate  (n <= 16: a lane per sample; n <= 64: the MFMA path; n <= 1024: strips of 64
    # columns on the matrix cores; beyond: the plain path)
    "MOMENT2": [(5000, 64, 0), (4097, 64, 1), (3, 64, 0), (100000, 64, 0), (1000, 20, 0), (3, 5, 1), (700, 70, 0),
                (50, 300, 0), (200, 65, 1), (40, 1024, 0), (9, 1030, 0), (1000, 6, 0), (300000, 13, 1), (70, 16, 0),
                (5, 1, 0), (600, 17, 0), (1000, 128, 0), (37, 130, 1), (300, 1000, 0), (5, 100, 0), (2100, 192, 0),
                (37, 190, 0), (50, 513, 0), (9, 250, 1)],   # n % 4 != 0 with three or more strips
    # moment4: N n accumulate  (17 <= n <= 52: register tiles on the vector ALUs, also run here for smaller n;
    # 53 <= n <= 256: the matrix-core path, table in the workspace; n <= 16 is the COVARSMALL family's)
    "MOMENT4": [(300, 64, 0), (65, 64, 1), (1, 64, 0), (200, 20, 0), (130, 63, 0), (3, 5, 1), (9, 70, 0),
                (70, 65, 1), (3, 129, 0), (100, 80, 0), (37, 75, 1), (20, 130, 0), (9, 200, 1), (70, 13, 0),
                (300, 40, 0), (130, 52, 1), (90, 17, 0), (70, 30, 0), (200, 45, 1), (65, 29, 0)],
    # one-pass covariance for at most sixteen features: N n accumulate  (n <= 6: every lane holds all entries;
    # 7 <= n <= 16: the entries are split over the waves)
    "COVARSMALL": [(1000, 6, 0), (3, 6, 1), (257, 5, 0), (300000, 4, 0), (70, 1, 1), (513, 3, 0), (1000, 13, 0),
                   (65, 7, 1), (130, 16, 0), (3, 10, 0), (200, 9, 1), (50000, 14, 0)],
    # cover of the matrix-core moment kernels: order n  (every unique entry kept at exactly one tile position)
    "MCOVER": [(4, 30), (4, 32), (4, 41), (4, 48), (4, 64), (4, 56), (4, 80), (4, 75), (4, 100), (4, 128), (3, 65), (3, 80), (3, 100), (3, 128), (3, 200),
               (3, 256), (3, 250)],
    # cover of the second moment's strip path: n  (every pair i <= j kept at exactly one tile position of one task)
    "M2COVER": [(65,), (100,), (128,), (150,), (192,), (200,), (258,), (320,), (513,), (960,), (1000,), (1024,)],
    # expand: n order | n 10+kind w p0 count  (device unrank of kind 2, 3, 4 = band, 5 = sym4)
    "EXPAND": [(64, 3), (100, 2), (7, 3), (1, 2), (17, 4), (32, 4), (100, 12, 0, 17, 5000), (100, 13, 0, 17, 5000),
               (100, 14, 7, 17, 1000), (40, 15, 0, 17, 5000)],
    # table: op (0 thp | 1 mttkrp with fixed indices | 2 band expand), structure | kind | w, ni, nj | nk, nl, R
    "TABLE": [(0, 0, 33, 40, 20, 0), (0, 0, 7, 5, 3, 0), (0, 1, 9, 31, 64, 0), (0, 2, 31, 9, 6, 0), (0, 3, 50, 50, 12, 0),
              (0, 3, 1, 1, 1, 0), (1, 0, 5, 7, 33, 70), (1, 1, 5, 100, 64, 48), (1, 1, 3, 9, 7, 300),
              (1, 2, 77, 6, 128, 32), (1, 2, 9, 4, 10, 3), (2, 3, 20, 0, 8, 0), (2, 0, 9, 0, 5, 0), (2, 40, 13, 0, 4, 0)],
}


@pytest.fixture(scope="module")
def builds(tmp_path_factory):
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    out = tmp_path_factory.mktemp("emul")

    def build(fam):
        exe = str(out / ("bounds_" + fam.lower()))
        opt = "-O0" if fam == "COVARSMALL" else "-O1"       # its unrolled loop nests take minutes to optimise
        # (a shared array is a local array of the emulated thread; locals start at zero so that a thread which reads
        # what the other threads of its workgroup would have written reads zeros, not stack contents)
        cmd = [CLANG, "-std=c++17", opt, "-g", "-fsanitize=address", "-fno-omit-frame-pointer", "-ftrivial-auto-var-init=zero",
               "-DCHECK_" + fam, "-I", EMUL, "-x", "c++", os.path.join(EMUL, "bounds_check.cpp"), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, "host build of %s failed:\n%s" % (fam, r.stderr[-4000:])
        return fam, exe

    # the families build side by side (the one-pass covariance kernels alone take two minutes to compile)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(pool.map(build, list(CASES)))


@pytest.mark.parametrize("fam", sorted(CASES))
def test_kernel_addressing_in_bounds(builds, fam):
    for case in CASES[fam]:
        r = subprocess.run([builds[fam]] + [str(v) for v in case], capture_output=True, text=True, timeout=600)
        assert r.returncode == 0 and "rc=0" in r.stdout, "%s %s:\n%s\n%s" % (fam, case, r.stdout[-500:], r.stderr[-4000:])


def test_random_ttm_shapes_in_bounds(builds):
    """The contraction launcher picks among five kernels by shape (one-shot, persistent split-K, streaming split-K,
    general MFMA, plain): a seeded sweep of 400 random shapes, dense around the row counts where the choice changes,
    through the same bounds check."""
    import random
    rng = random.Random(20221118)
    for _ in range(400):
        nl = rng.choice([64, 128, 192, 256, 320, 384, 448, 512, 576, 1024, 33, 100, 7, 1, 16, 48])
        R = rng.choice([16, 32, 48, 64, 5, 20, 50, 63, 1, 128, 250, 300])
        rows = rng.choice([rng.randint(1, 600), rng.randint(3900, 4300), rng.randint(8000, 8400), rng.randint(12000, 12400),
                           rng.randint(16300, 16500), rng.randint(1, 40000)])
        if rows * nl > 12_000_000:
            continue
        r = subprocess.run([builds["TTM"], str(rows), str(nl), str(R)], capture_output=True, text=True, timeout=600)
        assert r.returncode == 0 and "rc=0" in r.stdout, "TTM %s:\n%s" % ((rows, nl, R), r.stderr[-3000:])
