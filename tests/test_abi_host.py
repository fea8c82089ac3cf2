"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/fda.h declares, validates arguments and plans launches."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import fda_synth as S
import paper_2405_20988_amd as F
from paper_2405_20988_amd.binding import make_desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fda.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fda_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = F.load_library()
    names = declared_functions()
    assert {"fda_local_state", "fda_estimate_variance", "fda_sync", "fda_sync_xi", "fda_update_xi"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    # the binding offers the same names
    for n in names:
        assert hasattr(F, n), n


def test_struct_layouts_match_header():
    assert C.sizeof(F.FdaEstimate) == 64
    assert F.FdaEstimate.sync_linear.offset == 40 and F.FdaEstimate.sync_sketch.offset == 44
    assert C.sizeof(F.FdaDesc) == 56
    assert C.sizeof(F.FdaPlanInfo) == 104


def test_strerror():
    assert F.fda_strerror(0) == "success"
    assert "invalid" in F.fda_strerror(-1)
    assert "unknown" in F.fda_strerror(-99)


def _desc(**kw):
    args = dict(K=5, d=61706, dtype=F.FDA_F32, variants=3, l=5, m=250, eps=0.06,
                hash_coef=S.hash_coefficients(0, kw.get("l", 5) if kw.get("l", 5) > 0 else 1))
    args.update(kw)
    return make_desc(**args)


@pytest.mark.parametrize("kw,code", [
    (dict(K=0), -1), (dict(d=0), -1), (dict(d=2**31 - 1), -2), (dict(dtype=7), -1),
    (dict(variants=0), -1), (dict(variants=8), -1), (dict(l=0), -1), (dict(l=17), -1),
    (dict(m=0), -1), (dict(row_stride=100), -1), (dict(eps=-1.0), -1),
    (dict(hash_coef=None), -1), (dict(l=1, m=60000), -2),
])
def test_plan_rejects_bad_descriptions(kw, code):
    desc, keep = _desc(**kw)
    with pytest.raises(F.FdaError) as e:
        F.fda_plan(desc, 256, 163840)
    assert e.value.code == code
    assert F.fda_last_error() != ""


def test_plan_rejects_large_coefficient():
    coef = S.hash_coefficients(0, 5)
    coef[2, 1, 3] = 2**31 - 1
    desc, keep = _desc(hash_coef=coef)
    with pytest.raises(F.FdaError) as e:
        F.fda_plan(desc, 256, 163840)
    assert e.value.code == -2


def test_create_rejects_before_touching_the_device():
    desc, keep = _desc(K=-3)
    with pytest.raises(F.FdaError) as e:
        F.fda_create(desc, 256, 1 << 20)
    assert e.value.code == -1


@pytest.mark.parametrize("name", list(S.CONFIGS))
def test_plan_of_the_five_configs(name):
    c = S.CONFIGS[name]
    dt = F.FDA_F32 if c["dtype"] == "f32" else F.FDA_BF16
    desc, keep = make_desc(c["K"], c["d"], dt, 3, c["l"], c["m"], 0.06, S.hash_coefficients(0, c["l"]))
    p = F.fda_plan(desc, 256, 163840)
    assert p.state_floats == 2 + c["l"] * c["m"]
    assert p.worker_groups * p.workers_per_group >= c["K"]
    assert p.workers_per_group <= 8
    assert p.partitions >= 1
    assert p.lds_bytes <= 163840
    assert p.partitions * p.chunk >= c["d"]
    tile = p.threads * 4                       # a lane owns 4 coordinates of a tile, whatever the slab type
    assert p.chunk % tile == 0
    assert p.worker_slots >= p.workers_per_group and p.sign_split_rows in (0, 1)
    # all five have LDS to spare for sign-split rows (an even number of worker slots, paired additions)
    assert p.sign_split_rows == 1 and p.worker_slots % 2 == 0
    assert p.worker_groups * p.row_groups * p.partitions <= 4 * 256
    # the partial buffers fit in the workspace
    need = p.partitions * c["K"] * (16 + 8 * c["l"] * c["m"])
    assert p.workspace_bytes >= need
    # the mean-state pass: one row group, one round (two workgroups per CU for bf16 slabs), partials fit too
    assert p.mean_row_groups == 1 and p.mean_rows_per_group == c["l"]
    assert p.mean_workgroups_per_cu == (2 if dt == F.FDA_BF16 else 1) and 2 * p.mean_lds_bytes <= 163840
    assert p.mean_partitions % 8 == 0 and p.mean_partitions <= 512
    assert p.mean_partitions * p.mean_chunk >= c["d"] and p.mean_chunk % (p.threads * 4) == 0
    assert p.workspace_bytes >= p.mean_partitions * (24 + 8 * c["l"] * c["m"])
    # sketch bytes the paper quotes for 5 x 250: l * m * 4 = 5 kB (Section 3.3)
    if (c["l"], c["m"]) == (5, 250):
        assert (p.state_floats - 2) * 4 == 5000


def test_plan_chooses_the_rows_the_lds_allows():
    """Sign-split rows need 2 m buckets per row: where even a single row of them does not fit, or more
    worker groups would cost more than the selects they save, the rows stay plain."""
    coef = S.hash_coefficients(0, 16)

    def plan(K, l, m, d=10**6, dt=F.FDA_F32, flags=0):
        desc, keep = make_desc(K, d, dt, 3, l, m, 0.06, coef[:l], flags=flags)
        return F.fda_plan(desc, 256, 163840)
    p = plan(2, 3, 6_000)                  # 3 x 6000 x 2 slots: 144 KB plain, split would need 288
    assert (p.worker_groups, p.worker_slots, p.row_groups, p.sign_split_rows) == (1, 2, 1, 0)
    p = plan(4, 2, 4_500)                  # two groups of two slots with split rows instead of one of four
    assert (p.worker_groups, p.worker_slots, p.sign_split_rows) == (2, 2, 1)
    p = plan(1, 5, 250)                    # a single worker: one slot, 32-bit additions, plain rows
    assert (p.worker_slots, p.sign_split_rows) == (1, 0)
    p = plan(3, 5, 250)                    # three workers take a kernel of four slots (one spare), rows placed
    assert (p.worker_groups, p.worker_slots, p.sign_split_rows, p.placed_row_group) == (1, 4, 1, 5)
    p = plan(3, 5, 250, flags=F.FDA_DESC_PLAIN_TABLE)    # ... or not
    assert (p.worker_groups, p.worker_slots, p.sign_split_rows, p.placed_row_group) == (1, 4, 1, 0)
    p = plan(3, 1, 19_000)                 # one slot per workgroup: the row fills the LDS
    assert (p.worker_groups, p.worker_slots, p.sign_split_rows) == (3, 1, 0)
    p = plan(8, 7, 1000, 350_000_000, F.FDA_BF16)       # cfg5: four groups of two, one round of 256 workgroups
    assert (p.worker_groups, p.worker_slots, p.partitions, p.sign_split_rows) == (4, 2, 64, 1)
    assert p.placed_row_group == 4         # fields of 13 bits: four rows of 2000 buckets per placement group
    p = plan(8, 7, 2049, 10**6, F.FDA_BF16)
    assert p.placed_row_group == 0         # two rows of 4098 buckets are beyond 13 bits
    p = plan(30, 5, 250, 7_000_000)                       # cfg3: one round of 255 workgroups, not three of 760
    assert (p.worker_groups, p.worker_slots, p.partitions) == (5, 6, 51)
    assert p.lds_bytes <= 163840
    # a 32-bit cell takes 16384 terms at most: narrow sketches get more partitions than one round of
    # workgroups needs, so that a cell of a workgroup expects about 12000 terms at most
    for K, l, m, d in ((8, 9, 250, 350_000_000), (2, 2, 8, 300_000_000), (1, 1, 1, 40_000_000)):
        p = plan(K, l, m, d, F.FDA_BF16)
        cells_per_row = m * (2 if p.sign_split_rows else 1)
        terms = 3_500 if p.sign_split_rows else 12_000      # cells of one hash sign do not cancel a common lean
        assert p.chunk <= cells_per_row * terms + p.threads * 4, (K, l, m, p.as_dict())
        assert p.partitions * p.chunk >= d


def test_plan_of_the_mean_state_pass_splits_rows_only_when_it_must():
    coef16 = S.hash_coefficients(0, 16)
    # 16 rows: more than the 8 row slots of a workgroup -> two row groups of 8
    desc, keep = make_desc(8, 10**6, F.FDA_F32, 3, 16, 64, 0.06, coef16)
    p = F.fda_plan(desc, 256, 163840)
    assert (p.mean_row_groups, p.mean_rows_per_group) == (2, 8)
    assert p.mean_row_groups * p.mean_partitions <= 2 * 256
    # 3 x 19000 8-byte cells: one row per workgroup, one workgroup per CU
    desc, keep = make_desc(3, 10**6, F.FDA_F32, 3, 3, 19_000, 0.06, coef16[:3])
    p = F.fda_plan(desc, 256, 163840)
    assert (p.mean_row_groups, p.mean_rows_per_group, p.mean_workgroups_per_cu) == (3, 1, 1)
    assert p.mean_lds_bytes <= 163840
    # a tiny vector: no more partitions than tiles (rounded up to the 8 XCDs)
    desc, keep = make_desc(4, 5000, F.FDA_F32, 3, 5, 250, 0.06, coef16[:5])
    p = F.fda_plan(desc, 256, 163840)
    assert p.mean_partitions == 8 and p.mean_chunk == 2048
    # a sketch row that does not fit in LDS with 8-byte cells is refused
    desc, keep = make_desc(4, 10**6, F.FDA_F32, 3, 2, 30_000, 0.06, coef16[:2])
    with pytest.raises(F.FdaError) as e:
        F.fda_plan(desc, 256, 163840)
    assert e.value.code == -2


def test_plan_linear_only_needs_no_sketch():
    desc, keep = make_desc(60, 10**6, F.FDA_F32, F.FDA_VARIANT_LINEAR)
    p = F.fda_plan(desc, 256, 163840)
    assert p.state_floats == 2 and p.worker_groups == 10 and p.row_groups == 1


def test_header_is_plain_c(tmp_path):
    """include/fda.h is the boundary: it must compile as C99 and as C++ on its own, and the struct
    sizes the binding mirrors must be the compiler's."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "hdr.c"
    src.write_text('#include "fda.h"\n#include <stdio.h>\n'
                   'int main(void) { printf("%d %d %d\\n", (int)sizeof(fda_desc), (int)sizeof(fda_estimate),'
                   ' (int)sizeof(fda_plan_info)); return 0; }\n')
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    exe = tmp_path / "hdr"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe)], check=True)
    sizes = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(x) for x in sizes] == [C.sizeof(F.FdaDesc), C.sizeof(F.FdaEstimate), C.sizeof(F.FdaPlanInfo)]
    gxx = shutil.which("g++")
    if gxx is not None:
        subprocess.run([gxx, "-std=c++11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-x", "c++", "-fsyntax-only",
                        "-I", os.path.join(root, "include"), str(src)], check=True)


def test_cell_tolerance_rule():
    """tests/fda_tolerance.py: cells holding at least half of what their number of average terms
    would give are held to 1e-5 * sum|u|; only the nearly empty rest gets the extra allowance."""
    import numpy as np
    from fda_tolerance import cell_bounds, check_cells
    sk_abs = np.array([[[10.0, 4.0, 0.0, 5.0]]])          # one worker, one row, four cells
    sk_cnt = np.array([[10, 10, 10, 10]])
    bound, dense = cell_bounds(sk_abs, sk_cnt, np.array([1.0]))
    assert dense.tolist() == [[[True, False, False, True]]]
    assert np.allclose(bound, 1e-5 * np.array([[[10.0, 14.0, 10.0, 5.0]]]))
    want = np.zeros((1, 1, 4))
    worst, frac = check_cells(want + np.array([9e-5, 1.3e-4, 9e-5, 2.5e-5]), want, sk_abs, sk_cnt, np.array([1.0]))
    assert worst == pytest.approx(0.9) and frac == 0.5
    with pytest.raises(AssertionError):
        check_cells(want + np.array([1.1e-4, 0, 0, 0]), want, sk_abs, sk_cnt, np.array([1.0]))
    with pytest.raises(AssertionError):                   # a dense cell does not get the allowance
        check_cells(want + np.array([0, 0, 0, 9e-5]), want, sk_abs, sk_cnt, np.array([1.0]))
