"""CPU checks of the C-ABI library: it loads, exports what the header declares, and its host-side
validation answers without a GPU.  No compute entry point is launched here."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2509_06362_amd import binding, workloads as W

ROOT = Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "maaso.h"


@pytest.fixture(scope="module")
def lib():
    if not binding.LIB_PATH.exists():
        from paper_2509_06362_amd import build
        build.build_library()
    return binding.load_library()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(maaso_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"maaso_profile_tables_load", "maaso_score_assign", "maaso_placement_sweep"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in maaso.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_the_header():
    # sizes follow from the C declaration order on LP64
    assert C.sizeof(binding.ProfileDesc) == 64
    assert C.sizeof(binding.Requests) == 40
    assert C.sizeof(binding.Placements) == 48
    assert C.sizeof(binding.Params) == 20
    assert C.sizeof(binding.AssignOut) == 48
    assert C.sizeof(binding.ScoreWeights) == 16
    assert C.sizeof(binding.ScoreOut) == 48
    assert C.sizeof(binding.PartitionWork) == 19 * 8


def test_strerror(lib):
    assert binding.strerror(0) == "ok"
    for s in range(-9, 0):
        assert binding.strerror(s) not in ("ok", "unknown status")
    assert binding.strerror(-99) == "unknown status"


def _load(w, **over):
    kw = dict(n_tp=w.n_tp, b_cap=w.b_cap, prefill_a=w.prefill_a, prefill_p=w.prefill_p, tbt=w.tbt,
              d_ttft=w.d_ttft, d_tbt=w.d_tbt, tp_degree=w.tp_degree, device=0)
    kw.update(over)
    return binding.maaso_profile_tables_load(**kw)


def test_load_validates_on_the_host(lib):
    w = W.config0(n_req=8)
    out = C.c_void_p(123)
    assert lib.maaso_profile_tables_load(None, 0, C.byref(out)) == -1 and out.value is None
    bad = w.tbt.copy(); bad[1, 3] = -1.0
    with pytest.raises(binding.MaasoError) as e:
        _load(w, tbt=bad)
    assert e.value.status == -3
    bad = w.prefill_p.copy(); bad[0, 1] = np.inf
    with pytest.raises(binding.MaasoError) as e:
        _load(w, prefill_p=bad)
    assert e.value.status == -3
    with pytest.raises(binding.MaasoError) as e:
        _load(w, d_ttft=np.array([0.5, 0.0, 1.0], np.float32))
    assert e.value.status == -3
    with pytest.raises(binding.MaasoError) as e:
        _load(w, d_ttft=np.full(17, 1.0, np.float32), d_tbt=np.full(17, 0.1, np.float32))
    assert e.value.status == -2
    big = np.ones((4, 2000), np.float32)
    with pytest.raises(binding.MaasoError) as e:
        _load(w, b_cap=1999, prefill_a=big, prefill_p=big, tbt=big)
    assert e.value.status == -2


def test_null_context_is_rejected(lib):
    assert lib.maaso_score_assign(None, None, None, None, None, None) == -1
    assert lib.maaso_placement_sweep(None, None, None, None, None, None, None, None) == -1
    assert lib.maaso_placement_score(None, None, None, None, None, None, None) == -1
    assert lib.maaso_placement_score_sets(None, None, 1, None, None, None, None, None) == -1
    assert lib.maaso_placement_score_sets(None, None, 0, None, None, None, None, None) == -1
    assert lib.maaso_score_assign_selected(None, None, None, None, None, None, None) == -1
    assert lib.maaso_profile_fit(0, 1, None, None, None, 8, 1.0, 2.0, None, None) == -1
    assert lib.maaso_split_by_slo(None, None, 0, None, None, None, None, None, None) == -1
    assert lib.maaso_ins_deploy_select(None, None, None, None, 0, 0, None, None, None) == -1
    assert lib.maaso_resource_partition(None, 0, None, None, None, None, None, None, 0, 0, None, None,
                                        None) == -1
    assert lib.maaso_ctx_device_status(None, None) == -1
    assert lib.maaso_ctx_set_launch_shape(None, 0, 0, 0, 0) == -1
    assert lib.maaso_ctx_set_wait_limit(None, 1) == -1
    assert lib.maaso_ctx_kernel_timing(None, 1) == -1
    assert lib.maaso_ctx_kernel_elapsed(None, None, None) == -1
    assert lib.maaso_ctx_sweep_evaluated(None, None, None) == -1
    lib.maaso_ctx_destroy(None)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", tmp_path / "libmaaso.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()


def test_product_package_does_not_touch_the_oracle():
    pkg = ROOT / "paper_2509_06362_amd"
    for f in list(pkg.rglob("*.py")) + list(pkg.rglob("*.hip")) + list(pkg.rglob("*.hpp")):
        text = f.read_text()
        assert "import oracle" not in text and "from oracle" not in text, f
        assert "maaso_oracle" not in text, f


def test_header_is_plain_c_and_layouts_agree_with_the_binding(lib, tmp_path):
    """maaso.h compiles as C99 with nothing but <stdint.h>, a C program links against the library,
    and the C compiler's struct sizes are the ones the ctypes binding marshals."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "abi_check.c"
    src.write_text(
        '#include <stdio.h>\n#include "maaso.h"\n'
        "int main(void) {\n"
        '  printf("%zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(maaso_profile_desc), sizeof(maaso_requests),\n'
        "         sizeof(maaso_placements), sizeof(maaso_params), sizeof(maaso_assign_out),\n"
        "         sizeof(maaso_score_weights), sizeof(maaso_score_out), sizeof(maaso_partition_work));\n"
        '  printf("%s\\n", maaso_strerror(MAASO_OK));\n'
        '  printf("%d\\n", maaso_score_assign(NULL, NULL, NULL, NULL, NULL, NULL));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "abi_check"
    pkg = binding.LIB_PATH.parent
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", f"-I{HEADER.parent}",
                    str(src), "-o", str(exe), f"-L{pkg}", "-lmaaso", f"-Wl,-rpath,{pkg}",
                    "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    sizes = [int(x) for x in out[0].split()]
    assert sizes == [C.sizeof(t) for t in (binding.ProfileDesc, binding.Requests, binding.Placements,
                                           binding.Params, binding.AssignOut, binding.ScoreWeights,
                                           binding.ScoreOut, binding.PartitionWork)]
    assert out[1] == "ok" and int(out[2]) == -1


def test_static_scratch_array_is_visible_to_the_runtime(lib, tmp_path):
    """hipGetSymbolAddress finds a device variable by name in the code object, so the static scratch
    array of maaso_placement_sweep_noalloc must be a GLOBAL symbol there (a file-local one makes the
    runtime abort at load).  Checked on the code object embedded in the built library."""
    import shutil
    import subprocess
    llvm = Path("/opt/rocm/lib/llvm/bin")
    bundler, readelf = llvm / "clang-offload-bundler", llvm / "llvm-readelf"
    if not (bundler.exists() and readelf.exists() and shutil.which("objcopy")):
        pytest.skip("llvm binutils not available")
    fat = tmp_path / "fatbin"
    subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", str(binding.LIB_PATH),
                    str(fat)], check=True)
    co = tmp_path / "gfx950.co"
    subprocess.run([str(bundler), "--unbundle", "--type=o", f"--input={fat}",
                    "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={co}"], check=True)
    syms = subprocess.run([str(readelf), "-s", str(co)], check=True, capture_output=True, text=True).stdout
    rows = [l.split() for l in syms.splitlines() if l.strip().endswith("scratch") and "OBJECT" in l]
    assert rows, "no scratch object in the device code object"
    assert all(r[4] == "GLOBAL" for r in rows), rows
    assert int(rows[0][2]) == binding.MAASO_NOALLOC_SCRATCH_BYTES


def test_partition_work_fields_follow_the_header():
    """The binding fills maaso_partition_work by position: its field list must be the header's, in order."""
    text = HEADER.read_text()
    body = text[text.index("typedef struct {", text.index("Arrays that maaso_resource_partition_requests")):
                text.index("} maaso_partition_work;")]
    import re
    fields = re.findall(r"^\s*(?:uint32_t|uint8_t|int32_t|float)\*\s*(\w+);", body, flags=re.M)
    assert fields == [name for name, _ in binding.PARTITION_WORK_FIELDS]


def test_every_export_has_declared_argument_types(lib):
    """ctypes passes an integer without a declared type as a C int: a device pointer would be cut to
    32 bits.  The loader refuses to come up with an undeclared signature; check that it looked."""
    for name in binding.EXPORTS:
        if name != "maaso_strerror":
            assert getattr(lib, name).argtypes is not None, name


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = HEADER.parent.parent
    res = subprocess.run([sys.executable, str(root / "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, cwd=root)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)


def test_traffic_figures_go_stale_with_the_kernel_source(monkeypatch):
    """roofline.traffic is a counter reading of a particular kernel: it is reported while the digest of
    that kernel's sources matches and withheld, with both digests, once they have changed."""
    import bench
    nbytes, info = bench.measured_traffic("cfg4_skewed_stress")
    assert info["source"] == "profiles/sweep_kernel_cfg4.md"
    assert (nbytes is None) == info["stale"]
    monkeypatch.setattr(bench, "kernel_source_digest", lambda kernel: "0" * 16)
    nbytes, info = bench.measured_traffic("cfg4_skewed_stress")
    assert nbytes is None and info["stale"] and info["kernel_digest_now"] == "0" * 16
    assert bench.measured_traffic("cfg0_tiny_distributor")[0] is None
