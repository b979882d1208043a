"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2110_08450_amd import binding as smfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "smfg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(smfg_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert sorted(smfg.EXPORTS) == names
    lib = ctypes.CDLL(smfg.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_bounds_and_host_validation():
    mn, me = smfg.bounds(1024, (15, 10, 5), 111_000_000)
    assert mn == [1024, 16384, 180224, 1081344] and me == [15360, 163840, 901120]
    mn, me = smfg.bounds(1024, (15, 10, 5), 169_000)        # capped by the graph size
    assert mn[-1] == 169_000 and mn[2] == 169_000
    for bad, code in [((0,), smfg.ERR_BAD_FANOUT), ((1025,), smfg.ERR_BAD_FANOUT), ((-2,), smfg.ERR_BAD_FANOUT),
                      ((), smfg.ERR_TOO_MANY_LAYERS), ((1,) * 9, smfg.ERR_TOO_MANY_LAYERS)]:
        with pytest.raises(smfg.SmfgError) as ei:
            smfg.bounds(4, bad, 100)
        assert ei.value.code == code
    assert "fanout" in smfg.strerror(smfg.ERR_BAD_FANOUT)
    assert "duplicate" in smfg.strerror(smfg.ST_DUPLICATE_SEED)


def test_packed_weight_size_is_host_only():
    """smfg_sage_packed_bytes: whole 32-column slices of halfs; 0 for widths the layer does not take."""
    L = smfg.lib()
    assert L.smfg_sage_packed_bytes(128, 256) == 256 * 256 * 2
    assert L.smfg_sage_packed_bytes(8, 1) == 32 * 16 * 2
    assert L.smfg_sage_packed_bytes(256, 33) == 64 * 512 * 2
    for dim, out_dim in [(0, 8), (12, 8), (264, 8), (128, 0), (-8, 8)]:
        assert L.smfg_sage_packed_bytes(dim, out_dim) == 0


def test_oracle_and_library_agree_on_bounds():
    import oracle
    for seeds, fan, n in [(256, (10, 5), 10_000), (4096, (20, 20, 20), 111_000_000), (5, (32,), 20),
                          (64, (100, 100), 5000), (8, (3, -1, 2), 900), (8, (-1,), 900)]:
        assert tuple(smfg.bounds(seeds, fan, n)) == tuple(oracle.worst_case(seeds, fan, n))


def test_header_is_plain_c(tmp_path):
    """include/smfg.h compiles as C99 on its own (plain pointers and sizes, no C++ or torch types)
    and every declared function can be referenced from C."""
    import subprocess
    names = [n for n in _declared()]
    src = tmp_path / "use_header.c"
    body = "\n".join(f"  p[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text('#include "smfg.h"\n#include <stddef.h>\n'
                   f"void (*p[{len(names)}])(void);\n"
                   "int use_all(void) {\n" + body + "\n  smfg_output_t o; o.node_capacity = 0;\n"
                   "  return (int)sizeof(o) + SMFG_MAX_LAYERS + SMFG_FANOUT_ALL;\n}\n")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "use_header.o")])


def test_output_struct_layout_matches_the_binding(tmp_path):
    """The ctypes mirror of smfg_output_t has the size and field offsets the C compiler gives."""
    import subprocess
    src = tmp_path / "layout.c"
    fields = ["indptr", "indices", "node_ids", "features", "counts", "node_capacity", "edge_capacity", "labels"]
    prints = "\n".join(f'  printf("{f} %zu\\n", offsetof(smfg_output_t, {f}));' for f in fields)
    src.write_text('#include "smfg.h"\n#include <stddef.h>\n#include <stdio.h>\nint main(void) {\n'
                   '  printf("size %zu\\n", sizeof(smfg_output_t));\n' + prints + "\n  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    assert int(got["size"]) == ctypes.sizeof(smfg._Output)
    for f in fields:
        assert int(got[f]) == getattr(smfg._Output, f).offset, f
    assert smfg.MAX_LAYERS == 8 and smfg.MAX_BATCHES == 16 and smfg.MAX_FANOUT == 32


def test_graph_create_refuses_bad_arguments_before_touching_a_device():
    """Null, negative and misaligned arguments of smfg_graph_create are turned down by host checks
    that come before the first HIP call, so they can be exercised without a GPU."""
    L = smfg.lib()
    h = ctypes.c_void_p()
    vp = ctypes.c_void_p
    ok_ptr = 0x7f0000001000      # never dereferenced: every case below is refused first
    create = L.smfg_graph_create
    assert create(None, 4, 8, vp(ok_ptr), vp(ok_ptr), None, 0, 0, 0) == smfg.ERR_NULL_PTR
    assert create(ctypes.byref(h), 4, 8, None, vp(ok_ptr), None, 0, 0, 0) == smfg.ERR_NULL_PTR
    assert create(ctypes.byref(h), 4, 8, vp(ok_ptr), None, None, 0, 0, 0) == smfg.ERR_NULL_PTR
    assert create(ctypes.byref(h), -1, 8, vp(ok_ptr), vp(ok_ptr), None, 0, 0, 0) == smfg.ERR_INVALID_ARG
    assert create(ctypes.byref(h), 1 << 31, 8, vp(ok_ptr), vp(ok_ptr), None, 0, 0, 0) == smfg.ERR_INVALID_ARG
    assert create(ctypes.byref(h), 4, 8, vp(ok_ptr + 4), vp(ok_ptr), None, 0, 0, 0) == smfg.ERR_INVALID_ARG
    assert create(ctypes.byref(h), 4, 8, vp(ok_ptr), vp(ok_ptr + 2), None, 0, 0, 0) == smfg.ERR_INVALID_ARG
    assert create(ctypes.byref(h), 4, 8, vp(ok_ptr), vp(ok_ptr), vp(ok_ptr), 0, 2, 0) == smfg.ERR_INVALID_ARG
    assert create(ctypes.byref(h), 4, 8, vp(ok_ptr), vp(ok_ptr), vp(ok_ptr), 8, 2, 15) == smfg.ERR_INVALID_ARG
    assert h.value is None
    # entry points that take raw arrays: null and misaligned pointers, before any launch
    i64 = ctypes.c_int64
    assert L.smfg_gather_rows(None, vp(ok_ptr), vp(ok_ptr), i64(4), vp(ok_ptr), None) == smfg.ERR_NULL_PTR
    assert L.smfg_mean_aggregate(vp(ok_ptr + 2), vp(ok_ptr), i64(8), vp(ok_ptr), i64(4), vp(ok_ptr), i64(4), 8, 2,
                                 vp(ok_ptr), None) == smfg.ERR_INVALID_ARG
    assert L.smfg_mean_aggregate(vp(ok_ptr), vp(ok_ptr), i64(8), vp(ok_ptr + 4), i64(4), vp(ok_ptr), i64(4), 8, 2,
                                 vp(ok_ptr), None) == smfg.ERR_INVALID_ARG
    assert L.smfg_sage_layer(vp(ok_ptr), vp(ok_ptr + 1), i64(8), vp(ok_ptr), i64(4), vp(ok_ptr), i64(4), 8,
                             vp(ok_ptr), None, 8, 0, vp(ok_ptr), 2, None) == smfg.ERR_INVALID_ARG
    assert L.smfg_sample_mfg_static(None, vp(ok_ptr), 4, None, 1, ctypes.c_uint64(1), None, None) == smfg.ERR_NULL_PTR
    assert "internal" in smfg.strerror(smfg.ST_INTERNAL)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bucket_levels_of_the_partition_strategy(tmp_path):
    """Host logic shared with the kernels: how 2^lg hash buckets are laid out in one or two levels.
    Both levels stay within what the kernels' LDS arrays hold, together they give exactly 2^lg
    buckets, and a hop takes two levels only when one cannot hold it."""
    import shutil
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2110_08450_amd", "csrc")
    src = tmp_path / "levels.hip"
    src.write_text('#include <cstdio>\n#include "kernels_part.h"\n'
                   'int main() {\n'
                   '  std::printf("%d %d %d\\n", smfg_dev::kPartMaxLgB, smfg_dev::kPartMaxLg2, smfg_dev::kPartSplitLgB);\n'
                   '  for (int lg = 0; lg <= smfg_dev::kPartMaxLgB + smfg_dev::kPartMaxLg2; ++lg) {\n'
                   '    int a = -1, b = -1;\n    smfg_dev::part_levels(lg, a, b);\n    std::printf("%d %d %d\\n", lg, a, b);\n  }\n'
                   '  return 0;\n}\n')
    exe = tmp_path / "levels"
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-I", csrc, "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True, capture_output=True, timeout=300)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=60).stdout.split("\n")
    max_b, max_2, split_b = map(int, lines[0].split())
    rows = [tuple(map(int, l.split())) for l in lines[1:] if l.strip()]
    assert [r[0] for r in rows] == list(range(max_b + max_2 + 1))
    for lg, lg_b, lg_2 in rows:
        assert lg_b + lg_2 == lg and 0 <= lg_b <= max_b and 0 <= lg_2 <= max_2
        if lg <= max_b:
            assert lg_2 == 0
        else:
            assert lg_b >= min(split_b, max_b) and lg_2 > 0
