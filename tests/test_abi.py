"""The C-ABI library loads, exports every entry point include/smoe.h declares,
and the Python binding's struct layouts match the compiler's."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "smoe.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\bint\s+(moe_\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    import paper_2508_18983_amd as M
    lib = M.load_library()
    names = _declared()
    assert {"moe_cache_init", "moe_decode_layer", "moe_cache_stats"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in smoe.h but not exported"
        assert callable(getattr(M, n)), f"binding lacks {n}"
    assert M.moe_last_hip_error() == 0


def test_header_is_plain_c_and_struct_layouts_match_binding(tmp_path):
    import paper_2508_18983_amd as M
    prog = tmp_path / "sizes.c"
    prog.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "smoe.h"\n'
                    'int main(void){printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(moe_cfg_t),'
                    'sizeof(moe_buffers_t), sizeof(moe_trace_t), sizeof(moe_stats_t), sizeof(moe_profile_t),'
                    'offsetof(moe_cfg_t, alpha), offsetof(moe_trace_t, n_fetched), sizeof(moe_prefetch_info_t),'
                    'offsetof(moe_cfg_t, cpu_cost_us), offsetof(moe_stats_t, cpu_computed), offsetof(moe_stats_t, prefetches),'
                    'offsetof(moe_trace_t, on_cpu), offsetof(moe_trace_t, inflight_mask) + 1000 * offsetof(moe_prefetch_info_t, bytes_withdrawn));return 0;}\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(prog), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    got = [int(v) for v in out]
    want = [ctypes.sizeof(M.MoeCfg), ctypes.sizeof(M.MoeBuffers), ctypes.sizeof(M.MoeTrace),
            ctypes.sizeof(M.MoeStats), ctypes.sizeof(M.MoeProfile), M.MoeCfg.alpha.offset,
            M.MoeTrace.n_fetched.offset, ctypes.sizeof(M.MoePrefetchInfo), M.MoeCfg.cpu_cost_us.offset,
            M.MoeStats.cpu_computed.offset, M.MoeStats.prefetches.offset, M.MoeTrace.on_cpu.offset,
            M.MoeTrace.inflight_mask.offset + 1000 * M.MoePrefetchInfo.bytes_withdrawn.offset]
    assert got == want


def test_product_path_does_not_import_the_oracle():
    code = ("import sys; import paper_2508_18983_amd, paper_2508_18983_amd.session, smoe_inputs; "
            "bad=[m for m in sys.modules if m.split('.')[0]=='oracle']; assert not bad, bad")
    subprocess.run([sys.executable, "-c", code], check=True, cwd=ROOT)
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2508_18983_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().lower(), f


def test_session_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from smoe_inputs import SHAPES, make_workload
    from paper_2508_18983_amd.session import session_from_workload
    with pytest.raises(RuntimeError):
        session_from_workload(make_workload(SHAPES["c1"].with_(tokens=1)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 2 and "one-GPU" in r.stderr and r.stdout.strip() == ""
