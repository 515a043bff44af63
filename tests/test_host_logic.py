"""Host-side checks of device logic that can run without a GPU: the product's own NF4 index
schemes (bucket table, binary search) against a plain threshold count, compiled for the host."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2305_14314_amd", "csrc")


def test_nf4_index_schemes_agree(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "nf4_index_check")
    src = os.path.join(ROOT, "tests", "host_checks", "nf4_index_check.cpp")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-ffp-contract=off", "-x", "hip", "-I", CSRC,
                    src, "-o", exe], check=True, capture_output=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True, timeout=300).stdout
    assert out.startswith("OK "), out
    assert int(out.split()[1]) > 30_000_000


def test_list_partition_tiles_the_work(tmp_path):
    """The range formula of the few-token list kernels (evaluated alike by the size queries, the launcher and the
    kernels): exact tiling, inverse map, contributor counts against brute force, for thousands of shape lists."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2305_14314_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    exe = str(tmp_path / "list_partition_check")
    src = os.path.join(ROOT, "tests", "host_checks", "list_partition_check.cpp")
    pkg = os.path.dirname(binding.LIB_PATH)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-x", "hip", "-I", CSRC, src, "-o", exe,
                    "-L", pkg, "-lqlora_hip", "-Wl,-rpath," + pkg], check=True, capture_output=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True, timeout=300).stdout
    assert out.startswith("OK "), out
    assert int(out.split()[1]) > 2000


def test_fused_gemm_row_loads_stay_inside_the_weight(tmp_path):
    """The fused backward GEMM loads a weight row's codes and block constant per K-step: every load its schedule asks
    for lies inside the buffers, for ragged N, K shorter and longer than the prefetch ring, with and without an adapter."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2305_14314_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    exe = str(tmp_path / "fused_gemm_index_check")
    src = os.path.join(ROOT, "tests", "host_checks", "fused_gemm_index_check.cpp")
    pkg = os.path.dirname(binding.LIB_PATH)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-x", "hip", "-I", CSRC, src, "-o", exe,
                    "-L", pkg, "-lqlora_hip", "-Wl,-rpath," + pkg], check=True, capture_output=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True, timeout=300).stdout
    assert out.startswith("OK "), out
    assert int(out.split()[1]) > 500


def test_fused_gemm_reads_no_register_in_flight(tmp_path):
    """The fused GEMM kernel's hand-placed asynchronous loads and lookups: in the compiled kernel no instruction touches
    a register between its asynchronous write and the wait that covers it (the compiler is free to schedule or copy
    such registers early: this checks what it actually did).  With the main loop's vmcnt waits deleted from the same
    text the check must fail, which shows that it sees the loads."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    import importlib.util
    spec = importlib.util.spec_from_file_location("async_register_check",
                                                  os.path.join(ROOT, "tests", "host_checks", "async_register_check.py"))
    chk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(chk)
    from paper_2305_14314_amd import build
    asm = str(tmp_path / "gemm.s")
    subprocess.run([hipcc, *build.FLAGS, "-x", "hip", "--cuda-device-only",
                    "-S", os.path.join(CSRC, "gemm.hip"), "-o", asm], check=True, capture_output=True)
    text = open(asm).read()
    bad, seen = chk.check(text)
    assert seen >= 5 and not bad, (seen, bad[:5])
    for plain in ("gemm_nt_kernelILi256ELi4ELb0EE", "gemm_nt_kernelILi128ELi4ELb0EE"):   # their fragment reads alike
        bad, seen = chk.check(text, plain)
        assert seen >= 5 and not bad, (plain, seen, bad[:5])
    broken = text.replace("s_waitcnt vmcnt(8)", "s_nop 0")
    assert broken != text
    bad, _ = chk.check(broken)
    assert bad
