"""include/liver.h is valid, self-contained C99, and the library can be driven from plain C."""
import os
import subprocess

import paper_2605_22014_amd as lv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_is_c99_and_library_links_from_c(tmp_path):
    exe = str(tmp_path / "c_abi_smoke")
    libdir = os.path.dirname(lv.library_path())
    torch_lib = os.path.join(os.path.dirname(__import__("torch").__file__), "lib")
    build = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I" + os.path.join(ROOT, "include"),
                            os.path.join(ROOT, "tests", "c_abi_smoke.c"), "-o", exe, "-L" + libdir, "-l:libliver.so",
                            "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, LD_LIBRARY_PATH=torch_lib + ":/opt/rocm/lib:" + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.stdout, run.stderr[-2000:])
    assert "chunks 35 descriptors 175 stream_bytes 35766272" in run.stdout, run.stdout
    assert "bad chunk_bytes -> -1" in run.stdout


def test_library_exports_every_symbol_the_headers_declare():
    import ctypes
    import glob
    import re
    lib = ctypes.CDLL(lv.library_path())
    declared = set()
    for path in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)        # declarations only, no comments
        declared |= set(re.findall(r"\b(liver_[a-z_0-9]+)\s*\(", text))
    assert {"liver_plan_create", "liver_pack", "liver_unpack", "liver_reshard", "liver_plan_destroy"} <= declared
    missing = [name for name in sorted(declared) if not hasattr(lib, name)]
    assert not missing, missing


def test_debug_entry_points_are_not_in_the_product_header():
    text = open(os.path.join(ROOT, "include", "liver.h")).read()
    assert "liver_debug_" not in text
    assert "liver_debug_emulate_host" in open(os.path.join(ROOT, "include", "liver_debug.h")).read()


def test_strerror_appends_the_detail_only_to_the_code_that_failed():
    spec = lv.ModelSpec(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=4, ffn=128, vocab=64)
    try:
        lv.liver_plan_create(spec, lv.Layout(tp=3, pp=1, dp=1), lv.Layout(tp=1, pp=1, dp=1), 1 << 20)
        raise AssertionError("tp=3 does not divide 4 heads: must be refused")
    except lv.LiverError as e:
        assert e.code == -2 and ":" in str(e).split("liver error -2: ", 1)[1]     # base text + detail
    assert lv.liver_strerror(-2).startswith("unsupported configuration: ")
    assert lv.liver_strerror(-1) == "invalid argument"                             # another code: no stale detail
    assert lv.liver_strerror(0) == "ok"


def test_static_staging_entry_refuses_on_the_host_what_it_cannot_run():
    """liver_reshard_static (for callers that cannot allocate): size limit and missing device are argument errors."""
    assert lv.liver_static_staging_bytes() == 64 << 20
    spec = lv.ModelSpec(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=4, ffn=128, vocab=64)
    lay = lv.Layout(tp=1, pp=1, dp=1)
    big = lv.liver_plan_create(spec, lv.Layout(tp=2, pp=1, dp=1), lay, (64 << 20) + 256)
    try:
        lv.liver_reshard_static(big, {}, {}, stream=0)
        raise AssertionError("a chunk beyond the static array must be refused")
    except lv.LiverError as e:
        assert e.code == -1 and "exceeds the library's static staging array" in str(e) and "67108864" in str(e)
    import torch
    if not torch.cuda.is_available():
        small = lv.liver_plan_create(spec, lv.Layout(tp=2, pp=1, dp=1), lay, 4096)
        try:
            lv.liver_reshard_static(small, {}, {}, stream=0)
            raise AssertionError("a host-only plan cannot run")
        except lv.LiverError as e:
            assert e.code == -5
