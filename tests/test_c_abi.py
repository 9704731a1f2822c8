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
