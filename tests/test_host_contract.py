"""No GPU: the header is valid C and C++, and bench.py refuses more than one GPU before touching any."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_compiles_as_c_and_as_cxx(tmp_path):
    hdr = os.path.join(ROOT, "include", "agg.h")
    for lang, std, cc in (("c", "-std=c99", "gcc"), ("c++", "-std=c++11", "g++")):
        src = tmp_path / ("use." + ("c" if lang == "c" else "cc"))
        src.write_text('#include "agg.h"\nint use(void) { agg_tune_result r; r.tile_config = AGG_OK; return r.tile_config + AGG_SIGNAL_STRIDE; }\n')
        r = subprocess.run([cc, "-x", lang, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                            "-I", os.path.dirname(hdr), str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
