"""CPU-side checks of the boundary: the shared library loads and exports every entry
point the header declares (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


HEADERS = ["swarm.h", "swarm_bench.h"]


def declared_symbols(headers=HEADERS):
    names = set()
    for header in headers:
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(swarm_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_calls_of_the_interaction():
    names = declared_symbols(["swarm.h"])
    for must in ["swarm_init", "swarm_local_steps", "swarm_gossip_round", "swarm_quantize", "swarm_dequantize",
                 "swarm_read_models", "swarm_interact", "swarm_run_sequential", "swarm_sample_matching", "swarm_potential"]:
        assert must in names
    # the measurement aids are kept out of the product header
    for aid in ["swarm_stream_copy", "swarm_stream_mix", "swarm_timing_reset", "swarm_kernel_times"]:
        assert aid not in names and aid in declared_symbols(["swarm_bench.h"])


def test_library_loads_and_exports_every_declared_symbol():
    import paper_1910_12308_amd as swarm
    if not os.path.exists(swarm.LIB_PATH):
        pytest.fail("libswarm.so is not built: run __graft_entry__.build()")
    lib = ctypes.CDLL(swarm.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} declared in swarm.h but not exported"
    assert sorted(swarm.EXPORTS) == declared_symbols()


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    import paper_1910_12308_amd as swarm
    monkeypatch.setattr(swarm, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(ImportError):
        swarm.load_library()


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1910_12308_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".hpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f


def test_header_is_plain_c_and_the_config_struct_matches_the_binding(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, and the binding's ctypes mirror of
    swarm_config has the size and field offsets the C compiler gives."""
    import ctypes
    import shutil
    import subprocess
    import paper_1910_12308_amd as swarm
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    fields = [name for name, _ in swarm._Config._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "swarm.h"\n#include "swarm_bench.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(swarm_config));\n'
                   + "".join(f'  printf("%zu\\n", offsetof(swarm_config, {f}));\n' for f in fields)
                   + "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(swarm._Config)
    assert out[1:] == [getattr(swarm._Config, f).offset for f in fields]
