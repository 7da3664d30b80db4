"""The C ABI used from plain C: include/loco.h compiles as strict C99 and as C++11 (CPU), and
a C99 program with no Python, C++ or torch in it drives the library on the GPU and matches the
oracle byte for byte (tests/c_abi_client.c)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")
CLIENT_SRC = os.path.join(ROOT, "tests", "c_abi_client.c")
CLIENT_BIN = os.path.join(ROOT, "tests", "c_abi_client.bin")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_client(out=CLIENT_BIN):
    """gcc, C99: the client, the oracle's C file, libloco.so and the HIP runtime."""
    pkg = os.path.join(ROOT, "paper_2407_04480_amd")
    cmd = ["gcc", "-std=c99", "-O1", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-I", INCLUDE,
           "-I", os.path.join(ROCM, "include"), "-o", out, CLIENT_SRC, os.path.join(ROOT, "oracle", "loco_ref.c"),
           "-L", pkg, "-lloco", "-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2407_04480_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return out


def test_header_is_strict_c99_and_cxx11(tmp_path):
    src = tmp_path / "use_header.c"
    src.write_text('#include "loco.h"\nint main(void) { return (int)loco_code_bytes(8, 4) - 4; }\n')
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "c++")):
        res = subprocess.run([cc, std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", INCLUDE, "-x", lang,
                              "-c", str(src), "-o", str(tmp_path / f"out_{lang}.o")], capture_output=True, text=True)
        assert res.returncode == 0, f"{cc} {std}: {res.stderr}"


def test_c_client_builds(tmp_path):
    """Links on a box without a GPU too (nothing is run)."""
    from paper_2407_04480_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2407_04480_amd import build
        build.build()
    build_client(str(tmp_path / "client.bin"))


@pytest.mark.gpu
def test_c_client_matches_the_oracle():
    if not os.path.exists(CLIENT_BIN):
        build_client()
    res = subprocess.run([CLIENT_BIN], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, (res.returncode, res.stdout[-2000:], res.stderr[-2000:])
    assert res.stdout.strip().endswith("c client ok"), res.stdout[-500:]
