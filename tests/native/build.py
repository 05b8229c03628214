"""Build tests/native/zpp_client (plain C, gcc) against the HIP library and the oracle.

Test infrastructure: links both, so it lives with the tests and not in the package.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "zpp_client.c")
OUT = os.path.join(HERE, "zpp_client")
SAN_OUT = os.path.join(HERE, "zpp_client_san")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


SANITIZE = ["-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
            "-static-libasan"]


def build(force=True, sanitize=False, out=None):
    """Compile the client; returns its path.  With force=False an up-to-date binary is kept.
    sanitize: instrument the client's own (host) code with ASan + UBSan and write it to `out`."""
    OUT = out or (SAN_OUT if sanitize else globals()["OUT"])
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    from paper_2306_10209_amd import build as lib_build
    oracle_so = oracle_build.build(force=False)
    lib_so = lib_build.LIB if os.path.exists(lib_build.LIB) else lib_build.build()
    deps = [SRC, os.path.join(ROOT, "include", "zpp.h"), oracle_so, lib_so]
    if not force and os.path.exists(OUT) and all(os.path.getmtime(OUT) >= os.path.getmtime(d) for d in deps):
        return OUT
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-Werror", *(SANITIZE if sanitize else []),
           f"-I{ROCM}/include", f"-I{ROOT}/include", SRC, "-o", OUT,
           f"-L{os.path.dirname(lib_so)}", "-lzpp_gfx950", f"-L{os.path.dirname(oracle_so)}", "-loracle",
           f"-L{ROCM}/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2306_10209_amd/lib", "-Wl,-rpath,$ORIGIN/../../oracle",
           f"-Wl,-rpath,{ROCM}/lib"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build())
