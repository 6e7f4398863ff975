"""Build libmi355attn.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2512_18134_amd.build

Two libraries come out of the same sources: libmi355attn.so (the product) and
libmi355attn_debug.so (-DATTN_DEBUG_ENTRY_POINTS: the same code plus test-only entry
points that let a test pick the kernel, e.g. the program-order reference of the
schedule-equivalence tests).  Nothing in the package loads the debug library.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "attn_fwd.hip"), os.path.join(HERE, "csrc", "attn_bwd.hip")]
LIB_PATH = os.path.join(HERE, "libmi355attn.so")
DEBUG_LIB_PATH = os.path.join(HERE, "libmi355attn_debug.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU ops are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def _run_generator(cmd, verbose):
    """The generators take everything from their command line: run them with an empty environment so
    that nothing set in the caller's shell can change what is built."""
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, env={})


def generate_sources(verbose=False, out_dir=None):
    """Run the loop generators: csrc/generated/*.inc (or out_dir)."""
    gen = os.path.join(HERE, "csrc", "gen_attn_loop.py")
    out_dir = out_dir or os.path.join(HERE, "csrc", "generated")
    os.makedirs(out_dir, exist_ok=True)
    for name, dtype in (("d64", "bf16"), ("d64", "f16"), ("d64_w4", "bf16"), ("d128", "bf16"), ("d128", "f16"),
                        ("d128a", "bf16"), ("d128a", "f16"), ("d256a", "bf16"), ("d256a", "f16")):
        out = os.path.join(out_dir, "attn_loop_%s%s.inc" % (name, "" if dtype == "bf16" else "_" + dtype))
        _run_generator([sys.executable, gen, name, out, dtype], verbose)
    gen3 = os.path.join(HERE, "csrc", "gen_attn_bwd_loop.py")
    for kind, d, dtype in (("kv", 128, "bf16"), ("q", 128, "bf16"), ("kv", 128, "f16"), ("q", 128, "f16"),
                           ("kv", 64, "bf16"), ("q", 64, "bf16"), ("kv", 64, "f16"), ("q", 64, "f16")):
        out = os.path.join(out_dir, "attn_bwd_loop_%s_d%d%s.inc" % (kind, d, "" if dtype == "bf16" else "_" + dtype))
        _run_generator([sys.executable, gen3, kind, str(d), out, dtype], verbose)


def _compile(lib_path, extra, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib_path + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + extra + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, lib_path)
    return lib_path


def build_library(verbose=False, debug=True):
    """Generate the scheduled loops, then compile every HIP source into LIB_PATH (and, with the test-only
    entry points, into DEBUG_LIB_PATH).  Raises on failure."""
    generate_sources(verbose)
    _compile(LIB_PATH, [], verbose)
    if debug:
        _compile(DEBUG_LIB_PATH, ["-DATTN_DEBUG_ENTRY_POINTS"], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
