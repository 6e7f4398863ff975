"""Build libmi355attn.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2512_18134_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "attn_fwd.hip"), os.path.join(HERE, "csrc", "attn_bwd.hip")]
LIB_PATH = os.environ.get("ATTN_FWD_LIB_OUT", os.path.join(HERE, "libmi355attn.so"))  # override: experiments only

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU ops are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def generate_sources(verbose=False):
    """Run the loop generator: csrc/generated/attn_loop_d{64,128}.inc."""
    gen = os.path.join(HERE, "csrc", "gen_attn_loop.py")
    out_dir = os.path.join(HERE, "csrc", "generated")
    os.makedirs(out_dir, exist_ok=True)
    for d, dtype, nw in ((64, "bf16", 8), (128, "bf16", 8), (64, "f16", 8), (128, "f16", 8), (64, "bf16", 4)):
        out = os.path.join(out_dir, "attn_loop_d%d%s%s.inc" % (d, "" if dtype == "bf16" else "_" + dtype,
                                                               "" if nw == 8 else "_w%d" % nw))
        cmd = [sys.executable, gen, str(d), out, dtype, str(nw)]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    gen2 = os.path.join(HERE, "csrc", "gen_attn_loop2.py")
    for name, dtype in (("d128a", "bf16"), ("d256a", "bf16"), ("d256a", "f16")):
        out = os.path.join(out_dir, "attn_loop_%s%s.inc" % (name, "" if dtype == "bf16" else "_" + dtype))
        cmd = [sys.executable, gen2, name, out, dtype]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    gen3 = os.path.join(HERE, "csrc", "gen_attn_bwd_loop.py")
    for kind, d, dtype in (("kv", 128, "bf16"), ("q", 128, "bf16"), ("kv", 128, "f16"), ("q", 128, "f16"),
                           ("kv", 64, "bf16"), ("q", 64, "bf16"), ("kv", 64, "f16"), ("q", 64, "f16")):
        out = os.path.join(out_dir, "attn_bwd_loop_%s_d%d%s.inc" % (kind, d, "" if dtype == "bf16" else "_" + dtype))
        cmd = [sys.executable, gen3, kind, str(d), out, dtype]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)


def build_library(verbose=False):
    """Generate the scheduled loops, then compile every HIP source into LIB_PATH.  Raises on failure."""
    generate_sources(verbose)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", tmp] + SOURCES
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
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
