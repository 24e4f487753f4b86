"""Bench-only comparator (one graph operator per kernel, everything stashed).  Not part of
the library: only `bench.py --compare-unfused` and its test load it."""
import ctypes as C
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libgnnunfused.so")
SOURCES = ["unfused_gat.hip", "unfused_edgeconv_gmm.hip"]


def build(verbose=True):
    cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           *[os.path.join(HERE, f) for f in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    text = "\n".join(l for l in out.stdout.splitlines() if "packed-fp32-ops" not in l)
    if text.strip() and verbose:
        print(text)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed for the unfused comparator")
    return LIB


def load():
    if not os.path.exists(LIB):
        raise ImportError(f"{LIB} is missing: run __graft_entry__.build()")
    lib = C.CDLL(LIB)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.unfused_gat_graph_fwd.argtypes = [C.c_int32, i64, i32, i32, f32] + [vp] * 13 + [vp]
    lib.unfused_gat_graph_bwd.argtypes = [C.c_int32, i64, i32, i32, f32] + [vp] * 19 + [vp]
    lib.unfused_ec_u_sub_v.argtypes = [i64, i32] + [vp] * 4 + [vp]
    lib.unfused_ec_add_max.argtypes = [C.c_int32, i64, i32] + [vp] * 7 + [vp]
    lib.unfused_gmm_graph_fwd.argtypes = [C.c_int32, i64, i32, i32] + [vp] * 10 + [vp]
    lib.unfused_marker.argtypes = [i32, vp]
    for f in (lib.unfused_ec_u_sub_v, lib.unfused_ec_add_max, lib.unfused_gmm_graph_fwd, lib.unfused_marker):
        f.restype = C.c_int
    lib.unfused_gat_graph_fwd.restype = C.c_int
    lib.unfused_gat_graph_bwd.restype = C.c_int
    return lib
