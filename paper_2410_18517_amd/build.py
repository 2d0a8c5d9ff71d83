"""Build libkvs.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvs.so")
SOURCES = ["kvs_host.cpp", "kvs_store_ops.hip", "kvs_attention.hip", "kvs_decode.hip", "kvs_distance.hip", "kvs_similarity.hip", "kvs_projection.hip",
           "kvs_static.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "kvs_internal.h"), os.path.join(CSRC, "kvs_device.h"), os.path.join(CSRC, "kvs_attn_tiles.h"), os.path.join(CSRC, "kvs_flat_plan.h"),
                        os.path.join(HERE, "..", "include", "kvs.h"), os.path.join(HERE, "..", "include", "kvs_testing.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    objs = []
    for src in sources():
        obj = os.path.splitext(src)[0] + ".o"
        cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stderr)
        if verbose and r.stderr:
            print(r.stderr)
        objs.append(obj)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
