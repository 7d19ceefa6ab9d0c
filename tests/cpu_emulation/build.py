"""Builds the CPU emulation of libtt_emb: the unchanged HIP sources of the library compiled for
the host against a stand-in for the HIP runtime (hip/hip_runtime.h, emu_runtime.cpp) that runs one
workgroup at a time, one OS thread per wavefront and one fiber per lane.  Test infrastructure only:
nothing in the product path loads what is built here.

  build_shared(out_dir)            -> libtt_emb_emu.so, driven through ctypes by the CPU tests
  build_harness(out_dir, sanitize) -> harness executable under "address" (+UBSan), "memory" or "thread"

Two textual changes are made to the copies that are compiled: `extern __shared__ float x[];`
becomes a pointer to the emulated dynamic LDS, and the switch that keeps the batched entry points
off is turned on, so that their host logic and kernels are exercised here although they are not
run on the GPU.
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2507_14668_amd", "csrc")
CLANG = os.environ.get("TT_EMU_CXX", "/opt/rocm/llvm/bin/clang++")
UNITS = ("tt_api", "tt_reorder", "tt_forward", "tt_forward_mfma", "tt_forward_sample", "tt_bf16", "tt_index_graph", "tt_fuse", "tt_backward",
         "tt_backward_mfma")


def available() -> bool:
    return os.path.exists(CLANG)


def _generate(gen: str) -> list:
    shutil.rmtree(gen, ignore_errors=True)
    os.makedirs(gen)
    out = []
    for u in UNITS:
        text = open(os.path.join(CSRC, u + ".hip")).read()
        text = re.sub(r"extern __shared__ float (\w+)\[\];", r"float *\1 = (float *)emu::dyn_lds();", text)
        text = text.replace("kBatchedCallsEnabled = false", "kBatchedCallsEnabled = true")
        # the host copies of the table descriptors are for the host only: kernels get the uploaded array
        text = text.replace("  if (!host) return TT_ERR_INVALID_ARG;\n",
                            "  if (!host) return TT_ERR_INVALID_ARG;\n  emu::host_only(host, (size_t)T * sizeof(TTDev));\n")
        text = text.replace("  free(host);\n  return st;", "  emu::host_only_release(host);\n  free(host);\n  return st;")
        path = os.path.join(gen, u + ".cpp")
        open(path, "w").write(text)
        out.append(path)
    shutil.copy(os.path.join(CSRC, "tt_internal.h"), gen)
    return out


def _compile(sources, flags, out_dir, tag):
    base = [CLANG, "-std=c++17", "-g", "-D__HIPCC__", "-I" + HERE, "-I" + os.path.join(out_dir, "gen_" + tag),
            "-I" + os.path.join(ROOT, "include"), "-pthread", "-Wno-unused-value"] + flags

    def one(src):
        obj = os.path.join(out_dir, "gen_" + tag, os.path.basename(src).rsplit(".", 1)[0] + ".o")
        res = subprocess.run(base + ["-c", src, "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("compiling %s failed:\n%s" % (src, res.stderr[-4000:]))
        return obj

    with ThreadPoolExecutor(max_workers=8) as pool:
        return list(pool.map(one, sources)), base


def build_shared(out_dir: str) -> str:
    os.makedirs(out_dir, exist_ok=True)
    srcs = _generate(os.path.join(out_dir, "gen_so")) + [os.path.join(HERE, "emu_runtime.cpp")]
    objs, base = _compile(srcs, ["-O2", "-fPIC"], out_dir, "so")
    lib = os.path.join(out_dir, "libtt_emb_emu.so")
    subprocess.run(base + ["-O2", "-fPIC", "-shared"] + objs + ["-o", lib], check=True)
    return lib


SANITIZERS = {
    "address": ["-fsanitize=address,undefined", "-fno-sanitize=vptr", "-fno-omit-frame-pointer"],
    "memory": ["-fsanitize=memory", "-fsanitize-memory-track-origins=2", "-DEMU_MSAN"],
    "thread": ["-fsanitize=thread"],
}


def build_harness(out_dir: str, sanitize: str = "address") -> str:
    os.makedirs(out_dir, exist_ok=True)
    tag = "h_" + sanitize
    srcs = _generate(os.path.join(out_dir, "gen_" + tag)) + [os.path.join(HERE, "emu_runtime.cpp"),
                                                             os.path.join(HERE, "harness.cpp")]
    flags = ["-O1"] + SANITIZERS[sanitize]
    objs, base = _compile(srcs, flags, out_dir, tag)
    exe = os.path.join(out_dir, "harness_" + sanitize)
    subprocess.run(base + flags + objs + ["-o", exe], check=True)
    return exe


if __name__ == "__main__":
    import sys
    out = os.path.join(HERE, "_build")
    print(build_shared(out))
    for s in sys.argv[1:] or ["address"]:
        print(build_harness(out, s))
