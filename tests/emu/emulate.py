"""CPU emulation of the HIP kernels (test infrastructure only).

The kernel sources of `paper_2410_21951_amd/csrc` are compiled for the host against a small
stand-in for the HIP runtime (`shim/hip/hip_runtime.h`, `emu_rt.cpp`): every GPU thread is an
OS thread, the blocks of a launch run one after another, wave collectives (shuffles, votes,
the bf16 MFMA) are rendezvous between the 64 lanes, and the "device" arena sits between
inaccessible guard pages.  The same C ABI is then driven through the ordinary Python binding, so
the kernels' index arithmetic and control flow can be checked against the oracle (and under
host sanitizers) without a GPU.  It says nothing about timing, caches or memory ordering across
workgroups: a persistent launch is emulated with a single workgroup.
"""
import ctypes as C
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2410_21951_amd", "csrc")
CXX = "/opt/rocm/llvm/bin/clang++"


def build(out_dir, extra_flags=()):
    """Translate the .hip sources for the host compiler and build libvadusa_emu.so in out_dir."""
    gen = os.path.join(out_dir, "gen")
    os.makedirs(gen, exist_ok=True)
    cpp = []
    for name in sorted(os.listdir(CSRC)):
        if not name.endswith((".hip", ".h")):
            continue
        text = open(os.path.join(CSRC, name)).read()
        # dynamic LDS, the one inline-asm wait, and the cooperative launch have host stand-ins
        text = text.replace("extern __shared__ uint4 smem[];", "uint4* smem = (uint4*)emu_dyn_lds;")
        text = text.replace("extern __shared__ float s_s[];", "float* s_s = (float*)emu_dyn_lds;")
        text = "\n".join(l for l in text.split("\n") if "s_waitcnt" not in l)
        text = re.sub(r"hipLaunchCooperativeKernel\(\(const void\*\)(\w+), (.*), st\);", r"emu_launch_coop(\1, \2);", text)
        dst = os.path.join(gen, name[:-4] + ".cpp" if name.endswith(".hip") else name)
        open(dst, "w").write(text)
        if dst.endswith(".cpp"):
            cpp.append(dst)
    out = os.path.join(out_dir, "libvadusa_emu.so")
    cmd = [CXX, "-std=c++17", "-g", "-O1", "-fPIC", "-shared", "-pthread", "-fno-omit-frame-pointer", *extra_flags,
           "-I" + os.path.join(HERE, "shim"), "-I" + os.path.join(ROOT, "include"), "-I" + gen,
           *cpp, os.path.join(HERE, "emu_rt.cpp"), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return out


def install(libpath, fill=0xAB):
    """Make paper_2410_21951_amd.Vadusa use the emulated library and a guarded host arena."""
    sys.path.insert(0, ROOT)
    import paper_2410_21951_amd.vadusa as V
    lib = V.load_library(libpath)
    lib.emu_alloc.restype = C.c_void_p
    lib.emu_alloc.argtypes = [C.c_size_t, C.c_int]
    V._lib = lib

    def init(self, model, max_batch=1, max_tree_nodes=64, ignore_eos=False, stream=None, prefill_chunk=0):
        self.lib = lib
        self.cfg = V.make_config(model, max_batch, max_tree_nodes, ignore_eos, prefill_chunk)
        msg = C.create_string_buffer(256)
        rc = lib.vadusa_config_check(C.byref(self.cfg), msg, 256)
        if rc:
            raise V.VadusaError(rc, msg.value.decode())
        nbytes = lib.vadusa_arena_bytes(C.byref(self.cfg))
        base = lib.emu_alloc(nbytes, fill)      # garbage-filled: nothing may rely on zeroed memory
        h = C.c_void_p()
        rc = lib.vadusa_create(C.byref(self.cfg), C.c_void_p(base), nbytes, None, C.byref(h))
        if rc:
            raise V.VadusaError(rc, "vadusa_create failed")
        self.h, self.batch, self.M = h, 0, 0
        self.Hh, self.V1 = self.cfg.n_draft_heads, self.cfg.speech_vocab + 1

    V.Vadusa.__init__ = init
