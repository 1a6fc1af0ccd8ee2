"""Builds and loads the lock-step CPU emulation of the kernels (tests/emu): the same device source
and host planner as the GPU library, with the wavefront primitives replaced by fibers.  Used only by
the host-side checks of the kernel logic; the product binding never loads it."""
import fcntl
import os
import subprocess

from paper_1812_01776_amd import estimator as binding

_HERE = os.path.dirname(os.path.abspath(__file__))
_EMU = os.path.join(_HERE, "emu")
_CSRC = os.path.join(os.path.dirname(_HERE), "paper_1812_01776_amd", "csrc")
_LIB = os.path.join(_EMU, "libestimator_emu.so")


def build():
    srcs = [os.path.join(_EMU, "backend_emu.cpp"), os.path.join(_CSRC, "est_host.cpp"), os.path.join(_CSRC, "est_planner.cpp")]
    deps = srcs + [os.path.join(_EMU, "wave_emu.h")] + [os.path.join(_CSRC, f) for f in os.listdir(_CSRC)] + \
        [os.path.join(os.path.dirname(_HERE), "include", "estimator.h")]
    def fresh():
        return os.path.exists(_LIB) and all(os.path.getmtime(_LIB) >= os.path.getmtime(d) for d in deps)

    if fresh():
        return _LIB
    # one builder at a time (test workers start together), and the library appears under its name only when complete
    with open(_LIB + ".lock", "w") as lock:
        fcntl.flock(lock, fcntl.LOCK_EX)
        if not fresh():
            tmp = _LIB + ".tmp%d" % os.getpid()
            subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-DEST_EMU_CHECKS", "-Wall", "-Wno-unused-parameter",
                                   "-o", tmp] + srcs)
            os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = binding.load_library(build())
    return _lib


def make(w):
    return binding.Estimator(w.parents, w.lat_us, w.cost_uusd_hr, _lib=lib())
