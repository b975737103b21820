"""bench.py's MFMA issue-rate probe: builds bench_probe.hip into libbench_probe.so beside this
file and calls it.  A measurement aid, not part of the KV-cache library or its C ABI."""
import ctypes as C
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bench_probe.hip")
LIB = os.path.join(HERE, "libbench_probe.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
_lib = None


def build() -> str:
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", LIB + ".tmp", SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def lib():
    """Load the built probe; build it only if nothing is built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = C.CDLL(LIB)
        _lib.bench_mfma_probe_operand_bytes.restype = C.c_size_t
        _lib.bench_mfma_probe.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                          C.POINTER(C.c_int64), C.c_void_p]
    return _lib


def operand_bytes() -> int:
    return int(lib().bench_mfma_probe_operand_bytes())


def mfma_probe(dtype: int, operands, blocks: int, iters: int, sink, stream: int) -> int:
    """Launches the probe on torch tensors; returns the floating-point operations issued."""
    flops = C.c_int64(0)
    rc = lib().bench_mfma_probe(dtype, operands.data_ptr(), blocks, iters, sink.data_ptr(),
                                C.byref(flops), stream)
    if rc != 0:
        raise RuntimeError(f"bench_mfma_probe failed ({rc})")
    return int(flops.value)
