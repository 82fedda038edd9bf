"""Hardware yardsticks used by `bench.py --hardware-rates` only (random single-word operations,
the workgroup-to-XCD map).  Built in-tree by build(); needs a GPU to run."""
import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "probes.hip")
_SO = os.path.join(_HERE, "libbench_probes.so")
_lib = None


def build(force=False):
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["hipcc", "-O3", "--offload-arch=gfx950", "-shared", "-fPIC",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-o", _SO, _SRC])
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise RuntimeError("bench_probes library not built: run __graft_entry__.build()")
        _lib = C.CDLL(_SO)
        _lib.bp_random_ops.restype = C.c_int
        _lib.bp_random_ops.argtypes = [C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_uint64, C.c_void_p]
        _lib.bp_xcd_map.restype = C.c_int
        _lib.bp_xcd_map.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
    return _lib


def random_ops(mode, table, n_ops, salt=0):
    """n_ops random single-word operations over an int64 device tensor.
    mode 0 atomicMin u64, 1 atomicMin u32, 2 store 8 B, 3 load 8 B, 4 atomicMin u64 at workgroup
    scope, 5 / 6 atomicMin u64 at device / workgroup scope with each XCD confined to its own eighth
    of the table, 7 load 8 B confined likewise."""
    import torch
    rc = _load().bp_random_ops(mode, table.data_ptr(), table.numel(), n_ops, salt,
                               torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("bp_random_ops failed: hip error %d" % rc)


def xcd_map(n_blocks):
    """int32 tensor: the XCD that ran each of n_blocks workgroups of one launch."""
    import torch
    out = torch.zeros(n_blocks, dtype=torch.int32, device="cuda")
    rc = _load().bp_xcd_map(out.data_ptr(), n_blocks, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("bp_xcd_map failed: hip error %d" % rc)
    return out
