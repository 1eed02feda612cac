"""The shared library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2604_11554_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "relax_rollout.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rlx_\w+|rollout_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None
        assert callable(getattr(B, n))


def test_struct_layouts_match_header():
    # field order and C types as written in the header: 1 uint32, 11 int32, 2 float, 5 int32
    assert ctypes.sizeof(B.ModelConfig) == 4 * 19
    assert ctypes.sizeof(B.Weights) == 8 + 8 * 3 + 8 * 11
    assert B.rlx_last_error() == "" or isinstance(B.rlx_last_error(), str)


def test_host_side_validation_needs_no_gpu():
    # NULL / size-mismatch arguments are rejected on the host before any HIP call
    lib = B.lib()
    h = ctypes.c_void_p()
    cfg = B.ModelConfig()
    w = B.Weights()
    assert lib.rlx_model_create(ctypes.byref(cfg), ctypes.byref(w), ctypes.byref(h)) == B.RLX_EINVAL
    assert "struct_size" in B.rlx_last_error()
    assert lib.rlx_model_create(None, None, None) == B.RLX_EINVAL
    out = ctypes.c_size_t()
    assert lib.rlx_kv_pool_bytes(None, 4, ctypes.byref(out)) == B.RLX_EINVAL
    assert lib.rollout_decode_step(*([None] * 2), 0, None, 0, 0, None, None, None, 0, *([None] * 10)) == B.RLX_EINVAL


def test_build_refuses_scratch_memory_and_loops_left_rolled():
    """The build reads hipcc's resource remarks: a kernel with scratch memory, or a loop the compiler declined to
    unroll (accumulators indexed at run time then live in scratch), fails it."""
    from paper_2604_11554_amd import build
    ok = ("k.hip:5:1: remark: Function Name: _Z1av [-Rpass-analysis=kernel-resource-usage]\n"
          "k.hip:5:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n")
    assert build._resource_problems(ok) == []
    bad = ok + ("k.hip:9:1: remark: Function Name: _Z1bv [-Rpass-analysis=kernel-resource-usage]\n"
                "k.hip:9:1: remark:     ScratchSize [bytes/lane]: 576 [-Rpass-analysis=kernel-resource-usage]\n"
                "k.hip:12:3: warning: loop not unrolled: the optimizer was unable to perform the requested "
                "transformation [-Wpass-failed=transform-warning]\n")
    got = build._resource_problems(bad)
    assert len(got) == 2 and "_Z1bv uses 576 bytes" in got[0] and "loop not unrolled" in got[1]
