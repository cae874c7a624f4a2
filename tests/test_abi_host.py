"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and validates configurations."""
import os
import re

import pytest

from paper_2504_15364_amd import binding as kd

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "keydiff.h")


def test_library_exports_every_declared_symbol():
    lib = kd.load_library()
    text = open(HEADER).read()
    declared = set(re.findall(r"KEYDIFF_API[^;(]*?\b(keydiff_\w+)\s*\(", text))
    assert declared == set(kd.EXPORTS) and len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.keydiff_version() == 1


def test_workspace_sizes():
    cfg = kd.KeyDiffConfig(1, 32, 8, 128, 8192, 128)
    k, v, meta, scratch = kd.workspace_bytes(cfg)
    assert k == v == 8 * (8192 + 128) * 128 * 2
    assert meta >= 8 * (8192 + 128) * 4
    assert scratch > 8 * (8192 + 128) * 4


@pytest.mark.parametrize("kw,code", [
    (dict(n_q_heads=5), kd.ESHAPE),            # not a multiple of the KV heads
    (dict(head_dim=96), kd.ESHAPE),
    (dict(budget_N=0), kd.ESHAPE),
    (dict(budget_N=40000), kd.ESHAPE),
    (dict(anchor_mode=7), kd.EINVAL),
    (dict(layout=9), kd.EINVAL),
    (dict(window_W=256), kd.ESHAPE),           # the window must leave room in the budget
])
def test_bad_configs_are_rejected_with_a_message(kw, code):
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, budget_N=256, block_B=32)
    base.update(kw)
    with pytest.raises(kd.KeyDiffError) as e:
        kd.workspace_bytes(kd.KeyDiffConfig(**base))
    assert e.value.code == code and len(str(e.value)) > 20


def test_null_handles_are_rejected_before_anything_is_enqueued():
    # argument checks precede every launch: with no GPU in the process these calls still return errors
    lib = kd.load_library()
    assert lib.keydiff_finish(None, None) == kd.EINVAL
    assert lib.keydiff_prefill_block_deferred(None, None, None, None, 1, 0, None, None, None) == kd.EINVAL
    assert lib.keydiff_prefill_block(None, None, None, None, 1, 0, None, None, None) == kd.EINVAL
    assert b"null" in lib.keydiff_last_error()
    import ctypes as C
    none4 = (C.c_void_p * 4)()
    assert lib.keydiff_prefill_block_layers(None, 4, none4, none4, none4, 1, 0, none4, None) == kd.EINVAL
    assert lib.keydiff_prefill_block_layers(none4, 0, none4, none4, none4, 1, 0, none4, None) == kd.ESHAPE
    assert lib.keydiff_prefill_block_layers(none4, 4, none4, none4, none4, 1, 0, none4, None) == kd.EINVAL
    assert b"layer 0" in lib.keydiff_last_error()


def test_static_scratch_array_is_visible_to_the_runtime(tmp_path):
    # keydiff_prefill_block_static reaches its device array through hipGetSymbolAddress, which aborts
    # the process when the code object holds the array as a local symbol: check the built object
    import shutil
    import subprocess
    tools = "/opt/rocm/lib/llvm/bin"
    obj = os.path.join(os.path.dirname(kd.LIB_PATH), "csrc", "keydiff_abi.o")
    if not (os.path.exists(obj) and os.path.exists(f"{tools}/llvm-objdump") and os.path.exists(f"{tools}/llvm-readelf")):
        pytest.skip("needs the built object and the LLVM binary tools")
    work = tmp_path / "keydiff_abi.o"
    shutil.copy(obj, work)
    subprocess.run([f"{tools}/llvm-objdump", "--offloading", str(work)], check=True, capture_output=True, cwd=tmp_path)
    device = [p for p in tmp_path.iterdir() if "gfx950" in p.name]
    assert device, "no gfx950 code object in keydiff_abi.o"
    syms = subprocess.run([f"{tools}/llvm-readelf", "--dyn-syms", "-W", str(device[0])], check=True,
                          capture_output=True, text=True).stdout
    rows = [l.split() for l in syms.splitlines() if l.strip().endswith("scratch")]
    assert rows and all(r[4] == "GLOBAL" and int(r[2]) == 40 << 20 for r in rows), syms


def test_wrapper_refuses_tensors_smaller_than_the_configuration():
    """The C ABI takes bare pointers, so the wrapper checks every tensor's shape against the cache's
    configuration before a call: a tensor of a smaller batch or head count would be read past its end."""
    import torch

    from paper_2504_15364_amd.binding import check_block_shapes, check_load_shapes, check_rope_tables

    cfg = kd.KeyDiffConfig(2, 8, 2, 64, 256, 32)
    q = torch.zeros((2, 8, 32, 64), dtype=torch.bfloat16)
    k = torch.zeros((2, 2, 32, 64), dtype=torch.bfloat16)
    assert check_block_shapes(cfg, q, k, k, out=q) == 32
    assert check_block_shapes(cfg, q[:, :, :5].contiguous(), k[:, :, :5].contiguous(), k[:, :, :5].contiguous()) == 5
    with pytest.raises(ValueError, match="q has shape"):
        check_block_shapes(cfg, q[:1], k, k)                      # one sequence instead of two
    with pytest.raises(ValueError, match="k_new has shape"):
        check_block_shapes(cfg, q, k[:, :1], k)                   # one KV head instead of two
    with pytest.raises(ValueError, match="v_new has shape"):
        check_block_shapes(cfg, q, k, k[:, :, :16])               # fewer rows than k_new
    with pytest.raises(ValueError, match="out has shape"):
        check_block_shapes(cfg, q, k, k, out=q[:, :4])
    cap = 288
    k0 = torch.zeros((2, 2, 100, 64), dtype=torch.bfloat16)
    p0 = torch.zeros((2, 2, 100), dtype=torch.int32)
    assert check_load_shapes(cfg, cap, k0, k0, p0) == 100
    with pytest.raises(ValueError):
        check_load_shapes(cfg, cap, k0[:1], k0[:1], p0[:1])       # the mistake that reads 2x past the end
    with pytest.raises(ValueError):
        check_load_shapes(cfg, cap, k0, k0, p0.to(torch.int64))
    with pytest.raises(ValueError):
        check_load_shapes(cfg, cap, torch.zeros((2, 2, 300, 64), dtype=torch.bfloat16), k0, p0)
    cos = torch.zeros((128, 32), dtype=torch.float32)
    check_rope_tables(cfg, cos, cos)
    with pytest.raises(ValueError):
        check_rope_tables(cfg, cos[:, :16].contiguous(), cos)


def test_build_refuses_kernels_that_use_scratch_memory():
    """The build reads the compiler's per-kernel resource remarks and fails on any kernel with scratch
    memory (such a kernel runs several times slower on this chip): the parser on remarks as hipcc prints them."""
    from paper_2504_15364_amd.build import scratch_users

    remarks = """evict.hip:387:1: remark: Function Name: _ZN2kd17ksum_final_kernelEPKdPdii [-Rpass-analysis=kernel-resource-usage]
evict.hip:387:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]
evict.hip:387:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
evict.hip:255:1: remark: Function Name: _ZN2kd22compact_ordered_kernelILi128EEEvNS_10StepParamsEPiii [-Rpass-analysis=kernel-resource-usage]
evict.hip:255:1: remark:     ScratchSize [bytes/lane]: 700 [-Rpass-analysis=kernel-resource-usage]
evict.hip:255:1: remark:     Occupancy [waves/SIMD]: 4 [-Rpass-analysis=kernel-resource-usage]""".splitlines()
    assert scratch_users(remarks) == [("_ZN2kd22compact_ordered_kernelILi128EEEvNS_10StepParamsEPiii", 700)]
    assert scratch_users(remarks[:3]) == []
