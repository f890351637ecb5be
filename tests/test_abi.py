"""CPU-only checks of the C ABI: the shared library loads, exports every
function include/dllm.h declares, and rejects bad arguments before touching a
GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

from paper_2506_10848_amd import binding as b

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "dllm.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dllm_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = b.lib()
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(b.EXPORTS) == names          # the binding covers the whole header


def test_struct_layouts_match_the_header():
    assert C.sizeof(b.Config) == 11 * 4
    assert C.sizeof(b.StageParams) == 9 * 4
    assert C.sizeof(b.DecodeParams) == 12 * 4
    assert C.sizeof(b.StepStat) == 5 * 4
    assert C.sizeof(b.CommitListC) == 8 + 7 * 8


def good_config(**kw):
    c = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=2048, mask_id=2047,
             rms_eps=1e-5, rope_theta=1e4, max_batch=1, max_seq=96)
    c.update(kw)
    return b.Config(*[c[k] for k in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id",
                                     "rms_eps", "rope_theta", "max_batch", "max_seq")])


@pytest.mark.parametrize("kw,needle", [
    (dict(head_dim=32, n_heads=8), "head_dim"), (dict(n_heads=3), "differs from d_model"),
    (dict(mask_id=2048), "mask_id"), (dict(mask_id=-1), "mask_id"), (dict(max_batch=0), "max_batch"),
    (dict(max_batch=65), "max_batch"), (dict(max_seq=8193), "max_seq"), (dict(d_ffn=684), "multiples of 8"),
    (dict(vocab=2050, mask_id=5), "multiples of 8"), (dict(rope_theta=0.0), "rope_theta"),
])
def test_create_rejects_bad_configs(kw, needle):
    lib = b.lib()
    h = C.c_void_p()
    w = b.Weights()
    c = good_config(**kw)
    rc = lib.dllm_create(C.byref(c), C.byref(w), None, C.byref(h))
    assert rc == b.EINVAL and not h.value
    assert needle in lib.dllm_last_error(None).decode()


def test_create_rejects_null_weights_and_arguments():
    lib = b.lib()
    h = C.c_void_p()
    c = good_config()
    assert lib.dllm_create(C.byref(c), C.byref(b.Weights()), None, C.byref(h)) == b.EINVAL
    assert "null embed" in lib.dllm_last_error(None).decode()
    assert lib.dllm_create(None, C.byref(b.Weights()), None, C.byref(h)) == b.EINVAL
    assert lib.dllm_create(C.byref(c), C.byref(b.Weights()), None, None) == b.EINVAL


def test_null_handles_and_pointers_are_errors_not_crashes():
    lib = b.lib()
    assert lib.dllm_step(None, 1, 8, None, None, None, None, None) == b.EINVAL
    assert lib.dllm_decode(None, 1, 8, 0, None, None, None, None, None, 0) == b.EINVAL
    assert lib.dllm_forward(None, 1, 8, None) == b.EINVAL
    assert lib.dllm_debug_logits(None, None) == b.EINVAL
    assert lib.dllm_profile_begin(None, 4) == b.EINVAL
    assert lib.dllm_select(None, None, 1, 8, 64, 63, None, None, None, None, None, None, None) == b.EINVAL
    assert lib.dllm_op_linear(None, None, None, None, 8, 8, 8) == b.EINVAL
    assert lib.dllm_op_attention(None, None, None, 1, 8, 1, 64) == b.EINVAL
    lib.dllm_destroy(None)                       # no-op


def test_select_validates_before_launching():
    lib = b.lib()
    fake = C.c_void_p(0x1000)                    # never dereferenced: validation fails first
    cl = b.CommitListC(8, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    sp = (b.StageParams * 1)(b.stage_params(0, 0, 7, 0, .1, .9, 0, 0, 8))     # top_k = 0
    rc = lib.dllm_select(None, fake, 1, 8, 64, 63, fake, fake, fake, sp, fake, fake, C.byref(cl))
    assert rc == b.EINVAL and "top_k" in lib.dllm_last_error(None).decode()
    sp[0].top_k = 1
    cl.capacity = 3
    rc = lib.dllm_select(None, fake, 1, 8, 64, 63, fake, fake, fake, sp, fake, fake, C.byref(cl))
    assert rc == b.ECAPACITY
    rc = lib.dllm_select(None, fake, 65, 8, 64, 63, fake, fake, fake, sp, fake, fake, C.byref(cl))
    assert rc == b.EINVAL
    rc = lib.dllm_select(None, fake, 1, 8, 64, 64, fake, fake, fake, sp, fake, fake, C.byref(cl))
    assert rc == b.EINVAL and "mask_id" in lib.dllm_last_error(None).decode()


def test_split_count_never_exceeds_the_slabs_that_fit():
    """The O and down projections write one fp32 slab per K split into a workspace sized at create;
    each launch tells the planner how many slabs of its row count fit.  Sweep of row counts (cached
    steps recompute arbitrary subsets) for a narrow and a wide model: the plan obeys the limit, also
    between the multiples of the tile heights."""
    b.reload_env()
    for d, f in [(256, 688 + 16), (4096, 12288)]:
        for rows in list(range(4090, 4110)) + list(range(4097, 12289, 97)) + [12288]:
            for limit in (1, 2, 8):
                for N, K in [(d, d), (d, f)]:
                    if K % 64:
                        continue
                    p = b.gemm_plan(2, rows, N, K, limit)
                    assert 1 <= p["splits"] <= limit
    # no limit given: at most 8
    assert b.gemm_plan(2, 512, 4096, 12288)["splits"] <= 8
    # other epilogues never split
    assert b.gemm_plan(1, 512, 24576, 4096)["splits"] == 1 and b.gemm_plan(5, 256, 126464, 4096)["splits"] == 1
