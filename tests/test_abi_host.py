"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes the workspace, and turns bad arguments into status codes before any
device work.  (No compute call is made here.)"""
import os
import re

import pytest

from paper_2103_13262_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000   # an aligned, non-null address; never dereferenced because validation fails first


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_size_and_regions():
    d = B.make_desc(4096, 1024, 4096, 16, 2)
    total = B.moe_workspace_bytes(d)
    M = 8192
    need = 2 * (3 * M * 4096 + 4 * M * 1024)         # Z, H, dZ and Xs, Ys, dYs, dXs in bf16
    # plus the gate scratch, tile tables and 128 MiB of partial-sum tiles (2 phases x 256 persistent workgroups x 256 KiB)
    assert need + (128 << 20) <= total <= need + (128 << 20) + (8 << 20)
    prev_end = 0
    for name in ("Xs", "Z", "H", "Ys", "dYs", "dZ", "dXs", "dl"):   # ("status" lies behind the tables)
        off, n = B.moe_workspace_region(d, name)
        assert off % 256 == 0 and off >= prev_end and off + n <= total
        prev_end = off + n
    with pytest.raises(B.MoeError):
        B.moe_workspace_region(d, "nope")
    assert B.moe_workspace_bytes(B.make_desc(0, 64, 64, 4, 2)) > 0


@pytest.mark.parametrize("kw,status", [
    (dict(N=-1), B.MOE_ERR_INVALID_ARG),
    (dict(k=0), B.MOE_ERR_INVALID_ARG),
    (dict(k=5, E=4), B.MOE_ERR_INVALID_ARG),
    (dict(d=48), B.MOE_ERR_UNSUPPORTED),
    (dict(h=100), B.MOE_ERR_UNSUPPORTED),
    (dict(E=2048), B.MOE_ERR_UNSUPPORTED),
    (dict(k=9, E=16), B.MOE_ERR_UNSUPPORTED),
    (dict(dtype=7), B.MOE_ERR_UNSUPPORTED),
    (dict(dtype=B.MOE_F32, grad_dtype=B.MOE_BF16), B.MOE_ERR_UNSUPPORTED),
    (dict(accumulate=2), B.MOE_ERR_INVALID_ARG),
    (dict(score_all=2), B.MOE_ERR_INVALID_ARG),
    (dict(balance_stats=3), B.MOE_ERR_INVALID_ARG),
])
def test_bad_descriptions_are_rejected(kw, status):
    base = dict(N=16, d=64, h=64, E=4, k=2, dtype=B.MOE_BF16, grad_dtype=None, accumulate=0, score_all=0, balance_stats=0)
    base.update(kw)
    d = B.make_desc(**base)
    assert B.moe_workspace_bytes(d) == 0
    plan = B.make_plan(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    with pytest.raises(B.MoeError) as ei:
        B.moe_plan(d, FAKE, FAKE, None, plan, FAKE, 1 << 30)
    assert ei.value.status == status
    assert B.moe_last_error() != ""


def test_reserved_fields_must_be_zero():
    d = B.make_desc(16, 64, 64, 4, 2)
    d.reserved[3] = 1
    assert B.moe_workspace_bytes(d) == 0


def test_scores_over_all_experts_need_more_workspace_and_the_standalone_backwards_refuse_them():
    a, b = B.make_desc(512, 64, 64, 8, 2), B.make_desc(512, 64, 64, 8, 2, score_all=1)
    assert B.moe_workspace_bytes(b) >= B.moe_workspace_bytes(a) + 512 * 8 * 12 + 512 * 64 * 4
    plan = B.make_plan(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    for c in (lambda: B.moe_gather_backward(b, plan, FAKE, FAKE, FAKE, FAKE),
              lambda: B.moe_scatter_backward(b, plan, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, B.moe_workspace_bytes(b))):
        with pytest.raises(B.MoeError) as ei:
            c()
        assert ei.value.status == B.MOE_ERR_UNSUPPORTED


def test_null_misaligned_and_small_workspace_arguments():
    d = B.make_desc(16, 64, 64, 4, 2)
    ws = B.moe_workspace_bytes(d)
    plan = B.make_plan(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    cases = [
        lambda: B.moe_plan(d, None, FAKE, None, plan, FAKE, ws),                         # X NULL
        lambda: B.moe_plan(d, FAKE + 2, FAKE, None, plan, FAKE, ws),                     # X misaligned
        lambda: B.moe_plan(d, FAKE, FAKE, None, B.make_plan(FAKE, None, FAKE, FAKE, FAKE, FAKE), FAKE, ws),
        lambda: B.moe_forward(d, plan, FAKE, None, FAKE, None, None, FAKE, FAKE, ws),    # W1 NULL
        lambda: B.moe_backward(d, plan, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, ws),
        lambda: B.moe_scatter(d, plan, None, FAKE),                                      # X NULL
        lambda: B.moe_scatter(d, plan, FAKE, FAKE + 4),                                  # Xs misaligned
        lambda: B.moe_gather(d, plan, FAKE, None),                                       # Y NULL
        lambda: B.moe_gather_backward(d, plan, FAKE, FAKE, FAKE, None),                  # dl NULL
        lambda: B.moe_gather_backward(d, None, FAKE, FAKE, FAKE, FAKE),                  # plan NULL
        lambda: B.moe_scatter_backward(d, plan, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, ws),   # dWg NULL
    ]
    for c in cases:
        with pytest.raises(B.MoeError) as ei:
            c()
        assert ei.value.status == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError) as ei:
        B.moe_plan(d, FAKE, FAKE, None, plan, FAKE, ws - 1)
    assert ei.value.status == B.MOE_ERR_WORKSPACE
    with pytest.raises(B.MoeError) as ei:
        B.moe_scatter_backward(d, plan, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, ws - 1)
    assert ei.value.status == B.MOE_ERR_WORKSPACE
    for c in (lambda: B.moe_forward(d, plan, FAKE, FAKE, FAKE, FAKE + 2, None, FAKE, FAKE, ws),   # b1 misaligned
              lambda: B.moe_bias_backward(d, plan, FAKE + 4, None, FAKE, ws),                          # db1 misaligned
              lambda: B.moe_bias_backward(d, None, FAKE, FAKE, FAKE, ws)):                            # plan NULL
        with pytest.raises(B.MoeError) as ei:
            c()
        assert ei.value.status == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError) as ei:
        B.moe_bias_backward(d, plan, FAKE, FAKE, FAKE, ws - 1)
    assert ei.value.status == B.MOE_ERR_WORKSPACE


def test_static_scratch_call_rejects_bad_arguments_and_what_does_not_fit():
    """moe_scatter_backward_static: same checks as moe_scatter_backward, and a problem whose partial sums exceed the
    fixed 16 MiB array is refused with the sizes in the message -- all before any device work."""
    plan = B.make_plan(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    d = B.make_desc(16, 64, 64, 4, 2)
    for c in (lambda: B.moe_scatter_backward_static(d, plan, FAKE, FAKE, FAKE, FAKE, FAKE, None, None),      # dWg NULL
              lambda: B.moe_scatter_backward_static(d, plan, FAKE, FAKE + 2, FAKE, FAKE, FAKE, FAKE, None),  # Xs misaligned
              lambda: B.moe_scatter_backward_static(d, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None)):     # plan NULL
        with pytest.raises(B.MoeError) as ei:
            c()
        assert ei.value.status == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError) as ei:
        B.moe_scatter_backward_static(B.make_desc(16, 64, 64, 4, 2, score_all=1), plan, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    assert ei.value.status == B.MOE_ERR_UNSUPPORTED
    big = B.make_desc(1 << 20, 4096, 32, 8, 2)     # (2^21 / 64 + 8) pieces x 4096 floats = 512 MiB of partial sums
    with pytest.raises(B.MoeError) as ei:
        B.moe_scatter_backward_static(big, plan, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    assert ei.value.status == B.MOE_ERR_WORKSPACE and "16777216" in str(ei.value)
