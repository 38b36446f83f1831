"""The entry point that allocates nothing (hybrid_attn_forward_static: scratch in a static device array) against
hybrid_attn_forward with a caller workspace, through the C ABI: bit-for-bit equal outputs, two calls in a row with the
second on a smaller input (the array keeps the first call's contents), and a third back on the larger one."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W

pytestmark = pytest.mark.gpu

BIG = W.Workload("static_big", 2, 3, 2741, 128, "bf16", 128, 4, 128, 128, seed=301)
SMALL = W.Workload("static_small", 1, 2, 333, 128, "bf16", 64, 3, 128, 128, seed=302)
LINEAR = W.Workload("static_linear", 1, 2, 1500, 64, "f32", 128, 0, 64, 64, seed=303)


def _both(w):
    q, k, v, fq, fk = ha.to_device(W.make_inputs(w))
    ref = ha.hybrid_attn_forward(q, k, v, fq, fk, w.R, w.block_size, w.scale)
    out = torch.full_like(q, float("nan"))
    free_before = torch.cuda.memory_allocated()
    got = ha.hybrid_attn_forward_static(q, k, v, fq, fk, w.R, out, w.block_size, w.scale)
    assert torch.cuda.memory_allocated() == free_before       # torch's allocator was not asked for anything
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.isfinite(out.float()).all().item(), w.name
    assert torch.equal(out, ref), w.name


def test_static_scratch_matches_workspace_entry_point():
    assert ha.hybrid_attn_static_scratch_bytes() == 64 << 20
    print("  case big", flush=True)
    _both(BIG)
    print("  case small after big", flush=True)
    _both(SMALL)          # smaller input right after: stale contents of the larger call must not matter
    print("  case linear only", flush=True)
    _both(LINEAR)
    print("  case big again", flush=True)
    _both(BIG)


def test_static_scratch_on_a_side_stream():
    w = SMALL
    q, k, v, fq, fk = ha.to_device(W.make_inputs(w))
    ref = ha.hybrid_attn_forward(q, k, v, fq, fk, w.R, w.block_size, w.scale)
    out = torch.empty_like(q)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ha.hybrid_attn_forward_static(q, k, v, fq, fk, w.R, out, w.block_size, w.scale, stream=side)
    side.synchronize()
    assert torch.equal(out, ref)


def test_oversize_problem_is_refused_with_a_clear_error():
    """480p / 81 frames with B = 4: the workspace is far beyond the static array; refused on the host, nothing runs."""
    prob = ha.ha_problem(4, 12, 32760, 128, ha.HA_BF16, 128, 1, 128 ** -0.5, 12 * 32760 * 128, 32760 * 128, 128, 0, 0, 0, 0)
    assert ha.hybrid_attn_workspace_bytes(prob) > ha.hybrid_attn_static_scratch_bytes()
    fake = 0x7F0000001000
    st = ha._lib().hybrid_attn_forward_static(ctypes.byref(prob), fake, fake, fake, None, None, fake, None)
    assert st == ha.HA_ERR_WORKSPACE
    assert "workspace" in ha.hybrid_attn_status_string(st)
