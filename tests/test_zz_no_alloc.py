"""The entry point that allocates nothing (cos_verify_noalloc, the library's built-in scratch array) against
cos_verify_ex with a caller-owned workspace, through the C ABI: same inputs, identical outputs, on calls in a
row that share the array, the later ones on smaller inputs."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_01662_amd import cos_verify as C
from paper_2502_01662_amd import workloads as W


def _both(w, step, **ext):
    inp = W.generate(w, device="cuda", step=step)
    B, gamma = inp["draft_tokens"].shape
    args = (inp["logits"], inp["draft_tokens"], inp["proposer_idx"], w.mode, w.weights, inp["u_accept"],
            inp["u_resample"])
    d_ref = C.Diagnostics.allocate(B, gamma, "cuda")
    a_ref, t_ref = C.cos_verify(*args, diag=d_ref, **ext)
    d_new = C.Diagnostics.allocate(B, gamma, "cuda")
    a_new = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    t_new = torch.full((B, gamma + 1), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    C.cos_verify_noalloc(*args, accepted_len=a_new, out_tokens=t_new, diag=d_new, **ext)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before, "the binding allocated device memory"
    assert torch.equal(a_new, a_ref), (w.name, step)
    assert torch.equal(t_new, t_ref), (w.name, step)
    # same kernels on the same launch plan: the diagnostics are bit-identical as well
    for name in ("r_at_draft", "q_at_draft", "sample_mass", "cdf_lo", "cdf_hi", "flags"):
        assert torch.equal(getattr(d_new, name), getattr(d_ref, name)), (w.name, step, name)
    return a_ref


@pytest.mark.gpu
def test_noalloc_matches_the_workspace_entry_point_on_calls_in_a_row():
    # a larger input first, then smaller ones: the array keeps the last call's contents
    big = W.C3.scaled(B=24)
    small = W.C3.scaled(B=5, V=50048, gamma=3)
    lens = _both(big, 0)
    assert len(set(lens.tolist())) > 1          # rejections and full acceptances both occur
    _both(small, 1)
    _both(W.C2.scaled(B=6), 2)                  # masked contrastive: another set of kernels, same array
    _both(W.C1, 3)
    _both(big, 4)
    _both(small, 5, stop_window=1)              # several streaming launches, several counter sets
    alpha = torch.empty((small.B, small.gamma), dtype=torch.float64, device="cuda")
    _both(small, 6, alpha=alpha)


@pytest.mark.gpu
def test_noalloc_full_size_c4_then_smaller():
    for w, step in ((W.C4, 0), (W.C4.scaled(B=32), 1)):
        _both(w, step)


def test_noalloc_rejects_shapes_beyond_its_array():
    lib = C.load_library()
    cap = C.cos_verify_noalloc_capacity()
    assert cap == 8 << 20
    assert C.cos_verify_workspace_bytes(4, 512, 6, 256000, C.COS_DTYPE_BF16, C.COS_COMBINE_ENSEMBLE) <= cap
    assert C.cos_verify_workspace_bytes(4, 4096, 6, 256000, C.COS_DTYPE_BF16, C.COS_COMBINE_ENSEMBLE) > cap
    w = (ctypes.c_double * 4)(0.25, 0.25, 0.25, 0.25)
    fake = 0x1000   # never dereferenced: the size check comes before any HIP call
    st = lib.cos_verify_noalloc(fake, C.COS_DTYPE_BF16, 4, 4096, 6, 256000, fake, fake, C.COS_COMBINE_ENSEMBLE, w,
                                fake, fake, fake, fake, None, None, None)
    assert st == -10
    assert "scratch" in C.cos_status_string(st)
    # argument validation is the shared one
    assert lib.cos_verify_noalloc(fake, C.COS_DTYPE_BF16, 0, 1, 6, 256, fake, fake, 0, w, fake, fake, fake, fake,
                                  None, None, None) == -2
