"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes its workspace, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2502_01662_amd import cos_verify as C

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cos_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cos_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = C.load_library()
    names = _declared_functions()
    assert {"cos_verify", "cos_verify_workspace_bytes", "cos_status_string", "cos_verify_version"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_version_and_status_strings():
    assert C.cos_verify_version() == 7
    assert C.cos_status_string(0) == "ok"
    for code in range(-10, 0):
        assert C.cos_status_string(code) not in ("ok", "unknown status")


def test_workspace_bytes():
    assert C.cos_verify_workspace_bytes(4, 512, 6, 256000, C.COS_DTYPE_BF16, C.COS_COMBINE_ENSEMBLE) > 0
    small = C.cos_verify_workspace_bytes(2, 1, 5, 32000, C.COS_DTYPE_F32, C.COS_COMBINE_ENSEMBLE)
    big = C.cos_verify_workspace_bytes(2, 2, 5, 32000, C.COS_DTYPE_F32, C.COS_COMBINE_ENSEMBLE)
    assert 0 < small < big
    assert C.cos_verify_workspace_bytes(0, 1, 5, 32000, 0, 0) == 0            # n < 1
    assert C.cos_verify_workspace_bytes(9, 1, 5, 32000, 0, 0) == 0            # n > COS_MAX_MODELS
    assert C.cos_verify_workspace_bytes(2, 1, 0, 32000, 0, 0) == 0            # gamma < 1
    assert C.cos_verify_workspace_bytes(2, 1, 32, 32000, 0, 0) == 0           # gamma > COS_MAX_GAMMA
    assert C.cos_verify_workspace_bytes(2, 1, 5, (1 << 20) + 1, 0, 0) == 0    # V > COS_MAX_VOCAB
    for dt in (C.COS_DTYPE_F32, C.COS_DTYPE_BF16, C.COS_DTYPE_F16):          # every format, every mode
        for mode, n in ((C.COS_COMBINE_ENSEMBLE, 3), (C.COS_COMBINE_CONTRASTIVE, 2), (C.COS_COMBINE_LOGIT_MIX, 3)):
            assert C.cos_verify_workspace_bytes(n, 4, 5, 32000, dt, mode) >= 256
    assert C.cos_verify_workspace_bytes(2, 4, 5, 32000, C.COS_DTYPE_F16, 0) == \
        C.cos_verify_workspace_bytes(2, 4, 5, 32000, C.COS_DTYPE_BF16, 0)    # both are 2-byte formats
    assert C.cos_verify_workspace_bytes(2, 1, 5, 32000, 7, 0) == 0            # dtype
    assert C.cos_verify_workspace_bytes(2, 1, 5, 32000, 0, 7) == 0            # mode


def _call(n=2, B=1, gamma=2, V=16, dt=0, mode=0, weights=(0.5, 0.5), logits=0x1000, draft=0x1000,
          prop=0x1000, ua=0x1000, ur=0x1000, alen=0x1000, toks=0x1000, ws=0x1000, ws_bytes=1 << 20):
    """Call cos_verify with fake (never dereferenced) device pointers: validation runs on the host
    and every case here must be rejected before any HIP call."""
    lib = C.load_library()
    w = (ctypes.c_double * len(weights))(*weights)
    return lib.cos_verify(logits, dt, n, B, gamma, V, draft, prop, mode, w, ua, ur, alen, toks, ws, ws_bytes,
                          None, None)


def test_argument_validation_needs_no_gpu():
    assert _call(n=0) == -2
    assert _call(gamma=0) == -2
    assert _call(V=0) == -2
    assert _call(B=-1) == -2
    assert _call(dt=5) == -3
    assert _call(mode=3) == -4
    assert _call(mode=2, weights=(1.5, -0.5)) not in (-4, -5)     # logit mix: any finite weights ...
    assert _call(mode=2, weights=(1.5, float("inf"))) == -5       # ... but finite
    assert _call(dt=2, logits=0x1001) == -7                       # binary16 logits at an odd address
    assert _call(mode=1, n=3, weights=(0.5, 0.1, 0.0)) == -4      # contrastive needs n == 2
    assert _call(weights=(0.5, 0.6)) == -5
    assert _call(weights=(1.5, -0.5)) == -5
    assert _call(weights=(float("nan"), 0.5)) == -5
    assert _call(mode=1, weights=(0.5, 1.5)) == -5                # alpha_cd outside [0,1]
    assert _call(mode=1, weights=(float("inf"), 0.1)) == -5       # mu not finite
    assert _call(logits=0) == -1
    assert _call(draft=0) == -1
    assert _call(toks=0) == -1
    assert _call(dt=0, logits=0x1002) == -7                       # float32 logits at a 2-byte address
    assert _call(ws=0) == -6
    assert _call(ws=0x1010) == -6                                 # workspace not 256-byte aligned
    assert _call(ws_bytes=16) == -6
    assert _call(B=0, logits=0, draft=0) == 0                     # empty batch: a no-op


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(C.CosVerifyError):
        C.cos_verify(torch.zeros((2, 1, 3, 8)), torch.zeros((1, 2), dtype=torch.int32),
                     torch.zeros(1, dtype=torch.int32), 0, [0.5, 0.5], torch.zeros((1, 2), dtype=torch.float64),
                     torch.zeros(1, dtype=torch.float64))


class _Options(ctypes.Structure):
    _fields_ = C.CosOptions._fields_


def _call_ex(opt, mode=0, weights=(0.5, 0.5), gamma=2):
    lib = C.load_library()
    w = (ctypes.c_double * len(weights))(*weights)
    return lib.cos_verify_ex(0x1000, 0, 2, 1, gamma, 16, 0x1000, 0x1000, mode, w, 0x1000, 0x1000, 0x1000, 0x1000,
                             0x1000, 16, None, ctypes.byref(opt), None)     # workspace too small: -6 if all else passes


def test_option_validation_needs_no_gpu():
    size = ctypes.sizeof(C.CosOptions)
    ok = C.CosOptions(size, 0.0, None, None, None, 0, 0, None, 0)
    assert _call_ex(ok) == -6                                               # options accepted, workspace rejected
    assert _call_ex(C.CosOptions(size - 8, 0.0, None, None, None, 0, 0, None, 0)) == -9      # another ABI's struct
    assert _call_ex(C.CosOptions(size, -1.0, None, None, None, 0, 0, None, 0)) == -5         # temperature < 0
    assert _call_ex(C.CosOptions(size, float("nan"), None, None, None, 0, 0, None, 0)) == -5
    assert _call_ex(C.CosOptions(size, 0.0, None, None, None, -1, 0, None, 0)) == -2         # stop_window < 0
    assert _call_ex(C.CosOptions(size, 0.0, None, None, None, 0, 1, None, 0)) == -6          # greedy ensemble: built
    assert _call_ex(C.CosOptions(size, 0.0, None, 0x1000, None, 0, 1, None, 0)) == -6        # ... with per-position proposers
    assert _call_ex(C.CosOptions(size, 0.0, None, None, 0x1000, 0, 1, None, 0)) == -9        # ... but not with acceptance rates
    assert _call_ex(C.CosOptions(size, 0.0, None, None, None, 0, 1, None, 0), mode=2) == -6  # greedy logit mix: built
    assert _call_ex(C.CosOptions(size, 0.0, None, 0x1000, None, 0, 1, None, 0), mode=2) == -9  # ... not per-position proposers
    assert _call_ex(C.CosOptions(size, 0.0, None, None, None, 0, 1, None, 0), mode=1, weights=(0.5, 0.1)) == -6
    assert _call_ex(C.CosOptions(size, 0.0, None, None, 0x1000, 1, 0, None, 0)) == -9        # alpha with windows
    assert _call_ex(C.CosOptions(size, 0.0, None, None, 0x1000, 5, 0, None, 0)) == -6        # window > gamma: one launch
    assert _call_ex(C.CosOptions(size, 0.0, None, None, None, 0, 0, 0x1000, 1)) == -6        # ragged, no bonus


def test_cpp_driver_links_the_library_and_validates_its_arguments():
    """The plain C++ caller is built with the library; bad arguments end it before any GPU call."""
    import subprocess
    from paper_2502_01662_amd import build as B
    if not os.path.exists(B.DRIVER):
        B.build_driver()
    assert subprocess.run([B.DRIVER, "0"], capture_output=True).returncode == 2              # n = 0
    assert subprocess.run([B.DRIVER, "2", "1", "2", "16", "int8"], capture_output=True).returncode == 2
    assert subprocess.run([B.DRIVER, "2", "1", "2", "16", "bf16", "vote"], capture_output=True).returncode == 2


def test_workspace_bytes_follow_the_launch_shape_of_the_call():
    """Shorter chunks for the last sequences need more room for chunk partials: the size function and the
    call agree on it because both take the same options (a workspace sized for other options is rejected)."""
    shape = (2, 2048, 4, 128256, C.COS_DTYPE_BF16, C.COS_COMBINE_ENSEMBLE)   # whole rows per workgroup by default
    plain = C.cos_verify_workspace_bytes_ex(*shape, C.LaunchShape(tail_sequences=-1))
    finer_shape = C.LaunchShape(tail_sequences=8, tail_factor=16)
    finer = C.cos_verify_workspace_bytes_ex(*shape, finer_shape)
    assert finer > plain > 0
    assert C.cos_verify_workspace_bytes_ex(*shape, None) == C.cos_verify_workspace_bytes(*shape) >= plain
    lib = C.load_library()
    w = (ctypes.c_double * 2)(0.5, 0.5)
    opt = C._options(shape=finer_shape)
    call = lambda nbytes, o: lib.cos_verify_ex(0x1000, 1, 2, 2048, 4, 128256, 0x1000, 0x1000, 0, w, 0x1000, 0x1000,
                                               0x1000, 0x1000, 0x1000, nbytes, None, o, None)
    assert call(plain, ctypes.byref(opt)) == -6                  # too small for these options: rejected on the host
    bad = C._options()
    bad.struct_bytes = 8
    assert call(finer, ctypes.byref(bad)) == -9                  # an options struct of another size
    assert lib.cos_verify_workspace_bytes_ex(*shape, ctypes.byref(bad)) == 0


def test_the_library_keeps_no_settings_between_calls():
    """Every exported function is declared in the header, and none of them sets process-wide state:
    no cos_tune_* / cos_profile_* symbols exist any more."""
    lib = C.load_library()
    for name in ("cos_tune_set_chunk_vectors", "cos_tune_set_sample_blocks", "cos_tune_set_tail", "cos_profile_enable",
                 "cos_profile_recorded", "cos_profile_kernel_ms"):
        assert not hasattr(lib, name), name


def test_input_checker_validates_its_own_arguments_on_the_host():
    lib = C.load_library()
    bad = ctypes.c_int(-1)
    call = lambda n, B, ws, ws_bytes, draft=0x1000: lib.cos_verify_check_inputs(
        n, B, 2, 16, draft, 0x1000, 0x1000, 0x1000, None, ws, ws_bytes, ctypes.byref(bad), None)
    assert call(0, 1, 0x1000, 256) == -2                          # n out of range
    assert call(2, 1, 0x1000, 256, draft=0) == -1                 # a required array is missing
    assert call(2, 1, 0, 256) == -6 and call(2, 1, 0x1010, 256) == -6 and call(2, 1, 0x1000, 16) == -6
    assert call(2, 0, 0, 0) == 0 and bad.value == 0               # empty batch: nothing to check
    assert lib.cos_verify_check_inputs(2, 1, 2, 16, 0x1000, 0x1000, 0x1000, 0x1000, None, 0x1000, 256, None, None) == -1


def test_workspace_of_an_empty_batch_and_of_every_refinement_route():
    """Sizing never divides by the batch size, and does not depend on how residuals of little mass are refined."""
    for mode, n in ((C.COS_COMBINE_ENSEMBLE, 3), (C.COS_COMBINE_CONTRASTIVE, 2), (C.COS_COMBINE_LOGIT_MIX, 3)):
        assert C.cos_verify_workspace_bytes(n, 0, 4, 1000, C.COS_DTYPE_BF16, mode) >= 256
        sizes = {C.cos_verify_workspace_bytes_ex(n, 17, 4, 70000, C.COS_DTYPE_BF16, mode, C.LaunchShape(refine_kernels=r))
                 for r in (-1, 0, 1)}
        assert len(sizes) == 1 and min(sizes) > 256


def test_launch_info_whole_rows_routes_and_windows():
    """What a call would enqueue, without a GPU.  Once a call has thousands of rows a workgroup takes a whole
    row -- never a long chunk and a sliver (float32 rows of 64000 vectors were once cut into 63488 + 512)."""
    ens, cd, mix = C.COS_COMBINE_ENSEMBLE, C.COS_COMBINE_CONTRASTIVE, C.COS_COMBINE_LOGIT_MIX
    for dt, V in ((C.COS_DTYPE_F32, 256000), (C.COS_DTYPE_BF16, 256000), (C.COS_DTYPE_F32, 128256), (C.COS_DTYPE_F16, 152064)):
        info = C.cos_verify_launch_info(4, 512, 6, V, dt, ens, [0.25] * 4)
        nvec = -(-V // (4 if dt == C.COS_DTYPE_F32 else 8))
        assert info["chunks_per_row"] == 1 and info["chunk_vectors"] >= nvec, info
        assert info["tail_sequences"] > 0 and info["tail_chunks_per_row"] == 4
        assert info["streaming_launches"] == 1 and info["sample_workgroups"] == 2 and info["refine_launches"] == 1
        assert info["workspace_bytes"] == C.cos_verify_workspace_bytes(4, 512, 6, V, dt, ens)
    # a cut row: chunks of at least one full group of loads (2048 vectors), the last one not empty
    for n, B, gamma, V in ((3, 64, 4, 152064), (2, 16, 5, 128256), (2, 1, 5, 32000), (4, 8, 6, 256000), (2, 40, 3, 50257)):
        info = C.cos_verify_launch_info(n, B, gamma, V, C.COS_DTYPE_BF16, ens, [1.0 / n] * n)
        nvec = -(-V // 8)
        last = nvec - (info["chunks_per_row"] - 1) * info["chunk_vectors"]
        assert info["chunks_per_row"] > 1 and info["chunk_vectors"] >= 2048 and 0 < last <= info["chunk_vectors"], info
    # small row-sets keep the lone refinement, windows multiply the streaming launches
    small = C.cos_verify_launch_info(2, 1, 5, 32000, C.COS_DTYPE_F32, ens, [0.5, 0.5])
    assert small["refine_launches"] == 0 and small["sample_workgroups"] > 1
    assert C.cos_verify_launch_info(2, 1, 5, 32000, C.COS_DTYPE_F32, ens, [0.5, 0.5],
                                    shape=C.LaunchShape(refine_kernels=1))["refine_launches"] == 1
    assert C.cos_verify_launch_info(2, 8, 5, 32000, C.COS_DTYPE_F32, ens, [0.5, 0.5], stop_window=2)["streaming_launches"] == 3
    # masked contrastive mode: one read while the mask can be expected to be sparse
    for alpha_cd, T, one in ((0.1, 1.0, 1), (0.05, 1.0, 1), (0.03, 1.0, 0), (0.1, 2.0, 0), (0.002, 0.5, 1), (0.0, 1.0, 0)):
        info = C.cos_verify_launch_info(2, 16, 5, 128256, C.COS_DTYPE_BF16, cd, [0.5, alpha_cd], temperature=T)
        assert info["one_read_mask"] == one and (info["sample_workgroups"] == 0) == bool(one), (alpha_cd, T, info)
    forced = C.cos_verify_launch_info(2, 16, 5, 128256, C.COS_DTYPE_BF16, cd, [0.5, 0.001], shape=C.LaunchShape(two_pass_mask=-1))
    assert forced["one_read_mask"] == 1
    assert C.cos_verify_launch_info(3, 16, 5, 128256, C.COS_DTYPE_BF16, mix, [0.5, 0.3, 0.2], greedy=True)["greedy"] == 1
    with pytest.raises(C.CosVerifyError):
        C.cos_verify_launch_info(3, 16, 5, 128256, C.COS_DTYPE_BF16, cd, [0.5, 0.1])
