"""The cross-workgroup hand-off rests on which instructions gfx950 code gets for it: agent-scope
write-through stores, a wait for their completion, an agent-scope atomic increment, agent-scope loads --
and no cache-wide write-back or invalidate.  This compiles a few lines that use the hand-off primitives
of csrc/cos_device.h for gfx950 (no GPU needed) and checks the instruction stream."""
import os
import re
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SNIPPET = r'''
#include "cos_device.h"
extern "C" __global__ void handoff_roundtrip(Partial* slot, int* counter, int total, double* out) {
  __shared__ int s_flag;
  if (threadIdx.x == 0) {
    slot[blockIdx.x].Z.publish(1.5 * blockIdx.x);
    slot[blockIdx.x].o.publish((int)blockIdx.x);
    wait_stores();
  }
  if (arrive_last(counter, total, &s_flag)) {
    double z = 0.0;
    for (int i = threadIdx.x; i < total; i += blockDim.x) z += slot[i].Z.read() + slot[i].o.read();
    out[threadIdx.x] = z;
  }
}
'''


def _asm():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as d:
        src, out = os.path.join(d, "snippet.hip"), os.path.join(d, "snippet.s")
        open(src, "w").write(SNIPPET)
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-value",
                        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2502_01662_amd", "csrc"),
                        "-o", out, src], check=True, capture_output=True)
        text = open(out).read()
    body = text[text.index("handoff_roundtrip:"):text.index(".Lfunc_end0")]
    return [ln.strip() for ln in body.splitlines() if ln.strip() and not ln.strip().startswith((";", "."))]


def test_handoff_compiles_to_write_through_stores_a_wait_and_agent_scope_loads():
    ins = _asm()
    stores = [i for i, ln in enumerate(ins) if ln.startswith("global_store")]
    atomics = [i for i, ln in enumerate(ins) if ln.startswith("global_atomic_inc")]   # wraps to zero at the last arrival
    loads = [i for i, ln in enumerate(ins) if re.match(r"global_load_dword(x2)? ", ln)]
    waits = [i for i, ln in enumerate(ins) if ln.startswith("s_waitcnt") and "vmcnt(0)" in ln]
    assert len(atomics) == 1
    publish = [i for i in stores if i < atomics[0]]
    assert len(publish) == 2
    for i in publish:                                    # published values: write-through at agent scope
        assert re.search(r"\bsc1\b", ins[i]) and not re.search(r"\bsc0\b", ins[i]), ins[i]
    assert any(max(publish) < w < atomics[0] for w in waits), "no wait between the stores and the counter bump"
    hand_off_loads = [i for i in loads if i > atomics[0]]
    assert hand_off_loads
    for i in hand_off_loads:                             # hand-off reads: agent-scope loads
        assert re.search(r"\bsc1\b", ins[i]), ins[i]
    # no cache-wide write-back or invalidate anywhere: the protocol does not need them
    assert not any(ln.startswith(("buffer_wbl2", "buffer_inv")) for ln in ins)
    # a barrier separates the atomic's return from the reads
    assert any(ln.startswith("s_barrier") and atomics[0] < i < min(hand_off_loads) for i, ln in enumerate(ins))
