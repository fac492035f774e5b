"""The streaming loop of the decode kernels, checked in the compiler's output (CPU only: hipcc cross-compiles).

The loop is written so that every wait counts exactly the loads issued after the one it needs: with 4 K
and 4 V loads of 16 bytes in flight per lane, the K tile of a step is consumed piece by piece under
s_waitcnt vmcnt(7), (6), (5), (4) (the four pieces of V, requested later, may still be outstanding), and
so is the V tile under the same counts after the next K tile has been requested.  Small changes
around the loop -- a load left pending across it, a branch inside it -- have made the compiler rotate the
loop or merge the waits into vmcnt(0), which serialises loads and arithmetic and costs 4 to 8 % of a
launch without failing any numerical test.  This test fails then."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2602_11937_amd import build as B

KERNELS = {
    "pz_attn.hip": "_ZN12_GLOBAL__N_118decode_attn_kernelILi64ELi1EEEvN2pz10AttnParamsE",
    "pz_attn_balanced.hip": "_ZN12_GLOBAL__N_127decode_attn_balanced_kernelILi64ELi1EEEvN2pz10AttnParamsE",
}


def kernel_asm(source, symbol):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
        r = subprocess.run([B.HIPCC, *flags, "--cuda-device-only", "-S", "-o", out, os.path.join(B.CSRC, source)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    start = text.index("\n" + symbol + ":")
    return text[start:text.index("s_endpgm", start)]


@pytest.mark.parametrize("source", sorted(KERNELS))
def test_streaming_loop_waits_count_the_loads_in_flight(source):
    asm = kernel_asm(source, KERNELS[source])
    # the first innermost loop that holds the non-temporal tile loads: its body follows its header
    bodies = [b for b in re.split(r"This Inner Loop Header: Depth=\d+", asm)[1:]
              if len(re.findall(r"global_load_dwordx4 .* nt", b[:b.find("Loop Header") if "Loop Header" in b else len(b)])) >= 8]
    assert bodies, "no streaming loop found"
    waits = [int(x) for x in re.findall(r"s_waitcnt vmcnt\((\d+)\)", bodies[0])][:12]
    # K pieces, then (after the next K tile is requested) V pieces: 7 6 5 4 each time, never a full drain
    assert len(waits) == 12 and 0 not in waits, waits
    assert waits == [7, 6, 5, 4] * 3, waits
