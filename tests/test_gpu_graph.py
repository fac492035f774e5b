"""The three calls of a decode step recorded into a HIP graph and replayed: every replay must give
the eager result (the library only enqueues kernels on the stream it is given)."""
import numpy as np
import pytest
import torch

import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_cache

pytestmark = pytest.mark.gpu


def test_decode_step_in_a_hip_graph():
    case = wl.make_case("g", B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1500, 64, 700, 129], seed=40)
    cache = gpu_cache(case)
    last = case.offsets[1:] - 1
    k_new, v_new = dev_bits(case.k[last]), dev_bits(case.v[last])
    slots = torch.from_numpy(case.slot_mapping[last]).to(DEV)
    q = dev_bits(case.q)
    bt = torch.from_numpy(case.block_table).to(DEV)
    sl = torch.from_numpy(case.seq_lens).to(DEV)
    sinks = torch.from_numpy(case.sinks).to(DEV)
    split = 256
    S = pz.pz_decode_attn_n_splits(1500, 0, split)
    wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S)
    ws = torch.zeros(wsb // 4, dtype=torch.float32, device=DEV)
    out = torch.zeros((case.B, case.Hq, case.d), dtype=torch.float32, device=DEV)

    def step():
        pz.pz_kv_append_fp8(cache, k_new, v_new, slots, case.B, case.k_scale, case.v_scale)
        pz.pz_decode_attn(cache, q, bt, case.max_pages, sl, case.B, case.Hq, sinks, case.sm_scale, case.k_scale,
                          case.v_scale, 0, split, S, ws, wsb, out)
        pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, 0, split, sinks, case.v_scale, out)

    step()
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                     # warm-up on the capture stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for i in range(4):
        out.fill_(float("nan"))                                    # eager work between the replays
        ws.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), i
