"""Two layers stepped on two HIP streams at once (default priorities): the library keeps no state between
calls and only enqueues on the stream it is given, so interleaved steps on separate caches and workspaces
must give what each layer gives alone."""
import numpy as np
import pytest
import torch

import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_cache

pytestmark = pytest.mark.gpu


class LayerStep:
    def __init__(self, seed, window, split):
        case = wl.make_case("st", B=6, Hq=16, Hkv=2, d=64, P=64, seq_lens=[2500, 64, 700, 129, 1, 1300],
                            window=window, seed=seed)
        self.case, self.window, self.split = case, window, split
        last = case.offsets[1:] - 1
        prefix = case.slot_mapping.copy()
        prefix[last] = -1
        self.cache = gpu_cache(case, slots=prefix)
        self.k_new, self.v_new = dev_bits(case.k[last]), dev_bits(case.v[last])
        self.q, self.bt = dev_bits(case.q), torch.from_numpy(case.block_table).to(DEV)
        self.sl, self.sinks = torch.from_numpy(case.seq_lens).to(DEV), torch.from_numpy(case.sinks).to(DEV)
        self.S = pz.pz_decode_attn_n_splits(int(case.seq_lens.max()), window, split) if split else 0
        self.wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, self.S) if split else 0
        self.ws = torch.zeros(max(self.wsb, 4) // 4, dtype=torch.float32, device=DEV)
        self.out = torch.zeros((case.B, case.Hq, case.d), dtype=torch.float32, device=DEV)

    def step(self, stream=None):
        c = self.case
        pz.pz_decode_attn_append(self.cache, self.k_new, self.v_new, self.q, self.bt, c.max_pages, self.sl, c.B, c.Hq,
                                 self.sinks, c.sm_scale, c.k_scale, c.v_scale, self.window, self.split, self.S,
                                 self.ws if self.split else None, self.wsb, self.out, stream=stream)
        if self.split:
            pz.pz_decode_attn_splitk_reduce(self.ws, self.wsb, c.B, c.Hq, c.d, self.S, self.sl, self.window, self.split,
                                            self.sinks, c.v_scale, self.out, stream=stream)


def test_two_streams_step_two_layers_concurrently():
    layers = [LayerStep(50, 0, 256), LayerStep(51, 300, 0)]
    alone = []
    for l in layers:
        l.step()
        torch.cuda.synchronize()
        alone.append(l.out.clone())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]            # default priority
    for rep in range(10):
        for l in layers:
            l.out.fill_(float("nan"))
        torch.cuda.synchronize()
        for _ in range(5):                                          # several steps queued on each stream
            for l, s in zip(layers, streams):
                l.step(stream=s)
        torch.cuda.synchronize()
        for l, want in zip(layers, alone):
            assert torch.equal(l.out, want), rep


def test_host_threads_call_the_library_concurrently():
    """Four host threads, each stepping its own layer on its own stream (ctypes releases the GIL during a call):
    the library's only shared state is an occupancy figure initialised once."""
    import threading
    layers = [LayerStep(60 + i, 0 if i % 2 == 0 else 200, 128 if i < 3 else 0) for i in range(4)]
    alone = []
    for l in layers:
        l.step()
        torch.cuda.synchronize()
        alone.append(l.out.clone())
        l.out.fill_(float("nan"))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in layers]
    errors = []

    def work(l, s):
        try:
            for _ in range(25):
                l.step(stream=s)
            s.synchronize()
        except Exception as e:                                       # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(l, s)) for l, s in zip(layers, streams)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for l, want in zip(layers, alone):
        assert torch.equal(l.out, want)
