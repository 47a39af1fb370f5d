"""Small batches are replayed from captured HIP graphs (wf_encoder_set_graphs): every replay must be
bit-identical to the kernel-by-kernel launch of the same batch, also with the program's own eager work
and synchronisations between the replays, with new data in the same input buffer, after other batches
went through the same encoder, and after the cache evicted and re-captured an entry."""
import numpy as np
import pytest

from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _setup(name, slack_frames=0):
    import torch
    wl, w, hush, mels = H.inputs(name)
    enc = wf.encoder_for_workload(wl, w, hush, wf.WF_PRECISION_BF16)
    flat, offs, nf = wf.pack_mels(mels)
    mel = torch.from_numpy(flat).cuda()
    M = wf.plan_batch(enc.cfg, nf)[2]
    return wl, enc, mel, offs, nf, M


@pytest.mark.parametrize("name", ["cfg1", "tiny-ragged", "cfg2-4s"])
def test_every_replay_equals_the_eager_result(name):
    import torch
    wl, enc, mel, offs, nf, M = _setup(name)
    try:
        out = torch.empty((M, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
        enc.set_graphs(False)
        enc.encode(mel, offs, nf, out=out)
        torch.cuda.synchronize()
        eager = out.clone()
        assert enc.graph_stats() == {"replays": 0, "captures": 0, "direct_calls": 1}
        enc.set_graphs(True)
        scratch = torch.empty(1 << 20, device="cuda")
        for it in range(6):                      # call 0 launches directly, call 1 captures and replays, 2.. replay
            out.fill_(float("nan"))
            enc.encode(mel, offs, nf, out=out)
            scratch.normal_()                    # eager work of the program between the replays
            s = float(scratch.sum())             # a library reduction and a host synchronisation
            assert np.isfinite(s)
            torch.cuda.synchronize()
            assert torch.equal(out, eager), it
        st = enc.graph_stats()
        assert st["captures"] == 1 and st["replays"] == 5 and st["direct_calls"] == 2
        # new data in the same buffer: the replay reads it (nothing of the input is baked into the graph)
        mel2 = (mel * 0.5 - 0.1).contiguous()
        enc.set_graphs(False)
        ref2 = torch.empty_like(out)
        tmp = mel.clone()
        mel.copy_(mel2)
        enc.encode(mel, offs, nf, out=ref2)
        torch.cuda.synchronize()
        assert not torch.equal(ref2, eager)
        enc.set_graphs(True)
        enc.encode(mel, offs, nf, out=out)
        torch.cuda.synchronize()
        assert torch.equal(out, ref2)
        assert enc.graph_stats()["replays"] == 6
        mel.copy_(tmp)
        # a different output buffer or different offsets are different keys: direct launch, same values
        out_b = torch.empty_like(out)
        enc.encode(mel, offs, nf, out=out_b)
        torch.cuda.synchronize()
        assert torch.equal(out_b, eager)
        assert enc.graph_stats()["captures"] == 1
    finally:
        enc.close()


def test_other_batches_between_replays_and_cache_eviction():
    """One encoder, many different single-stream lengths (what successive rounds of one stream look like): each
    length seen twice is captured; more than 64 distinct keys evict the least recently used; an evicted key is
    captured again later; every result equals the eager one."""
    import torch
    wl = synth.workload("cfg1")
    w, hush, _ = synth.materialize(wl)
    T_max = 400
    cfg = wf.make_config(wl.shape, wl.hush_frames, 1, T_max + wl.hush_frames, T_max + wl.hush_frames, wf.WF_PRECISION_BF16)
    enc = wf.Encoder(cfg, w, hush)
    rng = np.random.default_rng(11)
    mel = torch.from_numpy(np.clip(rng.normal(-0.3, 0.4, size=(T_max, wl.shape.n_mels)), -1, 1).astype(np.float32)).cuda()
    out = torch.empty(((T_max + wl.hush_frames + 1) // 2, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
    try:
        lengths = list(range(100, 100 + 70))                       # 70 keys > 64 cache entries
        enc.set_graphs(False)
        eager = {}
        for T in lengths:
            enc.encode(mel, [0], [T], out=out)
            torch.cuda.synchronize()
            eager[T] = out[:(T + wl.hush_frames + 1) // 2].clone()
        enc.set_graphs(True)
        base = enc.graph_stats()
        for T in lengths:                                          # first sighting of each: direct
            enc.encode(mel, [0], [T], out=out)
        torch.cuda.synchronize()
        assert enc.graph_stats()["captures"] == 0
        for rep in range(2):
            for T in lengths[-40:]:                                # second sighting: capture; third: replay
                out.fill_(float("nan"))
                enc.encode(mel, [0], [T], out=out)
                torch.cuda.synchronize()
                assert torch.equal(out[:eager[T].shape[0]], eager[T]), (rep, T)
        st = enc.graph_stats()
        assert st["captures"] == 40 and st["replays"] == 80
        for T in lengths[:30]:                                     # these keys were evicted by now: direct again, then capture
            for _ in range(2):
                out.fill_(float("nan"))
                enc.encode(mel, [0], [T], out=out)
                torch.cuda.synchronize()
                assert torch.equal(out[:eager[T].shape[0]], eager[T]), T
        assert enc.graph_stats()["captures"] == 70                 # the 30 new ones; six captured graphs were evicted for them
        for T in lengths[30:36] + lengths[-5:]:                    # evicted graphs are captured again, surviving ones replayed
            out.fill_(float("nan"))
            enc.encode(mel, [0], [T], out=out)
            enc.encode(mel, [0], [T], out=out)
            torch.cuda.synchronize()
            assert torch.equal(out[:eager[T].shape[0]], eager[T]), T
        assert enc.graph_stats()["direct_calls"] > base["direct_calls"]
    finally:
        enc.close()


def test_replay_is_opt_in_and_profiled_calls_are_never_replayed():
    import torch
    wl, enc, mel, offs, nf, M = _setup("cfg3")                     # 4951 tokens: one lane, so it is replayed
    try:
        out = torch.empty((M, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
        for _ in range(3):                                         # replay is opt-in: nothing is captured by default
            enc.encode(mel, offs, nf, out=out)
        torch.cuda.synchronize()
        assert enc.graph_stats() == {"replays": 0, "captures": 0, "direct_calls": 3}
        enc.set_graphs(True)
        for _ in range(3):
            enc.encode(mel, offs, nf, out=out)
        torch.cuda.synchronize()
        a = out.clone()
        assert enc.graph_stats()["replays"] == 2
        enc.set_profiling(True)                                    # per-kernel events need real launches
        enc.encode(mel, offs, nf, out=out)
        torch.cuda.synchronize()
        assert sum(s["launches"] for s in enc.kernel_stats()) == 4 + 7 * wl.shape.n_layers   # prep, two convolutions, 7 per block (4951 tokens: separate LayerNorm kernels), final LayerNorm
        enc.set_profiling(False)
        assert torch.equal(out, a)
        assert enc.graph_stats()["replays"] == 2
    finally:
        enc.close()
