"""The attention calls of one block's denoising steps only enqueue kernels, so they can be
recorded into a HIP graph and replayed (Introduction, generate-and-cache loop: the same cache is
read by every step of a block, only the block's own Q/K/V change).  Every replay, with other eager
work and synchronisations in between, is checked against the eager call and the oracle."""
import numpy as np
import pytest
import torch

from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import OracleCacheF, assert_attention_close, oracle_rows, to_np_exact

pytestmark = pytest.mark.gpu


def test_attention_calls_replay_from_a_graph(gpu_device):
    dev = gpu_device
    L, H, D, n, cap = 2, 3, 128, 200, 3
    with ifx.KVCache(L, H, D, cap * n, n, ifx.IFX_BF16) as cache:
        ocs = [OracleCacheF(cap, torch.bfloat16) for _ in range(L)]
        for b in range(cap + 1):  # the rings have wrapped
            for layer in range(L):
                _, k, v = synth.draw_qkv(31, b, 0, layer, n, H, D, torch.bfloat16, dev, True)
                cache.commit(layer, k, v)
                ocs[layer].commit(k, v)
        # static buffers of the graph: the block's Q/K/V of both layers, and the outputs
        qs, ks, vs = ([torch.empty((n, H, D), dtype=torch.bfloat16, device=dev) for _ in range(L)] for _ in range(3))
        outs = [torch.empty((n, H, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
        lses = [torch.empty((n, H), dtype=torch.float32, device=dev) for _ in range(L)]
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        cache.profile(True)  # no sample is taken on a capturing stream, so this must not disturb the capture
        with torch.cuda.graph(graph, stream=side):
            s = torch.cuda.current_stream().cuda_stream
            cache.attention(0, qs[0], ks[0], vs[0], outs[0], s)
            cache.attention_blocks(1, qs[1], ks[1], vs[1], [2, 0], outs[1], lses[1], s)
        assert cache.profile_read()[1] == 0  # attention launches sampled so far: none
        cache.profile(False)
        rows, heads = np.repeat(np.arange(n), H), np.tile(np.arange(H), n)
        eager = torch.empty((n, H, D), dtype=torch.bfloat16, device=dev)
        for step in range(4):
            for layer in range(L):
                q, k, v = synth.draw_qkv(31, 100 + step, step, layer, n, H, D, torch.bfloat16, dev, True)
                qs[layer].copy_(q), ks[layer].copy_(k), vs[layer].copy_(v)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got0, got1 = outs[0].clone(), outs[1].clone()
            # eager work of the program's own between the replays, same inputs: identical bits (a
            # replayed call is the same single kernel launch on the same cache as the eager one)
            cache.attention(0, qs[0], ks[0], vs[0], eager)
            torch.cuda.synchronize()
            assert torch.equal(got0.view(torch.int16), eager.view(torch.int16)), step
            cache.attention_blocks(1, qs[1], ks[1], vs[1], [2, 0], eager)
            torch.cuda.synchronize()
            assert torch.equal(got1.view(torch.int16), eager.view(torch.int16)), step
            want = oracle_rows(qs[0], ks[0], vs[0], ocs[0], rows, heads)
            assert_attention_close(to_np_exact(got0)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, f"replay {step}")
            assert torch.isfinite(lses[1]).all()
