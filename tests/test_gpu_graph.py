"""The hot calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
caller can capture them in a HIP graph: decode attention captured once and replayed with new queries in the same
buffers, every replay compared with the eager call, with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2507_20030_amd import binding as B
from paper_2507_20030_amd import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,cfg", [
    ("fft", wl.Config("g_fft", 2, 2, 2, 4, 128, 1024, 200, 4, "bf16", "mixed", n_sink=3, n_recent=5, seed=21)),
    ("chirp", wl.Config("g_chirp", 1, 2, 2, 2, 128, 1000, 150, 4, "f32", "low", seed=22)),
    # long context with many slices: kernels A and B pipelined over groups of slices (10 launches per call)
    ("pipelined", wl.Config("g_pipe", 16, 8, 8, 4, 128, 16384, 1100, 4, "bf16", "mixed", seed=23)),
])
def test_decode_attention_in_a_captured_graph(name, cfg):
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype,
                    cfg.L, bins, device=DEV, n_sink=cfg.n_sink, n_recent=cfg.n_recent)
    assert B.iwdft_attn_kind(cache.ctx) == ("chirp" if name == "chirp" else "fft")
    assert B.iwdft_attn_pipelined(cache.ctx) == (name == "pipelined")
    cache.prefill(K, V)
    for i in range(2):
        tk, tv, _ = wl.decode_step(cfg, i, DEV)
        cache.append(tk, tv)
    qs = [wl.decode_step(cfg, 10 + i, DEV)[2] for i in range(4)]
    q_buf, out_buf = qs[0].clone(), torch.empty_like(qs[0])
    cache.attend(q_buf, out_buf)                      # eager once: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cache.attend(q_buf, out_buf, 0.0, torch.cuda.current_stream())
    for i, q in enumerate(qs):
        ref = cache.attend(q).clone()                 # eager work between the replays
        torch.cuda.synchronize()
        q_buf.copy_(q)
        out_buf.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_buf, ref), f"{name}: replay {i} differs from the eager call"
    cache.close()
