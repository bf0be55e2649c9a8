"""Encode + decode captured once into a HIP graph and replayed, the way a serving loop would run them.

Every replay, with the program's own eager work (new input copied in, outputs overwritten) and a
synchronisation between the replays, must give byte for byte what the oracle gives for the input that is
in the buffer at that moment.  Covers one shape per encoder family, through `slicer_encode` (caller's
workspace) and through `slicer_encode_static` (the entry point that allocates nothing).
"""
import numpy as np
import pytest

from paper_2511_11608_amd import synth

pytestmark = pytest.mark.gpu

SHAPES = {
    "llm": lambda seed: synth.llm_prefill(seed=seed, rows=300),                      # one wavefront per row, two finishing launches
    "vit": lambda seed: synth.vit_tokens(seed=seed, rows=200),                       # fp32 rows, one finishing launch
    "ar_step": lambda seed: synth.ar_decode_step(seed=seed, step=seed, rows=64),     # one workgroup per row
    "resnet_2rows": lambda seed: synth.resnet_stage3(seed=seed, rows=2),             # long-row stages
}


@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("name", list(SHAPES))
def test_graph_replays_match_the_oracle(oracle, name, static):
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device, to_host
    wls = [SHAPES[name](seed) for seed in (11, 12)]
    wl = wls[0]
    x = to_device(wl.x, wl.dtype)                       # the graph's input buffer
    sb, meta, ws = binding.alloc_buffers(x, wl.keep_ratio, wl.n_blocks, wl.bit_set)
    y = torch.empty_like(x)

    def step():
        if static:
            binding.slicer_encode_static(x, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, sb, meta)
        else:
            binding.slicer_encode(x, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, sb, meta, ws)
        binding.slicer_decode_as(sb, meta, y, wl.n_blocks)

    step()                                              # first use outside the capture (per-device set-up of the library)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    view = np.uint32 if wl.dtype == "f32" else np.uint16
    for it in (1, 0, 1, 1):
        cur = wls[it]
        x.copy_(to_device(cur.x, cur.dtype))            # eager work between the replays
        sb.fill_(-1)
        meta.fill_(0xFF)
        y.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        s_ref, m_ref = oracle.encode(cur.x, cur.dtype, cur.keep_ratio, cur.n_blocks, cur.bit_set, cur.budget, n_threads=8)
        y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
        words = binding.slicer_stream_words(meta)
        assert np.array_equal(m_ref, meta.cpu().numpy()), (name, static, it)
        assert np.array_equal(s_ref, sb[:words].cpu().numpy().view(np.uint32)), (name, static, it)
        assert np.array_equal(y_ref.view(view), to_host(y).view(view)), (name, static, it)
