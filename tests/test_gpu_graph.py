"""The library under HIP graph capture.

Every entry point is asynchronous on the caller's stream and, once the scratch buffer of
kvra_chunk_attn exists (it is allocated on the first call on a device), allocates nothing: a whole
chunk sequence then records into a graph.  Each replay has to reproduce the eager result bit for
bit (the kernels are deterministic); eager work and synchronisations run between the replays.
"""
import numpy as np
import pytest
import torch

from paper_2405_05329_amd import kvra, synth

pytestmark = pytest.mark.gpu


def _sequence(q, q_master, k_in, v_in, k_cache, v_cache, out, bounds, H, Hkv, d, scale, stream):
    with torch.cuda.stream(stream):
        q.copy_(q_master)            # append rotates Q in place: start every run from the master copy
    C = bounds[-1]
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        kvra.kvra_append_kv(k_in[lo:hi], v_in[lo:hi], q[lo:hi], k_cache, v_cache, lo, hi - lo, C,
                            H, Hkv, d, synth.ROPE_BASE, stream=stream)
        kvra.kvra_chunk_attn(q[lo:hi], k_cache, v_cache, lo, hi - lo, H, Hkv, d, scale, out[lo:hi],
                             stream=stream)


@pytest.mark.parametrize("H,Hkv,d,bounds", [
    (8, 8, 128, [0, 2400, 2700, 3000]),      # chunks 1 and 2: 16 units behind 2400+ keys -> cut units, merged in the kernel
    (8, 2, 64, [0, 1111, 1500]),
])
def test_chunk_sequence_replays_from_a_graph(H, Hkv, d, bounds):
    from gpu_pipeline import to_dev, to_bits
    C = bounds[-1]
    qb, kb, vb = synth.make_qkv(3, 90, C, H, Hkv, d)
    q_master, k_in, v_in = to_dev(qb), to_dev(kb), to_dev(vb)
    q = torch.empty_like(q_master)
    k_cache = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros_like(k_cache)
    out = torch.zeros((C, H, d), dtype=torch.bfloat16, device="cuda")
    scale = synth.default_scale(d)
    args = (q, q_master, k_in, v_in, k_cache, v_cache, out, bounds, H, Hkv, d, scale)

    # eager run: the expected bits, and the warm-up that allocates the scratch
    _sequence(*args, torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = {name: to_bits(t).copy() for name, t in (("out", out), ("k", k_cache), ("v", v_cache), ("q", q))}

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        _sequence(*args, torch.cuda.current_stream())

    scratch_q = torch.empty_like(q_master)
    for replay in range(3):
        for t in (out, k_cache, v_cache, q):
            t.zero_()
        # unrelated eager work of the program between the replays
        kvra.kvra_append_kv(k_in[:64], v_in[:64], scratch_q[:64], torch.zeros_like(k_cache), torch.zeros_like(v_cache),
                            0, 64, C, H, Hkv, d, synth.ROPE_BASE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in (("out", out), ("k", k_cache), ("v", v_cache), ("q", q)):
            np.testing.assert_array_equal(to_bits(t), want[name], err_msg=f"replay {replay}: {name}")
