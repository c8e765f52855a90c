"""kvra_chunk_attn_noalloc (the entry point for callers that cannot allocate) against kvra_chunk_attn,
through the C-ABI: same kernels and launch plan, so the outputs must be equal bit for bit; and against
the fp64 oracle at the usual bars.  Two calls in a row, the second on a smaller input, with nothing in
between that could refresh the shared scratch array."""
import numpy as np
import pytest

from oracle import kvra_oracle as orc
from paper_2405_05329_amd import synth

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3

# (H, Hkv, d, prefix, c): launches whose units are cut (few long units), large then small, then one that is not
SEQUENCE = [(32, 8, 128, 6000, 700), (32, 32, 128, 9000, 8), (8, 8, 64, 5000, 1), (4, 4, 128, 0, 300)]


def _prepare(kvra, torch, to_dev, case, seed):
    H, Hkv, d, prefix, c = case
    C = prefix + c
    q, k, v = synth.make_qkv(seed, 60, C, H, Hkv, d)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    kc = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    kvra.kvra_append_kv(dk, dv, dq, kc, vc, 0, C, C, H, Hkv, d, synth.ROPE_BASE)
    return dict(case=case, q=q, k=k, v=v, dq=dq[prefix:].contiguous(), kc=kc, vc=vc,
                scale=synth.default_scale(d))


def test_noalloc_equals_the_allocating_entry_point_two_calls_in_a_row():
    import torch
    from gpu_pipeline import to_dev, to_bits
    from paper_2405_05329_amd import kvra

    cus = torch.cuda.get_device_properties(0).multi_processor_count
    preps = [_prepare(kvra, torch, to_dev, case, seed) for seed, case in enumerate(SEQUENCE)]
    split = []
    for p in preps:
        H, Hkv, d, prefix, c = p["case"]
        plan = kvra.kvra_chunk_attn_plan(prefix, c, H, Hkv, d, cus)
        assert plan["scratch_bytes"] <= kvra.kvra_chunk_attn_noalloc_scratch_bytes()
        split.append(plan["partial_pieces"] > 0)
    assert split[:3] == [True, True, True] and not split[3], split   # the first three go through the scratch
    torch.cuda.synchronize()

    # the calls under test, back to back on one stream: large, smaller, smallest, unsplit
    outs_static = []
    for p in preps:
        H, Hkv, d, prefix, c = p["case"]
        out = torch.full((c, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        kvra.kvra_chunk_attn_noalloc(p["dq"], p["kc"], p["vc"], prefix, c, H, Hkv, d, p["scale"], out)
        outs_static.append(out)
    torch.cuda.synchronize()
    # again in reverse order (small before large) on the same, now used, array
    outs_static_rev = {}
    for i in reversed(range(len(preps))):
        p = preps[i]
        H, Hkv, d, prefix, c = p["case"]
        out = torch.full((c, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        kvra.kvra_chunk_attn_noalloc(p["dq"], p["kc"], p["vc"], prefix, c, H, Hkv, d, p["scale"], out)
        outs_static_rev[i] = out
    torch.cuda.synchronize()

    for i, p in enumerate(preps):
        H, Hkv, d, prefix, c = p["case"]
        ref = torch.full((c, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        kvra.kvra_chunk_attn(p["dq"], p["kc"], p["vc"], prefix, c, H, Hkv, d, p["scale"], ref)
        torch.cuda.synchronize()
        got, got_rev, want_bits = to_bits(outs_static[i]), to_bits(outs_static_rev[i]), to_bits(ref)
        np.testing.assert_array_equal(got, want_bits, err_msg=f"{p['case']}: differs from kvra_chunk_attn")
        np.testing.assert_array_equal(got_rev, want_bits, err_msg=f"{p['case']}: second pass differs")
        rows = list(range(prefix, prefix + c))
        want = orc.attention_rows(orc.bf16_bits_to_f64(p["q"]), orc.bf16_bits_to_f64(p["k"]),
                                  orc.bf16_bits_to_f64(p["v"]), rows, p["scale"], rope_base=synth.ROPE_BASE)
        err = np.abs(orc.bf16_bits_to_f64(got) - want)
        assert np.isfinite(orc.bf16_bits_to_f64(got)).all()
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (p["case"], err.max(), err.mean())


def test_noalloc_rejects_bad_arguments_before_any_launch():
    import torch
    from paper_2405_05329_amd import kvra
    t = torch.zeros((4, 2, 64), dtype=torch.bfloat16, device="cuda")
    assert kvra.kvra_chunk_attn_noalloc(None, t, t, 0, 4, 2, 2, 64, 0.125, t, check=False) == kvra.KVRA_EINVAL
    assert kvra.kvra_chunk_attn_noalloc(t, t, t, 0, 0, 2, 2, 64, 0.125, t, check=False) == kvra.KVRA_EINVAL
    assert kvra.kvra_chunk_attn_noalloc(t, t, t, 0, 4, 2, 2, 96, 0.125, t, check=False) == kvra.KVRA_EUNSUPPORTED
    assert kvra.kvra_chunk_attn_noalloc(t, t, t, 0, 4, 3, 2, 64, 0.125, t, check=False) == kvra.KVRA_EINVAL
    torch.cuda.synchronize()
