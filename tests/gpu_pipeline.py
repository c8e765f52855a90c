"""Test-side driver of the HIP path: moves bf16 bit patterns to the GPU, runs the chunks of a
partition through the C-ABI (append, then attention) and brings bit patterns back."""
import numpy as np
import torch

from paper_2405_05329_amd import kvra


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_chunked(qbits, kbits, vbits, boundaries, scale, rope_base, capacity=None, sentinel=0x7FC0):
    """Returns dict(out, k_cache, v_cache, q_rot) of uint16 arrays.  Caches start filled with
    `sentinel` (a bf16 NaN pattern) so that reads of rows that were never written show up."""
    C, H, d = qbits.shape
    Hkv = kbits.shape[1]
    cap = capacity or C
    dev_q = to_dev(qbits)
    dev_k = to_dev(kbits)
    dev_v = to_dev(vbits)
    fill = np.full((cap, Hkv, d), sentinel, dtype=np.uint16)
    k_cache = to_dev(fill)
    v_cache = to_dev(fill)
    out = torch.zeros((C, H, d), dtype=torch.bfloat16, device="cuda")
    b = [int(x) for x in boundaries]
    for i in range(len(b) - 1):
        lo, hi = b[i], b[i + 1]
        kvra.kvra_append_kv(dev_k[lo:hi], dev_v[lo:hi], dev_q[lo:hi], k_cache, v_cache, lo, hi - lo, cap,
                            H, Hkv, d, rope_base if rope_base is not None else 0.0)
        kvra.kvra_chunk_attn(dev_q[lo:hi], k_cache, v_cache, lo, hi - lo, H, Hkv, d, scale, out[lo:hi])
    torch.cuda.synchronize()
    return dict(out=to_bits(out), k_cache=to_bits(k_cache), v_cache=to_bits(v_cache), q_rot=to_bits(dev_q))
