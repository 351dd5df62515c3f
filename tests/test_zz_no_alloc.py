"""The allocation-free decode entry point against the ordinary one, through the C ABI.

qjl_decode_attention_noalloc keeps its per-chunk records in a device array
inside the library instead of a caller's workspace.  Same kernels, same plan:
the outputs must agree to the attention bar (2e-3 absolute; in fact to the
bit), and with the oracle, on two calls in a row, the second on a smaller
input, so that whatever the first call left in the array is there when the
second runs.
"""
import os

import numpy as np
import pytest
import torch

import paper_2406_03482_amd as qjl
from paper_2406_03482_amd import inputs
from oracle import qjl_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(B, Hq, Hkv, n, m, seed):
    d, scale = 128, 128 ** -0.5
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, seed, DEV)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, seed + 1, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, seed + 2, DEV)
    S = qjl.qjl_make_sketch(seed + 3, m, d, torch.bfloat16, DEV)
    K64, S64 = inputs.to_f64(K), inputs.to_f64(S)
    bits, nu16, _ = orc.quantize_keys(K64, S64)
    ref = orc.decode_attention(inputs.to_f64(Q), S64, bits, nu16, inputs.to_f64(V), scale)
    return dict(Q=Q, S=S, bits=torch.from_numpy(bits).to(DEV), norms=torch.from_numpy(nu16).to(DEV), V=V,
                scale=scale, ref=ref, out=torch.empty((B, Hq, d), dtype=torch.float32, device=DEV))


def test_noalloc_entry_point_matches_the_workspace_one_twice_in_a_row():
    assert torch.cuda.is_available() and os.path.exists(qjl.lib_path())
    L = qjl.lib()
    assert L.qjl_decode_noalloc_max_bytes() == 4 << 20
    big = _case(2, 8, 2, 20000, 256, 7001)          # GQA x4, many chunks
    small = _case(1, 4, 4, 700, 256, 7101)          # fewer heads, fewer chunks, ragged
    for name, c in (("first call", big), ("second, smaller call", small)):
        print(f"[noalloc] {name}: Q {tuple(c['Q'].shape)} n={c['V'].shape[2]}", flush=True)
        want = qjl.qjl_decode_attention(c["Q"], c["S"], c["bits"], c["norms"], c["V"], c["scale"])
        before = torch.cuda.memory_allocated()
        got = qjl.qjl_decode_attention_noalloc(c["Q"], c["S"], c["bits"], c["norms"], c["V"], c["scale"], c["out"])
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before       # nothing came from torch's allocator either
        g, w = got.cpu().numpy().astype(np.float64), want.cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - w))) <= 2e-3
        assert torch.equal(got, want)                        # same kernels, same plan, same summation order
        assert float(np.max(np.abs(g - c["ref"]))) <= 2e-3   # and the oracle
    # once more on the first input: the array now holds the smaller call's records
    got = qjl.qjl_decode_attention_noalloc(big["Q"], big["S"], big["bits"], big["norms"], big["V"], big["scale"], big["out"])
    assert float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - big["ref"]))) <= 2e-3


def test_noalloc_entry_point_rejects_what_its_array_cannot_hold():
    """B * Hq * chunks records of 528 bytes must fit 4 MiB: 8192 query heads of 4096 keys need at least 8192."""
    L = qjl.lib()
    sh = qjl.QJLShape(256, 32, 32, 4096, 128, 256, qjl.QJL_BF16, 1.0)
    assert L.qjl_decode_workspace_bytes(sh) > L.qjl_decode_noalloc_max_bytes()
    x = torch.zeros(64, dtype=torch.uint8, device=DEV)       # never read: the size check comes before any launch
    rc = L.qjl_decode_attention_noalloc(sh, x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(),
                                        x.data_ptr(), None)
    assert rc == -3
