"""GPU-vs-oracle parity on inputs at the edges of what the entry points accept:
signed zeros through the matrix-core path, more (batch, kv head) segments than one
launch's grid holds, malformed outlier-channel lists, outliers large enough that
a difference of squared norms would cancel.  Through the C ABI; bars as in the
other parity tests (bits exact outside the near-zero band, norms 1e-3 relative).
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
DT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    assert os.path.exists(qjl.lib_path()), "libqjl.so must be built before the GPU tests run"
    qjl.lib()


def _dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


@pytest.mark.parametrize("dt,m", [("bf16", 256), ("bf16", 512), ("f16", 128), ("bf16", 1024), ("f32", 256)])
def test_signed_zero_keys(dt, m):
    """sign(0) := +1 whatever the zero's sign bit (Definition 3.1 with that reading): a key of -0.0 everywhere, and
    keys with +0.0 and -0.0 mixed, have every projection equal to zero, hence all code bits 1 and norm 0.  Keys with
    some -0.0 elements among ordinary ones are ordinary keys: their code is that of the key with +0.0 there."""
    say(f"[signed zeros] dt={dt} m={m}")
    d, n = 128, 130
    K = inputs.make_keys(1, 1, n, d, DT[dt], 91, DEV)
    K[0, 0, 0] = -0.0
    K[0, 0, 1] = 0.0
    K[0, 0, 1, ::2] = -0.0
    K[0, 0, 65] = -0.0
    K[0, 0, n - 1, 1::3] = -0.0
    K[0, 0, 7, :64] = -0.0                       # an ordinary key, half of its elements -0.0
    K[0, 0, 70, 5::7] = -0.0
    S = qjl.qjl_make_sketch(17, m, d, DT[dt], DEV)
    bits, norms = qjl.qjl_quantize_keys(K, S)
    bits, norms = bits.cpu().numpy(), norms.cpu().numpy()
    K64, S64 = inputs.to_f64(K), inputs.to_f64(S)
    assert np.signbit(K64[0, 0, 0]).all() and np.signbit(K64[0, 0, 1, ::2]).all()      # the zeros kept their sign
    ref_bits, ref_nu, P = orc.quantize_keys(K64, S64)
    for row in (0, 1, 65):
        assert np.all(ref_bits[0, 0, row] == 0xFF)                                    # the oracle's reading
        assert np.all(bits[0, 0, row] == 0xFF), (row, bits[0, 0, row])
        assert norms[0, 0, row] == 0
    diff = orc.unpack_signs(bits, m) != orc.unpack_signs(ref_bits, m)
    band = np.abs(P) < 1e-5 * np.linalg.norm(S64, axis=1) * np.linalg.norm(K64, axis=-1, keepdims=True)
    assert not (diff & ~band).any()
    assert np.all(np.abs(norms.astype(np.float64) - np.linalg.norm(K64, axis=-1)) <= 1e-3 * np.linalg.norm(K64, axis=-1))


def test_dual_quantize_with_more_segments_than_one_grid_dimension():
    """Two-part codes walk one segment per (batch, kv head); a grid dimension holds 65535 of them, so 65600 heads
    take two launches.  Sampled heads on both sides of the seam against the oracle; every head's norms against
    torch's."""
    B, Hkv, n, d, m, m_out, count = 2, 32800, 3, 128, 128, 128, 2
    say(f"[dual segments] {B * Hkv} (batch, kv head) segments of {n} keys")
    g = torch.Generator(device=DEV)
    g.manual_seed(4242)
    K = torch.randn((B, Hkv, n, d), generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    ch = torch.stack([torch.randperm(d, generator=g, device=DEV)[:count] for _ in range(64)])   # 64 channel lists, reused
    ch = ch[torch.arange(B * Hkv, device=DEV) % 64].reshape(B, Hkv, count).to(torch.int32).contiguous()
    S_in = qjl.qjl_make_sketch(61, m, d, torch.bfloat16, DEV)
    S_out = qjl.qjl_make_sketch(62, m_out, d, torch.bfloat16, DEV)
    # (the stacked-sketch call takes at most 65535 heads at a time)
    S_dual = torch.cat([qjl.qjl_make_dual_sketch(S_in, S_out, ch[b:b + 1].contiguous()) for b in range(B)])
    bits, nu_in, nu_out = qjl.qjl_quantize_keys_dual(K, S_dual, ch, m_out)
    torch.cuda.synchronize()
    # every head: norms of the two parts
    mask = torch.zeros((B, Hkv, 1, d), dtype=torch.bool, device=DEV)
    mask.scatter_(3, ch.long()[:, :, None, :], True)
    Kf = K.float()
    ref_out = (Kf * mask).norm(dim=-1)
    ref_in = (Kf * ~mask).norm(dim=-1)
    assert torch.all((nu_in.float() - ref_in).abs() <= 1e-3 * ref_in)
    assert torch.all((nu_out.float() - ref_out).abs() <= 1e-3 * ref_out)
    # sampled heads, the seam between the two launches among them: codes against the oracle
    S_in64, S_out64 = inputs.to_f64(S_in), inputs.to_f64(S_out)
    flat = [0, 1, 63, 64, 32799, 32800, 65533, 65534, 65535, 65536, 65537, 65599]
    bad = 0
    for u in flat:
        b, h = divmod(u, Hkv)
        K64 = inputs.to_f64(K[b, h])[None, None]
        c = ch[b, h].cpu().numpy()[None, None]
        rb, ri, ro, P_in, P_out = orc.quantize_keys_dual(K64, S_in64, S_out64, c)
        got = bits[b, h].cpu().numpy()[None, None]
        K_in, K_out = orc.split_channels(K64, c)
        cm = np.zeros(d); cm[c[0, 0]] = 1.0
        for lo, mm, P, Sm, Kp in ((0, m, P_in, S_in64 * (1 - cm), K_in), (m // 8, m_out, P_out, S_out64 * cm, K_out)):
            diff = orc.unpack_signs(got[..., lo:lo + mm // 8], mm) != orc.unpack_signs(rb[..., lo:lo + mm // 8], mm)
            band = np.abs(P) < 1e-5 * np.linalg.norm(Sm, axis=1) * np.linalg.norm(Kp, axis=-1, keepdims=True)
            bad += int((diff & ~band).sum())
    say(f"  {len(flat)} sampled heads: {bad} code bits differ outside the near-zero band")
    assert bad == 0


@pytest.mark.parametrize("dt,n,m,m_out", [("bf16", 200, 256, 128), ("f16", 77, 128, 128), ("bf16", 70, 512, 512),
                                          ("f32", 50, 256, 128)])
def test_dual_channel_list_with_repeats_and_entries_out_of_range(dt, n, m, m_out):
    """One rule on every path: a channel listed twice counts once, an entry outside [0, d) is ignored.  The list
    (5, 130, 5, -1, 77) therefore means the channels {5, 77}."""
    say(f"[dual channel list] dt={dt} n={n} m={m}+{m_out}")
    B, Hkv, d = 1, 2, 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 800 + n, DEV, outliers=0)
    K[..., 5] *= 15
    K[..., 77] *= 15
    raw = np.array([[[5, 130, 5, -1, 77], [77, 77, 77, 5, 1000]]])
    clean = np.array([[[5, 77], [5, 77]]])
    S_in = qjl.qjl_make_sketch(71, m, d, DT[dt], DEV)
    S_out = qjl.qjl_make_sketch(72, m_out, d, DT[dt], DEV)
    S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, _dev_i32(raw))
    assert torch.equal(S_dual, qjl.qjl_make_dual_sketch(S_in, S_out, _dev_i32(clean)))
    bits, nu_in, nu_out = qjl.qjl_quantize_keys_dual(K, S_dual, _dev_i32(raw), m_out)
    b2, i2, o2 = qjl.qjl_quantize_keys_dual(K, S_dual, _dev_i32(clean), m_out)
    assert torch.equal(bits, b2) and torch.equal(nu_in, i2) and torch.equal(nu_out, o2)
    K64 = inputs.to_f64(K)
    K_in, K_out = orc.split_channels(K64, clean)
    for got, ref in ((nu_in, np.linalg.norm(K_in, axis=-1)), (nu_out, np.linalg.norm(K_out, axis=-1))):
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - ref) <= 1e-3 * ref)


@pytest.mark.parametrize("dt,m,m_out", [("bf16", 256, 128), ("bf16", 512, 512), ("f32", 256, 128)])
def test_dual_norms_with_dominant_outliers(dt, m, m_out):
    """Outlier channels 300 times the rest: ||k||^2 is about 3.6e5 times the inlier part, so an inlier norm taken as
    sqrt(||k||^2 - ||k_out||^2) in float32 would be off by percents; each part is summed on its own instead."""
    say(f"[dual dominant outliers] dt={dt} m={m}+{m_out}")
    B, Hkv, n, d = 1, 2, 300, 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 900, DEV, outliers=4, outlier_scale=300.0)
    K64 = inputs.to_f64(K)
    ch = orc.select_outlier_channels(K64, 4)
    S_in = qjl.qjl_make_sketch(81, m, d, DT[dt], DEV)
    S_out = qjl.qjl_make_sketch(82, m_out, d, DT[dt], DEV)
    S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, _dev_i32(ch))
    bits, nu_in, nu_out = qjl.qjl_quantize_keys_dual(K, S_dual, _dev_i32(ch), m_out)
    K_in, K_out = orc.split_channels(K64, ch)
    ref_in, ref_out = np.linalg.norm(K_in, axis=-1), np.linalg.norm(K_out, axis=-1)
    e_in = float(np.max(np.abs(nu_in.cpu().numpy().astype(np.float64) - ref_in) / ref_in))
    e_out = float(np.max(np.abs(nu_out.cpu().numpy().astype(np.float64) - ref_out) / ref_out))
    say(f"  worst relative error: inlier norm {e_in:.2e}, outlier norm {e_out:.2e}")
    assert e_in <= 1e-3 and e_out <= 1e-3
    rb, _, _, _, _ = orc.quantize_keys_dual(K64, inputs.to_f64(S_in), inputs.to_f64(S_out), ch)
    assert float(np.mean(bits.cpu().numpy() != rb)) < 1e-3          # near-zero projections may differ
