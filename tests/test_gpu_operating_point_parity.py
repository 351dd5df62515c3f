"""GPU-vs-oracle parity of the paper's operating point as one path (Section 4.1 two-part key codes + Section 3.2
quantized values + Algorithm 1's stream), through the C ABI: qjl_decode_attention_dual_vq and
qjl_generation_step.  Bars as everywhere: attention 2e-3 absolute, code bits exact outside the near-zero band,
norms 1e-3 relative, value codes bit-identical to the oracle's.  The oracle builds every cache that the GPU
reads; the GPU's own writes (the new token's row) are compared with the oracle's."""
import os

import numpy as np
import pytest
import torch

import paper_2406_03482_amd as qjl
from paper_2406_03482_amd import inputs
from oracle import qjl_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda"
DT = {"bf16": torch.bfloat16, "f16": torch.float16}


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    assert os.path.exists(qjl.lib_path()), "libqjl.so must be built before the GPU tests run"
    qjl.lib()


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _problem(dt, B, Hq, Hkv, n, m, m_out, seed, count=4):
    d = 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], seed, DEV, outliers=4)
    Q = inputs.make_normal((B, Hq, d), DT[dt], seed + 1, DEV)
    V = inputs.make_normal((B, Hkv, n, d), DT[dt], seed + 2, DEV)
    S_in = qjl.qjl_make_sketch(seed + 3, m, d, DT[dt], DEV)
    S_out = qjl.qjl_make_sketch(seed + 4, m_out, d, DT[dt], DEV)
    K64 = inputs.to_f64(K)
    ch = orc.select_outlier_channels(K64, count)
    S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, _dev(ch.astype(np.int32)))
    return dict(K=K, Q=Q, V=V, S_in=S_in, S_out=S_out, S_dual=S_dual, ch=ch, K64=K64, Q64=inputs.to_f64(Q),
                V64=inputs.to_f64(V), S_in64=inputs.to_f64(S_in), S_out64=inputs.to_f64(S_out))


DUAL_VQ_CASES = [
    # dtype, B, Hq, Hkv, n, m, m_out, vbits, scale
    ("bf16", 2, 4, 4, 1000, 256, 128, 4, 0.0884),     # MHA, 384-bit codes + 4-bit values: 3 bits per key coordinate
    ("bf16", 1, 8, 2, 1500, 128, 128, 4, 0.0884),     # GQA x4 on 256-bit codes
    ("bf16", 1, 8, 2, 700, 256, 128, 2, 0.0884),      # GQA x4 on 384-bit codes -> two heads at a time, 2-bit values
    ("f16", 1, 6, 3, 333, 256, 128, 8, 1.0),          # GQA x2, 8-bit values, the paper's literal scale
    ("bf16", 1, 3, 1, 260, 256, 128, 4, 0.0884),      # GQA x3 -> one head at a time
    ("bf16", 1, 2, 2, 1, 256, 128, 4, 1.0),           # n = 1
    ("bf16", 1, 2, 1, 20000, 256, 128, 4, 0.0884),    # many chunks
]


@pytest.mark.parametrize("dt,B,Hq,Hkv,n,m,m_out,vbits,scale", DUAL_VQ_CASES)
def test_decode_attention_dual_vq_parity(dt, B, Hq, Hkv, n, m, m_out, vbits, scale):
    say(f"[decode dual+vq] dt={dt} B={B} Hq={Hq} Hkv={Hkv} n={n} m={m}+{m_out} vbits={vbits} scale={scale}")
    p = _problem(dt, B, Hq, Hkv, n, m, m_out, 900 + n)
    bits, nu_in, nu_out, _, _ = orc.quantize_keys_dual(p["K64"], p["S_in64"], p["S_out64"], p["ch"])
    vc, vs, vz = orc.quantize_values(p["V64"], vbits)
    ref = orc.decode_attention_dual_vq(p["Q64"], p["S_in64"], p["S_out64"], p["ch"], bits, nu_in, nu_out, vc, vs, vz, vbits, scale)
    args = (p["Q"], p["S_dual"], _dev(bits), _dev(nu_in), _dev(nu_out), _dev(vc), _dev(vs), _dev(vz), m_out, vbits, scale)
    out = qjl.qjl_decode_attention_dual_vq(*args)
    err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))
    say(f"  max abs error {err:.3g}")
    assert err <= 2e-3
    assert torch.equal(out, qjl.qjl_decode_attention_dual_vq(*args))


STEP_CASES = [
    # dtype, B, Hq, Hkv, cap, m, m_out, vbits, positions
    ("bf16", 1, 4, 4, 700, 256, 128, 4, [0, 1, 63, 64, 65, 300, 511, 512, 699]),
    ("bf16", 2, 8, 2, 1100, 128, 128, 4, [0, 5, 255, 256, 1023, 1024, 1099]),      # GQA x4
    ("f16", 1, 8, 2, 600, 256, 128, 2, [0, 77, 511, 599]),                         # two heads at a time, 2-bit values
    ("bf16", 1, 3, 1, 300, 256, 128, 8, [0, 128, 299]),
    ("bf16", 1, 2, 1, 9000, 256, 128, 4, [4095, 4096, 8999]),                      # several chunks: the new row sits in the last one
]


@pytest.mark.parametrize("dt,B,Hq,Hkv,cap,m,m_out,vbits,positions", STEP_CASES)
def test_generation_step_parity(dt, B, Hq, Hkv, cap, m, m_out, vbits, positions):
    """Each step starts from the oracle's caches for rows 0..pos-1 (stale bytes behind them), appends the token of
    position pos on both sides and compares the attention output and the row that the GPU wrote."""
    say(f"[generation step] dt={dt} B={B} Hq={Hq} Hkv={Hkv} cap={cap} m={m}+{m_out} vbits={vbits}")
    d, scale = 128, 0.0884
    p = _problem(dt, B, Hq, Hkv, cap, m, m_out, 1300 + cap)
    ob, oi, oo, P_in, P_out = orc.quantize_keys_dual(p["K64"], p["S_in64"], p["S_out64"], p["ch"])
    oc, os_, oz = orc.quantize_values(p["V64"], vbits)
    K_in, K_out = orc.split_channels(p["K64"], p["ch"])
    ch_d = _dev(p["ch"].astype(np.int32))
    rng = np.random.default_rng(cap)
    flips = 0
    for pos in positions:
        caches = [np.ascontiguousarray(x.copy()) for x in (ob, oi, oo, oc, os_, oz)]
        for x in caches:                                               # rows pos.. hold stale contents
            x[:, :, pos:] = rng.integers(1, 120, size=x[:, :, pos:].shape).astype(x.dtype)
        ref_caches = [x.copy() for x in caches]
        Qs = inputs.make_normal((B, Hq, d), DT[dt], 5000 + pos, DEV)
        ref = orc.generation_step(inputs.to_f64(Qs), p["S_in64"], p["S_out64"], p["ch"], *ref_caches,
                                  p["K64"][:, :, pos:pos + 1], p["V64"][:, :, pos:pos + 1], pos, vbits, scale)
        dc = [_dev(x) for x in caches]
        out = qjl.qjl_generation_step(Qs, p["K"][:, :, pos:pos + 1].contiguous(), p["V"][:, :, pos:pos + 1].contiguous(),
                                      p["S_dual"], ch_d, *dc, pos, m_out, vbits, scale)
        torch.cuda.synchronize()
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))
        assert err <= 2e-3, (pos, err)
        got = [x.cpu().numpy() for x in dc]
        for g, c0 in zip(got, caches):                                 # only row pos was written
            assert np.array_equal(g[:, :, :pos], c0[:, :, :pos]) and np.array_equal(g[:, :, pos + 1:], c0[:, :, pos + 1:])
        # the new row: value codes, scale and zero point are the oracle's; key code bits exact outside the band
        assert np.array_equal(got[3][:, :, pos], oc[:, :, pos])
        assert np.array_equal(got[4][:, :, pos], os_[:, :, pos]) and np.array_equal(got[5][:, :, pos], oz[:, :, pos])
        for lo, mm, P, S64, Kp, is_out in ((0, m, P_in, p["S_in64"], K_in, False), (m // 8, m_out, P_out, p["S_out64"], K_out, True)):
            diff = orc.unpack_signs(got[0][:, :, pos:pos + 1, lo:lo + mm // 8], mm) != orc.unpack_signs(ob[:, :, pos:pos + 1, lo:lo + mm // 8], mm)
            for b in range(B):
                for h in range(Hkv):
                    mask = np.zeros(d); mask[p["ch"][b, h]] = 1.0
                    Sm = S64 * (mask if is_out else 1 - mask)
                    band = np.abs(P[b, h, pos]) < 1e-5 * np.linalg.norm(Sm, axis=1) * np.linalg.norm(Kp[b, h, pos])
                    assert not (diff[b, h, 0] & ~band).any(), (pos, b, h)
                    flips += int((diff[b, h, 0] & band).sum())
        for g16, Kp in ((got[1], K_in), (got[2], K_out)):
            refn = np.linalg.norm(Kp[:, :, pos], axis=-1)
            assert np.all(np.abs(g16[:, :, pos].astype(np.float64) - refn) <= 1e-3 * refn)
    say(f"  {len(positions)} steps, {flips} near-zero sign flips in the appended rows")


def test_generation_steps_stream_into_the_caches():
    """Forty consecutive steps on the GPU alone (each step reads what the steps before wrote), against the oracle's
    own stream; and the caches end up as the bulk quantizers would have written them."""
    dt, B, Hq, Hkv, cap, m, m_out, vbits, scale = "bf16", 1, 8, 2, 300, 256, 128, 4, 0.0884
    p = _problem(dt, B, Hq, Hkv, cap, m, m_out, 1717)
    say("[generation stream] 40 steps from position 240")
    start, steps = 240, 40
    ob, oi, oo, _, _ = orc.quantize_keys_dual(p["K64"][:, :, :start], p["S_in64"], p["S_out64"], p["ch"])
    oc, os_, oz = orc.quantize_values(p["V64"][:, :, :start], vbits)
    shapes = [((m + m_out) // 8, np.uint8), (None, np.float16), (None, np.float16), (128 * vbits // 8, np.uint8), (None, np.float16), (None, np.float16)]
    host = []
    for (last, tp), first in zip(shapes, (ob, oi, oo, oc, os_, oz)):
        full = np.zeros((B, Hkv, cap) + ((last,) if last else ()), dtype=tp)
        full[:, :, :start] = first
        host.append(full)
    ref_caches = [x.copy() for x in host]
    dc = [_dev(x) for x in host]
    ch_d = _dev(p["ch"].astype(np.int32))
    ws = torch.empty((qjl.qjl_decode_dual_workspace_bytes(B, Hq, Hkv, cap, 128, m, m_out),), dtype=torch.uint8, device=DEV)
    worst = 0.0
    for pos in range(start, start + steps):
        Qs = inputs.make_normal((B, Hq, 128), DT[dt], 7000 + pos, DEV)
        out = qjl.qjl_generation_step(Qs, p["K"][:, :, pos:pos + 1].contiguous(), p["V"][:, :, pos:pos + 1].contiguous(),
                                      p["S_dual"], ch_d, *dc, pos, m_out, vbits, scale, workspace=ws)
        ref = orc.generation_step(inputs.to_f64(Qs), p["S_in64"], p["S_out64"], p["ch"], *ref_caches,
                                  p["K64"][:, :, pos:pos + 1], p["V64"][:, :, pos:pos + 1], pos, vbits, scale)
        worst = max(worst, float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref))))
    say(f"  worst error over the stream {worst:.3g}")
    assert worst <= 2e-3                    # (a near-zero sign flip in an appended row moves the output far less than this)
    e = start + steps
    bulk_b, bulk_i, bulk_o = qjl.qjl_quantize_keys_dual(p["K"][:, :, :e].contiguous(), p["S_dual"], ch_d, m_out)
    bulk_c, bulk_s, bulk_z = qjl.qjl_quantize_values(p["V"][:, :, :e].contiguous(), vbits)
    assert torch.equal(dc[3][:, :, :e], bulk_c) and torch.equal(dc[4][:, :, :e], bulk_s) and torch.equal(dc[5][:, :, :e], bulk_z)
    assert torch.equal(dc[1][:, :, :e], bulk_i) and torch.equal(dc[2][:, :, :e], bulk_o)
    assert float((dc[0][:, :, :e] != bulk_b).float().mean()) < 1e-3


def test_generation_loop_replayed_from_a_graph():
    """The step with its position in device memory (qjl_generation_step_devpos), recorded once into a HIP graph
    together with the increment of the position and replayed for 40 tokens, with eager work (the next token's
    inputs, the comparison) and synchronizations between the replays: every replay against the oracle's stream.
    The capacity is cut into three chunks of 512 rows and the loop starts at row 1000, so the last chunk is empty
    for the first 24 steps and takes the new rows after that."""
    dt, B, Hq, Hkv, cap, m, m_out, vbits, scale = "bf16", 1, 8, 2, 1400, 256, 128, 4, 0.0884
    p = _problem(dt, B, Hq, Hkv, cap, m, m_out, 2323)
    say("[generation graph] 40 replays from position 1000")
    assert qjl.qjl_decode_plan(B, Hq, Hkv, cap, 128, m, m_out)[2:] == (3, 512)
    start, steps = 1000, 40
    ob, oi, oo, _, _ = orc.quantize_keys_dual(p["K64"][:, :, :start], p["S_in64"], p["S_out64"], p["ch"])
    oc, os_, oz = orc.quantize_values(p["V64"][:, :, :start], vbits)
    shapes = [((m + m_out) // 8, np.uint8), (None, np.float16), (None, np.float16), (128 * vbits // 8, np.uint8), (None, np.float16), (None, np.float16)]
    host = []
    for (last, tp), first in zip(shapes, (ob, oi, oo, oc, os_, oz)):
        full = np.full((B, Hkv, cap) + ((last,) if last else ()), 9, dtype=tp)     # stale contents behind the rows in use
        full[:, :, :start] = first
        host.append(full)
    ref_caches = [x.copy() for x in host]
    dc = [_dev(x) for x in host]
    ch_d = _dev(p["ch"].astype(np.int32))
    ws = torch.empty((qjl.qjl_decode_dual_workspace_bytes(B, Hq, Hkv, cap, 128, m, m_out),), dtype=torch.uint8, device=DEV)
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device=DEV)
    Qs = torch.empty((B, Hq, 128), dtype=DT[dt], device=DEV)
    Kn = torch.empty((B, Hkv, 1, 128), dtype=DT[dt], device=DEV)
    Vn = torch.empty((B, Hkv, 1, 128), dtype=DT[dt], device=DEV)
    pos_t = torch.tensor([start], dtype=torch.int32, device=DEV)

    def feed(pos):
        Qs.copy_(inputs.make_normal((B, Hq, 128), DT[dt], 9000 + pos, DEV))
        Kn.copy_(p["K"][:, :, pos:pos + 1])
        Vn.copy_(p["V"][:, :, pos:pos + 1])

    def step():
        qjl.qjl_generation_step(Qs, Kn, Vn, p["S_dual"], ch_d, *dc, pos_t, m_out, vbits, scale, out=out, workspace=ws)
        pos_t.add_(1)

    feed(start)
    step()                                            # once eagerly (what it writes to row `start` the first replay writes again)
    pos_t.fill_(start)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    pos_t.fill_(start)
    worst = 0.0
    for pos in range(start, start + steps):
        feed(pos)
        g.replay()
        torch.cuda.synchronize()
        ref = orc.generation_step(inputs.to_f64(Qs), p["S_in64"], p["S_out64"], p["ch"], *ref_caches,
                                  p["K64"][:, :, pos:pos + 1], p["V64"][:, :, pos:pos + 1], pos, vbits, scale)
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))
        assert err <= 2e-3, (pos, err)
        worst = max(worst, err)
        assert int(pos_t.item()) == pos + 1
    say(f"  worst error over the replays {worst:.3g}")
    e = start + steps
    bulk_c, bulk_s, bulk_z = qjl.qjl_quantize_values(p["V"][:, :, :e].contiguous(), vbits)
    assert torch.equal(dc[3][:, :, :e], bulk_c) and torch.equal(dc[4][:, :, :e], bulk_s) and torch.equal(dc[5][:, :, :e], bulk_z)
    assert torch.all(dc[3][:, :, e:] == 9)            # nothing behind the newest row was touched
    # a position outside the caches cannot be reported from the kernel: it is clamped
    for bad, used in ((cap + 5, cap - 1), (-3, 0)):
        caches = [x.copy() for x in ref_caches]
        dcc = [_dev(x) for x in caches]
        feed(used)
        pos_t.fill_(bad)
        qjl.qjl_generation_step(Qs, Kn, Vn, p["S_dual"], ch_d, *dcc, pos_t, m_out, vbits, scale, out=out, workspace=ws)
        torch.cuda.synchronize()
        ref = orc.generation_step(inputs.to_f64(Qs), p["S_in64"], p["S_out64"], p["ch"], *caches,
                                  p["K64"][:, :, used:used + 1], p["V64"][:, :, used:used + 1], used, vbits, scale)
        assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref))) <= 2e-3, bad


def test_unsupported_combinations_are_reported():
    L = qjl.lib()
    x = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    P = x.data_ptr()
    sh = qjl.QJLShape(1, 4, 4, 64, 128, 256, qjl.QJL_F32, 1.0)
    assert L.qjl_decode_attention_dual_vq(sh, 128, 4, P, P, P, P, P, P, P, P, P, P, 1 << 20, None, None, None) == -2   # fp32
    sh = qjl.QJLShape(1, 4, 4, 64, 128, 256, qjl.QJL_BF16, 1.0)
    assert L.qjl_decode_attention_dual_vq(sh, 128, 3, P, P, P, P, P, P, P, P, P, P, 1 << 20, None, None, None) == -2   # 3-bit values
    assert L.qjl_decode_attention_dual_vq(sh, 64, 4, P, P, P, P, P, P, P, P, P, P, 1 << 20, None, None, None) == -2    # m_out = 64
    assert L.qjl_generation_step(sh, 128, 4, 64, P, P, P, P, P, 4, P, P, P, P, P, P, P, P, 1 << 20, None) == -1        # pos = capacity
    assert L.qjl_generation_step(sh, 128, 4, 3, P, P, P, P, P, 4, P, P, P, P, P, P, P, P, 16, None) == -3              # workspace


@pytest.mark.parametrize("name,units", [("c3o_long_context_b4_32k_dual_v4", 4), ("c5bo_llama3_8b_gqa_b16_8k_dual_v4", 6),
                                        ("c2o_llama2_7b_generation_step_4k_dual_v4", 8)])
def test_full_size_operating_point_sampled(name, units):
    """The benchmark's workloads at full size, in the launch configuration it times.  The oracle handles sampled
    (batch, kv head) units: it quantizes their keys and values, the GPU reads exactly those caches for them, and
    the attention outputs of all their query heads are compared; for the generation step the last row is left
    for the GPU to append and is compared as well.  Every other unit gets the range check that holds at any size."""
    w = inputs.WORKLOADS[name]
    say(f"[full operating point] {name}")
    K, Q, V = inputs.make_workload_tensors(w, DEV)
    S_in = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    S_out = qjl.qjl_make_sketch(w.sketch_seed + 1000, w.m_out, w.d, w.dtype, DEV)
    S_in64, S_out64, Q64 = inputs.to_f64(S_in), inputs.to_f64(S_out), inputs.to_f64(Q)
    ch_d = qjl.qjl_select_outliers(K, 4)
    S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, ch_d)
    bits_d, in_d, out_d = qjl.qjl_quantize_keys_dual(K, S_dual, ch_d, w.m_out)
    vc_d, vs_d, vz_d = qjl.qjl_quantize_values(V, w.vbits)
    G = w.q_heads // w.kv_heads
    pos = w.n - 1
    rng = np.random.default_rng(w.data_seed)
    picked = sorted(rng.choice(w.batch * w.kv_heads, size=units, replace=False).tolist())
    refs = {}
    for u in picked:
        b, g = divmod(u, w.kv_heads)
        K64 = inputs.to_f64(K[b, g])[None, None]
        V64 = inputs.to_f64(V[b, g])[None, None]
        ch = orc.select_outlier_channels(K64, 4)
        assert np.array_equal(ch_d[b, g].cpu().numpy(), ch[0, 0])
        rb, ri, ro, _, _ = orc.quantize_keys_dual(K64, S_in64, S_out64, ch)
        rc, rs, rz = orc.quantize_values(V64, w.vbits)
        assert np.array_equal(vc_d[b, g].cpu().numpy(), rc[0, 0])            # value codes: bit-identical
        for dst, src in ((bits_d, rb), (in_d, ri), (out_d, ro), (vc_d, rc), (vs_d, rs), (vz_d, rz)):
            dst[b, g] = torch.from_numpy(src[0, 0]).to(DEV)                  # both sides use the oracle's caches
        refs[(b, g)] = (orc.decode_attention_dual_vq(Q64[b:b + 1, g * G:(g + 1) * G], S_in64, S_out64, ch, rb, ri, ro, rc, rs, rz,
                                                     w.vbits, w.scale)[0], rb, rc, rs, rz)
    if w.stream:
        k_last, v_last = K[:, :, pos:pos + 1].contiguous(), V[:, :, pos:pos + 1].contiguous()
        for t in (bits_d, in_d, out_d, vc_d, vs_d, vz_d):
            t[:, :, pos] = 0                                                 # the row the step has to write
        out = qjl.qjl_generation_step(Q, k_last, v_last, S_dual, ch_d, bits_d, in_d, out_d, vc_d, vs_d, vz_d, pos, w.m_out,
                                      w.vbits, w.scale).cpu().numpy()
    else:
        out = qjl.qjl_decode_attention_dual_vq(Q, S_dual, bits_d, in_d, out_d, vc_d, vs_d, vz_d, w.m_out, w.vbits, w.scale).cpu().numpy()
    worst = 0.0
    for (b, g), (ref, rb, rc, rs, rz) in refs.items():
        worst = max(worst, float(np.max(np.abs(out[b, g * G:(g + 1) * G].astype(np.float64) - ref))))
        if w.stream:                                                         # the appended row
            assert np.array_equal(vc_d[b, g, pos].cpu().numpy(), rc[0, 0, pos])
            assert vs_d[b, g, pos].item() == rs[0, 0, pos] and vz_d[b, g, pos].item() == rz[0, 0, pos]
            assert float(np.mean(bits_d[b, g, pos].cpu().numpy() != rb[0, 0, pos])) < 0.1   # near-zero projections may differ
    say(f"  worst attention error over {len(refs) * G} heads: {worst:.3g}")
    assert worst <= 2e-3 and np.all(np.isfinite(out))
    deq_max = (vz_d.float() + vs_d.float() * (2 ** w.vbits - 1)).amax(dim=2).cpu().numpy().repeat(G, axis=1)
    deq_min = vz_d.float().amin(dim=2).cpu().numpy().repeat(G, axis=1)
    assert np.all(out <= deq_max[..., None] + 1e-3) and np.all(out >= deq_min[..., None] - 1e-3)
