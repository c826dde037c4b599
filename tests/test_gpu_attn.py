"""Instrumented bf16 attention forward through the C ABI: outputs against the fp64 oracle and the
uninstrumented kernel (bitwise); traces against closed forms and the CPU decoder oracle."""
import math

import numpy as np
import pytest
import torch

import inputs
from oracle import ref_attn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_attn(kp, q, k, v, causal, mask, trace_cap=None, scale=None, dev=None):
    B, H, S, D = q.shape
    if dev is None:
        dev = (q.cuda(), k.cuda(), v.cuda())
    O = torch.full((B, H, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    n_wg, waves, R = kp.kp_attn_launch_shape(B, H, S, D)
    trace = None
    if mask & 0x7FFFFFFF:
        trace = torch.full((kp.kp_trace_bytes(n_wg, waves, trace_cap),), 0x33, dtype=torch.uint8, device="cuda")
    kp.kp_attn_instrumented(*dev, O, B, H, S, D, causal, scale if scale else 1.0 / math.sqrt(D), mask, trace,
                            trace_cap or 0)
    torch.cuda.synchronize()
    return O, trace, (n_wg, waves, R)


def assert_head_close(O, q, k, v, b, h, causal, rows=None, scale=None):
    ref = ref_attn(q[b, h], k[b, h], v[b, h], causal=causal, rows=rows, scale=scale)
    got = O[b, h].float().cpu().numpy().astype(np.float64)
    if rows is not None:
        got = got[np.asarray(rows)]
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.abs(got - ref)
    assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms), (b, h, float(err.max()), float(rms))
    assert np.linalg.norm(got - ref) <= 1e-2 * np.linalg.norm(ref)


@pytest.mark.parametrize("causal", [True, False])
def test_small_attention_matches_oracle_and_vanilla(kp, causal):
    q, k, v = inputs.attn_inputs(2, 3, 384, 128, seed=7)
    o_van, _, shape = run_attn(kp, q, k, v, causal, 0)
    assert shape == (2 * 3 * 3, 4, 3)
    for b in range(2):
        for h in range(3):
            assert_head_close(o_van, q, k, v, b, h, causal)
    o_ins, _, _ = run_attn(kp, q, k, v, causal, 0b111, trace_cap=1024)
    assert torch.equal(o_ins.view(torch.int16), o_van.view(torch.int16))
    o_fl, _, _ = run_attn(kp, q, k, v, causal, 0b101 | (1 << 31), trace_cap=1024)
    assert torch.equal(o_fl.view(torch.int16), o_van.view(torch.int16))
    o_sc, _, _ = run_attn(kp, q, k, v, causal, 0, scale=0.2)
    assert_head_close(o_sc, q, k, v, 1, 2, causal, scale=0.2)


def test_heads_in_multiples_of_eight_take_the_xcd_mapping(kp):
    """With a multiple of 8 (batch x head) pairs the workgroups are renumbered so that all query blocks
    of a head run on one XCD; every head must still come out right, and the recorded workgroup ids
    stay head-major: workgroup w of the trace is head w // blocks, query block blocks - 1 - w % blocks."""
    B, H, S = 2, 8, 384
    q, k, v = inputs.attn_inputs(B, H, S, 128, seed=12)
    o_van, _, shape = run_attn(kp, q, k, v, True, 0)
    blocks = S // 128
    assert shape == (B * H * blocks, 4, 3)
    for b in range(B):
        for h in range(H):
            assert_head_close(o_van, q, k, v, b, h, True)
    o_ins, trace, _ = run_attn(kp, q, k, v, True, 0b111, trace_cap=1024)
    assert torch.equal(o_ins.view(torch.int16), o_van.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32)
    hdr = raw[16:16 + 32 * shape[0]].reshape(shape[0], 32)
    assert (hdr[:, 0] == np.arange(shape[0])).all()
    # query block qb writes 6 records per KV tile and wave, 2 * (qb + 1) tiles
    want = np.array([6 * 2 * (blocks - w % blocks) for w in range(shape[0])])
    assert (hdr[:, 8] == want).all()


def test_attention_special_cases(kp):
    q, k, v = inputs.attn_inputs(1, 1, 256, 128, seed=8)
    vc = torch.full_like(v, 0.75)
    o, _, _ = run_attn(kp, q, k, vc, True, 0b111, trace_cap=256)
    assert torch.allclose(o.float().cpu(), torch.full((1, 1, 256, 128), 0.75), atol=4e-3)
    o, _, _ = run_attn(kp, q, k, v, True, 0)
    assert torch.equal(o[0, 0, 0].cpu().view(torch.int16), v[0, 0, 0].view(torch.int16))  # row 0 sees key 0 only
    o, _, _ = run_attn(kp, torch.zeros_like(q), k, v, True, 0)
    want = torch.cumsum(v[0, 0].double(), 0) / torch.arange(1, 257, dtype=torch.float64)[:, None]
    assert torch.allclose(o[0, 0].double().cpu(), want, atol=1e-2, rtol=1e-2)


def test_attention_trace_closed_form(kp, oracle_mod):
    from tests.gpu_util import assert_stats_equal

    B, H, S = 1, 2, 512
    q, k, v = inputs.attn_inputs(B, H, S, 128, seed=9)
    _, trace, (n_wg, waves, R) = run_attn(kp, q, k, v, True, 0b111, trace_cap=64)  # 16 slots per wave
    raw = trace.cpu().numpy().view(np.uint32).copy()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 16, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    # query block qb runs 2*(qb+1) KV tiles and writes 6 records per tile and wave
    totals = np.array([6 * 2 * (qb + 1) for qb in range(S // 128)])
    assert st["n_dropped"] == B * H * waves * int(np.maximum(totals - 16, 0).sum())
    assert st["n_slots_valid"] == B * H * waves * int(np.minimum(totals, 16).sum())
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    assert sorted(hdr[:, 8].tolist()) == sorted(list(totals) * (B * H))
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_disorder"] == 0


def test_attention_wave_group_records(kp, oracle_mod):
    """KP_MASK_WAVE_GROUP: the four waves of a workgroup form one group, so the trace holds one
    stream per workgroup, written by wave 0, with the per-wave record count."""
    from tests.gpu_util import assert_stats_equal

    B, H, S = 1, 2, 512
    q, k, v = inputs.attn_inputs(B, H, S, 128, seed=10)
    Q, K, V = q.cuda(), k.cuda(), v.cuda()
    O, O0 = torch.empty_like(Q), torch.empty_like(Q)
    n_wg, waves, R = kp.kp_attn_launch_shape(B, H, S, 128)
    cap = 64
    trace = torch.full((kp.kp_trace_bytes(n_wg, 1, cap),), 0x33, dtype=torch.uint8, device="cuda")
    scale = 1.0 / np.sqrt(128.0)
    kp.kp_attn_instrumented(Q, K, V, O, B, H, S, 128, True, scale, 0b111 | kp.KP_MASK_WAVE_GROUP, trace, cap)
    kp.kp_attn_instrumented(Q, K, V, O0, B, H, S, 128, True, scale, 0, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), O0.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[2:8]) == (n_wg, 1, R, cap, 0, 0)
    out = torch.zeros(kp.kp_stats_bytes(n_wg, 1, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * cap, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    totals = np.array([6 * 2 * (qb + 1) for qb in range(S // 128)])
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    assert sorted(hdr[:, 8].tolist()) == sorted(list(totals) * (B * H)) and (hdr[:, 9:24] == 0).all()
    assert st["n_slots_valid"] == B * H * int(totals.sum()) and st["n_dropped"] == 0
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_disorder"] == 0


@pytest.mark.parametrize("option", ["realtime", "collab", "collab_flush"])
def test_attention_record_variants(kp, oracle_mod, option):
    """KP_MASK_REALTIME (constant-rate clock in the records, Sec. 3.1 MetricType) and KP_MASK_COLLAB
    (64-lane store and hardware ids in the header, Sec. 4.2) on the attention kernel: the output stays
    bit-identical, the trace decodes like the oracle says and holds 6 records per KV tile and wave."""
    from tests.gpu_util import assert_stats_equal

    B, H, S = 1, 2, 512
    q, k, v = inputs.attn_inputs(B, H, S, 128, seed=12)
    Q, K, V = q.cuda(), k.cuda(), v.cuda()
    O, O0 = torch.empty_like(Q), torch.empty_like(Q)
    n_wg, waves, R = kp.kp_attn_launch_shape(B, H, S, 128)
    cap_wave = 64
    bits = {"realtime": kp.KP_MASK_REALTIME, "collab": kp.KP_MASK_COLLAB, "collab_flush": kp.KP_MASK_COLLAB | kp.KP_MASK_FLUSH}[option]
    flags = {"realtime": kp.KP_FLAG_REALTIME, "collab": kp.KP_FLAG_HW_IDS, "collab_flush": kp.KP_FLAG_HW_IDS | 1}[option]
    trace = torch.full((kp.kp_trace_bytes(n_wg, waves, waves * cap_wave),), 0x44, dtype=torch.uint8, device="cuda")
    scale = 1.0 / np.sqrt(128.0)
    kp.kp_attn_instrumented(Q, K, V, O, B, H, S, 128, True, scale, 0b111 | bits, trace, waves * cap_wave)
    kp.kp_attn_instrumented(Q, K, V, O0, B, H, S, 128, True, scale, 0, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), O0.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[2:6]) == (n_wg, waves, R, cap_wave) and raw[7] == flags
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * cap_wave, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    totals = np.array([6 * 2 * (qb + 1) for qb in range(S // 128)])
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    assert sorted(hdr[:, 8].tolist()) == sorted(list(totals) * (B * H)) and (hdr[:, 8:12] == hdr[:, 8:9]).all()
    assert st["n_slots_valid"] == waves * B * H * int(totals.sum()) and st["n_dropped"] == 0
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_orphan_start"] == 0 and st["n_orphan_end"] == 0
    ids = hdr[:, 24:32].copy().view(np.uint16).reshape(n_wg, 16)
    if option == "realtime":
        assert (ids == 0).all()
        h64 = hdr[:, 2:8].copy().view(np.uint64)
        ghz = h64[:, 2].astype(np.float64).sum() / (h64[:, 1] - h64[:, 0]).astype(np.float64).sum() * 0.1
        assert 1.0 < ghz < 2.6, ghz
    else:
        assert (ids[:, waves:] == 0).all() and ((ids[:, :waves] >> 8) == (ids[:, :1] >> 8)).all()
        assert all(len(set((row & 0x3F).tolist())) == waves for row in ids[:, :waves])


def test_full_size_attention(kp, oracle_mod):
    """Benchmark configuration: batch 4, 32 heads, sequence 4096, head dim 128, causal, ring of 1024
    records per workgroup (256 per wave), which wraps for query blocks 21..31."""
    from tests.gpu_util import assert_stats_equal

    B, H, S, D = 4, 32, 4096, 128
    q, k, v = inputs.attn_inputs(B, H, S, D, seed=3)
    dev = (q.cuda(), k.cuda(), v.cuda())
    o_van, _, shape = run_attn(kp, q, k, v, True, 0, dev=dev)
    assert shape == (4096, 4, 3)
    rng = np.random.default_rng(1)
    for b, h in ((0, 0), (3, 31), (1, 17)):
        rows = np.sort(rng.choice(S, size=96, replace=False))
        assert_head_close(o_van, q, k, v, b, h, True, rows=rows)
    o_ins, trace, (n_wg, waves, R) = run_attn(kp, q, k, v, True, 0b111, trace_cap=1024, dev=dev)
    assert torch.equal(o_ins.view(torch.int16), o_van.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 256, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 16), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    totals = np.array([12 * (qb + 1) for qb in range(S // 128)])
    assert st["n_dropped"] == B * H * waves * int(np.maximum(totals - 256, 0).sum()) > 0
    assert st["n_slots_valid"] == B * H * waves * int(np.minimum(totals, 256).sum())
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_span_overflow_wgs"] == 0


@pytest.mark.parametrize("regions", [0b111, 0b101, 0b010])
@pytest.mark.parametrize("trace_cap", [8, 64, 1024])
def test_attention_chained_sites_write_the_generic_sites_records(kp, regions, trace_cap):
    """The kernel keeps only the clocks of its record sites in LDS and makes the records when it copies the
    trace out.  Slot by slot the tags must be those the generic sites write (KP_MASK_COLLAB selects them), with
    a region mask and where the ring wrapped too, and along the sequence numbers of a wave the clocks must
    not decrease."""
    B, H, S = 1, 2, 640
    q, k, v = inputs.attn_inputs(B, H, S, 128, seed=21)
    dev = (q.cuda(), k.cuda(), v.cuda())
    _, t_chain, (n_wg, waves, R) = run_attn(kp, q, k, v, True, regions, trace_cap=trace_cap, dev=dev)
    _, t_gen, _ = run_attn(kp, q, k, v, True, regions | kp.KP_MASK_COLLAB, trace_cap=trace_cap, dev=dev)
    cap = trace_cap // waves
    a, b = (t.cpu().numpy().view(np.uint32).copy() for t in (t_chain, t_gen))
    assert tuple(a[2:6]) == tuple(b[2:6]) == (n_wg, waves, R, cap)
    ha, hb = (x[16:16 + 32 * n_wg].reshape(n_wg, 32) for x in (a, b))
    assert (ha[:, 8:24] == hb[:, 8:24]).all() and (ha[:, 0] == hb[:, 0]).all()
    ra, rb = (x[16 + 32 * n_wg:].reshape(n_wg, waves, cap, 2) for x in (a, b))
    for w in range(n_wg):
        for j in range(waves):
            total = int(ha[w, 8 + j])
            n = min(total, cap)
            assert total == 2 * bin(regions).count("1") * 2 * (S // 128 - w % (S // 128))
            assert (ra[w, j, :n, 0] == rb[w, j, :n, 0]).all(), (w, j)
            assert (ra[w, j, n:] == 0).all()
            seq = ra[w, j, :n, 0] & 0xFFFFF
            order = np.argsort(seq)
            assert (np.sort(seq) == np.arange(total - n, total)).all()
            ts = ra[w, j, :n, 1][order].astype(np.int64)
            assert (np.diff(ts) >= 0).all() and ts[0] > 0
            span = int(ha[w, 4:6].copy().view(np.uint64)[0] - ha[w, 2:4].copy().view(np.uint64)[0])
            assert ts[-1] < span


@pytest.mark.parametrize("case", range(8))
def test_attention_chained_sites_with_every_option(kp, case):
    """Seeded combinations of region mask, wave-group records, constant-rate clock, causal or not, ring capacity
    and sequence length: the chained sites must leave the record counts and tags of the generic sites
    (KP_MASK_COLLAB on top of the same options), slot by slot, and clocks that do not decrease along a stream."""
    rng = np.random.default_rng(300 + case)
    regions = int(rng.integers(1, 8))
    group = bool(rng.integers(2))
    realtime = bool(rng.integers(2))
    causal = bool(rng.integers(2))
    S = int(rng.choice([128, 384, 1024]))
    cap_wave = int(rng.choice([2, 16, 256]))
    q, k, v = inputs.attn_inputs(1, 3, S, 128, seed=60 + case)
    dev = (q.cuda(), k.cuda(), v.cuda())
    n_wg, waves, R = kp.kp_attn_launch_shape(1, 3, S, 128)
    streams = 1 if group else waves
    opts = regions | (kp.KP_MASK_WAVE_GROUP if group else 0) | (kp.KP_MASK_REALTIME if realtime else 0)
    raws = []
    for extra in (0, kp.KP_MASK_COLLAB):
        O = torch.empty(1, 3, S, 128, dtype=torch.bfloat16, device="cuda")
        trace = torch.full((kp.kp_trace_bytes(n_wg, streams, cap_wave * streams),), 0x5C, dtype=torch.uint8, device="cuda")
        kp.kp_attn_instrumented(*dev, O, 1, 3, S, 128, causal, 0.09, opts | extra, trace, cap_wave * streams)
        torch.cuda.synchronize()
        raws.append(trace.cpu().numpy().view(np.uint32).copy())
    x, y = raws
    what = (regions, group, realtime, causal, S, cap_wave)
    assert tuple(x[2:6]) == tuple(y[2:6]) == (n_wg, streams, R, cap_wave), what
    hx, hy = (r[16:16 + 32 * n_wg].reshape(n_wg, 32) for r in (x, y))
    rx, ry = (r[16 + 32 * n_wg:].reshape(n_wg, streams, cap_wave, 2) for r in (x, y))
    assert (hx[:, 8:24] == hy[:, 8:24]).all(), what
    blocks = S // 128
    for w in range(n_wg):
        tiles = 2 * (blocks - w % blocks) if causal else S // 64
        total = int(hx[w, 8])
        assert total == 2 * bin(regions).count("1") * tiles, what
        n = min(total, cap_wave)
        assert (rx[w, :, :n, 0] == ry[w, :, :n, 0]).all(), what
        assert (rx[w, :, n:] == 0).all()
        order = np.argsort(rx[w, :, :n, 0] & 0xFFFFF, axis=1)
        ts = np.take_along_axis(rx[w, :, :n, 1], order, 1).astype(np.int64)
        assert (np.diff(ts, axis=1) >= 0).all() and (ts > 0).all(), what


def test_attention_errors(kp):
    t = torch.zeros(1, 1, 128, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kp.KperfError) as e:
        kp.kp_attn_instrumented(t, t, t, t, 1, 1, 128, 64, 1, 0.1, 0, None, 0)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(kp.KperfError) as e:
        kp.kp_attn_instrumented(t, t, t, t, 1, 1, 100, 128, 1, 0.1, 0, None, 0)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(kp.KperfError) as e:
        kp.kp_attn_instrumented(t, t, t, t, 1, 1, 128, 128, 1, 0.1, 7, None, 64)
    assert e.value.status == kp.KP_ERR_INVALID_ARG
    tr = torch.zeros(kp.kp_trace_bytes(1, 4, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError) as e:
        kp.kp_attn_instrumented(t, t, t, t, 1, 1, 128, 128, 1, 0.1, 7, tr, 60)
    assert e.value.status == kp.KP_ERR_TRACE_TOO_SMALL
