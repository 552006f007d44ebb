"""GPU parity of the range variants (one visit of a key chunk to a query chunk, the building block
of context parallelism) and of the log-sum-exp merge, through the C ABI, against the fp64
reference of oracle/range_oracle.py; and the property that makes them useful: the visits of a
ring merge to the plain forward, their partial gradients sum to the plain backward."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from oracle import range_oracle as rorc
from paper_2412_07894_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu

A = binding.RANGE_ALIGN
O_SENT, LSE_SENT = 7.0, 123.0            # what unwritten rows must still hold


def setup(lengths, hq, hkv, seed, gain=1.0):
    d = 128
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", seed)
    do = do * np.float32(gain)
    scale = 1.0 / np.sqrt(d)
    dev = dict(cu=torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda(), q=gu.to_dev(q, "bf16"),
               k=gu.to_dev(k, "bf16"), v=gu.to_dev(v, "bf16"), do=gu.to_dev(do, "bf16"))
    return cu, q, k, v, do, scale, dev


def rows_of(cu, rng_list, which):
    """Boolean mask over the T packed rows: inside the query (which=0) or key (which=1) range."""
    m = np.zeros(int(cu[-1]), dtype=bool)
    for s, r in enumerate(rng_list):
        L = int(cu[s + 1] - cu[s])
        b, e = r[2 * which], min(r[2 * which + 1], L)
        if e > b:
            m[cu[s] + b:cu[s] + e] = True
    return m


def split(ranges):
    return [(r[0], r[1]) for r in ranges], [(r[2], r[3]) for r in ranges]


def check_lse(got, ref):
    """-inf must match exactly in place; the finite entries meet the bf16 bar."""
    assert np.array_equal(np.isneginf(got), np.isneginf(ref)), "LSE: -inf entries differ"
    fin = np.isfinite(ref)
    assert np.all(np.isfinite(got[fin]))
    if fin.any():
        gu.check("lse", got[fin], ref[fin], "bf16")


def run_fwd_range(dev, cu, ranges, scale, hq):
    T = int(cu[-1])
    lens = np.diff(cu)
    out = torch.full((T, hq, 128), O_SENT, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((hq, T), LSE_SENT, dtype=torch.float32, device="cuda")
    binding.varlen_attn_fwd_range(dev["q"], dev["k"], dev["v"], dev["cu"], ranges, int(lens.max()), scale, out, lse,
                                  cu_seqlens_host=[int(x) for x in cu])
    torch.cuda.synchronize()
    return gu.to_np(out), gu.to_np(lse)


CASES = [
    # (lengths, hq, hkv, ranges)
    ([700, 300, 1100, 90, 0, 256], 4, 2,
     [(256, 768, 0, 512), (0, 256, 0, 300), (512, 1100, 256, 768), (256, 512, 0, 256), (0, 0, 0, 0), (0, 256, 0, 256)]),
    # keys strictly before the queries (no diagonal tile at all), and keys after them (nothing visible)
    ([1500, 1024], 8, 8, [(1024, 1500, 0, 512), (0, 512, 512, 1024)]),
    # the whole sequence as one range reproduces the plain call; an empty key range; an empty query range
    ([600, 520, 515], 2, 1, [(0, 600, 0, 600), (0, 520, 256, 256), (512, 512, 0, 515)]),
]


@pytest.mark.parametrize("lengths,hq,hkv,ranges", CASES)
def test_forward_visit(lengths, hq, hkv, ranges):
    print(f"\nfwd range case lengths={lengths} hq={hq} hkv={hkv} ranges={ranges}", flush=True)
    cu, q, k, v, do, scale, dev = setup(lengths, hq, hkv, seed=51)
    o, lse = run_fwd_range(dev, cu, ranges, scale, hq)
    qr, kr = split(ranges)
    o_ref, lse_ref = rorc.fwd_range(q, k, v, cu, scale, qr, kr)
    inq = rows_of(cu, ranges, 0)
    assert np.all(o[~inq] == O_SENT) and np.all(lse[:, ~inq] == LSE_SENT), "rows outside the query range were written"
    assert not np.isnan(o_ref[inq]).any()
    if inq.any():
        gu.check("o", o[inq], o_ref[inq], "bf16")
        check_lse(lse[:, inq], lse_ref[:, inq])
        blind = np.isneginf(lse_ref[:, inq]).T              # [rows, heads]
        assert np.all(o[inq][blind] == 0.0)


def chunk_bounds(L, cp):
    """cp chunks of a sequence with boundaries on the granule (the last chunk takes the rest)."""
    per = -(-L // cp)
    per = -(-per // A) * A
    return [(c * per, (c + 1) * per if c + 1 < cp else max(L, cp * per)) for c in range(cp)]


@pytest.mark.parametrize("lengths,hq,hkv,cp", [([1300, 257, 2048, 40], 4, 2, 2), ([3000, 700, 100], 2, 2, 4)])
def test_ring_of_visits_merges_to_the_plain_forward(lengths, hq, hkv, cp):
    """Every (query chunk, key chunk) pair is one visit - also the pairs in which the keys lie
    after the queries, which contribute the neutral element - merged in place as a ring would."""
    print(f"\nring case lengths={lengths} hq={hq} hkv={hkv} cp={cp}", flush=True)
    cu, q, k, v, do, scale, dev = setup(lengths, hq, hkv, seed=52)
    T = int(cu[-1])
    bounds = [chunk_bounds(L, cp) for L in lengths]
    acc_o = torch.zeros((T, hq, 128), dtype=torch.bfloat16, device="cuda")
    acc_l = torch.full((hq, T), float("-inf"), dtype=torch.float32, device="cuda")
    part_o = torch.zeros_like(acc_o)
    part_l = torch.full_like(acc_l, float("-inf"))
    hc = [int(x) for x in cu]
    for step in range(cp):                       # ring step: rank r meets key chunk (r - step) mod cp
        for r in range(cp):
            c = (r - step) % cp
            ranges = [(b[r][0], b[r][1], b[c][0], b[c][1]) for b in bounds]
            part_o.zero_(); part_l.fill_(float("-inf"))
            binding.varlen_attn_fwd_range(dev["q"], dev["k"], dev["v"], dev["cu"], ranges, max(lengths), scale,
                                          part_o, part_l, cu_seqlens_host=hc)
            binding.attn_merge(acc_o, acc_l, part_o, part_l, out=acc_o, lse_out=acc_l)
    torch.cuda.synchronize()
    o_ref, lse_ref = orc.fwd(q, k, v, cu, scale)
    gu.check("o", gu.to_np(acc_o), o_ref, "bf16")
    gu.check("lse", gu.to_np(acc_l), lse_ref, "bf16")


def test_ring_at_head_dim_64():
    lengths, hq, hkv, cp = [1300, 257, 600], 4, 2, 2
    d = 64
    cu, q, k, v, do = wl.custom(lengths, hq, hkv, d, "bf16", 55)
    scale = 1.0 / np.sqrt(d)
    dev = [gu.to_dev(x, "bf16") for x in (q, k, v)]
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    T = int(cu[-1])
    bounds = [chunk_bounds(L, cp) for L in lengths]
    acc_o = torch.zeros((T, hq, d), dtype=torch.bfloat16, device="cuda")
    acc_l = torch.full((hq, T), float("-inf"), dtype=torch.float32, device="cuda")
    part_o, part_l = torch.zeros_like(acc_o), torch.full_like(acc_l, float("-inf"))
    for r in range(cp):
        for c in range(r + 1):
            ranges = [(b[r][0], b[r][1], b[c][0], b[c][1]) for b in bounds]
            binding.varlen_attn_fwd_range(dev[0], dev[1], dev[2], cu_d, ranges, max(lengths), scale, part_o, part_l,
                                          cu_seqlens_host=[int(x) for x in cu])
            binding.attn_merge(acc_o, acc_l, part_o, part_l, out=acc_o, lse_out=acc_l)
            part_o.zero_(); part_l.fill_(float("-inf"))
    torch.cuda.synchronize()
    o_ref, lse_ref = orc.fwd(q, k, v, cu, scale)
    gu.check("o", gu.to_np(acc_o), o_ref, "bf16")
    gu.check("lse", gu.to_np(acc_l), lse_ref, "bf16")


def test_merge_kernel_alone():
    rng = np.random.default_rng(7)
    T, hq = 1000, 3
    oa = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(rng.standard_normal((T, hq, 128)).astype(np.float32)))
    ob = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(rng.standard_normal((T, hq, 128)).astype(np.float32)))
    la = rng.uniform(-30, 30, size=(hq, T)).astype(np.float32)
    lb = (la + rng.uniform(-12, 12, size=(hq, T))).astype(np.float32)
    la[0, :100] = -np.inf                       # a alone blind, b alone blind, both blind
    lb[1, 50:150] = -np.inf
    la[2, 200:260] = -np.inf; lb[2, 230:300] = -np.inf
    o_ref, l_ref = rorc.merge(oa, la, ob, lb)
    d = [gu.to_dev(oa, "bf16"), torch.from_numpy(la).cuda(), gu.to_dev(ob, "bf16"), torch.from_numpy(lb).cuda()]
    o, l = binding.attn_merge(*d)
    torch.cuda.synchronize()
    gu.check("o", gu.to_np(o), o_ref, "bf16")
    got_l = gu.to_np(l)
    assert np.array_equal(np.isneginf(got_l), np.isneginf(l_ref))
    fin = np.isfinite(l_ref)
    assert np.max(np.abs(got_l[fin] - l_ref[fin])) <= 1e-5 * np.maximum(1.0, np.abs(l_ref[fin])).max()
    # a partial with weight zero is taken out even when its rows hold non-finite bits
    oa_bad = d[0].clone()
    oa_bad[:100, 0] = float("nan")
    o2, l2 = binding.attn_merge(oa_bad, d[1], d[2], d[3])
    # in place over either input pair
    a_o, a_l = d[0].clone(), d[1].clone()
    binding.attn_merge(a_o, a_l, d[2], d[3], out=a_o, lse_out=a_l)
    b_o, b_l = d[2].clone(), d[3].clone()
    binding.attn_merge(d[0], d[1], b_o, b_l, out=b_o, lse_out=b_l)
    torch.cuda.synchronize()
    for oo, ll in ((o2, l2), (a_o, a_l), (b_o, b_l)):
        assert torch.equal(oo, o) and torch.equal(ll, l)


@pytest.mark.parametrize("lengths,hq,hkv,ranges", CASES)
def test_backward_visit(lengths, hq, hkv, ranges):
    print(f"\nbwd range case lengths={lengths} hq={hq} hkv={hkv} ranges={ranges}", flush=True)
    cu, q, k, v, do, scale, dev = setup(lengths, hq, hkv, seed=53)
    T = int(cu[-1])
    o_full, lse_full = orc.fwd(q, k, v, cu, scale)
    dvec = np.einsum("thd,thd->ht", do.astype(np.float64), o_full)
    o_in = gu.to_dev(o_full.astype(np.float32), "bf16")
    lse_in = torch.from_numpy(lse_full.astype(np.float32)).cuda()
    sent = 5.0
    dq = torch.full((T, hq, 128), sent, dtype=torch.bfloat16, device="cuda")
    dk = torch.full((T, hkv, 128), sent, dtype=torch.bfloat16, device="cuda")
    dv = torch.full((T, hkv, 128), sent, dtype=torch.bfloat16, device="cuda")
    binding.varlen_attn_bwd_range(dev["q"], dev["k"], dev["v"], o_in, lse_in, dev["do"], dev["cu"], ranges,
                                  max(lengths), scale, dq, dk, dv, cu_seqlens_host=[int(x) for x in cu])
    torch.cuda.synchronize()
    qr, kr = split(ranges)
    dq_ref, dk_ref, dv_ref = rorc.bwd_range(q, k, v, do, cu, scale, lse_full, dvec, qr, kr)
    inq, ink = rows_of(cu, ranges, 0), rows_of(cu, ranges, 1)
    g = {"dq": gu.to_np(dq), "dk": gu.to_np(dk), "dv": gu.to_np(dv)}
    assert np.all(g["dq"][~inq] == sent), "dQ rows outside the query range were written"
    assert np.all(g["dk"][~ink] == sent) and np.all(g["dv"][~ink] == sent), "dK/dV rows outside the key range were written"
    for name, ref, m in (("dq", dq_ref, inq), ("dk", dk_ref, ink), ("dv", dv_ref, ink)):
        assert not np.isnan(ref[m]).any()
        if m.any():
            gu.check(name, g[name][m], ref[m], "bf16")


def test_partial_gradients_of_a_ring_sum_to_the_plain_backward():
    lengths, hq, hkv, cp = [1300, 257, 2048, 40], 4, 2, 2
    cu, q, k, v, do, scale, dev = setup(lengths, hq, hkv, seed=54, gain=0.5)
    T = int(cu[-1])
    hc = [int(x) for x in cu]
    o, lse = binding.varlen_attn_fwd(dev["q"], dev["k"], dev["v"], dev["cu"], max(lengths), scale, cu_seqlens_host=hc)
    bounds = [chunk_bounds(L, cp) for L in lengths]
    tot = {n: np.zeros((T, h, 128)) for n, h in (("dq", hq), ("dk", hkv), ("dv", hkv))}
    for r in range(cp):
        for c in range(cp):
            ranges = [(b[r][0], b[r][1], b[c][0], b[c][1]) for b in bounds]
            bufs = [torch.zeros((T, h, 128), dtype=torch.bfloat16, device="cuda") for h in (hq, hkv, hkv)]
            binding.varlen_attn_bwd_range(dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dev["cu"], ranges,
                                          max(lengths), scale, *bufs, cu_seqlens_host=hc)
            torch.cuda.synchronize()
            for n, t in zip(("dq", "dk", "dv"), bufs):
                tot[n] += gu.to_np(t)
    dq, dk, dv = orc.bwd(q, k, v, do, cu, scale)
    for name, ref in (("dq", dq), ("dk", dk), ("dv", dv)):
        gu.check(name, tot[name], ref, "bf16")


def test_config2_ring_at_full_size():
    """Configuration 2 (the benchmark's headline buffer) under CP = 2, every visit of both ranks:
    the merged forward and the summed partial gradients against sampled oracle rows and keys."""
    import cp_study
    cid, cp = 2, 2
    cfg = wl.CONFIGS[cid]
    lengths = [int(x) for x in wl.seqlens(cid)]
    cu = wl.cu_seqlens(lengths)
    T, hq, hkv = cfg.total_tokens, cfg.hq, cfg.hkv
    q = wl.normal_tensor(cid, "q", T, hq, cfg.d, "bf16"); k = wl.normal_tensor(cid, "k", T, hkv, cfg.d, "bf16")
    v = wl.normal_tensor(cid, "v", T, hkv, cfg.d, "bf16"); do = wl.normal_tensor(cid, "do", T, hq, cfg.d, "bf16")
    print(f"\nconfig 2 ring: T={T} seqs={len(lengths)} longest={max(lengths)}", flush=True)
    qd, kd, vd, dod = (gu.to_dev(x, "bf16") for x in (q, k, v, do))
    cu_d = torch.from_numpy(cu).cuda()
    hc, ml = [int(x) for x in cu], max(lengths)
    bounds = cp_study.chunk_ranges(lengths, cp, A)
    acc_o = torch.zeros_like(qd)
    acc_l = torch.full((hq, T), float("-inf"), dtype=torch.float32, device="cuda")
    part_o, part_l = torch.zeros_like(qd), torch.full_like(acc_l, float("-inf"))
    visits = [(r, c) for r in range(cp) for c in range(r + 1)]
    for r, c in visits:
        ranges = [(b[r][0], b[r][1], b[c][0], b[c][1]) for b in bounds]
        binding.varlen_attn_fwd_range(qd, kd, vd, cu_d, ranges, ml, cfg.scale, part_o, part_l, cu_seqlens_host=hc)
        binding.attn_merge(acc_o, acc_l, part_o, part_l, out=acc_o, lse_out=acc_l)
        part_o.zero_(); part_l.fill_(float("-inf"))
    tot = [torch.zeros((T, h, cfg.d), dtype=torch.float32, device="cuda") for h in (hq, hkv, hkv)]
    for r, c in visits:
        ranges = [(b[r][0], b[r][1], b[c][0], b[c][1]) for b in bounds]
        bufs = [torch.zeros((T, h, cfg.d), dtype=torch.bfloat16, device="cuda") for h in (hq, hkv, hkv)]
        binding.varlen_attn_bwd_range(qd, kd, vd, acc_o, acc_l, dod, cu_d, ranges, ml, cfg.scale, *bufs, cu_seqlens_host=hc)
        for a, t in zip(tot, bufs):
            a += t.float()
    torch.cuda.synchronize()
    rng = np.random.default_rng(77)
    toks, heads = gu.sample_rows(cu, hq, rng, 60)
    ro, rlse, rdq = orc.rows(q, k, v, do, cu, cfg.scale, toks, heads)
    ti, hi = torch.from_numpy(toks.astype(np.int64)).cuda(), torch.from_numpy(heads.astype(np.int64)).cuda()
    gu.check("o[rows]", gu.to_np(acc_o[ti, hi]), ro, "bf16")
    gu.check("lse[rows]", gu.to_np(acc_l[hi, ti]), rlse, "bf16")
    gu.check("dq[rows]", gu.to_np(tot[0][ti, hi]), rdq, "bf16")
    lens = np.diff(cu)
    s = int(np.argsort(-lens)[1])                       # the second longest sequence: keys of both chunks
    L, g = int(lens[s]), 3 % hkv
    cols = np.array(sorted({0, 1, 127, 128, 255, 256, L // 2, L - 2, L - 1} & set(range(L))), dtype=np.int32)
    rk, rv = orc.cols(q, k, v, do, cu, cfg.scale, s, g, cols)
    idx = torch.from_numpy((cu[s] + cols).astype(np.int64)).cuda()
    gu.check("dk[keys]", gu.to_np(tot[1][idx, g]), rk, "bf16")
    gu.check("dv[keys]", gu.to_np(tot[2][idx, g]), rv, "bf16")
