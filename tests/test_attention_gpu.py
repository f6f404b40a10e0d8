"""GPU parity of the attention primitives (rotary embedding, causal grouped-query attention forward and backward,
bf16 with head size 128) against the fp64 oracle on the same seeded bf16 inputs."""
import numpy as np
import pytest

from oracle import attn_oracle as ao
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
HD = 128


def _bf(a):
    return wk.round_to_bf16(np.asarray(a, dtype=np.float32))


def _offsets(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


@pytest.mark.parametrize("lens,heads", [([1, 130, 0, 64, 257], 3), ([4100], 2)], ids=["ragged", "long"])
def test_rope_matches_oracle(lens, heads):
    import torch
    from paper_2602_07263_amd import tlora
    seq = _offsets(lens)
    T = int(seq[-1])
    x = _bf(np.random.default_rng(3).normal(size=(T, heads * HD)))
    att = tlora.Attention(seq, heads, heads, "cuda")
    for inverse in (False, True):
        X = torch.from_numpy(x).to(device="cuda", dtype=torch.bfloat16)
        att.rope(X, heads, 10000.0, inverse)
        torch.cuda.synchronize()
        ref = ao.rope(x, seq, heads, HD, 10000.0, transpose=inverse)
        r = pu.worst_ratio(X.float().cpu().numpy(), ref, pu.BF16_TOL)
        assert r <= 1.0, f"inverse={inverse}: worst error / tolerance {r}"


# (sequence lengths, query heads, key/value heads): ragged lengths around the 32 / 64 / 128 tile edges, an empty
# sequence, single tokens, one sequence of many tiles; group sizes 1, 2 and 4
CASES = [([1, 130, 0, 64, 257, 31, 128], 4, 2),
         ([33, 1, 1, 200], 2, 2),
         ([1500, 7], 8, 2),
         ([5000], 1, 1)]


@pytest.mark.parametrize("case", CASES, ids=["ragged_g2", "small_g1", "long_g4", "one_long_sequence"])
def test_attention_fwd_bwd_match_oracle(case):
    import torch
    from paper_2602_07263_amd import tlora
    lens, Hq, Hkv = case
    seq = _offsets(lens)
    T = int(seq[-1])
    rng = np.random.default_rng(11)
    Q, K, V, dO = (_bf(rng.normal(size=(T, h * HD))) for h in (Hq, Hkv, Hkv, Hq))
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    nan = lambda h: torch.full((T, h * HD), float("nan"), dtype=torch.bfloat16, device="cuda")
    att = tlora.Attention(seq, Hq, Hkv, "cuda")
    tQ, tK, tV, tdO = up(Q), up(K), up(V), up(dO)
    O, dQ, dK, dV = nan(Hq), nan(Hq), nan(Hkv), nan(Hkv)
    lse = torch.full((T, Hq), float("nan"), dtype=torch.float32, device="cuda")
    att.fwd(tQ, tK, tV, O, lse)
    att.bwd(tQ, tK, tV, O, tdO, lse, dQ, dK, dV)
    torch.cuda.synchronize()
    O_r, _ = ao.attention(Q, K, V, seq, Hq, Hkv, HD)
    lse_r = ao.attention_lse(Q, K, seq, Hq, Hkv, HD) / np.log(2.0)      # the kernel stores the statistic in base 2
    dQ_r, dK_r, dV_r = ao.attention_backward(Q, K, V, dO, seq, Hq, Hkv, HD)
    res = {"O": pu.worst_ratio(O.float().cpu().numpy(), O_r, pu.BF16_TOL),
           "lse": pu.worst_ratio(lse.cpu().numpy(), lse_r, 1e-4),
           "dQ": pu.worst_ratio(dQ.float().cpu().numpy(), dQ_r, pu.BF16_TOL),
           "dK": pu.worst_ratio(dK.float().cpu().numpy(), dK_r, pu.BF16_TOL),
           "dV": pu.worst_ratio(dV.float().cpu().numpy(), dV_r, pu.BF16_TOL)}
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {res}"


def test_attention_backward_is_deterministic():
    import torch
    from paper_2602_07263_amd import tlora
    seq = _offsets([700, 90])
    T, Hq, Hkv = int(seq[-1]), 4, 1
    rng = np.random.default_rng(5)
    up = lambda a: torch.from_numpy(_bf(a)).to(device="cuda", dtype=torch.bfloat16).contiguous()
    Q, K, V, dO = (up(rng.normal(size=(T, h * HD))) for h in (Hq, Hkv, Hkv, Hq))
    att = tlora.Attention(seq, Hq, Hkv, "cuda")
    O = torch.empty_like(Q)
    lse = torch.empty((T, Hq), dtype=torch.float32, device="cuda")
    att.fwd(Q, K, V, O, lse)
    outs = []
    for _ in range(2):
        g = [torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)]
        att.bwd(Q, K, V, O, dO, lse, *g)
        torch.cuda.synchronize()
        outs.append([t.view(torch.int16).cpu() for t in g])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_attention_rejects_bad_arguments():
    import ctypes
    from paper_2602_07263_amd import tlora
    L = tlora.lib()
    seq = (ctypes.c_int64 * 2)(0, 8)
    assert L.tlora_attention_workspace_bytes(1, seq, 0) == 0
    bad = (ctypes.c_int64 * 3)(0, 8, 4)
    assert L.tlora_attention_workspace_bytes(2, bad, 4) == 0
    ws = L.tlora_attention_workspace_bytes(1, seq, 4)
    assert ws > 0
    # head size other than 128, and query heads not a multiple of key/value heads
    assert L.tlora_attention_fwd(None, None, None, None, None, 1, seq, 4, 2, 64, None, 0, None) != 0
    assert L.tlora_attention_fwd(None, None, None, None, None, 1, seq, 3, 2, 128, None, 0, None) != 0


def test_attention_at_bench_shape_sampled_sequences():
    """The decoder-layer leg's attention shape (32 query / 8 key-value heads, 41 sequences of 2048 tokens): three
    sampled (sequence, key/value head) groups, each compared in full (all 2048 positions, the group's four query
    heads) with the oracle, which is run on that group's slices alone."""
    import torch
    from paper_2602_07263_amd import tlora
    Hq, Hkv, n, S = 32, 8, 2048, 41
    G = Hq // Hkv
    T = n * S
    seq = _offsets([n] * S)
    g = torch.Generator(device="cuda"); g.manual_seed(21)
    rn = lambda h: torch.randn(T, h * HD, device="cuda", generator=g).to(torch.bfloat16)
    Q, K, V, dO = rn(Hq), rn(Hkv), rn(Hkv), rn(Hq)
    O, dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    lse = torch.empty(T, Hq, dtype=torch.float32, device="cuda")
    att = tlora.Attention(seq, Hq, Hkv, "cuda")
    att.fwd(Q, K, V, O, lse)
    att.bwd(Q, K, V, O, dO, lse, dQ, dK, dV)
    torch.cuda.synchronize()
    for t in (O, dQ, dK, dV):                      # nothing left unwritten anywhere
        assert bool(torch.isfinite(t.float()).all())
    worst = {}
    for s, hk in [(0, 0), (17, 3), (40, 7)]:
        rows = slice(s * n, (s + 1) * n)
        qc, kc = slice(hk * G * HD, (hk + 1) * G * HD), slice(hk * HD, (hk + 1) * HD)
        f = lambda t, c: t[rows, c].double().cpu().numpy()
        q, k, v, do = f(Q, qc), f(K, kc), f(V, kc), f(dO, qc)
        O_r, _ = ao.attention(q, k, v, [0, n], G, 1, HD)
        lse_r = ao.attention_lse(q, k, [0, n], G, 1, HD) / np.log(2.0)
        dQ_r, dK_r, dV_r = ao.attention_backward(q, k, v, do, [0, n], G, 1, HD)
        res = {"O": pu.worst_ratio(f(O, qc), O_r, pu.BF16_TOL),
               "lse": pu.worst_ratio(lse[rows, hk * G:(hk + 1) * G].double().cpu().numpy(), lse_r, 1e-4),
               "dQ": pu.worst_ratio(f(dQ, qc), dQ_r, pu.BF16_TOL),
               "dK": pu.worst_ratio(f(dK, kc), dK_r, pu.BF16_TOL),
               "dV": pu.worst_ratio(f(dV, kc), dV_r, pu.BF16_TOL)}
        for name, r in res.items():
            worst[name] = max(worst.get(name, 0.0), r)
    print({k_: round(v_, 3) for k_, v_ in worst.items()})
    assert all(v_ <= 1.0 for v_ in worst.values()), worst


@pytest.mark.parametrize("seed", range(10))
def test_attention_random_shapes(seed):
    """Random sequence counts and lengths (1 .. 400 tokens, occasionally empty), head counts and group sizes.  Odd seeds
    scale the queries by 3 (a much sharper softmax than unit-variance scores give).  The gradients are products of the
    bf16-rounded score gradients with Q and K, so their rounding noise grows with the operand scale while the "1 +" floor
    of the tolerance does not: for those cases the floor is the query scale, |err| <= tol (3 + |ref|) (a float64
    emulation of nothing but the kernel's three rounding points -- P, dS and the stored O -- already shows 2.3 x the
    unit-floor tolerance on dK there)."""
    import torch
    from paper_2602_07263_amd import tlora
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    lens = [int(x) for x in rng.integers(1, 400, size=int(rng.integers(1, 6)))]
    if seed % 3 == 0:
        lens.insert(int(rng.integers(0, len(lens) + 1)), 0)
    seq = _offsets(lens)
    T = int(seq[-1])
    Q, K, V, dO = (_bf(rng.normal(size=(T, h * HD)) * s) for h, s in ((Hq, 1.0), (Hkv, 1.0), (Hkv, 1.0), (Hq, 1.0)))
    floor = 1.0
    if seed % 2:                                    # sharper softmax: larger queries
        Q = _bf(Q * 3.0)
        floor = 3.0
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    nan = lambda h: torch.full((T, h * HD), float("nan"), dtype=torch.bfloat16, device="cuda")
    att = tlora.Attention(seq, Hq, Hkv, "cuda")
    tQ, tK, tV, tdO = up(Q), up(K), up(V), up(dO)
    O, dQ, dK, dV = nan(Hq), nan(Hq), nan(Hkv), nan(Hkv)
    lse = torch.full((T, Hq), float("nan"), dtype=torch.float32, device="cuda")
    att.fwd(tQ, tK, tV, O, lse)
    att.bwd(tQ, tK, tV, O, tdO, lse, dQ, dK, dV)
    torch.cuda.synchronize()
    O_r, _ = ao.attention(Q, K, V, seq, Hq, Hkv, HD)
    lse_r = ao.attention_lse(Q, K, seq, Hq, Hkv, HD) / np.log(2.0)      # the kernel stores the statistic in base 2
    dQ_r, dK_r, dV_r = ao.attention_backward(Q, K, V, dO, seq, Hq, Hkv, HD)
    def grad_ratio(got, ref):
        got = np.asarray(got, dtype=np.float64)
        assert np.all(np.isfinite(got))
        return float(np.max(np.abs(got - ref) / (pu.BF16_TOL * (floor + np.abs(ref)))))
    res = {"O": pu.worst_ratio(O.float().cpu().numpy(), O_r, pu.BF16_TOL),
           "lse": pu.worst_ratio(lse.cpu().numpy(), lse_r, 1e-4),
           "dQ": grad_ratio(dQ.float().cpu().numpy(), dQ_r),
           "dK": grad_ratio(dK.float().cpu().numpy(), dK_r),
           "dV": grad_ratio(dV.float().cpu().numpy(), dV_r)}
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"lens {lens}, heads {Hq}/{Hkv}: worst error / tolerance ratios {res}"
