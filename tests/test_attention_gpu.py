"""GPU parity of decode attention (through the C ABI) against the fp64 oracle.

Bar: |gpu - y| <= 4e-3 * S per output element, S = sum_j p_j |v_j| (tests/parity.py), on seeded inputs
with the ragged length mix of a decode batch; empty and one-position requests, grouped heads whose
group is not a power of two, both head sizes, and chunked as well as single-pass launches."""
import numpy as np
import pytest

from tests.gpu_common import say, to_dev, to_host
from tests.parity import check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def thi():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_25655_amd as thi
    thi.load_library()
    return thi


def f16(a):
    return np.asarray(a, dtype=np.float16)


def make_case(seed, B, Hq, Hkv, D, S_max, lens):
    rng = np.random.Generator(np.random.Philox(key=seed))
    q = f16(rng.standard_normal((B, Hq, D)))
    k = f16(rng.standard_normal((B, Hkv, S_max, D)))
    v = f16(rng.standard_normal((B, Hkv, S_max, D)))
    # whatever lies past a request's length must not matter: poison it
    for b in range(B):
        k[b, :, lens[b]:] = np.float16(np.nan)
        v[b, :, lens[b]:] = np.float16(np.inf)
    return q, k, v


def run(thi, q, k, v, lens, scale):
    import torch
    B, Hq, D = q.shape
    _, Hkv, S_max, _ = k.shape
    ws = thi.Workspace(thi.thi_attention_workspace_bytes(B, Hq, Hkv, D, S_max), init=False)
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float16, device="cuda")
    ld = torch.from_numpy(np.ascontiguousarray(lens, dtype=np.int32)).cuda()
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    thi.thi_decode_attention(qd, kd, vd, ld, scale, out, ws)
    first = to_host(out)
    out2 = torch.full((B, Hq, D), float("nan"), dtype=torch.float16, device="cuda")
    thi.thi_decode_attention(qd, kd, vd, ld, scale, out2, ws)
    assert np.array_equal(first.view(np.uint16), to_host(out2).view(np.uint16)), "not reproducible"
    return first


CASES = [
    # B, Hq, Hkv, D, S_max, lengths
    (1, 4, 4, 128, 64, [64]),
    (2, 4, 4, 128, 300, [300, 1]),
    (3, 8, 8, 128, 1000, [1000, 517, 0]),
    (4, 16, 2, 128, 777, [777, 64, 65, 3]),          # group of 8
    (2, 6, 2, 128, 500, [123, 500]),                  # group of 3: two passes, the second with one head
    (2, 8, 4, 64, 600, [600, 257]),                   # head size 64, group of 2
    (5, 4, 1, 64, 130, [130, 129, 128, 127, 1]),      # group of 4
    (40, 32, 32, 128, 200, None),                     # many workgroups: one pass per request
    (1, 8, 1, 128, 4096, [4096]),                     # one request, long: cut into chunks
    (2, 64, 8, 128, 2050, [2050, 999]),               # 70B-like heads
    (2, 8, 2, 128, 333, [333, 200]),                  # group of 4, head size 128
    (1, 24, 2, 128, 450, [450]),                      # group of 12: a pass of 8 heads and a pass of 4
    (3, 32, 8, 128, 150, [150, 17, 16]),              # Llama-3-8B-like heads, short
]


@pytest.mark.parametrize("B,Hq,Hkv,D,S_max,lens", CASES)
def test_decode_attention_matches_oracle(thi, oracle_mod, B, Hq, Hkv, D, S_max, lens):
    say(f"[case] decode attention B={B} Hq={Hq} Hkv={Hkv} D={D} S_max={S_max}")
    if lens is None:
        lens = (np.arange(B) * 37 % S_max + 1).tolist()
    lens = np.asarray(lens, dtype=np.int32)
    q, k, v = make_case(9000 + B + Hq + D + S_max, B, Hq, Hkv, D, S_max, lens)
    scale = float(np.float32(1.0 / np.sqrt(D)))
    got = run(thi, q, k, v, lens, scale)
    kc, vc = k.copy(), v.copy()
    for b in range(B):                       # the oracle never reads past the length either; keep it finite anyway
        kc[b, :, lens[b]:] = 0
        vc[b, :, lens[b]:] = 0
    y, s = oracle_mod.decode_attention(q, kc, vc, lens, scale)
    check(got.reshape(B * Hq, D), y.reshape(B * Hq, D), s.reshape(B * Hq, D) + 1e-30, "decode attention", argmax=False)
    for b in range(B):
        if lens[b] == 0:
            assert not got[b].astype(np.float32).any(), "an empty request must give zeros"


def test_sharp_softmax_selects_one_row(thi, oracle_mod):
    # a dominant key: the weights are one-hot to fp32 precision, so the output is that value row bit for bit
    rng = np.random.default_rng(7)
    B, H, D, S = 2, 4, 128, 900
    q = f16(np.full((B, H, D), 4.0))
    k = f16(rng.uniform(-0.05, 0.05, (B, H, S, D)))
    v = f16(rng.standard_normal((B, H, S, D)))
    pick = [[5, 899, 400, 64], [0, 63, 128, 700]]
    for b in range(B):
        for h in range(H):
            k[b, h, pick[b][h]] = 4.0
    got = run(thi, q, k, v, np.array([S, S]), 1.0)
    for b in range(B):
        for h in range(H):
            assert np.array_equal(got[b, h].view(np.uint16), v[b, h, pick[b][h]].view(np.uint16))


@pytest.mark.parametrize("B,Hq,Hkv", [(32, 32, 32), (32, 64, 8), (1, 64, 8)])
def test_full_size_properties_without_an_oracle(thi, B, Hq, Hkv):
    """At the benchmark's size (2048 cached positions per request, heads of 128): permuting the requests
    permutes the outputs bit for bit (requests are independent), and scaling V by a power of two scales the
    output exactly (the weights do not depend on V)."""
    import torch
    D, S = 128, 2048
    say(f"[case] attention properties B={B} Hq={Hq} Hkv={Hkv} S={S}")
    g = torch.Generator(device="cuda")
    g.manual_seed(5 + B + Hkv)
    q = torch.randn((B, Hq, D), generator=g, device="cuda", dtype=torch.float32).half()
    k = torch.randn((B, Hkv, S, D), generator=g, device="cuda", dtype=torch.float32).half()
    v = torch.randn((B, Hkv, S, D), generator=g, device="cuda", dtype=torch.float32).half()
    lens = torch.randint(1, S + 1, (B,), generator=g, device="cuda", dtype=torch.int32)
    lens[0] = S
    ws = thi.Workspace(thi.thi_attention_workspace_bytes(B, Hq, Hkv, D, S), init=False)
    scale = 1.0 / D ** 0.5

    def call(q_, k_, v_, l_):
        out = torch.full((B, Hq, D), float("nan"), dtype=torch.float16, device="cuda")
        thi.thi_decode_attention(q_, k_, v_, l_, scale, out, ws)
        torch.cuda.synchronize()
        return out

    a = call(q, k, v, lens)
    assert torch.isfinite(a.float()).all()
    perm = torch.randperm(B, generator=g, device="cuda")
    ap = call(q[perm].contiguous(), k[perm].contiguous(), v[perm].contiguous(), lens[perm].contiguous())
    assert torch.equal(a[perm].view(torch.int16), ap.view(torch.int16))
    a4 = call(q, k, (v.float() * 4).half(), lens)
    ok = a.float().abs() >= 2.0 ** -12
    assert ok.float().mean() > 0.95
    assert torch.equal((a.float() * 4)[ok], a4.float()[ok])


def test_attention_argument_errors(thi):
    import torch
    z = lambda *sh: torch.zeros(sh, dtype=torch.float16, device="cuda")
    ws = thi.Workspace(1 << 20, init=False)
    lens = torch.ones(1, dtype=torch.int32, device="cuda")
    assert thi.thi_decode_attention(z(1, 3, 128), z(1, 2, 8, 128), z(1, 2, 8, 128), lens, 1.0, z(1, 3, 128), ws, check=False) == 2
    assert thi.thi_decode_attention(z(1, 2, 96), z(1, 2, 8, 96), z(1, 2, 8, 96), lens, 1.0, z(1, 2, 96), ws, check=False) == 2
    assert thi.thi_decode_attention(z(1, 2, 128), z(1, 2, 8, 128), z(1, 2, 8, 128), None, 1.0, z(1, 2, 128), ws, check=False) == 1
    assert thi.thi_attention_workspace_bytes(1, 3, 2, 128, 8) == 0
