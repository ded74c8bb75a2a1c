"""Exact key identity at full size (40 heads, 4680 queries, 0..8 cached blocks of 4680 tokens).

With N(0,1) inputs at 32760 keys a single dropped, duplicated or misplaced key moves the output
by far less than the tolerance. Here every output element is tied to ONE key instead:

  position of key j in head h:   pos = j + off_h            (off_h shifts the windows per head)
  window (class) of the key:     cls = (pos // 128) % 128   -> K[j,h,:] = 14 * e_cls
  dim the key's value lives in:  d = pos % 128              -> V[j,h,:] = val * e_d,
                                 val = 1 + pos // 16384     (1, 2, 3: which repeat of the class)
  query row i of head h:         Q[i,h,:] = 16 * e_w,  w = (i + 3 h) % n_classes

so row (i, h) puts weight exp(19.8) on the (up to three) 128-key windows of class w and weight 1
on every other key, and out[i,h,d] = val / (window keys) if and only if key "window start + d" was
read exactly once, from the right place, with its own V row. A key dropped from a window zeroes
its element, a duplicated one doubles it, a misplaced one moves it to another element: all far
beyond the 2^-7 relative tolerance (bf16 rounding of P and of the output is 2^-9 each). Windows
start at every residue modulo the 64-key tile across heads, so the cache/block seam, the first
block tile, the ragged last tile and the last key are all inside windows of some (row, head).
Rows whose class is absent from tile 0 also take the kernel's raise-the-maximum path.

Two comparisons: against the oracle on a row sample (all heads, including the ragged last wave
tile), and -- for ALL 4680 x 40 x 128 outputs -- against the closed form of the same definition
(weights are exp(19.8) or 1, so every sum is a count)."""
import math

import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si

pytestmark = pytest.mark.gpu

T, H, D = 4680, 40, 128
A_Q, B_K = 16.0, 14.0
REL_TOL = 2.0 ** -7


def build_case(n_k, dev):
    j = torch.arange(n_k, device=dev, dtype=torch.int64)[:, None]
    off = (17 * torch.arange(H, device=dev, dtype=torch.int64) + 5)[None, :] % 128
    pos = j + off                                   # [n_k, H]
    cls = (pos // 128) % 128
    d = pos % 128
    val = 1 + pos // 16384
    n_classes = min(128, int((n_k + 127 + 127) // 128))
    K = torch.zeros((n_k, H, D), dtype=torch.bfloat16, device=dev)
    K.scatter_(2, cls[:, :, None], torch.full((n_k, H, 1), B_K, dtype=torch.bfloat16, device=dev))
    V = torch.zeros((n_k, H, D), dtype=torch.bfloat16, device=dev)
    V.scatter_(2, d[:, :, None], val[:, :, None].to(torch.bfloat16))
    i = torch.arange(T, device=dev, dtype=torch.int64)[:, None]
    w = (i + 3 * torch.arange(H, device=dev, dtype=torch.int64)[None, :]) % n_classes   # [T, H]
    Q = torch.zeros((T, H, D), dtype=torch.bfloat16, device=dev)
    Q.scatter_(2, w[:, :, None], torch.full((T, H, 1), A_Q, dtype=torch.bfloat16, device=dev))
    return Q, K, V, cls, d, val, w


def closed_form(n_k, cls, d, val, w):
    """out[i,h,:] for every row, from counts: weight E = exp(scale * 16 * 14) inside the row's
    class, 1 outside (fp64)."""
    dev = cls.device
    E = math.exp(A_Q * B_K / math.sqrt(D))
    hh = torch.arange(H, device=dev)[None, :].expand(n_k, H)
    table = torch.zeros((H, 128, D), dtype=torch.float64, device=dev)       # sum of val by (head, class, dim)
    table.index_put_((hh.reshape(-1), cls.reshape(-1), d.reshape(-1)), val.reshape(-1).double(), accumulate=True)
    count = torch.zeros((H, 128), dtype=torch.float64, device=dev)          # keys by (head, class)
    count.index_put_((hh.reshape(-1), cls.reshape(-1)), torch.ones(n_k * H, dtype=torch.float64, device=dev),
                     accumulate=True)
    s_all = table.sum(dim=1)                                                 # [H, D]
    hsel = torch.arange(H, device=dev)[None, :].expand(T, H)
    t_in = table[hsel, w]                                                    # [T, H, D]
    n_in = count[hsel, w]                                                    # [T, H]
    return (E * t_in + (s_all[None] - t_in)) / (E * n_in + (n_k - n_in))[:, :, None]


@pytest.mark.parametrize("k", list(range(9)))
def test_every_output_element_names_its_key(k):
    import paper_2604_17397_amd as P
    dev = torch.device("cuda:0")
    c = k * T
    n_k = c + T
    Q, K, V, cls, d, val, w = build_case(n_k, dev)
    cap = c + 9                                       # poisoned tokens past cache_len
    kc = torch.empty((max(cap, 1), H, D), dtype=torch.bfloat16, device=dev)
    vc = torch.empty_like(kc)
    kc.view(torch.int16).fill_(0x7FC1)
    vc.view(torch.int16).fill_(0x7FC1)
    kc[:c], vc[:c] = K[:c], V[:c]
    kb, vb = K[c:].contiguous(), V[c:].contiguous()
    out = torch.full((T, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
    P.block_attn(Q, kc, vc, kb, vb, c, out=out)
    torch.cuda.synchronize()
    got = out.double()
    assert not torch.isnan(got).any()

    # (1) all rows, all heads, all dims against the closed form
    exp = closed_form(n_k, cls, d, val, w)
    bad = (got - exp).abs() > REL_TOL * exp.abs() + 1e-10
    assert not bad.any(), ("k=%d: %d elements off, first at %s" % (k, int(bad.sum()), bad.nonzero()[0].tolist()))
    # every element that names an in-window key is large: the test is not vacuous
    assert (exp.max(dim=2).values > 1.0 / 400).all()

    # (2) the oracle on a row sample that includes the ragged last wave tile (rows 4672..4679)
    rows = np.array(sorted(set(range(0, 8)) | set(range(2336, 2344)) | set(range(T - 40, T))), dtype=np.int64)
    f = si.bits_from_device
    ref = oracle.block_attn(f(Q), f(kc[:max(c, 1)]), f(vc[:max(c, 1)]), f(kb), f(vb), c, rows=rows)
    g = si.bf16_bits_to_f64(f(out)[rows])
    assert np.all(np.abs(g - ref) <= REL_TOL * np.abs(ref) + 1e-10)
    # and the closed form is the oracle's answer (pins the closed form itself)
    assert np.allclose(exp[torch.from_numpy(rows).to(dev)].cpu().numpy(), ref, rtol=1e-9, atol=1e-14)
