"""GPU parity, bit-exact: sdvg_worst_frame_route / sdvg_avg_frame_route and their batched forms
through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


def gpu_route(P, scores, tau, b):
    return P.worst_frame_route(torch.from_numpy(np.asarray(scores, np.float32)).cuda(), tau, b)


def same_route(a, b):
    return a[0] == b[0] and np.float32(a[1]).view(np.uint32) == np.float32(b[1]).view(np.uint32)


def test_tiny_config_route():
    import paper_2604_17397_amd as P
    scores = si.normal(si.SEED, si.TID_SCORES, 12).astype(np.float32)
    for b in (0, 1):
        assert same_route(gpu_route(P, scores, -0.7, b), oracle.route(scores, -0.7, b))
    assert gpu_route(P, scores, -0.7, 0)[0] == 0


@pytest.mark.parametrize("F", [1, 3, 9, 12, 63, 64, 65, 200])
def test_route_frame_counts(F):
    import paper_2604_17397_amd as P
    for trial in range(4):
        s = si.frame_scores_iid(50 + trial, 1, n_frames=F)[0]
        for tau in (-1.0, -0.7, -0.4, float(s.min())):
            assert same_route(gpu_route(P, s, tau, 3), oracle.route(s, tau, 3))


def test_route_edge_values():
    import paper_2604_17397_amd as P
    cases = [[0.0, -0.0, 1.0], [-0.0, 0.0], [1.0, 0.0, -0.0], [np.inf] * 12, [-np.inf, 1.0],
             [0.2, np.nan, 0.1], [np.nan], [np.inf, -np.inf, np.nan], [1e-45, -1e-45], [3.0]]
    for c in cases:
        for tau in (0.0, -0.0, -0.7, np.inf, -np.inf):
            for b in (0, 2):
                assert same_route(gpu_route(P, c, tau, b), oracle.route(c, tau, b)), (c, tau, b)


def test_route_batch_matches_oracle_for_both_score_generators():
    import paper_2604_17397_amd as P
    n = 4096
    for gen in (si.frame_scores_iid, si.frame_scores_correlated):
        scores = gen(77, n)
        idx = (np.arange(n) % 9).astype(np.int32)
        for tau in (-1.0, -0.7, -0.4):
            dec, qb = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), tau,
                                                block_idx=torch.from_numpy(idx).cuda())
            dec, qb = dec.cpu().numpy(), qb.cpu().numpy()
            for i in range(n):
                d, q = oracle.route(scores[i], tau, int(idx[i]))
                assert d == dec[i] and q.view(np.uint32) == qb[i].view(np.uint32)
            assert dec[idx == 0].sum() == 0
        dec2, _ = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), -0.7, first_block_idx=0)
        assert dec2[0].item() == 0


def test_avg_frame_route_matches_oracle():
    """The ablation's average-frame router (fp64 sum in frame order), bit-exact, single and batched."""
    import paper_2604_17397_amd as P

    def gpu(scores, tau, b):
        return P.worst_frame_route(torch.from_numpy(np.asarray(scores, np.float32)).cuda(), tau, b, mode="mean")

    for F in (1, 3, 12, 65, 200):
        for trial in range(3):
            s = si.frame_scores_iid(90 + trial, 1, n_frames=F)[0]
            for tau in (-0.5, -0.3, float(np.float32(s.astype(np.float64).mean()))):
                for b in (0, 4):
                    assert same_route(gpu(s, tau, b), oracle.route(s, tau, b, mode="mean")), (F, tau, b)
    cases = [[16777216.0, 1.0, 1.0, -16777216.0], [0.5, 0.25, 0.25], [np.inf, 1.0], [np.inf, -np.inf],
             [0.2, np.nan, 0.1], [-0.0, -0.0], [1e-45, 1e-45, 0.0], [3.4e38, 3.4e38]]
    for c in cases:
        for tau in (0.0, 0.5, -np.inf):
            assert same_route(gpu(c, tau, 2), oracle.route(np.array(c, np.float32), tau, 2, mode="mean")), (c, tau)
    n = 2048
    scores = si.frame_scores_correlated(78, n)
    idx = (np.arange(n) % 9).astype(np.int32)
    for tau in (-0.5, -0.3):
        dec, qb = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), tau,
                                            block_idx=torch.from_numpy(idx).cuda(), mode="mean")
        dec, qb = dec.cpu().numpy(), qb.cpu().numpy()
        for i in range(n):
            d, q = oracle.route(scores[i], tau, int(idx[i]), mode="mean")
            assert d == dec[i] and q.view(np.uint32) == qb[i].view(np.uint32)
        assert dec[idx == 0].sum() == 0
