"""GPU parity of the expert-skipping rule (Sec. 3.5, Eq. 15-16) and of acceptance / resampling
(Sec. 2.1, Eq. 2-3), through the C ABI, against the fp64 oracle on the same seeded inputs.

Bars.  Thresholds (medians of fp32 ratios) within 2e-6; skip counts and keep masks bit-exact except
tokens with some r_i within 1e-6 of its threshold (counted); acceptance counts bit-exact except
sequences with u within 1e-6 (relative) of alpha at the deciding position; a resampled token is
right when the target mass lies inside its interval of the oracle's cumulative residual, the
interval widened by 1e-5 of the total (fp32 sums in a different order) - it is the oracle's own
token in almost every case (counted)."""
import numpy as np
import pytest
import torch

import paper_2512_21911_amd as S
from oracle import spec_rules_oracle as R
from workloads import rules as WR

pytestmark = pytest.mark.gpu


def gpu_skip(w, beta, m):
    T, k = w.shape
    wg = w.cuda()
    n = torch.full((T,), -7, dtype=torch.int32, device="cuda")
    mask = torch.zeros(T, dtype=torch.int32, device="cuda")
    S.svf_moe_skip(wg, m, torch.as_tensor(beta, dtype=torch.float32).cuda(), n, mask)
    torch.cuda.synchronize()
    bits = mask.cpu().numpy().view(np.uint32)
    keep = ((bits[:, None] >> np.arange(k, dtype=np.uint32)[None, :]) & 1).astype(bool)
    assert (bits >> np.uint32(k) == 0).all() if k < 32 else True
    return n.cpu().numpy(), keep


@pytest.mark.parametrize("T,k", [(1, 2), (7, 8), (4096, 8), (1000, 6), (333, 32), (65, 3)])
def test_calibrated_thresholds_and_skipping(T, k):
    cal = WR.routing_weights(max(T, 50) * 3 + (T % 2), k, seed=T + k)
    beta_ref = R.calibrate_beta(cal.numpy())
    beta = torch.zeros(k - 1, device="cuda")
    S.svf_moe_calibrate(cal.cuda(), beta)
    torch.cuda.synchronize()
    np.testing.assert_allclose(beta.cpu().numpy(), beta_ref, rtol=0, atol=2e-6)
    w = WR.routing_weights(T, k, seed=100 + T)
    r = R.skip_ratios(w.numpy())
    excused = 0
    for m in sorted({1, max(1, k // 2), k - 1}):
        n_ref, keep_ref = R.moe_skip(w.numpy(), beta_ref, m)
        n_gpu, keep_gpu = gpu_skip(w, beta_ref, m)
        near = (np.abs(r[:, :m] - beta_ref[None, :m]) <= 1e-6).any(axis=1)
        bad = (n_gpu != n_ref) | (keep_gpu != keep_ref).any(axis=1)
        assert not (bad & ~near).any(), f"m={m}: {int((bad & ~near).sum())} tokens differ away from a threshold"
        assert (keep_gpu.sum(axis=1) == k - n_gpu).all()
        excused += int(bad.sum())
    print(f"[rules] skip T={T} k={k}: {excused} near-threshold tokens", flush=True)


def test_even_and_odd_calibration_sets_and_ties():
    for T in (2, 3, 1000, 1001):
        cal = WR.routing_weights(T, 4, seed=T)
        beta = torch.zeros(3, device="cuda")
        S.svf_moe_calibrate(cal.cuda(), beta)
        torch.cuda.synchronize()
        np.testing.assert_allclose(beta.cpu().numpy(), R.calibrate_beta(cal.numpy()), rtol=0, atol=2e-6)
    # equal weights: the expert listed first is the lower one
    w = torch.full((3, 5), 0.2)
    n, keep = gpu_skip(w, [0.5, 0.5, 0.7, 0.9], 2)
    assert n.tolist() == [2, 2, 2] and keep[0].tolist() == [False, False, True, True, True]


def gpu_accept(x):
    g = {k: v.cuda() for k, v in x.items()}
    B = x["p_target"].shape[0]
    n = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    r = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    S.svf_accept_resample(g["p_target"], g["p_draft"], g["draft_tokens"], g["u_accept"], g["u_resample"], n, r)
    torch.cuda.synchronize()
    return n.cpu().numpy(), r.cpu().numpy()


def check_accept(x):
    n_gpu, r_gpu = gpu_accept(x)
    n_ref, r_ref, det = R.accept_resample(*(x[k].numpy() for k in ("p_target", "p_draft", "draft_tokens", "u_accept",
                                                                     "u_resample")))
    pt, pd = x["p_target"].double().numpy(), x["p_draft"].double().numpy()
    tok, ua = x["draft_tokens"].numpy(), x["u_accept"].double().numpy()
    B, gamma, V = pt.shape
    same = 0
    for b in range(B):
        if n_gpu[b] != n_ref[b]:
            j = min(n_gpu[b], n_ref[b])
            alpha = min(1.0, pt[b, j, tok[b, j]] / pd[b, j, tok[b, j]])
            assert abs(ua[b, j] - alpha) <= 1e-6 * alpha, f"sequence {b}: accepted {n_gpu[b]} against {n_ref[b]}"
            continue
        if n_ref[b] == gamma:
            assert r_gpu[b] == -1
            continue
        v = int(r_gpu[b])
        assert 0 <= v < V
        cdf, target = det[b]["cdf"], det[b]["target"]
        lo = cdf[v - 1] if v > 0 else 0.0
        slack = 1e-5 * cdf[-1]
        assert lo - slack <= target <= cdf[v] + slack, f"sequence {b}: token {v} does not hold the target mass"
        assert det[b]["resid"][v] > 0 or v == V - 1
        same += int(v == r_ref[b])
    rejected = int((n_ref < gamma).sum())
    print(f"[rules] accept B={B} gamma={gamma} V={V}: mean accepted {n_ref.mean():.2f}, "
          f"{same}/{rejected} resampled tokens identical", flush=True)
    return n_gpu, r_gpu


@pytest.mark.parametrize("B,gamma,V", [(1, 1, 1), (3, 4, 1000), (64, 4, 129280), (16, 8, 128256), (5, 64, 777),
                                        (2, 3, 1025)])
def test_accept_resample(B, gamma, V):
    check_accept(WR.acceptance_inputs(B, gamma, V, seed=B + gamma))


def test_by_hand_and_identical_distributions():
    pt = torch.tensor([[[0.5, 0.2, 0.2, 0.1], [0.1, 0.6, 0.2, 0.1], [0.25, 0.25, 0.25, 0.25]]])
    pd = torch.tensor([[[0.25, 0.25, 0.25, 0.25], [0.1, 0.2, 0.6, 0.1], [0.7, 0.1, 0.1, 0.1]]])
    tok = torch.tensor([[0, 2, 0]], dtype=torch.int32)
    for ua, ur, want in (([0.99, 0.30, 0.0], 0.0, (3, -1)), ([0.99, 0.34, 0.0], 0.5, (1, 1)),
                         ([0.99, 0.2, 0.5], 0.70, (2, 3)), ([0.99, 0.2, 0.5], 0.0, (2, 1))):
        n, r = gpu_accept({"p_target": pt, "p_draft": pd, "draft_tokens": tok, "u_accept": torch.tensor([ua]),
                           "u_resample": torch.tensor([ur])})
        assert (int(n[0]), int(r[0])) == want
    x = WR.acceptance_inputs(4, 4, 5000, seed=9)
    x["p_draft"] = x["p_target"].clone()
    n, r = gpu_accept(x)
    assert n.tolist() == [4] * 4 and r.tolist() == [-1] * 4
    x["u_accept"] = torch.ones(4, 4)                      # u = 1 rejects even alpha = 1: resample from p_theta
    n, r = check_accept(x)
    assert n.tolist() == [0] * 4


def test_same_bits_on_repeated_calls():
    x = WR.acceptance_inputs(32, 4, 129280, seed=3)
    a = gpu_accept(x)
    for _ in range(3):
        b = gpu_accept(x)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
