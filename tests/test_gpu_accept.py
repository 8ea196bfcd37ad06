"""GPU parity of the softmax statistics and the modified rejection step against the CPU oracle.

Decisions (n_accepted, next token) are integer results and must be bit-exact given identical p, q
and uniforms; probabilities produced by the GPU softmax are compared by tolerance
(1e-6 + 1e-5 * p) and then handed, bit for bit, to the oracle's rejection step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _dists(seed, B, K, V, zero_frac=0.0):
    g = torch.Generator().manual_seed(seed)
    def mk(rows):
        x = torch.rand((B, rows, V), generator=g).pow(6)
        if zero_frac:
            x = x * (torch.rand((B, rows, V), generator=g) > zero_frac)
            x[..., 0] += 1e-3
        return (x / x.sum(-1, keepdim=True)).float()
    p = mk(K + 1)
    q = p[:, :K] * (0.25 + 1.5 * torch.rand((B, K, V), generator=g))     # a draft that resembles the target
    q = (q / q.sum(-1, keepdim=True).clamp_min(1e-30)).float()
    return p, q


@pytest.mark.parametrize("B,K,V", [(3, 4, 1024), (5, 8, 1000), (2, 1, 50), (4, 0, 333), (64, 8, 4099), (2, 15, 32000),
                                   (3, 4, 40001), (1, 2, 131071)])   # the last two: several vocabulary segments, rows not 16-byte aligned
def test_speculative_accept_bit_exact(B, K, V):
    p, q = _dists(B * 1000 + K, B, K, V, zero_frac=0.3 if V < 2000 else 0.0)
    # draft tokens drawn from q by the oracle's sampler so that acceptance is non-trivial
    ud = si.uniforms(1, "ud", (B, max(K, 1))).numpy()
    d = np.array([[oracle.sample(q[b, i].numpy(), ud[b, i]) for i in range(K)] for b in range(B)], dtype=np.int32).reshape(B, K)
    u = si.uniforms(2, "u", (B, K + 1))
    ona, onx = oracle.speculative_accept(p.numpy(), q.numpy(), d, u.numpy())
    na, nx = sv.ss_speculative_accept(p.to(dev()), q.to(dev()) if K else torch.zeros(1, device=dev()),
                                      torch.tensor(d).to(dev()) if K else torch.zeros(1, dtype=torch.int32, device=dev()),
                                      u.to(dev()))
    assert na.cpu().tolist() == ona.tolist()
    assert nx.cpu().tolist() == onx.tolist()
    if K >= 4 and B >= 3:
        assert len(set(ona.tolist())) > 1          # the case really mixes accept counts


def test_accept_special_cases_match_oracle():
    B, K, V = 4, 3, 257
    p, q = _dists(7, B, K, V)
    u = si.uniforms(3, "u", (B, K + 1))
    d = si.token_ids(3, "d", (B, K), V)
    cases = []
    cases.append((p, p[:, :K].clone(), d))                                   # q = p: everything accepted
    qd = torch.zeros_like(q); qd[..., :5] = 0.2
    pd = p.clone(); pd[..., :5] = 0; pd = pd / pd.sum(-1, keepdim=True)
    cases.append((pd, qd, si.token_ids(4, "d", (B, K), 5)))                 # disjoint supports: a = 0
    tiny = torch.full_like(p, 1e-12)
    cases.append((tiny, tiny[:, :K].clone(), d))                             # all weights quantise to 0 -> argmax
    onehot_p = torch.nn.functional.one_hot(si.token_ids(5, "t", (B, K + 1), V).long(), V).float()
    cases.append((onehot_p, torch.nn.functional.one_hot(d.long(), V).float(), d))   # greedy as one-hot
    for pp, qq, dd in cases:
        ona, onx = oracle.speculative_accept(pp.numpy(), qq.numpy(), dd.numpy(), u.numpy())
        na, nx = sv.ss_speculative_accept(pp.to(dev()), qq.to(dev()), dd.to(dev()), u.to(dev()))
        assert na.cpu().tolist() == ona.tolist() and nx.cpu().tolist() == onx.tolist()


@pytest.mark.parametrize("rows,V,T", [(7, 1024, 1.0), (3, 1000, 0.8), (2, 50, 2.5), (5, 32000, 1.0), (17, 128256, 0.8)])
def test_softmax_close_to_oracle(rows, V, T):
    l = si.normal(11, "l", (rows, V), 2.0)
    got = sv.ss_softmax(l.to(dev()), T).cpu().numpy()
    ref = oracle.softmax(l.numpy(), T)
    assert np.all(np.abs(got - ref) <= 1e-6 + 1e-5 * ref)
    assert np.allclose(got.astype(np.float64).sum(-1), 1.0, atol=1e-5)


@pytest.mark.parametrize("B,K,V,T", [(4, 4, 1024, 1.0), (6, 8, 5000, 0.8), (3, 2, 333, 1.3)])
def test_fused_logits_path_equals_materialised_path_and_oracle(B, K, V, T):
    pl, ql, u, ud = si.accept_workload(21, B, K, V)
    qp = oracle.softmax(ql.numpy(), T)
    d = np.array([[oracle.sample(qp[b, i], ud[b, i].item()) for i in range(K)] for b in range(B)], dtype=np.int32)
    D = dev()
    p_out = torch.empty((B, K + 1, V), device=D)
    q_out = torch.empty((B, K, V), device=D)
    na, nx = sv.ss_speculative_accept_logits(pl.to(D), ql.to(D), T, torch.tensor(d).to(D), u.to(D), p_out=p_out, q_out=q_out)
    # (1) the materialised probabilities are the ones ss_softmax produces, bit for bit
    assert torch.equal(p_out, sv.ss_softmax(pl.to(D), T)) and torch.equal(q_out, sv.ss_softmax(ql.to(D), T))
    # (2) the fused result equals the rejection step on those probabilities, on the GPU and in the oracle
    na2, nx2 = sv.ss_speculative_accept(p_out, q_out, torch.tensor(d).to(D), u.to(D))
    ona, onx = oracle.speculative_accept(p_out.cpu().numpy(), q_out.cpu().numpy(), d, u.numpy())
    assert na.cpu().tolist() == na2.cpu().tolist() == ona.tolist()
    assert nx.cpu().tolist() == nx2.cpu().tolist() == onx.tolist()
    # (3) and the probabilities are within tolerance of the oracle's fp64 softmax
    ref = oracle.softmax(pl.numpy(), T)
    assert np.all(np.abs(p_out.cpu().numpy() - ref) <= 1e-6 + 1e-5 * ref)


@pytest.mark.parametrize("B,K,V", [(24, 3, 50000), (16, 8, 32000), (10, 5, 128256), (20, 4, 65536)])
def test_staged_row_statistics_skip_rows_without_changing_the_result(B, K, V):
    """Large logits without materialised outputs: the statistics are taken in stages that skip the rows
    behind a sequence's first rejection.  Same counts and tokens as the path that covers every row (which
    the tests above pin to the oracle), whatever stale statistics the workspace holds for skipped rows."""
    T, D = 0.8, dev()
    other = si.accept_workload(50, B, K, V, device=D)
    sv.ss_speculative_accept_logits(other[0], other[1], T, torch.zeros((B, K), dtype=torch.int32, device=D), other[2])  # leaves foreign statistics behind
    pl, ql, u, ud = si.accept_workload(51, B, K, V, device=D)
    q = sv.ss_softmax(ql, T)
    d = torch.empty((B, K), dtype=torch.int32, device=D)
    for i in range(K):
        _, tok = sv.ss_speculative_accept(q[:, i].contiguous()[:, None], torch.zeros(1, device=D), torch.zeros(1, dtype=torch.int32, device=D),
                                          ud[:, i:i + 1].contiguous())
        d[:, i] = tok
    p_out = torch.empty((B, K + 1, V), device=D)
    na_full, nx_full = sv.ss_speculative_accept_logits(pl, ql, T, d, u, p_out=p_out)
    na, nx = sv.ss_speculative_accept_logits(pl, ql, T, d, u)
    assert na.cpu().tolist() == na_full.cpu().tolist() and nx.cpu().tolist() == nx_full.cpu().tolist()
    ona, onx = oracle.speculative_accept(p_out.cpu().numpy(), q.cpu().numpy(), d.cpu().numpy(), u.cpu().numpy())
    assert na.cpu().tolist() == ona.tolist() and nx.cpu().tolist() == onx.tolist()
    assert 0 < sum(na.cpu().tolist()) < B * K     # both early rejections and surviving sequences occur


def test_gpu_rejection_step_emits_the_target_distribution():
    """The guarantee of Section 3, measured on the kernels themselves (no oracle involved): 2^18 sequences
    share one pair of rows p, q over 8 tokens; each draws d ~ q with the library's sampler, runs the
    rejection step, and emits d if accepted, else the resampled token.  The histogram of the emitted
    token must be p (chi-square, 7 degrees of freedom, p-value > 1e-4; the same test rejects q), and the
    acceptance rate must be 1 - ||p - q||_1 / 2 within four standard deviations."""
    from scipy import stats
    B, V, D = 1 << 18, 8, dev()
    g = torch.Generator().manual_seed(77)
    p1 = torch.softmax(torch.randn(V, generator=g), 0)
    q1 = torch.softmax(torch.randn(V, generator=g) * 1.5, 0)
    p = p1.to(D).repeat(B, 1, 1).repeat(1, 2, 1).contiguous()       # [B, K + 1 = 2, V]: the bonus row is p again
    q = q1.to(D).repeat(B, 1, 1).contiguous()                        # [B, 1, V]
    ud = si.uniforms(77, "chi_ud", (B, 1), device=D)
    ua = si.uniforms(77, "chi_ua", (B, 2), device=D)
    zf, zi = torch.zeros(1, device=D), torch.zeros(1, dtype=torch.int32, device=D)
    _, d = sv.ss_speculative_accept(q, zf, zi, ud)                   # K = 0: a plain sample from q per sequence
    na, nx = sv.ss_speculative_accept(p, q, d[:, None].contiguous(), ua)
    emitted = torch.where(na == 1, d, nx).cpu().numpy()
    counts = np.bincount(emitted, minlength=V).astype(np.float64)
    pe, qe = p1.double().numpy(), q1.double().numpy()
    chi_p = ((counts - B * pe) ** 2 / (B * pe)).sum()
    chi_q = ((counts - B * qe) ** 2 / (B * qe)).sum()
    assert stats.chi2.sf(chi_p, V - 1) > 1e-4
    assert stats.chi2.sf(chi_q, V - 1) < 1e-12
    rate, expect = float((na == 1).float().mean()), 1.0 - 0.5 * np.abs(pe - qe).sum()
    assert abs(rate - expect) < 4.0 * np.sqrt(expect * (1 - expect) / B)


def test_greedy_accept_matches_oracle_with_ties():
    B, K, V = 9, 5, 1024
    l = si.normal(31, "l", (B, K + 1, V), 2.0)
    l[0, 2, 700] = l[0, 2, 20] = l[0, 2].max() + 1            # tie: lowest index wins
    tgt = l.argmax(-1)
    d = tgt[:, :K].to(torch.int32).clone()
    for b in range(B):
        if b % (K + 1) < K:
            d[b, b % (K + 1)] = (d[b, b % (K + 1)] + 1) % V
    ona, onx = oracle.greedy_accept(l.numpy(), d.numpy())
    na, nx = sv.ss_greedy_accept(l.to(dev()), d.to(dev()))
    assert na.cpu().tolist() == ona.tolist() and nx.cpu().tolist() == onx.tolist()
    assert onx[0] == 20 or ona[0] < 2


def test_standalone_accept_workload_full_size():
    """batch 64, K = 8, vocab 128256, temperature 0.8: the launch configuration the bench times."""
    B, K, V, T = 64, 8, 128256, 0.8
    D = dev()
    pl, ql, u, ud = si.accept_workload(41, B, K, V, device=D)
    q = sv.ss_softmax(ql, T)
    d = torch.empty((B, K), dtype=torch.int32, device=D)
    for i in range(K):   # draft tokens ~ q: the K = 0 case of the rejection step is a plain sample (checked below)
        qi = q[:, i].contiguous()
        _, tok = sv.ss_speculative_accept(qi[:, None], torch.zeros(1, device=D), torch.zeros(1, dtype=torch.int32, device=D), ud[:, i:i + 1].contiguous())
        d[:, i] = tok
    p_out = torch.empty((B, K + 1, V), device=D)
    q_out = torch.empty((B, K, V), device=D)
    na, nx = sv.ss_speculative_accept_logits(pl, ql, T, d, u, p_out=p_out, q_out=q_out)
    assert torch.equal(q_out, q)
    # oracle on the GPU's own probability bits: every sequence, bit-exact
    pc, qc, dc, uc = p_out.cpu().numpy(), q_out.cpu().numpy(), d.cpu().numpy(), u.cpu().numpy()
    ona, onx = oracle.speculative_accept(pc, qc, dc, uc)
    assert na.cpu().tolist() == ona.tolist() and nx.cpu().tolist() == onx.tolist()
    # sampled draft tokens: spot-check against the oracle's sampler
    udc = ud.cpu().numpy()
    for b in range(0, B, 7):
        for i in (0, K - 1):
            assert dc[b, i] == oracle.sample(qc[b, i], udc[b, i])
    # sampled rows of the probabilities against the oracle's fp64 softmax
    plc = pl.cpu().numpy()
    for b, i in ((0, 0), (17, 3), (63, 8)):
        ref = oracle.softmax(plc[b, i], T)
        assert np.all(np.abs(pc[b, i] - ref) <= 1e-6 + 1e-5 * ref)
    mean_acc = float(np.mean(ona))
    assert 1.0 < mean_acc < 6.0       # sanity band for this workload (per-position accept ~ 0.75)


def test_bad_arguments_are_rejected_on_the_host():
    D = dev()
    p = torch.zeros((1, 2, 8), device=D)
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_softmax(p, 0.0)
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_accept_logits(p, p[:, :1].contiguous(), -1.0, torch.zeros((1, 1), dtype=torch.int32, device=D),
                                        torch.zeros((1, 2), device=D))
