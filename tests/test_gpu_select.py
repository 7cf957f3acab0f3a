"""GPU parity of the integer / decision kernels, through the C ABI: fan-out selection (bit-exact on the
oracle's logits), the branch sampler and lossless verification (decisions equal wherever the oracle's own
margin is above 1e-4)."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import MARGIN, dev_f32, dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


@pytest.mark.parametrize("V,rows,F,ties", [(1024, 10, 2, 3), (1000, 7, 5, 40), (128256, 6, 4, 2), (128256, 6, 8, 500),
                                           (33, 3, 16, 8), (128256, 96, 4, 0), (128256, 1, 16, 2), (9000, 24, 3, 9),
                                           (128256, 600, 2, 0)])
def test_top_f_bit_exact_on_oracle_logits(B, V, rows, F, ties):
    z = I.make_logits(rows, V, seed=V + rows, n_ties=ties)
    g = np.random.default_rng(V)
    z[0, g.integers(0, V, 3)] = np.nan                      # NaN ranks last
    z[min(1, rows - 1), g.integers(0, V, 3)] = -np.inf
    z[min(2, rows - 1), :4] = [0.0, -0.0, 0.0, -0.0]        # signed zeros tie
    exclude = np.array([int(np.argmax(np.nan_to_num(z[r], nan=-np.inf))) if r % 3 != 2 else -1 for r in range(rows)],
                       dtype=np.int32)                      # greedy drafting: the excluded token is the row's top-1
    want = np.stack([O.top_f_ids(z[r], F, exclude=None if exclude[r] < 0 else int(exclude[r])) for r in range(rows)])
    ids = torch.full((rows, F), -7, dtype=torch.int32, device="cuda")
    B.ssd_top_f(dev_f32(z), dev_i32(exclude), F, ids)
    torch.cuda.synchronize()
    assert np.array_equal(ids.cpu().numpy(), want)
    # the same with a workspace: several workgroups share a row when the vocabulary is large (the second call finds
    # the first call's candidates in the workspace and must not be misled by them)
    ws = torch.full((B.ssd_top_f_workspace_bytes(rows),), 0xff, dtype=torch.uint8, device="cuda")
    for _ in range(2):
        ids.fill_(-7)
        B.ssd_top_f(dev_f32(z), dev_i32(exclude), F, ids, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), want)
    # no exclusion list at all
    want = np.stack([O.top_f_ids(z[r], F) for r in range(rows)])
    for w in (None, ws):
        ids.fill_(-7)
        B.ssd_top_f(dev_f32(z), None, F, ids, workspace=w)
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), want)


def test_top_f_rejects_bad_sizes(B):
    z = dev_f32(np.zeros((2, 8)))
    ids = torch.zeros((2, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(B.SsdError) as e:
        B.ssd_top_f(z, None, 8, ids)                        # F + 1 > V
    assert e.value.status == B.SSD_EINVAL
    with pytest.raises(B.SsdError):
        B.ssd_top_f(z, None, 17, ids)                       # F > SSD_MAX_F
    # zero rows is a no-op
    assert B.lib.ssd_top_f(z.data_ptr(), 8, None, 0, 8, 2, ids.data_ptr(), None, None) == B.SSD_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("V,rows", [(1024, 10), (128256, 24)])
def test_sampler_greedy_and_gumbel(B, V, rows):
    z = I.make_logits(rows, V, seed=5 * V, n_ties=2)
    out = torch.zeros(rows, dtype=torch.int32, device="cuda")
    temps = np.zeros(rows, np.float32)
    B.ssd_sample(dev_f32(z), dev_f32(temps), seed=99, row_base=0, step=0, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), [int(O.top_f_ids(z[r], 1)[0]) for r in range(rows)])
    temps = np.where(np.arange(rows) % 2 == 0, 1.0, 0.7).astype(np.float32)
    for step in (0, 3):
        B.ssd_sample(dev_f32(z), dev_f32(temps), seed=99, row_base=48, step=step, out=out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        n_checked = 0
        for r in range(rows):
            tok, margin = O.sample_token(z[r], float(temps[r]), O.gumbel(99, O.STREAM_DRAFT, 48 + r, step, V))
            if margin > MARGIN:
                assert got[r] == tok, (r, step)
                n_checked += 1
        assert n_checked >= rows - 1
    # the draws differ between steps and rows (not all equal to the greedy token)
    greedy = np.array([int(O.top_f_ids(z[r], 1)[0]) for r in range(rows)])
    assert (got != greedy).any()


@pytest.mark.parametrize("V,rows,scale,temp", [(128256, 24, 1.0, 1.0), (128256, 48, 3.0, 0.3), (4099, 7, 50.0, 0.05),
                                               (128256, 6, 0.01, 2.0), (1024, 300, 1.0, 0.7)])
def test_sampler_fp32_preselection_gives_the_fp64_token(B, V, rows, scale, temp):
    """Sampled rows are scanned in fp32 and only the tokens within the error bound of the maximum are scored in fp64.
    The token must be the one a full fp64 scan gives, also with large logits over a small temperature, planted
    near-ties, infinities and NaN."""
    z = (I.make_logits(rows, V, seed=7 * V + rows, n_ties=5) * scale).astype(np.float32)
    g = np.random.default_rng(V + rows)
    for r in range(rows):
        top = int(np.argmax(np.nan_to_num(z[r], nan=-np.inf)))
        z[r, g.integers(0, V, 4)] = np.nextafter(z[r, top], np.float32(-np.inf))     # runners-up one ulp below the top
    z[0, 5] = np.nan
    z[min(1, rows - 1), 9] = -np.inf
    if rows > 3:
        z[3, 11] = np.inf                                       # an infinite logit wins whatever the noise
    temps = dev_f32(np.full(rows, temp, np.float32))
    zd = dev_f32(z)
    outs = []
    for sample in (B.ssd_sample_fp64_scan, B.ssd_sample):
        per_step = []
        for step in range(3):
            out = torch.full((rows,), -5, dtype=torch.int32, device="cuda")
            sample(zd, temps, seed=1234, row_base=17, step=step, out=out)
            torch.cuda.synchronize()
            per_step.append(out.cpu().numpy())
        outs.append(np.stack(per_step))
    assert np.array_equal(outs[0], outs[1])
    if rows > 3:
        assert (outs[1][:, 3] == 11).all()
    # and it is a sample, not the argmax: steps differ somewhere
    assert (outs[1][0] != outs[1][1]).any() or rows <= 7


def _verify_case(B, V, K, nb, seed, temps, close_draft):
    g = np.random.default_rng(seed)
    zt = (g.standard_normal((nb, K + 1, V)) * 2.0).astype(np.float32)
    if close_draft:
        zd = (zt[:, :K] + g.standard_normal((nb, K, V)).astype(np.float32) * 0.3).astype(np.float32)
    else:
        zd = (g.standard_normal((nb, K, V)) * 2.0).astype(np.float32)
    spec = np.zeros((nb, K), np.int32)
    for b in range(nb):
        for i in range(K):
            if temps[b] == 0:
                # greedy draft: mostly the target's argmax so that long accept runs occur
                spec[b, i] = int(np.argmax(zt[b, i])) if g.random() < 0.8 else int(g.integers(0, V))
            else:
                q = O.softmax_T(zd[b, i], float(temps[b]))
                spec[b, i] = int(min(np.searchsorted(np.cumsum(q), g.random()), V - 1))
    k_out = torch.full((nb,), -9, dtype=torch.int32, device="cuda")
    t_out = torch.full((nb,), -9, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
    B.ssd_verify(dev_f32(zt), dev_f32(zd), dev_i32(spec), dev_f32(temps), seed, k_out, t_out, ws)
    torch.cuda.synchronize()
    return zt, zd, spec, k_out.cpu().numpy(), t_out.cpu().numpy()


@pytest.mark.parametrize("V,K,nb,close", [(1024, 4, 12, True), (1024, 5, 8, False), (128256, 5, 3, True),
                                          (40000, 2, 40, True),      # rows and sequences are cut into different numbers of parts
                                          (3, 15, 2, True), (17, 1, 33, False), (128256, 15, 2, True)])
def test_verify_matches_oracle(B, V, K, nb, close):
    temps = np.array([0.0 if b % 3 == 0 else (1.0 if b % 3 == 1 else 0.6) for b in range(nb)], np.float32)
    seed = 4242 + V + K
    zt, zd, spec, k_got, t_got = _verify_case(B, V, K, nb, seed, temps, close)
    ks = []
    for b in range(nb):
        want = O.verify(zt[b], zd[b], spec[b], float(temps[b]), seed, seq=b)
        ks.append(want.accept_len)
        if all(m > MARGIN for m in want.accept_margin):
            assert k_got[b] == want.accept_len, b
            if want.bonus_margin > MARGIN:
                assert t_got[b] == want.bonus, b
    assert len(set(ks)) > 1 or nb < 8                         # several accept lengths were exercised


def test_verify_greedy_without_draft_logits_and_full_acceptance(B):
    V, K, nb = 1024, 5, 4
    g = np.random.default_rng(8)
    zt = g.standard_normal((nb, K + 1, V)).astype(np.float32)
    spec = np.argmax(zt[:, :K], axis=-1).astype(np.int32)      # the draft proposes exactly the target's choices
    spec[2, 3] = (spec[2, 3] + 1) % V                          # one mismatch
    k_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    t_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
    temps = dev_f32(np.full(nb, 1.0, np.float32))              # ignored: no draft logits => greedy
    B.ssd_verify(dev_f32(zt), None, dev_i32(spec), temps, 1, k_out, t_out, ws)
    torch.cuda.synchronize()
    assert list(k_out.cpu().numpy()) == [K, K, 3, K]
    assert list(t_out.cpu().numpy()) == [int(np.argmax(zt[b, k])) for b, k in zip(range(nb), [K, K, 3, K])]


def test_verify_identical_models_accept_all(B):
    V, K, nb = 1024, 5, 6
    g = np.random.default_rng(9)
    z = g.standard_normal((nb, K + 1, V)).astype(np.float32)
    temps = np.full(nb, 1.0, np.float32)
    spec = g.integers(0, V, (nb, K)).astype(np.int32)
    k_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    t_out = torch.zeros(nb, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
    B.ssd_verify(dev_f32(z), dev_f32(z[:, :K]), dev_i32(spec), dev_f32(temps), 77, k_out, t_out, ws)
    torch.cuda.synchronize()
    assert (k_out.cpu().numpy() == K).all()


def test_backup_random_tokens_equal_the_oracles(B):
    """Sec. 4.3 random-token backup: bit-exact against the oracle's generator, batch of sequences, full vocabulary."""
    for seed, nb, K, V in [(0, 1, 5, 128256), (12345678901234567, 16, 7, 128256), (7, 3, 15, 97), (1, 5, 1, 1)]:
        out = torch.full((nb, K), -1, dtype=torch.int32, device="cuda")
        B.ssd_backup_random(seed, V, out)
        torch.cuda.synchronize()
        want = np.array([O.random_speculation(seed, b, K, V)[0] for b in range(nb)], np.int32)
        assert np.array_equal(out.cpu().numpy(), want), (seed, nb, K, V)
