"""GPU parity: rapid_retrieve (C ABI) against the oracle.  Similarities: fp32 dot products of `dim`
terms against float64, |gpu - ref| <= 2e-6.  Selection: an integer decision taken from floating point
values, so it must equal the oracle's exactly unless the oracle's own margin (distance of a similarity
to the threshold, or of the k-th to the k+1-th value) is below 1e-5; such cases are counted, and the
GPU's selection is then checked against its own similarities instead."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_20330_amd import binding
from paper_2502_20330_amd import workloads as wl

pytestmark = pytest.mark.gpu

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    import gpu_util
    gu = gpu_util
    yield


def run(emb, q, k, thr, what):
    sim, sel, cnt = gu.rapid().rapid_retrieve(torch.from_numpy(emb).cuda(), torch.from_numpy(q).cuda(), k, thr)
    torch.cuda.synchronize()
    sim, sel, cnt = sim.cpu().numpy(), sel.cpu().numpy(), int(cnt.cpu()[0])
    ref_sim, ref_sel, margin = oracle.retrieve(emb, q, k, thr)
    assert np.max(np.abs(sim - ref_sim)) <= 2e-6, what
    assert np.all(sel[cnt:] == -1) and np.all(np.diff(sel[:cnt]) > 0), what
    near = margin < 1e-5
    if not near:
        assert cnt == len(ref_sel) and np.array_equal(sel[:cnt], ref_sel), what
    else:       # valid with respect to the GPU's own similarities: same rule applied to them with numpy
        order = sorted(range(len(sim)), key=lambda i: (-sim[i], i))[:k]
        own = sorted(i for i in order if sim[i] >= np.float32(thr))
        assert sel[:cnt].tolist() == own, what
    print(f"[{what}] n={len(emb)} k={k} selected={cnt} margin={margin:.2e} near_tie={near} "
          f"max_sim_err={np.max(np.abs(sim - ref_sim)):.2e}")
    return near


def test_paper_setting_128k_context():
    """256 chunks of 512 tokens (a 128K-token context), dimension 1024, k from the 1/24 rule, threshold 0.3."""
    emb, q = wl.gen_retrieval_inputs(256)
    k = oracle.retrieval_top_k(131072)
    assert k == 10
    assert not run(emb, q, k, 0.3, "128k")


@pytest.mark.parametrize("n,dim,k,thr,salt", [(1, 4, 1, 0.3, 0), (3, 8, 5, -1.0, 1), (64, 1024, 8, 0.3, 2),
                                               (257, 768, 20, 0.2, 3), (1000, 256, 85, 0.0, 4),
                                               (1024, 64, 1024, -2.0, 5), (500, 1024, 7, 0.95, 6)])
def test_sizes_thresholds_and_top_k(n, dim, k, thr, salt):
    emb, q = wl.gen_retrieval_inputs(n, dim, salt=salt)
    run(emb, q, k, thr, f"n{n}_dim{dim}_k{k}_thr{thr}")


def test_exact_ties_take_the_lower_index_and_zero_vectors_score_zero():
    q = np.zeros(8, dtype=np.float32); q[0] = 1.0
    emb = np.zeros((6, 8), dtype=np.float32)
    emb[0, 0] = 1; emb[1, 1] = 1; emb[2, 0] = 1; emb[2, 1] = 1; emb[3, 0] = -1; emb[5, 0] = 2
    for k, expect in ((1, [0]), (2, [0, 5]), (3, [0, 2, 5]), (6, [0, 2, 5])):
        sim, sel, cnt = gu.rapid().rapid_retrieve(torch.from_numpy(emb).cuda(), torch.from_numpy(q).cuda(), k, 0.3)
        torch.cuda.synchronize()
        assert sel.cpu().numpy()[:int(cnt.cpu()[0])].tolist() == expect
        assert sim.cpu().numpy()[4] == 0.0


def test_bad_arguments_return_error_codes():
    r = gu.rapid()
    e = torch.zeros(1025, 8, device="cuda"); q = torch.zeros(8, device="cuda")
    with pytest.raises(binding.RapidError) as ex:
        r.rapid_retrieve(e, q, 4)
    assert ex.value.status == binding.RAPID_EUNSUPPORTED
    with pytest.raises(binding.RapidError) as ex:
        r.rapid_retrieve(e[:10, :6].contiguous(), q[:6].contiguous(), 4)
    assert ex.value.status == binding.RAPID_EUNSUPPORTED
