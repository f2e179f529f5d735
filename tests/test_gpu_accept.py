"""GPU parity of the acceptance rule as a call of its own (sd_accept; Section 3.1) against the oracle's
orc_accept on the same fp32 logits, draft distributions, candidates and uniforms."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import api
from paper_2505_08600_amd import datagen as dg

pytestmark = pytest.mark.gpu


def synthetic_case(seed, B, gamma, V, rho, T):
    """Config-5 style inputs without a model: target logits N(0, 3), q = softmax(rho * logits + (1 - rho) * 4 N(0,1)),
    candidates drawn from q by the oracle's own inverse CDF, uniforms on the 2^-24 grid."""
    logits = np.stack([3.0 * dg.make_logit_noise(seed, b, 100 + i, V) for b in range(B) for i in range(gamma + 1)])
    logits = logits.reshape(B, gamma + 1, V).astype(np.float32)
    q = np.zeros((B, max(gamma, 1), V), np.float32)
    cand = np.zeros((B, max(gamma, 1)), np.int32)
    for b in range(B):
        ud = dg.make_uniforms(seed, dg.DRAFT_STREAM, b, 0, max(gamma, 1))
        for i in range(gamma):
            z = rho * logits[b, i] + (1.0 - rho) * 4.0 * dg.make_logit_noise(seed, b, i, V)
            q[b, i] = oracle.softmax_T(z.astype(np.float32), T if T > 0 else 1.0)
            cand[b, i] = oracle.sample_cdf(q[b, i].astype(np.float64), float(ud[i]))[0]
    u = np.stack([dg.make_uniforms(seed, dg.VERIFY_STREAM, b, 0, gamma + 1) for b in range(B)])
    return logits, q[:, :gamma], cand[:, :gamma], u


def check_against_oracle(logits, q, cand, u, T, na, nx, thr=1e-5):
    """Bit-exact decisions, unless the oracle's own margin is below the fp32 threshold.  -> flagged count"""
    B, rows, V = logits.shape
    gamma = rows - 1
    flagged = 0
    for b in range(B):
        r_na, r_nx, mg = oracle.accept(logits[b], q[b] if gamma and T > 0 else None, cand[b], u[b], T)
        if (int(na[b]), int(nx[b])) == (r_na, r_nx):
            continue
        flagged += 1
        if int(na[b]) != r_na:
            i = min(int(na[b]), r_na)
            lim = thr if T > 0 else thr * float(np.abs(logits[b, i]).max())
            assert mg[i] < lim, (b, int(na[b]), r_na, mg)
        elif T > 0:
            w = oracle.next_weights(logits[b], q[b] if gamma else None, r_na, T)
            assert oracle.cdf_distance(w, float(u[b, gamma]), int(nx[b])) < thr, (b, int(nx[b]), r_nx)
        else:
            assert mg[gamma] < thr * float(np.abs(logits[b, r_na]).max())
    return flagged


@pytest.mark.parametrize("V,gamma,T,rho", [(32000, 8, 1.0, 0.5), (32000, 8, 0.7, 0.9), (32000, 5, 1.0, 0.0),
                                           (32000, 5, 0.0, 0.9), (50000, 3, 1.0, 0.5), (1024, 4, 1.0, 0.5),
                                           (32000, 0, 1.0, 0.0)])
def test_accept_alone_matches_oracle(V, gamma, T, rho):
    print(f"sd_accept V={V} gamma={gamma} T={T} rho={rho}", flush=True)
    B = 6
    logits, q, cand, u = synthetic_case(91, B, gamma, V, rho, T)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    na = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    nx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    ws = torch.full((3 * B * (gamma + 1),), float("nan"), device="cuda")   # contents on entry must not matter
    api.sd_accept(dev(logits), gamma, T, dev(cand) if gamma else None, dev(q) if gamma and T > 0 else None,
                  dev(u) if T > 0 else None, na, nx, ws)
    torch.cuda.synchronize()
    na_h, nx_h = na.cpu().numpy(), nx.cpu().numpy()
    flagged = check_against_oracle(logits, q, cand, u, T, na_h, nx_h)
    print(f"  n_acc={na_h.tolist()} flagged={flagged}", flush=True)
    assert flagged <= 1
    if gamma >= 5 and 0 < rho < 1 and T > 0:
        assert len(set(na_h.tolist())) >= 2   # the case exercises accept, reject and the residual draw


def test_accept_argument_errors():
    L = api.lib()
    x = torch.zeros(8, device="cuda")
    i = torch.zeros(8, dtype=torch.int32, device="cuda")
    p = lambda t: t.data_ptr()
    assert L.sd_accept(None, 1, 1, 8, 1.0, p(i), p(x), p(x), p(i), p(i), p(x), None) == api.SD_EINVAL
    assert L.sd_accept(p(x), 1, 16, 8, 1.0, p(i), p(x), p(x), p(i), p(i), p(x), None) == api.SD_ECAP
    assert L.sd_accept(p(x), 1, 1, 6, 1.0, p(i), p(x), p(x), p(i), p(i), p(x), None) == api.SD_EINVAL
    assert L.sd_accept(p(x), 1, 1, 8, 1.0, p(i), None, p(x), p(i), p(i), p(x), None) == api.SD_EINVAL
    assert L.sd_accept(p(x), 1, 1, 8, 1.0, p(i), p(x), p(x), p(i), p(i), None, None) == api.SD_EINVAL


@pytest.mark.parametrize("nt", [1, 0])
def test_stream_read_probe_reads_every_word_exactly_once(nt):
    """In its checking mode the read probe folds every 32-bit word it reads into the scratch word with XOR: the
    result equals the XOR of the buffer iff both patterns cover every 16-byte vector exactly once, for sizes on
    and off the grid's granularity; and in measuring mode the word is left alone."""
    print(f"stream read probe, nontemporal pattern = {nt}", flush=True)
    try:
        rng = np.random.default_rng(7)
        for n_words in (4, 4 * 255, 4 * 2048 + 4, 4 * 65536 * 3 + 12, 1 << 22):
            w = rng.integers(0, 1 << 32, n_words, dtype=np.uint64).astype(np.uint32)
            buf = torch.from_numpy(w.view(np.int32)).cuda()
            word = torch.zeros(1, dtype=torch.int32, device="cuda")
            api.set_option("stream_read_nt", nt + 2)
            api.stream_read(buf, word)
            torch.cuda.synchronize()
            assert int(word.item()) & 0xffffffff == int(np.bitwise_xor.reduce(w)), f"{n_words} words: a vector was skipped or read twice"
            api.set_option("stream_read_nt", nt)
            word.zero_()
            api.stream_read(buf, word)
            torch.cuda.synchronize()
            assert int(word.item()) == 0
    finally:
        api.set_option("stream_read_nt", 1)
