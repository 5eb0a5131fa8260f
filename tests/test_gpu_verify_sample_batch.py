"""GPU: la_verify_sample_batch (sampling verification of several sequences in one launch) gives,
sequence by sequence, exactly what la_verify_sample gives for it alone - the same arithmetic in the
same order - and la_verify_sample is checked against the oracle in test_gpu_verify_sample.py.  The
oracle is also asked directly for a few sequences (it may legitimately differ on a near-tie, so
most, not all, must agree)."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def make(shape, extra, temperature):
    cur, cnd, cand, u_test, u_final = wl.verify_sample_inputs(shape, extra)
    host = (cur, cnd, cand, u_test, u_final, temperature)
    t = [torch.from_numpy(np.ascontiguousarray(a)).cuda() if a.size else None for a in (cur, cnd, cand, u_test, u_final)]
    return host, dict(logits_cur=t[0], logits_cand=t[1], cand_tokens=t[2], u_test=t[3], u_final=t[4],
                      temperature=temperature,
                      out_tokens=torch.full((shape.N,), -7, dtype=torch.int32, device="cuda"),
                      n_out=torch.full((1,), -7, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("shape,n", [(wl.TINY, 6), (wl.LLAMA2_7B, 8), (wl.LLAMA2_70B, 40), (wl.ragged_shape(1, 10), 3)],
                         ids=lambda x: getattr(x, "name", str(x)))
def test_equals_the_single_calls_and_mostly_the_oracle(shape, n):
    s = shape
    print("case", s.name, n, flush=True)
    temps = [0.5 + 0.25 * (i % 5) for i in range(n)]
    pairs = [make(s, i, temps[i]) for i in range(n)]
    seqs = [d for _, d in pairs]
    binding.la_verify_sample_batch(seqs, s.N, s.G, s.V)
    torch.cuda.synchronize()
    agree = 0
    for i, (host, d) in enumerate(pairs):
        out = torch.full((s.N,), -9, dtype=torch.int32, device="cuda")
        n_out = torch.full((1,), -9, dtype=torch.int32, device="cuda")
        binding.la_verify_sample(d["logits_cur"], d["logits_cand"], d["cand_tokens"], d["u_test"], d["u_final"],
                                 temps[i], s.N, s.G, s.V, out, n_out)
        torch.cuda.synchronize()
        k = int(n_out.item())
        assert int(d["n_out"].item()) == k and torch.equal(d["out_tokens"][:k], out[:k]), i
        if i < 4:
            cur, cnd, cand, u_test, u_final, t = host
            want = orc.verify_sample(cur, cnd, cand, u_test, float(u_final[0]), t, s.N, s.G, s.V)
            agree += d["out_tokens"][:k].tolist() == want
    assert agree >= 3


def test_no_candidates_and_argument_errors():
    V, N = 1000, 4
    rng = np.random.default_rng(0)
    seqs = [dict(logits_cur=torch.from_numpy(rng.standard_normal(V).astype(np.float32)).cuda(),
                 u_final=torch.tensor([0.1 + 0.2 * i], device="cuda"), temperature=1.0,
                 out_tokens=torch.full((N,), -7, dtype=torch.int32, device="cuda"),
                 n_out=torch.full((1,), -7, dtype=torch.int32, device="cuda")) for i in range(3)]
    binding.la_verify_sample_batch(seqs, N, 0, V)
    torch.cuda.synchronize()
    for x in seqs:
        assert int(x["n_out"].item()) == 1 and 0 <= int(x["out_tokens"][0].item()) < V
        want = orc.verify_sample(x["logits_cur"].cpu().numpy(), np.zeros((0, N - 1, V), np.float32),
                                 np.zeros((0, N - 1), np.int32), np.zeros((N - 1, 0), np.float32),
                                 float(x["u_final"].item()), 1.0, N, 0, V)
        assert x["out_tokens"][:1].tolist() == want
    seqs[1]["temperature"] = 0.0
    with pytest.raises(binding.LaError, match="descriptor 1"):
        binding.la_verify_sample_batch(seqs, N, 0, V)
