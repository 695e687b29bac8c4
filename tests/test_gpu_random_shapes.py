"""Seeded random shapes: m, n (from 1 upward, so also n < m, where g_bar lies
inside span{u_k} and G c cancels it), storage type (fp32, bf16, fp16), leading
dimension and base-pointer offset drawn at random (ragged tiles, every alignment,
row shards of a wider matrix), each compared with the oracle: Gram, whole step
and the operator on a random vector.  The tolerance of the whole step is the one
the header documents, computed from the oracle's own quantities."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_05069_amd as qn
from parity_util import rel, step_tolerance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
M_CHOICES = [1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 31, 32, 33, 40, 48, 49, 63, 64]
N_EDGES = [1, 2, 3, 63, 64, 65, 255, 256, 257, 511, 513, 1023, 1025, 2047, 2049, 4095, 4097,
           8193, 16383, 16384, 16385, 16897]


def stored(t):
    t = t.contiguous()      # bf16 goes to the oracle as bit patterns, fp16 and fp32 as numpy's types
    return t.view(torch.uint16).cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_match_the_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    for case in range(14):
        m = int(rng.choice(M_CHOICES))
        u = rng.random()
        if u < 0.3:
            n = int(rng.choice(N_EDGES))
        elif u < 0.55:
            n = int(rng.integers(1, 3 * m + 2))            # n of the order of m and below
        else:
            n = int(rng.integers(1, 60_000))
        kind = str(rng.choice(["f32", "f32", "bf16", "f16"]))
        bf = kind != "f32"
        ld = n + int(rng.integers(0, 9))
        off = int(rng.integers(0, 8))
        lam = float(rng.choice([0.01, 0.05, 0.3]))
        tau = float(rng.choice([1.0, 0.5]))
        tag = f"seed={seed} case={case} m={m} n={n} storage={kind} ld={ld} offset={off} lam={lam}"
        print(tag, flush=True)
        dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[kind]
        buf_t = torch.empty(m * ld + off + 8, dtype=dt, device=DEV)
        buf_g = torch.empty_like(buf_t)
        th = buf_t[off:off + m * ld].view(m, ld)[:, :n]
        gr = buf_g[off:off + m * ld].view(m, ld)[:, :n]
        rnd = lambda *shape: torch.randn(*shape, device=DEV, generator=gen)
        a = torch.exp(1.5 * rnd(n))
        b = rnd(n)
        th.copy_((rnd(n)[None, :] + 0.01 * rnd(m, n)).to(dt))
        gr.copy_((a[None, :] * th.float() - b[None, :] + 0.01 * rnd(m, n)).to(dt))
        th_np, gr_np = stored(th), stored(gr)

        C, w = qn.qn_gram(gr)
        Co, wo = oracle.gram_accumulate(gr_np)
        if m > 1:
            assert rel(C.cpu().numpy(), Co) <= 1e-5 and rel(w.cpu().numpy(), wo) <= 1e-5, tag
        else:
            assert torch.all(C == 0) and torch.all(w == 0), tag
        ref = oracle.update_streaming(th_np, gr_np, tau, np.float32(lam))
        sig = ref["sigma"]
        # "same j" is well posed when no singular value sits at the cutoff; with
        # n < m - 1 the trailing ones are rounding noise of either side
        rank = min(m - 1, n)
        margin = (np.min(np.abs(sig[:max(rank, 1)] / sig[0] - np.float32(lam)))
                  if sig[0] > 0 else 1.0)
        noise_ok = sig[0] == 0 or rank >= m - 1 or sig[rank] < 1e-3 * np.float32(lam) * sig[0]
        out, j = qn.qn_update(th, gr, tau, lam)
        z = rnd(n)
        h, jh = qn.qn_hinv(th, gr, z, lam)
        if margin > 1e-5 and noise_ok:
            assert int(j.item()) == ref["j"] and int(jh.item()) == ref["j"], tag
            base = 1e-3 if bf else 1e-5
            tol = step_tolerance(ref, th_np, gr_np, tau, base)
            assert rel(out.cpu().numpy(), ref["theta_new"]) <= tol, (tag, tol)
            tb, gb = oracle.row_means(th_np), oracle.row_means(gr_np)
            href = oracle.apply_Hinv_literal(oracle.centre(th_np, tb), oracle.centre(gr_np, gb),
                                             ref["sigma"], ref["V"], ref["j"],
                                             z.cpu().numpy().astype(np.float64))
            assert rel(h.cpu().numpy(), href) <= max(base, 1e-4), tag
