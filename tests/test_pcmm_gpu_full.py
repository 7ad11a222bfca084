"""Parity at the full workload sizes, in the launch configuration bench.py times (GPU).

The full oracle would need 4e11 .. 8e12 128-bit multiply-accumulates per workload, so at these sizes
the GPU result is checked by
  * a slab computed by the oracle and compared bit for bit: the first 16, last 16 and 32 seeded
    random rows x all columns, and the first 64, last 64 and the 64 columns straddling N (the a|b
    boundary) x all rows, for every limb;
  * a Freivalds check of the WHOLE output on the host: C_j.r = W.(A_j.r) mod q_j for two seeded
    vectors r per limb (a wrong row survives one vector with probability 1/q_j), plus a range check.
Inputs are the seeded synthetic workloads of pcmm_inputs (drawn on the GPU with torch integer ops, the
same numbers the host generator draws).
"""
import numpy as np
import pytest

import pcmm_inputs as pi

pytestmark = pytest.mark.gpu


def _slab_rows(wl, rng):
    rows = list(range(16)) + list(range(wl.M - 16, wl.M)) + sorted(rng.choice(wl.M, size=32, replace=False).tolist())
    return sorted(set(rows))


def _slab_cols(wl):
    N = wl.N
    return list(range(64)) + list(range(N - 32, N + 32)) + list(range(wl.Ncols - 64, wl.Ncols))


@pytest.mark.parametrize("name", ["attn_proj", "ffn_up_gate", "ffn_down", "wide_pc_attn", "attn_proj_w16_q62"])
def test_full_size_workload(gpu_device, name):
    import torch

    import paper_2601_18511_amd as pkg
    from oracle import pcmm_freivalds, pcmm_oracle_select

    wl = pi.WORKLOADS[name]
    primes = wl.primes
    rng = np.random.default_rng(2024)
    W = pi.gen_W(wl)
    print("[%s] generating A on the GPU" % name, flush=True)
    A_dev = pi.gen_A_torch(wl, gpu_device)
    C_dev = torch.empty((wl.L, wl.M, wl.Ncols), dtype=torch.int64, device=gpu_device)
    plan = pkg.pcmm_plan_create(torch.from_numpy(W).to(gpu_device), primes, wl.prime_bits, wl.Ncols)
    assert pkg.pcmm_plan_digits(plan) == wl.digits
    pkg.pcmm_run(plan, A_dev, C_dev)
    torch.cuda.synchronize()
    pkg.pcmm_plan_destroy(plan)

    rows, cols = _slab_rows(wl, rng), _slab_cols(wl)
    all_rows, all_cols = np.arange(wl.M), np.arange(wl.Ncols)
    for j in range(wl.L):                      # limb by limb bounds the host memory
        q = primes[j]
        print("[%s] limb %d: copy, slab, Freivalds" % (name, j), flush=True)
        Aj = A_dev[j].cpu().numpy().view(np.uint64)
        Cj = C_dev[j].cpu().numpy().view(np.uint64)
        # generator agreement on a few columns (the GPU drew the same numbers as the host would)
        probe = [0, wl.N, wl.Ncols - 1]
        assert (pi.gen_A_columns(wl, j, probe) == Aj[:, probe]).all()
        want = pcmm_oracle_select(W, Aj[None], [q], rows, all_cols)[0]
        assert (Cj[rows, :] == want).all(), "row slab differs in limb %d" % j
        want = pcmm_oracle_select(W, Aj[None], [q], all_rows, cols)[0]
        assert (Cj[:, cols] == want).all(), "column slab differs in limb %d" % j
        for t in range(2):
            r = pi.uniform_mod_q(99, 100 + 2 * j + t, np.arange(wl.Ncols, dtype=np.uint64), q, wl.prime_bits)
            assert pcmm_freivalds(W, Aj, Cj, r, q) == 0, "Freivalds check failed in limb %d" % j
        del Aj, Cj
