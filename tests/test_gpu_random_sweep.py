"""Seeded random sweep over valid inputs of every entry point (GPU): 260 cases drawn from all
supported widths, both dtypes, token counts around the tokens-per-workgroup and grid boundaries,
plain / in-place / optional-output variants, each compared with the oracle at the usual bar."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_2603_08343_amd as wht
from paper_2603_08343_amd import synth
from parity import assert_grad_close, assert_io_close, to_gpu

pytestmark = pytest.mark.gpu


def test_random_sweep_of_every_entry_point():
    rnd = random.Random(2024)
    widths_bf16 = [32, 64, 128, 256, 512, 768, 1024, 1536, 2048, 3072, 4096, 6144, 8192, 12288, 16384]
    widths_f32 = [32, 64, 128, 256, 512, 1024, 2048, 4096, 8192]
    cases = 0
    for it in range(260):
        dtype = rnd.choice(["bf16", "bf16", "f32"])
        d = rnd.choice(widths_bf16 if dtype == "bf16" else widths_f32)
        budget = 3_000_000 // d
        N = rnd.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 255, 257, 511, 513, 1023, 1025, 2047, 2049, 4097])
        N = max(1, min(N, budget))
        seed = rnd.randrange(1 << 30)
        inp = synth.make_inputs(N, d, dtype, seed=seed, outliers=rnd.random() < 0.2)
        x, dy = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
        a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
        meth = "matrix" if d <= 256 and N <= 64 else "fast"
        mode = rnd.choice(["fwd", "fwd_inplace", "resid", "resid_inplace", "stats", "bwd", "bwd_dx", "bwd_pg", "bwd_alias"])
        tag = f"case {it}: {mode} d={d} {dtype} N={N} seed={seed}"
        print(f"[parity] {tag}", flush=True)
        if mode == "fwd":
            assert_io_close(wht.wht_affine_forward(x, a, b), oracle.forward(inp.x, inp.alpha, inp.beta, meth), dtype, tag)
        elif mode == "fwd_inplace":
            x2 = x.clone(); wht.wht_affine_forward(x2, a, b, y=x2)
            assert_io_close(x2, oracle.forward(inp.x, inp.alpha, inp.beta, meth), dtype, tag)
        elif mode == "resid":
            assert_io_close(wht.wht_affine_forward_residual(x, a, b, dy), oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, meth), dtype, tag)
        elif mode == "resid_inplace":
            r2 = dy.clone(); wht.wht_affine_forward_residual(x, a, b, r2, y=r2)
            assert_io_close(r2, oracle.forward_residual(inp.x, inp.alpha, inp.beta, inp.dy, meth), dtype, tag)
        elif mode == "stats":
            y, ss = wht.wht_affine_forward_residual_stats(x, a, b, dy)
            ry, rss = oracle.forward_residual_stats(inp.x, inp.alpha, inp.beta, inp.dy, meth)
            assert_io_close(y, ry, dtype, tag)
            assert np.max(np.abs(ss.cpu().numpy() - rss) / rss) <= 1e-5, tag
        else:
            rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, meth)
            if mode == "bwd":
                dx, da, db = wht.wht_affine_backward(dy, x, a)
            elif mode == "bwd_dx":
                dx, da, db = wht.wht_affine_backward(dy, None, a, want_param_grads=False)
            elif mode == "bwd_pg":
                dx, da, db = wht.wht_affine_backward(dy, x, a, want_dx=False)
            else:
                g2 = dy.clone(); dx, da, db = wht.wht_affine_backward(g2, x, a, dx=g2)
            if dx is not None: assert_io_close(dx, rdx, dtype, tag + " dx")
            if da is not None:
                assert_grad_close(da, rda, tag + " dalpha"); assert_grad_close(db, rdb, tag + " dbeta")
        torch.cuda.synchronize()
        cases += 1
    assert cases == 260
