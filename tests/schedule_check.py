"""Stand-alone parity check of one (schedule, shape) set, run in its own process because the
library reads WHT_AFFINE_SCHEDULE once per process.  Used by test_gpu_schedules.py:

    WHT_AFFINE_SCHEDULE=butterfly python tests/schedule_check.py

Checks forward and backward against the CPU oracle for bf16 at d = 1024 ... 16384 with ragged token
counts, to the same tolerances as tests/test_gpu_parity.py.  Exit status 0 iff everything passes."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import torch  # noqa: E402

import oracle  # noqa: E402
import paper_2603_08343_amd as wht  # noqa: E402
from paper_2603_08343_amd import synth  # noqa: E402
from parity import assert_grad_close, assert_io_close, to_gpu  # noqa: E402


def main():
    for d, N in ((1024, 263), (2048, 131), (4096, 67), (8192, 1031), (16384, 35)):
        inp = synth.make_inputs(N, d, "bf16", seed=100 + d)
        print(f"[schedule_check] {os.environ.get('WHT_AFFINE_SCHEDULE', 'default')} d={d} N={N}", flush=True)
        x, dy = to_gpu(inp.x, "bf16"), to_gpu(inp.dy, "bf16")
        a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
        y = wht.wht_affine_forward(x, a, b)
        dx, da, db = wht.wht_affine_backward(dy, x, a)
        torch.cuda.synchronize()
        assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, "fast"), "bf16", f"y d={d}")
        rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, "fast")
        assert_io_close(dx, rdx, "bf16", f"dx d={d}")
        assert_grad_close(da, rda, f"dalpha d={d}")
        assert_grad_close(db, rdb, f"dbeta d={d}")
    print("[schedule_check] ok", flush=True)


if __name__ == "__main__":
    main()
