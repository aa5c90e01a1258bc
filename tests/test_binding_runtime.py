"""The binding and PyTorch must share one HIP runtime whatever the import order: device pointers and
streams that PyTorch hands out are only good for kernels launched through the runtime that made them."""
import subprocess
import sys
import textwrap

import pytest

MAPPED = 'print(sorted({l.split()[-1] for l in open("/proc/self/maps") if "libamdhip64" in l}))'


@pytest.mark.parametrize("first", ["library", "torch"])
def test_one_hip_runtime_is_mapped_whatever_the_import_order(first):
    lines = ["from paper_2603_08734_amd import binding", "binding.lib()"]
    lines = lines + ["import torch"] if first == "library" else ["import torch"] + lines
    out = subprocess.run([sys.executable, "-c", "\n".join(lines + [MAPPED])], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    mapped = eval(out.stdout.strip().splitlines()[-1])
    assert len(mapped) == 1, mapped


@pytest.mark.gpu
def test_plan_first_then_torch():
    """A process that plans and uploads before it ever imports PyTorch: PyTorch must still find the
    GPU, and the product must be right."""
    code = textwrap.dedent('''
        import numpy as np
        from paper_2603_08734_amd import Plan
        from workloads import make_config, dense_B
        A, N, dist = make_config(1, small=True)
        plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N)      # HIP is initialised here
        import torch
        assert torch.cuda.is_available()
        B = dense_B(A.n_cols, N, dist, seed=1)
        Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
        C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
        plan.spmm(Bd, C)
        torch.cuda.synchronize()
        from oracle import spmm as ospmm
        C_ref, S, _ = ospmm.spmm(A.row_ptr, A.col_idx, A.val, B)
        err = np.abs(C.cpu().numpy().astype(np.float64) - C_ref)
        assert (err <= 1e-4 * S).all()
        print("ok")
    ''')
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr
