"""The C ABI from plain C: the example program (no Python, no PyTorch in the process) is compiled
with gcc, run on the GPU, and its printed sums are compared with the same steps driven through the
Python binding on the same integer-pattern inputs (the library is deterministic: equal to the last
printed digit)."""
import math
import os
import shutil
import subprocess

import pytest
import torch

import paper_2412_05270_amd as A

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("rank", [32, 1])
def test_c_example_matches_the_python_binding(tmp_path, rank):
    cc = shutil.which("gcc") or shutil.which("cc")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if cc is None or not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime_api.h")):
        pytest.skip("no C compiler or HIP headers")
    libdir = os.path.dirname(A.library_path())
    exe = str(tmp_path / "c_abi_example")
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
                    "-D__HIP_PLATFORM_AMD__", os.path.join(ROOT, "paper_2412_05270_amd", "examples", "c_abi_example.c"),
                    "-L", libdir, "-lapollo_mi355x", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", exe], check=True)
    out = subprocess.run([exe, str(rank)], check=True, capture_output=True, text=True, timeout=120).stdout.split()
    got = {out[i]: out[i + 1] for i in range(0, len(out), 2)}

    rows, cols, steps = 256, 512, 3
    k = torch.arange(rows * cols, dtype=torch.int64)
    w = (((k * 37 + 11) % 201 - 100).to(torch.float32) * torch.tensor(1e-4, dtype=torch.float32)).reshape(rows, cols).cuda()
    g = torch.empty((rows, cols), dtype=torch.float32, device="cuda:0")
    cfg = A.ApolloConfig(rank=rank, mode=A.APOLLO_TENSOR if rank == 1 else A.APOLLO_CHANNEL, seed=2024, beta1=0.9,
                         beta2=0.999, eps=1e-8, scale=math.sqrt(128.0) if rank == 1 else 1.0, weight_decay=0.0,
                         nl_gamma=1.01, refresh_interval=2, bias_correction=1, side=A.APOLLO_SIDE_AUTO)
    st = A.ApolloStepper(cfg, [w], [g])
    for t in range(1, steps + 1):
        g.copy_((((k * 53 + 29 * t) % 127 - 63).to(torch.float32) * torch.tensor(1e-4, dtype=torch.float32)).reshape(rows, cols))
        st.step(t, 1e-2)
    torch.cuda.synchronize()
    hw = w.cpu().double().reshape(-1)
    assert int(got["rank"]) == rank and int(got["steps"]) == steps
    assert float(got["w0"]) == float("%.9e" % hw[0].item())
    assert float(got["w_last"]) == float("%.9e" % hw[-1].item())
    # the C program sums in index order in double precision; so does this
    s = 0.0
    sa = 0.0
    for v in hw.tolist():
        s += v
        sa += abs(v)
    assert float(got["sum"]) == float("%.9e" % s) and float(got["sum_abs"]) == float("%.9e" % sa)
    st.close()
