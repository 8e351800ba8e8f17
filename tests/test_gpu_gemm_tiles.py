"""Every tile shape of the bf16 MFMA GEMM accumulates the k index of an output element in the same
order with the same instruction, so all shapes must give bit-identical results (the batch invariance
of forwards above 384 token rows rests on this: the shape is chosen from M).  Each shape is forced through the
PVF_GEMM_TILE environment variable, which the library reads once per process, hence subprocesses."""
import hashlib
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import hashlib, sys, torch
sys.path.insert(0, %r)
from paper_2601_12247_amd import binding as B
g = torch.Generator(device="cuda").manual_seed(11)
M, N, K = 700, 1536, 512                       # ragged last row tile for every tile height
A = torch.randn(M, K, device="cuda", generator=g).to(torch.bfloat16)
W = (torch.randn(N, K, device="cuda", generator=g) * 0.05).to(torch.bfloat16)
W2 = (torch.randn(2 * N, K, device="cuda", generator=g) * 0.05).to(torch.bfloat16)
R = torch.randn(M, N, device="cuda", generator=g).to(torch.bfloat16)
outs = [B.gemm(A, W), B.gemm(A, W, residual=R), B.gemm_swiglu(A, W2)]
torch.cuda.synchronize()
print(" ".join(hashlib.sha256(o.view(torch.int16).cpu().numpy().tobytes()).hexdigest() for o in outs))
""" % ROOT


def run_child(tile):
    env = dict(os.environ)
    env["PVF_GEMM_TILE"] = tile
    r = subprocess.run([sys.executable, "-c", CHILD], capture_output=True, text=True, env=env, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    return r.stdout.strip().splitlines()[-1].split()


def test_all_tile_shapes_agree_bit_for_bit():
    want = run_child("")                           # the shapes the cost model picks
    assert len(want) == 3
    for tile in range(10):
        got = run_child(str(tile))
        assert got == want, f"tile shape {tile} differs from the default choice"
