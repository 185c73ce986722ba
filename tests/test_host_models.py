"""Host-side models of the library's index arithmetic, built with g++ and run on the CPU (no GPU).

* gemm_dma_model: every address the ring GEMM kernel's operand DMA can form, for every tile variant, operand
  layout, split-K chunk and a list of ragged shapes, checked against the operand as the caller's contract defines
  it; and the same schedule with the K loop padded to five K tiles and no clamp on the tile index (a variant that
  was tried on the GPU and faulted), which the model shows reading past the operand.
* plan_sanitize: the planning code of csrc/ntp_plan.cpp under AddressSanitizer and UndefinedBehaviorSanitizer
  with invariants on every result.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_06095_amd", "csrc")
MODEL = os.path.join(ROOT, "tests", "host_model")

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")


def _build(tmp_path, name, sources, flags):
    exe = str(tmp_path / name)
    cmd = ["g++", "-std=c++17", *flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *sources, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def test_every_dma_address_of_the_ring_kernel_lies_inside_its_operand(tmp_path):
    exe = _build(tmp_path, "gemm_dma_model", [os.path.join(MODEL, "gemm_dma_model.cpp")], ["-O2"])
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    tag, cases, loads = res.stdout.split()
    assert tag == "OK" and int(cases) > 10000 and int(loads) > 10 ** 8


def test_unclamped_padded_k_loop_reads_past_the_operand(tmp_path):
    """The withdrawn run-on ring variant: K loop padded to a multiple of five K tiles.  Without the clamp on the
    K tile index its loads reach megabytes past the operand; with the range check of the DMA switched off, as
    it was then, that is an illegal address."""
    exe = _build(tmp_path, "gemm_dma_model", [os.path.join(MODEL, "gemm_dma_model.cpp")], ["-O2"])
    res = subprocess.run([exe, "padded"], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    tag, overrun = res.stdout.split()
    assert tag == "OVERRUN" and int(overrun) > 1 << 20


def test_planning_code_under_address_and_ub_sanitizers(tmp_path):
    exe = _build(tmp_path, "plan_sanitize", [os.path.join(MODEL, "plan_sanitize.cpp"), os.path.join(CSRC, "ntp_plan.cpp")],
                 ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"])
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("OK ")
