"""Failure handling of the weight-streaming (few-row) FFN kernels.  Their waits on other workgroups are
bounded; a wait that gives up sets a word in host memory, and the library reports BB_ERR_TIMEOUT from the
next FFN call on the device (or from bb_check_fault) instead of handing back a silently wrong result.
Every kernel in these tests exits normally: the condition is forced from the host, either by setting the
word directly or by a poll limit of zero (each wait then gives up at once and the kernel runs to its end).
"""
import pytest
import torch

import bb_inputs
import bb_parity
import paper_2505_07829_amd as bb
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
EPS = 1e-6


@pytest.fixture(scope="module", autouse=True)
def _lib():
    bb.load()
    yield
    bb.bb_debug_set_spin_limit(8000000)
    bb.bb_set_variant(bb.VARIANT_AUTO)


def _run(cpu, transposed=False):
    X, g, W1, W3, W2 = [t.cuda() for t in cpu]
    if transposed:
        Y = bb.bb_rmsnorm_swiglu_ffn_t(X, g, W1.t().contiguous(), W3.t().contiguous(), W2.t().contiguous(), EPS)
    else:
        Y = bb.bb_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, EPS)
    torch.cuda.synchronize()
    return Y


@pytest.mark.parametrize("transposed", [False, True])
def test_flag_set_by_host_is_reported_once_and_the_next_call_is_correct(transposed):
    cpu = bb_inputs.make_ffn(8, 512, 1408, seed=31)
    ref = orc.rmsnorm_swiglu_ffn(*cpu, EPS)
    bb_parity.check(_run(cpu, transposed), ref, "before")
    bb.bb_debug_inject_fault()
    with pytest.raises(bb.BBError) as e:
        _run(cpu, transposed)
    assert e.value.status == bb.BB_ERR_TIMEOUT
    bb.bb_check_fault()                                    # reported once: now clear
    bb_parity.check(_run(cpu, transposed), ref, "after")   # the synchronisation words were set up again


@pytest.mark.parametrize("transposed", [False, True])
def test_a_wait_that_gives_up_ends_the_kernel_and_is_reported(transposed):
    cpu = bb_inputs.make_ffn(16, 1024, 2816, seed=32)
    ref = orc.rmsnorm_swiglu_ffn(*cpu, EPS)
    bb_parity.check(_run(cpu, transposed), ref, "before")
    bb.bb_debug_set_spin_limit(0)
    try:
        _run(cpu, transposed)          # every wait gives up after its first poll; the launch still completes
    finally:
        bb.bb_debug_set_spin_limit(8000000)
    # a workgroup that was not the last to arrive has given up: the flag is set (unless every workgroup
    # happened to find the barrier complete at its first poll, which 256 workgroups do not)
    with pytest.raises(bb.BBError) as e:
        bb.bb_check_fault()
    assert e.value.status == bb.BB_ERR_TIMEOUT
    bb.bb_check_fault()
    bb_parity.check(_run(cpu, transposed), ref, "after")


def test_check_fault_is_clean_without_a_failure():
    bb.bb_check_fault()
