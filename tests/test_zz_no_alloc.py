"""bb_rmsnorm_swiglu_ffn_static (the entry point that allocates nothing: its scratch is a static device
array) against bb_rmsnorm_swiglu_ffn, through the C ABI: same kernels, so the outputs must be bit-identical
(and both meet the parity gates against the oracle).  Two calls in a row share the array, the second with a
smaller input; then the other kernel family, and the size limit."""
import numpy as np
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
    bb.bb_init()
    bb.bb_set_variant(bb.VARIANT_AUTO)
    yield


def both(shape, seed):
    cpu = bb_inputs.make_ffn(*shape, seed=seed)
    dev = [t.cuda() for t in cpu]
    Y_static = torch.full((shape[0], shape[1]), float("nan"), dtype=torch.bfloat16, device="cuda")
    bb.bb_rmsnorm_swiglu_ffn_static(*dev, EPS, Y_static)
    Y = bb.bb_rmsnorm_swiglu_ffn(*dev, EPS)
    torch.cuda.synchronize()
    assert np.array_equal(bb_inputs.bits(Y_static.cpu()), bb_inputs.bits(Y.cpu())), shape
    bb_parity.check(Y_static, orc.rmsnorm_swiglu_ffn(*cpu, EPS), f"static {shape}")


def test_two_calls_in_a_row_second_smaller_streaming_kernels():
    both((16, 1024, 2816), 41)       # few rows: the weight-streaming kernel (partial sums, barrier words in the array)
    both((5, 512, 1408), 42)
    both((16, 1024, 2816), 43)       # and the larger one again after the smaller


def test_two_calls_in_a_row_second_smaller_tiled_kernels():
    both((200, 1024, 2816), 44)      # tiled kernels: hidden and split partial results in the array
    both((72, 512, 1408), 45)
    both((7, 512, 1408), 46)         # back to the streaming kernel: its zone was overwritten and is cleared again


def test_memory_allocated_by_torch_does_not_change_and_no_workspace_is_made():
    cpu = bb_inputs.make_ffn(64, 512, 1408, seed=47)
    dev = [t.cuda() for t in cpu]
    Y = torch.empty((64, 512), dtype=torch.bfloat16, device="cuda")
    bb.bb_shutdown()                                     # the library's own workspace is gone
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        bb.bb_rmsnorm_swiglu_ffn_static(*dev, EPS, Y)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 >= free0                                # nothing was allocated on the device
    bb_parity.check(Y, orc.rmsnorm_swiglu_ffn(*cpu, EPS), "static after shutdown")


def test_sizes_beyond_the_array_are_rejected():
    M, D, F = 1024, 4096, 11008
    assert bb.load().bb_workspace_bytes(0, M, D, F) > bb.STATIC_SCRATCH_BYTES
    X = torch.zeros((M, D), dtype=torch.bfloat16, device="cuda")
    g = torch.ones((D,), dtype=torch.bfloat16, device="cuda")
    W1 = torch.zeros((D, F), dtype=torch.bfloat16, device="cuda")
    W3 = torch.zeros((D, F), dtype=torch.bfloat16, device="cuda")
    W2 = torch.zeros((F, D), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, D), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(bb.BBError) as e:
        bb.bb_rmsnorm_swiglu_ffn_static(X, g, W1, W3, W2, EPS, Y)
    assert e.value.status == bb.BB_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())                        # nothing was launched
