"""The decode attention entry point that allocates nothing (its partial results live in a device array inside
the library): called through the C ABI, its output is bit for bit that of eet_op_attention_decode with a
caller-provided scratch buffer, and within the operator tolerance of the CPU oracle -- on two calls in a row,
the second with a smaller input, so that whatever the first call left in the array is there when the second runs."""
import numpy as np
import pytest
import torch

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl
from tests.gpu_util import dev, gate, host

pytestmark = pytest.mark.gpu

OP_MAX, OP_MEAN = 6e-3, 6e-4


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def run_both(eet, d, heads, cap, n_keys, seed):
    B = len(n_keys)
    q = wl.normal(seed, 1, (B, heads, d))
    kc = wl.normal(seed, 2, (B, heads, cap, d))
    vc = wl.normal(seed, 3, (B, heads, cap, d))
    want = orc.attention_decode(q, kc, vc, n_keys)
    for b, n in enumerate(n_keys):               # slots past a sequence's keys are never read
        kc[b, :, n:] = np.nan
        vc[b, :, n:] = np.nan
    need = eet.eet_op_attention_decode_scratch_bytes(B, heads, d, cap)
    assert need > 256, "the case must split the key range, or no scratch is used"
    qd, kd, vd, nd = dev(q.reshape(B, heads * d)), dev(kc), dev(vc), dev(np.asarray(n_keys, np.int32))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    ref = torch.full((B, heads * d), float("nan"), dtype=torch.float16, device="cuda:0")
    got = torch.full_like(ref, float("nan"))
    eet.eet_op_attention_decode(qd, kd, vd, ref, nd, ws)
    eet.eet_op_attention_decode_static(qd, kd, vd, got, nd)
    torch.cuda.synchronize()
    assert np.array_equal(host(got).view(np.uint16), host(ref).view(np.uint16)), f"d={d} heads={heads}: differs from eet_op_attention_decode"
    gate(host(got).reshape(B, heads, d), want, f"static-scratch decode attention d={d} heads={heads}", OP_MAX, OP_MEAN)


def test_static_scratch_decode_attention_equals_the_workspace_form_on_two_calls(eet):
    print("no-alloc decode attention: call 1 (2 sequences x 16 heads of 128, capacity 4224)", flush=True)
    run_both(eet, 128, 16, 4224, [4224, 2049], 7101)
    print("no-alloc decode attention: call 2, smaller (1 sequence x 12 heads of 64, capacity 512)", flush=True)
    run_both(eet, 64, 12, 512, [389], 7102)


def test_static_scratch_rejects_bad_arguments_without_launching(eet):
    L = eet.lib()
    assert L.eet_op_attention_decode_static(None, None, None, None, None, 1, 1, 64, 16, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_attention_decode_static(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1, 1, 96, 16, None) == eet.EET_ERR_UNSUPPORTED_SHAPE
    assert L.eet_op_attention_decode_static(0x1000, 0x1000, 0x1000, 0x1008, 0x1000, 1, 1, 64, 16, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_last_error()
