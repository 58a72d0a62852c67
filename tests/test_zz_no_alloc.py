"""jpp_op_attention_bwd_static, the entry point for callers that cannot allocate device memory:
the attention backward with its fp32 scratch (one float per batch, query head and position)
in a device array that belongs to the library.  Through the C ABI, against
jpp_op_attention_bwd on the same inputs: identical bits, on two calls in a row, the second
with a smaller input (the array then still holds the first call's values beyond what the
second one writes), and a refusal beyond the array's size with nothing launched.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def stream():
    return torch.cuda.current_stream().cuda_stream


def both_backwards(dtype, mb, seq, Hq, Hkv, hd, seed):
    """dqkv of the existing entry point and of the no-allocation one, on the same inputs."""
    tdt = torch.bfloat16 if dtype == inp.DT_BF16 else torch.float32
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    T, nqkv = mb * seq, (Hq + 2 * Hkv) * hd
    qkv = torch.randn((T, nqkv), generator=g, device=DEV).to(tdt)
    dout = torch.randn((T, Hq * hd), generator=g, device=DEV).to(tdt)
    out = torch.zeros((T, Hq * hd), dtype=tdt, device=DEV)
    lse = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    delta = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    ref = torch.full((T, nqkv), 3.0, dtype=tdt, device=DEV)
    got = torch.full((T, nqkv), 5.0, dtype=tdt, device=DEV)
    torch.cuda.synchronize()
    B.jpp_op_attention_fwd(dtype, mb, seq, Hq, Hkv, hd, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(), stream())
    B.jpp_op_attention_bwd(dtype, mb, seq, Hq, Hkv, hd, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(),
                           dout.data_ptr(), ref.data_ptr(), delta.data_ptr(), stream())
    torch.cuda.synchronize()
    # everything the call needs exists now: from here to the synchronisation nothing allocates
    before = torch.cuda.memory_allocated(DEV)
    B.jpp_op_attention_bwd_static(dtype, mb, seq, Hq, Hkv, hd, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                  dout.data_ptr(), got.data_ptr(), stream())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(DEV) == before
    return ref, got


def same_bits(a, b):
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8))


# (first call, second and smaller call)
CASES = {
    # the benchmark layer's attention shape (786 432 floats of scratch), then a ragged, grouped-query one
    "bf16-mfma": ((inp.DT_BF16, 1, 2048, 96, 96, 128), (inp.DT_BF16, 2, 328, 8, 2, 128)),
    # the generic kernels (fp32, head_dim 32), two sequences, then one short sequence
    "fp32-generic": ((inp.DT_F32, 2, 200, 4, 4, 32), (inp.DT_F32, 1, 37, 3, 1, 24)),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_static_scratch_backward_gives_the_bits_of_the_allocating_one(name):
    first, second = CASES[name]
    for k, shape in enumerate((first, second)):
        dtype, mb, seq, Hq, Hkv, hd = shape
        assert 4 * mb * Hq * seq <= B.JPP_STATIC_SCRATCH_BYTES
        print("attention backward without allocation:", name, "call", k, shape, flush=True)
        ref, got = both_backwards(*shape, seed=7 + k)
        assert bool(torch.isfinite(got.float()).all())
        assert float(ref.float().abs().max()) > 0.0
        assert same_bits(ref, got), (name, k)


def test_static_scratch_backward_refuses_what_does_not_fit():
    mb, seq, Hq, Hkv, hd = 1, 16384, 128, 128, 128           # 2 097 152 floats: twice the array
    assert 4 * mb * Hq * seq > B.JPP_STATIC_SCRATCH_BYTES
    one = torch.zeros(8, dtype=torch.bfloat16, device=DEV)   # never read: the sizes are refused first
    with pytest.raises(B.JppError) as e:
        B.jpp_op_attention_bwd_static(inp.DT_BF16, mb, seq, Hq, Hkv, hd, one.data_ptr(), one.data_ptr(),
                                      one.data_ptr(), one.data_ptr(), one.data_ptr(), stream())
    assert e.value.status == B.JPP_EINVAL
    assert "static scratch" in str(e.value)
    # exactly at the limit is accepted by the size check (1 x 128 heads x 8192 positions): small
    # tensors cannot back that, so only the arithmetic of the bound is checked here
    assert 4 * 1 * 128 * 8192 == B.JPP_STATIC_SCRATCH_BYTES
