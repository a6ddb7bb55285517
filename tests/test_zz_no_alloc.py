"""fd_verify_draft_attn_static (the entry point that allocates nothing: split partials go to a
static device buffer inside the library) against fd_verify_draft_attn on the same inputs, through
the C ABI: two calls in a row, the second with a smaller input, so that whatever the first call
left in the shared buffer is in the way of the second.  Both entry points run the same kernels over
the same partition of the work, so the results are required to be identical bit for bit -- tighter
than the 2e-2 (bf16) / 1e-5 (fp32) bound the parity tests hold the kernels to against the oracle."""
import numpy as np
import pytest
import torch

from paper_2605_20022_amd import workloads as W
from paper_2605_20022_amd.devcall import AttnCall, from_dev

pytestmark = pytest.mark.gpu


def _both(fd, inp, **kw):
    call = AttnCall(fd, inp, **kw)
    ref, ref_lse = call.run()                                   # the existing entry point, caller's workspace
    call.out.fill_(float("nan")); call.lse.fill_(float("nan"))
    call.args.workspace = None; call.args.workspace_bytes = 0   # ignored by the static entry point
    fd.fd_verify_draft_attn_static(call.args)
    torch.cuda.synchronize()
    assert int(call.status.item()) == 0
    got, got_lse = from_dev(call.out), from_dev(call.lse)
    assert np.isfinite(got).all()
    assert np.array_equal(got, ref) and np.array_equal(got_lse, ref_lse)


def test_static_scratch_matches_workspace_call_twice(fd):
    big = W.AttnWorkload("st_big", "bf16", 6, 32, 8, 128, 16, (300, 3000), (4, 16), 16, 1.0, seed=91)       # 128-row tiles, many split items
    small = W.AttnWorkload("st_small", "bf16", 2, 8, 2, 128, 16, (40, 500), (1, 3), 2, 1.0, seed=92)        # 64-row tiles, fewer work-groups in use
    _both(fd, W.make_attention_inputs(big))
    _both(fd, W.make_attention_inputs(small))
    _both(fd, W.make_attention_inputs(small), kv_chunk=128)     # every item split: partials everywhere
    d64 = W.AttnWorkload("st_d64", "bf16", 3, 16, 4, 64, 16, (100, 1500), (2, 8), 8, 1.0, seed=95)            # head dim 64, smaller partial rows
    _both(fd, W.make_attention_inputs(d64), kv_chunk=128)
    f32 = W.AttnWorkload("st_f32", "f32", 2, 4, 1, 64, 16, (10, 300), (2, 4), 3, 1.0, seed=93)              # the fp32 kernel's workspace fits too
    _both(fd, W.make_attention_inputs(f32))


def test_static_scratch_rejects_what_does_not_fit(fd):
    """The fp32 kernel's workspace grows with rows x chunks: a call beyond the buffer is refused on the host."""
    w = W.AttnWorkload("st_large", "f32", 1, 32, 8, 128, 16, (64, 64), (1, 1), 0, 1.0, seed=94)
    call = AttnCall(fd, W.make_attention_inputs(w))
    call.args.total_rows = 40000                                # scalars only: the host rejects before any launch
    call.args.max_kv_len = 1 << 20
    assert fd.fd_verify_draft_attn_workspace(call.args) > fd.FD_STATIC_SCRATCH_BYTES
    with pytest.raises(fd.FlexDraftError) as e:
        fd.fd_verify_draft_attn_static(call.args)
    assert e.value.code == 3 and "static" in str(e.value)
