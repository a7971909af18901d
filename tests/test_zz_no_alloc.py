"""The allocation-free decode entry point (mux_decode_attn_static) against mux_decode_attn.

Both run the same kernels; the first takes its scratch from the library's fixed device array,
the second from a workspace of the caller.  Outputs must be bit-identical to each other and
within tolerance of the CPU oracle, on two calls in a row, the second smaller than the first
(it must not see what the first left in the scratch).
"""
import numpy as np
import pytest
import torch

import mux_harness as H
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _static_gpu(ls, job, q, scale):
    out = torch.full_like(q, float("nan"))
    lens_dev = torch.from_numpy(job.lens).to(ls.device)
    mx.mux_decode_attn_static(ls.lib, out, q, job.tables_dev, lens_dev, int(job.lens.max()), scale)
    return out


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (16, 2)])
def test_static_scratch_decode_equals_workspace_decode_twice_in_a_row(n_q, n_kv):
    print("[case] static-scratch decode Hq=%d Hkv=%d" % (n_q, n_kv), flush=True)
    rng = np.random.Generator(np.random.PCG64(77 + n_q))
    n_blocks = 6000
    ls = H.Lockstep(n_blocks, 16, 128, "bf16", wl.placement_order(rng, n_blocks))
    scale = H.default_scale(128)
    # first call: a few long rows, so the plan splits them into spans and the partial results
    # go through the scratch; second call: fewer, shorter rows
    cases = [np.array([4000, 3000, 17, 0, 2500, 1], np.int32), np.array([700, 5, 333], np.int32)]
    for call, lens in enumerate(cases):
        shape = wl.ModelShape("t", n_q, n_kv, 128)
        job = H.open_job(ls, call, shape, lens.size, int(lens.max()) + 16)
        H.extend(ls, job, lens, seed=500 + 10 * call + n_q)
        q = H.make_q(ls, job, 900 + call)
        ws_bytes = mx.mux_decode_workspace_bytes(ls.lib, lens.size, n_q, n_kv, int(lens.max()))
        assert 0 < ws_bytes <= mx.MUX_STATIC_SCRATCH_BYTES
        if call == 0:
            assert ws_bytes > 16 + lens.size * 8 + 16      # the plan did split: partial results use the scratch
        got = _static_gpu(ls, job, q, scale)
        ref = H.decode_gpu(ls, job, q, scale)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), "call %d differs from mux_decode_attn" % call
        err = H.assert_close(got, H.decode_oracle(ls, job, q, scale), "bf16", "call %d" % call)
        print("call %d: %d rows, scratch use %d bytes, max abs err vs oracle %.2e" % (call, lens.size, ws_bytes, err), flush=True)
    ls.check_counters()


def test_static_scratch_refuses_what_does_not_fit():
    print("[case] static-scratch decode, oversized call", flush=True)
    ls = H.Lockstep(64, 16, 128, "bf16")
    n_seqs, n_q, n_kv, max_blocks = 4096, 32, 32, 1024
    assert mx.mux_decode_workspace_bytes(ls.lib, n_seqs, n_q, n_kv, max_blocks * 16) > mx.MUX_STATIC_SCRATCH_BYTES
    q = torch.zeros(n_seqs, n_q, 128, dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 7.0)
    tables = torch.zeros(n_seqs, n_kv, max_blocks, dtype=torch.int32, device="cuda")
    lens = torch.zeros(n_seqs, dtype=torch.int32, device="cuda")
    with pytest.raises(mx.MuxError) as e:
        mx.mux_decode_attn_static(ls.lib, out, q, tables, lens, max_blocks * 16, 1.0)
    assert e.value.status == mx.MUX_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert (out == 7.0).all()          # nothing was launched
