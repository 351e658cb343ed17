"""The decode-attention entry point that allocates nothing (static device scratch) against
the existing entry point that takes caller-provided scratch: same output, bit for bit, on
two calls in a row, the second with a smaller input; and both within tolerance of the
oracle."""
import numpy as np
import pytest

import tally_inputs as TI
from oracle import kernels as OK
from oracle import schedules as OS

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_allocating_one():
    import torch
    import paper_2410_07381_amd.binding as B
    from gpu_util import dev, host, assert_bf16_close
    assert torch.cuda.is_available()
    hi, be = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(hi, be)
    try:
        for tokens, heads, seed_stream in ((2048, 32, 4), (333, 5, 5)):   # second call: smaller
            at = TI.attn_decode_inputs(tokens, heads, 128, scale=0.5, config_index=4)
            a = dict(at, out=np.zeros((heads, 128), np.uint16))
            OS.run_native("attn_decode_bf16", OK.grid_of("attn_decode_bf16", a), a)
            q, Kc, Vc = dev(at["q"]), dev(at["K"]), dev(at["V"])
            out_ref = dev(np.zeros((heads, 128), np.uint16))
            out_new = dev(np.zeros((heads, 128), np.uint16))
            scratch = torch.zeros(B.attn_decode_scratch_bytes(heads), dtype=torch.uint8, device="cuda")
            torch.cuda.synchronize()
            ctx.launch_native(B.attn_decode_bf16(q, Kc, Vc, out_ref, scratch))
            torch.cuda.synchronize()
            ctx.launch_attn_decode_static(q, Kc, Vc, out_new)
            torch.cuda.synchronize()
            assert (host(out_new) == host(out_ref)).all()
            assert_bf16_close(host(out_new), a["out"])
            # on the high-priority stream too
            out_new.zero_()
            torch.cuda.synchronize()
            ctx.launch_attn_decode_static(q, Kc, Vc, out_new, hi=True)
            torch.cuda.synchronize()
            assert (host(out_new) == host(out_ref)).all()
        # beyond the static array's size the call is refused
        big = torch.zeros((8, 129, 128), dtype=torch.int16, device="cuda")
        qb = torch.zeros((129, 128), dtype=torch.int16, device="cuda")
        with pytest.raises(B.TallyError):
            ctx.launch_attn_decode_static(qb, big, big, qb)
    finally:
        ctx.close()
