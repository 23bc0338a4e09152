"""dx_route_static (the entry point for callers that cannot allocate: static device scratch) against
dx_route on a context: every output bit for bit, on two calls in a row, the second smaller, and the
size limit refused with a message."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_route_static_matches_route_on_two_calls_in_a_row():
    from paper_2511_15015_amd import binding as B
    B.load()
    E, k = 128, 8
    rng = np.random.default_rng(7)
    t_big, t_small = 1000, 200                     # 16 chunks with a ragged tail, then 4 chunks (both multi-chunk)
    ctx = B.Context(L=1, E=E, d=256, f=128, top_k=k, group=64, max_tokens=t_big)
    stream = torch.cuda.current_stream().cuda_stream

    def buffers(T):
        return (torch.full((T, k), -1, dtype=torch.int32, device="cuda"), torch.full((T, k), -1.0, device="cuda"),
                torch.full((E,), -1, dtype=torch.int32, device="cuda"), torch.full((E + 1,), -1, dtype=torch.int32, device="cuda"),
                torch.full((T * k,), -1, dtype=torch.int32, device="cuda"))

    for T in (t_big, t_small, 64, 1):             # the last two finish in the single-chunk launch (no scratch)
        print(f"dx_route_static T={T} E={E} k={k}", flush=True)
        lg = torch.from_numpy(rng.standard_normal((T, E)).astype(np.float32)).cuda()
        ref, got = buffers(T), buffers(T)
        ctx.dx_route(0, lg, T, *ref)
        torch.cuda.synchronize()
        # everything the static call needs exists before it starts: it must not allocate
        before = torch.cuda.memory_allocated()
        B.dx_route_static(lg, T, E, k, *got, stream=stream)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for name, a, b in zip(("ids", "w", "counts", "offsets", "perm"), ref, got):
            assert torch.equal(a, b), (T, name)
    ctx.close()
    # beyond the static scratch: refused, nothing launched
    with pytest.raises(B.DxError) as err:
        B.dx_route_static(lg, 8192, 1024, k, *got, stream=stream)
    assert err.value.status == B.DX_ERR_INVALID and "exceeds the static scratch" in str(err.value)
    with pytest.raises(B.DxError):
        B.dx_route_static(lg, 64, 2048, k, *got, stream=stream)
