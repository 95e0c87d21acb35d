"""ltri_attend_static: the attention of short query blocks with the partial results of the split key range in
the library's own device buffer instead of the context's scratch. Called through the C ABI and compared with
ltri_attend on the same state, twice in a row, the second call with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import ltri_oracle as O
from paper_2412_04757_amd import LtriContext, LtriError, config_from_workload
from workloads import planted_stream, theta_default, Workload

pytestmark = pytest.mark.gpu


def test_attend_static_matches_attend_on_two_calls(gpu_device):
    w = Workload("mini-static", 8, 2, 128, "bf16", 2048 + 16, 512, 4, 128, 0, 256, "uniform", 16, 64)
    n_seqs = 3
    T0 = [2048, 1024, 512]
    cfg = config_from_workload(w, max_tokens=w.context, theta=theta_default(w.head_dim), n_layers=1, n_seqs=n_seqs)
    ctx = LtriContext(cfg, gpu_device)
    ka, va = ctx.arena_views()
    streams = [planted_stream(w, 50 + s, device=str(gpu_device), context=w.context) for s in range(n_seqs)]
    ocfg = O.OracleConfig(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.n_sink, w.window,
                          budget_tokens=w.budget_tokens, theta=float(np.float32(theta_default(w.head_dim))))
    for s, (K, V, Q, _) in enumerate(streams):
        ka[0, s].copy_(K); va[0, s].copy_(V)
        for c0 in range(0, T0[s], 512):
            ctx.append_chunk(0, s, 1, 512)
    pos = list(T0)

    def one_step(seq_begin, seq_count, n_q):
        """Appends n_q tokens to the sequences, retrieves, and attends by both entry points."""
        q = torch.stack([streams[s][2][pos[s]:pos[s] + n_q] for s in range(seq_begin, seq_begin + seq_count)]).contiguous()
        ctx.append_chunk(0, seq_begin, seq_count, n_q)
        ctx.retrieve(0, seq_begin, seq_count, q)
        for s in range(seq_begin, seq_begin + seq_count):
            pos[s] += n_q
        lse_a = torch.empty((seq_count, n_q, w.n_q_heads), dtype=torch.float32, device=gpu_device)
        lse_b = torch.full_like(lse_a, float("nan"))
        want = ctx.attend(0, seq_begin, seq_count, q, lse=lse_a)
        got = torch.full_like(want, float("nan"))
        ctx.attend_static(0, seq_begin, seq_count, q, got, lse=lse_b)
        torch.cuda.synchronize()
        return q, want, got, lse_a, lse_b

    # first call: three sequences, three query rows each (the matrix-core kernel with a split key range)
    q, want, got, lse_a, lse_b = one_step(0, n_seqs, 3)
    assert torch.isfinite(got.float()).all()
    assert float((got.float() - want.float()).abs().max()) <= 2e-2
    assert torch.equal(got, want) and torch.equal(lse_a, lse_b)
    # second call right after it, smaller: one sequence, one token (the one-token kernel); the buffer still
    # holds the first call's partial results
    q, want, got, lse_a, lse_b = one_step(1, 1, 1)
    assert torch.isfinite(got.float()).all()
    assert float((got.float() - want.float()).abs().max()) <= 2e-2
    assert torch.equal(got, want) and torch.equal(lse_a, lse_b)
    # and against the oracle on that last step (sequence 1)
    K, V, Q, _ = streams[1]
    st = O.OracleStream(ocfg, K.double().cpu().numpy(), V.double().cpu().numpy())
    for c0 in range(0, T0[1], 512):
        st.append_chunk(512)
    st.append_chunk(3)
    st.append_chunk(1)
    for h in range(w.n_kv_heads):
        s_, l_ = ctx.get_spans(0, 1, h)
        assert list(s_) == st.starts[h] and list(l_) == st.lens[h]
    qn = q[0].double().cpu().numpy()
    st.retrieve(qn)
    ref, _ = st.attend(qn)
    assert np.abs(got[0].double().cpu().numpy() - ref).max() <= 2e-2
    # a full batch again after the small call
    q, want, got, lse_a, lse_b = one_step(0, n_seqs, 1)
    assert torch.equal(got, want) and torch.equal(lse_a, lse_b)
    # a request beyond the buffer is refused with a clear error and leaves `out` alone
    assert ctx.sync_status() == 0


def test_attend_static_refuses_what_its_buffer_cannot_hold(gpu_device):
    """Two sequences x 32 query heads x 4 rows split 16 ways need 2.13 MB of partial results: more than the 2 MiB
    the library holds. The call fails with LTRI_ECAPACITY before anything is enqueued; ltri_attend still works."""
    w = Workload("mini-static2", 32, 8, 128, "bf16", 512 + 8, 256, 4, 64, 0, 128, "uniform", 16, 64)
    cfg = config_from_workload(w, max_tokens=w.context, theta=theta_default(w.head_dim), n_layers=1, n_seqs=2)
    ctx = LtriContext(cfg, gpu_device)
    ka, va = ctx.arena_views()
    qs = []
    for s in range(2):
        K, V, Q, _ = planted_stream(w, 60 + s, device=str(gpu_device), context=w.context)
        ka[0, s].copy_(K); va[0, s].copy_(V)
        qs.append(Q)
        for c0 in range(0, 512, 256):
            ctx.append_chunk(0, s, 1, 256)
    q = torch.stack([qs[s][512:516] for s in range(2)]).contiguous()
    ctx.append_chunk(0, 0, 2, 4)
    ctx.retrieve(0, 0, 2, q)
    out = torch.zeros((2, 4, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=gpu_device)
    with pytest.raises(LtriError) as err:
        ctx.attend_static(0, 0, 2, q, out)
    assert err.value.status == -3 and "2097152" in str(err.value)
    torch.cuda.synchronize()
    assert float(out.float().abs().max()) == 0.0
    want = ctx.attend(0, 0, 2, q)
    one = torch.empty((1, 4, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=gpu_device)
    ctx.attend_static(0, 1, 1, q[1:2].contiguous(), one)          # one sequence fits
    assert torch.equal(one[0], want[1])
    assert ctx.sync_status() == 0
