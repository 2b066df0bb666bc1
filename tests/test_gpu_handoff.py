"""GPU checks of the chunked payload hand-off: byte-exact reassembly in pinned host memory, the order
of transfers against the CPU model replayed from the points at which each payload became visible, and
the bound the method is built for (a decode transfer never waits behind a prefill chunk chosen after
the decode payload became visible)."""
import pytest
import torch

from oracle import handoff_oracle as M
from paper_2507_05043_amd import handoff, synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def _pinned_like(t):
    return torch.zeros(t.shape, dtype=t.dtype, pin_memory=True)


def _bits(t):
    return t.view(torch.int16)


def _check_log_against_model(records, submits, visible, row_bytes, chunk_bytes):
    got = [r.as_tuple() for r in records]
    assert [r.pick for r in records] == list(range(len(records)))
    want = M.drain_order([(visible[k], q) for k, q in enumerate(submits)], row_bytes, chunk_bytes)
    assert got == want, "order of transfers differs from the model's"
    for i, r in enumerate(records):
        if r.kind == handoff.DECODE:
            late = [j for j in range(visible[r.ticket], i) if records[j].kind == handoff.PREFILL]
            assert late == [], "a prefill chunk was chosen while a visible decode transfer waited"
    for a, b in zip(records, records[1:]):
        assert b.begin_ms >= a.end_ms - 1e-6, "two transfers overlapped: the sender moves one at a time"


def test_mixed_payload_is_reassembled_byte_exact_in_model_order():
    torch.manual_seed(0)
    q_lens = [37, 1, 1, 1, 300, 1, 2, 1, 1]
    t, hdim = sum(q_lens), 512
    payload = synth.draw_normal_bf16(0, 1, t * hdim, device="cuda:0").view(t, hdim)
    host = _pinned_like(payload)
    chunk = 64 * 1024
    s = handoff.Sender(chunk)
    ticket = s.submit(payload, host, q_lens)
    s.wait(ticket, handoff.DECODE)
    s.wait(ticket)
    assert torch.equal(_bits(host), _bits(payload.cpu()))
    recs = s.log()
    assert [r.as_tuple()[1:] for r in recs] == handoff.plan(q_lens, hdim * 2, chunk)
    _check_log_against_model(recs, [q_lens], [s.visible_pick(ticket)], hdim * 2, chunk)
    s.close()


def test_a_decode_payload_overtakes_the_remaining_prefill_chunks():
    # prefill payloads of Qwen2-7B width (16 chunks of 2048 rows of 3584 bf16, 235 MB in all) are draining in
    # 256 KB pieces when a decode payload of 128 rows is submitted
    import time
    hdim = 3584
    rows = 16 * 2048
    pre = synth.draw_normal_bf16(1, 1, rows * hdim, device="cuda:0").view(rows, hdim)
    dec = synth.draw_normal_bf16(2, 1, 128 * hdim, device="cuda:0").view(128, hdim)
    pre_host, dec_host = _pinned_like(pre), _pinned_like(dec)
    torch.cuda.synchronize()
    chunk = 256 * 1024
    s = handoff.Sender(chunk)
    t0 = s.submit(pre, pre_host, [2048] * 16)
    deadline = time.time() + 20.0
    while s.picks() < 20:                             # about ten milliseconds of chunks are queued; let some go
        assert time.time() < deadline, "the sender made no progress"
    t1 = s.submit(dec, dec_host, [1] * 128)
    s.wait(t1, handoff.DECODE)
    s.wait(t0)
    s.wait(t1)
    assert torch.equal(_bits(pre_host), _bits(pre.cpu())) and torch.equal(_bits(dec_host), _bits(dec.cpu()))
    recs = s.log()
    visible = [s.visible_pick(t0), s.visible_pick(t1)]
    _check_log_against_model(recs, [[2048] * 16, [1] * 128], visible, hdim * 2, chunk)
    n_chunks = 16 * ((2048 * hdim * 2 + chunk - 1) // chunk)
    dec_pick = [r.pick for r in recs if r.ticket == t1][0]
    print(f"  {n_chunks} prefill chunks; decode payload visible after {visible[1]} picks, sent as pick {dec_pick}; "
          f"its transfer took {[r.end_ms - r.begin_ms for r in recs if r.ticket == t1][0] * 1e3:.0f} us, "
          f"a chunk {sum(r.end_ms - r.begin_ms for r in recs if r.ticket == t0) / n_chunks * 1e3:.0f} us", flush=True)
    assert dec_pick == visible[1], "the decode transfer was not the first choice after its payload became visible"
    assert visible[1] >= 20
    if visible[1] >= n_chunks:
        pytest.skip("the prefill payload had drained before the decode payload arrived: nothing to overtake")
    waited = [r for r in recs if r.ticket == t1][0].begin_ms - recs[visible[1] - 1].begin_ms
    print(f"  the decode transfer started {waited * 1e3:.0f} us after the chunk that was on the wire when it arrived",
          flush=True)
    s.close()


def test_hand_off_overlaps_the_next_forward_and_delivers_the_stage_output():
    shape, mb = synth.workload("tiny", seed=0)
    st = H.make_stage(shape, mb, 0, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=0, device="cuda:0")
    outs = [torch.empty_like(hidden) for _ in range(3)]
    hosts = [_pinned_like(hidden) for _ in range(3)]
    s = handoff.Sender(4096)
    tickets = []
    for i in range(3):
        H.fill_pool(st, shape, mb, 0)
        st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, out=outs[i])
        tickets.append(s.submit(outs[i], hosts[i], mb.q_lens))       # no synchronisation: the sender waits for the stream
    for tk in tickets:
        s.wait(tk)
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(_bits(hosts[i]), _bits(outs[i].cpu()))
        assert torch.equal(_bits(hosts[i]), _bits(hosts[0]))          # same inputs, same cache: same payload
    recs = s.log()
    _check_log_against_model(recs, [mb.q_lens] * 3, [s.visible_pick(t) for t in tickets], shape.hidden * 2, 4096)
    st.close()
    s.close()


def test_invalid_submissions_are_rejected():
    s = handoff.Sender(1024)
    x = torch.zeros(4, 8, dtype=torch.bfloat16, device="cuda:0")
    h = _pinned_like(x)
    with pytest.raises(handoff.HandoffError):
        s.submit(x, h, [2, 0, 2])
    with pytest.raises(ValueError):
        s.submit(x, torch.zeros(4, 8, dtype=torch.bfloat16), [4])        # host buffer not pinned
    with pytest.raises(handoff.HandoffError):
        s.wait(5)
    with pytest.raises(handoff.HandoffError):
        handoff.Sender(0)
    s.close()
