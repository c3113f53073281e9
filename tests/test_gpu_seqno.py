"""Stream-ordered sequence-number wait / signal (Sec. 4.1, device-side polling receive).

The writer of the sequence number is a host thread, or another stream of the same device;
every wait is bounded, so each kernel exits whether or not the writer ever shows up."""
import threading
import time

import pytest
import torch

from paper_2405_01814_amd import lamina

pytestmark = pytest.mark.gpu


def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    return torch.device("cuda:0")


def test_work_behind_a_wait_sees_what_the_host_released_before_the_seqno():
    d = dev()
    sq = lamina.Seqno()
    payload = torch.zeros(1 << 16, dtype=torch.int32).pin_memory()
    landed = torch.full((1 << 16,), -1, dtype=torch.int32, device=d)
    s = torch.cuda.Stream(device=d)
    print("enqueue wait + copy", flush=True)
    with torch.cuda.stream(s):
        sq.wait(1, timeout_us=5_000_000, stream=s)
        landed.copy_(payload, non_blocking=True)         # must not start before seqno >= 1

    def sender():
        time.sleep(0.05)
        payload.fill_(1234)                               # the data ...
        sq.value = 1                                      # ... then the sequence number

    t = threading.Thread(target=sender)
    t0 = time.perf_counter()
    t.start()
    s.synchronize()
    waited = time.perf_counter() - t0
    t.join()
    assert sq.status == lamina.LAMINA_SEQNO_REACHED
    assert waited >= 0.04, "the stream did not wait for the sequence number"
    assert bool((landed == 1234).all())
    sq.close()


def test_wait_is_bounded_when_the_writer_never_comes():
    d = dev()
    sq = lamina.Seqno()
    s = torch.cuda.Stream(device=d)
    after = torch.zeros(4, device=d)
    t0 = time.perf_counter()
    with torch.cuda.stream(s):
        sq.wait(7, timeout_us=20_000, stream=s)           # nobody writes 7
        after.add_(1)                                     # later work still runs
    s.synchronize()
    took = time.perf_counter() - t0
    assert sq.status == lamina.LAMINA_SEQNO_TIMED_OUT
    assert 0.02 <= took < 2.0
    assert bool((after == 1).all())
    sq.close()


def test_a_target_already_reached_does_not_wait():
    d = dev()
    sq = lamina.Seqno()
    sq.value = 5
    s = torch.cuda.Stream(device=d)
    t0 = time.perf_counter()
    sq.wait(3, timeout_us=5_000_000, stream=s)            # >= semantics
    sq.wait(5, timeout_us=5_000_000, stream=s)
    s.synchronize()
    assert time.perf_counter() - t0 < 1.0
    assert sq.status == lamina.LAMINA_SEQNO_REACHED
    sq.close()


def test_signal_on_one_stream_releases_a_wait_on_another_with_its_data():
    d = dev()
    sq = lamina.Seqno()
    produced = torch.zeros(1 << 20, device=d)
    consumed = torch.full((1 << 20,), -1.0, device=d)
    producer, consumer = torch.cuda.Stream(device=d), torch.cuda.Stream(device=d)
    torch.cuda.synchronize()
    with torch.cuda.stream(consumer):                     # receiver first: it has to wait
        sq.wait(3, timeout_us=5_000_000, stream=consumer)
        consumed.copy_(produced)
    time.sleep(0.02)
    with torch.cuda.stream(producer):
        produced.fill_(7.0)
        sq.signal(3, stream=producer)
    producer.synchronize()
    consumer.synchronize()
    assert sq.value == 3 and sq.status == lamina.LAMINA_SEQNO_REACHED
    assert bool((consumed == 7.0).all())
    sq.close()


def test_decode_attention_behind_a_wait_uses_the_query_that_arrived():
    # the receive path as the attention device runs it: poll, then attend (Sec. 4.1, Sec. 3.1)
    import numpy as np
    import oracle
    from paper_2405_01814_amd import workloads as W
    d = dev()
    b = W.generate(W.WORKLOADS["tiny"])
    op = lamina.DecodeAttention(8, 2, max_batch=4, max_seq_len=256)
    sq = lamina.Seqno()
    q_host = torch.zeros_like(b["q"]).pin_memory()        # the receive buffer, empty so far
    q_dev = torch.zeros_like(b["q"], device=d)
    k, v, lens = b["k"].to(d), b["v"].to(d), b["seq_lens"].to(d)
    s = torch.cuda.Stream(device=d)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        sq.wait(1, timeout_us=5_000_000, stream=s)
        q_dev.copy_(q_host, non_blocking=True)
        out, lse = op(q_dev, k, v, lens, stream=s)

    def sender():
        time.sleep(0.03)
        q_host.copy_(b["q"])
        sq.value = 1

    t = threading.Thread(target=sender)
    t.start()
    s.synchronize()
    t.join()
    assert sq.status == lamina.LAMINA_SEQNO_REACHED
    ref, ref_lse = oracle.decode_attention(b["q"], b["k"], b["v"], b["seq_lens"], num_kv_heads=2,
                                           scale=1.0 / 128 ** 0.5)
    assert np.abs(out.cpu().double().numpy() - ref).max() <= 2e-3
    assert np.abs(lse.cpu().double().numpy() - ref_lse).max() <= 1e-3
    sq.close()
    op.close()


def test_argument_errors():
    dev()
    assert lamina.lamina_seqno_wait(None, 1, 10, None, None) == lamina.LAMINA_ERR_INVALID_ARG
    assert lamina.lamina_seqno_signal(None, 1, None) == lamina.LAMINA_ERR_INVALID_ARG
    assert lamina.lamina_seqno_free(None, None) == lamina.LAMINA_OK
