"""Signal ingest ring (include/tide_ingest.h) through the C ABI: the bytes that reach the device are the
bytes the producer wrote, a training step that consumes an ingested batch equals the step on directly
uploaded data, the slot state machine (free -> filling -> copying -> free) and the error codes."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_05145_amd import workloads as W
from tests.gpu_util import sync

pytestmark = pytest.mark.gpu


def host_view(addr, nbytes):
    return np.ctypeslib.as_array((ctypes.c_uint8 * nbytes).from_address(addr))


def test_ingested_batch_trains_like_a_direct_upload():
    from paper_2602_05145_amd import binding as B, runtime
    cfg = W.get_config("small", batch=2, seq=128, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    ref = runtime.trainer_from_workload(cfg, wl)
    ref.train_step(cfg["lr"])
    sync()

    tr = runtime.trainer_from_workload(cfg, wl)
    hid_bits = W.f32_to_bf16_bits(wl["hidden"].astype(np.float32)).reshape(-1)          # what the producer holds
    nbytes = hid_bits.nbytes
    rc, q = B.tide_ingest_create(nbytes, 3)
    assert rc == 0, B.tide_ingest_last_error()
    try:
        dst = torch.zeros_like(tr.hidden)                    # device buffer the step will read
        rc, slot, addr = B.tide_ingest_acquire(q)
        assert rc == 0 and slot == 0
        host_view(addr, nbytes)[:] = hid_bits.view(np.uint8)
        assert B.tide_ingest_submit(q, slot, dst, nbytes) == 0
        assert B.tide_ingest_wait(q, slot, tr._stream()) == 0
        tr.hidden = dst
        tr.train_step(cfg["lr"])                             # ordered after the copy by the stream wait
        sync()
        assert B.tide_ingest_done(q, slot) == 1
        assert torch.equal(dst.view(torch.int16), ref.hidden.view(torch.int16))
        assert float(tr.loss.item()) == float(ref.loss.item())
        for k in tr.grads:
            assert torch.equal(tr.grads[k], ref.grads[k]), k
    finally:
        assert B.tide_ingest_destroy(q) == 0


def test_double_buffer_without_host_syncs_equals_direct_uploads():
    """Six different batches streamed through a two-slot ring into a device double buffer with no host
    synchronisation between the steps: the copy of batch i+1 into the buffer that step i-1 read is ordered after
    that step through the reader-stream argument of tide_ingest_submit.  Every step's loss and the final gradients
    and parameters must equal, bit for bit, a second trainer fed by direct uploads with a sync after every step."""
    from paper_2602_05145_amd import binding as B, runtime
    cfg = W.get_config("small", batch=4, seq=512, target_hidden=512, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=512, vocab=2048, mask="prefix", mask_p=0.1)
    batches = [W.make_workload(cfg, seed=500 + i) for i in range(6)]
    ref = runtime.trainer_from_workload(cfg, batches[0])
    ref_losses = []
    for wl in batches:
        ref.set_batch(wl["hidden"], wl["tokens"], wl["mask"])
        ref.train_step(cfg["lr"])
        sync()
        ref_losses.append(float(ref.loss.item()))

    tr = runtime.trainer_from_workload(cfg, batches[0])
    bits = [W.f32_to_bf16_bits(wl["hidden"].astype(np.float32)).reshape(-1) for wl in batches]
    toks = [torch.from_numpy(np.ascontiguousarray(wl["tokens"], dtype=np.int32)).to(tr.device) for wl in batches]
    masks = [torch.from_numpy(np.ascontiguousarray(wl["mask"], dtype=np.uint8)).to(tr.device) for wl in batches]
    nbytes = bits[0].nbytes
    rc, q = B.tide_ingest_create(nbytes, 2)
    assert rc == 0, B.tide_ingest_last_error()
    try:
        bufs = [torch.zeros_like(tr.hidden), torch.zeros_like(tr.hidden)]
        losses = []
        sync()
        # batch 0 goes in first; from then on the copy of batch i+1 is submitted BEFORE step i is enqueued, into the
        # buffer that step i-1 (possibly still running) reads
        rc, slot, addr = B.tide_ingest_acquire(q)
        assert rc == 0
        host_view(addr, nbytes)[:] = bits[0].view(np.uint8)
        assert B.tide_ingest_submit(q, slot, bufs[0], nbytes, tr._stream(), True) == 0
        for i in range(len(batches)):
            assert B.tide_ingest_wait(q, slot, tr._stream()) == 0
            if i + 1 < len(batches):
                while True:                                     # the other slot frees up when its copy has completed
                    rc, nslot, addr = B.tide_ingest_acquire(q)
                    if rc == 0:
                        break
                    assert rc == B.TIDE_INGEST_ERR_BUSY
                host_view(addr, nbytes)[:] = bits[i + 1].view(np.uint8)
                assert B.tide_ingest_submit(q, nslot, bufs[(i + 1) & 1], nbytes, tr._stream(), True) == 0
            tr.hidden, tr.tokens, tr.mask = bufs[i & 1], toks[i], masks[i]
            tr.train_step(cfg["lr"])
            losses.append(tr.loss.clone())                      # device-side copy on the compute stream, no sync
            if i + 1 < len(batches):
                slot = nslot
        sync()
        assert [float(x.item()) for x in losses] == ref_losses
        for k in tr.grads:
            assert torch.equal(tr.grads[k], ref.grads[k]), k
            assert torch.equal(tr.params[k], ref.params[k]), k
    finally:
        assert B.tide_ingest_destroy(q) == 0


def test_ring_states_and_errors():
    from paper_2602_05145_amd import binding as B
    rc, q = B.tide_ingest_create(0, 3)
    assert rc == B.TIDE_INGEST_ERR_ARG
    rc, q = B.tide_ingest_create(1024, 1)
    assert rc == B.TIDE_INGEST_ERR_ARG and "n_slots" in B.tide_ingest_last_error()
    nbytes = 1 << 20
    rc, q = B.tide_ingest_create(nbytes, 3)
    assert rc == 0
    try:
        dev = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0") for _ in range(4)]
        slots = []
        for i in range(3):
            rc, slot, addr = B.tide_ingest_acquire(q)
            assert rc == 0 and slot == i
            host_view(addr, nbytes)[:] = (np.arange(nbytes) * (i + 3) % 251).astype(np.uint8)
            slots.append(slot)
        rc, slot, addr = B.tide_ingest_acquire(q)
        assert rc == B.TIDE_INGEST_ERR_BUSY                                  # every slot is being filled
        assert B.tide_ingest_wait(q, 0, 0) == B.TIDE_INGEST_ERR_BUSY         # nothing submitted yet
        assert B.tide_ingest_submit(q, 0, dev[0], nbytes + 1) == B.TIDE_INGEST_ERR_ARG
        assert B.tide_ingest_submit(q, 7, dev[0], nbytes) == B.TIDE_INGEST_ERR_ARG
        assert B.tide_ingest_submit(q, 0, None, nbytes) == B.TIDE_INGEST_ERR_NULL
        for i in slots:
            assert B.tide_ingest_submit(q, i, dev[i], nbytes) == 0
        assert B.tide_ingest_submit(q, 0, dev[0], nbytes) == B.TIDE_INGEST_ERR_BUSY   # already copying
        s = torch.cuda.current_stream().cuda_stream
        for i in slots:
            assert B.tide_ingest_wait(q, i, s) == 0
        sync()                                                                # the compute stream waited for all three
        for i in slots:
            assert B.tide_ingest_done(q, i) == 1
            want = torch.from_numpy((np.arange(nbytes) * (i + 3) % 251).astype(np.uint8))
            assert torch.equal(dev[i].cpu(), want)
        # completed slots are recycled in ring order; a partial copy moves only its bytes
        rc, slot, addr = B.tide_ingest_acquire(q)
        assert rc == 0 and slot == 0
        host_view(addr, nbytes)[:] = 255
        assert B.tide_ingest_submit(q, slot, dev[3], 4096) == 0
        assert B.tide_ingest_wait(q, slot, s) == 0
        sync()
        assert int(dev[3][:4096].min()) == 255 and int(dev[3][4096:].max()) == 0
    finally:
        assert B.tide_ingest_destroy(q) == 0
    assert B.tide_ingest_destroy(None) == B.TIDE_INGEST_ERR_NULL
