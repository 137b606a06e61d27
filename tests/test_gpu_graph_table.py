"""The table of pre-recorded decode steps (Sec. 3.2.2): steps of two layers recorded for capacities 4, 8,
12 and 16; batches of several sizes replay the smallest capacity that holds them, their surplus rows
padded.  Every replay is compared with the fp64 oracle (appended caches bit for bit, the last layer's
attention within the gate), with eager work and synchronisation between the replays; one table is
recorded for a stream confined to a few compute units."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_20552_amd as adr
import workloads as W
from gpu_util import compare, dev, say

pytestmark = pytest.mark.gpu

INTERVAL, MAX_CAP, PART, LAYERS, STEPS = 4, 16, 256, 2, 3


def build(seed, flags, capture_stream):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, 1400, size=MAX_CAP).astype(np.int32)
    wl = W.Workload(94, "case", B=MAX_CAP, Hq=16, Hkv=4, d=128, lengths="given")
    b = W.make_batch(wl, device="cpu", headroom_tokens=STEPS * 8, seed_offset=seed, lens_before=lens)
    pools = [(b.k_cache, b.v_cache)] + [W.layer_pools(wl, b, i, "cpu") for i in range(1, LAYERS)]
    caches = [adr.KVCache(dev(k), dev(v)) for k, v in pools]
    host = [(W.bits(k).copy(), W.bits(v).copy()) for k, v in pools]
    max_len = int(lens.max()) + STEPS * 8
    bufs = dict(out=torch.zeros((MAX_CAP, wl.Hq, wl.d), dtype=torch.float32, device="cuda:0"),
                lse=torch.zeros((MAX_CAP, wl.Hq), dtype=torch.float32, device="cuda:0"),
                q=dev(b.q), k_new=dev(b.k_new), v_new=dev(b.v_new), table=dev(b.block_table),
                seq=torch.zeros(MAX_CAP, dtype=torch.int32, device="cuda:0"))
    ws = torch.empty(adr.adr_decode_workspace_bytes(MAX_CAP, wl.Hq, wl.d, max_len, PART), dtype=torch.uint8,
                     device="cuda:0")
    table = adr.GraphTable(bufs["out"], bufs["q"], bufs["k_new"], bufs["v_new"], caches, bufs["table"], bufs["seq"],
                           wl.scale, max_len, PART, ws, INTERVAL, MAX_CAP, capture_stream, lse=bufs["lse"],
                           flags=flags)
    return wl, b, lens, caches, host, bufs, table


def replay_and_check(wl, b, lens, caches, host, bufs, table, stream, what):
    cur = lens.copy()                                   # tokens each row holds
    for step, n in enumerate((16, 9, 5, 1, 12, 16)):
        assert table.capacity(n) == -(-n // INTERVAL) * INTERVAL
        seq = np.zeros(MAX_CAP, dtype=np.int32)
        seq[:n] = cur[:n] + 1                           # rows >= n are padded
        bufs["seq"].copy_(dev(seq))
        bufs["out"].fill_(float("nan")); bufs["lse"].fill_(float("nan"))
        torch.cuda.synchronize()
        table.launch(n, stream)
        torch.cuda.synchronize()
        pos = np.where(seq > 0, seq - 1, -1).astype(np.int32)
        for (kh, vh), c in zip(host, caches):
            oracle.kv_append(kh, vh, W.bits(b.k_new), W.bits(b.v_new), b.block_table, pos)
            assert np.array_equal(W.bits(c.k), kh) and np.array_equal(W.bits(c.v), vh), "%s step %d" % (what, step)
        ref, ref_lse, _ = oracle.decode_attention(W.bits(b.q), host[-1][0], host[-1][1], b.block_table, seq, wl.scale)
        cap = table.capacity(n)                         # the replayed step covers that many rows and no more
        compare(bufs["out"][:cap], bufs["lse"][:cap], ref[:cap], ref_lse[:cap],
                what="%s step %d, %d rows" % (what, step, n))
        assert torch.all(bufs["out"][n:cap] == 0) and torch.isnan(bufs["out"][cap:]).all()
        cur[:n] += 1
        # eager work of the program's own between the replays
        scratch = torch.empty_like(bufs["out"]).normal_()
        torch.cuda.synchronize()
        del scratch


def test_table_over_a_capacity_grid_serves_batches_of_any_size():
    side = torch.cuda.Stream()
    say("graph table, capacities 4..16")
    wl, b, lens, caches, host, bufs, table = build(31, adr.KERNEL_AUTO, side)
    try:
        assert table.capacity(17) == -1 and table.capacity(0) == INTERVAL
        with pytest.raises(adr.AdrError):
            table.launch(17, side)
        replay_and_check(wl, b, lens, caches, host, bufs, table, side, "table")
    finally:
        torch.cuda.synchronize()
        table.destroy()


def test_table_recorded_for_a_stream_confined_to_a_few_compute_units():
    """The recording cannot ask the stream for its mask: ADR_GRID_CUS sizes the grid for the 16 units."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    handle = adr.adr_stream_create_cu_mask([i < 16 for i in range(cus)])
    masked = torch.cuda.ExternalStream(handle)
    say("graph table on a CU-masked stream")
    wl, b, lens, caches, host, bufs, table = build(32, adr.KERNEL_MFMA | adr.GRID_CUS(16), masked)
    try:
        replay_and_check(wl, b, lens, caches, host, bufs, table, masked, "masked table")
    finally:
        torch.cuda.synchronize()
        table.destroy()
        adr.adr_stream_destroy(handle)


def test_create_rejects_bad_arguments_without_leaving_the_stream_recording():
    side = torch.cuda.Stream()
    wl = W.Workload(94, "case", B=8, Hq=16, Hkv=4, d=128, lengths="given")
    b = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=33, lens_before=np.full(8, 40, dtype=np.int32))
    cache = adr.KVCache(dev(b.k_cache), dev(b.v_cache))
    out = torch.zeros((8, 16, 128), dtype=torch.float32, device="cuda:0")
    seq = dev(b.seq_lens)
    args = (out, dev(b.q), dev(b.k_new), dev(b.v_new), [cache], dev(b.block_table), seq, wl.scale)
    say("graph table, rejected arguments")
    for kw in (dict(interval=3, max_capacity=8),               # not a multiple
               dict(interval=0, max_capacity=8)):
        with pytest.raises(adr.AdrError):
            adr.GraphTable(*args, 64, 16, None, capture_stream=side, **kw)
    with pytest.raises(adr.AdrError):                          # a split pass without a workspace: refused inside the recording
        adr.GraphTable(*args, 64, 16, None, 4, 8, side)
    # the stream is usable afterwards
    with torch.cuda.stream(side):
        out.fill_(1.0)
    torch.cuda.synchronize()
    assert torch.all(out == 1.0)
