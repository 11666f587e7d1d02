"""Swap engine on the GPU: bit-exact round trips, ordering against the
compute stream, the event-aware arena, and state errors."""
import numpy as np
import pytest
import torch

from paper_1812_07816_amd import swap as sw
from paper_1812_07816_amd._lib import Mi3dError

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def _engine(sizes, budget, arena_bytes=0, lookahead=1, policy=sw.POLICY_ALL, **kw):
    n = len(sizes)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda") if arena_bytes else None
    e = sw.SwapEngine(budget_bytes=budget, host_pool_bytes=sum((s + 4095) // 4096 * 4096 for s in sizes) + 4096,
                      arena=arena, lookahead=lookahead, policy=policy, **kw)
    e.set_timeline(n, 2 * n)
    for i, s in enumerate(sizes):
        e.register(i, s, i, min(i + 1, n - 1), 2 * n - 1 - i, 2 * n - 1 - i, sw.TAG_ENCODER)
    e.plan(allow_over_budget=True)
    return e


def test_round_trip_is_bit_exact(device):
    sizes = [8 * MiB + 256, 3 * MiB, 4096, 2]
    e = _engine(sizes, budget=1 << 40)
    g = torch.Generator(device="cuda").manual_seed(7)
    src = [torch.randint(0, 256, (s,), dtype=torch.uint8, device="cuda", generator=g) for s in sizes]
    keep = [t.clone() for t in src]
    for i, t in enumerate(src):
        e.swap_out(i, t.data_ptr())
        e.release(i)
        t.fill_(0xFF)            # reuse of the device block on the same stream must be safe after release
    dst = [torch.zeros_like(t) for t in src]
    for i in reversed(range(len(sizes))):
        e.swap_in(i, dst[i].data_ptr())
    for i in reversed(range(len(sizes))):
        e.wait_in(i)
        assert torch.equal(dst[i], keep[i])      # runs on the waiting stream
        e.done(i)
    st = e.stats()
    assert st["bytes_out"] == st["bytes_in"] == sum(sizes)
    assert st["n_swapped_out"] == st["n_swapped_in"] == len(sizes)
    assert st["copy_ms_out"] > 0 and st["copy_ms_in"] > 0 and 0 < st["busy_ms"] <= st["copy_ms_out"] + st["copy_ms_in"] + 1e-3
    e.close()


def test_bf16_activation_round_trip_through_arena(device):
    n = 1 << 22
    arena_bytes = 3 * n * 2 + 1024
    e = _engine([2 * n, 2 * n], budget=1 << 40, arena_bytes=arena_bytes)
    p0 = e.alloc(2 * n)
    p1 = e.alloc(2 * n)
    assert p0 % 256 == 0 and p1 % 256 == 0 and p1 >= p0 + 2 * n
    import ctypes
    def view(ptr):
        base = e.arena.data_ptr()
        return e.arena[ptr - base: ptr - base + 2 * n].view(torch.bfloat16)
    a0, a1 = view(p0), view(p1)
    a0.copy_(torch.randn(n, device="cuda").bfloat16()); a1.copy_(torch.randn(n, device="cuda").bfloat16())
    k0, k1 = a0.clone(), a1.clone()
    e.swap_out(0, p0); e.release(0)
    e.swap_out(1, p1); e.release(1)
    # blocks come back only with the copy events attached: writing into a fresh
    # allocation right away must not corrupt the data in flight
    q = e.alloc(2 * n); view(q).fill_(-1.0)
    q2 = e.alloc(2 * n); view(q2).fill_(-2.0)
    e.free(q); e.free(q2)
    r1 = e.alloc(2 * n); e.swap_in(1, r1)
    r0 = e.alloc(2 * n); e.swap_in(0, r0)
    e.wait_in(1); e.wait_in(0)
    assert torch.equal(view(r1).view(torch.int16), k1.view(torch.int16))
    assert torch.equal(view(r0).view(torch.int16), k0.view(torch.int16))
    assert e.stats()["peak_arena_bytes"] <= arena_bytes
    with pytest.raises(Mi3dError) as ei:
        e.alloc(arena_bytes)
    assert ei.value.status == -6
    e.close()


def test_copy_waits_for_the_producer_and_consumer_waits_for_the_copy(device):
    n = 32 * MiB
    e = _engine([n], budget=1 << 40)
    x = torch.zeros(n, dtype=torch.uint8, device="cuda")
    # a long chain of kernels on the compute stream produces the final value
    for _ in range(50):
        x.add_(1)
    e.swap_out(0, x.data_ptr())      # must see 50, not an intermediate value
    e.release(0)
    x.zero_()
    y = torch.empty_like(x)
    e.swap_in(0, y.data_ptr())
    e.wait_in(0)
    z = y.clone()                    # enqueued behind the wait
    torch.cuda.synchronize()
    assert int(z.min()) == 50 and int(z.max()) == 50
    e.close()


def test_state_errors(device):
    e = _engine([4096, 4096], budget=1 << 40, policy=sw.POLICY_FIRST_N, n_tensors=1)
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    def status(fn):
        with pytest.raises(Mi3dError) as ei:
            fn()
        return ei.value.status
    assert status(lambda: e.swap_out(1, buf.data_ptr())) == -7      # not in the swap set
    assert status(lambda: e.swap_in(0, buf.data_ptr())) == -7       # still on the device
    assert status(lambda: e.swap_out(7, buf.data_ptr())) == -7      # unknown id
    e.swap_out(0, buf.data_ptr())
    assert status(lambda: e.swap_out(0, buf.data_ptr())) == -7      # double swap-out
    assert status(lambda: e.wait_in(0)) == -7
    e.release(0)
    assert status(lambda: e.release(0)) == -7
    e.swap_in(0, buf.data_ptr())
    assert status(lambda: e.swap_in(0, buf.data_ptr())) == -7
    assert status(lambda: e.done(0)) == -7                           # not waited for yet
    e.wait_in(0); e.done(0)
    e.reset_step()
    e.swap_out(0, buf.data_ptr()); e.release(0)                      # the step can run again
    e.sync()
    e.close()


def test_pool_too_small_is_reported(device):
    e = sw.SwapEngine(budget_bytes=1 << 40, host_pool_bytes=8192, policy=sw.POLICY_ALL)
    e.set_timeline(2, 4)
    e.register(0, 8192, 0, 1, 3, 3)
    e.register(1, 8192, 1, 1, 2, 2)
    with pytest.raises(Mi3dError) as ei:
        e.plan()
    assert ei.value.status == -5
    e.close()


def _checksum_ref(raw):
    """The documented function, written out with numpy: sum of word_i * (2 i + 1) modulo 2^64 over the 8-byte
    little-endian words, the tail zero-extended."""
    b = np.frombuffer(raw, dtype=np.uint8)
    pad = (-b.size) % 8
    w = np.concatenate([b, np.zeros(pad, dtype=np.uint8)]).view("<u8")
    with np.errstate(over="ignore"):
        return int(np.sum(w * (2 * np.arange(w.size, dtype=np.uint64) + np.uint64(1)), dtype=np.uint64))


@pytest.mark.parametrize("nbytes", [8, 13, 4096, 3 * MiB + 5])
def test_checksum_function_and_what_it_notices(device, nbytes):
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    t = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    c0 = sw.checksum64(t)
    assert c0 == _checksum_ref(t.cpu().numpy().tobytes())
    u = t.clone()
    u[nbytes // 2] ^= 1                                  # one flipped bit
    assert sw.checksum64(u) != c0
    if nbytes >= 24:                                     # two words that changed places
        v = t.clone().view(-1)[: nbytes // 8 * 8].view(torch.int64)
        if int(v[0]) != int(v[1]):
            a, b = int(v[0]), int(v[1])
            v[0], v[1] = b, a
            full = t.clone()
            full[: v.numel() * 8] = v.view(torch.uint8)
            assert sw.checksum64(full) != c0


def test_checksum_mode_confirms_every_round_trip(device):
    sizes = [6 * MiB + 24, 2 * MiB, 4096, 10]
    e = _engine(sizes, budget=1 << 40)
    e.set_verify(True)
    g = torch.Generator(device="cuda").manual_seed(11)
    src = [torch.randint(0, 256, (s,), dtype=torch.uint8, device="cuda", generator=g) for s in sizes]
    keep = [t.clone() for t in src]
    for step in range(2):                                # the second step reuses the checksum slots
        e.reset_step()
        for i, t in enumerate(src):
            e.swap_out(i, t.data_ptr())
            e.release(i)
        dst = [torch.zeros_like(t) for t in src]
        for i in reversed(range(len(sizes))):
            e.swap_in(i, dst[i].data_ptr())
            e.wait_in(i)
            e.done(i)
        st = e.stats()
        assert st["n_checksummed"] == len(sizes) and st["n_checksum_mismatch"] == 0, st
        assert all(torch.equal(a, b) for a, b in zip(dst, keep))
    e.close()
