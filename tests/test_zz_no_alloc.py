"""The entry point that allocates nothing (sentry_merkle_root_noalloc, for callers that cannot
call hipMalloc) against the entry point it is a variant of, sentry_merkle_root, through the C
ABI: the same 32 bytes, on calls in a row that share the library's fixed scratch array, the
later ones with smaller inputs than the earlier ones left behind.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import binding
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def both_roots(d, size, leaf, stream=0):
    a = torch.zeros(32, dtype=torch.uint8, device="cuda")
    b = torch.zeros(32, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()     # torch fills the outputs on its own stream, which `stream` does not wait for
    sentry.sentry_merkle_root_noalloc(d.data_ptr() if size else 0, size, leaf, a.data_ptr(), stream)
    sentry.sentry_merkle_root(d.data_ptr() if size else 0, size, leaf, b.data_ptr(), stream)
    torch.cuda.synchronize()
    return bytes(a.cpu().numpy()), bytes(b.cpu().numpy())


def test_two_calls_in_a_row_the_second_smaller():
    # first call: 600,001 leaves of 64 bytes and a ragged tail (2344 workgroup nodes, two reduce
    # levels through the level buffers of the fixed array); second call: 16 MiB in 4 KiB leaves
    # (64 nodes, folded by the last workgroup of the one launch, which takes the ticket counter);
    # third: one leaf.  Each must equal the allocating entry point bit for bit, and the oracle.
    big = wl.uniform_bytes(9001, 0, 64 * 600_000 + 17)
    d = to_dev(big)
    for size, leaf in ((big.size, 64), (16 << 20, 4096), (4096, 4096), (big.size, 64), (100, 64)):
        got, ref = both_roots(d, size, leaf)
        assert got == ref, (size, leaf)
        assert got == oracle.merkle_root(big[:size], leaf), (size, leaf)


def test_smaller_then_larger_and_sizes_around_the_one_launch_limit():
    # 512 workgroup nodes is the most the last workgroup folds; 513 goes through the reduce kernel
    buf = wl.uniform_bytes(9002, 0, 64 * (64 * 513 + 5))
    d = to_dev(buf)
    for n_leaves in (2, 64, 65, 64 * 511 + 1, 64 * 512, 64 * 512 + 1, 64 * 513 + 5, 1):
        got, ref = both_roots(d, 64 * n_leaves, 64)
        assert got == ref, n_leaves
        assert got == oracle.merkle_root(buf[:64 * n_leaves], 64), n_leaves
    # the same limit with leaves long enough for the two-wave kernel (512-byte leaves)
    for n_leaves in (64 * 3 + 1, 64 * 256, 64 * 256 + 1, 64 * 512, 64 * 512 + 1):
        size = 512 * n_leaves - 5
        if size > buf.size:
            continue
        got, ref = both_roots(d, size, 512)
        assert got == ref, n_leaves
        assert got == oracle.merkle_root(buf[:size], 512), n_leaves


def test_empty_buffer_and_other_stream():
    st = torch.cuda.Stream()
    e = torch.empty(0, dtype=torch.uint8, device="cuda")
    got, ref = both_roots(e, 0, 4096, st.cuda_stream)
    assert got == ref == oracle.sha256(np.zeros(0, dtype=np.uint8))
    buf = wl.uniform_bytes(9003, 0, 1 << 20)
    d = to_dev(buf)
    got, ref = both_roots(d, buf.size, 4096, st.cuda_stream)
    assert got == ref == oracle.merkle_root(buf, 4096)


def test_the_call_makes_no_allocation_and_can_be_captured():
    # a captured graph may not contain an allocation: capturing the very first use of a size on a
    # fresh stream fails for sentry_merkle_root (it grows its scratch) and works for this one
    buf = wl.uniform_bytes(9004, 0, (8 << 20) + 100)
    d = to_dev(buf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    want = {n: oracle.merkle_root(buf[:n], 4096) for n in ((8 << 20) + 100, 1 << 20)}
    sentry.sentry_merkle_root_noalloc(d.data_ptr(), 4096, 4096, out.data_ptr())   # loads the kernels' code object
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        sentry.sentry_merkle_root_noalloc(d.data_ptr(), (8 << 20) + 100, 4096, out.data_ptr(), st.cuda_stream)
    for _ in range(3):
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want[(8 << 20) + 100]
        # a plain call with a smaller input between the replays: same array, other contents
        sentry.sentry_merkle_root_noalloc(d.data_ptr(), 1 << 20, 4096, out.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want[1 << 20]
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after >= free_before - (4 << 20)    # nothing grew (torch's own small buffers aside)


def test_sizes_beyond_the_fixed_array_are_rejected():
    d = torch.zeros(64, dtype=torch.uint8, device="cuda")
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    with pytest.raises(sentry.SentryError) as e:
        sentry.sentry_merkle_root_noalloc(d.data_ptr(), 64 * ((1 << 22) + 1), 64, out.data_ptr())
    assert e.value.code == binding.ERR_INVALID_ARG and "4194304" in str(e.value)
    # the largest size is accepted: 2^22 leaves of 64 bytes
    big = torch.zeros(64 << 22, dtype=torch.uint8, device="cuda")
    got, ref = both_roots(big, big.numel(), 64)
    assert got == ref
