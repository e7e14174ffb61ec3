"""GPU parity: the HIP Merkle path against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def gpu_root(buf_np, leaf, stream=0, out=None):
    d = to_dev(buf_np) if buf_np.size else torch.empty(0, dtype=torch.uint8, device="cuda")
    out = torch.zeros(32, dtype=torch.uint8, device="cuda") if out is None else out
    sentry.sentry_merkle_root(d.data_ptr() if buf_np.size else 0, buf_np.size, leaf, out.data_ptr(), stream)
    torch.cuda.synchronize()
    return bytes(out.cpu().numpy())


@pytest.mark.parametrize("leaf", [64, 128, 4096])
def test_edge_lengths(leaf):
    for n in (0, 1, 3, 4, 55, 56, 63, 64, 65, 119, 120, 127, 128, leaf - 1, leaf, leaf + 1,
              2 * leaf, 2 * leaf + 57, 3 * leaf, 5 * leaf - 8):
        buf = wl.uniform_bytes(100 + leaf, 0, n)
        assert gpu_root(buf, leaf) == oracle.merkle_root(buf, leaf), (leaf, n)


@pytest.mark.parametrize("n_leaves", [2, 3, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1025,
                                      256 * 512 - 1, 256 * 512, 256 * 512 + 1, 256 * 512 + 257])
def test_leaf_counts_across_group_boundaries(n_leaves):
    # 64-byte leaves: group boundaries of the leaf kernel (256) and of the reduce kernel (512)
    for tail in (0, 17):
        size = 64 * n_leaves - (64 - tail if tail else 0)
        buf = wl.uniform_bytes(200, 0, size)
        assert gpu_root(buf, 64) == oracle.merkle_root(buf, 64), (n_leaves, tail)


def test_very_long_leaves():
    # 16 MiB leaves (262,144 blocks per lane): three full leaves and a short one; one leaf that
    # is the whole buffer; through the root, the leaf digests and the BLAKE2b tree
    leaf = 16 << 20
    buf = wl.uniform_bytes(210, 0, 3 * leaf + 12345)
    assert gpu_root(buf, leaf) == oracle.merkle_root(buf, leaf)
    d = to_dev(buf)
    leaves = torch.zeros(4 * 32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_leaves(d.data_ptr(), buf.size, leaf, leaves.data_ptr())
    out = torch.zeros(64, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_root_h(sentry.HASH_BLAKE2B, d.data_ptr(), buf.size, leaf, out.data_ptr())
    torch.cuda.synchronize()
    assert (leaves.cpu().numpy().reshape(4, 32) == oracle.merkle_leaves(buf, leaf)).all()
    assert bytes(out.cpu().numpy()) == oracle.merkle_root_h(sentry.HASH_BLAKE2B, buf, leaf)
    one = buf[:leaf // 2 + 77]
    assert gpu_root(one, leaf) == oracle.sha256(one)


def test_config1_16mib_4k_leaves():
    buf = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20)
    want = oracle.merkle_root(buf, 4096)
    got = gpu_root(buf, 4096)
    assert got == want
    assert sentry.sentry_verify(got, want) == 0


def test_leaves_and_reduce_entry_points():
    buf = wl.uniform_bytes(300, 0, 192 * 1000 + 100)
    d = to_dev(buf)
    n = 1001
    leaves = torch.zeros(n * 32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_leaves(d.data_ptr(), buf.size, 192, leaves.data_ptr())
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_reduce(leaves.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    want_leaves = oracle.merkle_leaves(buf, 192)
    assert (leaves.cpu().numpy().reshape(n, 32) == want_leaves).all()
    assert bytes(out.cpu().numpy()) == oracle.merkle_root(buf, 192)


@pytest.mark.parametrize("n", [1, 2, 3, 511, 512, 513, 262143, 262145, 2_105_001])
def test_reduce_node_counts(n):
    # 2,105,001 is the leaf count of the 70B checkpoint at 64 KiB leaves
    nodes = wl.uniform_bytes(400 + n % 7, 0, 32 * n)
    d = to_dev(nodes)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_reduce(d.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == oracle.merkle_reduce(nodes.reshape(n, 32))
    assert (d.cpu().numpy() == nodes).all()          # input not modified


def test_input_is_not_modified_and_runs_are_deterministic():
    buf = wl.uniform_bytes(500, 0, 4096 * 300 + 77)
    d = to_dev(buf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    seen = set()
    for _ in range(10):
        sentry.sentry_merkle_root(d.data_ptr(), buf.size, 4096, out.data_ptr())
        torch.cuda.synchronize()
        seen.add(bytes(out.cpu().numpy()))
    assert seen == {oracle.merkle_root(buf, 4096)}
    assert (d.cpu().numpy() == buf).all()


def test_output_to_pinned_host_unaligned_and_on_a_side_stream():
    buf = wl.uniform_bytes(600, 0, 1 << 20)
    want = oracle.merkle_root(buf, 8192)
    d = to_dev(buf)
    pinned = torch.zeros(64, dtype=torch.uint8).pin_memory()
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    sentry.sentry_merkle_root(d.data_ptr(), buf.size, 8192, pinned.data_ptr() + 3, s.cuda_stream)
    s.synchronize()
    assert bytes(pinned[3:35].numpy()) == want
    assert not pinned[:3].any() and not pinned[35:].any()
    dev_out = torch.zeros(64, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()     # torch fills dev_out on its own stream, which s does not wait for
    sentry.sentry_merkle_root(d.data_ptr(), buf.size, 8192, dev_out.data_ptr() + 5, s.cuda_stream)
    s.synchronize()
    assert bytes(dev_out[5:37].cpu().numpy()) == want


def test_byte_flip_changes_root():
    buf = wl.uniform_bytes(700, 0, 64 * 1024)
    a = gpu_root(buf, 1024)
    buf2 = buf.copy()
    buf2[33 * 1024 + 5] ^= 1
    b = gpu_root(buf2, 1024)
    assert a != b and b == oracle.merkle_root(buf2, 1024)
    assert sentry.sentry_verify(a, b) == 1


def segments_case(sizes, leaf, want_roots=True, misalign_roots=False):
    segs = [wl.uniform_bytes(800 + i, 0, s) for i, s in enumerate(sizes)]
    devs = [to_dev(s) if s.size else torch.empty(16, dtype=torch.uint8, device="cuda") for s in segs]
    n = len(sizes)
    roots = torch.zeros(32 * n + 16, dtype=torch.uint8, device="cuda")
    top = torch.zeros(32, dtype=torch.uint8, device="cuda")
    roots_ptr = (roots.data_ptr() + (8 if misalign_roots else 0)) if want_roots else 0
    sentry.sentry_merkle_segments([d.data_ptr() for d in devs], list(sizes), leaf, roots_ptr, top.data_ptr())
    torch.cuda.synchronize()
    want_seg, want_top = oracle.merkle_segments(segs, leaf)
    assert bytes(top.cpu().numpy()) == want_top
    if want_roots:
        o = 8 if misalign_roots else 0
        got = roots.cpu().numpy()[o:o + 32 * n].reshape(n, 32)
        assert [bytes(r) for r in got] == want_seg
    for d, s in zip(devs, segs):
        if s.size:
            assert (d.cpu().numpy() == s).all()


def test_segments_small_and_edge():
    segments_case([4096 * 3, 17, 4096, 0, 4096 * 2 + 1, 64], 4096)
    segments_case([100], 64)
    segments_case([64 * 5, 64 * 7], 64, want_roots=False)
    segments_case([64 * 5, 64 * 7, 64], 64, misalign_roots=True)


def test_segments_multi_stage():
    # more than 256 leaves per segment: later stages; more than 256*512: three stages
    segments_case([64 * 300, 64 * 256, 64 * 257 + 3, 64, 64 * 1000], 64)
    segments_case([64 * (256 * 512 + 5), 64 * 10, 64 * (256 * 3)], 64)


def test_segments_tiny_checkpoint_layout():
    lay = wl.layout_tiny()
    tensors = wl.checkpoint_bytes_np(lay)
    devs = [to_dev(t) for t in tensors]
    n = len(tensors)
    roots = torch.zeros(32 * n, dtype=torch.uint8, device="cuda")
    top = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments([d.data_ptr() for d in devs], [t.size for t in tensors], 4096,
                                  roots.data_ptr(), top.data_ptr())
    torch.cuda.synchronize()
    want_seg, want_top = oracle.merkle_segments(tensors, 4096)
    assert [bytes(r) for r in roots.cpu().numpy().reshape(n, 32)] == want_seg
    assert bytes(top.cpu().numpy()) == want_top
    # one segment is the plain root
    one = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments([devs[0].data_ptr()], [tensors[0].size], 4096, 0, one.data_ptr())
    torch.cuda.synchronize()
    assert bytes(one.cpu().numpy()) == oracle.merkle_root(tensors[0], 4096)


def test_changed_tensors_update_the_model_root_through_their_roots():
    # the per-layer granularity of section 4.1 (fine-tuning changes some layers, the rest is frozen):
    # with the tensor roots kept, a changed tensor costs its own tree (sentry_merkle_root into its
    # place among the roots) and the tree over the roots (sentry_merkle_reduce), and the result is
    # the model root that hashing everything again gives
    lay = wl.layout_tiny()
    tensors = [t.copy() for t in wl.checkpoint_bytes_np(lay)]
    devs = [to_dev(t) for t in tensors]
    n = len(tensors)
    ptrs, lens = [d.data_ptr() for d in devs], [t.size for t in tensors]
    roots = torch.zeros(32 * n, dtype=torch.uint8, device="cuda")
    top = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments(ptrs, lens, 4096, roots.data_ptr(), top.data_ptr())
    torch.cuda.synchronize()
    before = bytes(top.cpu().numpy())
    for i in (0, n // 2, n - 1):
        tensors[i][tensors[i].size // 3] ^= 0x40
        devs[i].copy_(torch.from_numpy(tensors[i]))
        sentry.sentry_merkle_root(ptrs[i], lens[i], 4096, roots.data_ptr() + 32 * i)
    sentry.sentry_merkle_reduce(roots.data_ptr(), n, top.data_ptr())
    torch.cuda.synchronize()
    want_seg, want_top = oracle.merkle_segments(tensors, 4096)
    assert [bytes(r) for r in roots.cpu().numpy().reshape(n, 32)] == want_seg
    assert bytes(top.cpu().numpy()) == want_top != before
    again = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments(ptrs, lens, 4096, 0, again.data_ptr())
    torch.cuda.synchronize()
    assert bytes(again.cpu().numpy()) == want_top


@pytest.mark.parametrize("leaf,n_leaves,tail", [
    (512, 64 * 300 + 5, 0), (512, 64 * 257 + 1, 57), (1024, 64 * 256, 0), (1024, 64 * 256 + 1, 3),
    (512, 64 * 511 + 63, 511), (512, 64 * 512, 0), (512, 64 * 513, 9), (576, 129, 0), (4096, 65, 56),
])
def test_two_wave_split_kernel_group_counts(leaf, n_leaves, tail):
    # leaves of 512 bytes and more in launches of up to 512 groups of 64 leaves take the
    # producer/consumer kernel: one pair per workgroup up to 256 groups, two pairs above
    size = leaf * (n_leaves - 1) + (tail if tail else leaf)
    buf = wl.uniform_bytes(900 + n_leaves % 11, 0, size)
    assert gpu_root(buf, leaf) == oracle.merkle_root(buf, leaf)
    d = to_dev(buf)
    leaves = torch.zeros(n_leaves * 32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_leaves(d.data_ptr(), size, leaf, leaves.data_ptr())
    torch.cuda.synchronize()
    assert (leaves.cpu().numpy().reshape(n_leaves, 32) == oracle.merkle_leaves(buf, leaf)).all()


def inplace_case(sizes, leaf):
    segs = [wl.uniform_bytes(950 + i, 0, s) for i, s in enumerate(sizes)]
    devs = [to_dev(s) if s.size else torch.empty(16, dtype=torch.uint8, device="cuda") for s in segs]
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_inplace([d.data_ptr() for d in devs], list(sizes), leaf, out.data_ptr())
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == oracle.merkle_inplace(segs, leaf), (sizes, leaf)
    for d, s in zip(devs, segs):
        if s.size:
            assert (d.cpu().numpy() == s).all()


def test_inplace_flat_tree():
    # Algorithm 3: one tree over the blocks of all tensors, short tails kept short
    inplace_case([4096 * 3, 17, 4096, 0, 4096 * 2 + 1, 64], 4096)
    inplace_case([100], 64)
    inplace_case([0, 0], 64)
    inplace_case([64 * 300, 64 * 256, 64 * 257 + 3, 64, 64 * 1000], 64)
    inplace_case([512 * 70 + 9, 512 * 64, 5, 512 * 200], 512)            # two-wave kernel
    inplace_case([64 * (256 * 512 + 5), 64 * 10, 64 * (256 * 3)], 64)    # 256-leaf groups, three reduce passes
    # whole blocks everywhere: equal to the tree over the concatenation (Algorithm 1)
    sizes = [4096 * 5, 4096, 4096 * 11]
    segs = [wl.uniform_bytes(990 + i, 0, s) for i, s in enumerate(sizes)]
    devs = [to_dev(s) for s in segs]
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_inplace([d.data_ptr() for d in devs], sizes, 4096, out.data_ptr())
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == oracle.merkle_root(np.concatenate(segs), 4096)


@pytest.mark.parametrize("n_seg,leaf,max_leaves", [
    (300, 1024, 5),      # under 512 waves of 1 KiB leaves: the two-wave kernel, one pair per workgroup and two
    (700, 512, 60),
    (3000, 64, 70),      # single-wave workgroups of the plain kernel
    (9000, 64, 40),      # 256-lane workgroups
])
def test_packed_leaf_stage_many_small_tensors(n_seg, leaf, max_leaves):
    # few leaves per tensor: the leaf stage packs leaves of different tensors into one wave and
    # finds each lane's tensor by bisection; empty tensors, short tails, runs of one-leaf tensors
    rng = np.random.default_rng(n_seg)
    sizes = (rng.integers(0, max_leaves, n_seg) * leaf + rng.integers(0, leaf, n_seg) * (rng.random(n_seg) < 0.5)).astype(np.int64)
    sizes[rng.integers(0, n_seg, n_seg // 20)] = 0
    sizes[5:25] = leaf - 3                     # one short leaf each
    sizes[-1] = 0                              # the list ends with an empty tensor
    sizes = [int(x) for x in sizes]
    segments_case(sizes, leaf)
    inplace_case(sizes, leaf)


def test_inplace_tiny_checkpoint_layout():
    lay = wl.layout_tiny()
    tensors = wl.checkpoint_bytes_np(lay)
    devs = [to_dev(t) for t in tensors]
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    for leaf in (8192, 4096, 1 << 20):
        sentry.sentry_merkle_inplace([d.data_ptr() for d in devs], [t.size for t in tensors], leaf, out.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == oracle.merkle_inplace(tensors, leaf), leaf
