"""GPU parity: lattice hash of a model (Algorithm 4, block index in front of every block)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import golden_lines, to_dev

pytestmark = pytest.mark.gpu


def gpu_model(segs, block, want_layers=True):
    devs = [to_dev(s) if s.size else torch.empty(16, dtype=torch.uint8, device="cuda") for s in segs]
    n = len(segs)
    layers = torch.full((n * 32,), 0x7777, dtype=torch.int16, device="cuda")
    total = torch.full((32,), 0x7777, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_model([d.data_ptr() for d in devs], [s.size for s in segs], block,
                               layers.data_ptr() if want_layers else 0, total.data_ptr())
    torch.cuda.synchronize()
    for d, s in zip(devs, segs):
        if s.size:
            assert (d.cpu().numpy() == s).all()
    return layers.cpu().numpy().view(np.uint16).reshape(n, 32), total.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("block", [16, 112, 128, 256, 8192])
def test_edge_lengths(block):
    sizes = [0, 1, 7, 8, 9, 15, 16, 17, 111, 112, 113, 119, 120, 121, 127, 128, 129, 247, 248, 249, 255, 256, 257,
             block - 1, block, block + 1, 3 * block, 3 * block + 5, 2 * block - 9]
    segs = [wl.uniform_bytes(3000 + i, 0, s) for i, s in enumerate(sizes)]
    want_layers, want_total = oracle.lthash_model(segs, block)
    got_layers, got_total = gpu_model(segs, block)
    assert (got_layers == want_layers).all(), np.nonzero((got_layers != want_layers).any(axis=1))
    assert (got_total == want_total).all()


def test_many_blocks_several_groups_and_no_layer_output():
    segs = [wl.uniform_bytes(3100 + i, 0, s) for i, s in enumerate([256 * 700 + 3, 256 * 256, 256 * 257, 5])]
    want_layers, want_total = oracle.lthash_model(segs, 256)
    got_layers, got_total = gpu_model(segs, 256)
    assert (got_layers == want_layers).all() and (got_total == want_total).all()
    _, only_total = gpu_model(segs, 256, want_layers=False)
    assert (only_total == want_total).all()


def test_tiny_checkpoint_default_block_size():
    tensors = wl.checkpoint_bytes_np(wl.layout_tiny())
    want_layers, want_total = oracle.lthash_model(tensors, 8192)
    got_layers, got_total = gpu_model(tensors, 8192)
    assert (got_layers == want_layers).all() and (got_total == want_total).all()


def test_block_order_matters():
    a = wl.uniform_bytes(3200, 0, 4 * 8192)
    b = a.copy()
    b[:8192], b[8192:16384] = a[8192:16384], a[:8192]
    ta = gpu_model([a], 8192)[1]
    tb = gpu_model([b], 8192)[1]
    assert (ta != tb).any() and (tb == oracle.lthash_model([b], 8192)[1]).all()


def test_a_run_of_tensors_with_its_first_block_index_and_an_update_of_one_tensor():
    # section 2.2 / 4.2.2: the digests of disjoint runs of tensors add up to the model's, so a model
    # digest is brought up to date from the digests of the changed tensor alone
    block = 256
    sizes = [256 * 5 + 3, 0, 256 * 300, 77, 256 * 40, 256 * 257 + 1]
    segs = [wl.uniform_bytes(3300 + i, 0, s) for i, s in enumerate(sizes)]
    blocks = [-(-s // block) for s in sizes]
    want_layers, want_total = oracle.lthash_model(segs, block)
    devs = [to_dev(s) if s.size else torch.empty(16, dtype=torch.uint8, device="cuda") for s in segs]
    ptrs = [d.data_ptr() for d in devs]
    total = torch.zeros(32, dtype=torch.int16, device="cuda")
    part = torch.zeros(32, dtype=torch.int16, device="cuda")
    layers = torch.zeros(6 * 32, dtype=torch.int16, device="cuda")
    for lo, hi in ((0, 2), (2, 3), (3, 6)):                        # three runs, each numbered from its first block
        first = sum(blocks[:lo])
        sentry.sentry_lthash_model_from(ptrs[lo:hi], sizes[lo:hi], block, first, layers.data_ptr() + 64 * lo, part.data_ptr())
        sentry.sentry_lthash32_combine(total.data_ptr(), part.data_ptr())
        torch.cuda.synchronize()
        w_layers, w_part = oracle.lthash_model(segs[lo:hi], block, first_index=first)
        assert (part.cpu().numpy().view(np.uint16) == w_part).all(), (lo, hi)
    assert (total.cpu().numpy().view(np.uint16) == want_total).all()
    assert (layers.cpu().numpy().view(np.uint16).reshape(6, 32) == want_layers).all()
    # tensor 4 changes: model' = model - digest(old tensor 4) + digest(new tensor 4)
    new4 = wl.uniform_bytes(3399, 0, sizes[4])
    d_new = to_dev(new4)
    first = sum(blocks[:4])
    old_digest = torch.zeros(32, dtype=torch.int16, device="cuda")
    new_digest = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_model_from([ptrs[4]], [sizes[4]], block, first, 0, old_digest.data_ptr())
    sentry.sentry_lthash_model_from([d_new.data_ptr()], [sizes[4]], block, first, 0, new_digest.data_ptr())
    sentry.sentry_lthash32_remove(total.data_ptr(), old_digest.data_ptr())
    sentry.sentry_lthash32_combine(total.data_ptr(), new_digest.data_ptr())
    torch.cuda.synchronize()
    changed = segs[:4] + [new4] + segs[5:]
    assert (total.cpu().numpy().view(np.uint16) == oracle.lthash_model(changed, block)[1]).all()
    # with the wrong first index the digest is another one: the index is part of what is hashed
    sentry.sentry_lthash_model_from([ptrs[4]], [sizes[4]], block, first + 1, 0, part.data_ptr())
    torch.cuda.synchronize()
    assert (part.cpu() != old_digest.cpu()).any()


def test_config3_checkpoint_model_lattice_hash():
    # the 7B checkpoint (291 fragmented tensors), 8 KiB blocks, against the stored oracle digests
    lines = golden_lines("config3_model_lthash.txt")
    want_total = np.array([int(x, 16) for x in lines[0].split()], np.uint16)
    want_layers = np.array([[int(x, 16) for x in ln.split()[1:]] for ln in lines[1:]], np.uint16)
    lay = wl.layout_7b()
    tensors = [wl.checkpoint_tensor(lay, i, base_seed=wl.SEED_C3, device="cuda") for i in range(len(lay))]
    layers = torch.zeros(len(lay) * 32, dtype=torch.int16, device="cuda")
    total = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_model([t.data_ptr() for t in tensors], [2 * t.numel() for t in tensors], 8192,
                               layers.data_ptr(), total.data_ptr())
    torch.cuda.synchronize()
    assert (layers.cpu().numpy().view(np.uint16).reshape(len(lay), 32) == want_layers).all()
    assert (total.cpu().numpy().view(np.uint16) == want_total).all()
    del tensors
    import gc
    gc.collect()
    torch.cuda.empty_cache()
