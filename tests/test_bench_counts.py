"""The operation counts behind bench.py's roofline fractions, checked against counts obtained by
walking the definitions (FIPS 180-4 padding, the pairwise tree, BLAKE2b block counts)."""
import random

import bench


def sha_blocks(n):            # compressions of SHA-256 over n bytes: n + 1 + 8 bytes in 64-byte blocks
    return (n + 9 + 63) // 64


def tree_nodes(n_leaves):     # inner nodes hashed by the pairwise rule (a lone last node moves up unhashed)
    nodes = 0
    while n_leaves > 1:
        nodes += n_leaves // 2
        n_leaves = (n_leaves + 1) // 2
    return nodes


def leaves_of(n, leaf, empty_has_leaf=True):
    if n == 0:
        return [0] if empty_has_leaf else []
    return [min(leaf, n - s) for s in range(0, n, leaf)]


def walk_sha(lens, leaf, flat):
    ops, tops = 0, 0
    for n in lens:
        ls = leaves_of(n, leaf, empty_has_leaf=not flat)
        for l in ls:
            b = sha_blocks(l)
            # a whole number of blocks ends in one padding block whose schedule is a constant
            const = 1 if l % 64 == 0 and l > 0 else 0
            ops += (b - const) * bench.SHA_BLOCK_OPS + const * bench.SHA_CONST_BLOCK_OPS
        if flat:
            tops += len(ls)
        else:
            ops += tree_nodes(len(ls)) * (bench.SHA_BLOCK_OPS + bench.SHA_CONST_BLOCK_OPS)
            tops += 1
    return ops + tree_nodes(max(tops, 1)) * (bench.SHA_BLOCK_OPS + bench.SHA_CONST_BLOCK_OPS)


def test_sha_tree_ops_match_a_walk_over_the_definitions():
    rng = random.Random(5)
    for _ in range(200):
        leaf = rng.choice([64, 128, 4096])
        lens = [rng.choice([0, 1, 55, 56, 63, 64, 65, leaf - 1, leaf, leaf + 1, 3 * leaf, 3 * leaf + 57,
                            rng.randrange(0, 20 * leaf)]) for _ in range(rng.randrange(1, 9))]
        for flat in (False, True):
            if flat and sum(lens) == 0:
                continue      # the single empty leaf of an all-empty flat tree is priced by the caller
            assert bench.sha_tree_ops(lens, leaf, flat=flat) == walk_sha(lens, leaf, flat), (lens, leaf, flat)
    # tree levels of the chain floor
    assert [bench.tree_levels(n) for n in (1, 2, 3, 4, 5, 64, 65, 4096)] == [0, 1, 2, 2, 3, 6, 7, 12]


def test_instruction_mixes_and_issue_bound():
    # totals per unit, as the hot loops compile (cross-checked against SQ_INSTS_VALU in profiles/)
    assert bench.SHA_BLOCK_OPS == 64 * 14 + 48 * 10 + 16 + 8 == 1400
    assert bench.SHA_CONST_BLOCK_OPS == 64 * 14 + 8 == 904
    assert bench.B2_BLOCK_OPS == 96 * 20 + 32 == 1952          # a 64-bit add is one instruction
    assert bench.B2_EXPAND_OPS == 1952 - 96 + 16 == 1872
    assert bench.KECCAK_BLOCK_OPS == 24 * 190 + 34 == 4594
    # a mix of one opcode is bound by that opcode's rate; a mix of two by their harmonic blend
    for op, rate in bench.ISSUE_RATE_TOPS.items():
        assert abs(bench.issue_bound(bench.Mix({op: 123})) - rate * 1e12) < 1e3
    m = bench.Mix({"v_xor_b32": 100, "v_alignbit_b32": 100})
    want = 200 / (100 / bench.ISSUE_RATE_TOPS["v_xor_b32"] + 100 / bench.ISSUE_RATE_TOPS["v_alignbit_b32"]) * 1e12
    assert abs(bench.issue_bound(m) - want) < 1e3
    # every hash's ceiling lies between its slowest and its fastest opcode, and every opcode of every
    # mix has a measured rate
    for mix in (bench.SHA_BLOCK_MIX, bench.SHA_CONST_BLOCK_MIX, bench.B2_BLOCK_MIX, bench.B2_EXPAND_MIX, bench.KECCAK_BLOCK_MIX):
        rates = [bench.ISSUE_RATE_TOPS[op] for op in mix]
        assert min(rates) * 1e12 <= bench.issue_bound(mix) <= max(rates) * 1e12
    # mixes add and scale like the counts they stand for
    assert (3 * bench.SHA_BLOCK_MIX + bench.SHA_CONST_BLOCK_MIX).total() == 3 * 1400 + 904
    assert bench.sha_tree_mix([4096 * 5 + 3], 4096).total() == bench.sha_tree_ops([4096 * 5 + 3], 4096)
    # fractions: an entry that runs exactly at its issue bound has issue_frac 1 and alu_frac = bound / nominal
    mix = 1000 * bench.B2_BLOCK_MIX
    e = bench.rated({"ms": mix.total() / bench.issue_bound(mix) * 1e3, "bytes": 128000}, mix)
    assert abs(e["issue_frac"] - 1) < 1e-9 and abs(e["alu_frac"] - bench.issue_bound(mix) / bench.ALU_PEAK_OPS) < 1e-9


def test_blake2b_and_keccak_counts():
    rng = random.Random(6)
    lens = [rng.randrange(0, 5000) for _ in range(50)] + [0, 1, 127, 128, 129, 256]
    want = sum(max(1, -(-n // 128)) for n in lens) * bench.B2_BLOCK_OPS + len(lens) * 32 * bench.B2_EXPAND_OPS
    assert bench.lthash_ops(lens) == want
    # the 32-partition hash: the same root blocks, no expansion, 16 packed adds per digest
    assert bench.lthash32_mix(lens).total() == want - len(lens) * 32 * bench.B2_EXPAND_OPS + 16 * len(lens)
    # model lattice hash: 8 index bytes in front of every block
    for n, blk in ((0, 8192), (1, 8192), (8192, 8192), (8193, 8192), (3 * 112 + 5, 112), (120, 120), (121, 120)):
        blocks = leaves_of(n, blk, empty_has_leaf=False)
        assert bench.model_lthash_ops([n], blk) == sum(-(-(b + 8) // 128) for b in blocks) * bench.B2_BLOCK_OPS, (n, blk)
    # trees over the other two hashes: one leaf, and two leaves with their node
    assert bench.other_tree_ops("blake2b", [100], 128) == bench.B2_BLOCK_OPS
    assert bench.other_tree_ops("blake2b", [300], 128) == 3 * bench.B2_BLOCK_OPS + 2 * bench.B2_BLOCK_OPS
    assert bench.other_tree_ops("sha3_256", [135], 4096) == bench.KECCAK_BLOCK_OPS
    assert bench.other_tree_ops("sha3_256", [136], 4096) == 2 * bench.KECCAK_BLOCK_OPS      # rate 136: padding needs a block
    assert bench.other_tree_ops("sha3_256", [8192, 8192], 8192, flat=True) == (2 * 61 + 1) * bench.KECCAK_BLOCK_OPS
