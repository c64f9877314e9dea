"""GPU parity where a dropped or doubled token would hide inside the tolerance on N(0,1) data: one key that
carries all the softmax weight (score about 40 above the rest) sits at the last live token of a partial tile,
on either side of a tile, chunk and block boundary, at the first and last token of each tier and in the partly
filled newest block of a selected host tier.  With that key the output must be its (decompressed) value row, so
losing the token, reading the neighbour's row or counting it twice fails by O(1), not by 1/N."""
import numpy as np
import pytest
import torch

from paper_2604_19769_amd import binding as B
from paper_2604_19769_amd import synth
from ttkv_testlib import Pair, assert_close, dev

pytestmark = pytest.mark.gpu

ALPHA = 5.0          # planted key = ALPHA * direction; score = ALPHA * |u|^2 / sqrt(128) ~ 56, the rest stay below ~15


def directions(g, n, Hkv, dtype):
    return synth.normal(g, (n, Hkv, 128), dtype)


def queries_along(g, u, B_, Hq, Hkv, dtype):
    """Every query head of KV head h points along u[h], with its own noise: q = u + 0.5 eps."""
    G = Hq // Hkv
    q = np.repeat(u[None], B_, 0).repeat(G, axis=1) + 0.5 * g.standard_normal((B_, Hq, 128), dtype=np.float32)
    return synth.round_to(q, dtype)


def tier_positions(lo, hi, chunk, bt):
    """Sequence positions inside [lo, hi) worth a planted key: both sides of the first 16-, 32- and 64-token tile
    boundaries, of the first chunk boundary, of the last whole chunk and block, and the range's two ends."""
    n = hi - lo
    rel = {0, 1, 2, 3, 4, 15, 16, 17, 18, 19, 31, 32, 63, 64, chunk - 1, chunk, bt - 1, bt, n - 2, n - 1, n - 31, n - 32, n - 33,
           n // chunk * chunk - 1, n // chunk * chunk, n // bt * bt - 1, n // bt * bt, n // 64 * 64 - 1, n // 64 * 64,
           n // 16 * 16 - 1, n // 16 * 16}
    return sorted(lo + r for r in rel if 0 <= r < n)


def finest_items(n_tokens):
    """Tokens per work item of a run of n_tokens in HBM under the finest split (ttkv_set_split with a huge target):
    ceil(n / 256) items of equal size, a multiple of 64 tokens."""
    n = -(-n_tokens // 256)
    return (-(-n_tokens // n) + 63) // 64 * 64


def run_planted(p, B_, Hq, Hkv, dtype, lens, seed, chunks):
    """Load B_ sequences of lens[b] tokens whose keys at the listed positions point along one direction each, then
    one attention call (no append, no eviction) per direction.  The split is forced to its finest, so that the item
    boundaries are known here: chunks[t] for a host tier (fixed items), finest_items for a run in HBM."""
    B.ttkv_set_split(p.gpu.h, 1 << 20)
    g = synth.rng(seed)
    ks, vs = [], []
    for b in range(B_):
        k, v = synth.kv(seed * 31 + b, Hkv, lens[b], dtype)
        ks.append(k), vs.append(v)
    # where the tiers will sit (the loader fills tier 0 with capacity - 1 tokens, then each tier up to its capacity)
    pos = []
    for b in range(B_):
        rest, hi, P = lens[b], lens[b], []
        for t, spec in enumerate(p.tiers):
            take = rest if t == len(p.tiers) - 1 else min(rest, spec["capacity"] - 1 if t == 0 else spec["capacity"])
            if take:
                chunk = chunks[t] if spec.get("mem") == "host" else finest_items(take)
                P += tier_positions(hi - take, hi, chunk, spec["block_tokens"])
            hi, rest = hi - take, rest - take
        pos.append(sorted(set(P)))
    n_dir = max(len(x) for x in pos)
    u = directions(g, n_dir, Hkv, dtype)
    for b in range(B_):
        for j, t in enumerate(pos[b]):
            ks[b][:, t] = synth.round_to(ALPHA * u[j], dtype)
            vs[b][:, t] = synth.round_to(2.0 * g.standard_normal((Hkv, 128), dtype=np.float32), dtype)
        p.load(b, ks[b], vs[b])
    p.assert_state_equal()
    G = Hq // Hkv
    worst = 0.0
    for j in range(n_dir):
        q = queries_along(g, u[j], B_, Hq, Hkv, dtype)
        out, lse = p.gpu.decode(dev(q, dtype))
        torch.cuda.synchronize()
        out, lse = out.cpu().numpy(), lse.cpu().numpy()
        ro, rl = p.ora.attend(q)
        worst = max(worst, assert_close(out, ro, f"out direction {j}"))
        assert_close(lse, rl, f"lse direction {j}")
        for b in range(B_):
            if j >= len(pos[b]):
                continue
            # the oracle's stored value row at the planted position: the answer, whatever the other tokens hold
            t, blk, row = p.ora.locate(b, pos[b][j])
            want = np.repeat(p.ora.seq[t][b].vhat[:, blk * p.tiers[t]["block_tokens"] + row], G, axis=0)
            assert np.max(np.abs(ro[b] - want)) < 1e-5, (b, j, "the planted key does not dominate in the oracle")
            assert np.max(np.abs(out[b] - want)) < 2e-3 * max(1.0, np.max(np.abs(want))), (b, j, pos[b][j], t, blk, row)
    return worst


FORMATS = [("f16", ("f16", "f16")), ("f16", ("i8", "i8")), ("f16", ("i8", "i4")), ("f16", ("i4", "i4")), ("bf16", ("bf16", "bf16")),
           ("bf16", ("i8", "i4"))]


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (8, 2), (16, 2), (32, 2), (6, 2)])
@pytest.mark.parametrize("dtype,slow", FORMATS)
def test_dominant_key_at_tile_chunk_and_tier_ends(Hq, Hkv, dtype, slow):
    """fp window + one older tier in HBM, every stored format x 1, 2, 3, 4, 8 and 16 query heads per KV head (the
    vector kernel, and the matrix-core kernel's one- and two-pass cases)."""
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=256, block_tokens=64, ring_blocks=5),
             dict(k_fmt=slow[0], v_fmt=slow[1], capacity=10**9, block_tokens=128, ring_blocks=24)]
    p = Pair(2, Hq, Hkv, tiers, dtype)
    try:
        run_planted(p, 2, Hq, Hkv, dtype, [1033, 2890], synth.SEED_BASE + 300 + Hq, chunks=(256, 256))
        assert (p.gpu.stats()["mfma_launches"] > 0) == (Hq > Hkv)
    finally:
        p.close()


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (8, 2), (16, 2), (32, 2)])
@pytest.mark.parametrize("dtype,kfmt", [("f16", "i8"), ("bf16", "i4")])
def test_dominant_key_with_values_stored_channel_major(Hq, Hkv, dtype, kfmt):
    """The last tier's values as Q_4bit stored channel-major per 32 tokens (whole groups only): every nibble position
    of a group, both sides of the 32-token group, tile, chunk and block boundaries inside the tier."""
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=256, block_tokens=64, ring_blocks=5),
             dict(k_fmt=kfmt, v_fmt="i4c", capacity=10**9, block_tokens=128, ring_blocks=24)]
    p = Pair(2, Hq, Hkv, tiers, dtype)
    try:
        run_planted(p, 2, Hq, Hkv, dtype, [255 + 32 * 25, 255 + 32 * 83], synth.SEED_BASE + 330 + Hq, chunks=(256, 256))
        assert p.gpu.stats()["mfma_launches"] > 0
    finally:
        p.close()


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2)])
def test_dominant_key_with_keys_grouped_over_tokens(Hq, Hkv):
    """The last tier's keys as int4 per channel over 128 tokens: whole groups only, so its ends are block-aligned;
    the tile and chunk boundaries inside it and the fp window's ragged ends are what is planted."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=256, block_tokens=128, ring_blocks=3),
             dict(k_fmt="i4t", v_fmt="i4", capacity=10**9, block_tokens=128, ring_blocks=30)]
    p = Pair(2, Hq, Hkv, tiers, "f16")
    try:
        run_planted(p, 2, Hq, Hkv, "f16", [255 + 128 * 7, 255 + 128 * 21], synth.SEED_BASE + 320 + Hq, chunks=(256, 256))
    finally:
        p.close()


@pytest.mark.parametrize("n_slots", [0, 2])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2)])
def test_dominant_key_in_a_host_tier(Hq, Hkv, n_slots):
    """Three tiers, the oldest in pinned host memory, read in place (2048-token items) and through staging slots
    (256-token items): ragged host lengths, planted keys at the ends of its items and of its partly filled block."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=256, block_tokens=64, ring_blocks=6),
             dict(k_fmt="i8", v_fmt="i8", capacity=512, block_tokens=128, ring_blocks=8),
             dict(k_fmt="i4", v_fmt="i4", capacity=10**9, block_tokens=256, ring_blocks=16, mem="host")]
    p = Pair(2, Hq, Hkv, tiers, "f16", n_slots=n_slots)
    try:
        run_planted(p, 2, Hq, Hkv, "f16", [255 + 512 + 2085, 255 + 512 + 3331], synth.SEED_BASE + 340 + Hq + n_slots,
                    chunks=(256, 256, 256 if n_slots else 2048))
    finally:
        p.close()


@pytest.mark.parametrize("mem", ["host", "device"])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2)])
def test_dominant_key_in_the_partly_filled_newest_selected_block(Hq, Hkv, mem):
    """Block identification with the ids left on the device: the attention kernels look up each selected block and
    take the live token count of the newest one from the launch arguments (a host tier block by block, a tier in HBM
    as one run over all selected blocks).  Every block is selected (k above their number); the planted keys include
    the last live token of that block."""
    tiers = [dict(k_fmt="bf16", v_fmt="bf16", capacity=256, block_tokens=64, ring_blocks=6),
             dict(k_fmt="i8", v_fmt="i8", capacity=512, block_tokens=128, ring_blocks=8),
             dict(k_fmt="i4", v_fmt="i4", capacity=10**9, block_tokens=128, ring_blocks=40, mem=mem, summary=True)]
    p = Pair(2, Hq, Hkv, tiers, "bf16")
    try:
        # steps with append and eviction (the device-side selection is part of the step call); the host tier only
        # grows at its tail by whole 128-token blocks every 128 steps, so 20 steps leave the planted positions alone
        g = synth.rng(synth.SEED_BASE + 360 + Hq)
        lens = [255 + 512 + 1100, 255 + 512 + 3001]
        ks, vs, u = [], [], directions(g, 4, Hkv, "bf16")
        pos = []
        for b in range(2):
            k, v = synth.kv((synth.SEED_BASE + 360) * 31 + b, Hkv, lens[b], "bf16")
            n_host = lens[b] - 255 - 512
            pos.append([n_host - 1, n_host - 2, n_host // 128 * 128, n_host // 128 * 128 - 1])
            for j, t in enumerate(pos[b]):
                k[:, t] = synth.round_to(ALPHA * u[j], "bf16")
                v[:, t] = synth.round_to(2.0 * g.standard_normal((Hkv, 128), dtype=np.float32), "bf16")
            p.load(b, k, v)
            ks.append(k), vs.append(v)
        G = Hq // Hkv
        for j in range(4):
            q = queries_along(g, u[j], 2, Hq, Hkv, "bf16")
            kn, vn = synth.normal(g, (2, Hkv, 128), "bf16"), synth.normal(g, (2, Hkv, 128), "bf16")
            r = p.step(q, kn, vn, select_k=1000)
            assert_close(r[0], r[2], f"out direction {j}")
            assert_close(r[1], r[3], f"lse direction {j}")
            for b in range(2):
                assert np.array_equal(r[4][b], r[5][b])
                s = p.ora.seq[2][b]
                want = np.repeat(s.vhat[:, pos[b][j]], G, axis=0)        # host tier ordinals = sequence positions here
                assert np.max(np.abs(r[2][b] - want)) < 1e-5
                assert np.max(np.abs(r[0][b] - want)) < 2e-3 * max(1.0, np.max(np.abs(want))), (b, j)
    finally:
        p.close()
