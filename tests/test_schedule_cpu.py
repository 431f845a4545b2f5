"""The host planner against the block mask: the work items of a call cover exactly the visible
(query token, key token) pairs of the Block-attention mask (Section 2.1, 2.4, 2.5), none twice, and no
item walks a key tile in which none of its rows sees anything.  Host only: the items come from the
code the calls themselves plan with, and the key-range arithmetic of a split is the kernel's."""
import numpy as np
import pytest

import oracle
from paper_2409_15355_amd import binding as ba


@pytest.fixture(scope="module", autouse=True)
def lib():
    import os
    if not os.path.exists(ba.LIB_PATH):
        from paper_2409_15355_amd import build
        build.build()
    return ba.load()


def coverage_of(items, G, problem_rows):
    """count[problem][token, key] over the items; keys = (context keys..., own tokens...).
    problem_rows: {problem: (n_ctx_keys, n_tokens)}.  Also checks the per-item invariants.
    Items that name their KV head (splits sized by XCD speed) are checked head by head: every head's
    items must give the same, complete coverage."""
    heads_named = sorted({w.kv_head for w in items})
    if heads_named and heads_named != [-1]:
        assert -1 not in heads_named
        covs = [_coverage_of([w for w in items if w.kv_head == h], G, problem_rows) for h in heads_named]
        for c in covs[1:]:
            assert all(np.array_equal(c[p], covs[0][p]) for p in c)
        return covs[0]
    return _coverage_of(items, G, problem_rows)


def _coverage_of(items, G, problem_rows):
    cov = {p: np.zeros((lq, tc + lq), dtype=np.int32) for p, (tc, lq) in problem_rows.items()}
    seen_rows = {p: np.zeros(lq * G, dtype=np.int32) for p, (tc, lq) in problem_rows.items()}
    for w in items:
        tc, lq = problem_rows[w.problem]
        assert 0 <= w.row_begin < w.row_end <= lq * G and w.row_end - w.row_begin <= w.tile_rows
        assert w.row_begin % w.tile_rows == 0
        assert 0 <= w.ctx_begin <= w.ctx_end <= tc and 0 <= w.self_begin <= w.self_end <= lq
        # whole key tiles, cut at the end of a segment
        assert w.ctx_begin % w.tile_keys == 0 or w.ctx_begin == tc
        assert w.self_begin % w.tile_keys == 0 or w.self_begin == lq
        toks = np.arange(w.row_begin, w.row_end) // G
        last_tok = int(toks[-1])
        # no fully masked tile: every tile of the causal range starts at or before the last row's token
        if w.self_end > w.self_begin:
            last_tile_key0 = (w.self_end - 1) // w.tile_keys * w.tile_keys
            assert last_tile_key0 <= last_tok, (w.problem, w.row_begin, w.self_begin, w.self_end)
        if w.split == 0:
            seen_rows[w.problem][w.row_begin:w.row_end] += 1
        for t in np.unique(toks):
            heads_here = int((toks == t).sum())  # every head of the group is a row: count a pair once per row
            cov[w.problem][t, w.ctx_begin:w.ctx_end] += heads_here
            hi = min(w.self_end, t + 1)
            if hi > w.self_begin:
                cov[w.problem][t, tc + w.self_begin:tc + hi] += heads_here
    for p, rows in seen_rows.items():
        assert (rows == 1).all(), f"problem {p}: rows not covered exactly once per split"
    return cov


def expected_final(tc, lq, G):
    """The mask of Section 2.5 for one prompt, from the oracle's block mask: context = one block
    per... any earlier blocks (all of them visible to the last block), then the final block."""
    m = oracle.block_mask([0, tc, tc + lq]) if tc else oracle.block_mask([0, lq])
    return m[tc:, :].astype(np.int32) * G


@pytest.mark.parametrize("hq,hkv", [(32, 8), (4, 4), (8, 1)])
@pytest.mark.parametrize("n_cu", [256, 8, 1])
def test_final_block_items_cover_the_mask_exactly(hq, hkv, n_cu):
    rng = np.random.default_rng(7 + hq + n_cu)
    h = ba.Heads(hq, hkv, 128, 500000.0)
    G = hq // hkv
    for case in range(12):
        n_prompts = int(rng.integers(1, 5))
        lqs = [int(rng.choice([1, 17, 64, 65, 130, 256])) for _ in range(n_prompts)]
        tcs = [int(rng.choice([0, 1, 63, 64, 700, 3001, 9000])) for _ in range(n_prompts)]
        cu_q, cu_ctx = np.concatenate([[0], np.cumsum(lqs)]), np.concatenate([[0], np.cumsum(tcs)])
        items = ba.ba_schedule_final_block(h, cu_q, cu_ctx, n_cu)
        assert len({w.n_splits for w in items}) == 1
        cov = coverage_of(items, G, {p: (tcs[p], lqs[p]) for p in range(n_prompts)})
        for p in range(n_prompts):
            assert np.array_equal(cov[p], expected_final(tcs[p], lqs[p], G)), (case, p, lqs, tcs)
        assert all(w.first_token == cu_q[w.problem] for w in items)


def test_config5_schedule_is_the_one_the_design_states():
    h = ba.Heads(32, 8, 128, 500000.0)
    items = ba.ba_schedule_final_block(h, [0, 256], [0, 31744], 256)
    assert len(items) == 8 * 4 and {w.n_splits for w in items} == {8}   # x 8 KV heads = 256 workgroups
    tiles = lambda w: (w.ctx_end - w.ctx_begin + w.self_end - w.self_begin) // 64
    per_split = sorted({(w.split, tiles(w)) for w in items if w.row_begin == 0})
    # equal shares, except that the split with the causal tiles gets fewer
    assert [t for _, t in per_split][:-1] == [62] * 6 + [63] or max(t for _, t in per_split) - min(t for _, t in per_split) <= 4
    assert per_split[-1][1] < per_split[0][1]


@pytest.mark.parametrize("hq,hkv", [(32, 8), (4, 4), (2, 1)])
def test_encode_items_cover_the_block_diagonal_mask_exactly(hq, hkv):
    rng = np.random.default_rng(11 + hq)
    h = ba.Heads(hq, hkv, 64, 10000.0)
    G = hq // hkv
    for case in range(8):
        lens = [int(x) for x in rng.choice([0, 1, 31, 32, 33, 100, 257, 300], size=int(rng.integers(1, 9)))]
        if case == 0:
            lens = [7000, 5, 0, 6144, 6145]   # both schedules in one call (the long-block core beyond 6144 tokens)
        offs = np.concatenate([[0], np.cumsum(lens)])
        items = ba.ba_schedule_encode_blocks(h, offs)
        live = {b: (0, lens[b]) for b in range(len(lens)) if lens[b] > 0}
        assert {w.problem for w in items} == set(live)
        cov = coverage_of(items, G, live)
        mask = oracle.block_mask(np.concatenate([offs, [offs[-1]]]))  # (a trailing empty block: no block is "last")
        for b, (_, L) in live.items():
            want = mask[offs[b]:offs[b] + L, offs[b]:offs[b] + L].astype(np.int32) * G
            assert np.array_equal(cov[b], want), (case, b, lens)
            assert not mask[offs[b]:offs[b] + L, :offs[b]].any()
        if case == 0 and G >= 4:
            assert {w.tile_rows for w in items if w.problem in (0, 4)} == {256}
            assert {w.tile_rows for w in items if w.problem in (1, 3)} == {128}


@pytest.mark.parametrize("hq,hkv", [(32, 8), (8, 2)])
def test_whole_prompt_items_cover_the_mask_of_section_2_4_exactly(hq, hkv):
    rng = np.random.default_rng(13 + hq)
    h = ba.Heads(hq, hkv, 128, 500000.0)
    G = hq // hkv
    for case in range(8):
        n_prompts = int(rng.integers(1, 4))
        cu_blk, lens = [0], []
        for _ in range(n_prompts):
            nb = int(rng.integers(1, 6))
            lens += [int(x) for x in rng.choice([0, 1, 31, 33, 100, 257], size=nb - 1)] + [int(rng.choice([1, 32, 70]))]
            cu_blk.append(len(lens))
        offs = np.concatenate([[0], np.cumsum(lens)])
        items = ba.ba_schedule_prompts(h, cu_blk, offs)
        T = int(offs[-1])
        count = np.zeros((T, T), dtype=np.int32)
        rows_seen = np.zeros(T * G, dtype=np.int32)
        for w in items:
            p0 = int(offs[cu_blk[w.problem]])          # first token of the prompt
            blk_len = None
            b = int(np.searchsorted(offs, w.first_token, side="right") - 1)
            while lens[b] == 0:
                b += 1
            assert offs[b] == w.first_token
            blk_len = lens[b]
            is_last = b == cu_blk[w.problem + 1] - 1
            dq = w.first_token - p0 if is_last else 0
            assert w.ctx_begin == 0 and w.ctx_end <= dq
            toks = np.arange(w.row_begin, w.row_end) // G
            assert toks[-1] < blk_len
            rows_seen[w.first_token * G + w.row_begin:w.first_token * G + w.row_end] += 1
            for t in np.unique(toks):
                nh = int((toks == t).sum())
                count[w.first_token + t, p0:p0 + w.ctx_end] += nh
                hi = min(w.self_end, t + 1)
                count[w.first_token + t, w.first_token:w.first_token + hi] += nh
            # the walk reaches the last row's own token, and its last key tile is not fully masked
            walked = w.ctx_end + w.self_end
            assert walked >= min(dq + toks[-1] + 1, dq + blk_len) and (walked - 1) // 32 * 32 <= dq + toks[-1]
        assert (rows_seen == 1).all()
        want = np.zeros((T, T), dtype=np.int32)
        for n in range(n_prompts):
            o = offs[cu_blk[n]:cu_blk[n + 1] + 1]
            m = oracle.block_mask(o - o[0])
            want[o[0]:o[-1], o[0]:o[-1]] = m.astype(np.int32) * G
        assert np.array_equal(count, want), (case, lens, cu_blk)


def test_split_range_arithmetic_partitions_every_walk():
    """split_tile_range through the final-block query: over every split count the planner can
    choose (1 .. 32, by varying the compute-unit count), the splits of a row tile partition its walk."""
    h = ba.Heads(8, 8, 64, 10000.0)
    seen_splits = set()
    for n_cu in (1, 2, 3, 5, 8, 13, 16, 24, 32, 64, 100, 256, 1000):
        for tc in (0, 5, 64, 1000, 4097, 20000):
            for lq in (1, 64, 200):
                items = ba.ba_schedule_final_block(h, [0, lq], [0, tc], n_cu)
                seen_splits.add(items[0].n_splits)
                by_tile = {}
                for w in items:
                    by_tile.setdefault(w.row_begin, []).append(w)
                for ws in by_tile.values():
                    ws.sort(key=lambda w: w.split)
                    assert [w.split for w in ws] == list(range(ws[0].n_splits))
                    at_ctx, at_self = 0, 0
                    for w in ws:   # contiguous, in order, nothing skipped
                        if w.ctx_end > w.ctx_begin:
                            assert w.ctx_begin == at_ctx
                            at_ctx = w.ctx_end
                        if w.self_end > w.self_begin:
                            assert w.self_begin == at_self and at_ctx == tc
                            at_self = w.self_end
                    assert at_ctx == tc and at_self == min(lq, ((ws[0].row_end - 1) // 64 + 1) * 64)  # (one head per group: row = token)
    assert len(seen_splits) >= 6 and max(seen_splits) >= 16


@pytest.mark.parametrize("speeds", [[1.0] * 8, [0.92, 1.0, 1.08, 1.0, 0.95, 1.05, 1.0, 1.0], [0.5, 2.0, 0.5, 2.0, 1.0, 1.0, 1.0, 1.0]])
def test_splits_sized_by_xcd_speed_still_cover_the_mask_exactly(speeds):
    """ba_heads.xcd_speed moves the boundaries between KV splits (faster XCDs get more key tiles); the
    work items must still cover every visible pair exactly once."""
    rng = np.random.default_rng(5)
    h = ba.Heads(32, 8, 128, 500000.0, xcd_speed=speeds)
    for case in range(6):
        n_prompts = int(rng.integers(1, 4))
        lqs = [int(rng.choice([1, 64, 130, 256])) for _ in range(n_prompts)]
        tcs = [int(rng.choice([0, 700, 3001, 9000, 31744])) for _ in range(n_prompts)]
        if case == 0:
            n_prompts, lqs, tcs = 1, [256], [31744]
        cu_q, cu_ctx = np.concatenate([[0], np.cumsum(lqs)]), np.concatenate([[0], np.cumsum(tcs)])
        items = ba.ba_schedule_final_block(h, cu_q, cu_ctx, 256)
        cov = coverage_of(items, 4, {p: (tcs[p], lqs[p]) for p in range(n_prompts)})
        for p in range(n_prompts):
            assert np.array_equal(cov[p], expected_final(tcs[p], lqs[p], 4)), (case, p, lqs, tcs)
        if case == 0:
            # config 5: 256 workgroups; a split's share of its KV head's key tiles follows the speed of the XCD
            # that runs it (which XCDs a KV head's splits lie on is the planner's choice)
            assert sorted({w.kv_head for w in items}) == list(range(8))
            for kvh in range(8):
                mine = [w for w in items if w.kv_head == kvh and w.row_begin == 0]
                assert [w.split for w in sorted(mine, key=lambda w: w.split)] == list(range(8))
                if len(set(speeds)) == 1:
                    assert {w.xcd for w in mine} == {kvh}   # nothing to balance: an XCD fetches one KV head's query rows
                else:
                    assert len({w.xcd for w in mine}) >= 2  # a KV head's splits lie on XCDs that can be balanced against each other
                tiles = {w.split: (w.ctx_end - w.ctx_begin + w.self_end - w.self_begin) // 64 for w in mine}
                sp = {w.split: speeds[w.xcd] for w in mine}
                if len(set(speeds)) == 1:
                    assert max(tiles[s] for s in range(7)) - min(tiles[s] for s in range(7)) <= 1
                else:
                    share = np.array([tiles[s] / sp[s] for s in range(7)])
                    assert share.max() / share.min() < 1.06   # equal time per split, to a tile
                    if sp[0] != sp[4]:
                        assert (tiles[0] < tiles[4]) == (sp[0] < sp[4])
            # every row tile of a (KV head, split) runs on the same XCD: they share its K/V tiles
            for kvh in range(8):
                for s_ in range(8):
                    assert len({w.xcd for w in items if w.kv_head == kvh and w.split == s_}) == 1


@pytest.mark.parametrize("speeds", [[1.0608, 0.9721, 1.0293, 0.9882, 1.0236, 0.9837, 1.0255, 0.9167],
                                    [1.0393, 0.9966, 0.9955, 0.9547, 1.0547, 0.9905, 1.0048, 0.9638],
                                    [0.93, 0.94, 0.95, 0.96, 1.04, 1.05, 1.06, 1.07]])
def test_xcds_are_dealt_to_kv_head_groups_by_speed(speeds):
    """With measured speeds the planner also chooses which XCD runs which stretch of the work items: XCDs
    that share KV heads can be balanced against each other, so slow ones are put with fast ones.  Every
    XCD still runs an eighth of the launch, and the launch is expected to end within 3 % of the time a
    perfect balance would give (speeds as measured on two devices, and a set sorted the worst way)."""
    h = ba.Heads(32, 8, 128, 500000.0, xcd_speed=speeds)
    items = ba.ba_schedule_final_block(h, [0, 256], [0, 31744], 256)
    assert len(items) == 256
    tiles = lambda w: -(-(w.ctx_end - w.ctx_begin) // 64) - (-(w.self_end - w.self_begin) // 64)
    per_xcd = {x: [w for w in items if w.xcd == x] for x in range(8)}
    assert all(len(v) == 32 for v in per_xcd.values())
    ends = [max(tiles(w) for w in per_xcd[x]) / speeds[x] for x in range(8)]
    ideal = sum(tiles(w) for w in items) / 32.0 / sum(speeds)
    assert max(ends) <= 1.03 * ideal, (ends, ideal)
    hosted = {x: frozenset(w.kv_head for w in per_xcd[x]) for x in range(8)}
    if 1 < len(hosted[0]) < 8:
        # groups of XCDs share KV heads; the slowest XCD sits in a group with the fastest
        assert hosted[int(np.argmin(speeds))] == hosted[int(np.argmax(speeds))]
        groups = {}
        for x in range(8):
            groups.setdefault(hosted[x], []).append(speeds[x])
        means = [np.mean(v) for v in groups.values()]
        assert max(means) - min(means) < 0.02, groups


def test_every_xcd_runs_its_share_whatever_the_speeds():
    """Drawn speeds and shapes: the work items of a launch are dealt to the XCDs in equal numbers (to
    within one), each (KV head, split, row tile) exactly once, whichever XCD runs which stretch."""
    rng = np.random.default_rng(77)
    for case in range(40):
        hkv = int(rng.choice([1, 2, 4, 8]))
        g = int(rng.choice([1, 4, 8]))
        speeds = [float(x) for x in rng.uniform(0.8, 1.25, 8)]
        h = ba.Heads(hkv * g, hkv, 128, 500000.0, xcd_speed=speeds)
        lq, tc = int(rng.choice([1, 50, 64, 256, 700])), int(rng.choice([0, 900, 8000, 31744, 100000]))
        items = ba.ba_schedule_final_block(h, [0, lq], [0, tc], 256)
        if not items or items[0].xcd < 0:
            continue  # equal splits (one split, or nothing to size): no XCDs in the answer
        seen = {(w.kv_head, w.split, w.row_begin) for w in items}
        assert len(seen) == len(items), (case, hkv, g, lq, tc)
        counts = np.bincount([w.xcd for w in items], minlength=8)
        assert counts.max() - counts.min() <= 1, (case, counts)


def test_bad_xcd_speeds_are_rejected():
    h = ba.Heads(32, 8, 128, 500000.0, xcd_speed=[1, 1, 1, 0.1, 1, 1, 1, 1])
    with pytest.raises(ba.BaError):
        ba.ba_schedule_final_block(h, [0, 256], [0, 31744], 256)
    h = ba.Heads(32, 8, 128, 500000.0, xcd_speed=[1, 1, 1, float("nan"), 1, 1, 1, 1])
    with pytest.raises(ba.BaError):
        ba.ba_schedule_final_block(h, [0, 256], [0, 31744], 256)
    with pytest.raises(ValueError):
        ba.Heads(32, 8, 128, xcd_speed=[1.0] * 7)
