"""Host side of the library without a GPU: the C ABI loads and exports every
symbol the header declares, argument validation returns the documented error
codes, and the tile table cuts sequences exactly as the scan needs."""
import os
import re

import numpy as np
import pytest

import paper_2411_19379_amd as ssm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    lib = ssm.load_library()
    header = open(os.path.join(ROOT, "include", "ssm_prefill.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(ssm_[a-z0-9_]+)\s*\(", header))
    assert names == {"ssm_plan_create", "ssm_plan_info", "ssm_plan_tile", "ssm_plan_launch_order", "ssm_plan_launch_item",
                     "ssm_plan_stretch",
                     "ssm_plan_workspace_bytes",
                     "ssm_prefill", "ssm_prefill_noalloc", "ssm_state_advance", "ssm_conv1d_prefill",
                     "ssm_profile_mark", "ssm_plan_destroy", "ssm_last_error"}
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"


def tiles_of(plan):
    return plan.tiles()  # (tok0, len, seq, ckpt_slot)


def check_cover(plan, cu, ckpt_pos, tile_tokens):
    """Tiles are sequence-local, in order, no longer than the tile size, cover
    every token once, and a tile ends at every checkpoint with the right slot."""
    tiles = tiles_of(plan)
    slot = 0
    ti = 0
    for s in range(len(cu) - 1):
        pos = int(cu[s])
        ends = {int(cu[s]) + p: None for p in ckpt_pos[s]}
        for p in ckpt_pos[s]:
            ends[int(cu[s]) + p] = slot
            slot += 1
        while pos < cu[s + 1]:
            tok0, ln, seq, cs = tiles[ti]
            assert tok0 == pos and seq == s and 1 <= ln <= tile_tokens
            inside = [e for e in ends if pos < e < pos + ln]
            assert not inside, "a checkpoint falls strictly inside a tile"
            pos += ln
            assert cs == (ends[pos] if pos in ends else -1)
            ti += 1
    assert ti == len(tiles) and slot == plan.info.n_ckpt


def test_paper_position_example_tiles():
    """100 tokens, chunk 32, states wanted at 64 (chunk boundary), 80 and 100:
    a tile ends exactly at each of them (Section 4.1)."""
    with open(os.path.join(GOLDEN, "position_example.txt")) as f:
        total, chunk, want, boundary, rest = (int(v) for v in
                                              [ln for ln in f if ln.strip() and not ln.startswith("#")][0].split())
    plan = ssm.Plan(4, 16, 16, 1, chunk, "f32", [0, total], [[boundary, want, total]])
    check_cover(plan, [0, total], [[boundary, want, total]], plan.info.tile_tokens)
    ends = [t[0] + t[1] for t in tiles_of(plan) if t[3] >= 0]
    assert ends == [boundary, want, total]
    # the second pass of a two-pass prefill is a plan over the remaining tokens
    plan2 = ssm.Plan(4, 16, 16, 1, chunk, "f32", [0, rest], [[rest]])
    assert sum(t[1] for t in tiles_of(plan2)) == rest


@pytest.mark.parametrize("io,shape,path,tile", [("f32", (4, 16, 16, 1), ssm.SSM_PATH_VALU_F32, 16),
                                                ("bf16", (128, 64, 128, 8), ssm.SSM_PATH_MFMA_BF16, 64),
                                                ("bf16", (6, 24, 40, 3), ssm.SSM_PATH_VALU_F32, 16)])
def test_random_batches_are_covered(io, shape, path, tile):
    rs = np.random.RandomState(7)
    H, P, N, G = shape
    for trial in range(20):
        nb = int(rs.randint(1, 9))
        lens = [int(v) for v in rs.randint(0, 400, size=nb)]
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        ck = [sorted(set(int(v) for v in rs.randint(1, L + 1, size=rs.randint(0, 4)))) if L else [] for L in lens]
        plan = ssm.Plan(H, P, N, G, 256, io, cu, ck)
        assert plan.info.path == path and plan.info.tile_tokens == tile
        assert plan.info.total_tokens == cu[-1] and plan.info.batch == nb
        check_cover(plan, cu, ck, tile)
        # the matrix-core scan keeps, per tile, one operand image per group and one transposed dt row per head
        want_ws = plan.info.n_tiles * (G * 38912 + H * 128) if path == ssm.SSM_PATH_MFMA_BF16 else 0
        assert ssm.ssm_plan_workspace_bytes(plan.handle) == (want_ws + 255) // 256 * 256
        split = 1
        if path == ssm.SSM_PATH_MFMA_BF16:
            # 32 channels of a head per workgroup, or 64 where that would take more than the 256 workgroups of a round
            busy = sum(1 for L in lens if L > 0)
            split = P // 64 if P % 64 == 0 and 2 * busy * H * (P // 64) > 256 else P // 32
        assert plan.info.n_workgroups == nb * H * split
        plan.close()


def test_chunk_bounds_the_tile():
    p16 = ssm.Plan(4, 64, 128, 2, 16, "bf16", [0, 100], None)
    assert p16.info.tile_tokens == 16 and p16.info.n_tiles == 7
    p256 = ssm.Plan(4, 64, 128, 2, 256, "bf16", [0, 100], None)
    assert p256.info.tile_tokens == 64 and p256.info.n_tiles == 2


@pytest.mark.parametrize("kwargs,status", [
    (dict(cu=[1, 5]), "SSM_ERR_BAD_CU_SEQLENS"),
    (dict(cu=[0, 5, 3]), "SSM_ERR_BAD_CU_SEQLENS"),
    (dict(ck=[[0]]), "SSM_ERR_BAD_CHECKPOINT"),
    (dict(ck=[[11]]), "SSM_ERR_BAD_CHECKPOINT"),
    (dict(ck=[[4, 4]]), "SSM_ERR_BAD_CHECKPOINT"),
    (dict(ck=[[7, 3]]), "SSM_ERR_BAD_CHECKPOINT"),
    (dict(shape=(4, 16, 16, 3)), "SSM_ERR_INVALID_ARG"),
    (dict(shape=(0, 16, 16, 1)), "SSM_ERR_INVALID_ARG"),
    (dict(chunk=8), "SSM_ERR_UNSUPPORTED_SHAPE"),
    (dict(chunk=100), "SSM_ERR_UNSUPPORTED_SHAPE"),
    (dict(shape=(4, 6, 16, 1)), "SSM_ERR_UNSUPPORTED_SHAPE"),       # 24-byte rows of x
    (dict(shape=(2, 128, 256, 1)), "SSM_ERR_UNSUPPORTED_SHAPE"),    # fp32 state too large for the VALU kernel
])
def test_rejected_arguments(kwargs, status):
    shape = kwargs.get("shape", (4, 16, 16, 1))
    cu = kwargs.get("cu", [0, 10])
    ck = kwargs.get("ck", None)
    if ck is not None and len(ck) != len(cu) - 1:
        ck = ck + [[]] * (len(cu) - 1 - len(ck))
    with pytest.raises(ssm.SsmError) as e:
        ssm.Plan(*shape, kwargs.get("chunk", 64), "f32", cu, ck)
    assert e.value.status == status
    assert ssm.ssm_last_error() != ""


def test_null_arguments_and_destroy():
    lib = ssm.load_library()
    assert lib.ssm_plan_create(None, 1, None, None, None, None) == -1
    lib.ssm_plan_destroy(None)  # accepted
    plan = ssm.Plan(4, 16, 16, 1, 64, "f32", [0, 0, 0], [[], []])
    assert plan.info.n_tiles == 0 and plan.info.total_tokens == 0
    with pytest.raises(ssm.SsmError):
        ssm.ssm_plan_tile(plan.handle, 0)
    plan.close()
    plan.close()  # idempotent


def test_launch_order_covers_every_item_once_and_balances_the_dies():
    """The matrix-core scan's work items (rank by length, head, slice): empty sequences get none, every item belongs
    to exactly one workgroup of the launch, each die (workgroups b with the same b % 8) meets its items in order of
    decreasing sequence length, and a greedy schedule of each die's queue on its 32 compute units ends close to the
    ideal (total work / 256) whenever there are enough items to go round."""
    import heapq

    rng = np.random.default_rng(11)
    for trial in range(40):
        batch = int(rng.integers(1, 40))
        lens = rng.integers(0, 9000, size=batch) * (rng.random(batch) > 0.15)
        if trial == 0:
            lens = np.asarray([32768])
        if trial == 1:
            lens = np.zeros(5, dtype=np.int64)
        if trial == 2:  # the 16 requests of the packed configuration
            lens = np.asarray([615, 7105, 5883, 1198, 4728, 3752, 1172, 5308, 3632, 3866, 5581, 2229, 1333, 4866, 552, 7494])
        batch = len(lens)
        H = 80 if trial == 2 else int(rng.choice([2, 16, 80, 128]))
        P = 64 if trial == 2 else int(rng.choice([32, 64, 128]))
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        plan = ssm.Plan(H, P, 128, 1 if H == 80 else 2, 64, "bf16", cu.tolist(), None)
        by_length, slices, n_items, n_blocks = plan.launch_order()
        stretches = plan.stretches()
        n_st = plan.info.n_stretches
        tiles = np.asarray([e - b for b, e, _ in stretches], dtype=np.int64)
        assert sorted(by_length) == list(range(n_st))
        ranked = tiles[by_length]
        assert all(ranked[i] >= ranked[i + 1] for i in range(n_st - 1))
        assert all(by_length[i] < by_length[i + 1] for i in range(n_st - 1) if ranked[i] == ranked[i + 1])
        per_seq = H * slices
        assert slices in (P // 32, P // 64) and plan.info.n_workgroups == n_st * per_seq
        assert n_items == int((tiles > 0).sum()) * per_seq
        assert n_blocks % 8 == 0 and n_items <= n_blocks < n_items + 256
        if n_items < 256:
            assert n_blocks < n_items + 8
        items = [ssm.ssm_plan_launch_item(plan.handle, b) for b in range(n_blocks)]
        assert sorted(i for i in items if i >= 0) == list(range(n_items))
        with pytest.raises(ssm.SsmError):
            ssm.ssm_plan_launch_item(plan.handle, n_blocks)
        weight = np.repeat(ranked, per_seq)
        ends = []
        for die in range(8):
            queue = [weight[i] for i in items[die::8] if i >= 0]
            assert all(a >= b for a, b in zip(queue, queue[1:]))
            cus = [0] * 32
            for wq in queue:
                heapq.heappush(cus, heapq.heappop(cus) + int(wq))
            ends.append(max(cus))
        if n_items >= 1024:
            assert max(ends) <= 1.12 * weight[:n_items].sum() / 256 + weight.max() * 0.25, (ends, lens)
        plan.close()


def test_long_sequences_of_small_batches_are_cut_into_stretches():
    """A batch with at most 128 (sequence, head, 64-channel slice) streams: its long sequences are cut into
    stretches of at least 64 tiles (sequences of at least 160 tiles), as many as fit one round of 256 workgroups, the stretches of a sequence partition
    its tiles in order, only
    the first does not start from zero, and the workspace has room for one fp32 state per later stretch and one fp32
    per (tile, head).  Batches that fill the GPU, short sequences and the fp32 path are left alone."""
    def plan_of(lens, H=128, P=64, io="bf16", ckpt=None):
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        return ssm.Plan(H, P, 128, 8 if H % 8 == 0 else 1, 64, io, cu.tolist(), ckpt)

    def check_partition(plan, lens):
        per_seq = {}
        for (_, _, seq, _) in plan.tiles():
            per_seq[seq] = per_seq.get(seq, 0) + 1
        st = plan.stretches()
        pos, later = 0, 0
        for i, n in enumerate((per_seq.get(i, 0) for i in range(len(lens)))):
            mine = []
            while pos < len(st) and (not mine or st[pos][2]):
                if mine or not st[pos][2]:
                    mine.append(st[pos])
                    pos += 1
            assert not mine[0][2] and all(z for _, _, z in mine[1:])
            assert all(a[1] == b[0] for a, b in zip(mine, mine[1:]))
            assert mine[-1][1] - mine[0][0] == n
            later += len(mine) - 1
        assert pos == len(st)
        return later

    p = plan_of([32768])  # 128 streams: two stretches of 256 tiles
    assert p.info.n_stretches == 2 and p.stretches() == [(0, 256, False), (256, 512, True)]
    assert check_partition(p, [32768]) == 1
    assert p.info.n_workgroups == 2 * 128
    base = 512 * (8 * 38912 + 128 * 128)
    assert ssm.ssm_plan_workspace_bytes(p.handle) == base + 512 * 128 * 4 + 128 * 64 * 128 * 4
    p.close()
    p = plan_of([32768], H=32)  # 32 streams: 8 stretches of 64 tiles
    assert p.info.n_stretches == 8 and check_partition(p, [32768]) == 7
    p.close()
    p = plan_of([32768], H=16)  # 16 streams: 8 stretches are the most, 128 streams in all: 32 channels per workgroup
    assert p.info.n_stretches == 8 and p.info.n_workgroups == 8 * 16 * 2
    p.close()
    p = plan_of([2048], H=80)   # too short to cut
    assert p.info.n_stretches == 1 and p.info.n_workgroups == 160
    p.close()
    p = plan_of([20000, 300, 0, 9000 + 1300], H=40)  # 120 streams: two stretches where long enough; 200 streams, 64 channels
    assert [e - b for b, e, _ in p.stretches()] == [156, 157, 5, 0, 80, 81]
    assert check_partition(p, [20000, 300, 0, 10300]) == 2 and p.info.n_workgroups == 6 * 40
    p.close()
    p = plan_of([10240 - 64, 10240], H=40)  # 159 and 160 tiles: only the second is long enough to be cut
    assert [e - b for b, e, _ in p.stretches()] == [159, 80, 80]
    p.close()
    p = plan_of([20000, 20000], H=80)  # 160 streams: a second round either way with 32 channels; 64 channels, uncut
    assert p.info.n_stretches == 2 and p.info.n_workgroups == 160
    p.close()
    p = plan_of([16384, 16384])  # 256 streams: nothing to cut
    assert p.info.n_stretches == 2 and not any(z for _, _, z in p.stretches())
    p.close()
    p = plan_of([32768], H=8, io="f32")
    assert p.info.n_stretches == 1
    p.close()


def test_stretch_queries_reject_bad_indices_and_cover_the_fp32_path():
    p = ssm.Plan(4, 16, 16, 1, 64, "f32", [0, 100, 100, 300], None)  # vector-ALU path: one stretch per sequence
    assert p.info.n_stretches == 3
    tiles = p.tiles()
    st = p.stretches()
    assert [z for _, _, z in st] == [False, False, False]
    for i, (b, e, _) in enumerate(st):
        assert all(t[2] == i for t in tiles[b:e]) and e - b == sum(1 for t in tiles if t[2] == i)
    for bad in (-1, 3):
        with pytest.raises(ssm.SsmError) as err:
            ssm.ssm_plan_stretch(p.handle, bad)
        assert err.value.status == "SSM_ERR_INVALID_ARG"
    p.close()
    q = ssm.Plan(128, 64, 128, 8, 256, "bf16", [0, 32768], None)
    with pytest.raises(ssm.SsmError):
        ssm.ssm_plan_stretch(q.handle, 2)
    q.close()
