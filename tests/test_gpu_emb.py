"""GPU parity: hctr_emb_forward / hctr_emb_backward_sgd (direct-index mode) against the oracle,
element by element, on seeded synthetic inputs."""
import numpy as np
import pytest
import torch

import datagen
import oracle
from parity import assert_close, check_table_update, oracle_backward, oracle_forward, to_dev

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED


def H():
    import paper_2210_08803_amd as h
    return h


def run_case(table_rows, dim, batch, *, dtype=torch.float32, combiner=0, alpha=1.05, hot=None, seed=SEED,
             lr=0.01, share_table=False, poison=0, slot_base=None):
    """One forward + backward comparison.  hot = None (one-hot), (lo, hi) hotness range, or an array
    with the number of keys of every bag."""
    h = H()
    S = len(table_rows)
    if share_table:
        base = np.zeros(S, dtype=np.int64)
        total = int(table_rows[0])
    else:
        ro = datagen.row_offsets(table_rows)
        base, total = ro[:-1].copy(), int(ro[-1])
    num = np.asarray(table_rows, dtype=np.int64)
    table = datagen.table_rows_at(seed, torch.arange(total), dim, dtype)
    n_bags = batch * S
    if hot is None:
        offsets = None
        keys = datagen.onehot_keys(seed, 0, table_rows, batch, alpha)
    else:
        if isinstance(hot, np.ndarray):
            offsets = torch.zeros(n_bags + 1, dtype=torch.int64)
            offsets[1:] = torch.from_numpy(np.cumsum(hot.astype(np.int64)))
        else:
            offsets = datagen.multihot_offsets(seed, 0, n_bags, hot[0], hot[1])
        keys = datagen.multihot_keys(seed, 0, table_rows, batch, alpha, offsets)
    if poison:
        g = np.random.default_rng(seed)
        idx = g.integers(0, len(keys), poison)
        keys[idx] = torch.from_numpy(g.choice([-1, -2**62, 2**40, int(num.max())], poison))
    dY = datagen.normal_grads(seed, 0, n_bags * dim).view(n_bags, dim)

    tab_np, keys_np, dY_np = table.numpy(), keys.numpy(), dY.numpy()
    off_np = None if offsets is None else offsets.numpy()
    rows, bad = oracle.rows_direct(base, num, keys_np, off_np, n_bags=n_bags)
    ref_out, mag_out = oracle_forward(tab_np, rows, off_np, combiner, n_bags)
    ref_tab, mag_tab, uniq, cnt = oracle_backward(tab_np, rows, off_np, combiner, n_bags, dY_np, lr)

    d_table = to_dev(table)
    layer = h.EmbeddingLayer(d_table, S, combiner, base, num)
    d_keys, d_off, d_dY = to_dev(keys), (None if offsets is None else to_dev(offsets)), to_dev(dY)
    out = layer.forward(batch, d_keys, d_off)
    torch.cuda.synchronize()
    assert layer.invalid_keys() == bad
    out_np = out.cpu().numpy().reshape(n_bags, dim)
    if hot is None:
        assert np.array_equal(out_np.view(np.uint32), ref_out.view(np.uint32)), "one-hot forward must be bit-exact"
    assert_close(out_np, ref_out, mag_out, "forward")
    out2 = layer.forward(batch, d_keys, d_off)
    assert torch.equal(out, out2), "forward is not deterministic"

    assert layer.invalid_keys() == 2 * bad            # the counter is a running total
    layer.reset_invalid_keys()
    layer.backward_sgd(batch, d_keys, d_dY, lr, d_off)
    torch.cuda.synchronize()
    assert layer.invalid_keys() == bad
    g_rows, g_cnt = layer.dedup_result(batch, len(keys_np))
    assert np.array_equal(g_rows.cpu().numpy(), uniq), "unique rows differ"
    assert np.array_equal(g_cnt.cpu().numpy(), cnt), "occurrence counts differ"
    got = d_table.cpu().numpy()
    check_table_update(got, tab_np, ref_tab, mag_tab, uniq, "backward")

    d_table2 = to_dev(table)
    layer2 = h.EmbeddingLayer(d_table2, S, combiner, base, num)
    layer2.backward_sgd(batch, d_keys, d_dY, lr, d_off)
    torch.cuda.synchronize()
    assert torch.equal(d_table, d_table2), "backward is not deterministic"
    return dict(nnz=len(keys_np), unique=len(uniq), max_count=int(cnt.max()) if len(cnt) else 0)


def test_tiny_config():
    """10,000 x 16 fp32, batch 256, 4 one-hot slots on the one table, uniform keys, lr 0.01."""
    info = run_case([10000] * 4, 16, 256, alpha=0.0, share_table=True)
    assert info["nnz"] == 1024


def test_dlrm_shape_scaled_onehot():
    """26 tables at 1/1000 of the full row counts, dim 128 fp32, Zipf 1.05; 2,051 samples give a
    ragged last tile in every kernel and segments far longer than a reduction window."""
    rows = datagen.scaled_table_rows(1e-3)
    info = run_case(rows, 128, 2051)
    assert info["max_count"] > 128 and info["unique"] < info["nnz"]


def test_multihot_fp16_mean():
    """fp16 storage, fp32 accumulate, mean combiner, hotness 1..100 per bag, Zipf 1.1."""
    rows = datagen.scaled_table_rows(2e-4)
    run_case(rows, 128, 96, dtype=torch.float16, combiner=1, alpha=1.1, hot=(1, 100))


def test_multihot_with_empty_bags_sum_fp32():
    run_case([50, 3000, 7], 64, 300, combiner=0, alpha=1.1, hot=(0, 9))


def test_multihot_mean_fp32_with_empty_bags():
    run_case([50, 3000, 7], 32, 300, combiner=1, alpha=1.1, hot=(0, 9))


@pytest.mark.parametrize("dim", [4, 8, 20, 64, 100, 256, 384])
def test_row_widths_fp32(dim):
    run_case([37, 1000], dim, 130, hot=(0, 5))
    run_case([37, 1000], dim, 130)


@pytest.mark.parametrize("dim", [8, 24, 128, 520])
def test_row_widths_fp16(dim):
    run_case([37, 1000], dim, 130, dtype=torch.float16, hot=(0, 5))
    run_case([37, 1000], dim, 130, dtype=torch.float16)


def test_keys_without_a_row():
    info = run_case([100, 2000, 30], 16, 500, poison=40)
    run_case([100, 2000, 30], 16, 200, poison=60, hot=(0, 6), combiner=1)
    assert info["nnz"] == 1500


def test_a_workspace_that_was_never_initialised_is_named():
    """Forward and backward work on raw memory (they never read the counter of keys without a row);
    asking for that counter is what fails, and initialising afterwards makes it count."""
    h = H()
    rows, dim, batch = [50, 70], 8, 40
    ro = datagen.row_offsets(rows)
    table = to_dev(datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float32))
    layer = h.EmbeddingLayer(table, 2, 0, ro[:-1].copy(), np.asarray(rows, dtype=np.int64))
    keys = datagen.onehot_keys(SEED, 0, rows, batch, 1.05)
    keys[3] = -5
    d_keys = to_dev(keys)
    raw = torch.full((layer.workspace_bytes(batch, keys.numel()),), 0xA5, dtype=torch.uint8, device="cuda")
    out_raw = layer.forward(batch, d_keys, ws=raw)
    with pytest.raises(h.HctrError) as e:
        layer.invalid_keys(raw)
    assert e.value.status == -3 and "initialised" in str(e.value)
    good = layer.new_workspace(raw.numel())
    out_good = layer.forward(batch, d_keys, ws=good)
    assert torch.equal(out_raw, out_good)
    assert layer.invalid_keys(good) == 1
    layer.reset_invalid_keys(raw)
    layer.forward(batch, d_keys, ws=raw)
    assert layer.invalid_keys(raw) == 1


@pytest.mark.parametrize("dim,dtype", [(8, torch.float32), (64, torch.float32), (128, torch.float32), (128, torch.float16),
                                       (256, torch.float16), (100, torch.float32)],
                         ids=["f32x8", "f32x64", "f32x128", "f16x128", "f16x256", "f32x100"])
@pytest.mark.parametrize("combiner", [0, 1], ids=["sum", "mean"])
def test_large_bags_and_long_runs_take_the_steps_that_only_add(dim, dtype, combiner):
    """Bags of up to 150 keys (whole steps of every lane-group width, a second chunk of 64 keys, a
    partial last step) on few, heavily reused rows (runs of one row that span many reduction steps and
    windows); a width that is no multiple of a wave's columns and keys without a row keep the general
    steps in the picture."""
    run_case([7, 300, 5000], dim, 257, dtype=dtype, combiner=combiner, alpha=1.3, hot=(0, 150))
    run_case([7, 300], dim, 64, dtype=dtype, combiner=combiner, alpha=1.3, hot=(60, 70), poison=25)


def test_allocate_table_with_and_without_room_for_the_spacer():
    h = H()
    for spacer in (0.0, 0.25, 1e6):   # none, one that fits, one that cannot fit (skipped, not an error)
        t = h.allocate_table(1000, 16, torch.float16, "cuda", spacer_gib=spacer)
        assert t.shape == (1000, 16) and t.dtype == torch.float16 and t.is_cuda and t.is_contiguous()
        assert t.data_ptr() % 256 == 0


def test_every_key_equal_one_long_segment():
    """All 9,000 keys hit one row: a segment spanning hundreds of windows and several sort tiles."""
    info = run_case([1], 128, 9000)
    assert info["unique"] == 1 and info["max_count"] == 9000


def test_more_long_rows_than_blocks_in_the_long_row_kernel():
    """The largest slot count (128), three rows per slot, uniform keys: all 384 rows collect about 830
    occurrences each, i.e. 13 reduction windows, so every row goes to the list of long rows and that
    list is longer than the grid of the kernel that walks it (256 blocks)."""
    info = run_case([3] * 128, 8, 2500, alpha=0.0)
    assert info["unique"] == 384 and info["nnz"] == 320000
    assert info["nnz"] // info["unique"] > 9 * 64


@pytest.mark.parametrize("combiner", [0, 1], ids=["sum", "mean"])
def test_bag_sizes_around_what_the_sorted_word_can_carry(combiner):
    """For a mean over bags given by offsets the backward keeps each bag's key count in the bits its
    sorted (row, bag) words do not need for the bag number, and reads the offsets again where the
    count does not fit.  600,000 bags need 20 bits and leave 12: counts up to 4,095 ride along,
    4,096 and more do not.  Most bags are empty; a few sit on either side of that edge."""
    n_bags = 600_000
    hot = np.zeros(n_bags, dtype=np.int64)
    g = np.random.default_rng(SEED)
    where = g.choice(n_bags, 40, replace=False)
    hot[where] = g.integers(1, 60, 40)
    hot[where[:8]] = [4095, 4096, 4097, 5000, 4094, 1, 8191, 8192]
    hot[n_bags - 1] = 4100                      # the last bag: its bound is the last offset
    info = run_case([3000], 8, n_bags, combiner=combiner, alpha=0.8, hot=hot)
    assert info["nnz"] == int(hot.sum())


@pytest.mark.parametrize("batch", [1, 31, 32, 33, 4095, 4096, 4097])
def test_sizes_around_window_and_tile_edges(batch):
    run_case([500], 32, batch)


@pytest.mark.parametrize("tiles", [768, 769, 770, 771, 773, 776, 1024, 1025])
def test_dedup_around_the_switches_of_the_sort(tiles):
    """The sort derives its offsets differently above 48 groups of 16 tiles (768 tiles of 4,096 keys),
    uses narrower blocks above 1,024 tiles, and its scatter hands tiles to blocks die by die, with a
    remainder when the tile count is no multiple of 8.  Distinct rows and their counts against numpy
    on 3.1 to 4.2 M keys with 28-bit row ids (three passes)."""
    h = H()
    S, D = 2, 4
    rows_t = [3_000_000, 130_000_000]
    base = [0, rows_t[0]]
    nnz = tiles * 4096 - 6
    B = nnz // S
    g = torch.Generator(device="cuda").manual_seed(tiles)
    k0 = torch.randint(0, rows_t[0], (B,), generator=g, device="cuda")
    hot = torch.randint(0, 1000, (B,), generator=g, device="cuda")
    cold = torch.randint(0, rows_t[1], (B,), generator=g, device="cuda")
    k1 = torch.where(torch.rand(B, generator=g, device="cuda") < 0.5, hot, cold)
    keys = torch.stack([k0, k1], dim=1).contiguous()
    table = torch.empty((sum(rows_t), D), dtype=torch.float32, device="cuda")   # the key-only half never reads it
    layer = h.EmbeddingLayer(table, S, 0, base, rows_t)
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    layer.backward_dedup(B, keys, ws=ws)
    d_rows, d_cnt = layer.dedup_result(B, nnz, ws=ws)
    torch.cuda.synchronize()
    g_rows = (keys.cpu().numpy() + np.asarray(base)[None, :]).reshape(-1)
    uniq, cnt = np.unique(g_rows, return_counts=True)
    assert np.array_equal(d_rows.cpu().numpy(), uniq)
    assert np.array_equal(d_cnt.cpu().numpy(), cnt)
    assert layer.invalid_keys(ws) == 0
    del table, ws


@pytest.mark.parametrize("batch", [(8 << 20), (8 << 20) + 1], ids=["8Mi-keys-windows-of-64", "8Mi+1-keys-windows-of-256"])
def test_both_sides_of_the_window_switch(batch):
    """The reduction cuts the sorted list into windows of 64 positions up to 8 Mi keys and of 256 above:
    one batch on either side of the switch, on few rows (runs of thousands of windows) and on many."""
    info = run_case([1000, 3_000_000], 4, batch // 2 + batch % 2, alpha=1.05) if batch % 2 == 0 else \
        run_case([3_000_000], 4, batch, alpha=0.0)
    assert info["nnz"] == batch


def test_all_keys_distinct():
    h = H()
    n = 5000
    table = datagen.table_rows_at(SEED, torch.arange(n), 16, torch.float32)
    keys = torch.randperm(n, generator=torch.Generator().manual_seed(3))
    dY = datagen.normal_grads(SEED, 1, n * 16).view(n, 16)
    d_table = to_dev(table)
    layer = h.EmbeddingLayer(d_table, 1, 0, [0], [n])
    layer.backward_sgd(n, to_dev(keys), to_dev(dY), 0.5)
    torch.cuda.synchronize()
    ref = table.clone()
    ref[keys] -= 0.5 * dY
    assert torch.equal(d_table.cpu(), ref)   # one term per row, lr a power of two: exact


def test_empty_batch_and_lr_zero():
    h = H()
    table = datagen.table_rows_at(SEED, torch.arange(64), 8, torch.float32)
    d_table = to_dev(table)
    layer = h.EmbeddingLayer(d_table, 2, 0, [0, 32], [32, 32])
    empty = torch.empty(0, dtype=torch.int64, device="cuda")
    out = layer.forward(0, empty)
    assert out.numel() == 0
    layer.backward_sgd(0, empty, torch.empty(0, device="cuda"), 0.1)
    keys = to_dev(torch.tensor([1, 2, 3, 4]))
    layer.backward_sgd(2, keys, to_dev(torch.ones(4, 8)), 0.0)
    torch.cuda.synchronize()
    assert torch.equal(d_table.cpu(), table)


def test_library_is_the_hip_build():
    h = H()
    import os
    assert os.path.exists(h.lib_path()) and h.lib_path().endswith("libhctr.so")


def test_split_backward_beside_forward_on_two_streams():
    """hctr_emb_backward_dedup on a second stream while hctr_emb_forward runs, then
    hctr_emb_backward_apply: same bits as the single-call backward."""
    h = H()
    rows = datagen.scaled_table_rows(1e-3)
    S, dim, batch = len(rows), 128, 1500
    ro = datagen.row_offsets(rows)
    table = datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float32)
    keys = to_dev(datagen.onehot_keys(SEED, 3, rows, batch, 1.05))
    dY = to_dev(datagen.normal_grads(SEED, 3, batch * S * dim).view(batch * S, dim))
    t1, t2 = to_dev(table), to_dev(table)
    a = h.EmbeddingLayer(t1, S, 0, ro[:-1], rows)
    b = h.EmbeddingLayer(t2, S, 0, ro[:-1], rows)
    out_a = a.forward(batch, keys)
    a.backward_sgd(batch, keys, dY, 0.01)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ws = b.workspace(batch, keys.numel())
    for _ in range(3):                       # several rounds: the workspace is reused across steps
        t2.copy_(to_dev(table))
        side.wait_stream(main)
        b.backward_dedup(batch, keys, ws=ws, stream=side)
        out_b = b.forward(batch, keys, ws=ws)
        main.wait_stream(side)
        b.backward_apply(batch, keys.numel(), dY, 0.01, ws=ws)
        torch.cuda.synchronize()
        assert torch.equal(out_a, out_b) and torch.equal(t1, t2)
    ra, ca = a.dedup_result(batch, keys.numel())
    rb, cb = b.dedup_result(batch, keys.numel(), ws=ws)
    assert torch.equal(ra, rb) and torch.equal(ca, cb)


def test_one_dedup_serves_several_applies():
    """hctr_emb_backward_dedup once, hctr_emb_backward_apply twice with different gradients on the
    same workspace: the same bits as two single-call backwards.  Every row here is frequent enough to
    go on the list of long rows, which each apply has to leave empty for the next."""
    h = H()
    rows, dim, batch = [3] * 8, 16, 4000
    S = len(rows)
    ro = datagen.row_offsets(rows)
    table = datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float32)
    keys = to_dev(datagen.onehot_keys(SEED, 5, rows, batch, 0.0))
    g1 = to_dev(datagen.normal_grads(SEED, 6, batch * S * dim).view(batch * S, dim))
    g2 = to_dev(datagen.normal_grads(SEED, 7, batch * S * dim).view(batch * S, dim))
    t1, t2 = to_dev(table), to_dev(table)
    a = h.EmbeddingLayer(t1, S, 0, ro[:-1], rows)
    b = h.EmbeddingLayer(t2, S, 0, ro[:-1], rows)
    a.backward_sgd(batch, keys, g1, 0.01)
    a.backward_sgd(batch, keys, g2, 0.02)
    ws = b.workspace(batch, keys.numel())
    b.backward_dedup(batch, keys, ws=ws)
    b.backward_apply(batch, keys.numel(), g1, 0.01, ws=ws)
    b.backward_apply(batch, keys.numel(), g2, 0.02, ws=ws)
    torch.cuda.synchronize()
    _, counts = b.dedup_result(batch, keys.numel(), ws=ws)
    assert int(counts.min()) > 9 * 64
    assert torch.equal(t1, t2)


def test_check_offsets_accepts_valid_and_names_broken_input():
    h = H()
    good = torch.tensor([0, 2, 2, 5, 9], dtype=torch.int64, device="cuda")
    h.check_offsets(good, 9)
    big = torch.arange(0, 3_000_001, dtype=torch.int64, device="cuda") * 3
    h.check_offsets(big, 9_000_000)
    for bad, nnz in [([1, 2, 2, 5, 9], 9), ([0, 2, 2, 5, 9], 10), ([0, 3, 2, 5, 9], 9), ([0, 2, 2, 5, -1], -1 + 10)]:
        with pytest.raises(h.HctrError) as e:
            h.check_offsets(torch.tensor(bad, dtype=torch.int64, device="cuda"), nnz)
        assert e.value.status == -1 and "CSR" in str(e.value)
    big[1_500_000] = 0
    with pytest.raises(h.HctrError):
        h.check_offsets(big, 9_000_000)


@pytest.mark.parametrize("hot", [None, (0, 5)])
def test_no_key_has_a_row(hot):
    """Every key outside its table: zeros out, table untouched, an empty dedup result, all keys counted."""
    h = H()
    rows, dim, batch, S = [50, 7, 300], 32, 700, 3
    ro = datagen.row_offsets(rows)
    table = datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float32)
    n_bags = batch * S
    if hot is None:
        offsets, nnz = None, n_bags
    else:
        offsets = datagen.multihot_offsets(SEED, 3, n_bags, hot[0], hot[1])
        nnz = int(offsets[-1])
    g = np.random.default_rng(4)
    keys = torch.from_numpy(g.choice([-1, -7, 300, 10 ** 12], nnz).astype(np.int64))
    d_table = to_dev(table)
    layer = h.EmbeddingLayer(d_table, S, h.MEAN, ro[:-1].copy(), rows)
    d_off = None if offsets is None else to_dev(offsets)
    out = layer.forward(batch, to_dev(keys), d_off)
    assert torch.count_nonzero(out) == 0
    dY = datagen.normal_grads(SEED, 3, n_bags * dim).view(n_bags, dim)
    layer.backward_sgd(batch, to_dev(keys), to_dev(dY), 0.5, d_off)
    assert torch.equal(d_table.cpu(), table)
    assert layer.invalid_keys() == 2 * nnz
    uniq, cnt = layer.dedup_result(batch, nnz)
    assert uniq.numel() == 0 and cnt.numel() == 0


def test_forward_and_backward_can_be_captured_in_a_graph():
    """The compute calls only enqueue kernels (no allocation, no synchronisation, no memset), so a
    step can be captured once and replayed; every replay must give the eager result."""
    h = H()
    rows, dim, batch = [5000, 60, 900], 64, 2048
    S = len(rows)
    ro = datagen.row_offsets(rows)
    table0 = datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float32)
    keys = to_dev(datagen.onehot_keys(SEED, 0, rows, batch, 1.05))
    dY = to_dev(datagen.normal_grads(SEED, 0, batch * S * dim).view(batch, S, dim))

    def make():
        t = to_dev(table0)
        layer = h.EmbeddingLayer(t, S, h.SUM, ro[:-1].copy(), rows)
        ws = layer.new_workspace(layer.workspace_bytes(batch, batch * S))
        out = torch.empty((batch, S, dim), device="cuda")
        return t, layer, ws, out

    t_e, layer_e, ws_e, out_e = make()     # eager reference: three steps
    eager = []
    for _ in range(3):
        layer_e.forward(batch, keys, out=out_e, ws=ws_e)
        layer_e.backward_sgd(batch, keys, dY, 0.05, ws=ws_e)
        eager.append((out_e.clone(), t_e.clone()))

    t_g, layer_g, ws_g, out_g = make()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            layer_g.forward(batch, keys, out=out_g, ws=ws_g)
            layer_g.backward_sgd(batch, keys, dY, 0.05, ws=ws_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert torch.equal(t_g, to_dev(table0))          # capturing runs nothing
    for i in range(3):
        g.replay()
        torch.cuda.synchronize()
        scratch = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between the replays
        assert scratch == scratch
        assert torch.equal(out_g, eager[i][0]), f"replay {i}: forward differs from the eager step"
        assert torch.equal(t_g, eager[i][1]), f"replay {i}: table differs from the eager step"


def _replays_like_eager(make, step, n=3):
    """Runs `step` n times eagerly on one state and replays a graph of one captured step n times on
    another (with eager work and synchronisations between the replays); what the states watch must be
    equal after every step."""
    st_e = make()
    eager = []
    for i in range(n):
        step(st_e)
        eager.append([t.clone() for t in st_e["watch"]])
    st_g = make()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(st_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for i in range(n):
        g.replay()
        torch.cuda.synchronize()
        assert torch.randn(1 << 20, device="cuda").sum().item() is not None   # eager work between the replays
        for k, (a, b) in enumerate(zip(st_g["watch"], eager[i])):
            assert torch.equal(a, b), f"replay {i}: watched tensor {k} differs from the eager step"


def test_multi_hot_step_can_be_captured_in_a_graph():
    h = H()
    rows, dim, batch = [5000, 60, 900], 64, 700
    S = len(rows)
    ro = datagen.row_offsets(rows)
    table0 = datagen.table_rows_at(SEED, torch.arange(int(ro[-1])), dim, torch.float16)
    offsets = datagen.multihot_offsets(SEED, 0, batch * S, 0, 40)
    keys = to_dev(datagen.multihot_keys(SEED, 0, rows, batch, 1.05, offsets))
    d_off = to_dev(offsets)
    dY = to_dev(datagen.normal_grads(SEED, 0, batch * S * dim).view(batch, S, dim))

    def make():
        t = to_dev(table0)
        layer = h.EmbeddingLayer(t, S, h.MEAN, ro[:-1].copy(), rows)
        ws = layer.new_workspace(layer.workspace_bytes(batch, keys.numel()))
        out = torch.empty((batch, S, dim), device="cuda")
        return dict(layer=layer, ws=ws, out=out, watch=[out, t])

    def step(s):
        s["layer"].forward(batch, keys, d_off, out=s["out"], ws=s["ws"])
        s["layer"].backward_sgd(batch, keys, dY, 0.05, d_off, ws=s["ws"])

    _replays_like_eager(make, step)


def test_hashed_step_with_insertion_can_be_captured_in_a_graph():
    """Insert-or-find takes its counts from device memory, so the captured step inserts on its first
    replay and finds on the later ones, as the eager steps do."""
    h = H()
    S, dim, batch, max_rows = 26, 32, 400, 20000
    table0 = datagen.table_rows_at(SEED, torch.arange(max_rows), dim, torch.float32)
    keys = to_dev(datagen.open_space_keys(SEED, 0, S, batch, 1.05))
    dY = to_dev(datagen.normal_grads(SEED, 1, batch * S * dim).view(batch, S, dim))

    def make():
        t = to_dev(table0)
        ht = h.HashTable(32768, max_rows)
        layer = h.EmbeddingLayer(t, S, h.SUM, hash_table=ht, insert_on_miss=True, reuse_forward_rows=True)
        ws = layer.new_workspace(layer.workspace_bytes(batch, batch * S))
        out = torch.empty((batch, S, dim), device="cuda")
        return dict(layer=layer, ws=ws, out=out, ht=ht, watch=[out, t])

    def step(s):
        s["layer"].forward(batch, keys, out=s["out"], ws=s["ws"])
        s["layer"].backward_sgd(batch, keys, dY, 0.05, ws=s["ws"])

    _replays_like_eager(make, step)
