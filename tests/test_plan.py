"""Host-side planning of a step (spec_k_plan_step: decoder passes, projection launch shapes, attention
plan), checked without a GPU: invariants over a sweep of shapes, batches and lookaheads -- everything a
launch writes fits what spec_verify_init would have allocated, every variant exists, every limit of the
kernels is respected -- and the plans of the named configurations."""
import random

import pytest

from paper_2411_00853_amd import binding as sv
from paper_2411_00853_amd import workload as wl


def _plan(shape, look, max_batch=None, max_kv_len=2048, kmax=None, cu=256, paged=False):
    cfg = sv.make_cfg(shape, max_batch or len(look), max_kv_len, max(look) if kmax is None else kmax)
    return cfg, sv.spec_k_plan_step(cfg, look, cu, paged)


def _check_invariants(shape, cfg, look, p, paged):
    B, rows = len(look), sum(k + 1 for k in look)
    # passes: consecutive sequences, all rows, none beyond what one launch of the projections takes
    assert p.rows == rows and 1 <= p.n_passes <= sv.PLAN_MAX_PASSES
    assert (p.n_passes == 1) == (rows <= 352)
    b0 = 0
    for g in range(p.n_passes):
        n = p.pass_seqs[g]
        assert n >= 1 and p.pass_rows[g] == sum(k + 1 for k in look[b0:b0 + n]) <= 352
        b0 += n
    assert b0 == B
    # as few passes as filling each to the brim would take, and no pass much above the mean
    fewest, acc = 1, 0
    for k in look:
        if acc + k + 1 > 352:
            fewest, acc = fewest + 1, 0
        acc += k + 1
    assert p.n_passes == fewest
    assert max(p.pass_rows[:p.n_passes]) <= -(-rows // p.n_passes) + 15
    # projections of the first pass
    dq = shape.n_q_heads * shape.head_dim
    n_in = [shape.d_model, dq, shape.d_model, shape.d_ffn, shape.d_model]
    n_out = [dq + 2 * shape.n_kv_heads * shape.head_dim, shape.d_model, 2 * shape.d_ffn, shape.d_model, shape.vocab]
    for i in range(sv.PLAN_PROJECTIONS):
        mt, nt, s, kbs = p.gemm_row_tiles[i], p.gemm_col_tiles[i], p.gemm_k_ranges[i], p.gemm_k_blocks_per_range[i]
        assert mt * 16 >= p.pass_rows[0] and mt in (1, 2, 3, 4, 5, 6, 8, 10, 12, 14, 16, 18, 20, 22)
        assert nt in (1, 2, 3, 4) and p.gemm_row_parts[i] in (1, 2) and p.gemm_col_groups[i] in (2, 3, 4)
        assert (p.gemm_row_parts[i] == 2) == (mt >= 8)
        assert s in (1, 2, 4, 8, 16) and kbs % 4 == 0 and s * kbs >= n_in[i] // 32
        with_work = -(-(n_in[i] // 32) // kbs)
        assert with_work * 8 >= s * 7, "at most one K range in eight may come out empty"
        n_pad = (n_out[i] + 15) // 16 * 16
        assert p.gemm_partial_floats[i] == s * p.pass_rows[0] * n_pad <= p.gemm_partial_capacity
        tiles_per_wg = nt * p.gemm_col_groups[i]
        assert p.gemm_workgroups[i] == -(-(n_pad // 16) // tiles_per_wg) * s
    # operand fragments fit their buffers; SwiGLU inside the GEMM only up to four row tiles
    assert p.xfrag_units <= p.xfrag_capacity and p.xfrag_act_units <= p.xfrag_act_capacity
    if p.gate_up_swiglu_inside:
        assert p.gemm_row_tiles[2] <= 4 and p.xfrag_act_units > 0
    # attention of the first pass
    group = shape.n_q_heads // shape.n_kv_heads
    window = max(look[:p.pass_seqs[0]]) + 1
    assert group % p.attn_kv_share == 0 and (group // p.attn_kv_share) * window <= 64
    assert p.attn_row_tiles == -(-(group // p.attn_kv_share) * window // 16) and 1 <= p.attn_row_tiles <= 4
    assert p.attn_chunk_keys % 32 == 0 and p.attn_chunks * p.attn_chunk_keys >= cfg.max_kv_len
    assert (p.attn_chunks - 1) * p.attn_chunk_keys < cfg.max_kv_len and 1 <= p.attn_chunks
    assert p.attn_chunks <= (16 if not paged else max(16, -(-cfg.max_kv_len // 2048)))
    assert p.attn_wavefronts in (0, 1, 2, 4, 8) and (p.attn_wavefronts == 0 or p.attn_chunks <= p.attn_wavefronts)
    if p.attn_wavefronts:                                   # chunk results of a workgroup fit 64 KiB of LDS
        assert p.attn_wavefronts * p.attn_row_tiles * 16 * (shape.head_dim + 2) * 4 <= 64 * 1024
    if p.attn_fused:
        assert not (shape.head_dim == 128 and p.attn_row_tiles >= 3) and p.attn_chunk_keys >= 192
    if paged:
        assert p.attn_chunk_keys <= 2048
    if p.attn_small:
        assert p.attn_chunks <= max(4, -(-cfg.max_kv_len // 2048) if paged else 1)
    assert p.attn_partial_floats <= p.attn_partial_capacity


@pytest.mark.parametrize("seed", range(40))
def test_plans_respect_every_limit(seed):
    r = random.Random(seed)
    for _ in range(25):
        hd = r.choice([64, 128])
        n_kv = r.choice([1, 2, 4, 8, 16, 32])
        group = r.choice([1, 2, 3, 4, 6, 8, 16])
        d = r.choice([256, 1024, 2048, 4096, 8192])
        shape = wl.ModelShape(r.choice([1, 4, 32]), d, n_kv * group, n_kv, hd, r.choice([512, 2752, 11008, 28672]),
                              r.choice([1000, 32000, 128256]))
        kmax = r.choice([0, 1, 5, 10, 15])
        max_batch = r.choice([1, 8, 32, 64, 200, 256])
        B = r.randrange(1, max_batch + 1)
        look = [r.randrange(0, kmax + 1) for _ in range(B)]
        look[r.randrange(B)] = kmax
        paged = r.random() < 0.3
        max_kv_len = r.choice([64, 1030, 2054, 4107, 16384, 32768, 131072])
        if max_kv_len < kmax + 1:
            max_kv_len = 64
        cu = r.choice([256, 256, 64, 304])
        cfg = sv.make_cfg(shape, max_batch, max_kv_len, kmax)
        p = sv.spec_k_plan_step(cfg, look, cu, paged)
        _check_invariants(shape, cfg, look, p, paged)


def test_capacity_holds_for_every_batch_and_row_count():
    """What a launch writes never exceeds what init allocates, for every batch size up to the handle's
    and the full range of row counts (the check the step itself makes before launching)."""
    for shape, max_batch, kmax, max_kv in ((wl.SEVEN_B, 32, 10, 4107), (wl.ONE_B, 16, 15, 2048),
                                           (wl.ModelShape(2, 512, 64, 8, 64, 1024, 50000), 64, 15, 700)):
        cfg = sv.make_cfg(shape, max_batch, max_kv, kmax)
        for B in range(1, max_batch + 1):
            for k in (0, kmax // 2, kmax):
                p = sv.spec_k_plan_step(cfg, [k] * B, 256, False)
                assert max(p.gemm_partial_floats) <= p.gemm_partial_capacity
                assert p.attn_partial_floats <= p.attn_partial_capacity


def test_plans_of_the_named_configurations():
    w = wl.workload_7b()
    cfg, p = _plan(w.shape, list(w.lookahead), w.batch, w.max_kv_len, w.max_lookahead)
    assert p.rows == 48 and p.n_passes == 1
    assert list(p.gemm_row_tiles) == [3] * 5
    # (the launch rounds these up to whole rounds of the 8 XCDs: 250 runs as a grid of 256)
    # (the QKV projection as 256 workgroups of three wavefronts: four per workgroup would leave 64 compute units idle)
    assert list(p.gemm_workgroups) == [256, 256, 172, 256, 250] and list(p.gemm_col_groups) == [3, 2, 4, 4, 4]
    # (two column groups where a workgroup's K range stays within 2048: the output projection in 4 ranges, not the down projection)
    assert list(p.gemm_k_ranges) == [2, 4, 2, 8, 2]
    assert (p.attn_kv_share, p.attn_small, p.attn_chunks, p.attn_wavefronts, p.attn_fused) == (1, 0, 2, 2, 1)
    assert p.gate_up_swiglu_inside == 1
    w = wl.workload_1b()
    cfg, p = _plan(w.shape, list(w.lookahead), w.batch, w.max_kv_len, w.max_lookahead)
    assert p.rows == 6 and list(p.gemm_row_tiles) == [1] * 5
    # a small launch: every query head a work item of its own, four chunks merged in the workgroup
    assert (p.attn_kv_share, p.attn_small, p.attn_chunks, p.attn_wavefronts, p.attn_fused) == (4, 1, 4, 4, 1)
    w = wl.workload_dyn()
    cfg, p = _plan(w.shape, list(w.lookahead), w.batch, w.max_kv_len, w.max_lookahead)
    assert p.rows == sum(k + 1 for k in w.lookahead) and p.n_passes == 1
    assert list(p.gemm_row_tiles) == [10] * 5 and list(p.gemm_row_parts) == [2] * 5
    assert (p.attn_kv_share, p.attn_small, p.attn_chunks, p.attn_wavefronts) == (1, 0, 1, 1)


def test_steps_beyond_one_pass_and_beyond_64_rows_per_kv_head():
    shape = wl.ModelShape(2, 256, 16, 2, 64, 512, 1000)          # 8 query heads per kv head
    cfg, p = _plan(shape, [15] * 40, 40, 400, 15)
    assert p.rows == 640 and p.n_passes == 2 and list(p.pass_rows[:2]) == [320, 320]
    assert p.attn_kv_share >= 2 and (8 // p.attn_kv_share) * 16 <= 64
    cfg, p = _plan(shape, [3] * 40, 40, 400, 15)                 # 8 x 4 = 32 rows: one item per kv head would do
    assert p.n_passes == 1 and (8 // p.attn_kv_share) * 4 <= 64


def test_bad_arguments_are_refused():
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    cfg = sv.make_cfg(shape, 4, 100, 5)
    with pytest.raises(sv.SpecError):
        sv.spec_k_plan_step(cfg, [6, 1], 256)                    # lookahead beyond the handle's
    with pytest.raises(sv.SpecError):
        sv.spec_k_plan_step(cfg, [1] * 5, 256)                   # batch beyond the handle's
    with pytest.raises(sv.SpecError):
        sv.spec_k_plan_step(cfg, [1], 0)
    fp32 = sv.make_cfg(wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32"), 4, 100, 5)
    with pytest.raises(sv.SpecError):
        sv.spec_k_plan_step(fp32, [1], 256)


def test_chunks_follow_the_resident_wavefronts_of_the_128_dim_fused_variant():
    """7B-shape (32 kv heads x 128): two chunks per pair as long as they fit the 1024 wavefronts the chip
    holds of that variant, one chunk where only that fits them, two again where neither does."""
    for B, chunks in ((8, 2), (16, 2), (18, 1), (20, 1), (24, 1), (27, 1), (28, 1), (32, 1), (33, 2), (48, 2)):
        cfg = sv.make_cfg(wl.SEVEN_B, B, 2054, 5)
        p = sv.spec_k_plan_step(cfg, [5] * B, 256, False)
        assert p.attn_chunks == chunks, (B, p.attn_chunks)
