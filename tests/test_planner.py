"""The conversion planner and swizzle synthesizer, checked on the CPU by invariants and against
the oracle's exhaustive wavefront enumerator (many swizzles are equally valid, so plans are not
compared bit for bit).  No GPU needed: planning is host-only."""
import numpy as np
import pytest

import oracle
import workloads as wl

import paper_2505_23819_amd as ll  # noqa: E402  (a missing library must fail loudly, not skip)


def span(vectors):
    s = {0}
    for v in vectors:
        s |= {x ^ v for x in s}
    return s


def random_invertible(rng, d):
    while True:
        cols = [int(rng.integers(0, 1 << d)) for _ in range(d)]
        if len(span(cols)) == 1 << d:
            return cols


def gfx950_phases(access_bytes, side="lds_read"):
    """Lanes served together by one LDS instruction, as measured on gfx950.  Reads: halves of the
    wave for accesses up to 8 bytes, the groups {l5, l2^l3^l4} for 16 bytes.  Writes: halves up to
    4 bytes, 16 consecutive lanes for 8 bytes, 8 consecutive lanes for 16 bytes."""
    if side == "lds_write":
        shift = 5 if access_bytes <= 4 else (4 if access_bytes == 8 else 3)
        return [l >> shift for l in range(64)]
    if access_bytes <= 8:
        return [l >> 5 for l in range(64)]
    return [(l >> 5) * 2 + (((l >> 2) ^ (l >> 3) ^ (l >> 4)) & 1) for l in range(64)]


def banks_of(info, side):
    return info["lds_banks_write"] if side == "lds_write" else info["lds_banks"]


def plan_of(cfg, strategy=None):
    a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
    return ll.ll_plan_convert(a, b, cfg.elem_bytes, None if strategy is None else ll.ll_options_init(strategy=strategy))


def test_conversion_matrix_equals_tabulated_composition():
    # B^-1 o A (Sec. 5.4) against the oracle's table-based inverse
    for cid in (1, 2, 3, 4):
        cfg = wl.config(cid)
        conv = plan_of(cfg).info()["conv"]
        inv_b = oracle.inverse_table(cfg.dst_bases)
        for k in range(cfg.d):
            assert conv[k] == int(inv_b[cfg.src_bases[k]])


def test_classification_of_the_configs():
    kinds = {cid: plan_of(wl.config(cid)).info()["kind_name"] for cid in (1, 2, 3, 4)}
    assert kinds == {1: "lds", 2: "lds", 3: "intra_wave", 4: "lds"}


def test_classification_rules():
    # Sec. 5.4: identity -> nothing to do; only register columns differ -> intra-thread;
    # wave part identity -> intra-warp; otherwise shared memory.
    d, nreg, nlane, nwave = 12, 4, 6, 2
    ident = [1 << k for k in range(d)]
    mk = lambda cols: ll.distributed_layout(nreg, nlane, nwave, [d], cols)
    kind = lambda a, b: ll.ll_plan_convert(mk(a), mk(b), 4).info()["kind_name"]
    assert kind(ident, ident) == "noop"
    regs_swapped = [2, 1] + ident[2:]
    assert kind(ident, regs_swapped) == "reg_only"
    reg_xor = [1, 3] + ident[2:]                       # register bit 1 -> r0 ^ r1: still registers only
    assert kind(ident, reg_xor) == "reg_only"
    lane_reg = ident[:]
    lane_reg[0], lane_reg[5] = lane_reg[5], lane_reg[0]
    assert kind(ident, lane_reg) == "intra_wave"
    wave_lane = ident[:]
    wave_lane[10], lane5 = wave_lane[5], wave_lane[10]
    wave_lane[5] = lane5
    assert kind(ident, wave_lane) == "lds"
    reg_into_wave = ident[:]
    reg_into_wave[0] = 1 | (1 << 11)                   # a register bit leaks into a wave bit
    assert kind(ident, reg_into_wave) == "lds"


def test_strategies_of_the_configs(monkeypatch):
    got = {cid: plan_of(wl.config(cid)).info() for cid in (1, 2, 3, 4)}
    # bit-permutation conversions need no LDS once the kernel picks its own lanes: registers only,
    # or a few lane <-> register stages
    assert got[1]["strategy_name"] in ("reg_permute", "wave_shuffle")
    assert got[2]["strategy_name"] == "reg_permute" and got[2]["register_transpose"] == 1
    assert got[3]["strategy_name"] in ("reg_permute", "wave_shuffle")
    assert got[4]["strategy_name"] == "lds_elem"          # XOR layouts: no common run, element-wide LDS
    for cid in (1, 2, 3, 4):
        assert got[cid]["global_vec_bytes"] == 16
    # with the register / shuffle planner switched off, configs 1-3 stage through LDS with 128-bit accesses
    for cid in (1, 2, 3):
        info = plan_of(wl.config(cid), ll.LL_STRATEGY_LDS_VEC).info()
        assert info["strategy_name"] == "lds_vec"
        assert info["lds_write_bytes"] == 16 and info["lds_read_bytes"] == 16 and info["register_transpose"] == 1


@pytest.mark.parametrize("force", [3, 4])
@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_swizzle_of_configs_is_conflict_free_by_enumeration(cid, force):
    info = plan_of(wl.config(cid), force).info()          # 3: element-wide LDS, 4: 128-bit LDS where it applies
    assert info["strategy_name"] in ("lds_elem", "lds_vec")
    if force == 3:
        assert info["strategy_name"] == "lds_elem"
    n = info["block_bits"]
    assert len(span(info["lds_mem"])) == 1 << n        # M is invertible
    for side in ("lds_write", "lds_read"):
        mx, tot, nph = oracle.wavefronts(info["lds_mem"], info[side], info["lds_write_reg_bits"], 6,
                                         info["elem_bytes"], info["lds_vec_bits"], banks_of(info, side),
                                         gfx950_phases(info["lds_write_bytes"], side))
        assert mx == 1 and tot == nph
    assert info["predicted_wavefronts_write"] == 1 and info["predicted_wavefronts_read"] == 1


@pytest.mark.parametrize("force", [3, 4])
def test_unswizzled_staging_of_config1_conflicts(force):
    # control: the same accesses against a linear (unswizzled) LDS layout do collide
    info = plan_of(wl.config(1), force).info()
    n = info["block_bits"]
    linear = [1 << k for k in range(n)]
    worst = max(oracle.wavefronts(linear, info[side], info["lds_write_reg_bits"], 6, 4, info["lds_vec_bits"],
                                  banks_of(info, side), gfx950_phases(info["lds_write_bytes"], side))[0]
                for side in ("lds_write", "lds_read"))
    assert worst > 1


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_random_layouts_plan_and_swizzle(w):
    rng = np.random.default_rng(100 + w)
    for d, nreg in [(8, 2), (10, 2), (12, 4), (13, 3), (15, 5), (16, 6)]:
        for trial in range(4):
            if trial % 2:
                ca = [1 << int(p) for p in rng.permutation(d)]
                cb = [1 << int(p) for p in rng.permutation(d)]
            else:
                ca, cb = random_invertible(rng, d), random_invertible(rng, d)
            nlane = min(6, d - nreg)
            a = ll.distributed_layout(nreg, nlane, d - nreg - nlane, [d], ca)
            b = ll.distributed_layout(nreg, nlane, d - nreg - nlane, [d], cb)
            info = ll.ll_plan_convert(a, b, w).info()      # runs the library's own table walk too
            if info["strategy_name"] not in ("lds_elem", "lds_vec"):
                continue
            assert info["lds_bytes"] == (1 << info["block_bits"]) * w <= 64 * 1024
            assert info["threads"] * info["vectors_per_thread"] * 16 == info["lds_bytes"]
            assert (1 << info["segment_bits"]) * w >= 16
            for side in ("lds_write", "lds_read"):
                mx, tot, nph = oracle.wavefronts(info["lds_mem"], info[side], info["lds_write_reg_bits"], 6, w,
                                                 info["lds_vec_bits"], banks_of(info, side),
                                                 gfx950_phases(info["lds_write_bytes"], side))
                assert mx == 1, (w, d, trial, side)


def test_common_vector_is_kept_wide(monkeypatch):
    # both layouts keep register bits 0,1 on logical bits 0,1 (4-byte elements): 16-byte LDS accesses
    d = 12
    rng = np.random.default_rng(3)
    rest_a = [1 << int(p) for p in (rng.permutation(d - 2) + 2)]
    rest_b = [1 << int(p) for p in (rng.permutation(d - 2) + 2)]
    a = ll.distributed_layout(4, 6, 2, [d], [1, 2] + rest_a)
    b = ll.distributed_layout(4, 6, 2, [d], [1, 2] + rest_b)
    assert ll.ll_plan_convert(a, b, 4).info()["strategy_name"] in ("reg_permute", "wave_shuffle", "lds_elem")
    info = ll.ll_plan_convert(a, b, 4, ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM)).info()
    assert info["strategy_name"] == "lds_elem"
    assert info["lds_vec_bits"] == 2 and info["lds_write_bytes"] == 16
    for side in ("lds_write", "lds_read"):
        assert oracle.wavefronts(info["lds_mem"], info[side], info["lds_write_reg_bits"], 6, 4, 2,
                                 banks_of(info, side), gfx950_phases(16, side))[0] == 1


def test_plan_errors():
    d = 8
    ident = [1 << k for k in range(d)]
    a = ll.distributed_layout(2, 5, 1, [d], ident)
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(a, ll.distributed_layout(3, 5, 1, [d + 1], ident + [1 << d]), 4)
    assert e.value.status == ll.LL_ERR_DIM_MISMATCH                  # output spaces differ
    tiled = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 5), (ll.LL_IN_TILE, 1)], [d], ident)
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(a, tiled, 4)
    assert e.value.status == ll.LL_ERR_DIM_MISMATCH                  # tile bits differ
    # the same tile split differently over registers, lanes and waves is a flat re-indexing
    assert ll.ll_plan_convert(a, ll.distributed_layout(3, 5, 0, [d], ident), 4).info()["strategy_name"] == "copy"
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(a, a, 3)
    assert e.value.status == ll.LL_ERR_INVALID_ARG
    singular = ident[:]
    singular[3] = singular[2]
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(a, ll.distributed_layout(2, 5, 1, [d], singular), 4)
    assert e.value.status == ll.LL_ERR_NOT_SURJECTIVE
    # a layout with a zero column broadcasts; it still has to cover the logical tensor
    hole = ll.distributed_layout(3, 5, 1, [d], [1, 2, 0, 4, 8, 16, 32, 64, 64])
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(a, hole, 4)
    assert e.value.status == ll.LL_ERR_NOT_SURJECTIVE
    # tile label must pass through
    t_in = [(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 5), (ll.LL_IN_TILE, 1)]
    ta = ll.ll_layout_create(t_in, [d], ident)
    mixed = ident[:]
    mixed[0], mixed[7] = mixed[7], mixed[0]
    with pytest.raises(ll.LLError) as e:
        ll.ll_plan_convert(ta, ll.ll_layout_create(t_in, [d], mixed), 4)
    assert e.value.status == ll.LL_ERR_TILE_MIXED


def surjective_bases(rng, d_in, d_out):
    """Random columns spanning F2^d_out; when d_in > d_out one column is zero (a plain replica bit)."""
    while True:
        cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
        if d_in > d_out:
            cols[int(rng.integers(0, d_in))] = 0
        seen = {0}
        for c in cols:
            seen |= {x ^ c for x in seen}
        if len(seen) == 1 << d_out:
            return cols


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_broadcast_plans_pull_from_the_right_inverse(w):
    """Sec. 5.1 broadcasting / Sec. 5.4 rule 2: the plan's pull map sends every destination index to
    the source index the oracle's right inverse (free variables zero) names for its logical element."""
    rng = np.random.default_rng(500 + w)
    for da, db, dl in [(9, 8, 8), (8, 10, 8), (12, 12, 10), (14, 13, 12), (16, 14, 12), (7, 9, 6), (10, 12, 10)]:
        ca, cb = surjective_bases(rng, da, dl), surjective_bases(rng, db, dl)
        a = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, da - 2)], [dl], ca)
        b = ll.ll_layout_create([(ll.LL_IN_REG, 3), (ll.LL_IN_LANE, db - 3)], [dl], cb)
        info = ll.ll_plan_convert(a, b, w).info()
        assert info["kind_name"] == "broadcast" and info["strategy_name"] == "lds_pull"
        assert info["d"] == da and info["d_dst"] == db
        rinv = oracle.right_inverse_table(ca, dl)
        hb = np.arange(1 << db, dtype=np.uint64)
        pulled = np.zeros(1 << db, dtype=np.uint64)
        logical = np.zeros(1 << db, dtype=np.uint64)
        for k in range(db):
            bit = ((hb >> np.uint64(k)) & np.uint64(1)).astype(bool)
            pulled[bit] ^= np.uint64(info["pull"][k])
            logical[bit] ^= np.uint64(cb[k])
        assert np.array_equal(pulled, rinv[logical].astype(np.uint64))
        assert info["predicted_wavefronts_write"] == 1 and info["lds_bytes"] <= 64 * 1024


def test_broadcast_plan_of_the_paper_zero_column_example():
    """Layout A of Sec. 4.1 with a zero column spliced in after its two register bits
    (Sec. 5.1 "Broadcasting"): 512 hardware slots hold 256 logical elements."""
    base = wl.PAPER_LAYOUT_A
    wide = base[:2] + [0] + base[2:]
    a = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 5), (ll.LL_IN_WAVE, 1)], [4, 4], base)
    b = ll.ll_layout_create([(ll.LL_IN_REG, 3), (ll.LL_IN_LANE, 5), (ll.LL_IN_WAVE, 1)], [4, 4], wide)
    for x, y, dx, dy in ((a, b, 8, 9), (b, a, 9, 8), (b, b, 9, 9)):
        info = ll.ll_plan_convert(x, y, 4).info()
        assert (info["kind_name"], info["d"], info["d_dst"]) == ("broadcast", dx, dy)
    # expanding A into its widened copy: the replica bit (destination bit 2) pulls from nowhere new
    info = ll.ll_plan_convert(a, b, 2).info()
    assert info["pull"][2] == 0
    assert info["pull"][:2] == [1, 2] and info["pull"][3:9] == [4, 8, 16, 32, 64, 128]


def test_device_entry_points_reject_bad_arguments_before_launch():
    cfg = wl.config(1)
    plan = plan_of(cfg)
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, 0, 0, 1, stream=0)
    assert e.value.status == ll.LL_ERR_INVALID_ARG                 # null pointers
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, 4096 + 4, 1 << 20, 1, stream=0)
    assert e.value.status == ll.LL_ERR_INVALID_ARG                 # misaligned
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, 4096, 4096 + 1024, 1, stream=0)
    assert e.value.status == ll.LL_ERR_INVALID_ARG                 # overlap
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, 4096, 1 << 20, -1, stream=0)
    assert e.value.status == ll.LL_ERR_INVALID_ARG
    ll.ll_convert(plan, 0, 0, 0, stream=0)                         # ntiles == 0: no-op
    tiny = ll.ll_plan_convert(ll.ll_layout_create([(ll.LL_IN_REG, 2)], [2], [2, 1]),
                              ll.ll_layout_create([(ll.LL_IN_REG, 2)], [2], [1, 2]), 1)
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(tiny, 4096, 1 << 20, 3, stream=0)            # 12 bytes: not a whole 16-byte vector
    assert e.value.status == ll.LL_ERR_INVALID_ARG

    with pytest.raises(ll.LLError) as e:
        ll.ll_copy(4096, 4096 + 32, 64, stream=0)                  # overlapping buffers
    assert e.value.status == ll.LL_ERR_INVALID_ARG
    g = wl.config(5)
    lay = ll.distributed_layout(g.nreg, g.nlane, g.nwave, g.out_dim_bits, g.src_bases)
    ll.ll_gather(lay, 0, 2, 0, 0, 0, 0, stream=0)                  # valid layout, nothing to move
    with pytest.raises(ll.LLError) as e:
        ll.ll_gather(lay, 2, 2, 0, 0, 0, 0, stream=0)
    assert e.value.status == ll.LL_ERR_INVALID_ARG
    # an axis that crosses waves: outside the paper's legality condition (reported, not an error).  The
    # columns of `big` live on 4 register and all 6 wave bits; the block closed under them is those
    # 10 bits plus 128-byte runs, not the aligned 256 KiB range: staged in LDS
    big = ll.distributed_layout(4, 6, 6, [6, 10], [1 << k for k in range(4)] + [1 << (10 + k) for k in range(6)] +
                                [1 << (4 + k) for k in range(6)])
    info = ll.ll_gather_info(big, 1, 4)
    assert info["kernel_name"] == "block_staged" and info["axis_wave_bits"] == 6 and info["block_bytes"] == 8192
    assert ll.ll_gather_info(big, 0, 4)["kernel_name"] == "shuffle_rows"      # 64 bytes per lane, axis on lane bits
    # 8192 rows of 32 two-byte elements: a block closed under the rows would need runs under 64 bytes
    # to fit LDS; the aligned 512 KiB range is walked through LDS in chunks.  Four times the rows: the
    # range is 2 MiB and the rows are gathered straight from memory
    tall = ll.distributed_layout(4, 6, 8, [13, 5], [1 << k for k in range(18)])
    info = ll.ll_gather_info(tall, 0, 2)
    assert info["kernel_name"] == "lds_phased" and info["block_bytes"] == 512 * 1024
    taller = ll.distributed_layout(4, 6, 10, [15, 5], [1 << k for k in range(20)])
    info = ll.ll_gather_info(taller, 0, 2)
    assert info["kernel_name"] == "global" and info["block_bytes"] == 2048 * 1024
    # a tile label on the axis
    tiled = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 6), (ll.LL_IN_TILE, 2)], [2, 8],
                                [1 << k for k in range(10)])
    with pytest.raises(ll.LLError) as e:
        ll.ll_gather(tiled, 0, 4, 0, 0, 0, 0, stream=0)
    assert e.value.status == ll.LL_ERR_TILE_MIXED


def test_gather_kernel_choice():
    """Sec. 5.5: an axis on lane bits needs one round of shuffles; register bits on the axis mean
    2^bits rounds in the paper and workgroup-LDS staging here; so do wave bits (when they fit)."""
    g = wl.config(5)
    lay = ll.distributed_layout(g.nreg, g.nlane, g.nwave, g.out_dim_bits, g.src_bases)
    info = ll.ll_gather_info(lay, 0, 2)
    assert (info["kernel_name"], info["axis_lane_bits"], info["axis_reg_bits"], info["paper_rounds"]) == ("wave_staged", 6, 0, 1)
    info = ll.ll_gather_info(lay, 1, 2)                            # columns live in registers and waves
    assert (info["kernel_name"], info["axis_reg_bits"], info["axis_wave_bits"], info["paper_rounds"]) == ("block_staged", 4, 4, 16)
    assert info["block_bytes"] == 8192          # 4 register + 4 wave bits and runs of 2^8 elements, not the aligned 32 KiB
    regaxis = ll.distributed_layout(2, 6, 0, [2, 6], [1 << 6, 1 << 7] + [1 << k for k in range(6)])
    info = ll.ll_gather_info(regaxis, 0, 4)
    assert (info["kernel_name"], info["axis_reg_bits"], info["paper_rounds"]) == ("block_staged", 2, 4)
    narrow = ll.distributed_layout(0, 6, 2, [6, 2], [1 << (2 + k) for k in range(6)] + [1, 2])
    assert ll.ll_gather_info(narrow, 0, 4)["kernel_name"] == "block_staged"       # 4 bytes per lane: staged
    rows16 = ll.distributed_layout(2, 6, 2, [6, 4], [1, 2] + [1 << (4 + k) for k in range(6)] + [4, 8])
    assert ll.ll_gather_info(rows16, 0, 4)["kernel_name"] == "shuffle"            # 16 bytes per lane: one shuffle round


def test_paper_shuffle_schedule_invariants():
    """Sec. 5.4 "Intra-warp Data Exchange": with V, I, E, F, G and the completion R as the paper
    defines them, every affine space R(i) + span(V u I u G) holds exactly one vectorized element per
    thread in layout A and in layout B, and the exchange takes 2^|R| rounds.  Checked by brute
    force over all hardware indices with the oracle's apply."""
    rng = np.random.default_rng(42)
    for w, nreg, nlane, nwave in [(4, 2, 5, 1), (4, 4, 6, 0), (2, 3, 6, 1), (1, 4, 6, 0), (4, 5, 5, 1), (2, 5, 4, 0)]:
        d = nreg + nlane + nwave
        low = nreg + nlane
        for trial in range(2):
            waves = [1 << int(x) for x in rng.choice(d, size=nwave, replace=False)]
            rest = [1 << k for k in range(d) if (1 << k) not in waves]
            ca = [rest[int(i)] for i in rng.permutation(low)] + waves
            cb = [rest[int(i)] for i in rng.permutation(low)] + waves
            a = ll.distributed_layout(nreg, nlane, nwave, [d], ca)
            b = ll.distributed_layout(nreg, nlane, nwave, [d], cb)
            info = ll.ll_plan_convert(a, b, w).info()
            if info["kind_name"] == "noop":
                continue
            assert info["kind_name"] in ("reg_only", "intra_wave") and info["sched_valid"] == 1
            V, I, G, R = info["sched_v"], info["sched_i"], info["sched_g"], info["sched_r"]
            assert len(V) <= {1: 2, 2: 1, 4: 0, 8: 0}[w]                     # 32-bit payload
            assert set(V) <= set(ca[:nreg]) & set(cb[:nreg])
            assert set(I) == set(ca[nreg:low]) & set(cb[nreg:low])
            assert len(G) == nlane - len(I) and len(R) + len(V) == nreg
            sub = span(V + I + G)
            assert len(sub) == 1 << (len(V) + len(I) + len(G))                # a basis
            for cols in (ca, cb):
                for wv in range(1 << nwave):
                    wave_img = oracle.apply(cols, wv << low)
                    for r in span(R):
                        coset = {r ^ wave_img ^ x for x in sub}
                        per_lane = {}
                        for h in range(1 << low):
                            x = oracle.apply(cols, h | (wv << low))
                            if x in coset:
                                per_lane.setdefault(h >> nreg, []).append(x)
                        assert len(per_lane) == 1 << nlane                    # every thread takes part
                        for xs in per_lane.values():
                            assert len(xs) == 1 << len(V)                     # exactly one vectorized element
                            assert {x ^ xs[0] for x in xs} == span(V)


def test_plan_of_config1_reports_the_hand_derived_conversion_matrix():
    """The columns of B^-1 o A for config 1, as derived by hand in tests/golden/config_spot_values.txt."""
    row = [l.split() for l in open("tests/golden/config_spot_values.txt") if l.startswith("P")][0]
    info = plan_of(wl.config(1)).info()
    assert info["conv"] == [int(x, 16) for x in row[1:]]


def test_planning_from_several_threads():
    """Layouts and plans are immutable after creation and the library keeps no shared mutable state:
    concurrent planning (ctypes releases the GIL) gives the same plans, and ll_last_error is per thread."""
    import threading
    cfgs = [wl.config(c) for c in (1, 2, 3, 4)]
    want = [plan_of(c).info() for c in cfgs]
    errors = []

    def work(k):
        try:
            for rep in range(5):
                for c, w in zip(cfgs, want):
                    got = plan_of(c).info()
                    assert got["conv"] == w["conv"] and got["strategy"] == w["strategy"] and got["lds_mem"] == w["lds_mem"]
                if k % 2:                                   # provoke an error on this thread only
                    with pytest.raises(ll.LLError) as e:
                        ll.ll_layout_create([(ll.LL_IN_REG, 2)], [1], [1, 7])
                    assert "does not fit" in str(e.value)
        except Exception as exc:                            # noqa: BLE001
            errors.append((k, exc))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_every_plan_keeps_wave_accesses_in_eight_lines():
    """D1 / D5: a wave-wide 16-byte access (1 KiB) must touch exactly 8 lines of 128 bytes on both
    sides, whatever the strategy (plans whose lanes would spread further are rejected in favour of
    the element-wide LDS kernel)."""
    rng = np.random.default_rng(77)
    seen = set()
    for trial in range(150):
        d = int(rng.integers(8, 17))
        w = int(rng.choice([1, 2, 4, 8]))
        nreg = int(rng.integers(0, 7))
        nlane = min(6, d - nreg)
        nwave = d - nreg - nlane
        if trial % 2:
            ca, cb = [1 << int(p) for p in rng.permutation(d)], [1 << int(p) for p in rng.permutation(d)]
        else:
            ca, cb = wl.random_invertible_bases(5000 + trial, d), wl.random_invertible_bases(6000 + trial, d)
        info = ll.ll_plan_convert(ll.distributed_layout(nreg, nlane, nwave, [d], ca),
                                  ll.distributed_layout(nreg, nlane, nwave, [d], cb), w).info()
        if info["kind_name"] == "noop":
            continue
        assert info["src_lines_per_access"] == 8 and info["dst_lines_per_access"] == 8, (trial, info["strategy_name"])
        seen.add(info["strategy_name"])
    for cid in (1, 2, 3, 4):
        info = plan_of(wl.config(cid)).info()
        assert info["src_lines_per_access"] == 8 and info["dst_lines_per_access"] == 8
    assert len(seen) >= 3


def test_sparse_sliced_sources_plan():
    """The slice left by a reduction along the dim the registers run along keeps one element in 2^r
    slots: for 1-byte elements and 16 registers per lane every 16-byte source vector holds a single
    useful byte.  The planner shrinks the destination block until the source vectors behind it fit
    one workgroup (LDS within 64 KiB), for every element size."""
    for regs_along_reduced in (2, 3, 4):
        parent = ll.ll_layout_blocked([1, regs_along_reduced], [3, 3], [1, 1], [1, 0])
        s = ll.ll_layout_slice(parent, 1)
        dl = sum(s.out_dims)
        compact = ll.ll_layout_create([(ll.LL_IN_REG, 1), (ll.LL_IN_LANE, dl - 1)], s.out_dims, [1 << k for k in range(dl)])
        for w in (1, 2, 4, 8):
            for a, b in ((s, compact), (compact, s), (s, s)):
                info = ll.ll_plan_convert(a, b, w).info()
                assert info["kind_name"] == "broadcast" and 0 < info["lds_bytes"] <= 65536
                assert info["predicted_wavefronts_write"] >= 1


def test_binding_rejects_host_and_short_tensors():
    """A tensor handed to a device entry point must be on the GPU and large enough: the binding checks
    before anything is launched (raw integer addresses are taken on trust)."""
    import torch
    c = wl.config(2)
    a = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.src_bases)
    b = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.dst_bases)
    plan = ll.ll_plan_convert(a, b, 2)
    host = torch.zeros(1 << 14, dtype=torch.int16)
    for call in (lambda: ll.ll_convert(plan, host, host.clone(), 1, stream=0),
                 lambda: ll.ll_copy(host, host.clone(), 1 << 15, stream=0),
                 lambda: ll.ll_gather(a, 0, 2, host, torch.zeros(1 << 14, dtype=torch.int32), host.clone(), 1, stream=0)):
        with pytest.raises(ll.LLError) as e:
            call()
        assert e.value.status == ll.LL_ERR_INVALID_ARG and "GPU tensor" in e.value.message
    assert plan.sizes() == (14, 14, 2) and a.d_in == 14


def test_gather_choice_is_remembered_per_layout_and_follows_the_options():
    """The kernel choice of a gather is kept with the layout; a repeated query returns the same
    description, other axes and element sizes get their own, and the options the choice was made
    under are part of the key."""
    cfg = wl.config(5)
    layout = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    first = ll.ll_gather_info(layout, 0, 2)
    assert first["kernel_name"] == "wave_staged"
    assert ll.ll_gather_info(layout, 0, 2) == first
    assert ll.ll_gather_info(layout, 1, 2)["kernel_name"] == "block_staged"
    assert ll.ll_gather_info(layout, 0, 1)["kernel_name"] == "block_staged"       # one-byte elements
    staged = ll.ll_options_init(gather_kernel=ll.LL_GATHER_BLOCK_STAGED)
    assert ll.ll_gather_info(layout, 0, 2, staged)["kernel_name"] == "block_staged"
    assert ll.ll_gather_info(layout, 0, 2, ll.ll_options_init(gather_kernel=ll.LL_GATHER_SHUFFLE))["kernel_name"] == "shuffle"
    assert ll.ll_gather_info(layout, 0, 2) == first
    assert ll.ll_gather_info(layout, 0, 2, ll.ll_options_init()) == first         # all-automatic options = no options
    # many distinct queries on one layout (the list is bounded) still answer correctly
    for rep in range(3):
        for w in (1, 2, 4, 8):
            for axis in (0, 1):
                for knob in (None, 0, 1, 2):
                    for blk in (-1, 4096, 16384, 32768):
                        opts = None if knob is None else ll.ll_options_init(gather_kernel=knob, gather_block_bytes=blk)
                        fresh = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
                        assert ll.ll_gather_info(layout, axis, w, opts) == ll.ll_gather_info(fresh, axis, w, opts)


def test_planning_from_many_threads_gives_the_single_thread_answer():
    """Layouts are immutable and planning keeps no shared state besides the per-layout gather choices:
    eight threads planning conversions and querying gathers on the SAME layout objects (ctypes drops
    the interpreter lock during the calls) get what one thread gets."""
    import threading
    cfg2, cfg5 = wl.config(2), wl.config(5)
    a = ll.distributed_layout(cfg2.nreg, cfg2.nlane, cfg2.nwave, cfg2.out_dim_bits, cfg2.src_bases)
    b = ll.distributed_layout(cfg2.nreg, cfg2.nlane, cfg2.nwave, cfg2.out_dim_bits, cfg2.dst_bases)
    g = ll.distributed_layout(cfg5.nreg, cfg5.nlane, cfg5.nwave, cfg5.out_dim_bits, cfg5.src_bases)
    want_plan = {w: ll.ll_plan_convert(a, b, w).info() for w in (1, 2, 4, 8)}
    fresh = ll.distributed_layout(cfg5.nreg, cfg5.nlane, cfg5.nwave, cfg5.out_dim_bits, cfg5.src_bases)
    want_gather = {(axis, w): ll.ll_gather_info(fresh, axis, w) for axis in (0, 1) for w in (1, 2, 4, 8)}
    errors = []

    def work(t):
        try:
            for i in range(12):
                w = 1 << ((i + t) & 3)
                if ll.ll_plan_convert(a, b, w).info() != want_plan[w]:
                    errors.append(("plan", t, i))
                axis = (i >> 2) & 1
                if ll.ll_gather_info(g, axis, w) != want_gather[(axis, w)]:
                    errors.append(("gather", t, i))
        except Exception as e:                      # noqa: BLE001 - report whatever a thread hit
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors
