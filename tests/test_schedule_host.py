"""Host-side checks that need no GPU: the C ABI loads and exports what include/mk.h
declares, the page-budget equations agree with the oracle and the paper's figures, and the
offline scheduler / verifier / serialiser behave (including rejecting corrupted schedules)."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_11581_amd import binding as mk, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KNONE = 0xFFFFFFFF
# dword indices of the instruction format (mk_isa.h)
OP, FLAGS, REF_SEQ, WAIT_CTR0, WAIT_CNT0, SIG_CTR, U0, NU = 0, 1, 2, 4, 6, 8, 13, 14


def build(name="c0_tiny", **opts):
    cfg = synth.model_cfg(synth.CONFIGS[name])
    opts.setdefault("n_workgroups", 256)
    return mk.mk_build_schedule(mk.make_config(cfg, **opts))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mk.h")).read()
    declared = set(re.findall(r"\b(mk_[a-z_0-9]+)\s*\(", hdr))
    assert declared, "no declarations found"
    lib = mk.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), f"libmk.so does not export {name}"
    assert declared == set(mk.EXPORTS)


def test_page_budget_equations_match_oracle_and_paper():
    rng = np.random.default_rng(0)
    for _ in range(200):
        a = [int(x) for x in rng.integers(0, 300000, size=6)]
        a[5] = max(a[5], 1)
        assert mk.mk_pages_available(*a) == oracle.pages_available(*a)
        b = [int(x) for x in rng.integers(0, 64, size=5)]
        b[4] = max(b[4], 1)
        assert mk.mk_pipeline_stages(*b) == oracle.pipeline_stages(*b)
    # Sec. 4.3.2: 64 KB -> 32 KB per iteration is 4 -> 2 pages of 16 KB
    assert mk.mk_pages_available(65536, 0, 0, 0, 0, 16384) == 4
    assert mk.mk_pages_available(32768, 0, 0, 0, 0, 16384) == 2
    # Sec. 1: 128 KB sustains 2 stages of a 4-page iteration; halving K (2 pages) restores 4
    n = mk.mk_pages_available(128 * 1024, 1, 0, 0, 0, 16384)
    assert mk.mk_pipeline_stages(n, 0, 0, 0, 4) == 2 and mk.mk_pipeline_stages(n, 0, 0, 0, 2) == 4


@pytest.mark.parametrize("name", ["c0_tiny", "c1_0p5b", "c2_1p5b", "c3_4b"])
def test_schedules_build_and_verify(name):
    h = build(name)
    mk.mk_schedule_verify(h)
    st = mk.mk_get_stats(h)
    full = synth.CONFIGS[name]
    L, H, d = full["n_layers"], full["hidden"], full["head_dim"]
    qd, kvd, I, V = full["n_q_heads"] * d, full["n_kv_heads"] * d, full["intermediate"], full["vocab"]
    algorithmic = 2 * (L * (H * (qd + 2 * kvd) + qd * H + 3 * H * I) + V * H)
    # the streamed (tile-padded) weights cover the algorithmic bytes with little padding
    assert algorithmic <= st["weight_bytes_per_step"] <= algorithmic * 1.06
    assert st["n_workgroups"] == 256 and st["lds_bytes"] <= 160 * 1024
    assert st["sim_makespan_us"] > 0 and 0 < st["sim_duty_cycle"] <= 1
    assert st["candidates_tried"] > st["candidates_pruned"] >= 0
    mk.mk_destroy(h)


def test_batched_schedule_uses_matrix_cores_and_fits_lds():
    cfg = synth.model_cfg(synth.CONFIGS["c4_7b"], n_layers=2, vocab=4096)
    h = mk.mk_build_schedule(mk.make_config(cfg, n_workgroups=256))
    st = mk.mk_get_stats(h)
    assert st["use_mfma"] == 1 and st["rows_qkv"] == 16 and st["lds_bytes"] <= 160 * 1024
    mk.mk_destroy(h)


@pytest.mark.parametrize("n_wg", [1, 7, 64, 304])
def test_other_grid_sizes(n_wg):
    h = build("c0_tiny", n_workgroups=n_wg)
    mk.mk_schedule_verify(h)
    assert mk.mk_get_stats(h)["n_workgroups"] == n_wg
    mk.mk_destroy(h)


def test_fixed_tiling_overrides_are_honoured():
    h = build("c0_tiny", split_qkv=2, split_o=2, split_gateup=2, split_down=2, attn_chunks=4)
    st = mk.mk_get_stats(h)
    assert (st["split_qkv"], st["split_o"], st["split_gateup"], st["split_down"], st["attn_chunks"]) == (2, 2, 2, 2, 4)
    mk.mk_schedule_verify(h)
    mk.mk_destroy(h)


@pytest.mark.parametrize("bad", [dict(head_dim=8), dict(hidden=100), dict(max_batch=17), dict(max_batch=0),
                                 dict(n_q_heads=3), dict(n_layers=0), dict(max_context=0),
                                 dict(max_batch=2, use_mfma=0), dict(ring_kb=200), dict(ring_kb=8), dict(ring_kb=-3),
                                 dict(split_down=10 ** 6)])
def test_bad_configs_are_rejected(bad):
    cfg = synth.model_cfg(synth.CONFIGS["c0_tiny"])
    opts = {k: bad.pop(k) for k in list(bad) if k in ("use_mfma", "ring_kb", "split_down")}
    cfg.update(bad)
    with pytest.raises(mk.MkError) as e:
        mk.mk_build_schedule(mk.make_config(cfg, n_workgroups=64, **opts))
    assert e.value.code in (mk.MK_EINVAL, mk.MK_EINFEASIBLE)


def test_page_ring_obeys_the_lds_budget():
    """Eq. 1-2 in the builder: the ring (pages of 1 KB, stages of 16) plus the staged activations,
    the reduction area and the instruction/flag areas never exceed 160 KB; a ring that cannot fit
    next to the attention scratch of the 1.5B shape is refused; the search mode picks a depth
    that fits."""
    h = build("c0_tiny", ring_kb=100)
    st = mk.mk_get_stats(h)
    assert st["ring_pages"] == 96 and st["page_bytes"] == 1024 and st["n_stage"] == 6
    assert st["lds_bytes"] <= 160 * 1024 and st["lds_bytes"] >= 96 * 1024
    mk.mk_schedule_verify(h)
    blob = mk.mk_schedule_dump(h)
    h2 = mk.mk_schedule_load(blob)
    assert mk.mk_get_stats(h2)["ring_pages"] == 96 and mk.mk_schedule_dump(h2) == blob
    mk.mk_destroy(h); mk.mk_destroy(h2)
    with pytest.raises(mk.MkError) as e:
        build("c2_1p5b", ring_kb=144)
    assert e.value.code == mk.MK_EINFEASIBLE
    h = build("c2_1p5b", ring_kb=-2)
    st = mk.mk_get_stats(h)
    assert st["ring_pages"] % 16 == 0 and st["lds_bytes"] <= 160 * 1024
    mk.mk_destroy(h)
    assert mk.mk_get_stats(build("c2_1p5b"))["ring_pages"] == 0     # auto: weights stay out of LDS


def test_recorded_profile_guided_tilings_build_and_verify():
    """Every line of the table of recorded tilings (written by the on-device search, read by the library)
    names a known configuration, and mk_build_schedule ALONE, given that configuration with no tiling
    field set, returns that tiling: the schedule the benchmark times is reachable through the C ABI."""
    from paper_2605_11581_amd import autotune
    table = autotune.read_table()
    assert table, "tuned_tilings.txt is empty"
    by_key = {}
    for name, full in synth.CONFIGS.items():
        for b in (1, 2, 4, 8, 16):
            for bits in (16, 4):
                by_key[autotune.shape_key(synth.model_cfg(full, max_batch=b), 256, bits)] = (name, b, bits)
    for key, opts in table.items():
        assert key in by_key, f"{key} matches no known configuration"
        name, b, bits = by_key[key]
        model = synth.model_cfg(synth.CONFIGS[name], max_batch=b)
        assert autotune.tuned_opts(model, 256, bits) == opts
        h = mk.mk_build_schedule(mk.make_config(model, n_workgroups=256, weight_bits=bits))
        mk.mk_schedule_verify(h)
        st = mk.mk_get_stats(h)
        assert st["from_table"] == 1, key
        for k, v in opts.items():
            assert st[k] == v, (key, k)
        mk.mk_destroy(h)
    assert autotune.tuned_opts(synth.model_cfg(synth.CONFIGS["c0_tiny"]), 7) == {}


def test_table_is_bypassed_on_request_or_when_a_tiling_field_is_set(tmp_path, monkeypatch):
    model = synth.model_cfg(synth.CONFIGS["c2_1p5b"])
    h = mk.mk_build_schedule(mk.make_config(model, n_workgroups=256, flags=mk.MK_F_NO_TABLE))
    assert mk.mk_get_stats(h)["from_table"] == 0
    mk.mk_destroy(h)
    h = mk.mk_build_schedule(mk.make_config(model, n_workgroups=256, attn_chunks=16))
    st = mk.mk_get_stats(h)
    assert st["from_table"] == 0 and st["attn_chunks"] == 16
    mk.mk_destroy(h)
    # another table through the environment; a malformed line is skipped, a line that does not build
    # leaves the cost model's choice in place
    from paper_2605_11581_amd import autotune
    key = autotune.shape_key(model, 256, 16)
    alt = tmp_path / "alt.txt"
    alt.write_text(f"{key} attn_chunks=8 rows_qkv=3\n")
    monkeypatch.setenv("MK_TUNED_TABLE", str(alt))
    h = mk.mk_build_schedule(mk.make_config(model, n_workgroups=256))
    assert mk.mk_get_stats(h)["from_table"] == 0
    mk.mk_destroy(h)
    alt.write_text(f"{key} attn_chunks=8 rows_qkv=4 bogus\n{key} attn_chunks=8 rows_qkv=4 rows_down=4 ms=1.5\n")
    h = mk.mk_build_schedule(mk.make_config(model, n_workgroups=256))
    st = mk.mk_get_stats(h)
    assert (st["from_table"], st["attn_chunks"], st["rows_qkv"], st["rows_down"]) == (1, 8, 4, 4)
    blob = mk.mk_schedule_dump(h)
    h2 = mk.mk_schedule_load(blob)          # the blob carries the tiling itself, not a reference to the table
    assert mk.mk_schedule_dump(h2) == blob
    mk.mk_destroy(h); mk.mk_destroy(h2)


def test_build_is_deterministic_and_roundtrips():
    h1, h2 = build("c0_tiny"), build("c0_tiny")
    b1, b2 = mk.mk_schedule_dump(h1), mk.mk_schedule_dump(h2)
    assert b1 == b2
    h3 = mk.mk_schedule_load(b1)
    assert mk.mk_schedule_dump(h3) == b1
    for wg in (0, 17, 255):
        n = mk.mk_instr_count(h1, wg)
        assert n == mk.mk_instr_count(h3, wg)
        for i in range(n):
            assert np.array_equal(mk.mk_instr_get(h1, wg, i), mk.mk_instr_get(h3, wg, i))
    with pytest.raises(mk.MkError):
        mk.mk_schedule_load(b1[:-8])
    with pytest.raises(mk.MkError):
        mk.mk_schedule_load(b"\0" * 64)
    bad = bytearray(b1); bad[0] ^= 0xFF
    with pytest.raises(mk.MkError):
        mk.mk_schedule_load(bytes(bad))
    for h in (h1, h2, h3):
        mk.mk_destroy(h)


def _first(h, wg, pred):
    for i in range(mk.mk_instr_count(h, wg)):
        w = mk.mk_instr_get(h, wg, i)
        if pred(w):
            return i, w
    raise AssertionError("no such instruction")


def _expect_rejected(h, needle=None):
    with pytest.raises(mk.MkError) as e:
        mk.mk_schedule_verify(h)
    assert e.value.code == mk.MK_ESCHED
    if needle:
        assert needle in str(e.value), str(e.value)
    mk.mk_destroy(h)


def test_verifier_rejects_swapped_dependent_instructions():
    h = build("c0_tiny", n_workgroups=4)
    a, b = mk.mk_instr_get(h, 0, 0), mk.mk_instr_get(h, 0, 1)
    assert a[REF_SEQ] != b[REF_SEQ]
    mk.mk_instr_set(h, 0, 0, b); mk.mk_instr_set(h, 0, 1, a)
    _expect_rejected(h)      # the later operator now blocks its own producer: deadlock


def test_verifier_rejects_wrong_counter_target():
    h = build("c0_tiny")
    i, w = _first(h, 3, lambda w: w[WAIT_CTR0] != KNONE)
    w[WAIT_CNT0] += 1
    mk.mk_instr_set(h, 3, i, w)
    _expect_rejected(h, "waits for")


def test_verifier_rejects_dropped_wait():
    h = build("c0_tiny")
    i, w = _first(h, 5, lambda w: w[WAIT_CTR0] != KNONE and w[OP] == 1)
    w[WAIT_CTR0] = KNONE
    mk.mk_instr_set(h, 5, i, w)
    _expect_rejected(h, "waits on nothing")


def test_verifier_rejects_wait_on_the_wrong_producer():
    """A task that waits on an existing counter with the right signal count, but not the one its
    input comes from, leaves a read-after-write pair unordered."""
    h = build("c0_tiny")
    # a down-projection task (stage 5) of layer 0 made to wait for the O projection instead of gate/up
    def anywhere(pred):
        for wg in range(256):
            for i in range(mk.mk_instr_count(h, wg)):
                w = mk.mk_instr_get(h, wg, i)
                if pred(w):
                    return wg, i, w
        raise AssertionError("no such instruction")
    wg, i, w = anywhere(lambda w: w[OP] == 1 and w[REF_SEQ] == 5)
    _, _, o = anywhere(lambda w: w[OP] == 1 and w[REF_SEQ] == 4)
    w[WAIT_CTR0], w[WAIT_CNT0] = o[WAIT_CTR0], o[WAIT_CNT0]
    mk.mk_instr_set(h, wg, i, w)
    _expect_rejected(h, "not ordered")


def test_verifier_guards_the_step_boundary():
    """Steps of a multi-step launch are ordered only by the arg-max counter: the first operator must
    wait for it at the previous step's target, nobody else may, and the arg-max must cover every
    LM-head partial."""
    F_WAIT_PREV, OP_ARGMAX, N_SLOTS = 64, 4, 25
    h = build("c0_tiny")
    i, w = _first(h, 0, lambda w: w[OP] == 1 and w[REF_SEQ] == 0)
    assert w[FLAGS] & F_WAIT_PREV
    w[FLAGS] = int(w[FLAGS]) & (0xFFFFFFFF ^ F_WAIT_PREV)
    mk.mk_instr_set(h, 0, i, w)
    _expect_rejected(h)          # waits inside the step for a counter signalled at its very end
    h = build("c0_tiny")
    done = False
    for wg in range(256):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if not done and w[OP] == 1 and w[REF_SEQ] == 3:
                w[FLAGS] |= F_WAIT_PREV
                mk.mk_instr_set(h, wg, i, w)
                done = True
    assert done
    _expect_rejected(h)
    h = build("c0_tiny")
    found = False
    for wg in range(256):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if w[OP] == OP_ARGMAX:
                w[N_SLOTS] -= 1
                mk.mk_instr_set(h, wg, i, w)
                found = True
    assert found
    _expect_rejected(h, "arg-max")


def test_verifier_rejects_dropped_signal_and_bad_counter():
    h = build("c0_tiny")
    i, w = _first(h, 9, lambda w: w[SIG_CTR] != KNONE)
    w[SIG_CTR] = KNONE
    mk.mk_instr_set(h, 9, i, w)
    _expect_rejected(h)
    h = build("c0_tiny")
    i, w = _first(h, 9, lambda w: w[SIG_CTR] != KNONE)
    w[SIG_CTR] = 10 ** 6
    mk.mk_instr_set(h, 9, i, w)
    _expect_rejected(h, "does not exist")


def test_verifier_rejects_missing_or_duplicated_tile():
    h = build("c0_tiny")
    i, w = _first(h, 11, lambda w: w[OP] == 1)
    w[U0] += 1
    mk.mk_instr_set(h, 11, i, w)
    _expect_rejected(h, "unit")


def _anywhere(h, pred, n_wg=256):
    for wg in range(n_wg):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if pred(w):
                return wg, i, w
    raise AssertionError("no such instruction")


# dword indices of the fields that address weights, vectors and the KV cache (mk_isa.h)
LAYER, W_CHUNK, KBT, GAIN, BIAS = 3, 9, 10, 25, 29
ATT_B, ATT_G, ATT_C, ATT_NC, ATT_BS, ATT_QN, ATT_OUT = 9, 10, 11, 12, 13, 18, 20


@pytest.mark.parametrize("what,pred,field,value,needle", [
    ("attention layer", lambda w: w[OP] == 2, LAYER, 1000, "layer"),
    ("attention kv head", lambda w: w[OP] == 2, ATT_G, 2, "kv head"),
    ("attention sequence", lambda w: w[OP] == 2, ATT_B, 1, "sequence"),
    ("attention chunk index", lambda w: w[OP] == 2, ATT_C, 1 << 20, "chunk"),
    ("attention chunk count", lambda w: w[OP] == 2, ATT_NC, 3, "chunk count"),
    ("attention block size", lambda w: w[OP] == 2, ATT_BS, 32, "block size"),
    ("attention q-norm gain", lambda w: w[OP] == 2, ATT_QN, 12345, "gain"),
    ("attention partial buffer", lambda w: w[OP] == 2, ATT_OUT, 7, "partial buffer"),
    ("combine sequence", lambda w: w[OP] == 3, ATT_B, 5, "sequence"),
    ("GEMV layer", lambda w: w[OP] == 1 and w[REF_SEQ] == 3, LAYER, 1, "layer"),
    ("GEMV weight chunk", lambda w: w[OP] == 1 and w[REF_SEQ] == 4, W_CHUNK, 1 << 30, "weight chunk"),
    ("GEMV chunks per row group", lambda w: w[OP] == 1 and w[REF_SEQ] == 5, KBT, 10 ** 6, "geometry"),
    ("GEMV norm gain", lambda w: w[OP] == 1 and w[REF_SEQ] == 0, GAIN, 1 << 28, "gain"),
    ("GEMV bias", lambda w: w[OP] == 1 and w[REF_SEQ] == 0, BIAS, 64, "bias"),
    ("arg-max sequence", lambda w: w[OP] == 4, ATT_B, 9, "sequence"),
], ids=lambda v: v if isinstance(v, str) and " " in v else None)
def test_verifier_rejects_fields_that_address_weights_vectors_or_the_cache(what, pred, field, value, needle):
    """These fields never show in the activation footprint of a task: a list that carries a wrong one
    would read or append outside its buffers.  Host only: such lists are never run."""
    h = build("c0_tiny")
    wg, i, w = _anywhere(h, pred)
    assert int(w[field]) != value
    w[field] = value
    mk.mk_instr_set(h, wg, i, w)
    _expect_rejected(h, needle)


S_FIELD, NKB, N_ROWS, CFG, XS_LO, XS_N = 12, 11, 15, 16, 22, 23
F_SLICE_MAJOR = 256


def test_k_sliced_down_projection_keeps_a_workgroups_units_inside_one_slice():
    """7B shape at batch 8: the down projection needs eight K slices to fit its staged input in LDS.  Units are numbered
    slice first there, so that a workgroup's share is a few row groups of ONE slice (one staged input, one contiguous
    weight range) rather than one task per (row group, slice) pair."""
    cfg = synth.model_cfg(synth.CONFIGS["c4_7b"], max_batch=8)
    h = mk.mk_build_schedule(mk.make_config(cfg, n_workgroups=256, flags=mk.MK_F_NO_TABLE, split_down=8))
    mk.mk_schedule_verify(h)
    st = mk.mk_get_stats(h)
    assert st["split_down"] == 8
    n_down, multi = 0, 0
    for wg in range(0, 256, 17):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if w[OP] != 1 or w[REF_SEQ] % 8 != 5 or w[LAYER] != 0:
                continue
            assert w[FLAGS] & F_SLICE_MAJOR
            rlog = (int(w[CFG]) >> 4) & 15
            groups = (int(w[N_ROWS]) + (1 << rlog) - 1) >> rlog
            slices = {u // groups for u in range(int(w[U0]), int(w[U0]) + int(w[NU]))}
            assert len(slices) == 1                                   # one K slice per task
            (sl,) = slices
            assert int(w[XS_LO]) == sl * int(w[NKB]) and int(w[XS_N]) <= int(w[NKB])
            n_down += 1
            multi += int(w[NU]) > 1
    assert n_down and multi                                           # ... and several row groups in it
    # a unit outside the staged slice is rejected
    wg, i, w = _anywhere(h, lambda w: w[OP] == 1 and w[REF_SEQ] % 8 == 5 and w[NU] > 1)
    w[XS_N] = 1
    mk.mk_instr_set(h, wg, i, w)
    _expect_rejected(h, "staged input range")


def test_residual_sum_level_exists_where_many_partial_rows_would_be_reread():
    """7B shape, batch 8, down projection in 8 K slices: 64 partial rows.  The schedule sums them in a level of its own
    (op 5, one slice of the hidden dimension per workgroup); the next layer's QKV tasks then read one row per sequence.
    At batch 1 there is no such level."""
    cfg = synth.model_cfg(synth.CONFIGS["c4_7b"], max_batch=8)
    h = mk.mk_build_schedule(mk.make_config(cfg, n_workgroups=256, flags=mk.MK_F_NO_TABLE, split_down=8))
    mk.mk_schedule_verify(h)
    covered = []
    for wg in range(256):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if w[OP] == 5 and w[LAYER] == 3:
                assert w[REF_SEQ] == 3 * 8 + 6 and (int(w[CFG]) >> 16) & 255 == 8
                covered.append((int(w[XS_LO]), int(w[XS_N])))       # (for this op: slice [lo, hi) of the hidden dimension)
            if w[OP] == 1 and w[REF_SEQ] == 4 * 8 + 0:
                assert (int(w[CFG]) >> 16) & 255 == 0                # the next QKV reads no partial rows
    covered.sort()
    assert covered[0][0] == 0 and covered[-1][1] == cfg["hidden"]
    assert all(a[1] == b[0] for a, b in zip(covered, covered[1:]))
    # a slice that overlaps its neighbour is rejected
    wg, i, w = _anywhere(h, lambda w: w[OP] == 5 and w[XS_LO] > 0)
    w[XS_LO] -= 4
    mk.mk_instr_set(h, wg, i, w)
    _expect_rejected(h)
    h1 = build("c2_1p5b")
    assert all(mk.mk_instr_get(h1, wg, i)[OP] != 5 for wg in (0, 100, 255) for i in range(mk.mk_instr_count(h1, wg)))
    mk.mk_destroy(h1)


def test_step_calls_refuse_a_handle_that_is_not_bound():
    """Call order is checked on the host, before anything touches a GPU."""
    h = build("c0_tiny")
    for call in (lambda: mk.lib().mk_decode_step(h, None, None, None, None, 1, None),
                 lambda: mk.lib().mk_fill_cache(h, None, None, None, 1, 4, None),
                 lambda: mk.lib().mk_decode_step_static(h, None, None, None, None, 1, None)):
        assert call() == mk.MK_ESTATE
        assert "before mk_bind_workspace" in mk.mk_last_error()
    mk.mk_destroy(h)


def test_verifier_rejects_list_without_end_and_unknown_opcode():
    h = build("c0_tiny")
    w = mk.mk_instr_get(h, 0, 0)
    w[OP] = 77
    mk.mk_instr_set(h, 0, 0, w)
    _expect_rejected(h, "opcode")


def test_weight_prefetch_is_independent_of_activations():
    """Sec. 4.2.3 (asynchronous prefetching): weight tiles carry no activation dependency, so
    every GEMV instruction names its weight chunks statically -- they are a pure function of the
    instruction, identical from step to step."""
    h = build("c2_1p5b")
    seen = 0
    for wg in (0, 100, 255):
        for i in range(mk.mk_instr_count(h, wg)):
            w = mk.mk_instr_get(h, wg, i)
            if w[OP] == 1:
                assert w[NU] >= 1 and w[9] < 2 ** 31      # w_chunk is a constant of the schedule
                seen += 1
    assert seen > 300
    mk.mk_destroy(h)


def test_no_oracle_in_product_path():
    pkg = os.path.join(ROOT, "paper_2605_11581_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
