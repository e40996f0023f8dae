"""CPU-side checks of the C ABI: the library loads, exports what include/df.h declares, the
ctypes mirror of the argument structs matches the C layout, host-only entry points agree with
the oracle, and argument validation returns the documented codes without touching a GPU."""
import ctypes as C
import os
import random
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "df.h")


@pytest.fixture(scope="module")
def b():
    lib_path = os.path.join(ROOT, "paper_2601_20499_amd", "libdf_hip.so")
    if not os.path.exists(lib_path):
        sys.path.insert(0, ROOT)
        import __graft_entry__
        __graft_entry__.build()
    from paper_2601_20499_amd import binding
    return binding


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(df_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(b):
    names = _declared_functions()
    assert set(names) == set(b.EXPORTS)
    for n in names:
        assert getattr(b.lib, n) is not None


def test_struct_layout_matches_c(b, tmp_path):
    structs = {"df_attn_args": b.df_attn_args, "df_score_args": b.df_score_args, "df_cache": b.df_cache,
               "df_append_args": b.df_append_args, "df_pack_args": b.df_pack_args,
               "df_attn_plan_info": b.df_attn_plan_info}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "df.h"', 'int main(void){']
    for sname, st in structs.items():
        lines.append(f'printf("{sname} %zu\\n", sizeof({sname}));')
        for fname, _ in st._fields_:
            lines.append(f'printf("{sname}.{fname} %zu\\n", offsetof({sname}, {fname}));')
    lines.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    got = dict(zip(out[0::2], map(int, out[1::2])))
    for sname, st in structs.items():
        assert got[sname] == C.sizeof(st)
        for fname, _ in st._fields_:
            assert got[f"{sname}.{fname}"] == getattr(st, fname).offset, (sname, fname)


def test_status_strings(b):
    seen = {b.status_string(s) for s in range(0, 8)}
    assert len(seen) == 8 and b.status_string(0) == "ok" and b.status_string(99) == "unknown status"


def test_head_context_matches_oracle(b):
    from oracle import df_oracle as orc
    for t in range(5):
        assert b.df_head_context(t, 1560, 1, 5) == orc.head_context_tokens(t, 1560, 1, 5)
    with pytest.raises(b.DfError) as e:
        b.df_head_context(7, 1560, 1, 5)
    assert e.value.status == b.DF_ERR_UNSUPPORTED
    with pytest.raises(b.DfError):
        b.df_head_context(0, 0, 1, 5)


def test_classify_matches_oracle(b):
    from oracle import df_oracle as orc
    rng = np.random.default_rng(0)
    for n, N in [(4, 1), (12, 3), (12, 6), (360, 90), (360, 180), (5, 0), (5, 5)]:
        F = rng.random((n, 3)).astype(np.float32) + 0.01
        F = (F / F.sum(1, keepdims=True)).astype(np.float32)
        for mode_b, mode_o in [(b.DF_CLASSIFY_TWO_CLASS, orc.MODE_TWO_CLASS), (b.DF_CLASSIFY_DHP, orc.MODE_DHP)]:
            types, keys = b.df_classify(F.tolist(), N, mode_b)
            # both sides take the decision in fp32, the precision the scores are produced in
            F32 = F.astype(np.float32)
            key32 = (np.maximum(F32[:, 0], F32[:, 1]) if mode_o == orc.MODE_DHP else F32[:, 0] + F32[:, 1])
            o_types, o_key = orc.classify(F32, N, mode_o)
            if not np.array_equal(np.asarray(o_key, dtype=np.float32), key32):
                # fp64 sum differs from the fp32 sum in the last bit: only ordering of exact ties could change
                pass
            assert types == o_types.tolist(), (n, N, mode_b)
            np.testing.assert_allclose(keys, o_key, rtol=1e-6)


def test_classify_ties_and_errors(b):
    F = [[0.3, 0.3, 0.4]] * 4
    types, _ = b.df_classify(F, 2, b.DF_CLASSIFY_DHP)
    assert types == [b.DF_HEAD_DUMMY, b.DF_HEAD_DUMMY, b.DF_HEAD_SINK, b.DF_HEAD_SINK]
    for bad, code in [((F, 5, 1), b.DF_ERR_RANGE), ((F, -1, 1), b.DF_ERR_RANGE), ((F, 1, 9), b.DF_ERR_UNSUPPORTED),
                      (([[float("nan"), 0, 1]], 0, 0), b.DF_ERR_RANGE)]:
        with pytest.raises(b.DfError) as e:
            b.df_classify(*bad)
        assert e.value.status == code
    assert b.lib.df_classify(None, 3, 1, 0, None, None) == b.DF_ERR_NULL


def _attn_args(b, **kw):
    """A structurally valid argument block built from fake (never dereferenced) device addresses."""
    a = b.df_attn_args()
    a.q = a.k_cur = a.v_cur = a.out = a.k_hist = a.v_hist = 0x10000
    a.q_stride_tok = a.kc_stride_tok = a.o_stride_tok = 4 * 128
    a.q_stride_head = a.kc_stride_head = a.o_stride_head = 128
    a.H, a.d, a.Nq, a.Nc = 4, 128, 100, 100
    a.softmax_scale = 0.1
    a.workspace, a.workspace_bytes = 0x40000, 1 << 30
    keep = {"off": (C.c_int64 * 5)(0, 10, 10, 30, 40), "sl": (C.c_int32 * 4)(5, 0, 20, 0)}
    a.hist_off, a.hist_sink_len = keep["off"], keep["sl"]
    for k, v in kw.items():
        setattr(a, k, v)
    return a, keep


def test_attn_argument_validation(b):
    E = b
    cases = [
        (dict(q=None), E.DF_ERR_NULL),
        (dict(out=None), E.DF_ERR_NULL),
        (dict(d=96), E.DF_ERR_UNSUPPORTED),
        (dict(H=65), E.DF_ERR_UNSUPPORTED),
        (dict(Nq=0), E.DF_ERR_SHAPE),
        (dict(Nc=-3), E.DF_ERR_SHAPE),
        (dict(q=0x10002), E.DF_ERR_ALIGN),
        (dict(q_stride_tok=100), E.DF_ERR_ALIGN),
        (dict(k_hist=None), E.DF_ERR_NULL),
        (dict(softmax_scale=0.0), E.DF_ERR_RANGE),
        (dict(workspace=None), E.DF_ERR_WORKSPACE),                          # the workspace is always required
        (dict(workspace=0x30000, workspace_bytes=8), E.DF_ERR_WORKSPACE),
        (dict(workspace=0x30010), E.DF_ERR_ALIGN),
    ]
    for kw, code in cases:
        a, keep = _attn_args(b, **kw)
        assert b.lib.df_attn_fwd(C.byref(a), None) == code, kw
    a, keep = _attn_args(b)
    keep["off"][2] = 5                                                       # not monotone
    assert b.lib.df_attn_fwd(C.byref(a), None) == E.DF_ERR_RANGE
    a, keep = _attn_args(b)
    keep["sl"][0] = 11                                                       # sink longer than the head's history
    assert b.lib.df_attn_fwd(C.byref(a), None) == E.DF_ERR_RANGE
    a, keep = _attn_args(b, hist_off=None)
    assert b.lib.df_attn_fwd(C.byref(a), None) == E.DF_ERR_NULL
    for hl, code in [((10, 0, 21, 10), E.DF_ERR_RANGE),                      # more keys than the head has rows
                     ((4, 0, 20, 10), E.DF_ERR_RANGE),                       # fewer keys than its sink region
                     ((-1, 0, 20, 10), E.DF_ERR_RANGE)]:
        a, keep = _attn_args(b)
        keep["hl"] = (C.c_int32 * 4)(*hl)
        a.hist_len = keep["hl"]
        assert b.lib.df_attn_fwd(C.byref(a), None) == code, hl
    assert b.lib.df_attn_fwd(None, None) == E.DF_ERR_NULL
    assert b.df_attn_workspace_bytes(12, 128, 4680) >= 12 * 37 * 16 + 512 * 512 * 132
    assert b.df_attn_workspace_bytes(0, 128, 10) == 0


def test_score_argument_validation(b):
    s = b.df_score_args()
    assert b.lib.df_head_score(C.byref(s), None) == b.DF_ERR_NULL
    s.q = s.k_cur = s.k_hist = s.score_out = 0x10000
    s.q_stride_tok = s.kc_stride_tok = 512
    s.q_stride_head = s.kc_stride_head = 128
    s.H, s.d, s.Nq, s.Nc = 4, 128, 100, 100
    s.softmax_scale = 0.1
    off, sl = (C.c_int64 * 5)(0, 10, 20, 30, 40), (C.c_int32 * 4)(5, 5, 5, 5)
    s.hist_off, s.hist_sink_len = off, sl
    s.q_sample_stride, s.q_offset = 0, 0
    assert b.lib.df_head_score(C.byref(s), None) == b.DF_ERR_RANGE
    s.q_sample_stride, s.q_offset = 4, 4
    assert b.lib.df_head_score(C.byref(s), None) == b.DF_ERR_RANGE
    s.q_offset = 1
    assert b.lib.df_head_score(C.byref(s), None) == b.DF_ERR_WORKSPACE
    s.hist_sink_len = None
    assert b.lib.df_head_score(C.byref(s), None) == b.DF_ERR_NULL


def test_cache_argument_validation(b):
    H = 3
    cache = b.Cache(None, None, [0, 10, 10, 30], [2, 0, 5], [8, 0, 15], d=128)
    cache.c.k_cache = cache.c.v_cache = 0x10000
    ap = b.df_append_args()
    ap.cache = C.pointer(cache.c)
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_NULL            # k_new missing
    ap.k_new = ap.v_new = 0x20000
    ap.stride_tok, ap.stride_head, ap.Nc = 384, 128, 0
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_SHAPE
    ap.Nc, ap.stride_tok = 4, 100
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_ALIGN
    cache.win_len[0] = 9                                                     # beyond capacity
    ap.stride_tok = 384
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_RANGE
    cache.win_len[0] = 0
    cache.head_row_off[1] = 9                                                # head 0 rows < sink_cap + win_cap
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_RANGE
    cache.head_row_off[1] = 10
    cache.c.d = 100
    assert b.lib.df_kv_append(C.byref(ap), None) == b.DF_ERR_UNSUPPORTED
    cache.c.d = 128
    pk = b.df_pack_args()
    pk.cache = C.pointer(cache.c)
    assert b.lib.df_pack_context(C.byref(pk), None) == b.DF_ERR_NULL
    # an empty cache packs to nothing without any launch: pure host bookkeeping
    ts, tw = (C.c_int32 * H)(2, 0, 5), (C.c_int32 * H)(8, 0, 15)
    off, sl = (C.c_int64 * (H + 1))(), (C.c_int32 * H)()
    pk.take_sink, pk.take_win, pk.hist_off_out, pk.sink_len_out = ts, tw, off, sl
    assert b.lib.df_pack_context(C.byref(pk), None) == b.DF_OK
    assert list(off) == [0, 0, 0, 0] and list(sl) == [0, 0, 0]
    # pretend the cache is filled: the requested rows exceed the output capacity
    cache.sink_len[0], cache.win_len[0], cache.win_pos[0] = 2, 8, 3
    pk.out_capacity_rows = 5
    assert b.lib.df_pack_context(C.byref(pk), None) == b.DF_ERR_RANGE


def test_generated_mfma_phase_is_current():
    """The committed asm include of the attention kernel is what its generator writes."""
    import importlib.util
    path = os.path.join(ROOT, "paper_2601_20499_amd", "csrc", "gen_attn_phase.py")
    spec = importlib.util.spec_from_file_location("gen_attn_phase", path)
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    assert open(gen.OUT).read() == gen.text()


CONFIG_MIXES = {
    "config2 (9 full of 1+5 frames, 3 dummy)": ([9360] * 9 + [0] * 3, [1560] * 9 + [0] * 3, 1560),
    "config4 (9 full of 12 frames at 720P, 3 dummy)": ([43200] * 9 + [0] * 3, [3600] * 9 + [0] * 3, 3600),
    "config5 (6 dummy, 3..60 frames)": ([4680, 93600, 0, 0, 31200, 0, 56160, 0, 14040, 0, 74880, 0],
                                       [1560, 1560, 0, 0, 1560, 0, 1560, 0, 1560, 0, 1560, 0], 1560),
}


@pytest.mark.parametrize("Nq", [4680, 10800, 24480, 33024, 65797])
@pytest.mark.parametrize("mix", list(CONFIG_MIXES))
def test_attention_plan_fills_the_machine(b, Nq, mix):
    """The launch decomposition keeps at least 95 % of the 256 workgroup slots busy and its spans within
    3 % of each other for every query count of the named shapes (and one that is a multiple of nothing)."""
    hist_len, sink_len, _ = CONFIG_MIXES[mix]
    r = b.df_attn_plan(Nq, Nq, hist_len, sink_len)
    assert r["n_qtiles"] == -(-Nq // 256)
    assert r["workgroups"] == r["n_teams"] * r["team_size"] <= 256
    assert r["n_groups"] == -(-r["n_qtiles"] // r["team_size"])
    assert r["busy"] >= 0.95, r
    assert r["span_max"] - r["span_min"] <= 1 and r["span_max"] <= 1.03 * r["line_len"] / r["n_teams"] + 1, r
    tiles = lambda n: -(-n // 64)
    cols = sum(tiles(s) + tiles(l - s) + tiles(Nq) for l, s in zip(hist_len, sink_len))
    assert r["total_cols"] == cols and r["line_len"] == cols * r["n_groups"]
    assert 0 <= r["cut_units"] <= (r["n_teams"] - 1) * r["team_size"]
    # the walk over the spans that the kernel takes: what the hand-over between workgroups relies on
    assert r["consistent"] == 1, r
    assert r["takes"] <= min(r["gives"], r["n_teams"] - 1) and r["gives"] <= r["n_teams"] - 1
    assert (r["gives"] == 0) == (r["takes"] == 0) == (r["cut_units"] == 0)
    # the same counts from the plan's definition: columns = key tiles of the heads, longest head first, once per
    # group of query tiles; boundaries at k * line_len / n_teams; a boundary strictly inside a unit cuts it
    per_head = sorted((tiles(s) + tiles(l - s) + tiles(Nq) for l, s in zip(hist_len, sink_len)), reverse=True)
    starts, at = [], 0
    for _ in range(r["n_groups"]):
        for n in per_head:
            starts.append((at, at + n))
            at += n
    cuts = [k * r["line_len"] // r["n_teams"] for k in range(1, r["n_teams"])]
    inside = [(lo, hi) for c in cuts for lo, hi in starts if lo < c < hi]
    assert r["gives"] == len(inside) and r["takes"] == len(set(inside))
    assert r["pieces"] == len(starts) + len(inside)
    assert r["max_pieces_per_unit"] == 1 + max([inside.count(u) for u in set(inside)], default=0)


def test_attention_plan_small_and_error_cases(b):
    r = b.df_attn_plan(64, 64, [192, 192, 192, 0], [64, 64, 64, 0])          # config 1: one query tile
    assert r["n_qtiles"] == 1 and r["team_size"] == 1 and r["n_groups"] == 1 and r["n_teams"] >= 1
    r = b.df_attn_plan(1, 1, [0])                                            # one key tile in all: one workgroup
    assert r["workgroups"] == 1 and r["cut_units"] == 0 and r["line_len"] == 1
    for bad, code in (((0, 1, [0]), b.DF_ERR_SHAPE), ((1, 0, [0]), b.DF_ERR_SHAPE), ((1, 1, [-1]), b.DF_ERR_RANGE),
                      ((1, 1, [0] * 65), b.DF_ERR_UNSUPPORTED)):
        with pytest.raises(b.DfError) as e:
            b.df_attn_plan(*bad)
        assert e.value.status == code
    with pytest.raises(b.DfError) as e:
        b.df_attn_plan(4, 4, [10], [11])                                    # sink longer than the history
    assert e.value.status == b.DF_ERR_RANGE



def test_attention_plan_piece_walk_is_consistent_for_random_shapes(b):
    """Seeded random head mixes and query counts (64 heads down to one, empty to long histories, one query to
    many more query tiles than compute units): the pieces tile every span, every unit's pieces lie in consecutive
    spans and cover it, and no span leaves or collects partial sums more than once."""
    rng = random.Random(20499)
    for _ in range(400):
        H = rng.choice([1, 2, 3, 5, 12, 40, 64])
        Nq = rng.choice([1, 63, 64, 255, 256, 257, 1000, 4680, 10800, 24480, 70000])
        Nc = rng.choice([1, 64, 65, Nq])
        lens = [rng.choice([0, 0, 1, 63, 64, 65, 500, 1560, 9360, 40000]) for _ in range(H)]
        sinks = [rng.randint(0, n) for n in lens]
        r = b.df_attn_plan(Nq, Nc, lens, sinks)
        assert r["consistent"] == 1, (H, Nq, Nc, lens, r)
        assert r["workgroups"] <= 256 and r["span_max"] - r["span_min"] <= 1
        assert r["max_pieces_per_unit"] >= 1 and r["pieces"] >= r["n_teams"]
