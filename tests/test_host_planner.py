"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, validates
its inputs, and the planner's work items cover every decode token and every visible prefill
(row, key) pair exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2508_15919_amd import binding as hb
from paper_2508_15919_amd import synth
from paper_2508_15919_amd.synth import DECODE, PREFILL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hb.LIB_PATH):
        from paper_2508_15919_amd import build
        build.build()
    return hb.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "hfxattn.h")).read()
    declared = set(re.findall(r"\b(hfx_[a-z_]+)\s*\(", header))
    assert declared == set(hb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert hb.hfx_status_string(0) == "ok" and "page id" in hb.hfx_status_string(hb.HFX_ERR_PAGE_ID)
    assert hb.hfx_version()[1] >= 1


def fill(b, scale=0.0):
    shape = hb.make_shape(b.num_q_heads, b.num_kv_heads, b.head_dim, b.num_pages, scale)
    hbts, dbts, wbts = hb.hfx_batch_desc_sizes(shape, b.kind, b.q_len, b.ctx_len)
    host = np.zeros(hbts, np.uint8)
    hb.hfx_fill_batch_desc(shape, b.kind, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages, host)
    d = hb.parse_desc(host)
    assert d["header"].total_bytes == hbts == dbts and d["header"].workspace_bytes == wbts
    return d


def lengths_only(Hq, Hkv, D, kind, q_len, ctx_len):
    """A step with a block table but a one-page dummy pool (the planner never reads the pool)."""
    kind, q_len, ctx_len = (np.asarray(a, np.int32) for a in (kind, q_len, ctx_len))
    npg = (ctx_len.astype(np.int64) + 15) // 16
    indptr = np.zeros(len(kind) + 1, np.int32)
    indptr[1:] = np.cumsum(npg)
    pages = np.arange(int(npg.sum()), dtype=np.int32)[::-1].copy()
    return synth.StepBatch(Hq, Hkv, D, max(1, int(npg.sum())), kind, q_len, ctx_len, indptr, pages,
                           np.zeros((int(q_len.sum()), Hq, D), np.uint16), np.zeros((1, Hkv, 2, 16 * D), np.uint16))


def check_class_order(b, items):
    """Queue of a prefill-dominated step: 8 position classes (position mod 8), one per die.

    The prefill items that read the same piece of the keys of one (request, kv-head), i.e. the same
    split index over row tiles and head blocks, form a unit; the planner may cut a unit into sub-units
    of consecutive row tiles.  A decode item is a unit of its own.  Checked here: the items of one
    (unit, row tile) share a home class; class loads differ by no more than the largest total a unit
    has in one class; the list of a class (its own items in position order, then what other classes
    took off its tail) is in descending cost; a class's positions hold foreign items only behind its
    own."""
    G = b.num_q_heads // b.num_kv_heads
    n = len(items)
    cost, home_of = items["cost"].astype(np.int64), items["home"]
    unit = {}
    by_tile = {}
    for i, it in enumerate(items):
        if it["type"] == 1:
            by_tile.setdefault((int(it["req"]), int(it["row0"]), int(it["h0"])), []).append((int(it["kb"]), i))
        else:
            unit[i] = ("d", i)
    for (req, row0, h0), lst in by_tile.items():
        for s, (_, i) in enumerate(sorted(lst)):
            unit[i] = ("p", req, h0 // G, s)
    home = {}
    for i, it in enumerate(items):
        assert 0 <= int(home_of[i]) < 8
        k = unit[i] + (int(it["row0"]),)
        assert home.setdefault(k, int(home_of[i])) == int(home_of[i]), "one home per unit and row tile"
    loads, unit_total = [], {}
    for c in range(8):
        seq = list(range(c, n, 8))
        own = [i for i in seq if int(home_of[i]) == c]
        assert seq[:len(own)] == own, "foreign items only behind the class's own"
        taken = [i for i in range(n) if int(home_of[i]) == c and i % 8 != c]
        full = own + taken[::-1]                    # taken off the tail, last first
        loads.append(int(cost[full].sum()))
        assert np.all(np.diff(cost[full]) <= 0), "a class's list is in descending cost"
        for i in full:
            unit_total[(c, unit[i])] = unit_total.get((c, unit[i]), 0) + int(cost[i])
    assert max(loads) - min(loads) <= max(unit_total.values()), (loads, max(unit_total.values()))


def check_coverage(b, d):
    h, items, reqs, groups = d["header"], d["items"], d["reqs"], d["groups"]
    Hq, Hkv = b.num_q_heads, b.num_kv_heads
    G = Hq // Hkv
    assert h.n_items == len(items) == h.n_decode_items + h.n_prefill_items
    ty = items["type"]
    n_dec, n_pre = int((ty == 0).sum()), int((ty == 1).sum())
    if np.all(items["home"] >= 0):
        assert h.queue_classes == 8
        check_class_order(b, items)
    else:
        assert np.all(items["home"] == -1) and h.queue_classes == 1
        for k in (0, 1):
            assert np.all(np.diff(items["cost"][ty == k]) <= 0), "each kind in descending modelled cost"
        if n_pre == 0 or n_dec == 0 or np.all(np.diff(items["cost"]) <= 0):
            pass                                   # one kind only, or plain descending order
        else:
            # decode-dominated mixed step: over the first two rounds of 512 positions the prefill items sit
            # at the positions of the workgroups of the first ceil(n_pre / 4) CUs (position mod 256), at
            # most 128 of them; behind that, blocks of 256, decode first, as long as both kinds last
            pair_cus = min((n_pre + 3) // 4, 128)
            want = []
            for pos in range(min(1024, n_dec + n_pre)):
                slot = (pos % 512) % 256 < pair_cus
                if (slot and n_pre) or not n_dec:
                    want.append(1); n_pre -= 1
                else:
                    want.append(0); n_dec -= 1
            while n_dec or n_pre:
                k = min(256, n_dec); want += [0] * k; n_dec -= k
                k = min(256, n_pre); want += [1] * k; n_pre -= k
            assert ty.tolist() == want
    assert np.all(d["ctrl"] == 0)
    # stored block table: exactly the needed pages, in order
    for r in range(b.num_requests):
        n = int(reqs["n_pages"][r])
        assert n == (int(b.ctx_len[r]) + 15) // 16
        assert np.array_equal(d["bt"][reqs["bt_start"][r]:reqs["bt_start"][r] + n],
                              b.bt_pages[b.bt_indptr[r]:b.bt_indptr[r] + n])
        # stored quad-aligned, with the last page repeated behind it
        m = int(reqs["bt_len"][r])
        assert reqs["bt_start"][r] % 4 == 0 and m == (n + 3) // 4 * 4 + 16
        assert np.all(d["bt"][reqs["bt_start"][r] + n:reqs["bt_start"][r] + m] == b.bt_pages[b.bt_indptr[r] + n - 1])
    qi = b.q_indptr()
    assert np.array_equal(reqs["q_start"], qi[:-1])
    # append runs: every new token exactly once, in its page and slot, never across a page boundary
    where = {}
    for row0, n, page, slot0 in d["runs"]:
        assert 1 <= n <= 16 and 0 <= slot0 and slot0 + n <= 16
        for k in range(n):
            assert row0 + k not in where
            where[row0 + k] = (page, slot0 + k)
    assert len(where) == h.total_q
    for r in range(b.num_requests):
        for i in range(int(b.q_len[r])):
            t = int(b.ctx_len[r]) - int(b.q_len[r]) + i
            assert where[qi[r] + i] == (int(b.bt_pages[b.bt_indptr[r] + t // 16]), t % 16)
    slot_owner = np.zeros(max(1, h.n_partial_rows), np.int32)
    group_count = np.zeros(max(1, h.n_groups), np.int32)
    for r in range(b.num_requests):
        mine = items[items["req"] == r]
        c, ql = int(b.ctx_len[r]), int(b.q_len[r])
        if b.kind[r] == DECODE:
            assert np.all(mine["type"] == 0)
            cover = np.zeros((Hkv, (c + 15) // 16), np.int32)
            for it in mine:
                assert it["hn"] in (1, 2, 4) and 0 <= it["kb"] < it["ke"] <= (c + 15) // 16 and it["kb"] % 2 == 0
                cover[it["h0"]:it["h0"] + it["hn"], it["kb"]:it["ke"]] += 1
            assert np.all(cover == 1)
        else:
            assert np.all(mine["type"] == 1)
            p = c - ql
            cover = np.zeros((Hq, ql, c), np.int16)
            for it in mine:
                assert it["hn"] in (1, 2, 4) and it["nrows"] == 32 * 4 // it["hn"] and it["kb"] % 64 == 0
                assert it["h0"] // G == (it["h0"] + it["hn"] - 1) // G, "an item stays inside one kv group"
                r1 = min(ql, it["row0"] + it["nrows"])
                cover[it["h0"]:it["h0"] + it["hn"], it["row0"]:r1, it["kb"]:it["ke"]] += 1
                # modelled cost: 4*D flops per visible pair per q-head at 2000 flops/ns, plus a fixed 3000 ns
                rows_i = np.arange(it["row0"], r1)
                pairs = int(np.clip(np.minimum(it["ke"], p + rows_i + 1) - it["kb"], 0, None).sum())
                assert it["cost"] == int(4.0 * b.head_dim * it["hn"] * pairs / 2000.0 + 3000.0)
            visible = (np.arange(c)[None, :] <= (p + np.arange(ql))[:, None])
            assert np.all(cover[:, visible] == 1), "every visible pair exactly once"
        for f in ("kind", "q_len", "ctx_len", "q_start", "bt_start", "n_pages", "bt_len"):
            assert np.all(mine["rq_" + f] == reqs[f][r]), "an item carries a copy of its request record"
        for it in mine:
            if it["group"] >= 0:
                g = groups[it["group"]]
                rows = g["rows_per_split"]
                assert rows == (it["hn"] * G if it["type"] == 0 else 128)
                s = (it["slot_row"] - g["base_row"]) // rows
                assert 0 <= s < g["nsplit"] and it["slot_row"] == g["base_row"] + s * rows
                slot_owner[it["slot_row"]:it["slot_row"] + rows] += 1
                group_count[it["group"]] += 1
            else:
                assert it["slot_row"] == -1
    if h.n_groups:
        assert np.array_equal(group_count[:h.n_groups], groups["nsplit"]) and np.all(groups["nsplit"] > 1)
        # merge units: every row of every group belongs to exactly one unit
        seen = [np.zeros(g["rows_per_split"], np.int32) for g in groups]
        for gi, chunk in d["units"]:
            per = 1 if groups[gi]["nsplit"] > 8 else 8
            seen[gi][chunk * per:(chunk + 1) * per] += 1
        assert all(np.all(x == 1) for x in seen) and h.n_units == len(d["units"])
        assert np.all(slot_owner[:h.n_partial_rows] == 1)
        assert h.workspace_bytes >= h.ws_off_ml + 8 * h.n_partial_rows >= 4 * h.n_partial_rows * b.head_dim
    else:
        assert h.workspace_bytes == 0


@pytest.mark.parametrize("idx,scale", [(1, 1.0), (2, 0.25), (3, 0.1), (4, 0.12), (5, 0.05)])
def test_planner_covers_scaled_configs(lib, idx, scale):
    b = synth.config(idx, scale)
    check_coverage(b, fill(b))


def test_planner_covers_full_size_lengths(lib):
    # full-size length mixes without materialising pools
    g = np.random.default_rng(0)
    c3 = g.integers(2048, 16385, 256)
    b = lengths_only(32, 8, 128, [DECODE] * 256, [1] * 256, c3)
    d = fill(b)
    check_coverage(b, d)
    assert d["header"].n_items >= 4 * 512, "enough items to balance 512 resident workgroups"
    b = lengths_only(8, 1, 128, [DECODE] * 4 + [PREFILL], [1] * 4 + [4096], [131072, 32768, 70001, 99999, 8192])
    d = fill(b)
    check_coverage(b, d)
    assert d["groups"]["nsplit"].max() <= 64


def test_queue_per_die_and_whole_rounds(lib):
    """Prefill-dominated steps of three to eight items per workgroup get one queue class per die;
    steps of few prefill items per workgroup are cut so that the prefill items fill whole rounds of 512."""
    # four prompts' chunks of 2048 tokens at different depths plus 32 decodes (the prefill-heavy mixed shape)
    g = np.random.default_rng(1)
    dec = g.integers(512, 4097, 32).tolist()
    b = lengths_only(32, 8, 128, [PREFILL] * 4 + [DECODE] * 32, [2048] * 4 + [1] * 32,
                     [2048, 6144, 10240, 14336] + dec)
    d = fill(b)
    assert d["header"].queue_classes == 8 and 3 * 512 <= d["header"].n_items <= 8 * 512
    check_coverage(b, d)
    # one long prompt on one kv-head, with and without decodes beside it
    b = lengths_only(8, 1, 128, [PREFILL] + [DECODE] * 16, [4096] + [1] * 16, [65536] + [90000] * 16)
    d = fill(b)
    assert d["header"].queue_classes == 8
    check_coverage(b, d)
    b = lengths_only(8, 1, 128, [PREFILL], [4096], [65536])
    d = fill(b)
    assert d["header"].n_prefill_items == 1024 and d["header"].queue_classes == 1
    check_coverage(b, d)
    # many short prompts, a decode-only step and a small step keep the single queue
    b = lengths_only(32, 8, 128, [PREFILL] * 256, [256] * 256, [256] * 256)
    assert fill(b)["header"].queue_classes == 1
    b = lengths_only(32, 8, 128, [DECODE] * 64, [1] * 64, [4096] * 64)
    assert fill(b)["header"].queue_classes == 1
    b = lengths_only(32, 8, 128, [PREFILL] * 2, [512] * 2, [512, 2048])
    assert fill(b)["header"].queue_classes == 1


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 64), (2, 2, 128), (16, 1, 64), (12, 4, 128), (6, 2, 64)])
def test_planner_head_layouts_and_ragged_chunks(lib, Hq, Hkv, D):
    b = lengths_only(Hq, Hkv, D, [PREFILL, DECODE, PREFILL, DECODE, PREFILL], [1, 1, 33, 1, 130],
                     [1, 1, 33, 500, 700])
    check_coverage(b, fill(b))


def test_planner_is_a_function_of_lengths_only(lib):
    b = synth.config(2, 0.25)
    p = synth.permute_pages(b, 5)
    d0, d1 = fill(b), fill(p)
    assert np.array_equal(d0["items"], d1["items"]) and np.array_equal(d0["groups"], d1["groups"])
    assert not np.array_equal(d0["bt"], d1["bt"])


def test_validation_errors(lib):
    b = synth.config(1)
    shape = hb.make_shape(4, 2, 64, b.num_pages)
    host = np.zeros(1 << 16, np.uint8)

    def code(fn, *a):
        with pytest.raises(hb.HfxError) as e:
            fn(*a)
        return e.value.code

    ok = (b.kind, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages)
    hb.hfx_fill_batch_desc(shape, *ok, host)
    for bad_shape in [hb.make_shape(4, 3, 64, 8), hb.make_shape(4, 2, 96, 8), hb.make_shape(4, 2, 64, 8, page_size=32),
                      hb.make_shape(4, 2, 64, 0), hb.make_shape(64, 2, 64, 8), hb.make_shape(12, 6, 64, 8)]:
        assert code(hb.hfx_fill_batch_desc, bad_shape, *ok, host) == hb.HFX_ERR_SHAPE
    k = b.kind.copy(); k[0] = 2
    assert code(hb.hfx_fill_batch_desc, shape, k, *ok[1:], host) == hb.HFX_ERR_KIND
    q = b.q_len.copy(); q[0] = 2                          # decode with q_len != 1
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, q, *ok[2:], host) == hb.HFX_ERR_LEN
    c = b.ctx_len.copy(); c[3] = 31                       # context shorter than the chunk
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, b.q_len, c, *ok[3:], host) == hb.HFX_ERR_LEN
    q = b.q_len.copy(); q[3] = 0
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, q, *ok[2:], host) == hb.HFX_ERR_LEN
    ip = b.bt_indptr.copy(); ip[1] = 2                    # request 0 needs 3 pages, gets 2
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, b.q_len, b.ctx_len, ip, b.bt_pages, host) == hb.HFX_ERR_PAGES
    ip = b.bt_indptr.copy(); ip[0] = 1
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, b.q_len, b.ctx_len, ip, b.bt_pages, host) == hb.HFX_ERR_PAGES
    pg = b.bt_pages.copy(); pg[4] = b.num_pages
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, b.q_len, b.ctx_len, b.bt_indptr, pg, host) == hb.HFX_ERR_PAGE_ID
    pg = b.bt_pages.copy(); pg[0] = -1
    assert code(hb.hfx_fill_batch_desc, shape, b.kind, b.q_len, b.ctx_len, b.bt_indptr, pg, host) == hb.HFX_ERR_PAGE_ID
    assert code(hb.hfx_fill_batch_desc, shape, *ok, np.zeros(64, np.uint8)) == hb.HFX_ERR_BUFSIZE
    # null pointers, through the raw ABI
    sz = ctypes.c_size_t()
    assert lib.hfx_batch_desc_sizes(ctypes.byref(shape), 4, None, None, None, ctypes.byref(sz), ctypes.byref(sz),
                                    ctypes.byref(sz)) == hb.HFX_ERR_NULL
    assert lib.hfx_batch_desc_sizes(None, 4, None, None, None, None, None, None) == hb.HFX_ERR_NULL
    assert lib.hfx_mixed_paged_attention(ctypes.byref(shape), None, None, None, None, None, 0, None, None) == hb.HFX_ERR_NULL
    # a blob that is not a descriptor
    junk = np.zeros(4096, np.uint8)
    assert lib.hfx_mixed_paged_attention(ctypes.byref(shape), 16, 16, junk.ctypes.data, 16, None, 0, 16, None) == hb.HFX_ERR_DESC
    # shape that differs from the descriptor's
    other = hb.make_shape(4, 2, 64, b.num_pages + 1)
    assert lib.hfx_mixed_paged_attention(ctypes.byref(other), 16, 16, host.ctypes.data, 16, None, 0, 16, None) == hb.HFX_ERR_SHAPE
    # misaligned device pointer
    assert lib.hfx_mixed_paged_attention(ctypes.byref(shape), 8, 16, host.ctypes.data, 16, None, 0, 16, None) == hb.HFX_ERR_ALIGN
    # the other calls that take their geometry from the staging buffer's header refuse the same blobs
    sh, oth = ctypes.byref(shape), ctypes.byref(other)
    assert lib.hfx_mixed_paged_attention_static(sh, 16, 16, junk.ctypes.data, 16, 16, None) == hb.HFX_ERR_DESC
    assert lib.hfx_mixed_paged_attention_static(oth, 16, 16, host.ctypes.data, 16, 16, None) == hb.HFX_ERR_SHAPE
    assert lib.hfx_gather_kv(sh, 16, junk.ctypes.data, 16, 0, 16, 16, None) == hb.HFX_ERR_DESC
    assert lib.hfx_gather_kv(oth, 16, host.ctypes.data, 16, 0, 16, 16, None) == hb.HFX_ERR_SHAPE
    assert lib.hfx_gather_kv(sh, 16, host.ctypes.data, 16, 4, 16, 16, None) == hb.HFX_ERR_LEN      # request out of range
    assert lib.hfx_append_kv(sh, 16, 16, 16, junk.ctypes.data, 16, None) == hb.HFX_ERR_DESC
    assert lib.hfx_append_kv(oth, 16, 16, 16, host.ctypes.data, 16, None) == hb.HFX_ERR_SHAPE
    stale = host.copy()
    stale[4] ^= 1                                         # a descriptor of another layout version
    assert lib.hfx_mixed_paged_attention(sh, 16, 16, stale.ctypes.data, 16, None, 0, 16, None) == hb.HFX_ERR_DESC
    # a header whose count of queue classes is neither 1 nor 8 (the kernel would index the counters with it)
    bent = host.copy()
    off = hb.DescHeader.queue_classes.offset
    bent[off:off + 4] = np.frombuffer(np.uint32(5).tobytes(), np.uint8)
    ws = 16 if hb.parse_desc(host)["header"].workspace_bytes else None
    assert lib.hfx_mixed_paged_attention(sh, 16, 16, bent.ctypes.data, 16, ws, 1 << 40, 16, None) == hb.HFX_ERR_DESC


def test_extra_reserved_pages_are_ignored(lib):
    b = synth.make_batch(4, 2, 64, [DECODE, PREFILL], [1, 20], [37, 50], 3, extra_pages_per_request=3)
    d = fill(b)
    assert d["header"].n_bt == (4 + 16) + (4 + 16)      # stored: rounded up to 4 entries, plus the padding
    check_coverage(b, d)


def test_copy_pages_validation(lib):
    # every check below fails on the host before anything is enqueued, so dummy device addresses do
    shape = hb.make_shape(8, 2, 64, 10, 0.0)
    stage = np.zeros(64, np.uint8)
    src, dst = 0x10000, 0x20000

    def call(s_ids, d_ids, src_pool=src, dst_pool=dst, dst_pages=6, host=stage, dev=0x30000):
        hb.hfx_copy_pages(shape, src_pool, dst_pool, dst_pages, s_ids, d_ids, host, dev, stage_bytes=64)

    call([], [])                                           # nothing to do
    for s_ids, d_ids, kw, code in [
            ([10], [0], {}, hb.HFX_ERR_PAGE_ID), ([-1], [0], {}, hb.HFX_ERR_PAGE_ID),
            ([0], [6], {}, hb.HFX_ERR_PAGE_ID), ([0, 1], [3, 3], {}, hb.HFX_ERR_PAGES),
            ([0, 1], [2, 0], {"dst_pool": src, "dst_pages": 10}, hb.HFX_ERR_PAGES),
            ([0], [1], {"src_pool": 0x10008}, hb.HFX_ERR_ALIGN),
            (list(range(9)), list(range(9)), {"dst_pages": 10}, hb.HFX_ERR_BUFSIZE),
            ([0], [1], {"dst_pages": 0}, hb.HFX_ERR_SHAPE)]:
        with pytest.raises(hb.HfxError) as e:
            call(s_ids, d_ids, **kw)
        assert e.value.code == code, (s_ids, d_ids, kw)


def test_header_is_plain_c_and_cpp(tmp_path):
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "hfxattn.h")
    for compiler, flags, ext in (("gcc", ["-std=c99", "-pedantic", "-Wall", "-Werror"], "c"),
                                 ("g++", ["-std=c++11", "-Wall", "-Werror"], "cpp")):
        if shutil.which(compiler) is None:
            pytest.skip(f"{compiler} not available")
        src = tmp_path / f"use.{ext}"
        src.write_text('#include "hfxattn.h"\nint main(void) { hfx_shape s; hfx_decision d; (void)s; (void)d; return HFX_OK; }\n')
        subprocess.run([compiler, *flags, "-fsyntax-only", "-I", os.path.dirname(hdr), str(src)], check=True)
