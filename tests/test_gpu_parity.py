"""GPU parity: the HIP path through the C ABI against the fp64 CPU oracle, element by element.

Tolerance (bf16 outputs, fp32 accumulation): max-abs <= 2e-2 and mean-abs <= 2e-3 over all
outputs of a step.  Paging (gather) and results that are bf16-representable by construction
are compared bit for bit."""
import numpy as np
import pytest

from paper_2508_15919_amd import synth
from paper_2508_15919_amd.synth import DECODE, PREFILL, bf16_bits_to_f64

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


@pytest.fixture(scope="module")
def hb():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2508_15919_amd import binding
    binding.load()
    return binding


def report(b, err):
    qi = b.q_indptr()
    lines = []
    for r in range(b.num_requests):
        e = err[qi[r]:qi[r + 1]]
        lines.append(f"  req {r} kind {int(b.kind[r])} q {int(b.q_len[r])} c {int(b.ctx_len[r])}: "
                     f"max {np.nanmax(e):.3e} nan {int(np.isnan(e).sum())} per-head {np.round(np.nanmax(e, axis=(0, 2)), 4).tolist()}")
    return "\n".join(lines[:40])


def run_gpu(hb, b):
    step = hb.DeviceStep(b)
    step.run()
    return step, step.out_bits()


def check_full(hb, oracle, b):
    step, bits = run_gpu(hb, b)
    got = bf16_bits_to_f64(bits)
    ref = oracle.attention_batch(b)
    err = np.abs(got - ref)
    msg = f"{b.name}: max {np.nanmax(err):.3e} mean {np.nanmean(err):.3e}\n" + report(b, err)
    print(f"{b.name}: T={b.total_q} max-abs {np.nanmax(err):.3e} mean-abs {np.nanmean(err):.3e}", flush=True)
    assert np.isfinite(got).all(), msg
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, msg
    return step, bits


def test_config1_tiny_mixed(hb, oracle):
    check_full(hb, oracle, synth.config(1))


@pytest.mark.parametrize("idx,scale", [(2, 0.25), (3, 0.1), (4, 0.12), (5, 0.05)])
def test_scaled_configs_full_compare(hb, oracle, idx, scale):
    check_full(hb, oracle, synth.config(idx, scale))


def test_config2_full_size(hb, oracle):
    check_full(hb, oracle, synth.config(2))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("idx", [3, 4, 5])
def test_large_configs_full_size_all_outputs(hb, oracle, idx):
    """The decode-heavy, prefill-heavy and long-context steps at full size, every output compared (the
    oracle takes seconds on the first and about half a minute on the other two with 16 host threads)."""
    check_full(hb, oracle, synth.config(idx))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("idx,scale,which", [(2, 1.0, PREFILL), (2, 1.0, DECODE), (4, 1.0, DECODE), (4, 0.25, PREFILL),
                                             (5, 0.1, PREFILL), (5, 0.1, DECODE), (4, 1.0, PREFILL)])
def test_pure_prefill_and_pure_decode_steps(hb, oracle, idx, scale, which):
    """Steps of one kind only (the prefill batch E_p and the decode iteration E_d of Section 3.3.1; what the
    prefill and decode instances of the disaggregated mode run): the all-prefill queue never has a decode
    item between two prompts' items, and the other way round."""
    check_full(hb, oracle, synth.config(idx, scale).sub_batch(which))


def test_table1_pure_prefill_step(hb, oracle):
    check_full(hb, oracle, synth.table1_short_context().sub_batch(PREFILL))


def test_single_token_context_returns_v_bit_exact(hb):
    b = synth.make_batch(32, 8, 128, [DECODE, PREFILL, DECODE], [1, 1, 1], [1, 1, 1], 5)
    _, bits = run_gpu(hb, b)
    for r in range(3):
        page = b.bt_pages[b.bt_indptr[r]]
        v = b.pool[page, :, 1].reshape(8, 128, 16)[:, :, 0]           # [g, d] at slot 0
        for h in range(32):
            assert np.array_equal(bits[r, h], v[h // 4]), (r, h)


def test_page_permutation_gives_identical_bits(hb):
    for b in (synth.config(1), synth.config(2, 0.25), synth.config(5, 0.05)):
        _, a = run_gpu(hb, b)
        _, c = run_gpu(hb, synth.permute_pages(b, 9))
        assert np.array_equal(a, c), b.name


def test_gather_is_bit_exact(hb, oracle):
    for b in (synth.config(1), synth.config(2, 0.1)):
        step = hb.DeviceStep(b)
        for r in range(b.num_requests):
            k, v = step.gather(r)
            ok, ov = oracle.gather_kv(b.num_kv_heads, b.head_dim, b.num_pages, b.ctx_len, b.bt_indptr, b.bt_pages,
                                      b.pool, r)
            assert np.array_equal(k, ok) and np.array_equal(v, ov), (b.name, r)


def test_descriptor_serves_repeated_launches(hb):
    import torch
    b = synth.config(4, 0.12)
    step = hb.DeviceStep(b)
    step.run()
    first = step.out_bits().copy()
    for _ in range(3):
        step.out.zero_()
        step.run()
        assert np.array_equal(step.out_bits(), first)
    torch.cuda.synchronize()
    d = hb.parse_desc(step.device_desc.cpu().numpy())
    assert np.all(d["ctrl"] == 0), "control words must be restored to zero"
    assert d["header"].n_groups > 0


def test_queue_per_die_step_and_repeated_launches(hb, oracle):
    """A prefill-dominated step of four items per workgroup: the planner lays the queue out in one class
    per die and the kernel keeps a ticket counter per class.  Compared with the oracle, launched again on
    the same descriptor (all counters must have been put back), and with a decode request beside it."""
    import torch
    kinds = [PREFILL] * 4 + [DECODE] * 6
    ql = [2048, 2048, 2048, 2000] + [1] * 6
    cl = [2048, 2304, 2560, 2100] + [700, 33, 1500, 257, 4096, 16]
    b = synth.make_batch(32, 8, 128, kinds, ql, cl, 4242)
    step, _ = check_full(hb, oracle, b)
    d = hb.parse_desc(step.host_desc.numpy())
    assert d["header"].queue_classes == 8 and np.all(d["items"]["home"] >= 0)
    first = step.out_bits().copy()
    for _ in range(3):
        step.out.zero_()
        step.run()
        assert np.array_equal(step.out_bits(), first)
    torch.cuda.synchronize()
    assert np.all(hb.parse_desc(step.device_desc.cpu().numpy())["ctrl"] == 0), "control words must be restored to zero"


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 64), (2, 2, 128), (16, 1, 64), (16, 1, 128), (12, 4, 128), (8, 8, 128),
                                      (6, 2, 64)])
def test_head_layouts_and_ragged_lengths(hb, oracle, Hq, Hkv, D):
    kinds = [PREFILL, DECODE, PREFILL, DECODE, PREFILL, DECODE, PREFILL, DECODE]
    ql = [1, 1, 33, 1, 130, 1, 64, 1]
    cl = [1, 16, 33, 500, 700, 17, 64, 2049]
    check_full(hb, oracle, synth.make_batch(Hq, Hkv, D, kinds, ql, cl, 100 + Hq + D, extra_pages_per_request=1))


@pytest.mark.parametrize("seed", range(8))
def test_random_steps(hb, oracle, seed):
    """Random shapes and length mixes: one-tile and many-tile prefill items and decode ranges of all
    sizes follow each other in every order in a workgroup's queue."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv, D = [(32, 8, 128), (8, 8, 64), (16, 2, 128), (4, 1, 64), (24, 8, 128), (32, 4, 64), (8, 2, 128),
                  (16, 16, 128)][seed]
    R = int(rng.integers(1, 48))
    kinds, ql, cl = [], [], []
    for _ in range(R):
        if rng.random() < 0.5:
            kinds.append(DECODE); ql.append(1); cl.append(int(rng.choice([1, 2, 15, 16, 17, 31, 33, 257, 1000, 3000, 6000])))
        else:
            q = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 100, 129, 300]))
            prior = int(rng.choice([0, 0, 1, 16, 63, 64, 100, 700]))
            kinds.append(PREFILL); ql.append(q); cl.append(q + prior)
    check_full(hb, oracle, synth.make_batch(Hq, Hkv, D, kinds, ql, cl, 2000 + seed, name=f"random-{seed}"))


def test_many_short_items_in_a_row(hb, oracle):
    """Far more items than resident workgroups, almost all of them one tile long: every workgroup chains
    through dozens of hand-overs, first on its two dealt items and then on counter tickets."""
    rng = np.random.default_rng(77)
    R = 700
    kinds = [PREFILL if i % 3 else DECODE for i in range(R)]
    ql = [int(rng.integers(1, 70)) if k == PREFILL else 1 for k in kinds]
    cl = [q if k == PREFILL else int(rng.integers(1, 200)) for k, q in zip(kinds, ql)]
    check_full(hb, oracle, synth.make_batch(32, 8, 128, kinds, ql, cl, 78, name="many-short"))


def test_items_of_one_to_six_tiles_and_pairs(hb, oracle):
    """The ticket for the item after next is asked for and published at tile (or page-pair) positions
    that depend on how long the current item is: prompts whose row tiles see 1..6 key tiles and decodes
    whose wavefronts walk 1..6 page pairs, far more of them than resident workgroups, in one queue."""
    rng = np.random.default_rng(91)
    kinds, ql, cl = [], [], []
    for rep in range(40):
        for tiles in range(1, 7):
            kinds.append(PREFILL); ql.append(32); cl.append(64 * tiles - int(rng.integers(0, 31)))
            kinds.append(DECODE); ql.append(1); cl.append(32 * tiles - int(rng.integers(0, 31)))
    check_full(hb, oracle, synth.make_batch(32, 8, 128, kinds, ql, cl, 92, name="ticket-points"))


def test_merge_of_two_to_sixty_splits(hb, oracle):
    """The merge launch has one body per slot count (2, 4, 8) and a wide form above 8 splits: decode
    contexts cut into 2, 3, 4, 5, 8, 9, 16, about 40 and about 60 pieces, and a prompt chunk on a
    long prior context whose row tiles are split along the keys."""
    ctx = [300, 500, 700, 900, 1450, 1650, 2950, 7400, 13000]
    kinds = [DECODE] * len(ctx) + [PREFILL]
    ql = [1] * len(ctx) + [96]
    cl = ctx + [6000]
    b = synth.make_batch(32, 8, 128, kinds, ql, cl, 93, name="split-counts")
    d = hb.parse_desc(hb.DeviceStep(b).host_desc.numpy())
    nsplit = sorted(set(int(x) for x in d["groups"]["nsplit"]))
    assert nsplit[0] == 2 and nsplit[-1] > 48 and any(2 < x <= 4 for x in nsplit) and any(4 < x <= 8 for x in nsplit) \
        and any(8 < x <= 16 for x in nsplit), nsplit
    check_full(hb, oracle, b)


def test_shared_prefix_pages(hb, oracle):
    b = synth.make_batch(32, 8, 128, [DECODE, DECODE, PREFILL], [1, 1, 40], [300, 300, 296], 13)
    n = 16
    for r in (1, 2):
        b.bt_pages[b.bt_indptr[r]:b.bt_indptr[r] + n] = b.bt_pages[0:n]      # first 256 tokens shared
    check_full(hb, oracle, b)


def test_table1_short_context_step(hb, oracle):
    check_full(hb, oracle, synth.table1_short_context())


def test_custom_softmax_scale(hb, oracle):
    b = synth.config(1)
    step = hb.DeviceStep(b, softmax_scale=0.05)
    step.run()
    got = bf16_bits_to_f64(step.out_bits())
    ref = oracle.attention_batch(b, scale=float(np.float32(0.05)))
    err = np.abs(got - ref)
    assert np.isfinite(got).all() and err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


@pytest.mark.parametrize("idx,scale", [(1, 1.0), (2, 0.25), (5, 0.05)])
def test_append_kv_is_bit_exact_and_feeds_attention(hb, oracle, idx, scale):
    import torch
    b = synth.config(idx, scale)
    rng = np.random.default_rng(idx)
    T, Hkv, D = b.total_q, b.num_kv_heads, b.head_dim
    k_new = synth.f32_to_bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    v_new = synth.f32_to_bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    step = hb.DeviceStep(b)
    hb.hfx_append_kv(step.shape, torch.from_numpy(k_new.view(np.int16)).cuda(), torch.from_numpy(v_new.view(np.int16)).cuda(),
                     step.pool, step.host_desc, step.device_desc, torch.cuda.current_stream())
    torch.cuda.synchronize()
    oracle.append_kv(Hkv, D, b.num_pages, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages, k_new, v_new, b.pool)
    assert np.array_equal(step.pool.cpu().numpy().view(np.uint16), b.pool), "pool after append must match bit for bit"
    step.run()
    got = bf16_bits_to_f64(step.out_bits())
    err = np.abs(got - oracle.attention_batch(b))
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS

@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 1, 64), (8, 2, 128)])
def test_append_kv_runs_that_start_and_end_inside_pages(hb, oracle, Hq, Hkv, D):
    """The append walks the new tokens page by page: chunks whose first and last tokens fall anywhere in a
    page (runs of 1 to 16 slots at every offset), next to single decode tokens at every slot."""
    import torch
    rng = np.random.default_rng(7 * Hq + D)
    kinds, ql, cl = [], [], []
    for slot in range(16):
        kinds.append(DECODE); ql.append(1); cl.append(40 + slot)
    for _ in range(40):
        q = int(rng.integers(1, 70)); prior = int(rng.integers(0, 100))
        kinds.append(PREFILL); ql.append(q); cl.append(prior + q)
    b = synth.make_batch(Hq, Hkv, D, kinds, ql, cl, 95, name="append-runs")
    T = b.total_q
    k_new = synth.f32_to_bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    v_new = synth.f32_to_bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    step = hb.DeviceStep(b)
    hb.hfx_append_kv(step.shape, torch.from_numpy(k_new.view(np.int16)).cuda(), torch.from_numpy(v_new.view(np.int16)).cuda(),
                     step.pool, step.host_desc, step.device_desc, torch.cuda.current_stream())
    torch.cuda.synchronize()
    oracle.append_kv(Hkv, D, b.num_pages, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages, k_new, v_new, b.pool)
    assert np.array_equal(step.pool.cpu().numpy().view(np.uint16), b.pool), "pool after append must match bit for bit"


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 1, 64), (12, 12, 128)])
def test_copy_pages_is_bit_exact_and_attention_follows_the_pages(hb, oracle, Hq, Hkv, D):
    """A request's pages move to another pool (bit for bit, nothing else touched); attention through the
    destination pool and the new block table gives the very bits it gave through the source pool."""
    import torch
    rng = np.random.default_rng(31)
    b = synth.make_batch(Hq, Hkv, D, [DECODE, PREFILL, DECODE], [1, 70, 1], [333, 150, 17], seed=31,
                         name=f"copy-{Hq}-{Hkv}-{D}")
    shape = hb.make_shape(Hq, Hkv, D, b.num_pages, 0.0)
    src_ids = b.bt_pages.copy()                      # every page of every request
    n_dst = len(src_ids) + 9
    dst_ids = rng.permutation(n_dst)[:len(src_ids)].astype(np.int32)
    dst_np = synth.f32_to_bf16_bits(rng.standard_normal((n_dst,) + b.pool.shape[1:]).astype(np.float32))
    want = dst_np.copy()
    oracle.copy_pages(Hkv, D, src_ids, dst_ids, b.pool, want)
    src_dev = torch.from_numpy(b.pool.view(np.int16)).cuda()
    dst_dev = torch.from_numpy(dst_np.view(np.int16)).cuda()
    host_stage = torch.empty(8 * len(src_ids), dtype=torch.uint8, pin_memory=True)
    dev_stage = torch.empty(8 * len(src_ids), dtype=torch.uint8, device="cuda")
    hb.hfx_copy_pages(shape, src_dev, dst_dev, n_dst, src_ids, dst_ids, host_stage, dev_stage)
    hb.hfx_copy_pages(shape, src_dev, dst_dev, n_dst, [], [], host_stage, dev_stage)       # no-op
    torch.cuda.synchronize()
    assert np.array_equal(dst_dev.cpu().numpy().view(np.uint16), want)
    assert np.array_equal(src_dev.cpu().numpy().view(np.uint16), b.pool)

    # inside one pool: move the last request's pages onto unused ids
    used = set(b.bt_pages.tolist())
    free = np.array([p for p in range(b.num_pages) if p not in used], np.int32)
    r = 2
    mine = b.bt_pages[b.bt_indptr[r]:b.bt_indptr[r + 1]]
    if len(free) >= len(mine):
        want2 = b.pool.copy()
        oracle.copy_pages(Hkv, D, mine, free[:len(mine)], b.pool, want2)
        hb.hfx_copy_pages(shape, src_dev, src_dev, b.num_pages, mine, free[:len(mine)], host_stage, dev_stage)
        torch.cuda.synchronize()
        assert np.array_equal(src_dev.cpu().numpy().view(np.uint16), want2)

    # attention over the moved pages
    first = hb.DeviceStep(b).run()
    import copy
    b2 = copy.copy(b)
    b2.num_pages, b2.bt_pages, b2.pool = n_dst, dst_ids.copy(), want
    second = hb.DeviceStep(b2, pool_dev=dst_dev).run()
    torch.cuda.synchronize()
    assert torch.equal(first, second)



def test_device_side_errors(hb):
    import torch
    b = synth.config(1)
    step = hb.DeviceStep(b)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_build_batch_desc(step.shape, b.kind, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages, step.host_desc,
                                small, torch.cuda.current_stream())
    assert e.value.code == hb.HFX_ERR_BUFSIZE
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_gather_kv(step.shape, step.pool, step.host_desc, step.device_desc, 99, step.q, step.q)
    assert e.value.code == hb.HFX_ERR_LEN
    big = synth.config(4, 0.12)
    s2 = hb.DeviceStep(big)
    assert s2.workspace_bytes > 0
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_mixed_paged_attention(s2.shape, s2.q, s2.pool, s2.host_desc, s2.device_desc, small, s2.out)
    assert e.value.code == hb.HFX_ERR_BUFSIZE
