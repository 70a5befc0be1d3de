"""The entry point that allocates nothing (hfx_mixed_paged_attention_static) against the entry point
it is a variant of, through the C ABI: the same bits, on two calls in a row of which the second is the
smaller step, so that the shared fixed workspace still holds the first call's partials."""
import numpy as np
import pytest

from paper_2508_15919_amd import synth

pytestmark = pytest.mark.gpu


def both_ways(hb, torch, b):
    step = hb.DeviceStep(b)
    assert step.workspace_bytes > 0, "the step must have split partials, or the workspace is not exercised"
    nan = torch.full_like(step.out, 0x7FC0)
    step.out.copy_(nan)
    step.run()
    want = step.out_bits().copy()
    step.out.copy_(nan)
    hb.hfx_mixed_paged_attention_static(step.shape, step.q, step.pool, step.host_desc, step.device_desc, step.out,
                                        torch.cuda.current_stream())
    got = step.out_bits()
    assert np.isfinite(synth.bf16_bits_to_f64(want)).all()
    assert np.array_equal(got, want), b.name
    return step


def test_static_workspace_entry_matches_on_two_calls_in_a_row():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2508_15919_amd import binding as hb
    hb.load()
    big = synth.config(2)                       # 18.7 MB of split partials: decode splits and prefill splits
    small = synth.config(4, 0.12)               # a smaller step, other split shapes, same workspace
    s1 = both_ways(hb, torch, big)
    s2 = both_ways(hb, torch, small)
    assert s2.workspace_bytes < s1.workspace_bytes
    # a step that does not fit the fixed workspace (64 MiB) is refused before anything is enqueued
    huge = synth.config(5, fill_pool=False)     # the long-context share: 72 MB of split partials
    shape = hb.make_shape(huge.num_q_heads, huge.num_kv_heads, huge.head_dim, huge.num_pages)
    hbytes, dbytes, wbytes = hb.hfx_batch_desc_sizes(shape, huge.kind, huge.q_len, huge.ctx_len)
    assert wbytes > (64 << 20), wbytes
    host = np.zeros(hbytes, np.uint8)
    hb.hfx_fill_batch_desc(shape, huge.kind, huge.q_len, huge.ctx_len, huge.bt_indptr, huge.bt_pages, host)
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_mixed_paged_attention_static(shape, s1.q, s1.pool, host, s1.device_desc, s1.out)
    assert e.value.code == hb.HFX_ERR_BUFSIZE
