"""Argument validation and page bookkeeping of the library, exercised on a bookkeeping-only handle
(device = H1BKV_DEVICE_NONE): no GPU is touched and no kernel is launched."""
import ctypes as C

import numpy as np
import pytest

from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl


def cfg(**kw):
    base = dict(n_q_heads=8, n_kv_heads=4, head_dim=128, sketch_bits=128, group_size=32, in_dtype=B.H1BKV_F16,
                page_tokens=0, max_seqs=4, max_pages=10, max_pages_per_seq=6, device=B.H1BKV_DEVICE_NONE)
    base.update(kw)
    return B.h1bkv_config(**base)


def make(**kw):
    c = cfg(**kw)
    R = wl.projection(c.sketch_bits, c.head_dim)
    rc, h = B.h1bkv_create(c, None, 0, R)
    assert rc == B.H1BKV_OK
    return c, h, R


@pytest.mark.parametrize("bad", [dict(n_q_heads=6), dict(head_dim=96), dict(sketch_bits=32), dict(sketch_bits=192),
                                 dict(group_size=16), dict(group_size=128, head_dim=64), dict(in_dtype=2),
                                 dict(page_tokens=128), dict(max_seqs=0), dict(max_pages=0), dict(max_pages_per_seq=0),
                                 dict(n_kv_heads=0), dict(device=-2)])
def test_bad_geometry_is_rejected(bad):
    c = cfg(**bad)
    assert B.h1bkv_pool_bytes(c) == 0
    rc, _ = B.h1bkv_create(c, None, 0, wl.projection(128, 128))
    assert rc == B.H1BKV_ESHAPE


def test_pool_bytes_formula():
    """sketch + nibbles + fp16 scale/zero per record (Sec. IV-B: a b-bit sketch and d 4-bit values per token),
    plus R, its transpose, its two fp16 pieces with the per-row guard bands (one for fp16, one for fp32 inputs), and the
    block table with 64 words behind it (the merge kernels' arrival counter), each rounded up to 256 bytes."""
    for w in (wl.WORKLOADS["tiny"], wl.WORKLOADS["decode_b16_32k"], wl.WORKLOADS["decode_gqa_128k"]):
        c = cfg(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                group_size=w.group_size, max_seqs=3, max_pages=7, max_pages_per_seq=5)
        al = lambda x: (x + 255) // 256 * 256
        rec = 7 * w.n_kv_heads * 256
        want = (2 * al(w.sketch_bits * w.head_dim * 4) + 2 * al(w.sketch_bits * w.head_dim * 2) + al(2 * w.sketch_bits * 4)
                + al((3 * 5 + 64) * 4) + al(rec * w.sketch_bits // 8)
                + al(rec * w.head_dim // 2) + al(rec * w.n_groups * 4))
        assert B.h1bkv_pool_bytes(c) == want
        assert (w.sketch_bits // 8 + w.head_dim // 2 + 4 * w.n_groups) == w.record_bytes


def test_create_null_arguments():
    c = cfg()
    assert B.lib().h1bkv_create(C.byref(c), None, 0, None, None) == B.H1BKV_ENULL       # nowhere to put the handle
    assert B.lib().h1bkv_create(None, None, 0, None, None) == B.H1BKV_ENULL
    # a real device handle needs a pool pointer
    rc, _ = B.h1bkv_create(cfg(device=0), None, 0, wl.projection(128, 128))
    assert rc == B.H1BKV_ENULL


def test_projection_round_trips():
    c, h, R = make()
    rc, back = B.h1bkv_get_projection(h, c.sketch_bits, c.head_dim)
    assert rc == B.H1BKV_OK and np.array_equal(back, R)
    B.h1bkv_destroy(h)


def test_append_bookkeeping_and_page_accounting():
    c, h, _ = make()
    S = (128 * 4, 128 * 4 * 300, 128)      # strides of a dense [n_seqs][300][4][128] tensor: seq, tok, head
    assert B.h1bkv_free_pages(h) == (0, 10)
    assert B.h1bkv_append_kv(h, [0, 2], 300, None, None, 300 * 512, 512, 128) == B.H1BKV_OK
    assert B.h1bkv_seq_len(h, 0) == (0, 300) and B.h1bkv_seq_len(h, 2) == (0, 300) and B.h1bkv_seq_len(h, 1) == (0, 0)
    assert B.h1bkv_free_pages(h) == (0, 6)               # two pages each
    assert B.h1bkv_append_kv(h, [0], 212, None, None, 0, 512, 128) == B.H1BKV_OK     # fills page 2 exactly
    assert B.h1bkv_seq_len(h, 0) == (0, 512) and B.h1bkv_free_pages(h) == (0, 6)
    assert B.h1bkv_append_kv(h, [0], 1, None, None, 0, 512, 128) == B.H1BKV_OK       # needs a third page
    assert B.h1bkv_free_pages(h) == (0, 5)
    # pool exhaustion leaves everything unchanged: 5 free pages, request needs 3 + 3
    assert B.h1bkv_append_kv(h, [1, 3], 700, None, None, 700 * 512, 512, 128) == B.H1BKV_ENOSPACE
    assert B.h1bkv_seq_len(h, 1) == (0, 0) and B.h1bkv_seq_len(h, 3) == (0, 0) and B.h1bkv_free_pages(h) == (0, 5)
    # per-sequence page cap: 6 pages = 1536 tokens
    assert B.h1bkv_append_kv(h, [2], 1536 - 300 + 1, None, None, 0, 512, 128) == B.H1BKV_ENOSPACE
    assert B.h1bkv_seq_len(h, 2) == (0, 300)
    # truncate / reset give pages back
    assert B.h1bkv_truncate_seq(h, 0, 513) == B.H1BKV_OK and B.h1bkv_free_pages(h) == (0, 5)
    assert B.h1bkv_truncate_seq(h, 0, 256) == B.H1BKV_OK and B.h1bkv_free_pages(h) == (0, 7)
    assert B.h1bkv_truncate_seq(h, 0, 257) == B.H1BKV_ERANGE and B.h1bkv_truncate_seq(h, 0, -1) == B.H1BKV_ERANGE
    assert B.h1bkv_reset_seq(h, 2) == B.H1BKV_OK and B.h1bkv_free_pages(h) == (0, 9)
    assert B.h1bkv_extend_seq(h, 3, 257, 0) == B.H1BKV_OK and B.h1bkv_seq_len(h, 3) == (0, 257)
    assert B.h1bkv_free_pages(h) == (0, 7)
    B.h1bkv_destroy(h)


def test_append_argument_errors():
    c, h, _ = make()
    ok = (512, 512, 128)
    assert B.lib().h1bkv_append_kv(h, None, 1, 1, None, None, *ok, None) == B.H1BKV_ENULL
    assert B.lib().h1bkv_append_kv(None, None, 1, 1, None, None, *ok, None) == B.H1BKV_ENULL
    assert B.h1bkv_append_kv(h, [4], 1, None, None, *ok) == B.H1BKV_ERANGE
    assert B.h1bkv_append_kv(h, [-1], 1, None, None, *ok) == B.H1BKV_ERANGE
    assert B.h1bkv_append_kv(h, [1, 1], 1, None, None, *ok) == B.H1BKV_EINVAL       # duplicate id
    assert B.h1bkv_append_kv(h, [1], 0, None, None, *ok) == B.H1BKV_EINVAL
    assert B.h1bkv_append_kv(h, [1], 1, None, None, 512, 512, 64) == B.H1BKV_EINVAL  # head stride < head_dim
    assert B.h1bkv_append_kv(h, [1], 1, None, None, -1, 512, 128) == B.H1BKV_EINVAL
    assert B.h1bkv_seq_len(h, 1) == (0, 0)
    assert B.h1bkv_seq_len(h, 9)[0] == B.H1BKV_ERANGE
    B.h1bkv_destroy(h)


def test_decode_argument_errors_and_workspace_size():
    c, h, _ = make()
    assert B.h1bkv_decode_attn(h, [0], None, 0.0, None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn(h, [0], None, -1.0, None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn(h, [0], None, float("nan"), None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn(h, [0], None, float("inf"), None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn(h, [7], None, 0.1, None, None, 0) == B.H1BKV_ERANGE
    assert B.h1bkv_decode_attn(h, [0, 0], None, 0.1, None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn(h, [0], None, 0.1, None, None, 0) == B.H1BKV_ENODEVICE   # valid, but no GPU behind it
    # workspace: query sketches + per-page partials, monotone
    al = lambda x: (x + 255) // 256 * 256
    heads = 3 * 8
    want = al(heads * 2 * 8) + al(heads * 5 * 2 * 4) + al(heads * 5 * 128 * 4)
    assert B.h1bkv_decode_workspace_bytes(h, 3, 1025) == want
    sizes = [B.h1bkv_decode_workspace_bytes(h, 3, t) for t in (0, 1, 256, 257, 5000)]
    assert sizes == sorted(sizes) and sizes[0] > 0
    assert B.h1bkv_decode_workspace_bytes(h, 0, 10) == 0
    B.h1bkv_destroy(h)


def test_misc_errors():
    c, h, _ = make()
    assert B.h1bkv_set_decode_chunk(h, 100) == B.H1BKV_EINVAL
    assert B.h1bkv_set_decode_chunk(h, 16384) == B.H1BKV_EINVAL
    assert B.h1bkv_set_decode_chunk(h, 512) == B.H1BKV_OK and B.h1bkv_set_decode_chunk(h, 0) == B.H1BKV_OK
    assert B.h1bkv_export_tokens(h, 0, 0, 0, 1, 2, 128, 4)[0] == B.H1BKV_ERANGE      # nothing cached yet
    assert B.h1bkv_append_kv(h, [0], 5, None, None, 0, 512, 128) == B.H1BKV_OK
    assert B.h1bkv_export_tokens(h, 0, 4, 0, 1, 2, 128, 4)[0] == B.H1BKV_ERANGE      # head out of range
    assert B.h1bkv_export_tokens(h, 0, 0, 3, 3, 2, 128, 4)[0] == B.H1BKV_ERANGE      # runs past the length
    assert B.h1bkv_export_tokens(h, 0, 0, 0, 5, 2, 128, 4)[0] == B.H1BKV_ENODEVICE
    assert B.h1bkv_profile_enable(h, 4, 0xF) == B.H1BKV_ENODEVICE and B.h1bkv_profile_enable(h, 0, 0) == B.H1BKV_OK
    assert B.h1bkv_stream_copy(None, None, 16) == B.H1BKV_ENULL
    assert B.h1bkv_stream_copy(4096, 8192, 24) == B.H1BKV_EINVAL
    assert B.h1bkv_stream_read(None, 16, None) == B.H1BKV_ENULL
    assert B.h1bkv_stream_read(4096, 24, 8192) == B.H1BKV_EINVAL
    assert B.h1bkv_stream_read_ms(None, 16, None)[0] == B.H1BKV_ENULL
    assert B.h1bkv_stream_read_ms(4096, 0, 8192)[0] == B.H1BKV_EINVAL          # nothing to time
    assert B.h1bkv_stream_read_ms(4096, 24, 8192) == (B.H1BKV_EINVAL, 0.0)
    assert B.h1bkv_destroy(h) == B.H1BKV_OK and B.h1bkv_destroy(None) == B.H1BKV_OK


def test_decode_step_validates_both_halves_before_changing_anything():
    c, h, _ = make()
    assert B.h1bkv_append_kv(h, [0, 1], 10, None, None, 10 * 512, 512, 128) == B.H1BKV_OK
    free = B.h1bkv_free_pages(h)
    args = dict(stride_seq=512, stride_head=128)
    # bad decode arguments are reported although the append half would be fine, and nothing is appended
    assert B.h1bkv_decode_step(h, [0, 1], None, None, 512, 128, None, 0.0, None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_step(h, [0, 0], None, None, 512, 128, None, 0.1, None, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_step(h, [0, 5], None, None, 512, 128, None, 0.1, None, None, 0) == B.H1BKV_ERANGE
    # a bookkeeping-only handle cannot decode: the step is refused as a whole
    assert B.h1bkv_decode_step(h, [0, 1], None, None, 512, 128, None, 0.1, None, None, 0) == B.H1BKV_ENODEVICE
    assert B.h1bkv_seq_len(h, 0) == (0, 10) and B.h1bkv_seq_len(h, 1) == (0, 10) and B.h1bkv_free_pages(h) == free
    assert B.lib().h1bkv_decode_step(None, None, 1, None, None, 512, 128, None, 0.1, None, None, 0, None) == B.H1BKV_ENULL
    B.h1bkv_destroy(h)


def test_value_bits_configuration():
    """The fp16-value variant replaces the code and scale/zero planes (d/2 + 4 n_g bytes per record) by 2d bytes."""
    c4, c16, cbad = cfg(), cfg(value_bits=16), cfg(value_bits=8)
    assert B.h1bkv_pool_bytes(cbad) == 0
    assert B.h1bkv_pool_bytes(cfg(value_bits=0)) == B.h1bkv_pool_bytes(cfg(value_bits=4)) == B.h1bkv_pool_bytes(c4)
    rec = c4.max_pages * c4.n_kv_heads * 256
    d, ng = c4.head_dim, c4.head_dim // c4.group_size
    diff = B.h1bkv_pool_bytes(c16) - B.h1bkv_pool_bytes(c4)
    assert abs(diff - rec * (2 * d - d // 2 - 4 * ng)) <= 512       # plane starts are 256-byte aligned


def test_prefill_workspace_size():
    """Query sketches of the chunk, plus per-row partial results of up to 16 context splits when the chunk alone brings
    too few workgroups to fill the chip once: fewer than 512 of heads x sequences x blocks of 128 positions,
    or, from 256 positions per chunk on, fewer than 256 of ... x blocks of 256 positions."""
    c, h, _ = make()                      # 8 query heads, d = 128, b = 128 (2 words)
    al = lambda x: (x + 255) // 256 * 256

    def want(n_seqs, n_q):
        rows = n_seqs * n_q * 8
        block, fill = (256, 256) if n_q >= 256 else (128, 512)
        wgs = 8 * n_seqs * ((n_q + block - 1) // block)
        splits = min(16, max(1, -(-fill // wgs)))
        return al(rows * 2 * 8) + (al(rows * splits * (128 + 2) * 4) if splits > 1 else 0)

    for n_seqs, n_q in [(1, 1), (1, 128), (1, 255), (1, 256), (3, 300), (1, 511), (1, 512), (2, 600), (2, 1000), (2, 1024), (1, 3000), (4, 4096), (4, 8192), (3, 129)]:
        assert B.h1bkv_prefill_workspace_bytes(h, n_seqs, n_q) == want(n_seqs, n_q), (n_seqs, n_q)
    assert want(4, 8192) == al(4 * 8192 * 8 * 16)       # a long prompt: one split, sketches only
    assert B.h1bkv_prefill_workspace_bytes(h, 0, 5) == 0 and B.h1bkv_prefill_workspace_bytes(h, 2, 0) == 0
    B.h1bkv_destroy(h)


def splitmix_box_muller(seed, n):
    """The draw h1bkv_create documents for R_host == NULL, written out with Python integers and numpy doubles."""
    mask = (1 << 64) - 1
    state = seed & mask
    out = np.empty(n, dtype=np.float64)

    def uniform():
        nonlocal state
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        z ^= z >> 31
        return ((z >> 11) + 0.5) * 2.0 ** -53

    for e in range(0, n, 2):
        u1, u2 = uniform(), uniform()
        rad, ang = np.sqrt(-2.0 * np.log(u1)), 2.0 * np.pi * u2
        out[e], out[e + 1] = rad * np.cos(ang), rad * np.sin(ang)
    return out


def test_projection_drawn_from_the_seed():
    """Sec. III: R_ij ~ N(0,1), drawn once.  Without a caller-supplied R the library draws it from cfg.seed with the
    documented generator; the same seed gives the same matrix, another seed another one, and the entries look Gaussian."""
    c = cfg(seed=0x1234ABCD5678EF01, sketch_bits=256)
    rc, h = B.h1bkv_create(c, None, 0, None)
    assert rc == B.H1BKV_OK
    rc, R1 = B.h1bkv_get_projection(h, 256, 128)
    assert rc == B.H1BKV_OK
    want = splitmix_box_muller(0x1234ABCD5678EF01, 256 * 128).reshape(256, 128)
    # libm may differ in the last place of log / cos / sin between this process's numpy and the library's host code
    assert np.allclose(R1, want.astype(np.float32), rtol=3e-7, atol=1e-9)
    rc, h2 = B.h1bkv_create(c, None, 0, None)
    assert np.array_equal(B.h1bkv_get_projection(h2, 256, 128)[1], R1)
    rc, h3 = B.h1bkv_create(cfg(seed=7, sketch_bits=256), None, 0, None)
    R3 = B.h1bkv_get_projection(h3, 256, 128)[1]
    assert not np.array_equal(R3, R1) and abs(np.corrcoef(R3.ravel(), R1.ravel())[0, 1]) < 0.03
    n = R1.size
    assert abs(R1.mean()) < 4 / np.sqrt(n) and abs(R1.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs((R1 ** 4).mean() - 3) < 0.25 and abs(np.mean(np.abs(R1) < 1) - 0.6827) < 0.01
    # neighbouring elements (the cos and sin of one pair) and rows are uncorrelated
    assert abs(np.corrcoef(R1[:, 0::2].ravel(), R1[:, 1::2].ravel())[0, 1]) < 0.03
    for x in (h, h2, h3):
        B.h1bkv_destroy(x)


def test_failed_launch_leaves_the_bookkeeping_unchanged():
    """An erroring call changes neither lengths nor page assignments: force the n-th launch attempt of a call to fail and
    compare the bookkeeping before and after, for every launch position of append and extend."""
    c, h, _ = make(max_pages=600, max_pages_per_seq=130)

    def state():
        return [B.h1bkv_seq_len(h, s)[1] for s in range(4)], B.h1bkv_free_pages(h)[1]

    assert B.h1bkv_append_kv(h, [0, 1], 300, None, None, 300 * 512, 512, 128) == B.H1BKV_OK
    before = state()
    # [0,1,3] x 700 tokens: 2 + 2 + 3 new pages -> one block-table launch + one append launch
    for nth, want in ((1, B.H1BKV_EHIP), (2, B.H1BKV_EHIP), (3, B.H1BKV_OK)):
        assert B.h1bkv_debug_fail_launch(h, nth) == B.H1BKV_OK
        rc = B.h1bkv_append_kv(h, [0, 1, 3], 700, None, None, 700 * 512, 512, 128)
        assert rc == want, (nth, rc)
        if rc != B.H1BKV_OK:
            assert state() == before, nth
    assert state() == ([1000, 1000, 0, 700], before[1] - 7)
    assert B.h1bkv_debug_fail_launch(h, 0) == B.H1BKV_OK
    # a long extension needs more block-table updates than one launch carries (240): the second launch fails
    before = state()
    assert B.h1bkv_debug_fail_launch(h, 2) == B.H1BKV_OK
    assert B.h1bkv_extend_seq(h, 2, 250 * 256 - 1, 0) == B.H1BKV_ENOSPACE        # beyond 130 pages: refused up front
    assert B.h1bkv_extend_seq(h, 2, 130 * 256, 0) == B.H1BKV_OK and state() != before   # 130 pages = one launch: attempt 1 passes
    assert B.h1bkv_reset_seq(h, 2) == B.H1BKV_OK and state() == before
    assert B.h1bkv_debug_fail_launch(h, 1) == B.H1BKV_OK
    assert B.h1bkv_extend_seq(h, 2, 1000, 0) == B.H1BKV_EHIP and state() == before
    # after the failure the same pages are handed out in the same order: a repeat succeeds and matches a fresh handle
    assert B.h1bkv_extend_seq(h, 2, 1000, 0) == B.H1BKV_OK and state() == ([1000, 1000, 1000, 700], before[1] - 4)
    assert B.h1bkv_debug_fail_launch(h, -1) == B.H1BKV_EINVAL and B.h1bkv_debug_fail_launch(None, 1) == B.H1BKV_ENULL
    B.h1bkv_destroy(h)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """h1bkv_decode_attn_static keeps sketches and per-chunk partials in a fixed array: a call that needs more is
    refused on the host (before the question of a device even arises); a call that fits is only missing a GPU here."""
    c, h, _ = make(n_q_heads=64, n_kv_heads=8, max_seqs=64, max_pages=64 * 9, max_pages_per_seq=9)
    for s in range(64):
        assert B.h1bkv_extend_seq(h, s, 2304, 0) == B.H1BKV_OK
    assert B.h1bkv_set_decode_chunk(h, 256) == B.H1BKV_OK          # 9 partials per head: 64 x 64 x 9 x (128 + 2) floats
    assert B.h1bkv_decode_attn_static(h, list(range(64)), None, 0.1, None, 0) == B.H1BKV_EWORKSPACE
    assert B.h1bkv_decode_attn_static(h, list(range(8)), None, 0.1, None, 0) == B.H1BKV_ENODEVICE
    assert B.h1bkv_decode_attn_static(h, [0, 0], None, 0.1, None, 0) == B.H1BKV_EINVAL
    assert B.h1bkv_decode_attn_static(h, [0], None, -0.1, None, 0) == B.H1BKV_EINVAL
    assert B.lib().h1bkv_decode_attn_static(None, None, 1, None, 0.1, None, None) == B.H1BKV_ENULL
    B.h1bkv_destroy(h)


def test_reserved_pages_and_device_position_step_bookkeeping():
    """h1bkv_reserve_seq takes pages without changing the length; appends use them up before taking new ones;
    h1bkv_set_seq_len moves the length only inside the reservation; truncating gives reserved pages back; the
    device-position step insists on pages for every position it may touch.  (Bookkeeping-only handle: nothing launches.)"""
    c, h, _ = make(max_pages=10, max_pages_per_seq=6)
    free = lambda: B.h1bkv_free_pages(h)[1]
    length = lambda s: B.h1bkv_seq_len(h, s)[1]
    assert B.h1bkv_append_kv(h, [0], 100, None, None, 100 * 512, 512, 128) == B.H1BKV_OK
    assert (length(0), free(), B.h1bkv_reserved_tokens(h, 0)[1]) == (100, 9, 256)
    assert B.h1bkv_reserve_seq(h, 0, 0) == B.H1BKV_OK and free() == 9                   # nothing to take
    assert B.h1bkv_reserve_seq(h, 0, 156) == B.H1BKV_OK and free() == 9                 # still inside the first page
    assert B.h1bkv_reserve_seq(h, 0, 157) == B.H1BKV_OK and free() == 8                 # position 256 needs a second one
    assert B.h1bkv_reserve_seq(h, 0, 600) == B.H1BKV_OK and (length(0), free()) == (100, 7)
    assert B.h1bkv_reserved_tokens(h, 0)[1] == 768
    assert B.h1bkv_reserve_seq(h, 0, 6 * 256 - 100 + 1) == B.H1BKV_ENOSPACE and free() == 7   # beyond the per-sequence limit
    assert B.h1bkv_reserve_seq(h, 0, -1) == B.H1BKV_EINVAL and B.h1bkv_reserve_seq(h, 9, 1) == B.H1BKV_ERANGE
    # an append inside the reservation takes no page, one that outgrows it takes the difference
    assert B.h1bkv_append_kv(h, [0], 500, None, None, 500 * 512, 512, 128) == B.H1BKV_OK and (length(0), free()) == (600, 7)
    assert B.h1bkv_append_kv(h, [0], 300, None, None, 300 * 512, 512, 128) == B.H1BKV_OK and (length(0), free()) == (900, 6)
    # lengths move forward inside the reservation only
    assert B.h1bkv_reserve_seq(h, 0, 300) == B.H1BKV_OK and free() == 5
    assert B.h1bkv_set_seq_len(h, 0, 899) == B.H1BKV_ERANGE                              # backwards is truncate's job
    assert B.h1bkv_set_seq_len(h, 0, 1281) == B.H1BKV_ERANGE                             # five pages hold 1280 tokens
    assert B.h1bkv_set_seq_len(h, 0, 1000) == B.H1BKV_OK and (length(0), free()) == (1000, 5)
    # truncating to the length that is cached drops what was reserved beyond it
    assert B.h1bkv_truncate_seq(h, 0, 1000) == B.H1BKV_OK and free() == 6
    # a forced launch failure while publishing reserved pages leaves everything as it was
    assert B.h1bkv_debug_fail_launch(h, 1) == B.H1BKV_OK
    assert B.h1bkv_reserve_seq(h, 1, 300) == B.H1BKV_EHIP and (length(1), free(), B.h1bkv_reserved_tokens(h, 1)[1]) == (0, 6, 0)
    assert B.h1bkv_debug_fail_launch(h, 0) == B.H1BKV_OK
    # the device-position step: argument checks that need no device
    step = lambda seqs, max_pos, tau=0.1, advance=1: B.h1bkv_decode_step_dev(h, seqs, None, None, 512, 128, None, tau, None, None,
                                                                             max_pos, None, 0, advance=advance)
    assert step([0], 1025) == B.H1BKV_ERANGE             # sequence 0 holds four pages
    assert step([0], 0) == B.H1BKV_EINVAL and step([0], 100, tau=0.0) == B.H1BKV_EINVAL
    assert step([0], 100, advance=2) == B.H1BKV_EINVAL and step([0], 1024, advance=0) == B.H1BKV_ENODEVICE
    assert step([0, 0], 100) == B.H1BKV_EINVAL and step([7], 100) == B.H1BKV_ERANGE
    assert step([0], 1024) == B.H1BKV_ENODEVICE          # everything else is in order: only the device is missing
    B.h1bkv_destroy(h)
