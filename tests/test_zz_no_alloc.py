"""The entry point that allocates nothing (tg_fingerprint_noalloc) against
tg_fingerprint, through the C ABI: two calls in a row on the same GPU, the
second with a smaller input, so that what the first call left in the fixed
scratch array would show if the second did not clear it."""
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2512_01357_amd import tangram as tg  # noqa: E402

DEV = "cuda:0"


def _spans(buf, lengths, gap=256):
    """Consecutive 256-byte-aligned extents of `buf` with the given lengths."""
    out, at = [], 0
    for n in lengths:
        out.append((buf.data_ptr() + at, n))
        at += (n + gap - 1) // gap * gap
    assert at <= buf.numel()
    return out


def test_noalloc_fingerprint_matches_the_allocating_entry_point_twice_in_a_row():
    print("[gpu-test] tg_fingerprint_noalloc: two calls, second smaller", flush=True)
    g = torch.Generator(device=DEV)
    g.manual_seed(20251201)
    buf = torch.randint(0, 256, (96 << 20,), dtype=torch.uint8, device=DEV, generator=g)
    # several tiles (a tile is 32 KiB), ragged tails, a one-byte and an empty extent
    first = [5 << 20, 1, 0, 32768, 32769, 1000003, 17, (3 << 20) + 5, 8, 40 << 20, 255, 4096] + [8192 + 16 * i for i in range(200)]
    second = [777, 2 << 20, 0, 65536 + 9]
    torch.cuda.synchronize()
    a_spans, b_spans = _spans(buf, first), _spans(buf, second)
    # the entry point under test goes first: run alone, this is the process's first call into
    # the library, so the array's address is looked up before any other kernel has run
    got_a = tg.tg_fingerprint_noalloc(a_spans)
    got_b = tg.tg_fingerprint_noalloc(b_spans)
    want_a = tg.tg_fingerprint(a_spans)
    want_b = tg.tg_fingerprint(b_spans)
    assert got_a == want_a
    assert got_b == want_b
    free_before, _ = torch.cuda.mem_get_info()
    assert tg.tg_fingerprint_noalloc(a_spans) == want_a
    assert tg.tg_fingerprint_noalloc(b_spans) == want_b
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before            # no device memory was taken
    # on a stream of the caller's, and once more: the array is reused call after call
    s = torch.cuda.Stream(device=DEV)
    assert tg.tg_fingerprint_noalloc(a_spans, s) == want_a
    assert tg.tg_fingerprint_noalloc(b_spans[:1], s) == want_b[:1]


def test_noalloc_fingerprint_rejects_what_does_not_fit():
    print("[gpu-test] tg_fingerprint_noalloc: limits", flush=True)
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device=DEV)
    too_many = [(buf.data_ptr(), 16)] * (tg.TG_NOALLOC_MAX_SPANS + 1)
    with pytest.raises(tg.TgError) as e:
        tg.tg_fingerprint_noalloc(too_many)
    assert e.value.status == tg.TG_ERR_INVALID
    with pytest.raises(tg.TgError) as e:
        tg.tg_fingerprint_noalloc([(buf.data_ptr() + 8, 64)])       # not 16-byte aligned
    assert e.value.status == tg.TG_ERR_INVALID
    # the maximum itself is accepted
    most = [(buf.data_ptr() + 256 * (i % 4096), 100 + i % 57) for i in range(tg.TG_NOALLOC_MAX_SPANS)]
    assert tg.tg_fingerprint_noalloc(most) == tg.tg_fingerprint(most)
    assert tg.tg_fingerprint_noalloc([]) == []
