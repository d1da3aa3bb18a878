"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every symbol
the header declares, and rejects bad arguments with the documented status before any launch."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2604_15408_amd import binding

ROOT = Path(__file__).resolve().parents[1]
FAKE = 0x10000          # non-null, 16-byte aligned; never dereferenced because validation fails first


@pytest.fixture(scope="module")
def lib():
    if not binding.LIB_PATH.exists():
        from paper_2604_15408_amd import build
        build.build()
    return binding.load()


def declared_functions():
    text = (ROOT / "include" / "ragged.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ragged_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_status_strings(lib):
    assert binding.version() >= 700
    assert binding.status_string(0) == "ok"
    texts = {binding.status_string(s) for s in range(6)}
    assert len(texts) == 6 and binding.status_string(99) == "unknown"


def _pack(lib, x=FAKE, keep=FAKE, B=2, N=8, C=64, dt=0, packed=FAKE, cap=16, cu=FAKE, gi=FAKE):
    return lib.ragged_pack(x, keep, B, N, C, dt, packed, cap, cu, gi, None)


def _attn(lib, q=FAKE, k=FAKE, v=FAKE, o=FAKE, cu=FAKE, B=2, ms=8, H=2, D=64, scale=0.125, i=0, od=0):
    return lib.ragged_attn(q, k, v, o, cu, B, ms, H, D, scale, i, od, None)


def _unpack(lib, src=FAKE, keep=FAKE, cu=FAKE, gi=FAKE, B=2, N=8, C=64, dt=0, out=FAKE, fm=0):
    return lib.ragged_unpack(src, keep, cu, gi, B, N, C, dt, out, fm, None)


def test_pack_validation(lib):
    for null in ("x", "keep", "packed", "cu", "gi"):
        assert _pack(lib, **{null: None}) == 1
    for bad in (dict(B=0), dict(N=-1), dict(C=0), dict(B=1 << 20, N=1 << 20)):
        assert _pack(lib, **bad) == 2
    for bad in (dict(dt=2), dict(dt=7), dict(C=12), dict(x=FAKE + 2), dict(packed=FAKE + 8)):
        assert _pack(lib, **bad) == 3
    assert _pack(lib, cap=0) == 4


def test_attn_validation(lib):
    for null in ("q", "k", "v", "o", "cu"):
        assert _attn(lib, **{null: None}) == 1
    for bad in (dict(B=0), dict(H=0), dict(D=0), dict(ms=0), dict(B=1 << 30, H=64)):
        assert _attn(lib, **bad) == 2
    # grid limits: 65535 q-tiles of 64 rows, 65535 dispatch batches of 512 (image, head) pairs, < 2^31 work-groups
    for bad in (dict(B=1, H=1, ms=64 * 65535 + 1), dict(B=512 * 65535 + 1, H=1, ms=8), dict(B=1 << 16, H=16, ms=1 << 17)):
        assert _attn(lib, **bad) == 2
    for bad in (dict(D=48), dict(i=2), dict(i=0, od=1), dict(i=1, od=0), dict(scale=float("inf")),
                dict(scale=float("nan")), dict(q=FAKE + 4), dict(o=FAKE + 8)):
        assert _attn(lib, **bad) == 3


def test_unpack_validation(lib):
    assert _unpack(lib, fm=2) == 3
    for null in ("src", "cu", "out"):
        assert _unpack(lib, **{null: None}) == 1
    assert _unpack(lib, gi=None, fm=0) == 1 and _unpack(lib, keep=None, fm=1) == 1
    for bad in (dict(B=0), dict(N=0), dict(C=-8)):
        assert _unpack(lib, **bad) == 2
    for bad in (dict(dt=2), dict(C=20), dict(src=FAKE + 1), dict(out=FAKE + 2)):
        assert _unpack(lib, **bad) == 3


def test_attn_padded_validation(lib):
    def call(q=FAKE, k=FAKE, v=FAKE, o=FAKE, keep=FAKE, B=2, N=8, H=2, D=64, scale=0.125, i=0, od=0, fm=0):
        return lib.ragged_attn_padded(q, k, v, o, keep, B, N, H, D, scale, i, od, fm, None)
    for null in ("q", "k", "v", "o", "keep"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(N=0), dict(H=-1), dict(D=0), dict(B=1 << 20, N=1 << 20)):
        assert call(**bad) == 2
    for bad in (dict(D=32), dict(N=1537), dict(fm=2), dict(i=1, od=0), dict(scale=float("nan")), dict(v=FAKE + 8)):
        assert call(**bad) == 3


def test_attn_strided_validation(lib):
    def call(q=FAKE, k=FAKE, v=FAKE, o=FAKE, cu=FAKE, B=2, ms=8, H=2, D=64, si=384, so=128, scale=0.125, i=0, od=0):
        return lib.ragged_attn_strided(q, k, v, o, cu, B, ms, H, D, si, so, scale, i, od, None)
    for null in ("q", "k", "v", "o", "cu"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(ms=0), dict(si=127), dict(so=64), dict(si=-384), dict(si=(1 << 23) + 8),
                dict(so=1 << 31)):
        assert call(**bad) == 2
    for bad in (dict(D=32), dict(si=132), dict(so=132), dict(i=0, od=1), dict(scale=float("inf")), dict(k=FAKE + 2)):
        assert call(**bad) == 3


def test_attn_checked_validation(lib):
    def call(q=FAKE, k=FAKE, v=FAKE, o=FAKE, cu=FAKE, B=2, ms=8, H=2, D=64, si=128, so=128, scale=0.125, i=0, od=0,
             flags=FAKE):
        return lib.ragged_attn_checked(q, k, v, o, cu, B, ms, H, D, si, so, scale, i, od, flags, None)
    for null in ("q", "k", "v", "o", "cu", "flags"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(ms=0), dict(si=64)):
        assert call(**bad) == 2
    for bad in (dict(D=32), dict(flags=FAKE + 2), dict(i=0, od=1), dict(scale=float("nan"))):
        assert call(**bad) == 3


def test_repack_validation(lib):
    def call(src=FAKE, kr=FAKE, cu=FAKE, B=2, cap_in=16, C=64, dt=0, dst=FAKE, cap_out=16, cuo=FAKE, gi=FAKE):
        return lib.ragged_repack(src, kr, cu, B, cap_in, C, dt, dst, cap_out, cuo, gi, None)
    for null in ("src", "kr", "cu", "dst", "cuo", "gi"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(C=0), dict(cap_in=1 << 31)):
        assert call(**bad) == 2
    for bad in (dict(dt=2), dict(C=12), dict(src=FAKE + 4), dict(dst=FAKE + 8)):
        assert call(**bad) == 3
    assert call(cap_in=0) == 4 and call(cap_out=0) == 4


def test_cls_extract_validation(lib):
    def call(src=FAKE, cu=FAKE, B=2, C=64, dt=0, out=FAKE):
        return lib.ragged_cls_extract(src, cu, B, C, dt, out, None)
    for null in ("src", "cu", "out"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(C=-8)):
        assert call(**bad) == 2
    for bad in (dict(dt=2), dict(C=20), dict(src=FAKE + 2), dict(out=FAKE + 8)):
        assert call(**bad) == 3


def test_pack_attn_unpack_validation(lib):
    def call(x=FAKE, keep=FAKE, q=FAKE, k=FAKE, v=FAKE, B=2, N=8, H=2, D=64, scale=0.125, dt=0, packed=FAKE, cap=16,
             cu=FAKE, gi=FAKE, o=FAKE, out=FAKE, fm=0):
        return lib.ragged_pack_attn_unpack(x, keep, q, k, v, B, N, H, D, scale, dt, packed, cap, cu, gi, o, out, fm, None)
    for null in ("x", "keep", "q", "k", "v", "packed", "cu", "gi", "o", "out"):
        assert call(**{null: None}) == 1
    for bad in (dict(B=0), dict(N=0), dict(H=0), dict(D=-1), dict(B=1 << 20, N=1 << 20)):
        assert call(**bad) == 2
    for bad in (dict(D=32), dict(N=1537, cap=1 << 20), dict(dt=2), dict(fm=3), dict(scale=float("nan")),
                dict(x=FAKE + 2), dict(out=FAKE + 8)):
        assert call(**bad) == 3
    assert call(cap=15) == 4


def test_linear_validation(lib):
    def call(x=FAKE, w=FAKE, b=FAKE, r=None, y=FAKE, rows=16, rd=None, hint=0, N=128, K=64, act=0, dt=0):
        return lib.ragged_linear(x, w, b, r, y, rows, rd, hint, N, K, act, dt, None)
    for null in ("x", "w", "y"):
        assert call(**{null: None}) == 1
    for bad in (dict(rows=0), dict(N=0), dict(K=-64), dict(K=(1 << 22) + 64), dict(rows=1 << 31),
                dict(hint=-1), dict(hint=17)):
        assert call(**bad) == 2
    for bad in (dict(N=160), dict(K=96), dict(act=2), dict(dt=2), dict(x=FAKE + 2), dict(b=FAKE + 8), dict(r=FAKE + 4)):
        assert call(**bad) == 3


def test_layernorm_validation(lib):
    def call(x=FAKE, g=FAKE, b=FAKE, y=FAKE, rows=16, rd=None, C=768, eps=1e-6, dt=0):
        return lib.ragged_layernorm(x, g, b, y, rows, rd, C, eps, dt, None)
    for null in ("x", "g", "b", "y"):
        assert call(**{null: None}) == 1
    for bad in (dict(rows=0), dict(C=0)):
        assert call(**bad) == 2
    for bad in (dict(C=100), dict(C=4096), dict(eps=-1.0), dict(eps=float("nan")), dict(dt=2), dict(y=FAKE + 8)):
        assert call(**bad) == 3


def test_mask_producer_validation(lib):
    assert lib.ragged_token_scores_l2(None, 8, 64, 0, FAKE, None) == 1
    assert lib.ragged_token_scores_l2(FAKE, 8, 64, 0, None, None) == 1
    assert lib.ragged_token_scores_l2(FAKE, 0, 64, 0, FAKE, None) == 2
    assert lib.ragged_token_scores_l2(FAKE, 8, 0, 0, FAKE, None) == 2
    for bad in ((8, 12, 0, FAKE), (8, 64, 2, FAKE), (8, 64, 0, FAKE + 4)):
        assert lib.ragged_token_scores_l2(FAKE, bad[0], bad[1], bad[2], bad[3], None) == 3
    assert lib.ragged_token_scores_l2(FAKE + 8, 8, 64, 0, FAKE, None) == 3
    assert lib.ragged_keep_topk(None, 2, 8, 3, FAKE, None) == 1 and lib.ragged_keep_topk(FAKE, 2, 8, 3, None, None) == 1
    for bad in ((0, 8, 3), (2, 0, 3), (2, 8, 0), (1 << 20, 1 << 20, 3)):
        assert lib.ragged_keep_topk(FAKE, bad[0], bad[1], bad[2], FAKE, None) == 2
    assert lib.ragged_keep_topk(FAKE, 2, 1537, 3, FAKE, None) == 3
    assert lib.ragged_keep_topk(FAKE + 4, 2, 8, 3, FAKE, None) == 3


def test_noop_validation(lib):
    assert lib.ragged_noop(0, None) == 2


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 4, 64, dtype=torch.float16)
    with pytest.raises(TypeError):
        binding.ragged_pack(x, torch.ones(1, 4, dtype=torch.uint8), torch.zeros(4, 64, dtype=torch.float16),
                            torch.zeros(2, dtype=torch.int32), torch.zeros(4, dtype=torch.int32), stream=0)
