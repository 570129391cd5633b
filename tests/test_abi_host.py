"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, agrees with the header on the struct layout, and decides every error / no-op case before any launch."""
import ctypes
import os
import re
import subprocess
import tempfile

import pytest

from paper_2410_01518_amd import infinipot as ip

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "infinipot.h")


def _declared():
    src = open(HEADER).read()
    return re.findall(r"CCD_API\s+[\w\s\*]+?\b(ccd_\w+)\s*\(", src)


def test_header_symbols_are_exported():
    names = _declared()
    assert set(names) == set(ip.EXPORTS) and len(names) == len(ip.EXPORTS)
    L = ip.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_struct_layout_matches_header():
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "infinipot.h"
int main(void){ printf("%zu %zu %zu %zu %zu %zu\n", sizeof(ccd_shape_t), offsetof(ccd_shape_t, scale),
  offsetof(ccd_shape_t, kv_stride_b), offsetof(ccd_shape_t, q_stride_h), offsetof(ccd_shape_t, nov_stride_h),
  offsetof(ccd_shape_t, window));
  printf("%d %d %d %d %d %d %d\n", CCD_OK, CCD_NOOP, CCD_EINVAL, CCD_EUNSUPPORTED, CCD_EALIGN, CCD_EWORKSPACE, CCD_ELAUNCH);
  return 0; }'''
    with tempfile.TemporaryDirectory() as td:
        c = os.path.join(td, "t.c"); exe = os.path.join(td, "t")
        open(c, "w").write(prog)
        subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe], check=True)
        out = subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split()
    vals = [int(v) for v in out]
    S = ip.ccd_shape_t
    assert vals[:6] == [ctypes.sizeof(S), S.scale.offset, S.kv_stride_b.offset, S.q_stride_h.offset, S.nov_stride_h.offset,
                        S.window.offset]
    assert vals[6:] == [ip.CCD_OK, ip.CCD_NOOP, ip.CCD_EINVAL, ip.CCD_EUNSUPPORTED, ip.CCD_EALIGN, ip.CCD_EWORKSPACE,
                        ip.CCD_ELAUNCH]


def _shape(**kw):
    s = ip.ccd_shape_t()
    base = dict(B=1, L=2, Hq=8, Hkv=2, d=128, n_valid=512, n_cap=512, k=256, P=16, T=128, pool_w=7,
                pool_mode=ip.CCD_POOL_MAX, dtype=ip.CCD_BF16, scale=0.0)
    base.update(kw)
    for k_, v in base.items():
        setattr(s, k_, v)
    d, n_cap = s.d, s.n_cap
    s.kv_stride_h = kw.get("kv_stride_h", n_cap * d); s.kv_stride_l = kw.get("kv_stride_l", s.Hkv * n_cap * d)
    s.kv_stride_b = kw.get("kv_stride_b", s.L * s.Hkv * n_cap * d)
    s.q_stride_h = kw.get("q_stride_h", s.P * d); s.q_stride_l = kw.get("q_stride_l", max(s.Hq, 1) * s.P * d)
    s.q_stride_b = kw.get("q_stride_b", s.L * max(s.Hq, 1) * s.P * d)
    s.nov_stride_b = kw.get("nov_stride_b", s.n_valid)
    s.nov_stride_l = kw.get("nov_stride_l", 0); s.nov_stride_h = kw.get("nov_stride_h", 0)
    return s


P = 0x1000  # a fake, aligned, non-null device address: never dereferenced because every case below fails on the host


def _compress(s, Q=P, K=P, V=P, nov=P, scores=None, keep=P, ws=0x10000, ws_bytes=None):
    nbytes = ip.ccd_workspace_bytes(s) if ws_bytes is None else ws_bytes
    return ip.lib().ccd_compress(ctypes.byref(s), Q, K, V, nov, scores, keep, ws, nbytes, None)


def test_workspace_bytes():
    s = _shape()
    n = ip.ccd_workspace_bytes(s)
    assert n > 0 and n % 256 == 0
    assert ip.ccd_workspace_bytes(_shape(k=0)) == 0
    assert ip.lib().ccd_workspace_bytes(None) == 0
    assert ip.ccd_workspace_bytes(_shape(n_valid=1024, n_cap=1024)) > n


@pytest.mark.parametrize("kw,code", [
    (dict(k=0), ip.CCD_EINVAL), (dict(k=513), ip.CCD_EINVAL), (dict(T=257), ip.CCD_EINVAL), (dict(T=-1), ip.CCD_EINVAL),
    (dict(Hq=7), ip.CCD_EINVAL), (dict(B=0), ip.CCD_EINVAL), (dict(P=0), ip.CCD_EINVAL),
    (dict(pool_w=4), ip.CCD_EINVAL), (dict(pool_w=0), ip.CCD_EINVAL), (dict(n_valid=600), ip.CCD_EINVAL),
    (dict(scale=-1.0), ip.CCD_EINVAL), (dict(scale=float("nan")), ip.CCD_EINVAL),
    (dict(kv_stride_h=100), ip.CCD_EINVAL), (dict(q_stride_h=8), ip.CCD_EINVAL),
    (dict(d=96), ip.CCD_EUNSUPPORTED), (dict(dtype=3), ip.CCD_EUNSUPPORTED), (dict(pool_mode=5), ip.CCD_EUNSUPPORTED),
    (dict(kv_stride_l=2 * 512 * 128 + 4), ip.CCD_EALIGN), (dict(q_stride_b=2 * 8 * 16 * 128 + 2), ip.CCD_EALIGN),
])
def test_bad_shapes_are_rejected_on_the_host(kw, code):
    s = _shape(**kw)
    assert ip.lib().ccd_compress(ctypes.byref(s), P, P, P, P, None, P, 0x10000, 1 << 40, None) == code
    assert ip.lib().ccd_score(ctypes.byref(s), P, P, P, P, 0x10000, 1 << 40, None) == code


def test_null_misaligned_and_workspace_errors():
    s = _shape()
    assert _compress(s, Q=None) == ip.CCD_EINVAL
    assert _compress(s, K=None) == ip.CCD_EINVAL
    assert _compress(s, V=None) == ip.CCD_EINVAL
    assert _compress(s, keep=None) == ip.CCD_EINVAL
    assert _compress(s, nov=None) == ip.CCD_EINVAL           # T > 0 needs novelty
    assert _compress(s, K=P + 8) == ip.CCD_EALIGN
    assert _compress(s, ws=None) == ip.CCD_EWORKSPACE
    assert _compress(s, ws=0x10010) == ip.CCD_EWORKSPACE      # not 256-byte aligned
    assert _compress(s, ws_bytes=ip.ccd_workspace_bytes(s) - 1) == ip.CCD_EWORKSPACE
    L = ip.lib()
    assert L.ccd_compress(None, P, P, P, P, None, P, 0x10000, 1 << 40, None) == ip.CCD_EINVAL
    assert L.ccd_select(ctypes.byref(s), None, P, None) == ip.CCD_EINVAL
    assert L.ccd_select(ctypes.byref(_shape(k=0)), P, P, None) == ip.CCD_EINVAL
    assert L.ccd_compact(ctypes.byref(s), P, P, None, P, P, None, None) == ip.CCD_EINVAL
    assert L.ccd_compact(ctypes.byref(s), P, P + 4, P, P, P, None, None) == ip.CCD_EALIGN
    assert L.ccd_compact(ctypes.byref(_shape(d=80)), P, P, P, P, P, None, None) == ip.CCD_EUNSUPPORTED


def test_cr_rope_argument_errors_are_decided_on_the_host():
    s = _shape()
    L = ip.lib()
    ws_bytes = ip.ccd_workspace_bytes(s)
    P2 = P + 0x100000

    def rope(K=P, cos=P, sin=P, count=10, Krot=P2):
        return L.ccd_cr_rope(ctypes.byref(s), K, cos, sin, count, Krot, None)

    assert rope(K=None) == ip.CCD_EINVAL and rope(cos=None) == ip.CCD_EINVAL and rope(sin=None) == ip.CCD_EINVAL
    assert rope(Krot=None) == ip.CCD_EINVAL and rope(Krot=P) == ip.CCD_EINVAL          # K_rot must not be K
    assert rope(count=-1) == ip.CCD_EINVAL and rope(count=s.n_cap + 1) == ip.CCD_EINVAL
    assert rope(cos=P + 4) == ip.CCD_EALIGN and rope(Krot=P2 + 8) == ip.CCD_EALIGN
    assert rope(count=0) == ip.CCD_OK                                                   # nothing to do, nothing launched

    def crope(cos=P, sin=P, Krot=P2, shape=s, Kscore=None, Kcap=None, lse=None):
        return L.ccd_compress_rope(ctypes.byref(shape), P, P, P, P, None, P, Kscore, Kcap, lse, cos, sin, Krot, 0x10000,
                                   ws_bytes, None)

    assert crope(Krot=None) == ip.CCD_EINVAL and crope(cos=None) == ip.CCD_EINVAL and crope(sin=None) == ip.CCD_EINVAL
    assert crope(Krot=P) == ip.CCD_EINVAL                                               # aliases K (and V)
    assert crope(sin=P + 4) == ip.CCD_EALIGN and crope(Kscore=P2 + 4) == ip.CCD_EALIGN
    assert crope(Kscore=P2, shape=_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP   # K_score may be K_rot
    assert crope(shape=_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP            # pot not full: nothing launched
    assert crope(Kcap=P) == ip.CCD_EINVAL and crope(Kcap=P2) == ip.CCD_EINVAL           # aliases K / K_rot
    assert crope(Kcap=P2 + 0x100004) == ip.CCD_EALIGN
    assert crope(Kcap=P2 + 0x100000, shape=_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP
    assert crope(Kcap=P2 + 0x100000, lse=P2 + 0x200000) == ip.CCD_EINVAL                # normalisers and CaP keys together
    assert crope(lse=P2 + 0x200004) == ip.CCD_EALIGN
    assert crope(lse=P2 + 0x200000, shape=_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP


def test_lse_argument_errors_are_decided_on_the_host():
    s = _shape()
    L = ip.lib()
    ws_bytes = ip.ccd_workspace_bytes(s)
    P2 = P + 0x100000
    assert L.ccd_score_lse(ctypes.byref(s), P, P, None, P, P, 0x10000, ws_bytes, None) == ip.CCD_EINVAL
    assert L.ccd_score_lse(ctypes.byref(s), P, P, P2 + 4, P, P, 0x10000, ws_bytes, None) == ip.CCD_EALIGN
    assert L.ccd_score_lse(ctypes.byref(s), P, P, P2, P, None, 0x10000, ws_bytes, None) == ip.CCD_EINVAL
    assert L.ccd_compress_lse(ctypes.byref(s), P, P, P, None, P, None, P, 0x10000, ws_bytes, None) == ip.CCD_EINVAL
    assert L.ccd_compress_lse(ctypes.byref(s), P, P, P, P2 + 8, P, None, P, 0x10000, ws_bytes, None) == ip.CCD_EALIGN
    assert L.ccd_compress_lse(ctypes.byref(s), P, P, P, P2, P, None, P, None, ws_bytes, None) == ip.CCD_EWORKSPACE
    noop = _shape(n_valid=300, n_cap=512, k=256)
    assert L.ccd_compress_lse(ctypes.byref(noop), P, P, P, P2, P, None, P, 0x10000, ws_bytes, None) == ip.CCD_NOOP


def test_kcat_argument_errors_are_decided_on_the_host():
    s = _shape()
    L = ip.lib()
    ws_bytes = ip.ccd_workspace_bytes(s)
    P2 = P + 0x100000

    def score(Kcap=P2, K=P, scores=P, ws=0x10000):
        return L.ccd_score_kcat(ctypes.byref(s), P, K, Kcap, P, scores, ws, ws_bytes, None)

    def compress(Kcap=P2, shape=s, K=P, V=P + 0x200000):
        return L.ccd_compress_kcat(ctypes.byref(shape), P, K, V, Kcap, P, None, P, 0x10000, ws_bytes, None)

    assert score(Kcap=None) == ip.CCD_EINVAL and compress(Kcap=None) == ip.CCD_EINVAL
    assert score(Kcap=P2 + 2) == ip.CCD_EALIGN and compress(Kcap=P2 + 2) == ip.CCD_EALIGN
    assert score(scores=None) == ip.CCD_EINVAL and score(ws=None) == ip.CCD_EWORKSPACE
    assert compress(Kcap=P) == ip.CCD_EINVAL and compress(Kcap=P + 0x200000) == ip.CCD_EINVAL   # aliases K / V
    assert compress(shape=_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP
    # an fp32 cache with CaP keys cannot take the matrix-core unit kernel: refused when named, not replaced silently
    f32 = _shape(dtype=ip.CCD_FP32, d=64, score_path=ip.CCD_PATH_MFMA_UNIT)
    assert L.ccd_compress_kcat(ctypes.byref(f32), P, P, P + 0x200000, P2, P, None, P, 0x10000, ip.ccd_workspace_bytes(f32),
                               None) == ip.CCD_EUNSUPPORTED


def test_window_errors_are_decided_on_the_host():
    assert _compress(_shape(window=-1)) == ip.CCD_EINVAL
    assert _compress(_shape(window=15)) == ip.CCD_EINVAL                      # shorter than the P = 16 CaP tokens
    assert _compress(_shape(score_path=4)) == ip.CCD_EINVAL and _compress(_shape(score_path=-1)) == ip.CCD_EINVAL
    # fp32 caches on the matrix cores: the unit kernel only, head dimension 64, no window (no CaP keys: next test)
    for path in (ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT):
        assert _compress(_shape(dtype=ip.CCD_FP32, score_path=path)) == ip.CCD_EUNSUPPORTED            # d = 128
    assert _compress(_shape(dtype=ip.CCD_FP32, d=64, score_path=ip.CCD_PATH_MFMA_SLICES)) == ip.CCD_EUNSUPPORTED
    assert _compress(_shape(dtype=ip.CCD_FP32, d=64, score_path=ip.CCD_PATH_MFMA_UNIT, window=400)) == ip.CCD_EUNSUPPORTED
    assert _compress(_shape(dtype=ip.CCD_FP32, d=64, score_path=ip.CCD_PATH_MFMA_UNIT, n_valid=300)) == ip.CCD_NOOP
    assert "fp32" in ip.ccd_strerror(ip.CCD_EUNSUPPORTED) and "2000" in ip.ccd_strerror(ip.CCD_EUNSUPPORTED)
    # more CaP tokens than the windowed matrix-core kernels take: refused when such a path is named (the automatic
    # choice scores on the vector ALUs then: tests/test_gpu_swa.py)
    for path in (ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT):
        big = _shape(n_valid=8192, n_cap=8192, k=4096, T=0, P=2100, window=4096, score_path=path)
        assert _compress(big) == ip.CCD_EUNSUPPORTED
    assert ip.ccd_workspace_bytes(_shape(window=512)) == ip.ccd_workspace_bytes(_shape())
    assert _compress(_shape(n_valid=300, n_cap=512, k=256, window=300)) == ip.CCD_NOOP


def test_pot_not_full_is_a_noop_decided_on_the_host():
    # Sec. 3.2: distillation only happens once the cache is full.  The fake pointers prove nothing is launched.
    assert _compress(_shape(n_valid=300, n_cap=512, k=256)) == ip.CCD_NOOP
    assert _compress(_shape(n_valid=512, n_cap=512, k=512, T=0)) == ip.CCD_NOOP


def test_strerror():
    for code in (0, 1, -1, -2, -3, -4, -5, 99):
        assert len(ip.ccd_strerror(code)) > 0
    with pytest.raises(ip.CCDError):
        ip._check(ip.CCD_EALIGN)


def test_nuc_from_logits_argument_errors_are_decided_on_the_host():
    L = ip.lib()

    def nuc(logits=P, labels=P, nov=P, rows=4, V=1000, stride=1000, dtype=ip.CCD_BF16):
        return L.ccd_nuc_from_logits(logits, labels, nov, rows, V, stride, dtype, None)

    assert nuc(logits=None) == ip.CCD_EINVAL and nuc(labels=None) == ip.CCD_EINVAL and nuc(nov=None) == ip.CCD_EINVAL
    assert nuc(rows=-1) == ip.CCD_EINVAL and nuc(V=0) == ip.CCD_EINVAL and nuc(stride=999) == ip.CCD_EINVAL
    assert nuc(dtype=5) == ip.CCD_EUNSUPPORTED
    assert nuc(logits=P + 2) == ip.CCD_EALIGN and nuc(V=1001, stride=1001) == ip.CCD_EALIGN     # rows 2002 bytes apart
    assert nuc(rows=0) == ip.CCD_OK                                                             # nothing launched


def test_append_argument_errors_are_decided_on_the_host():
    L = ip.lib()
    P2, P3, P4 = P + 0x100000, P + 0x200000, P + 0x300000

    def append(s, K=P, V=P2, nov=None, Kn=P3, Vn=P4, nn=None, count=10):
        return L.ccd_append(None if s is None else ctypes.byref(s), K, V, nov, Kn, Vn, nn, count, None)

    s = _shape(n_valid=100, n_cap=512)
    assert append(None) == ip.CCD_EINVAL
    assert append(s, K=None) == ip.CCD_EINVAL and append(s, Vn=None) == ip.CCD_EINVAL
    assert append(s, count=-1) == ip.CCD_EINVAL
    assert append(s, count=413) == ip.CCD_EINVAL                      # 100 + 413 > 512: the chunk does not fit
    assert append(s, count=0) == ip.CCD_OK and append(s, Kn=None, Vn=None, count=0) == ip.CCD_OK   # nothing to do, nothing launched
    assert append(s, nov=P, nn=None) == ip.CCD_EINVAL and append(s, nov=None, nn=P) == ip.CCD_EINVAL   # both or neither
    assert append(s, K=P + 2) == ip.CCD_EALIGN and append(s, Kn=P3 + 4) == ip.CCD_EALIGN
    assert append(_shape(n_valid=100, n_cap=512, d=96)) == ip.CCD_EUNSUPPORTED
    assert append(_shape(n_valid=100, n_cap=512, dtype=5)) == ip.CCD_EUNSUPPORTED
    assert append(_shape(n_valid=100, n_cap=512, kv_stride_h=100)) == ip.CCD_EINVAL
    assert append(_shape(n_valid=-1, n_cap=512)) == ip.CCD_EINVAL
    per_head = _shape(n_valid=100, n_cap=512, nov_stride_b=2 * 2 * 512, nov_stride_l=2 * 512, nov_stride_h=100)
    assert append(per_head, nov=P, nn=P2 + 64) == ip.CCD_EINVAL        # a head's novelty row shorter than the pot
