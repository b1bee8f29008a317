"""Host-side behaviour of the C ABI: the library loads without a GPU, exports every symbol the
header declares, sizes its workspace, and rejects bad arguments before touching the device.
Device pointers here are fake aligned addresses: every call below must fail validation (or be
a no-op) on the host, so nothing is ever dereferenced or launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_16886_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # aligned, never dereferenced


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return B.load_library()


def test_exports_every_declared_symbol(lib):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"RFKV_API\s+[\w\s\*]+?\b(rfkv_\w+)\s*\(", header))
    assert declared == set(B.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.rfkv_version() >= 100
    assert B.status_string(B.RFKV_OK) == "ok"
    assert "workspace" in B.status_string(B.RFKV_WORKSPACE_TOO_SMALL)
    assert B.rfkv_last_device_error() == 0


def test_params_struct_matches_header_layout():
    # 12 four-byte fields, 6 eight-byte strides, the padded-layout row count
    assert ctypes.sizeof(B.RfkvParams) == 104
    assert B.RfkvParams.granularity.offset == 44
    assert B.RfkvParams.out_pad_rows.offset == 96
    assert B.RfkvParams.k_stride_tok.offset == 48


def good(**kw):
    p = B.make_params(1, 32, 8, 128, 32, "bf16")
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_workspace_bytes(lib):
    p = good()
    small, big = B.rfkv_workspace_bytes(p, 8192, 8192), B.rfkv_workspace_bytes(p, 32768, 32768)
    assert 0 < small < big
    assert big >= 2 * 32768 * 8 * 4                         # padded index lists + scores at least
    assert B.rfkv_workspace_bytes(good(head_dim=96), 8192, 8192) == 0
    assert B.rfkv_workspace_bytes(p, 100, 200) == 0          # longest sequence exceeds the total
    assert lib.rfkv_workspace_bytes(None, 10, 10) == 0


CU = np.array([0, 4096], dtype=np.int32)


def score(p, q=FAKE, k=FAKE, cu_h=CU, cu_d=FAKE, s=FAKE, ws=FAKE, wsb=1 << 40):
    return B.rfkv_score(p, q, k, cu_h, cu_d, s, ws, wsb, stream=0, check=False)


def layer(p, q=FAKE, k=FAKE, v=FAKE, cu_h=CU, cu_d=FAKE, kept=FAKE, offs=FAKE, ko=FAKE, vo=FAKE, cap=1 << 20,
          ws=FAKE, wsb=1 << 40):
    return B.rfkv_compress_layer(p, q, k, v, cu_h, cu_d, None, kept, offs, None, ko, vo, cap, ws, wsb, stream=0,
                                 check=False)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    assert lib.rfkv_score(None, FAKE, FAKE, CU.ctypes.data, FAKE, FAKE, FAKE, 1 << 40, None) == B.RFKV_INVALID_ARG
    assert score(good(), q=None) == B.RFKV_INVALID_ARG
    assert score(good(), k=None) == B.RFKV_INVALID_ARG
    assert score(good(), s=None) == B.RFKV_INVALID_ARG
    assert score(good(), ws=None) == B.RFKV_INVALID_ARG
    assert score(good(), cu_h=None) == B.RFKV_INVALID_ARG
    assert score(good(), cu_d=None) == B.RFKV_INVALID_ARG
    assert score(good(), k=FAKE + 8) == B.RFKV_INVALID_ARG                  # misaligned
    assert score(good(n_q_heads=30)) == B.RFKV_INVALID_ARG                  # not a multiple of Hkv
    assert score(good(window=0)) == B.RFKV_INVALID_ARG
    assert score(good(n_sink=-1)) == B.RFKV_INVALID_ARG
    assert score(good(rank_mode=7)) == B.RFKV_INVALID_ARG
    assert score(good(softmax_scale=-1.0)) == B.RFKV_INVALID_ARG
    assert score(good(threshold=float("nan"))) == B.RFKV_INVALID_ARG
    assert score(good(k_stride_tok=100)) == B.RFKV_INVALID_ARG              # rows would overlap / misalign
    assert score(good(q_stride_head=132)) == B.RFKV_INVALID_ARG             # 264 bytes: not 16-byte aligned
    assert score(good(), cu_h=np.array([1, 4096], dtype=np.int32)) == B.RFKV_INVALID_ARG
    assert score(good(batch=2), cu_h=np.array([0, 500, 300], dtype=np.int32)) == B.RFKV_INVALID_ARG
    assert layer(good(), kept=None) == B.RFKV_INVALID_ARG
    assert layer(good(), offs=None) == B.RFKV_INVALID_ARG
    assert layer(good(), v=None) == B.RFKV_INVALID_ARG
    assert layer(good(), ko=None) == B.RFKV_INVALID_ARG
    assert layer(good(), cap=-1) == B.RFKV_INVALID_ARG
    assert layer(good(v_stride_head=64)) == B.RFKV_INVALID_ARG
    assert layer(good(), q=None) == B.RFKV_INVALID_ARG                      # queries are needed to score ...
    assert layer(good(threshold=0.0), q=None, k=None) == B.RFKV_INVALID_ARG  # ... and K and V always
    st = B.rfkv_compact(good(), FAKE, FAKE, CU, FAKE, FAKE, FAKE, None, FAKE, FAKE, 10, stream=0, check=False)
    assert st == B.RFKV_INVALID_ARG
    st = B.rfkv_select(good(), FAKE, CU, FAKE, None, FAKE, FAKE, FAKE, 1 << 40, stream=0, check=False)
    assert st == B.RFKV_INVALID_ARG


def test_unsupported_problems(lib):
    assert score(good(dtype=3)) == B.RFKV_UNSUPPORTED
    assert score(good(head_dim=96)) == B.RFKV_UNSUPPORTED
    assert score(good(window=20000)) == B.RFKV_UNSUPPORTED                   # 20000 * 4 rows > RFKV_MAX_WIDE_ROWS
    assert score(good(dtype=B.DTYPE_FP32, window=256)) == B.RFKV_UNSUPPORTED  # wide window: 256-byte rows at most
    assert score(good(dtype=B.DTYPE_FP32, window=128)) == B.RFKV_UNSUPPORTED  # fp32 queries do not fit in LDS
    assert score(good(batch=10000), cu_h=np.zeros(10001, dtype=np.int32)) == B.RFKV_UNSUPPORTED
    assert score(good(k_stride_tok=(1 << 22) + 8)) == B.RFKV_UNSUPPORTED      # above RFKV_MAX_STRIDE_TOK
    # a wide window over very many units: more work items than the kernels' 32-bit grids index
    cu = np.concatenate([[0], np.cumsum(np.r_[600000, np.full(7999, 1)])]).astype(np.int32)
    assert score(good(batch=8000, window=16384), cu_h=cu) == B.RFKV_UNSUPPORTED       # 512 x 37 x 64000 items


def test_workspace_too_small(lib):
    p = good()
    need = B.rfkv_workspace_bytes(p, 4096, 4096)
    assert score(p, wsb=need // 2) == B.RFKV_WORKSPACE_TOO_SMALL
    assert layer(p, wsb=16) == B.RFKV_WORKSPACE_TOO_SMALL
    st = B.rfkv_select(p, FAKE, CU, FAKE, FAKE, FAKE, FAKE, FAKE, 0, stream=0, check=False)
    assert st == B.RFKV_WORKSPACE_TOO_SMALL


def test_empty_batches_are_no_ops(lib):
    empty = np.array([0], dtype=np.int32)
    assert score(good(batch=0), cu_h=empty) == B.RFKV_OK
    assert layer(good(batch=0), cu_h=empty) == B.RFKV_OK
    assert score(good(batch=1), cu_h=np.array([0, 0], dtype=np.int32)) == B.RFKV_OK     # one empty sequence


def test_static_scratch_entry_point_host_checks(lib):
    """rfkv_compress_layer_static validates like rfkv_compress_layer and refuses, on the host, a batch
    whose scratch would not fit its fixed array (nothing is looked up or enqueued before that)."""
    def static(p, cu_h=CU, cap=8192 * 8):
        return B.rfkv_compress_layer_static(p, FAKE, FAKE, FAKE, cu_h, FAKE, None, FAKE, FAKE, None, FAKE, FAKE, cap,
                                            stream=0, check=False)
    assert static(good(window=0)) == B.RFKV_INVALID_ARG
    assert static(good(head_dim=96)) == B.RFKV_UNSUPPORTED
    assert static(good(), cu_h=None) == B.RFKV_INVALID_ARG
    n = 400000
    assert B.rfkv_workspace_bytes(good(), n, n) > B.STATIC_SCRATCH_BYTES
    assert static(good(), cu_h=np.array([0, n], dtype=np.int32), cap=n * 8) == B.RFKV_WORKSPACE_TOO_SMALL
    assert static(good(batch=0), cu_h=np.array([0], dtype=np.int32)) == B.RFKV_OK


def test_binding_raises_on_error(lib):
    with pytest.raises(B.RfkvError) as e:
        B.rfkv_score(good(window=0), FAKE, FAKE, CU, FAKE, FAKE, FAKE, 1 << 40, stream=0)
    assert e.value.status == B.RFKV_INVALID_ARG


def decode(p, n_new=64, q=FAKE, k=FAKE, v=FAKE, cu_h=CU, offs=FAKE, kept=None, out=FAKE, ws=FAKE, wsb=1 << 40):
    return B.rfkv_decode_attention(p, q, n_new, k, v, cu_h, offs, kept, out, ws, wsb, stream=0, check=False)


def masked(p, n_new=64, q=FAKE, k=FAKE, v=FAKE, cu_h=CU, cu_d=FAKE, mask=FAKE, out=FAKE, ws=FAKE, wsb=1 << 40):
    return B.rfkv_masked_attention(p, q, n_new, k, v, cu_h, cu_d, mask, out, ws, wsb, stream=0, check=False)


def test_decode_attention_host_checks(lib):
    """Everything the decode entry points can reject before touching the GPU (nothing is enqueued)."""
    need = B.rfkv_decode_workspace_bytes(good(), 64, 4096)
    assert need > 256 * 256 * 128 * 4                        # a partial output slot per workgroup at least
    assert B.rfkv_decode_workspace_bytes(good(), 65, 4096) == 0
    assert B.rfkv_decode_workspace_bytes(good(dtype=B.DTYPE_FP32, window=8), 4, 4096) == 0
    assert lib.rfkv_decode_workspace_bytes(None, 4, 4096) == 0
    assert decode(good(), n_new=65) == B.RFKV_UNSUPPORTED
    assert decode(good(dtype=B.DTYPE_FP32, window=8)) == B.RFKV_UNSUPPORTED
    assert decode(good(), n_new=-1) == B.RFKV_INVALID_ARG
    assert decode(good(), q=None) == B.RFKV_INVALID_ARG
    assert decode(good(), k=None) == B.RFKV_INVALID_ARG
    assert decode(good(), v=FAKE + 4) == B.RFKV_INVALID_ARG
    assert decode(good(), offs=None) == B.RFKV_INVALID_ARG
    # a padded cache is described by its kept counts: without them the attention would run over pad rows
    assert decode(good(out_pad_rows=8192)) == B.RFKV_INVALID_ARG
    assert decode(good(out_pad_rows=8192), kept=FAKE, wsb=need - 1) == B.RFKV_WORKSPACE_TOO_SMALL
    assert decode(good(), out=None) == B.RFKV_INVALID_ARG
    assert decode(good(), cu_h=None) == B.RFKV_INVALID_ARG
    assert decode(good(), cu_h=np.array([0, -5], dtype=np.int32)) == B.RFKV_INVALID_ARG
    assert decode(good(), wsb=need - 1) == B.RFKV_WORKSPACE_TOO_SMALL
    assert decode(good(), n_new=0) == B.RFKV_OK              # nothing to do
    assert decode(good(batch=0), cu_h=np.array([0], dtype=np.int32)) == B.RFKV_OK
    assert masked(good(), mask=None) == B.RFKV_INVALID_ARG
    assert masked(good(), cu_d=None) == B.RFKV_INVALID_ARG
    assert masked(good(k_stride_tok=100)) == B.RFKV_INVALID_ARG
    assert masked(good(), wsb=16) == B.RFKV_WORKSPACE_TOO_SMALL
    assert masked(good(v_stride_tok=(1 << 22) + 8)) == B.RFKV_UNSUPPORTED     # above RFKV_MAX_STRIDE_TOK


C_PROGRAM = r"""
#include "rfkv.h"
#include <stdio.h>
#include <string.h>
int main(void) {
  rfkv_params p;
  memset(&p, 0, sizeof p);
  p.batch = 1; p.n_q_heads = 32; p.n_kv_heads = 8; p.head_dim = 128; p.window = 32; p.n_sink = 4;
  p.threshold = 0.01f; p.rank_mode = RFKV_RANK_POSITION; p.dtype = RFKV_DTYPE_BF16;
  p.k_stride_tok = p.v_stride_tok = 8 * 128; p.k_stride_head = p.v_stride_head = 128;
  p.q_stride_row = 32 * 128; p.q_stride_head = 128;
  if (sizeof p != 104) return 1;
  if (rfkv_version() < 100) return 2;
  if (rfkv_workspace_bytes(&p, 32768, 32768) == 0) return 3;
  if (strcmp(rfkv_status_string(RFKV_OK), "ok") != 0) return 4;
  /* a null parameter block is rejected on the host, before anything touches a device */
  if (rfkv_score(0, 0, 0, 0, 0, 0, 0, 0, 0) != RFKV_INVALID_ARG) return 5;
  printf("%d\n", (int)rfkv_version());
  return 0;
}
"""


def test_header_is_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """include/rfkv.h compiles as strict C99 (and as C++), and a C program linked against the shared
    library reaches the host-side entry points.  No device call is made."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    src = tmp_path / "abi.c"
    src.write_text(C_PROGRAM)
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", f"-I{inc}", str(src)],
                   check=True)
    subprocess.run(["g++", "-std=c++11", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", f"-I{inc}",
                    str(src)], check=True)
    exe = tmp_path / "abi"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", f"-I{inc}", str(src), "-o", str(exe), B.LIB_PATH, f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120)
    assert int(out.stdout.strip()) == B.rfkv_version()
