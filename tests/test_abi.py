"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
before touching the GPU (no compute calls here)."""
import ctypes
import os
import re
import subprocess

import paper_2502_14477_amd as esa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "esa.h")).read()
    return sorted(set(re.findall(r"ESA_API\s+[\w\s\*]+?\b(esa_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert len(names) == 25 and "esa_attend" in names and "esa_select_topk" in names
    raw = ctypes.CDLL(esa.lib_path())
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(esa.EXPORTS) == names
    for n in ("esa_compress", "esa_score", "esa_select_topk", "esa_gather_kv", "esa_attend", "esa_segments"):
        assert callable(getattr(esa, n))
    assert esa.esa_version() >= 100


def test_segments_host_logic():
    assert esa.esa_segments(0, 128, 2048) == (0, 0)
    assert esa.esa_segments(100, 128, 2048) == (100, 100)
    assert esa.esa_segments(1000, 128, 2048) == (128, 128)
    assert esa.esa_segments(4608, 128, 2048) == (128, 2560)
    assert esa.esa_segments(130560, 128, 2048) == (128, 128512)
    L = esa.lib
    assert L.esa_segments(-1, 0, 0, ctypes.byref(ctypes.c_int64()), ctypes.byref(ctypes.c_int64())) == -1
    assert L.esa_segments(5, 1, 1, None, None) == -1


def test_argument_validation_returns_codes_without_a_gpu():
    L = esa.lib
    fake = ctypes.c_void_p(4096)          # never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(4097)
    # unsupported dtype / sizes
    assert L.esa_compress(fake, 4, 64, 64, fake, 0, None, 32, fake, 32, 7, 1, 0, 0, None) == -2
    assert L.esa_compress(fake, 4, 64, 64, fake, 0, None, 24, fake, 24, 0, 1, 0, 0, None) == -2
    assert L.esa_compress(fake, 4, 64, 32, fake, 0, None, 32, fake, 32, 0, 1, 0, 0, None) == -1     # ldx < d_in
    assert L.esa_compress(None, 4, 64, 64, fake, 0, None, 32, fake, 32, 0, 1, 0, 0, None) == -1     # null x
    assert L.esa_compress(odd, 4, 64, 64, fake, 0, None, 32, fake, 32, 0, 1, 0, 0, None) == -1      # misaligned
    assert L.esa_compress(fake, 4, 64, 64, fake, 5, None, 32, fake, 32, 0, 1, 0, 0, None) == -1     # unknown weight layout
    assert L.esa_compress(None, 0, 64, 64, None, 1, None, 32, None, 32, 0, 1, 0, 0, None) == 0      # empty: no-op
    assert L.esa_pack_weights(fake, 64, 32, 0, fake, None) == -1                                    # in place is refused
    assert L.esa_pack_weights(None, 64, 32, 0, fake, None) == -1
    assert b"esa_pack_weights" in L.esa_last_error()
    qk = lambda ldxk, ptr=fake: L.esa_compress_qk(ptr, 64, 64, fake, None, fake, 32, 0, 0, fake, 32, ldxk, fake, None, fake, 32, 0, 0,
                                                  4, 32, 1, 0, 1, None)
    assert qk(16) == -1                                                                             # key row stride < d_in
    assert qk(32, None) == -1
    # score: bad range, missing workspace
    assert L.esa_score(fake, 4, fake, 10, 5, 32, 0, fake, 0, 1, 0, 0, 0, fake, 1 << 20, None) == -1
    assert L.esa_score(fake, 4, fake, 0, 100, 32, 0, fake, 0, 1, 0, 0, 0, None, 0, None) == -3
    assert L.esa_score(fake, 4, fake, 0, 100, 32, 0, fake, 0, 1, 0, 0, 0, fake, 8, None) == -3
    assert L.esa_score(fake, 4, fake, 7, 7, 32, 0, fake, 0, 1, 0, 0, 0, None, 0, None) == 0       # empty middle
    # top-k
    assert L.esa_select_topk(fake, -1, 4, 0, fake, 1, 0, 0, fake, 1 << 20, None) == -1
    assert L.esa_select_topk(fake, 100, 4, 2**31 - 50, fake, 1, 0, 0, fake, 1 << 20, None) == -1  # positions overflow int32
    assert L.esa_select_topk(fake, 100000, 4, 0, fake, 1, 0, 0, fake, 16, None) == -3
    assert L.esa_select_topk(fake, 0, 4, 0, fake, 1, 0, 0, None, 0, None) == 0
    assert L.esa_select_topk_workspace_bytes(128384, 2048, 1) >= 3 * 2048 * 4
    # gather
    assert L.esa_gather_kv(fake, fake, 10, fake, 4, 2, 64, fake, fake, 0, 1, 0, 0, 0, None) == -1  # tok_stride < row
    assert L.esa_gather_kv(fake, fake, 128, None, 4, 2, 64, fake, fake, 0, 1, 0, 0, 0, None) == -1
    assert L.esa_gather_kv(fake, fake, 128, fake, 0, 2, 64, fake, fake, 0, 1, 0, 0, 0, None) == 0
    # attend: H not a multiple of H_kv, unsupported head size, more selected than middle tokens
    args = lambda h, h_kv, d, n_sel, t0: (fake, 8, h, h_kv, d, fake, fake, h_kv * d, t0, 4, 8, fake, fake, n_sel,
                                           ctypes.c_float(0.1), fake, None, 0, 1, 0, 0, 0, 0, fake, 1 << 20, None)
    assert L.esa_attend(*args(6, 4, 64, 0, 100)) == -1
    assert L.esa_attend(*args(4, 2, 48, 0, 100)) == -2
    assert L.esa_attend(*args(4, 2, 64, 200, 100)) == -1
    assert b"middle tokens" in L.esa_last_error()
    # the two-call form: unknown split
    assert L.esa_attend_local(fake, 8, 4, 2, 64, fake, fake, 128, 100, 4, 8, ctypes.c_float(0.1), 7, 0, 1, 0, 0,
                              fake, 1 << 20, None) == -1
    assert L.esa_attend_finish(fake, 8, 4, 2, 64, fake, fake, 128, 100, 4, 8, fake, fake, 0, ctypes.c_float(0.1), -1,
                               fake, None, 0, 1, 0, 0, 0, 0, fake, 1 << 20, None) == -1
    assert b"split" in L.esa_last_error()
    # rotary encoding: head size not a power of two, row stride smaller than the row, in place with unequal strides
    d64 = ctypes.c_double
    rope = lambda x, heads, d, ldx, out, ldo, base=5e5: L.esa_rope(x, 4, heads, d, ldx, d64(0.0), d64(1.0), d64(base), out,
                                                                    ldo, 1, 1, 0, 0, None)
    assert rope(fake, 2, 48, 96, fake, 96) == -2
    assert rope(fake, 2, 64, 100, fake, 128) == -1
    assert rope(fake, 2, 64, 128, fake, 256) == -1
    assert rope(fake, 2, 64, 128, None, 128) == -1
    assert rope(fake, 2, 64, 128, fake, 128, base=0.0) == -1
    assert L.esa_rope(None, 0, 2, 64, 128, d64(0.0), d64(1.0), d64(5e5), None, 128, 1, 1, 0, 0, None) == 0   # no rows: no-op
    # re-encoded attention: workspace too small, negative w
    re_args = lambda ws_bytes, w: (fake, 8, 4, 2, 64, fake, fake, 128, 100, 4, 8, fake, fake, 0, ctypes.c_float(0.1), d64(w),
                                   d64(5e5), fake, None, 0, 1, 0, 0, 0, 0, fake, ws_bytes, None)
    assert L.esa_attend_reencoded(*re_args(16, 4096.0)) == -3
    assert L.esa_attend_reencoded(*re_args(1 << 30, -1.0)) == -1
    assert L.esa_attend_reencoded_workspace_bytes(512, 32, 8, 128, 1, 1, 2048) > 2 * 512 * 4096 * 2 + 2 * 2560 * 1024 * 2


C_CLIENT = r"""
#include <stdio.h>
#include <string.h>
#include <dlfcn.h>
#include "esa.h"
int main(int argc, char** argv) {
  void* h = dlopen(argv[1], RTLD_NOW);
  if (!h) { printf("dlopen: %s\n", dlerror()); return 2; }
  int (*version)(void) = (int (*)(void))dlsym(h, "esa_version");
  int (*seg)(int64_t, int64_t, int64_t, int64_t*, int64_t*) =
      (int (*)(int64_t, int64_t, int64_t, int64_t*, int64_t*))dlsym(h, "esa_segments");
  const char* (*last)(void) = (const char* (*)(void))dlsym(h, "esa_last_error");
  size_t (*ws)(int64_t, int, int) = (size_t (*)(int64_t, int, int))dlsym(h, "esa_select_topk_workspace_bytes");
  if (!version || !seg || !last || !ws) return 3;
  int64_t i_end = -1, l_start = -1;
  if (seg(130560, 128, 2048, &i_end, &l_start) != ESA_OK) return 4;
  if (seg(-1, 0, 0, &i_end, &l_start) != ESA_EINVAL || !strstr(last(), "esa_segments")) return 5;
  seg(130560, 128, 2048, &i_end, &l_start);
  printf("%d %lld %lld %zu %d %d\n", version(), (long long)i_end, (long long)l_start, ws(128384, 2048, 1),
         ESA_SPLIT_ALGORITHM1, ESA_BF16);
  return 0;
}
"""


def test_header_is_plain_c_and_the_library_serves_a_c_client(tmp_path):
    """include/esa.h compiles as C99 and as C++ with no other header of this repository, and a C
    program that knows nothing but the header can load the library and call its host-side entry points."""
    inc = os.path.join(ROOT, "include")
    for lang, std in (("c", "-std=c99"), ("c++", "-std=c++11")):
        r = subprocess.run(["gcc", "-x", lang, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                            os.path.join(inc, "esa.h")], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    src = tmp_path / "client.c"
    src.write_text(C_CLIENT)
    exe = tmp_path / "client"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), "-ldl"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe), esa.lib_path()], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    version, i_end, l_start, ws_bytes, split, bf16 = (int(t) for t in r.stdout.split())
    assert version == esa.esa_version() and (i_end, l_start) == (128, 128512)
    assert ws_bytes == esa.lib.esa_select_topk_workspace_bytes(128384, 2048, 1)
    assert split == esa.ESA_SPLIT_ALGORITHM1 and bf16 == esa.ESA_BF16
