"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function the header declares, sizes its workspace and validates shapes."""
import ctypes
import os

import pytest

import paper_2404_18057_amd as kc


def test_library_is_built_in_tree_and_loads():
    assert os.path.dirname(kc.lib_path()).endswith("paper_2404_18057_amd")
    assert kc.version().startswith("kcache-gfx950")


def test_every_declared_function_is_exported():
    names = kc.declared_symbols()
    assert "kcache_prefill_store" in names and "kcache_decode_attention" in names
    assert len(names) >= 16
    raw = ctypes.CDLL(kc.lib_path())
    for n in names:
        assert hasattr(raw, n), n


def test_workspace_size_formula():
    # at least the unfused layout: fp32 scores [B][H][S_cap] + positions and weights [B][H][N]
    assert kc.workspace_bytes(8, 32, 32768, 256) >= 8 * 32 * 32768 * 4 + 2 * 8 * 32 * 256 * 4
    assert kc.workspace_bytes(8, 32, 32768, 256) <= 4 * 8 * 32 * 32768 * 4
    assert kc.workspace_bytes(1, 1, 1, 1) % 256 == 0 and kc.workspace_bytes(1, 1, 1, 1) > 0
    assert kc.workspace_bytes(0, 32, 1024, 8) == 0
    assert kc.workspace_bytes(8, 32, 1024, -1) == 0


@pytest.mark.parametrize("args,status", [
    ((1, 8, 2048, 128, 0, 8, 64), 0),
    ((16, 8, 8192, 128, 1, 32, 128), 0),      # GQA group of 4, bf16
    ((1, 8, 2048, 64, 0, 8, 64), 0),          # head_dim 64
    ((1, 8, 2048, 256, 1, 8, 64), 0),         # head_dim 256
    ((1, 8, 2048, 96, 0, 8, 64), -2),         # head_dim other than 64 / 128 / 256
    ((1, 8, 2048, 128, 0, 24, 64), -2),       # group of 3
    ((1, 2, 2048, 128, 0, 32, 64), 0),        # 32 query heads over 2 KV groups: group of 16
    ((1, 1, 2048, 128, 0, 64, 64), -2),       # group of 64
    ((1, 8, 2048, 128, 0, 12, 64), -1),       # H not a multiple of Hkv
    ((1, 8, 2048, 128, 2, 8, 64), -1),        # unknown dtype
    ((0, 8, 2048, 128, 0, 8, 64), -1),
    ((1, 8, 0, 128, 0, 8, 64), -1),
    ((1, 8, 2048, 128, 0, 8, 0), -1),         # N < 1
    ((1, 8, 2048, 128, 0, 0, 0), 0),          # store-only check ignores H and N
])
def test_shape_validation(args, status):
    assert kc.check_shapes(*args) == status


def test_calls_without_a_context_fail_cleanly():
    L = kc.lib()
    assert L.kcache_set_option(None, 0, 1) == -1
    assert L.kcache_synchronize(None) == -1
    assert L.kcache_destroy(None) == 0
    assert L.kcache_decode_attention(None, None, None, 0, None, 0, None, None, None, 0, None) == -1
    assert L.kcache_prefill_store(None, None, None, None, None, 1, None, None) == -1


def test_create_without_a_gpu_reports_an_error_instead_of_crashing():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(kc.KCacheError) as e:
        kc.Context(0)
    assert e.value.status == -5 and "HIP" in str(e.value)


def test_header_is_plain_c_and_a_c_caller_links(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with nothing but the standard
    headers, and a C program that names every entry point links against the library and can
    call the calls that need no GPU."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    names = kc.declared_symbols()
    src = tmp_path / "caller.c"
    refs = "\n".join("  p[%d] = (fn)%s;" % (i, n) for i, n in enumerate(names))
    src.write_text("""
#include <stdio.h>
#include "kcache.h"
typedef void (*fn)(void);
int main(void) {
  fn p[%d];
  kc_layer_cache c = {0};
%s
  c.B = 8; c.Hkv = 32; c.S_cap = 32768; c.d = 128; c.dtype = KC_F16;
  if (kcache_check_shapes(&c, 32, 256) != KC_OK) return 2;
  c.d = 96;
  if (kcache_check_shapes(&c, 32, 256) != KC_ERR_UNSUPPORTED) return 3;
  if (kcache_workspace_bytes(8, 32, 32768, 256) == 0) return 4;
  if (kcache_static_scratch_bytes() != ((size_t)48 << 20)) return 5;
  printf("%%s %%d\\n", kcache_version(), p[0] != 0);
  return 0;
}
""" % (len(names), refs))
    exe = tmp_path / "caller"
    libdir = os.path.dirname(kc.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, str(src),
                           "-o", str(exe), "-L", libdir, "-l:libkcache.so",
                           "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("kcache-gfx950")
