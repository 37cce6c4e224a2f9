"""The C-ABI library builds, loads and exports every function include/mkv.h declares; its
configuration checks and size arithmetic run without a GPU.  No compute calls here."""
import ctypes as C
import os
import re

import pytest

from paper_2605_29873_amd import binding as B
from paper_2605_29873_amd import inputs as X

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return B.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "mkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mkv_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported(lib):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mkv.h but not exported"


def _cfg(**kw):
    base = dict(n_layers=1, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64, dtype=B.MKV_F32,
                max_prefill=256, decode_budget=64, evict_trigger=72, decode_capacity=0,
                recent_window=8, alpha=0.9, softmax_scale=0.0, score_mode=0, split_keys=0)
    base.update(kw)
    return B.make_config(**base)


def test_required_bytes_covers_the_pools(lib):
    cfg = _cfg()
    need = B.mkv_required_bytes(cfg)
    pools = 2 * 2 * 2 * (256 + 73) * 64 * 4        # K and V, batch 2, 2 KV heads, fp32
    assert pools < need < pools + (1 << 20)
    wl = X.workloads()["cfg5"]
    big = _cfg(n_layers=32, batch=32, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=B.MKV_BF16,
               max_prefill=16384, decode_budget=4096, evict_trigger=4159, recent_window=128)
    kv = 32 * 32 * (16384 + 4160) * 4096          # layers x seqs x tokens x 4 KB per token per layer
    assert kv < B.mkv_required_bytes(big) < kv * 1.02 < 288e9
    assert wl.capacity == 4160


@pytest.mark.parametrize("bad", [
    dict(n_q_heads=7), dict(head_dim=96), dict(dtype=5), dict(decode_budget=0),
    dict(evict_trigger=63), dict(recent_window=65), dict(alpha=1.5), dict(alpha=-0.1),
    dict(alpha=float("nan")), dict(batch=0), dict(n_layers=0), dict(score_mode=3),
    dict(split_keys=100), dict(evict_trigger=B.MKV_NEVER_EVICT),            # capacity missing
    dict(evict_trigger=B.MKV_NEVER_EVICT, decode_capacity=64),              # not above the budget
    dict(decode_capacity=70),                                               # below trigger + 1
    dict(decode_budget=20000, evict_trigger=20000),                         # above the supported pool
    dict(batch=5000), dict(max_prefill=1 << 24), dict(softmax_scale=-1.0), dict(arena=12345, arena_bytes=1 << 30),
])
def test_bad_configurations_are_refused_without_touching_the_gpu(lib, bad):
    cfg = _cfg(**bad)
    assert B.mkv_required_bytes(cfg) == 0
    out = C.c_void_p()
    assert lib.mkv_create(C.byref(cfg), C.byref(out)) == B.MKV_ERR_ARG
    assert out.value is None
    assert B.mkv_last_error(None) != ""


def test_null_arguments(lib):
    assert lib.mkv_create(None, None) == B.MKV_ERR_ARG
    assert lib.mkv_destroy(None) == B.MKV_OK
    assert lib.mkv_evict(None, 0, 0) == B.MKV_ERR_ARG
    assert lib.mkv_get_lens(None, 0, 0, None, None, None) == B.MKV_ERR_ARG


def test_header_is_plain_c_and_the_binding_mirrors_its_struct(tmp_path):
    """include/mkv.h compiles as C99 on its own, and the ctypes mirror of mkv_config has the
    header's size and field offsets (checked with a small C program, no GPU involved)."""
    import subprocess
    fields = [name for name, _ in B.mkv_config._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "mkv.h"', 'int main(void) {',
             '  printf("%zu\\n", sizeof(mkv_config));']
    lines += [f'  printf("%zu\\n", offsetof(mkv_config, {f}));' for f in fields]
    lines += ['  return 0;', '}']
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == C.sizeof(B.mkv_config)
    for f, off in zip(fields, out[1:]):
        assert int(off) == getattr(B.mkv_config, f).offset, f


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The host side of the ABI (configuration checks, layout arithmetic, argument handling in
    csrc/mkv_api.hip) built with AddressSanitizer and UBSan on the host pass only, driven by
    tests/abi_host_driver.c.  No GPU code is sanitized and no GPU is needed."""
    import subprocess
    from paper_2605_29873_amd import build as Bd
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    csrc = os.path.join(ROOT, "paper_2605_29873_amd", "csrc")
    objs = []
    for src in Bd.SOURCES:                      # only the API file holds host logic; the others bring the launch stubs
        obj = tmp_path / src.replace(".hip", ".o")
        plain = os.path.join(ROOT, "paper_2605_29873_amd", "_build", src.replace(".hip", ".o"))
        if src != "mkv_api.hip" and os.path.exists(plain):
            objs.append(plain)
            continue
        flags = san if src == "mkv_api.hip" else []
        subprocess.run([hipcc, *Bd.FLAGS, *flags, "-I", os.path.join(ROOT, "include"), "-c",
                        os.path.join(csrc, src), "-o", str(obj)], check=True, capture_output=True)
        objs.append(str(obj))
    lib = tmp_path / "libmkv_san.so"
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", str(lib),
                    "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"], check=True, capture_output=True)
    exe = tmp_path / "abi_host_driver"
    clang = "/opt/rocm/llvm/bin/clang"
    subprocess.run([clang, "-std=c99", "-Wall", "-Werror", "-g", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-sanitize-recover=undefined", "-shared-libsan", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_host_driver.c"), "-o", str(exe),
                    f"-L{tmp_path}", "-lmkv_san", f"-Wl,-rpath,{tmp_path}"], check=True, capture_output=True)
    rt_dir = os.path.dirname(subprocess.run([clang, "--print-file-name=libclang_rt.asan-x86_64.so"],
                                            check=True, capture_output=True, text=True).stdout.strip())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               LD_LIBRARY_PATH=rt_dir + ":/opt/rocm/lib:" + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.strip().endswith("ok")
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
