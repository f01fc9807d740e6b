"""Host-side checks of the C ABI that need no GPU: the library loads, exports exactly the symbols
include/apbv.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2601_21444_amd as apbv
from paper_2601_21444_amd.binding import ApbvTensor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "apbv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(apbv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = apbv.load_library()
    names = declared_symbols()
    assert names == ["apbv_compress_kv", "apbv_compress_kv_noalloc", "apbv_compress_kv_reduced", "apbv_compress_reduced_workspace_bytes",
                     "apbv_compress_workspace_bytes", "apbv_host_attention", "apbv_host_attention_group",
                     "apbv_merge_lse",
                     "apbv_query_attention", "apbv_query_attention_workspace_bytes", "apbv_status_string",
                     "apbv_version"]
    for n in names:
        assert getattr(lib, n) is not None
    assert apbv.apbv_version() >= 100


def test_status_strings():
    for code, word in [(0, "OK"), (-1, "NULL"), (-2, "SHAPE"), (-3, "UNSUPPORTED"), (-4, "WORKSPACE"), (-5, "LAUNCH")]:
        assert word in apbv.status_string(code)
    assert "unknown" in apbv.status_string(-99)


def test_workspace_size_query():
    ws = apbv.apbv_compress_workspace_bytes
    assert ws(1, 2, 128, 16384, 1024) >= 2 * 16384 * 8 + 2 * 128 * 8
    assert ws(2, 2, 128, 16384, 1024) > ws(1, 2, 128, 16384, 1024)
    assert ws(1, 2, 128, 16384, 16384) > ws(1, 2, 128, 16384, 8192)     # large sort spills to the workspace
    assert ws(1, 2, 96, 16384, 10) == 0 and ws(0, 2, 128, 10, 1) == 0 and ws(1, 2, 128, 10, 11) == 0


def view(tokens, heads, d, ptr=0x1000, batch_stride=None):
    return ApbvTensor(ptr if tokens else None, tokens, heads * d, d, batch_stride or max(tokens, 1) * heads * d)


def call_attention(batch=1, hq=4, hkv=2, d=128, L=64, l_a=8, n_p=8, scale=0.1, out=0x2000, q=None, ka=None, va=None,
                   kp=None, vp=None, k=None, v=None):
    lib = apbv.load_library()
    return lib.apbv_host_attention(
        batch, hq, hkv, d,
        q or view(L, hq, d), ka or view(l_a, hkv, d), va or view(l_a, hkv, d), kp or view(n_p, hkv, d),
        vp or view(n_p, hkv, d), k or view(L, hkv, d), v or view(L, hkv, d),
        ctypes.c_float(scale), out, None, None)


def test_attention_rejects_bad_arguments_without_launching():
    assert call_attention(hq=3, hkv=2) == -2                     # Hq % Hkv
    assert call_attention(d=96) == -3                            # unsupported head_dim
    assert call_attention(batch=0) == -2
    assert call_attention(out=None) == -1
    assert call_attention(out=0x2004) == -2                      # misaligned output
    assert call_attention(scale=0.0) == -2 and call_attention(scale=float("nan")) == -2
    assert call_attention(q=view(63, 4, 128)) == -2              # q rows != local keys
    assert call_attention(va=view(7, 2, 128)) == -2              # K/V anchor mismatch
    assert call_attention(vp=view(9, 2, 128)) == -2
    assert call_attention(k=ApbvTensor(None, 64, 256, 128, 0)) == -1
    assert call_attention(k=ApbvTensor(0x1008, 64, 256, 128, 0)) == -2      # 8-byte aligned only
    assert call_attention(k=ApbvTensor(0x1000, 64, 252, 128, 0)) == -2      # stride not a multiple of 8
    assert call_attention(k=ApbvTensor(0x1000, 64, 64, 128, 0)) == -2       # rows overlap
    assert call_attention(L=0) == -2
    assert call_attention(k=view(0, 2, 128), v=view(0, 2, 128), l_a=0, n_p=0) == -2       # no key at all
    assert call_attention(k=view(0, 2, 128)) == -2                                        # K/V local mismatch
    assert call_attention(k=ApbvTensor(0x1000, 64, 1 << 24, 128, 0)) == -3     # token stride too large for 32-bit tile offsets


def call_compress(batch=1, hq=4, hkv=2, d=128, n_q=4, L=64, l_p=8, idx=0x3000, kc=0x4000, vc=0x5000, ws=0x10000,
                  ws_bytes=1 << 20, q=None, k=None, v=None):
    lib = apbv.load_library()
    return lib.apbv_compress_kv(batch, hq, hkv, d, q or view(n_q, hq, d), k or view(L, hkv, d), v or view(L, hkv, d),
                                l_p, idx, kc, vc, None, ws, ws_bytes, None)


def test_compress_rejects_bad_arguments_without_launching():
    assert call_compress(l_p=65) == -2 and call_compress(l_p=-1) == -2
    assert call_compress(hq=5) == -2
    assert call_compress(d=32) == -3
    assert call_compress(idx=None) == -1 and call_compress(kc=None) == -1 and call_compress(vc=None) == -1
    assert call_compress(ws=None) == -4 and call_compress(ws=0x10010) == -4 and call_compress(ws_bytes=64) == -4
    assert call_compress(n_q=0) == -2
    assert call_compress(v=view(63, 2, 128)) == -2
    assert call_compress(kc=0x4002) == -2


def test_compress_noalloc_rejects_bad_arguments_and_oversize_without_launching():
    lib = apbv.load_library()

    def call(batch=1, hq=4, hkv=2, d=128, n_q=4, L=64, l_p=8, idx=0x3000, kc=0x4000, vc=0x5000):
        return lib.apbv_compress_kv_noalloc(batch, hq, hkv, d, view(n_q, hq, d), view(L, hkv, d), view(L, hkv, d), l_p,
                                            idx, kc, vc, None, None)
    assert call(l_p=65) == -2 and call(hq=5) == -2 and call(d=32) == -3 and call(idx=None) == -1
    # a shape whose workspace exceeds the static array is refused with the workspace status
    assert apbv.apbv_compress_workspace_bytes(64, 2, 128, 16384, 8) > apbv.NOALLOC_MAX_WORKSPACE_BYTES
    assert call(batch=64, L=16384) == -4
    assert apbv.apbv_compress_workspace_bytes(2, 4, 128, 16384, 2048) <= apbv.NOALLOC_MAX_WORKSPACE_BYTES
    assert b"static scratch" in lib.apbv_status_string(-4)


def test_compress_reduced_rejects_bad_arguments_without_launching():
    lib = apbv.load_library()
    ws = apbv.apbv_compress_reduced_workspace_bytes
    base = apbv.apbv_compress_workspace_bytes(1, 2, 128, 4096, 64)
    assert ws("sum", 1, 4, 2, 128, 8, 4096, 64) == base
    assert ws("max", 1, 4, 2, 128, 8, 4096, 64) == (base + 255) // 256 * 256          # no row statistics
    # softmax-sum: 16 rows -> 32 padded, 16 chunks of 256 keys, 2 heads: partial statistics of 8 bytes, final of 4
    assert ws("softmax_sum", 1, 4, 2, 128, 8, 4096, 64) == (base + 255) // 256 * 256 + 2 * 16 * 32 * 8 + 2 * 32 * 4
    assert lib.apbv_compress_reduced_workspace_bytes(7, 1, 4, 2, 128, 8, 4096, 64) == 0
    assert lib.apbv_compress_reduced_workspace_bytes(1, 1, 5, 2, 128, 8, 4096, 64) == 0

    def call(reducer=2, scale=0.1, n_q=8, L=4096, ws_bytes=1 << 24, hq=4):
        return lib.apbv_compress_kv_reduced(reducer, scale, 1, hq, 2, 128, view(n_q, hq, 128), view(L, 2, 128),
                                            view(L, 2, 128), 64, 0x3000, 0x4000, 0x5000, None, 0x10000, ws_bytes, None)
    assert call(reducer=3) == -2 and call(reducer=-1) == -2
    assert call(scale=0.0) == -2 and call(scale=float("inf")) == -2
    assert call(reducer=1, scale=0.0, ws_bytes=64) == -4          # the scale is ignored by the maximum; workspace too small
    need = ws("softmax_sum", 1, 4, 2, 128, 8, 4096, 64)
    assert call(ws_bytes=need - 1) == -4
    assert call(n_q=4200, ws_bytes=1 << 30) == -3                 # 8400 rows: more than the softmax-sum kernels stage


def test_merge_rejects_bad_arguments_without_launching():
    lib = apbv.load_library()

    def call(n=2, rows=8, hq=4, d=128, po=0x1000, so=8 * 4 * 128, pl=0x9000, sl=32, out=0x20000):
        return lib.apbv_merge_lse(n, rows, hq, d, po, so, pl, sl, out, None, None)
    assert call(n=0) == -2 and call(rows=0) == -2 and call(d=96) == -3
    assert call(po=None) == -1 and call(pl=None) == -1 and call(out=None) == -1
    assert call(po=0x1008) == -2 and call(so=100) == -2 and call(sl=31) == -2


def test_query_attention_workspace_plan_and_rejections():
    lib = apbv.load_library()
    ws = apbv.apbv_query_attention_workspace_bytes
    assert ws(1, 24, 128, 256, 64 * 1024, 1) == 0                       # one range: the plain kernel, no workspace
    per_split = 256 * 24 * 128 * 2 + 256 * 24 * 4                       # bf16 partial + fp32 lse, already 256-aligned
    assert ws(1, 24, 128, 256, 64 * 1024, 8) == 8 * per_split
    assert ws(1, 24, 128, 256, 64 * 1024, 100000) == 256 * per_split    # clipped to 256 ranges
    assert ws(1, 24, 128, 256, 100, 8) == 2 * per_split                 # two 64-key tiles only
    auto = ws(1, 24, 128, 256, 64 * 1024, 0)
    assert auto % per_split == 0 and 2 <= auto // per_split <= 256      # a short block over a long context is split
    assert ws(1, 24, 128, 16384, 64 * 1024, 0) == 0                     # a full block fills the GPU by itself
    assert ws(0, 24, 128, 256, 1024, 0) == 0 and ws(1, 24, 96, 256, 1024, 0) == 0 and ws(1, 24, 128, 256, 1024, -1) == 0

    def call(n_splits=4, ws_ptr=0x100000, ws_bytes=1 << 30, out=0x2000, n_q=64, l_a=4096, hq=4):
        e = view(0, 2, 128)
        return lib.apbv_query_attention(1, hq, 2, 128, view(n_q, hq, 128), view(l_a, 2, 128), view(l_a, 2, 128),
                                        e, e, e, e, 0.1, n_splits, out, None, ws_ptr, ws_bytes, None)
    assert call(ws_ptr=None) == -4 and call(ws_ptr=0x100010) == -4 and call(ws_bytes=1024) == -4
    assert call(n_splits=-1) == -2 and call(out=None) == -1 and call(hq=3) == -2 and call(n_q=0) == -2


def test_attention_group_rejects_bad_arguments_without_launching():
    lib = apbv.load_library()

    def item(L=64, l_a=8, n_p=16, local=None, out=0x2000):
        it = apbv.ApbvAttentionItem()
        it.q_local = view(L, 4, 128)
        it.k_anchor = it.v_anchor = view(l_a, 2, 128)
        it.k_pass = it.v_pass = view(n_p, 2, 128)
        it.k_local = it.v_local = view(L if local is None else local, 2, 128)
        it.out, it.lse_out = out, None
        return it

    def call(items, n=None, hq=4, hkv=2, d=128, scale=0.1):
        arr = (apbv.ApbvAttentionItem * max(len(items), 1))(*items)
        return lib.apbv_host_attention_group(len(items) if n is None else n, arr, hq, hkv, d, scale, None)
    assert call([], n=0) == -2 and call([item()] * 9) == -2
    assert lib.apbv_host_attention_group(1, None, 4, 2, 128, 0.1, None) == -1
    assert call([item(), item(out=None)]) == -1
    assert call([item(), item(local=0)]) == -3              # no causal segment: not in a group
    assert call([item(), item(local=63)]) == -2
    assert call([item()], hq=3) == -2 and call([item()], d=96) == -3 and call([item()], scale=-1.0) == -2


def test_product_path_has_no_oracle_or_cpu_fallback():
    """The package must not import the oracle, and must raise when the library is absent."""
    pkg = os.path.join(ROOT, "paper_2601_21444_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
    import paper_2601_21444_amd.binding as b
    saved_lib, saved_path = b._lib, b._LIB_PATH
    try:
        b._lib, b._LIB_PATH = None, os.path.join(pkg, "does_not_exist.so")
        with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
            b.load_library()
    finally:
        b._lib, b._LIB_PATH = saved_lib, saved_path


SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g",
            "-static-libasan", "-static-libubsan"]       # static runtimes: independent of the process's preload list


def build_and_run_host_check(tmp_path, name):
    """Compile tests/host/<name>.cpp with the host compiler under the address and undefined-behaviour sanitizers
    (no HIP involved: the headers it includes are plain C++) and run it."""
    import subprocess
    exe = tmp_path / name
    src = os.path.join(ROOT, "tests", "host", name + ".cpp")
    incs = ["-I", os.path.join(ROOT, "paper_2601_21444_amd", "csrc"), "-I", os.path.join(ROOT, "include")]
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", *SANITIZE, *incs, src, "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([str(exe)], capture_output=True, text=True, env=env)


def test_group_schedule_covers_every_query_tile_once(tmp_path):
    """The merged heaviest-first schedule of apbv_host_attention_group, checked by brute force on the host, under
    the sanitizers."""
    res = build_and_run_host_check(tmp_path, "schedule_check")
    assert res.returncode == 0 and "schedule ok" in res.stdout, res.stdout + res.stderr


def test_host_validation_under_sanitizers(tmp_path):
    """Every rejection case of the C ABI's host-side validation and the workspace / key-split planners, compiled
    alone with g++ -fsanitize=address,undefined."""
    res = build_and_run_host_check(tmp_path, "validation_check")
    assert res.returncode == 0 and "host validation OK" in res.stdout, res.stdout + res.stderr
