"""CPU-only checks of the C ABI: the library loads, exports what the header declares, and its host
logic (plan arithmetic, argument validation) agrees with the paper's integers and the oracle's rules."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import pytest

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding
from paper_2505_00570_amd.binding import Layout, Plan, Profile
from oracle import freqkv_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "freqkv.h")


def _layout(dtype=fk.BF16, n_layers=32, batch=1, n_heads=8, cap=8192, d=128):
    L = Layout()
    L.dtype, L.n_layers, L.batch, L.token_capacity = dtype, n_layers, batch, cap
    L.stride_token = d
    L.stride_head = cap * d
    L.stride_batch = n_heads * cap * d
    L.stride_layer = batch * n_heads * cap * d
    return L


def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(freqkv_[a-z_0-9]+)\s*\(", text))
    assert {"freqkv_plan", "freqkv_compress", "freqkv_status_string", "freqkv_shutdown"} <= declared
    lib = fk.load()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert fk.version() >= 100


def test_struct_layout_matches_header():
    """sizeof/offsetof of the ctypes mirrors equal what a C compiler sees in freqkv.h."""
    src = r'''
#include <stdio.h>
#include <stddef.h>
#include "freqkv.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %zu\n", sizeof(freqkv_layout_t), offsetof(freqkv_layout_t, stride_token),
         offsetof(freqkv_layout_t, workspace), offsetof(freqkv_layout_t, tap_f32),
         sizeof(freqkv_plan_t), sizeof(freqkv_profile_t));
  printf("%zu %zu %zu\n", offsetof(freqkv_plan_t, workspace_bytes), offsetof(freqkv_plan_t, flops_dense),
         offsetof(freqkv_profile_t, ms_prepare));
  return 0; }
'''
    with tempfile.TemporaryDirectory() as td:
        c = os.path.join(td, "t.c")
        open(c, "w").write(src)
        exe = os.path.join(td, "t")
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe])
        out = subprocess.check_output([exe]).decode().split()
    got = [int(x) for x in out]
    want = [C.sizeof(Layout), Layout.stride_token.offset, Layout.workspace.offset, Layout.tap_f32.offset,
            C.sizeof(Plan), C.sizeof(Profile), Plan.workspace_bytes.offset, Plan.flops_dense.offset,
            Profile.ms_prepare.offset]
    assert got == want


def test_status_strings():
    assert fk.status_string(0) == "FREQKV_OK"
    assert fk.status_string(1) == "FREQKV_NOOP"
    assert fk.status_string(-3) == "FREQKV_E_WORKSPACE"
    assert "UNKNOWN" in fk.status_string(-99)


def test_plan_matches_paper_integers():
    # Sec. 4.1: window 4096, 4 sinks, ratio 0.5: 4092 states -> 2046
    rc, p = fk.plan(_layout(n_heads=32, cap=4096), 32, 128, 4096, 4096, 4, 0.5)
    assert rc == 0 and (p.span_len, p.retained_len, p.new_len) == (4092, 2046, 2050)
    assert p.head_tensors == 2 * 32 * 32
    # LLaMA-3 window
    rc, p = fk.plan(_layout(), 8, 128, 8192, 8192, 4, 0.5)
    # 8188 = 4 * 23 * 89, ratio 1/2: the factored transform, no workspace, tables of about 113 KiB
    assert (p.span_len, p.retained_len, p.new_len, p.head_tensors, p.variant) == (8188, 4094, 4098, 512, 6)
    assert p.workspace_bytes == 0 and p.workspace_min_bytes == 0
    assert p.basis_bytes == 2 * 18 * 1024 + 2 * 6 * 1024 + 45 * 12 * 64
    assert p.flops_dense == pytest.approx(2.0 * 4094 * 8188 * 128 * 512)
    assert p.bytes_algorithmic == pytest.approx((8188 + 4094) * 128 * 2 * 512)
    per_channel = 2.0 * (4 * 23 * 89 * 90 + 4 * 45 * 4 * 23 * 23 + 16 * 23 * 45 + 2 * 45 * 4 * 23 * 23 + 2 * 23 * 90 * 89)
    assert p.flops_executed == pytest.approx(per_channel * 128 * 512)
    assert p.flops_executed < p.flops_dense / 15
    # the matrix form on request
    Ld = _layout()
    Ld.flags = fk.FLAG_DENSE
    rc, p = fk.plan(Ld, 8, 128, 8192, 8192, 4, 0.5)
    assert (p.span_len, p.retained_len, p.new_len, p.head_tensors, p.variant) == (8188, 4094, 4098, 512, 5)
    assert p.flops_dense == pytest.approx(2.0 * 4094 * 8188 * 128 * 512)
    assert p.flops_executed == pytest.approx(p.flops_dense * 3 / 8)       # two-level even/odd fold
    assert p.bytes_algorithmic == pytest.approx((8188 + 4094) * 128 * 2 * 512)
    assert p.workspace_min_bytes <= p.workspace_bytes
    # even part: 2 x 1024 rows x 2048 columns, odd part: 2048 rows x 4096 columns, fp16
    assert p.basis_bytes == 2 * 1024 * 2048 * 2 + 2048 * 4096 * 2
    # the one-level fold on request
    L1 = _layout()
    L1.flags = fk.FLAG_SINGLE_FOLD
    rc, p1 = fk.plan(L1, 8, 128, 8192, 8192, 4, 0.5)
    assert p1.variant == 1 and p1.flops_executed == pytest.approx(p1.flops_dense / 2)
    assert p1.basis_bytes == 2 * 2048 * 4096 * 2


@pytest.mark.parametrize("window,sink,ratio,cur", [(4096, 4, 0.5, 4096), (4096, 0, 0.25, 5000), (512, 4, 0.5, 512),
                                                   (701, 4, 0.5, 701), (100, 8, 0.75, 130), (64, 2, 0.01, 64),
                                                   (50, 8, 1.0, 70), (4096, 4, 0.3, 4096)])
def test_plan_agrees_with_oracle_rules(window, sink, ratio, cur):
    rc, p = fk.plan(_layout(cap=max(cur, window)), 8, 128, cur, window, sink, ratio)
    assert rc == 0
    assert p.span_len == window - sink
    assert p.retained_len == orc.retained_len(window - sink, ratio)
    assert p.new_len == orc.new_len(cur, window, sink, ratio)
    if ratio == 1.0:
        assert p.variant == 0 and p.workspace_bytes == 0
    elif window - sink in (8188, 4092, 2044, 1020, 1260, 140) and p.retained_len * 2 == window - sink:
        assert p.variant == 6 and p.workspace_bytes == 0
    elif (window - sink) % 4 == 0 and p.retained_len % 2 == 0 and window - sink >= 2048:
        assert p.variant == 5                     # 32 layers x 8 heads: enough head-tensors for the two-level fold
    elif (window - sink) % 2 == 0 and p.retained_len % 2 == 0:
        assert p.variant == 1
    else:
        assert p.variant == 2


def test_plan_noop_below_window():
    rc, p = fk.plan(_layout(), 8, 128, 100, 8192, 4, 0.5)
    assert rc == 1 and p.retained_len == 4094
    assert p.new_len == 4 + 4094            # plan for a full cache without a tail


def test_trigger_schedule_from_plan_matches_paper_counts():
    # count compressions while T tokens stream in, using only the library's plan arithmetic
    def count(total, window, sink, ratio):
        cur, fed, n = 0, 0, 0
        while fed < total:
            if cur >= window:
                _, p = fk.plan(_layout(cap=window), 8, 128, cur, window, sink, ratio)
                cur, n = p.new_len, n + 1
            take = min(total - fed, window - cur)
            cur, fed = cur + take, fed + take
        return n
    for total, expect in [(4096, 0), (8192, 3), (12288, 5), (16384, 7), (32768, 15), (65536, 31),
                          (131072, 63), (262144, 127)]:
        assert count(total, 4096, 4, 0.5) == expect
        assert orc.trigger_count(total, 4096, 4, 0.5) == expect
    assert count(131072, 8192, 4, 0.5) == 31


BAD = [
    dict(n_heads=0), dict(head_dim=4), dict(n_sink=-1), dict(window=5, n_sink=4), dict(ratio=0.0),
    dict(ratio=1.5), dict(ratio=float("nan")), dict(cur_len=9000), dict(cur_len=-1),
]


@pytest.mark.parametrize("bad", BAD)
def test_plan_rejects_invalid_arguments(bad):
    a = dict(n_heads=8, head_dim=128, cur_len=8192, window=8192, n_sink=4, ratio=0.5)
    a.update(bad)
    rc, _ = fk.plan(_layout(), a["n_heads"], a["head_dim"], a["cur_len"], a["window"], a["n_sink"], a["ratio"],
                    check=False)
    assert rc == binding.E_INVALID


def test_plan_rejects_bad_layout():
    for field, val in [("dtype", 7), ("n_layers", 0), ("batch", 0), ("stride_token", 64), ("stride_token", 132),
                       ("stride_head", 12), ("pointer_table", 2), ("flags", 0x80)]:
        L = _layout()
        setattr(L, field, val)
        rc, _ = fk.plan(L, 8, 128, 8192, 8192, 4, 0.5, check=False)
        assert rc == binding.E_INVALID, field
    rc, _ = fk.plan(_layout(d=12), 8, 12, 8192, 8192, 4, 0.5, check=False)
    assert rc == binding.E_UNSUPPORTED
    assert fk.load().freqkv_plan(None, 8, 128, 1, 1, 0, 0.5, None) == binding.E_INVALID


def test_compress_validates_before_touching_the_device():
    """Every one of these returns before the first HIP call, so it runs without a GPU."""
    L = _layout()
    fake = 0x7F0000000000          # 16-byte aligned, never dereferenced on these paths
    # cache not full -> NOOP
    assert fk.compress(fake, fake, L, 8, 128, 100, 8192, 4, 0.5, check=False) == 1
    # ratio 1 -> identity, nothing enqueued
    assert fk.compress(fake, fake, L, 8, 128, 8192, 8192, 4, 1.0, check=False) == 0
    # null / misaligned cache pointers
    assert fk.compress(None, fake, L, 8, 128, 8192, 8192, 4, 0.5, check=False) == binding.E_INVALID
    assert fk.compress(fake + 2, fake, L, 8, 128, 8192, 8192, 4, 0.5, check=False) == binding.E_INVALID
    # missing / small / misaligned workspace (the matrix forms need one; the factored form does not)
    L.flags = fk.FLAG_DENSE
    assert fk.compress(fake, fake, L, 8, 128, 8192, 8192, 4, 0.5, check=False) == binding.E_WORKSPACE
    _, p = fk.plan(L, 8, 128, 8192, 8192, 4, 0.5)
    L.workspace, L.workspace_bytes = fake, p.workspace_min_bytes - 1
    assert fk.compress(fake, fake, L, 8, 128, 8192, 8192, 4, 0.5, check=False) == binding.E_WORKSPACE
    L.workspace, L.workspace_bytes = fake + 16, p.workspace_bytes
    assert fk.compress(fake, fake, L, 8, 128, 8192, 8192, 4, 0.5, check=False) == binding.E_WORKSPACE
    with pytest.raises(fk.FreqKVError):
        fk.compress(fake, fake, L, 8, 128, 8192, 8192, 4, 0.5)
    # invalid scalars
    assert fk.compress(fake, fake, L, 8, 128, 9000, 8192, 4, 0.5, check=False) == binding.E_INVALID


def test_plan_dropping_variant_needs_no_workspace():
    L = _layout()
    L.flags = fk.FLAG_DROPPING
    rc, p = fk.plan(L, 8, 128, 8192, 8192, 4, 0.5)
    assert rc == 0 and p.variant == 4
    assert (p.retained_len, p.new_len) == (4094, 4098)
    assert p.workspace_bytes == 0 and p.workspace_min_bytes == 0 and p.basis_bytes == 0 and p.flops_executed == 0
    assert p.bytes_algorithmic == pytest.approx(2 * 4094 * 128 * 2 * 512)


# ---------------------------------------------------------------- attention plan (host arithmetic only)

def test_attend_plan_llama3_shape():
    L = _layout()                                     # 32 layers x 8 KV heads x 8192 rows x 128, bf16
    rc, p = fk.attend_plan(L, 32, 8, 128, 8192)
    assert rc == 0
    assert p.heads_together == 4
    assert p.n_split >= 1 and p.chunk_rows % 32 == 0
    assert (p.n_split - 1) * p.chunk_rows < 8192 <= p.n_split * p.chunk_rows
    units = 32 * 8
    # K and V rows read once (bf16) plus the query read and the output written
    assert p.bytes_algorithmic == units * (2.0 * 8192 * 128 * 2 + 2.0 * 4 * 128 * 2)
    assert p.flops == units * 4 * 4.0 * 8192 * 128
    need = units * 4 * p.n_split * (128 + 2) * 4
    assert need <= p.workspace_bytes <= need + 256


@pytest.mark.parametrize("hq,hkv,gt", [(32, 32, 1), (8, 4, 2), (12, 4, 1), (24, 4, 2), (64, 8, 4)])
def test_attend_plan_head_grouping(hq, hkv, gt):
    L = _layout(n_heads=hkv, n_layers=2, cap=1024)
    _, p = fk.attend_plan(L, hq, hkv, 128, 1000)
    assert p.heads_together == gt
    assert (p.n_split - 1) * p.chunk_rows < 1000 <= p.n_split * p.chunk_rows


@pytest.mark.parametrize("cur", [1, 2, 15, 16, 17, 255, 256, 257, 8191])
def test_attend_plan_chunks_cover_any_length(cur):
    L = _layout(n_layers=1, n_heads=1, cap=8192)
    for d in (64, 128, 256):
        L.stride_token = d
        _, p = fk.attend_plan(L, 4, 1, d, cur)
        assert p.n_split >= 1
        assert (p.n_split - 1) * p.chunk_rows < cur <= p.n_split * p.chunk_rows


def test_attend_plan_invalid_arguments():
    L = _layout(n_layers=1, n_heads=2, cap=128)
    out = binding.AttendPlan()
    lib = fk.load()
    call = lambda *a: lib.freqkv_attend_plan(C.byref(L), *a, C.byref(out))
    assert call(4, 2, 128, 100) == 0
    assert call(5, 2, 128, 100) == -1           # query heads not a multiple of KV heads
    assert call(4, 0, 128, 100) == -1
    assert call(4, 2, 128, 0) == -1             # empty cache
    assert call(4, 2, 128, 129) == -1           # beyond the capacity
    assert call(4, 2, 96, 100) == -2            # head_dim not 64/128/256
    assert call(4, 2, 4, 100) == -1
    assert lib.freqkv_attend_plan(None, 4, 2, 128, 100, C.byref(out)) == -1
    assert lib.freqkv_attend_plan(C.byref(L), 4, 2, 128, 100, None) == -1
    # rows of one head are addressed by 32-bit byte offsets: a head whose rows span 4 GiB or more is refused
    big = _layout(n_layers=1, n_heads=1, cap=1 << 20)
    big.stride_token = 2048                     # token-major interleaving: 4 KiB between rows, 4 GiB per head
    big.stride_head = 128
    assert lib.freqkv_attend_plan(C.byref(big), 4, 1, 128, 1 << 19, C.byref(out)) == 0
    assert lib.freqkv_attend_plan(C.byref(big), 4, 1, 128, 1 << 20, C.byref(out)) == -2


def test_attend_decode_validates_without_gpu():
    """Argument errors are reported before any device call."""
    L = _layout(n_layers=1, n_heads=2, cap=128)
    lib = fk.load()
    f = lib.freqkv_attend_decode
    assert f(None, None, None, None, None, C.byref(L), 4, 2, 128, 100, -1, 10000.0, None) == -1
    assert f(16, 16, 16, 16, None, C.byref(L), 4, 2, 128, 100, -2, 10000.0, None) == -1       # q_pos
    assert f(16, 16, 16, 16, None, C.byref(L), 4, 2, 128, 100, -1, -5.0, None) == -1          # rotary base
    assert f(16, 16, 16, 16, None, C.byref(L), 4, 2, 128, 100, -1, 10000.0, None) == -3       # no workspace
    assert f(24, 16, 16, 16, None, C.byref(L), 4, 2, 128, 100, -1, 10000.0, None) == -1       # q misaligned


def test_compress_ragged_validates_without_gpu():
    L = _layout(n_layers=1, batch=3, n_heads=2, cap=128)
    lib = fk.load()
    f = lib.freqkv_compress_ragged
    lens = (C.c_int32 * 3)(10, 20, 30)
    out = (C.c_int32 * 3)()
    assert f(16, 16, C.byref(L), 2, 128, None, out, 64, 4, 0.5, None) == -1
    assert f(None, 16, C.byref(L), 2, 128, lens, out, 64, 4, 0.5, None) == -1
    assert f(16, 16, C.byref(L), 2, 128, lens, out, 64, 4, 0.5, None) == 1          # nobody reached the window
    assert list(out) == [10, 20, 30]
    lens[1] = 129                                                                     # beyond the capacity
    assert f(16, 16, C.byref(L), 2, 128, lens, out, 64, 4, 0.5, None) == -1
    lens[1] = 64                                                                      # triggers, but no workspace
    assert f(16, 16, C.byref(L), 2, 128, lens, out, 64, 4, 0.5, None) == -3
    assert f(16, 16, C.byref(L), 2, 128, lens, out, 64, 4, 1.5, None) == -1          # ratio


def test_prefill_plan():
    L = _layout()                                     # 32 layers x 8 KV heads x 8192 rows x 128, bf16
    out = binding.PrefillPlan()
    rc, p = fk.attend_prefill_plan(L, 32, 8, 128, 8192, 4094)
    assert rc == 0 and p.key_tiles == 256 and p.query_blocks == 128
    # causal flops: query i sees cur_len - q_len + i + 1 rows
    rows = sum(8192 - 4094 + i + 1 for i in range(4094))
    assert p.flops == 32 * 32 * 4.0 * 128 * rows
    units = 32 * 8
    need = 8192 * 64 * 8 + 2 * units * 256 * 32 * 128 * 2          # rotary table, rotated keys, transposed values
    assert need <= p.workspace_bytes <= need + 1024
    lib = fk.load()
    call = lambda *a: lib.freqkv_attend_prefill_plan(C.byref(L), *a, C.byref(out))
    assert call(32, 8, 128, 8192, 0) == -1 and call(32, 8, 128, 8192, 8193) == -1
    assert call(32, 8, 64, 8192, 100) == -2           # head_dim 128 only
    assert call(33, 8, 128, 8192, 100) == -1
    L.dtype = fk.F32
    assert call(32, 8, 128, 8192, 100) == -2          # bf16 only


def test_build_rejects_packed_fp32_in_device_code(tmp_path):
    """The build keeps the device assembly of every file and fails on packed fp32 arithmetic.  Here: a probe
    that the compiler turns into v_pk_fma_f32 without the feature flag and into scalar code with it (the host
    pass of hipcc does not know the flag and says so: harmless, the device pass is what counts)."""
    from paper_2505_00570_amd import build as hb
    src = tmp_path / "probe.hip"
    src.write_text("#include <hip/hip_runtime.h>\n"
                   "__global__ void k(float2* a, const float2* b) { int i = threadIdx.x; float2 x = a[i], y = b[i];\n"
                   "  x.x = x.x * y.x + 1.f; x.y = x.y * y.y + 1.f; a[i] = x; }\n")
    flag = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    counts = []
    for extra in ([], flag):
        out = tmp_path / ("with.s" if extra else "without.s")
        subprocess.check_call([hb.HIPCC, "--offload-arch=gfx950", "-O3", "--cuda-device-only", "-S"] + extra +
                              [str(src), "-o", str(out)], stderr=subprocess.DEVNULL)
        counts.append(hb.check_device_asm(str(out))[0])
    assert counts[0] >= 1 and counts[1] == 0
    # the library's own device code, as built: no packed fp32, no foreign use of M0
    for name in hb.SOURCES:
        asm = os.path.join(hb.OBJ_DIR, name.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s"))
        if os.path.exists(asm):
            assert hb.check_device_asm(asm) == (0, 0), name
