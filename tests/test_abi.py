"""The C-ABI library loads and exports every symbol the header declares; host-only entry
points and argument validation behave as documented (no GPU compute calls)."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qoq_w4a8.h")


@pytest.fixture(scope="module")
def api():
    from paper_2405_04532_amd import api as a
    if not os.path.exists(a.LIB_PATH):
        from paper_2405_04532_amd import build
        build.build()
    return a


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qoq_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header(api):
    names = _declared()
    assert len(names) >= 10
    handle = api.lib()
    for n in names:
        assert hasattr(handle, n), n
    assert set(names) == set(api.EXPORTS)


def test_header_compiles_as_c():
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", HEADER])


def test_packed_bytes_and_status(api):
    assert api.packed_bytes(256, 256) >= 256 * 256 // 2 + 256 * 2 * 2 + 256 * 2
    assert api.packed_bytes(256, 256) % 256 == 0
    # algorithmic size plus at most the 0.5-byte-per-group metadata padding and section alignment
    n, k = 4096, 4096
    algo = n * k // 2 + n * (k // 128) * 3 // 2 + 2 * n
    assert algo <= api.packed_bytes(n, k) <= algo + n * (k // 128) // 2 + 2048
    assert api.packed_bytes(256, 100) == 0 and api.packed_bytes(100, 256) == 0 and api.packed_bytes(256, 256, 7) == 0
    assert api.packed_bytes(256, 256, api.QOQ_PER_CHANNEL) >= 256 * 128 + 256 * 3
    assert api.status_string(0) == "QOQ_OK"
    assert "SHAPE" in api.status_string(2) and "UNKNOWN" in api.status_string(99)


def test_argument_validation_without_gpu(api):
    L = api.lib()
    buf = (ctypes.c_uint8 * 64)()
    p = ctypes.addressof(buf)
    p = (p + 15) & ~15
    assert L.qoq_pack_weights(p, 256, 100, 0, p, None) == 2       # K % 128
    assert L.qoq_pack_weights(p, 100, 256, 0, p, None) == 2       # N % 64
    assert L.qoq_pack_weights(None, 256, 256, 0, p, None) == 1
    assert L.qoq_pack_weights(p + 4, 256, 256, 0, p, None) == 3
    assert L.qoq_quant_act_per_token(p, 4, 100, p, p, None, None, None) == 2
    assert L.qoq_quant_act_per_token(None, 4, 128, p, p, None, None, None) == 1
    assert L.qoq_quant_act_per_token(None, 0, 128, None, None, None, None, None) == 0   # empty batch
    assert L.qoq_w4a8_gemm(p, p, None, p, 4, 256, 256, 3, p, None, 0, None) == 2
    assert L.qoq_w4a8_gemm(p, p, None, p, 4, 256, 256, 1, p, None, 0, None) == 1        # per-channel needs rowsum
    assert L.qoq_w4a8_gemm(p, p, None, p, 0, 256, 256, 0, p, None, 0, None) == 0        # M = 0
    assert L.qoq_w4a8_gemm(p, p, None, p, 4, 256, 256, 0, None, None, 0, None) == 1
    assert L.qoq_w4a8_gemm_i32(p, None, p, 4, 256, 256, 0, p + 8, None, 0, None) == 3
    # the per-token vectors are read in 4-byte words: a token-scale pointer that is only 2-byte aligned is refused
    assert L.qoq_w4a8_gemm(p, p + 2, None, p, 4, 256, 256, 0, p, None, 0, None) == api.QOQ_ERR_ALIGN == 3
    assert L.qoq_w4a8_gemm(p, p + 4, None, p, 4, 256, 256, 1, p, None, 0, None) == api.QOQ_ERR_NULL      # (aligned: next check)
    assert L.qoq_w4a8_gemm(p, p, p + 2, p, 4, 256, 256, 1, p, None, 0, None) == api.QOQ_ERR_ALIGN
    assert L.qoq_w4a8_gemm_token_sum(p, p, p + 2, p, 4, 256, 256, p, None, 0, None) == api.QOQ_ERR_ALIGN
    assert "BLOB" in api.status_string(api.QOQ_ERR_BLOB) and api.QOQ_ERR_BLOB == 4
    # a salience that is not finite has no place in an order
    sal = (ctypes.c_float * 4)(1.0, float("nan"), 3.0, 2.0)
    perm = (ctypes.c_int32 * 4)()
    assert L.qoq_channel_order_host(sal, 4, perm) == api.QOQ_ERR_SHAPE
    sal[1] = float("inf")
    assert L.qoq_channel_order_host(sal, 4, perm) == api.QOQ_ERR_SHAPE
    sal[1] = 0.5
    assert L.qoq_channel_order_host(sal, 4, perm) == 0 and list(perm) == [2, 3, 0, 1]
    assert L.qoq_set_gemm_config(48, 0) == 2 and L.qoq_set_gemm_config(0, -1) == 2 and L.qoq_set_gemm_config(0, 0) == 0
    # split-k problems must come with a workspace
    need = api.gemm_workspace_bytes(16, 256, 4096)
    assert need >= 2 * 16 * 256 * 4 and need % 16 == 0          # counters + at least two partial tiles
    assert L.qoq_w4a8_gemm(p, p, None, p, 16, 256, 4096, 0, p, None, 0, None) == api.QOQ_ERR_WORKSPACE == 5
    assert L.qoq_w4a8_gemm(p, p, None, p, 16, 256, 4096, 0, p, p, need - 16, None) == api.QOQ_ERR_WORKSPACE
    assert api.gemm_workspace_bytes(4096, 4096, 4096) == 0
    assert L.qoq_gemm_workspace_prepare(None, 64, None) == 1
    assert L.qoq_gemm_workspace_prepare(p, 24, None) == 3
    assert L.qoq_gemm_workspace_prepare(None, 0, None) == 0


def test_launch_plan_host_logic(api):
    """The host-side choice of kernel, tile and partition (no device work): always a runnable configuration (a streaming
    partition gives every workgroup at least two units and a token tile at most one workgroup per CU), narrow layers cut the tokens into
    smaller tiles that run side by side, wide layers keep the 64-token tile, forced values are honoured."""
    L = api.lib()
    t, k = ctypes.c_int(0), ctypes.c_int(0)
    assert L.qoq_query_gemm_config(4, 100, 256, 0, ctypes.byref(t), ctypes.byref(k)) == 2
    assert L.qoq_query_gemm_config(4, 256, 256, 0, None, ctypes.byref(k)) == 1
    for N in (64, 256, 4096, 12288, 22016, 57344):
        for K in (128, 1152, 4096, 11008, 28672):
            for M in (1, 7, 16, 17, 32, 33, 64, 65, 100, 128, 200, 256, 512, 1024, 4096):
                tile, split = api.query_gemm_config(M, N, K)
                assert tile in (16, 32, 64, 65, 66, 67, 68, 69, 70, 71, 128, 129, 130, 131, 132) and split >= 1, (M, N, K, tile, split)
                units = (N // 64) * (K // 128)
                if tile in (69, 70, 71):
                    assert split <= min(256, N // 16)
                elif tile in (65, 66, 67, 68):
                    width = 256 if tile == 66 else 128
                    assert N % width == 0 and split <= N // width
                elif tile <= 64:
                    assert split <= min(256, max(1, (units + 1) // 2)), (M, N, K, tile, split)
                else:
                    assert M > 64 and split <= K // 128
                assert api.gemm_workspace_bytes(M, N, K) % 16 == 0
    assert api.query_gemm_config(64, 4096, 4096) == (70, 128)       # narrow: two 32-token tiles x 128 workgroups, activations resident
    assert api.query_gemm_config(64, 12288, 4096) == (64, 192)      # one block per workgroup already
    assert api.query_gemm_config(64, 22016, 4096) == (71, 256)      # widest layer: activations resident, 16-channel fragments dealt to 256 workgroups
    assert api.query_gemm_config(64, 22016, 4096, api.QOQ_PER_CHANNEL) == (71, 256)   # in either mode
    assert api.query_gemm_config(64, 4096, 11008) == (32, 128)      # K too long for one workgroup's registers: K spread over the chip
    assert api.query_gemm_config(16, 12288, 4096) == (69, 256)
    assert api.query_gemm_config(1024, 12288, 4096)[0] == 131       # 256 tiles of 256 x 192
    api.set_gemm_config(32, 5)
    try:
        assert api.query_gemm_config(200, 4096, 4096) == (32, 5)
    finally:
        api.set_gemm_config(0, 0)


def test_layout_is_a_bijection(tmp_path):
    """Host logic of the packed layout: (n, k) -> (byte, nibble) is one-to-one and onto."""
    src = tmp_path / "t.cpp"
    src.write_text(r'''
#include <cstdio>
#include <set>
#include <utility>
#include "qoq_layout.h"
int main() {
  const long N = 128, K = 384, G = K / 128;
  std::set<std::pair<size_t,int>> seen;
  for (long n = 0; n < N; ++n) {
    long nf; int i; qoq::phys_row(n, nf, i);
    if (qoq::logical_row(nf, i) != n || i < 0 || i > 15 || nf < 0 || nf >= N / 16) return 1;
    for (long k = 0; k < K; ++k) {
      int sh; size_t off = qoq::code_dword_offset(nf, i, k / 128, G, (int)(k % 128), sh);
      if (off % 4 || off >= (size_t)N * K / 2 || sh % 4 || sh > 28) return 2;
      if (!seen.insert({off, sh}).second) return 3;
    }
  }
  if (seen.size() != (size_t)N * K) return 4;
  // one lane's 16 bytes hold 32 codes of ONE row and ONE group: k_local = kb*16+t and 64+kb*16+t
  for (int kb = 0; kb < 4; ++kb) for (int t = 0; t < 16; ++t) for (int s = 0; s < 2; ++s) {
    int sh; size_t off = qoq::code_dword_offset(3, 5, 1, G, s * 64 + kb * 16 + t, sh);
    size_t lane_base = ((size_t)(3 * G + 1) * 64 + (size_t)(kb * 16 + 5)) * 16;
    if (off < lane_base || off >= lane_base + 16 || (int)((off - lane_base) / 8) != s) return 5;
  }
  qoq::BlobLayout L = qoq::make_layout(4096, 4096, 0);
  if (L.codes_off % 256 || L.meta_off % 256 || L.scale_off % 256 || L.total % 256) return 6;
  if (L.meta_off < L.codes_off + (size_t)4096 * 4096 / 2) return 7;
  printf("ok\n");
  return 0;
}
''')
    exe = tmp_path / "t"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2405_04532_amd", "csrc"),
                           str(src), "-o", str(exe)])
    assert subprocess.run([str(exe)], capture_output=True, text=True).stdout.strip() == "ok"


def test_run_walk_closed_form(tmp_path):
    """Host logic of the streaming kernel: the closed form that gives any iteration of a workgroup's run
    (block, first group, units, segment end, whole block) equals stepping through the run unit by unit."""
    src = tmp_path / "w.cpp"
    src.write_text(r'''
#include "qoq_walk.h"
#include <cstdio>
#include <cstdlib>
using namespace qoq;
int main() {
    long checked = 0;
    for (int R = 1; R <= 8; R += (R == 2 ? 6 : 1))
    for (int G = 1; G <= 13; ++G)
        for (int u0 = 0; u0 < 4 * G + 3; ++u0)
            for (int U = 1; U <= 5 * G + 2; ++U) {
                const int u1 = u0 + U;
                RunShape r = make_run(u0, u1, G, R);
                // reference state machine
                int block = u0 / G, g = u0 - block * G, left = (G - g) < U ? (G - g) : U, rem = U - left, seg_first = g, it = 0;
                while (left > 0) {
                    const int n = left < R ? left : R;
                    if (it >= r.T) { printf("too many iterations G=%d u0=%d U=%d\n", G, u0, U); return 1; }
                    IterInfo o = run_iteration(r, it);
                    const bool wrapped = g + n >= G;
                    const int block_now = block, g_now = g;
                    g += n; left -= n;
                    bool seg_end = false;
                    if (left <= 0) { seg_end = true; if (rem > 0) { block += 1; g = 0; left = G < rem ? G : rem; rem -= left; } }
                    const bool complete = seg_end && seg_first == 0 && wrapped;
                    if (o.block != block_now || o.g != g_now || o.n != n || o.seg_end != seg_end || o.complete != complete) {
                        printf("mismatch G=%d u0=%d U=%d it=%d: got (%d,%d,%d,%d,%d) want (%d,%d,%d,%d,%d)\n", G, u0, U, it, o.block, o.g, o.n,
                               o.seg_end, o.complete, block_now, g_now, n, seg_end, complete);
                        return 1;
                    }
                    if (seg_end) seg_first = 0;
                    ++it; ++checked;
                }
                if (it != r.T) { printf("T mismatch G=%d u0=%d U=%d: %d vs %d\n", G, u0, U, it, r.T); return 1; }
            }
    printf("ok %ld iterations checked\n", checked);
    return 0;
}
''')
    exe = tmp_path / "w"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2405_04532_amd", "csrc"),
                           str(src), "-o", str(exe)])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok"), out.stdout
