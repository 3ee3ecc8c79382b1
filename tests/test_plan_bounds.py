"""Every address the GEMM kernels form under the launch configurations the library picks stays inside the buffers
the caller handed over -- checked on the host, for every kernel family, over a grid of shapes.

A host model walks each launch the way its kernel does: the same partition of the work over workgroups (taken from
the library's own qoq_query_gemm_config and qoq_gemm_workspace_bytes), the same iteration structure (csrc/qoq_walk.h,
the header the kernels themselves include), the same clamps for rows past M, groups past the end of a run or slice,
fragments past N, and the copies issued past the end of a run.  Each global address the model forms -- packed codes,
level-2 metadata, channel scales and zeros, INT8 activations, token scales and sums, partial tiles and counters in the
workspace -- is checked against the size of its buffer.  A copy that read group G of the last token row (128 bytes
past the activations) once went unnoticed until it faulted on the GPU; this test makes that class of mistake fail
on the CPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHECKER = r'''
#include "qoq_layout.h"
#include "qoq_walk.h"
#include <algorithm>
#include <cstdio>
#include <cstdlib>
using namespace qoq;
typedef long long ll;
static ll M, N, K, G, ws_bytes, counters_bytes; static int mode, tile, split;
static ll n_codes, n_meta, n_scales, n_zeros, n_qx, n_sx, n_rs;
static const char* fail = nullptr; static ll fail_off, fail_len, fail_size;
static inline void chk(const char* what, ll off, ll len, ll size) {
    if (!fail && (off < 0 || off + len > size)) { fail = what; fail_off = off; fail_len = len; fail_size = size; }
}
static ll cdiv(ll a, ll b) { return (a + b - 1) / b; }

// ---- LDS-staged and register-streaming kernels: units = (64-channel block, group) dealt in runs ----------------
static void check_stream(int MF, bool staged) {
    const ll blocks = N / 64, total = blocks * G, nwg = split, upw = cdiv(total, nwg), nf_total = N / 16, m_tiles = cdiv(M, 16 * MF);
    const ll kEl = MF * 256;                                   // int4 elements of a partial tile
    for (ll mt = 0; mt < m_tiles; ++mt) for (ll wg = 0; wg < nwg; ++wg) {
        const ll m0 = mt * 16 * MF;
        const int u0 = (int)std::min(total, wg * upw), u1 = (int)std::min(total, u0 + upw);
        if (u0 >= u1) continue;
        RunShape run = make_run(u0, u1, (int)G, staged ? 2 : 8);
        for (int it = 0; it < run.T; ++it) {                   // copies past the end of the run repeat iteration T-1
            const IterInfo o = run_iteration(run, it);
            if (staged) {
                for (int e = 0; e < 2; ++e) {
                    const ll gsel = std::min<ll>(o.g + (e < o.n ? e : 0), G - 1);
                    for (int f = 0; f < 4; ++f) chk("codes", ((o.block * 4 + f) * G + gsel) << 10, 1024, n_codes);
                    for (int b = 0; b < 2 * MF; ++b) for (int r = 0; r < 16; ++r) {
                        const ll row = std::min(m0 + (b >> 1) * 16 + r, M - 1);
                        chk("qx", row * K + gsel * kGroup + (b & 1) * 64, 64, n_qx);
                    }
                    if (mode == 0) chk("meta", gsel * nf_total * 32 + (ll)o.block * 128, 128, n_meta);
                }
                chk("scales", (ll)o.block * 128, 128, n_scales);
                if (mode == 1) chk("zeros", (ll)o.block * 64, 64, n_zeros);
            } else {
                for (int w = 0; w < o.n; ++w) {
                    const ll g = o.g + w;
                    for (int f = 0; f < 4; ++f) {
                        const ll nf = (ll)o.block * 4 + f;
                        chk("codes", (nf * G + g) * 1024, 1024, n_codes);
                        if (mode == 0) chk("meta", (g * nf_total + nf) * 32, 32, n_meta);
                    }
                    for (int mf = 0; mf < MF; ++mf) for (int r = 0; r < 16; ++r)
                        chk("qx", std::min(m0 + mf * 16 + r, M - 1) * K + g * kGroup, 128, n_qx);
                }
            }
            if (o.seg_end) {                                    // epilogue constants / partial tile of the block
                chk("scales", (ll)o.block * 128, 128, n_scales);
                if (mode == 1) chk("zeros", (ll)o.block * 64, 64, n_zeros);
                if (!o.complete) {
                    chk("counter", (mt * blocks + o.block) * 4, 4, counters_bytes);
                    const ll wf = ((ll)o.block * G) / upw, wl = ((ll)o.block * G + G - 1) / upw;   // contributors
                    for (ll ww = wf; ww <= wl; ++ww) for (int which = 0; which < 2; ++which)
                        chk("parts", counters_bytes + ((mt * nwg + ww) * 2 + which) * kEl * 16, kEl * 16, ws_bytes);
                }
            }
        }
        chk("sx", std::min(m0 + 16 * MF - 1, M - 1) * 2, 2, n_sx);
    }
}

// ---- blocks in lockstep: whole pairs / quads per workgroup ---------------------------------------------------------
static void check_lockstep(int NB, int MF) {
    const ll sets = N / (64 * NB), upw = cdiv(sets, split), nf_total = N / 16, m_tiles = cdiv(M, 16 * MF);
    if (N % (64 * NB)) { fail = "lockstep width"; return; }
    for (ll mt = 0; mt < m_tiles; ++mt) for (ll wg = 0; wg < split; ++wg) {
        const ll m0 = mt * 16 * MF, sb0 = std::min(sets, wg * upw), sb1 = std::min(sets, sb0 + upw);
        if (sb0 >= sb1) continue;
        const ll T = (sb1 - sb0) * ((G + 1) / 2);
        ll csb = sb0, cg = 0, cleft = T;
        for (ll it = 0; it < T + 2; ++it) {                   // the copy front, kRing - 1 issues past the end included
            const int two = cg + 1 < G ? 1 : 0;
            for (int pk = 0; pk < 2; ++pk) {
                const ll gsel = cg + (pk & two);
                for (int b = 0; b < 2 * MF; ++b) for (int r = 0; r < 16; ++r)
                    chk("qx", std::min(m0 + (b >> 1) * 16 + r, M - 1) * K + gsel * kGroup + (b & 1) * 64, 64, n_qx);
                if (mode == 0) chk("meta", gsel * nf_total * 32 + csb * NB * 128, NB * 128, n_meta);
                for (int f = 0; f < 4 * NB; ++f) chk("codes", ((csb * 4 * NB + f) * G + gsel) << 10, 1024, n_codes);
            }
            chk("scales", csb * NB * 128, NB * 128, n_scales);
            if (mode == 1) chk("zeros", csb * NB * 64, NB == 2 ? 128 : 256, n_zeros);
            if (cleft > 1) { --cleft; cg += 2; if (cg >= G) { cg = 0; ++csb; } }
        }
    }
}

// ---- activation-stationary kernels ---------------------------------------------------------------------------------
static void check_astat(int tl) {
    const int MF = tl / 16, waves = 8, cap = waves * (tl == 64 ? 4 : 8);
    ll S = cdiv(G, cap), gps = cdiv(G, S); S = cdiv(G, gps);
    const ll nf_total = N / 16, nwg = split, base = nf_total / nwg, rem = nf_total - base * nwg, m_tiles = cdiv(M, tl), kEl = MF * 64;
    const ll jeff = cdiv(gps, waves);
    if (jeff * MF > 16) { fail = "astat capacity"; return; }
    for (ll mt = 0; mt < m_tiles; ++mt) for (ll sl = 0; sl < S; ++sl) for (ll wg = 0; wg < nwg; ++wg) {
        const ll m0 = mt * tl, f0 = wg * base + std::min(wg, rem), f1 = f0 + base + (wg < rem ? 1 : 0);
        if (f0 >= f1) continue;
        const ll g_lo = sl * gps, g_hi = std::min(G, g_lo + gps);
        if (g_lo >= g_hi) { fail = "astat empty slice"; return; }
        if (wg == 0) {   // the activation preload does not depend on the workgroup's fragments
            // compiled group capacity per wave: the smallest instantiation that holds jeff groups
            const ll J = tl == 64 ? std::max<ll>(jeff, 2) : (jeff <= 4 ? 4 : 8);
            const ll JP = J >= 8 ? 8 : 4, RP = std::min<ll>(128 / JP, MF * 16), row_passes = MF * 16 / RP, j_passes = cdiv(J, JP), dma = RP * JP / 8;
            if (dma * 1024 > 16384) { fail = "astat staging"; return; }
            for (int w = 0; w < waves; ++w) for (ll rp = 0; rp < row_passes; ++rp) for (ll jp = 0; jp < j_passes; ++jp) {
                for (ll flat = 0; flat < dma * 64; ++flat) {
                    const ll row_local = flat / (JP * 8), pos = flat % (JP * 8);
                    const ll row = std::min(m0 + rp * RP + row_local, M - 1);
                    const ll col = std::min((g_lo + w * jeff + jp * JP) * kGroup + ((pos ^ (row_local & 15)) * 16), K - 16);
                    chk("qx", row * K + col, 16, n_qx);
                }
                for (ll mm = 0; mm < RP / 16; ++mm) for (ll jj = 0; jj < JP; ++jj) for (int lane = 0; lane < 64; ++lane) for (int ks = 0; ks < 2; ++ks) {
                    const ll row_local = mm * 16 + (lane & 15), L = jj * 8 + ks * 4 + (lane >> 4);
                    chk("staging", row_local * JP * 128 + ((L ^ (row_local & 15)) * 16), 16, dma * 1024);
                }
            }
        }
        for (ll nf = f0; nf < f1; ++nf) {
            for (int w = 0; w < waves; ++w) for (ll j = 0; j < std::max<ll>(jeff, 1) + 3; ++j) {   // slots past jeff re-read the last group
                const ll g = std::min(g_lo + w * jeff + std::min(j, jeff - 1), g_hi - 1);
                chk("codes", (nf * G + g) * 1024, 1024, n_codes);
                if (mode == 0) chk("meta", (g * nf_total + nf) * 32, 32, n_meta);
            }
            chk("scales", ((nf >> 2) * 64 + 48 + 4 * (nf & 3)) * 2, 8, n_scales);
            if (mode == 1) chk("zeros", (nf >> 2) * 64 + 48 + 4 * (nf & 3), 4, n_zeros);
            if (S > 1) {
                chk("counter", (mt * nf_total + nf) * 4, 4, counters_bytes);
                chk("parts", counters_bytes + ((mt * nf_total + nf) * S + sl) * kEl * 16, kEl * 16, ws_bytes);
            }
        }
    }
}

// ---- compute-bound kernel -------------------------------------------------------------------------------------------
static void check_mma() {
    const ll tm = (tile == 129 || tile == 132) ? 128 : 256, tn = tile == 130 ? 128 : tile == 131 ? 192 : 256;
    const ll n_tiles = cdiv(N, tn), m_tiles = cdiv(M, tm), S = split, gps = cdiv(G, S), nf_total = N / 16;
    const ll kACopies = tm / 64, kUnits = tn / 16, kWCopies = kUnits / 4, tiles = n_tiles * m_tiles;
    if (cdiv(G, gps) != S) { fail = "mma slices"; return; }
    for (ll t = 0; t < tiles; ++t) for (ll sl = 0; sl < S; ++sl) {
        const ll tmi = t / n_tiles, tni = t % n_tiles, m_base = tmi * tm, n_base = tni * tn, nf_base = tni * kUnits;
        const ll g_first = sl * gps, Gs = std::min(G - g_first, gps), g_last = g_first + Gs - 1;
        if (Gs < 1) { fail = "mma empty slice"; return; }
        for (ll g = g_first; g <= g_last; ++g) for (int wave = 0; wave < 4; ++wave) {
            for (int hf = 0; hf < 2; ++hf) for (ll c = 0; c < kACopies; ++c) for (int r = 0; r < 8; ++r)
                chk("qx", std::min(m_base + ((wave * 2 + hf) * kACopies + c) * 8 + r, M - 1) * K + g * kGroup, 128, n_qx);
            for (ll u = 0; u < kWCopies; ++u)
                chk("codes", std::min(nf_base + wave * kWCopies + u, nf_total - 1) * G * 1024 + g * 1024, 1024, n_codes);
            if (mode == 0) for (int lane = 0; lane < 64; ++lane) {
                const ll ml = std::min<ll>(lane, kWCopies * 8 - 1);
                chk("meta", g * nf_total * 32 + std::min(nf_base + wave * kWCopies + (ml >> 3), nf_total - 1) * 32 + (ml & 7) * 4, 4, n_meta);
            }
        }
        for (int d = 0; d < 256; ++d) {                        // epilogue constants: 256 of each, clamped
            if (d < 128) chk("sx", m_base * 2 + std::min<ll>(d, (M - m_base - 1) >> 1) * 4, 4, n_sx);
            if (d < 128) chk("scales", n_base * 2 + std::min<ll>(d, ((N - n_base) >> 1) - 1) * 4, 4, n_scales);
            if (mode == 1) chk("rowsum", (m_base + std::min<ll>(d, M - m_base - 1)) * 4, 4, n_rs);
            if (mode == 1 && d < 64) chk("zeros", n_base + std::min<ll>(d, ((N - n_base) >> 2) - 1) * 4, 4, n_zeros);
        }
        if (S > 1) {
            chk("counter", t * 4, 4, counters_bytes);
            chk("parts", counters_bytes + (t * S + sl) * tm * tn * 4, tm * tn * 4, ws_bytes);
        }
    }
}

int main(int argc, char** argv) {
    FILE* f = fopen(argv[1], "r");
    long checked = 0;
    while (fscanf(f, "%lld %lld %lld %d %d %d %lld %lld", &M, &N, &K, &mode, &tile, &split, &ws_bytes, &counters_bytes) == 8) {
        G = K / kGroup;
        n_codes = N * K / 2; n_meta = mode == 0 ? N * G * 2 : 0; n_scales = 2 * N; n_zeros = mode == 1 ? N : 0;
        n_qx = M * K; n_sx = (2 * M + 3) / 4 * 4; n_rs = 4 * M;       // (token scales are read in whole 4-byte words)
        fail = nullptr;
        if (tile == 64) check_stream(4, true);
        else if (tile == 32 || tile == 16) check_stream(tile / 16, false);
        else if (tile == 65) check_lockstep(2, 4);
        else if (tile == 66) check_lockstep(4, 4);
        else if (tile == 67) check_lockstep(2, 2);
        else if (tile == 68) check_lockstep(2, 1);
        else if (tile >= 69 && tile <= 71) check_astat(tile == 71 ? 64 : tile == 70 ? 32 : 16);
        else check_mma();
        if (fail) {
            printf("M=%lld N=%lld K=%lld mode=%d tile=%d split=%d: %s access [%lld, +%lld) outside %lld bytes\n", M, N, K, mode, tile,
                   split, fail, fail_off, fail_len, fail_size);
            return 1;
        }
        ++checked;
    }
    printf("ok %ld launch plans\n", checked);
    return 0;
}
'''


def _plans(api):
    shapes = [(N, K) for N in (64, 192, 256, 4096, 12288, 22016, 57344) for K in (128, 1152, 4096, 11008, 28672)]
    Ms = (1, 7, 16, 17, 32, 33, 63, 64, 65, 100, 128, 130, 200, 256, 300, 512, 1000, 1024, 4096)
    forced = [(0, 0), (16, 0), (16, 7), (32, 0), (32, 9), (64, 0), (64, 5), (65, 0), (65, 3), (66, 0), (67, 0), (68, 2),
              (69, 0), (69, 5), (70, 0), (71, 0), (71, 3), (128, 0), (128, 3), (129, 0), (129, 2), (130, 0), (131, 0), (131, 2),
              (132, 0)]
    lines = []
    for cfg in forced:
        api.set_gemm_config(*cfg)
        try:
            for N, K in shapes:
                if cfg != (0, 0) and (N, K) not in ((192, 1152), (256, 128), (4096, 4096), (4096, 11008), (22016, 4096), (12288, 1152)):
                    continue                                   # forced configurations: a smaller set of shapes
                for M in Ms:
                    if cfg != (0, 0) and M not in (1, 17, 64, 100, 300, 1024):
                        continue
                    for mode in (0, 1):
                        tile, split = api.query_gemm_config(M, N, K, mode)
                        ws = api.gemm_workspace_bytes(M, N, K, mode)
                        lines.append((M, N, K, mode, tile, split, ws))
        finally:
            api.set_gemm_config(0, 0)
    return lines


def test_every_launch_plan_stays_inside_its_buffers(tmp_path):
    import ctypes

    from paper_2405_04532_amd import api
    L = api.lib()
    plans = _plans(api)
    assert len(plans) > 1500
    # the counters sit at the start of the workspace: their size is what separates them from the partial tiles
    src = tmp_path / "bounds.cpp"
    src.write_text(CHECKER)
    exe = tmp_path / "bounds"
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-I", os.path.join(ROOT, "paper_2405_04532_amd", "csrc"), str(src), "-o", str(exe)])
    listing = tmp_path / "plans.txt"
    with open(listing, "w") as f:
        for M, N, K, mode, tile, split, ws in plans:
            f.write("%d %d %d %d %d %d %d %d\n" % (M, N, K, mode, tile, split, ws, _counter_bytes(M, N, K, tile, split, ws)))
    out = subprocess.run([str(exe), str(listing)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok"), out.stdout[-2000:]
    assert int(out.stdout.split()[1]) == len(plans)


def _counter_bytes(M, N, K, tile, split, ws):
    """Size of the counter area at the start of the workspace (256-byte aligned), as the header states the layout."""
    if ws == 0:
        return 0
    al = lambda v: (v + 255) // 256 * 256
    if tile <= 64:
        return al(-(-M // tile) * (N // 64) * 4)
    if 69 <= tile <= 71:
        t = {69: 16, 70: 32, 71: 64}[tile]
        return al(-(-M // t) * (N // 16) * 4)
    tm = 128 if tile in (129, 132) else 256
    tn = 128 if tile == 130 else 192 if tile == 131 else 256
    return al(-(-M // tm) * -(-N // tn) * 4)


def test_the_checker_catches_a_planted_overrun(tmp_path):
    """The mistake that once faulted on the GPU, planted in the host model's input: a run that is allowed to reach
    group G (one past the last) of the last token row must be reported."""
    src = tmp_path / "bounds.cpp"
    src.write_text(CHECKER.replace("const ll gsel = std::min<ll>(o.g + (e < o.n ? e : 0), G - 1);",
                                   "const ll gsel = o.g + e;"))
    exe = tmp_path / "bounds"
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-I", os.path.join(ROOT, "paper_2405_04532_amd", "csrc"), str(src), "-o", str(exe)])
    listing = tmp_path / "plans.txt"
    listing.write_text("64 256 1152 0 64 8 0 0\n")          # nine groups: the last iteration of a block has one unit
    out = subprocess.run([str(exe), str(listing)], capture_output=True, text=True)
    assert out.returncode == 1 and "outside" in out.stdout
