"""The C ABI used from plain C: tests/c_client/abi_client.c is compiled with gcc against
include/mmee.h, linked with the built library and run as its own process (no Python, no torch
in it); what it prints is compared with the oracle."""
import os
import subprocess

import pytest

import oracle as O

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIBDIR = os.path.join(ROOT, "paper_2604_03446_amd")
SRC = os.path.join(ROOT, "tests", "c_client", "abi_client.c")


def test_c_program_against_oracle(tmp_path):
    exe = str(tmp_path / "abi_client")
    subprocess.run(["gcc", "-O1", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), SRC, "-o", exe,
                    "-L", LIBDIR, "-lmmee", "-Wl,-rpath," + LIBDIR], check=True)
    w = dict(B=1, H=2, N=24, d=4, word_bytes=2, tiling_mode=1, c_softmax=10)
    h = dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=700,
             e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=8.0, gb_bw=32.0)
    first, n = 123456789, 4099
    args = [w[k] for k in ("B", "H", "N", "d", "word_bytes", "tiling_mode", "c_softmax")] + \
           [h[k] for k in ("pe_rows", "pe_cols", "n_arrays", "rf_bytes", "gb_bytes", "e_dram", "e_gb", "e_rf",
                           "e_mac", "dram_bw", "gb_bw")] + [first, n]
    run = subprocess.run([exe] + [repr(a) for a in args], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stderr
    lines = run.stdout.splitlines()
    ow, oh = O.workload(w), O.hw(h)
    assert lines[0] == "space %d" % O.space_size(ow, oh)
    want = O.eval_batch(ow, oh, first, n)
    got = [ln.split() for ln in lines if ln.startswith("cost ")]
    assert len(got) == n
    for rec, ln in zip(want, got):
        real = rec["reason"] != 1
        ints = [int(rec[f]) if real else 0 for f in ("bs_words", "da_words", "br_words", "mac_total", "comp_cycles")]
        assert [int(x) for x in ln[2:7]] == ints, ln
        assert float.fromhex(ln[7]) == rec["energy_pj"] and float.fromhex(ln[8]) == rec["latency_cycles"], ln
        assert (int(ln[9]), int(ln[10])) == (int(rec["valid"]), int(rec["reason"])), ln
    rc, idx, cost, n_valid, _ = O.search_all(ow, oh)
    assert rc == 0 and n_valid > 0
    best = [ln.split() for ln in lines if ln.startswith("best ")]
    assert len(best) == 4
    for obj, ln in enumerate(best):
        assert int(ln[1]) == obj and int(ln[2]) == idx[obj], ln
        assert float.fromhex(ln[3]) == cost[obj].energy_pj and float.fromhex(ln[4]) == cost[obj].latency_cycles
        m, _, _ = O.evaluate(ow, oh, idx[obj])
        assert [int(x) for x in ln[6:10]] == list(m.xG)
        assert ln[11] == "".join(str(x) for x in m.order) and ln[13] == "".join(str(x) for x in m.level)
        assert (int(ln[15]), int(ln[17]), int(ln[18]), int(ln[20])) == (m.recompute, m.stat1, m.stat2, m.fused)
