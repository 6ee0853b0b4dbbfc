"""CPU-only checks of the scripts that write the hand-scheduled assembly loops (head sizes 128 and 64):
the text is deterministic, stays inside the registers it declares, fits the LDS of a compute unit and uses
none of the instruction forms this code base rules out."""
import os
import re
import subprocess
import sys

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2407_00611_amd", "csrc")

# script, macro prefix, pinned input registers (VGPRs, SGPRs) handed over by the C++ shell
GENERATORS = [
    ("gen_fwd_asm.py", "ST_FWD_FAST", range(224, 240), range(32, 47)),
    ("gen_bwd_dq_asm.py", "ST_DQ_FAST", range(160, 180), range(32, 44)),
    ("gen_bwd_dkv_asm.py", "ST_DKV_FAST", range(176, 192), list(range(32, 64))),
]
CASES = [(g, d) for g in GENERATORS for d in (128, 64)]


def _run(script, d):
    args = [sys.executable, os.path.join(CSRC, script)] + (["64"] if d == 64 else [])
    r = subprocess.run(args, capture_output=True, text=True, env={k: v for k, v in os.environ.items() if not k.startswith("ST_GEN_")})
    assert r.returncode == 0, r.stderr
    return r.stdout


def _regs(kind, text):
    """Every register of one file (v, a or s) that the text names, single or as a range."""
    used = set()
    for m in re.finditer(rf"(?<![A-Za-z0-9_]){kind}(\d+)(?![\d:\]])", text):
        used.add(int(m.group(1)))
    for m in re.finditer(rf"(?<![A-Za-z0-9_]){kind}\[(\d+):(\d+)\]", text):
        used.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return used


@pytest.mark.parametrize("gen,d", CASES, ids=[f"{g[0]}-{d}" for g, d in CASES])
def test_generated_loop_invariants(gen, d):
    script, prefix, in_v, in_s = gen
    prefix += "64" if d == 64 else ""
    text = _run(script, d)
    assert text == _run(script, d), "generator output must be deterministic"
    lds = int(re.search(rf"#define {prefix}_LDS_BYTES (\d+)", text).group(1))
    assert 0 < lds <= 160 * 1024
    assert int(re.search(rf"#define {prefix}_NINSTR (\d+)", text).group(1)) > 500
    clob = re.search(rf"#define {prefix}_CLOBBERS (.*)", text).group(1)
    clobbered = set(re.findall(r'"([^"]+)"', clob))
    assert {"vcc", "scc", "memory"} <= clobbered        # m0 is a reserved register: written freely, never declared
    body = text[text.index(f"#define {prefix}_ASM"):]
    asm = "\n".join(re.findall(r'^\s*"(.*?)\\n\\t" \\$', body, flags=re.M))
    assert asm.count("\n") > 500
    # registers: everything written or read is a declared clobber or a pinned input
    for kind, inputs in (("v", set(in_v)), ("a", set()), ("s", set(in_s))):
        used = _regs(kind, asm)
        allowed = {int(c[1:]) for c in clobbered if re.fullmatch(rf"{kind}\d+", c)} | inputs
        assert used <= allowed, f"{kind}-registers outside clobbers and inputs: {sorted(used - allowed)}"
        assert max(used) < (256 if kind != "s" else 102)
    # LDS immediates fit their 16-bit field; every label is local to the statement
    for m in re.finditer(r"offset:(-?\d+)", asm):
        assert 0 <= int(m.group(1)) < 65536, m.group(0)
    for m in re.finditer(r"^\s*(\.L\w+):", asm, flags=re.M):
        assert m.group(1).endswith("%="), "labels must carry the per-statement suffix"
    # instruction forms that are ruled out: stores, atomics and cache maintenance of the scalar data cache,
    # hand-written packed fp32 arithmetic, wave priority changes
    banned = [r"\bs_store_", r"\bs_buffer_store_", r"\bs_atomic_", r"\bs_buffer_atomic_", r"\bs_dcache_", r"\bs_scratch_store",
              r"\bv_pk_(add|mul|fma)_f32\b", r"\bs_setprio\b", r"\bs_sethalt\b", r"\bs_trap\b"]
    for pat in banned:
        assert not re.search(pat, asm), pat
    # every barrier is unconditional top-level code of the loop: no branch may skip one wavefront's barrier
    assert "s_barrier" in asm and "s_endpgm" not in asm


def test_head_sizes_differ_where_they_should():
    for script, prefix, _, _ in GENERATORS:
        big, small = _run(script, 128), _run(script, 64)
        n = lambda t: t.count("v_mfma_f32_32x32x16_bf16")
        assert n(big) > n(small) > 0
        assert "_FAST64_" in small and "_FAST64_" not in big
