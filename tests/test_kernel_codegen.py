"""What the compiler made of the aggregation kernel (CPU only: hipcc cross-compiles for gfx950).

The kernel's speed rests on two properties of the generated code that a harmless-looking source
change can lose without any test of results noticing:
  * the U row gathers of a batch are issued back to back; a wait for vector memory between two
    of them (which the compiler inserts when an address register overlaps the destination of a
    load still in flight) makes every gather wait for the one before;
  * the register budget: no scratch (spilled registers) in the plain kernels, at least four
    wavefronts per SIMD everywhere, five for the 4-byte-lane kernels of the plain layout.
Both are read from the compiler's own output for every template variant."""
import re
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = ROOT / "paper_2204_02662_amd" / "csrc" / "epp_aggregate.hip"
VARIANT = re.compile(r"k_aggregateILi(\d)ELi(\d)ELi(\d+)ELb([01])ELb([01])ELb([01])ELb([01])E")


@pytest.fixture(scope="module")
def compiled(tmp_path_factory):
    d = tmp_path_factory.mktemp("codegen")
    out = subprocess.run(
        ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", f"-I{ROOT / 'include'}", f"-I{SRC.parent}", "-c", str(SRC), "-o", "agg.o", "--save-temps",
         "-Rpass-analysis=kernel-resource-usage"], cwd=d, capture_output=True, text=True, timeout=900)
    assert out.returncode == 0, out.stderr[-3000:]
    asm = next(d.glob("*gfx950*.s")).read_text()
    return asm, out.stderr


def test_register_budget_of_every_variant(compiled):
    _, remarks = compiled
    usage, cur = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = VARIANT.search(m.group(1))
            if cur:
                usage[cur.groups()] = {}
            continue
        if cur:
            for key, pat in (("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"), ("occupancy", r"Occupancy \[waves/SIMD\]: (\d+)")):
                m = re.search(pat, line)
                if m:
                    usage[cur.groups()][key] = int(m.group(1))
    assert len(usage) >= 200, len(usage)  # 3 lane widths x 7 lane counts x 10 flag combinations
    for (vec, log2t, u, ifelse, cold, part, inner), r in usage.items():
        assert r["occupancy"] >= 4, (vec, log2t, ifelse, cold, part, inner, r)
        if (ifelse, inner) == ("0", "0"):
            assert r["scratch"] == 0, (vec, log2t, ifelse, cold, part, inner, r)
        # (the variants for a path that runs on the next outer path's arrays are held to the plain
        # kernel's occupancy; that costs narrow lanes three spilled registers)
        assert r["scratch"] <= 16 or ifelse == "1", (vec, log2t, ifelse, cold, part, inner, r)
        if (vec, ifelse, part) == ("1", "0", "0"):
            assert r["occupancy"] >= 5, (vec, log2t, cold, inner, r)


def test_gathers_of_a_batch_are_issued_back_to_back(compiled):
    asm, _ = compiled
    checked = 0
    for m in re.finditer(r"^(_ZN12_GLOBAL__N_111k_aggregateILi(\d)ELi(\d)ELi(\d+)ELb([01])ELb([01])ELb([01])ELb([01])EEEvNS_7AggArgsE):(.*?)s_endpgm",
                         asm, re.S | re.M):
        vec, log2t, u, ifelse, cold, part, inner = m.groups()[1:8]
        if vec == "1":
            continue  # 4-byte gathers cannot be told from the kernel's other 4-byte loads by their opcode
        lines = [x.strip() for x in m.group(9).split("\n") if x.strip() and not x.strip().startswith((";", "."))]
        op = "global_load_dwordx4" if vec == "4" else "global_load_dwordx2"
        # the gathers: loads of that width that are not the streamed (nt) loads of the index pairs
        idx = [i for i, x in enumerate(lines) if x.startswith(op) and not (vec == "2" and x.rstrip().endswith(" nt") and cold == "0")]
        waits = 0
        for a, b in zip(idx, idx[1:]):
            if b - a < 40 and any(re.match(r"s_waitcnt.*vmcnt\(0\)", x) for x in lines[a + 1:b]):
                waits += 1
        assert waits <= 1, f"VEC={vec} LOG2T={log2t} if-else={ifelse} cold={cold} part={part} inner={inner}: {waits} full waits between gathers"
        checked += 1
    assert checked >= 120, checked
