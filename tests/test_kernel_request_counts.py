"""The small-M kernels wait on vector-memory requests with hand-counted `s_waitcnt vmcnt(n)`;
every n is built from ATile::LOADS, the number of requests that fetch one row tile.  This
test compiles the kernels to gfx950 assembly (no GPU needed) and checks that the requests
the compiler emitted are whole multiples of that number, so a request added to or dropped
from the tile fetch without the count following fails here, on the CPU, and not as a wrong
sum on the GPU."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_11582_amd", "csrc")


def _hipcc():
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.fixture(scope="module")
def smallm_asm(tmp_path_factory):
    """The small-M source compiled to gfx950 assembly, split into (kernel name, body) pairs."""
    hipcc = _hipcc()
    if hipcc is None:
        pytest.skip("hipcc not found")
    asm = str(tmp_path_factory.mktemp("asm") / "smallm.s")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                          "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "--cuda-device-only", "-S",
                          os.path.join(CSRC, "egt_mfma_smallm.hip"), "-o", asm], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    parts = re.split(r"\n(_Z\w+):[^\n]*\n", open(asm).read())
    return [(name, body.split(".Lfunc_end")[0]) for name, body in zip(parts[1::2], parts[2::2])]


def test_tile_requests_of_the_small_m_kernels_match_the_wait_counts(smallm_asm):
    text = open(os.path.join(CSRC, "egt_mfma_smallm.hip")).read()
    loads = re.search(r"static constexpr int LOADS = KIND == EGT_VAL_INT4 \? (\d+) : 1 \+ VW;", text)
    vw = re.search(r"static constexpr int VW = KIND == EGT_VAL_INT4 \? 1 : (\d+);", text)
    assert loads and vw, "ATile::LOADS / ATile::VW are not where this test reads them"
    per_tile = {0: int(loads.group(1)), 1: 1 + int(vw.group(1))}          # by value kind
    # no hand-written count survives beside the constant
    assert not re.search(r"wait_vmem<[^>]*\b[2-9]\b[^>]*>", text), "a literal request count in a wait"
    seen = 0
    for name, body in smallm_asm:
        m = re.search(r"k_sparse_smallm_ksILi(\d)ELi(\d+)ELi(\d+)E", name)   # KIND, NT, NIT
        if not m:
            continue
        kind, nit = int(m.group(1)), int(m.group(3))
        requests = [ln for ln in body.split("\n") if re.search(r"\bbuffer_load_dword", ln)]
        tile_requests = [ln for ln in requests if " lds" not in ln]           # X goes straight to LDS: counted apart
        assert tile_requests, name
        assert len(tile_requests) % (nit * per_tile[kind]) == 0, (name, len(tile_requests), nit, per_tile[kind])
        waits = {int(v) for v in re.findall(r"vmcnt\((\d+)\)", body)}
        assert max(waits) <= 2 * nit * per_tile[kind], (name, sorted(waits))   # at most two phases of tiles pending
        seen += 1
    assert seen >= 20


def test_requests_of_the_row_split_stack_kernel_match_its_wait_counts(smallm_asm):
    # k_smallm_rows<NG, Q, W> allows exactly the Q * LOADS requests of the next round's A tiles to stay pending at
    # the top of a round; the round body is compiled twice (two sets of fetch registers) after a prologue of two rounds
    text = open(os.path.join(CSRC, "egt_mfma_smallm.hip")).read()
    loads = int(re.search(r"static constexpr int LOADS = KIND == EGT_VAL_INT4 \? (\d+) : 1 \+ VW;", text).group(1))
    seen = 0
    for name, body in smallm_asm:
        m = re.search(r"k_smallm_rowsILi(\d+)ELi(\d+)ELi(\d+)ELb(\d)E", name)       # NG, Q, W, N1
        if not m:
            continue
        ng, q, w, n1 = (int(v) for v in m.groups())
        per_round, x_per_round = q * loads, ng * q * (16 if n1 else 8) // w      # (1:4: a request of X per token, 2:4: per pair)
        requests = [ln for ln in body.split("\n") if re.search(r"\bbuffer_load_dword", ln)]
        to_lds = [ln for ln in requests if " lds" in ln]
        assert len(requests) - len(to_lds) == 4 * per_round, (name, len(requests), len(to_lds))   # rounds 0, 1 and j + 2 twice
        assert len(to_lds) == 3 * x_per_round, (name, len(to_lds))                                # X(0) and X(j + 1) twice
        waits = [int(v) for v in re.findall(r"vmcnt\((\d+)\)", body)]
        assert waits.count(per_round) >= 2 and max(waits) <= 2 * per_round + x_per_round + 1, (name, sorted(set(waits)))
        assert len(re.findall(r"\bs_barrier\b", body)) == 2, name
        assert not re.search(r"\bscratch_|\bflat_", body), name
        seen += 1
    assert seen == 5
