"""Checks on the machine code hipcc generates for the tree-attention sweep (no GPU needed: the kernels are only
compiled).  Two properties that correctness or speed depend on and that a compiler update could silently break:
  - the LDS address register M0 is written by the kernel's own assembly (direct-to-LDS loads) and the compiler was
    not told; so no compiler-generated instruction may use M0;
  - in the steady-state loop of every sweep instantiation the only waits on the vector-memory counter are the
    kernel's own, one per tile, next to its barrier: an additional compiler-placed wait would make the LDS reads of
    the tile being computed wait for the loads of the next tile (bf16 prefix: two-tile loop of a double buffer; fp8
    prefix and small bf16 launches: four-tile loop of a four-stage ring)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def sweep_asm(tmp_path_factory):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("asm") / "tree_attention.s"
    csrc = os.path.join(ROOT, "paper_2409_10644_amd", "csrc")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(csrc, "tree_attention.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text().split("\n")


def _functions(lines):
    starts = [(i, l.split(":")[0]) for i, l in enumerate(lines) if re.match(r"^_Z\w+:", l)]
    for (i0, name), (i1, _) in zip(starts, starts[1:] + [(len(lines), "")]):
        yield name, lines[i0:i1]


def test_m0_is_only_touched_by_the_kernels_own_assembly(sweep_asm):
    inside, seen = False, 0
    for l in sweep_asm:
        if "#ASMSTART" in l:
            inside = True
        elif "#ASMEND" in l:
            inside = False
        elif re.search(r"\bm0\b", l.split(";")[0]):
            assert inside, f"compiler-generated use of M0: {l.strip()}"
            seen += 1
    assert seen > 0


def test_steady_state_loops_wait_for_memory_once_per_tile(sweep_asm):
    checked = 0
    for name, body in _functions(sweep_asm):
        if "tree_attn_bf16_kernel" not in name:
            continue
        labels = {m.group(1): i for i, l in enumerate(body) if (m := re.match(r"^(\.LBB\d+_\d+):", l))}
        loops = []
        for i, l in enumerate(body):
            m = re.search(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", l)
            if m and m.group(1) in labels and labels[m.group(1)] < i:
                loop = body[labels[m.group(1)]:i + 1]
                if any("global_load_lds" in x for x in loop) and any("v_mfma" in x for x in loop):
                    loops.append(loop)
        assert loops, f"no streaming loop found in {name}"
        D, QBP, NS, F8 = (int(x) for x in re.search(r"ILi(\d+)ELi(\d+)ELi(\d+)ELb(\d)E", name).groups())
        if NS == 2:
            loop = min(loops, key=len)                                # the innermost one
            code = [x.split(";")[0] for x in loop]
            waits = sum("vmcnt" in x for x in code)
            barriers = sum("s_barrier" in x for x in code)
            assert barriers == 2 and waits == 2, f"{name}: {waits} vmcnt waits, {barriers} barriers in the two-tile loop"
        else:
            # four-stage ring, four tiles per trip; a step waits for all loads but those of the two, one or zero tiles
            # requested after its own (three alternative instructions), right before its barrier, and nowhere else
            # (of the backward branches that span exactly the ring's four barriers the one with the fewest waits, the
            # longest of those: block placement adds backward jumps from the kernel's epilogue whose spans hold the
            # loop plus the waits before and after it; a wait the compiler added inside the loop is in every span)
            four = [x for x in loops if sum("s_barrier" in y.split(";")[0] for y in x) == 4]
            assert four, f"{name}: no four-tile loop found"
            loop = min(four, key=lambda x: (sum("vmcnt" in y.split(";")[0] for y in x), -len(x)))
            code = [x.split(";")[0] for x in loop if x.split(";")[0].strip() and not x.strip().startswith(".")]
            wait_at = [i for i, x in enumerate(code) if "vmcnt" in x]
            barrier_at = [i for i, x in enumerate(code) if "s_barrier" in x]
            assert len(barrier_at) == 4 and len(wait_at) == 12, f"{name}: {len(wait_at)} waits, {len(barrier_at)} barriers"
            for i in wait_at:
                assert any(0 < b - i <= 16 for b in barrier_at), f"{name}: a wait on vector memory away from the barriers"
            row_bytes = D if F8 else 2 * D                     # 64-key tiles: 2 (K, V) x 64 rows / rows per 1 KiB load / 4 wavefronts
            loads_per_tile = 2 * 64 * row_bytes // 1024 // 4
            assert sorted(set(int(re.search(r"vmcnt\((\d+)\)", code[i]).group(1)) for i in wait_at)) == \
                [0, loads_per_tile, 2 * loads_per_tile], name
        assert not any("scratch_" in x for x in code), f"{name}: register spills inside the streaming loop"
        checked += 1
    # head_dim 64 / 128 x 1, 2, 4 query blocks with two stages, x 2, 4 query blocks with four; fp8 prefix: head_dim 128 x 2, 4
    assert checked == 12
