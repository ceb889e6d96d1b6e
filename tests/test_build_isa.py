"""The generated code of the dominant kernel, checked at build time (no GPU): the stage loop of the
sparse matrix-core lookup (arXiv 2302.03213 Eq. 4 as a one-hot contraction) lives at the edge of the
register file - 256 accumulator registers and everything else in the other 256 - and a spill into
its loop, which the compiler reports nowhere but in the assembly, costs tens of per cent.  These
checks read the assembly hipcc writes for gfx950 and fail when the loop no longer fits."""
import os
import re
import subprocess

import pytest

from paper_2302_03213_amd import build


@pytest.fixture(scope="module")
def isa(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "lookup_smfmac.s")
    flags = [f for f in build.FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
    cmd = [build.HIPCC] + flags + ["-S", "--cuda-device-only", "-o", out,
                                   os.path.join(build.CSRC, "lookup_smfmac.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    with open(out) as f:
        return f.read().split("\n")


def kernel_body(lines, mangled_args):
    """(instructions by basic block, trailing metadata lines) of one lookup_smfmac_i8_kernel instance."""
    start = [i for i, l in enumerate(lines)
             if re.match(r"^_ZN5lutnn.*lookup_smfmac_i8_kernel" + mangled_args + r"EEvPK.*:", l)]
    assert len(start) == 1, (mangled_args, len(start))
    end = next(i for i in range(start[0], len(lines)) if lines[i].strip().startswith("s_endpgm"))
    blocks, name, cur = {}, "entry", []
    for l in lines[start[0]:end]:
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            blocks[name] = cur
            name, cur = m.group(1), []
        else:
            t = l.split(";")[0].strip()
            if t and not t.startswith("."):
                cur.append(t)
    blocks[name] = cur
    meta = {}
    for l in lines[end:end + 200]:
        m = re.match(r"^; (NumVgprs|NumAgprs|ScratchSize|LDSByteSize|Occupancy): (\d+)", l.strip())
        if m and m.group(1) not in meta:
            meta[m.group(1)] = int(m.group(2))
    return blocks, meta


# template arguments <TM, TN, SPLIT, STREAM> as the mangled name spells them
INSTANCES = {
    "512x128 streamed (config 5)": "ILi4ELi4ELb0ELb1E",
    "512x128": "ILi4ELi4ELb0ELb0E",
    "512x96": "ILi4ELi3ELb0ELb0E",
    "384x128": "ILi3ELi4ELb0ELb0E",
    "256x128": "ILi2ELi4ELb0ELb0E",
    "128x128": "ILi1ELi4ELb0ELb0E",
    "512x128 split": "ILi4ELi4ELb1ELb0E",
}


@pytest.mark.parametrize("name", list(INSTANCES))
def test_stage_loop_has_no_spills_and_fits_the_machine(isa, name):
    blocks, meta = kernel_body(isa, INSTANCES[name])
    # one workgroup per compute unit: up to 512 registers per lane, 160 KiB of LDS
    assert meta["NumVgprs"] <= 256 and meta["NumAgprs"] <= 256, meta
    assert meta["LDSByteSize"] <= 160 * 1024, meta
    loops = {b: ins for b, ins in blocks.items() if sum(x.startswith("v_smfmac") for x in ins) >= 48}
    assert loops, "no stage loop found"
    for b, ins in loops.items():
        spills = [x for x in ins if x.startswith(("scratch_", "buffer_store", "buffer_load_dword "))]
        assert not spills, "%s: %d scratch accesses in block %s" % (name, len(spills), b)
        # the loop's own waits leave the loads of the current stage in flight (six or more); a
        # wait for fewer would be the compiler's, for a load of its own, and would drain the ring
        for x in ins:
            m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", x)
            assert not m or int(m.group(1)) >= 6, "%s: '%s' in block %s" % (name, x, b)


def test_steady_state_loop_of_the_benchmark_instance_keeps_its_instruction_budget(isa):
    """Four stages' worth of the 512x128 streamed instance: 192 matrix instructions (three stages in
    the largest block), no scratch memory at all, and the vector-instruction count it was tuned to
    (391 when written; a fifth more means the allocator has started shuffling registers)."""
    blocks, meta = kernel_body(isa, INSTANCES["512x128 streamed (config 5)"])
    assert meta["ScratchSize"] == 0, meta
    body = max(blocks.values(), key=lambda ins: sum(x.startswith("v_smfmac") for x in ins))
    n_mfma = sum(x.startswith("v_smfmac_i32_32x32x64_i8") for x in body)
    n_valu = sum(x.startswith("v_") and not x.startswith("v_smfmac") for x in body)
    n_dma = sum(x.startswith("global_load_lds_dwordx4") for x in body)
    assert n_mfma == 192, n_mfma
    assert n_dma == 32, n_dma   # 3 stages x 8 table loads + their share of the index loads
    assert n_valu <= 430, "%d vector instructions per 192 matrix instructions" % n_valu
