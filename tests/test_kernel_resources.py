"""The streaming attention kernel's decode builds and the projection kernels must compile without register spills.

A spilled value inside the stream loop is reloaded through scratch memory, which shares the load
counter with the tile prefetches: every reload then waits for all loads in flight and the loop
stops overlapping memory and compute.  This check compiles the kernel for gfx950 (no GPU needed)
and reads the resource usage the compiler records in the assembly's metadata.
"""
import os
import re
import subprocess
import tempfile

from paper_2604_14889_amd import build as B


def compiled_kernels(source: str):
    """(assembly text, {kernel: resource usage}) of one source file compiled for gfx950."""
    src = os.path.join(B.CSRC, source)
    flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [B.hipcc(), *flags, f"-I{B.INCLUDE}", f"-I{B.CSRC}", "-c", src, "-o", os.path.join(tmp, "k.o"), "-save-temps=obj"]
        res = subprocess.run(cmd, capture_output=True, text=True, cwd=tmp)
        assert res.returncode == 0, res.stderr[-2000:]
        asm = [f for f in os.listdir(tmp) if f.endswith(".s") and "gfx950" in f]
        assert len(asm) == 1, os.listdir(tmp)
        text = open(os.path.join(tmp, asm[0])).read()
    kernels = {}
    for block in text.split("  - .agpr_count:")[1:]:
        name = re.search(r"\.name:\s+(\S+)", block).group(1)
        kernels[name] = {k: int(re.search(rf"\.{k}:\s+(\d+)", block).group(1))
                         for k in ("vgpr_count", "vgpr_spill_count", "sgpr_spill_count", "private_segment_fixed_size")}
    return text, kernels


def loops_with_priority_changes(lines, start, end):
    """(first, last) line of every loop (a backward branch to a label) between start and end whose body raises the wave priority."""
    label_at = {ln.split(":")[0]: i for i, ln in enumerate(lines[start:end], start) if ln.startswith(".LBB") and ":" in ln}
    loops = []
    for i in range(start, end):
        m = re.match(r"\s+s_c?branch\w*\s+(\.LBB\w+)", lines[i])
        if m and m.group(1) in label_at and label_at[m.group(1)] < i:
            first = label_at[m.group(1)]
            if any("s_setprio" in lines[j] for j in range(first, i)):
                loops.append((first, i))
    return loops


def test_projection_kernels_do_not_spill():
    """The few-row kernel keeps 16 loads in flight per wave and the tiled one runs two waves per SIMD
    (256 registers each): a spilled value inside their loops would put a wait for all loads there.  The
    tiled kernel may park a few registers around its K loops (stored before, reloaded after)."""
    text, kernels = compiled_kernels("gemm.hip")
    few = {n: r for n, r in kernels.items() if "skinny_mfma_bf16" in n}
    assert len(few) == 6, sorted(kernels)
    for name, r in few.items():
        assert r["vgpr_spill_count"] == 0 and r["private_segment_fixed_size"] == 0 and r["vgpr_count"] <= 128, (name, r)
    tiled = {n: r for n, r in kernels.items() if "gemm_tn_bf16" in n}
    assert len(tiled) == 4, sorted(kernels)
    lines = text.split("\n")
    for name, r in tiled.items():
        assert r["vgpr_spill_count"] <= 8 and r["vgpr_count"] <= 256, (name, r)
        start = next(i for i, ln in enumerate(lines) if ln.startswith(name + ":"))
        end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
        loops = loops_with_priority_changes(lines, start, end)
        multiplying = 0
        for first, last in loops:
            body = lines[first:last]
            multiplying += sum("v_mfma" in ln for ln in body) >= 8
            assert not [ln.strip() for ln in body if "scratch_" in ln], (name, first)
        assert multiplying >= 4, (name, loops)          # one K loop per number of valid row blocks (1 to 4; 0 only moves data)
    norm = [r for n, r in kernels.items() if "reduce_add_rmsnorm" in n]
    assert len(norm) == 1 and norm[0]["vgpr_spill_count"] == 0 and norm[0]["vgpr_count"] <= 128, norm


def test_decode_builds_of_the_stream_kernel_do_not_spill_in_the_stream_loop():
    text, kernels = compiled_kernels("attention_mfma.hip")
    decode = {n: r for n, r in kernels.items() if "pv_attn_mfma_stream" in n}
    assert len(decode) == 4, sorted(kernels)           # fixed / first-come tile assignment x small / large layer pool
    lines = text.split("\n")
    for name, r in decode.items():
        assert r["vgpr_count"] <= 256, (name, r)       # two waves per SIMD
        # the stream loop lies between the first and the last change of the wave priority
        start = next(i for i, ln in enumerate(lines) if ln.startswith(name + ":"))
        end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
        prio = [i for i in range(start, end) if "s_setprio" in lines[i]]
        assert len(prio) >= 3, name
        in_loop = [lines[i].strip() for i in range(prio[0], prio[-1]) if "scratch_" in lines[i]]
        assert not in_loop, (name, in_loop)
        if name.endswith("ELb0EEEvNS_8MfmaArgsE"):     # the small-pool builds do not spill at all
            assert r["vgpr_spill_count"] == 0 and r["private_segment_fixed_size"] == 0, (name, r)
        else:
            assert r["vgpr_spill_count"] <= 4, (name, r)
    # the wide-step kernel: spills are tolerated in its set-up and closing, not between the barriers of its tile loop
    wide = [n for n in kernels if "pv_attn_mfma_wide" in n]
    assert len(wide) == 1
    start = next(i for i, ln in enumerate(lines) if ln.startswith(wide[0] + ":"))
    end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
    assert kernels[wide[0]]["vgpr_count"] <= 256
    # its tile loop is the innermost loop that holds matrix instructions, a workgroup barrier and the
    # streaming (non-temporal) loads of V: the block between a label and the backward branch to it
    labels = {lines[i].split(":")[0]: i for i in range(start, end) if lines[i].startswith(".LBB")}
    loops = []
    for i in range(start, end):
        m = re.match(r"\s+s_c?branch\w* (\.LBB\d+_\d+)", lines[i])
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            body = lines[labels[m.group(1)]:i]
            if any("v_mfma" in b for b in body) and any("s_barrier" in b for b in body) and any("global_load" in b and " nt" in b for b in body):
                loops.append(body)
    assert loops, "tile loop of the wide kernel not found"
    inner = min(loops, key=len)
    assert not [b for b in inner if "scratch_" in b], [b.strip() for b in inner if "scratch_" in b]
