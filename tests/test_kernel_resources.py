"""The streaming attention kernel's decode builds must compile without register spills.

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


def test_decode_builds_of_the_stream_kernel_do_not_spill_in_the_stream_loop():
    src = os.path.join(B.CSRC, "attention_mfma.hip")
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
    decode = {n: r for n, r in kernels.items() if "pv_attn_mfma_streamILb0E" in n}
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
