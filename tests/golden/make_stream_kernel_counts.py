"""Writes tests/golden/stream_kernel_instruction_counts.txt: per kernel of csrc/gemm_big.hip the number of
vector-memory instructions of each kind, of hand-written and compiler-made waits on them, of barriers and of
matrix instructions, taken from the compiler's assembly.

Why: the streaming kernels wait for their global->LDS transfers with exact `s_waitcnt vmcnt(n)` values, which
are only right while the compiler puts no vector-memory instruction of its own (a spill, a hoisted load) between
the transfers and the waits.  The counts below were taken from the build whose kernels pass every corner-shape
and bit-exact test on the GPU; tests/test_stream_kernel_asm.py fails when a rebuild no longer matches them, which
tells whoever changed the source or the compiler to go through the wait counts again (and then to refresh this
file with this script).  Run from the repository root: python tests/golden/make_stream_kernel_counts.py
"""
import os
import re
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
OUT = os.path.join(ROOT, "tests", "golden", "stream_kernel_instruction_counts.txt")
KINDS = [("dma16", r"^\s*global_load_lds_dwordx4\b"), ("dma4", r"^\s*global_load_lds_dword\b"),
         ("global_load", r"^\s*global_load_(?!lds)"), ("global_store", r"^\s*global_store_"),
         ("scratch", r"^\s*scratch_"), ("buffer", r"^\s*buffer_"), ("vmcnt_waits", r"^\s*s_waitcnt[^\n]*vmcnt"),
         ("barriers", r"^\s*s_barrier\b"), ("mfma", r"^\s*v_mfma_")]


def kernel_counts():
    sys.path.insert(0, ROOT)
    from paper_2112_13509_amd import build as b
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "gemm_big.s")
        cmd = [b.HIPCC] + b.FLAGS + ["-S", "--cuda-device-only", "-o", asm, os.path.join(b.CSRC, "gemm_big.hip")]
        subprocess.run(cmd, check=True, capture_output=True)
        text = open(asm).read()
    out = {}
    for m in re.finditer(r"^(_ZN2ab\w+):.*?\n(.*?)\n\s*s_endpgm", text, re.S | re.M):
        name = subprocess.run(["c++filt", m.group(1)], capture_output=True, text=True).stdout.strip() or m.group(1)
        name = name.replace("void ", "").split("(")[0]
        out[name] = {k: len(re.findall(p, m.group(2), re.M)) for k, p in KINDS}
        out[name]["uses_scratch"] = int(bool(re.search(re.escape(m.group(1)) + r"\.private_seg_size, [1-9]", text)))
    return out


def main():
    counts = kernel_counts()
    with open(OUT, "w") as f:
        f.write("# kernel | " + " | ".join(k for k, _ in KINDS) + " | uses_scratch\n")
        for name in sorted(counts):
            c = counts[name]
            f.write(name + " | " + " | ".join(str(c[k]) for k, _ in KINDS) + " | %d\n" % c["uses_scratch"])
    print(open(OUT).read())


if __name__ == "__main__":
    main()
