"""Build-time guard of the streaming GEMM kernels' memory-operation accounting (CPU only: the compiler's assembly
is inspected, nothing runs).

Those kernels wait for their global->LDS transfers with exact `s_waitcnt vmcnt(n)` values; that is only right
while the compiler adds no vector-memory instruction of its own between a transfer and its wait (a register spill
to scratch, a load it hoisted) and no wait of its own.  The counts in tests/golden/stream_kernel_instruction_counts.txt
were taken from the build whose kernels pass the corner-shape and bit-exact tests on the GPU.  A rebuild that does
not reproduce them -- after a change to csrc/gemm_big.hip or to the compiler -- fails here, before anything runs
on a GPU: go through the wait counts again, run the GPU tests, then refresh the file with
tests/golden/make_stream_kernel_counts.py."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden", "stream_kernel_instruction_counts.txt")


def _load_generator():
    spec = importlib.util.spec_from_file_location("make_stream_kernel_counts",
                                                  os.path.join(ROOT, "tests", "golden", "make_stream_kernel_counts.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_streaming_kernels_compile_to_the_recorded_memory_operation_counts():
    gen = _load_generator()
    kinds = [k for k, _ in gen.KINDS] + ["uses_scratch"]
    want = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        cells = [c.strip() for c in line.split("|")]
        want[cells[0]] = dict(zip(kinds, map(int, cells[1:])))
    got = gen.kernel_counts()
    assert set(got) == set(want), (sorted(got), sorted(want))
    for name in sorted(want):
        assert got[name]["scratch"] == 0 and got[name]["uses_scratch"] == 0, (name, "spills to scratch")
        assert got[name] == want[name], (name, got[name], want[name])
    # the streaming kernels proper: nothing but transfers into LDS, the epilogue's stores and the one-off
    # table loads of the prologue; every matrix instruction of the four quarters of both slab copies is there
    for name, c in got.items():
        if "gemm_stream" in name:
            assert c["mfma"] == 64 and c["buffer"] == 0, (name, c)
