"""CPU-only: the C-ABI library builds/loads and exports every symbol include/moe_hip.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2603_07685_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()
    lib = ctypes.CDLL(build.LIB)
    names = _declared()
    assert "moe_route_topk" in names and "moe_grouped_gemm_wgrad" in names and len(names) >= 13
    for n in names:
        assert hasattr(lib, n), f"{n} declared in moe_hip.h but not exported"


def test_binding_names_match_header():
    import importlib.util
    spec = importlib.util.find_spec("torch")
    assert spec is not None
    from paper_2603_07685_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_host_only_calls():
    """moe_workspace_bytes is a pure host function; NULL contexts are rejected without touching a GPU."""
    from paper_2603_07685_amd import build
    lib = ctypes.CDLL(build.LIB)
    lib.moe_workspace_bytes.restype = ctypes.c_size_t
    small = lib.moe_workspace_bytes(256, 2, 8, 128, 256)
    big = lib.moe_workspace_bytes(16384, 8, 32, 7168, 2048)
    assert 0 < small <= big and big % 256 == 0
    assert lib.moe_workspace_bytes(-1, 2, 8, 128, 256) == 0
    assert lib.moe_route_topk(None, None, None, 1, 1, 1, 0, 0, ctypes.c_float(1.0), None, None, None) == -1
    assert lib.moe_ctx_destroy(None) == 0


def test_build_refuses_register_arrays_in_scratch():
    """The build reads the compiler's per-kernel resource report and fails when a kernel needs more scratch than a
    few spilled registers (a register array demoted to memory); the parser picks the largest figure and its kernel."""
    from paper_2603_07685_amd import build as b
    log = ("gemm.hip:1:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
           "gemm.hip:1:1: remark:     ScratchSize [bytes/lane]: 44 [-Rpass-analysis=kernel-resource-usage]\n"
           "gemm.hip:9:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]\n"
           "gemm.hip:9:1: remark:     ScratchSize [bytes/lane]: 640 [-Rpass-analysis=kernel-resource-usage]\n")
    assert b._max_scratch(log) == (640, "kernel_b")
    assert b._max_scratch("no remarks here") == (0, "")
    assert 0 < b.MAX_SCRATCH_BYTES_PER_LANE < 640


def test_header_is_plain_c_and_cxx():
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++11, warnings included."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "moe_hip.h")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", hdr])


def test_row_map_division_by_multiplication():
    """The gathered GEMMs turn a map entry s = t*k + slot into its token t = s / k with one multiplication,
    t = ((2 s + 1) * ceil(2^31 / k)) >> 32, and the host admits only T*k*k < 2^30.  The identity, checked in exact
    integer arithmetic for every k up to 64 (and a few large ones) on the extremes of the admitted range and on random
    entries: a wrong rounding of the constant, or a bound that is too generous, fails here."""
    import random
    rnd = random.Random(7)
    for k in list(range(1, 65)) + [100, 127, 128, 255, 1000, 4096]:
        m = ((1 << 31) + k - 1) // k
        assert m < (1 << 32)
        top = ((1 << 30) - 1) // k            # s * k < 2^30 at most (s < T*k and T*k*k < 2^30)
        cases = {0, 1, k - 1, k, k + 1, top, top - 1, max(top - k, 0), (top // k) * k, max((top // k) * k - 1, 0)}
        cases |= {rnd.randrange(0, top + 1) for _ in range(2000)}
        for s in cases:
            assert 2 * s + 1 < (1 << 32)
            assert ((2 * s + 1) * m) >> 32 == s // k, (k, s)


def test_quantiser_row_map_division_by_multiplication():
    """The gathering quantisers divide a map entry 0 <= s < 2^31 by k (k <= 32 admitted) as (s * m) >> (31 + l) with
    l = ceil(log2 k), m = ceil(2^(31 + l) / k): exact on the extremes and on random entries, m fits 32 bits and the
    product 64 (a constant of the form ceil(2^40 / k) would overflow 64 bits from s = 2^24 k on)."""
    import random
    rnd = random.Random(11)
    for k in list(range(1, 33)) + [33, 63, 64, 65, 100, 1000]:
        l = (k - 1).bit_length()
        assert (1 << l) >= k and (l == 0 or (1 << (l - 1)) < k)
        m = ((1 << (31 + l)) + k - 1) // k
        assert m < (1 << 32)
        top = (1 << 31) - 1
        cases = {0, 1, k - 1, k, k + 1, top, top - 1, top - k, (top // k) * k, (top // k) * k - 1, 1 << 24, (1 << 24) * k,
                 (1 << 24) * k - 1}
        cases |= {rnd.randrange(0, top + 1) for _ in range(2000)}
        for s in cases:
            if s > top:
                continue
            assert s * m < (1 << 64)
            assert (s * m) >> (31 + l) == s // k, (k, s)


def test_bench_refuses_more_than_one_gpu():
    """This build is the one-GPU path: bench.py --gpus N with N > 1 exits with a message that says so, before anything
    touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr and "--gpus 1" in r.stderr and r.stdout.strip() == ""
