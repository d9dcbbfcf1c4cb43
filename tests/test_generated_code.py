"""The expert FFN kernel's hand-scheduled parts rely on two things the compiler cannot check (see tests/generated_code.py):
registers that an explicit asynchronous load is still filling are not touched, and explicit memory instructions do not read a
scalar base too early.  These tests compile the kernel file to gfx950 assembly for every hidden size and look.  No GPU needed."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

import generated_code as gc
from paper_2602_08404_amd import build as tb

SRC = os.path.join(tb.CSRC, "ffn_bf16_kernel.hip")
JOBS = [(f"bf16 hidden {128 * ksa}", [f"-DFFN_KSA_THIS_FILE={ksa}"]) for ksa in (16, 8, 4, 2)] + \
       [(f"8-bit hidden {128 * ksa}", [f"-DFFN_KSA_THIS_FILE={ksa}", "-DFFN_W8_THIS_FILE=1"]) for ksa in (16, 8)]


def _assembly(job, out_dir):
    name, defines = job
    out = os.path.join(out_dir, name.replace(" ", "_") + ".s")
    subprocess.run([tb.HIPCC, *tb.FLAGS, *defines, "--cuda-device-only", "-S", SRC, "-o", out], check=True, stderr=subprocess.DEVNULL)
    with open(out) as f:
        return name, f.read()


@pytest.fixture(scope="module")
def assemblies(tmp_path_factory):
    d = str(tmp_path_factory.mktemp("asm"))
    with ThreadPoolExecutor(3) as ex:
        return dict(ex.map(lambda j: _assembly(j, d), JOBS))


def test_registers_of_requests_in_flight_are_left_alone(assemblies):
    checked = 0
    for name, text in assemblies.items():
        fns = gc.kernel_functions(text)
        assert fns, name
        for fn, lines in fns.items():
            groups, violations = gc.in_flight_register_uses(lines)
            assert not violations, (name, fn, violations[:5])
            # the X_AHEAD stages of every instance of the streaming body must have been found: bf16 kernels hold the instance with
            # one token tile per wavefront and the one with two, 8-bit kernels the first only
            instances = 1 if "8-bit" in name else 2
            assert len(gc.streaming_bodies(lines)) == instances, (name, fn)
            assert groups == 4 * instances, (name, fn, groups)
            checked += 1
    assert checked == 4 * 8 + 2 * 4              # bf16: 4 hidden sizes x 8 intermediate sizes; 8-bit: 2 x 4


def test_explicit_memory_instructions_do_not_read_a_fresh_scalar_base(assemblies):
    for name, text in assemblies.items():
        for fn, lines in gc.kernel_functions(text).items():
            assert not gc.stale_scalar_base_uses(lines), (name, fn)


def test_no_kernel_uses_scratch_memory(assemblies):
    """Scratch (private) memory traffic consists of vector-memory operations: it would join the queue whose length the
    kernel's explicit waits count, and every compiler-inserted wait for it would drain the weight stream."""
    import re
    for name, text in assemblies.items():
        sizes = [int(v) for v in re.findall(r"; ScratchSize: (\d+)", text)]
        assert sizes and all(v == 0 for v in sizes), (name, sizes)


def test_the_checks_catch_planted_mistakes():
    """A register copy between a request and its wait, and a memory instruction right behind v_readlane, in a minimal listing."""
    ok = """
        ;;#ASMSTART
        global_load_dwordx4 v[2:5], v[10:11], off offset:0
        ;;#ASMEND
        ;;#ASMSTART
        global_load_dwordx4 v[6:9], v[10:11], off offset:64
        ;;#ASMEND
        s_add_i32 s1, s1, 1
        ;;#ASMSTART
        s_waitcnt vmcnt(3)
        ;;#ASMEND
        v_mfma_f32_16x16x32_bf16 v[20:23], v[30:33], v[2:5], v[20:23]
        v_mfma_f32_16x16x32_bf16 v[20:23], v[34:37], v[6:9], v[20:23]
        ;;#ASMSTART
        global_load_dwordx4 v[2:5], v[10:11], off offset:0
        ;;#ASMEND
        ;;#ASMSTART
        global_load_dwordx4 v[6:9], v[10:11], off offset:64
        ;;#ASMEND
    """
    lines = [l.strip() for l in ok.split("\n")]
    assert gc.in_flight_register_uses(lines) == (1, [])
    copied = ok.replace("s_add_i32 s1, s1, 1", "v_mov_b32_e32 v40, v3")
    groups, violations = gc.in_flight_register_uses([l.strip() for l in copied.split("\n")])
    assert groups == 1 and len(violations) == 1 and "v_mov_b32_e32 v40, v3" in violations[0]
    reuse = ok.replace("v_mfma_f32_16x16x32_bf16 v[20:23], v[34:37], v[6:9], v[20:23]",
                       "v_mfma_f32_16x16x32_bf16 v[20:23], v[34:37], v[6:9], v[20:23]\n        v_lshl_add_u64 v[2:3], s[6:7], 1, v[10:11]")
    assert gc.in_flight_register_uses([l.strip() for l in reuse.split("\n")]) == (1, [])     # behind the wait the data is there
    base = """
        v_readlane_b32 s4, v191, 6
        v_readlane_b32 s5, v191, 7
        ;;#ASMSTART
        global_load_dword v1, v2, s[4:5]
        ;;#ASMEND
    """
    assert gc.stale_scalar_base_uses([l.strip() for l in base.split("\n")])
    fixed = base.replace("global_load_dword v1", "s_nop 4\n        global_load_dword v1")
    assert not gc.stale_scalar_base_uses([l.strip() for l in fixed.split("\n")])
