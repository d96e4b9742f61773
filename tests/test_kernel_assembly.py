"""What the compiler generated around the kernels' inline assembly.

The kernels rely on properties that the source cannot enforce by itself:
* the direct-to-LDS copies set M0 inside an inline-assembly statement, and the
  compiler does not accept M0 in a clobber list, so no compiler-generated
  instruction of these kernels may read or write M0;
* the 64-rows-per-wave kernel keeps its O^T accumulators in fixed accumulation
  registers that only its own assembly statements name; the register
  allocator is free to use whatever a statement does not clobber at that
  point, so it must not have picked any of them;
* nothing spills to scratch memory, and no packed-fp32 vector instruction is
  emitted (the build switches them off).
The device code is compiled to assembly with the flags of the build (no GPU
needed) and scanned."""
import re
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2605_08581_amd import build

KERNEL_SOURCES = ["prism_kernels.hip", "prism_attn64.hip"]


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("asm"))
    with ThreadPoolExecutor(max_workers=2) as ex:
        paths = list(ex.map(lambda s: build.emit_assembly(s, out), KERNEL_SOURCES))
    return {s: open(p).read().splitlines() for s, p in zip(KERNEL_SOURCES, paths)}


def _instructions(lines):
    """(kernel, in_inline_asm, instruction text) for every instruction line."""
    kernel, inline = None, False
    for line in lines:
        s = line.strip()
        if s.startswith(";;#ASMSTART"):
            inline = True
            continue
        if s.startswith(";;#ASMEND"):
            inline = False
            continue
        m = re.match(r"^(_Z\w+):", line)
        if m:
            kernel = m.group(1)
            continue
        if not s or s[0] in ";." or s.endswith(":"):
            continue
        yield kernel, inline, s.split(";")[0].strip()


def test_both_sources_define_their_kernels(assembly):
    names = {k for lines in assembly.values() for k, _, _ in _instructions(lines) if k}
    for want in ("kv_append_kernel", "prefill_attn_kernel", "prefill_attn64_kernel", "split_reduce_kernel"):
        assert any(want in n for n in names), want


def test_compiler_never_touches_m0(assembly):
    for src, lines in assembly.items():
        ours = 0
        for kernel, inline, ins in _instructions(lines):
            if re.search(r"\bm0\b", ins):
                assert inline, f"{src}: compiler-generated use of M0 in {kernel}: {ins}"
                assert ins.startswith("s_mov_b32 m0,"), ins
                ours += 1
        assert ours > 0, f"{src}: the LDS copies should set M0"


def test_fixed_accumulators_belong_to_the_inline_assembly(assembly):
    seen = 0
    for kernel, inline, ins in _instructions(assembly["prism_attn64.hip"]):
        if kernel is None or "prefill_attn64_kernel" not in kernel:
            continue
        head_dim = int(re.search(r"prefill_attn64_kernelILi(\d+)E", kernel).group(1))
        reserved = head_dim            # two row blocks x head_dim/32 tiles x 16 registers
        for m in re.finditer(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]", ins):
            low = int(m.group(1) if m.group(1) else m.group(2))
            if inline:
                seen += 1
                assert int(m.group(3) or low) < reserved, f"{kernel}: {ins}"
            else:
                assert low >= reserved, f"compiler-generated use of a reserved accumulator in {kernel}: {ins}"
    assert seen > 0


def test_no_spills_and_no_packed_fp32(assembly):
    for src, lines in assembly.items():
        for line in lines:
            m = re.match(r"\s*\.amdhsa_private_segment_fixed_size\s+(\d+)", line)
            if m:
                assert int(m.group(1)) == 0, f"{src}: a kernel uses scratch memory"
        for kernel, _, ins in _instructions(lines):
            assert not ins.startswith("scratch_"), f"{src}: {kernel}: {ins}"
            assert not re.match(r"v_pk_(add|mul|fma)_f32\b", ins), f"{src}: {kernel}: {ins}"
