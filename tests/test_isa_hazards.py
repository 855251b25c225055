"""Checks on the generated gfx950 code of the FFN kernels (no GPU needed).

The kernels for blocks of more than 32 tokens issue their loads from inline asm
and wait for them with explicit counts.  The compiler neither inserts the wait
states the hardware requires around instructions inside asm nor knows that the
loaded registers are valid only after the explicit wait, so three properties
of the generated code are checked here:
  * a scalar register written by a vector instruction (v_readlane /
    v_readfirstlane, e.g. a spilled scalar being restored) is not used as the
    base of a vector-memory load within the next five wait states;
  * the write of M0 and the direct-to-LDS load that uses it are at least one
    wait state apart;
  * those kernels spill no vector registers (a spill could copy a register whose
    asynchronous load has not landed yet).
"""
import os
import re

import pytest

from paper_2602_00879_amd import build as B


@pytest.fixture(scope="module")
def ffn_asm(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "des_ffn.s")
    B.device_asm("des_ffn.hip", out)
    return open(out).read()


def _kernels(text):
    """{kernel name: list of instructions} of every kernel in the assembly."""
    out = {}
    for m in re.finditer(r"\n(_ZN3des\w+):[^\n]*\n(.*?)\n\s*s_endpgm", text, re.S):
        ins = []
        for line in m.group(2).split("\n"):
            line = line.split(";")[0].strip()
            if line and not line.startswith(".") and not line.endswith(":"):
                ins.append(line)
        out[m.group(1)] = ins
    return out


def _wait_states(instr):
    m = re.match(r"s_nop (\d+)", instr)
    return int(m.group(1)) + 1 if m else 1


def test_no_vector_written_scalar_base_too_close_to_a_load(ffn_asm):
    kernels = _kernels(ffn_asm)
    assert any("lds_kernel" in k for k in kernels)
    for name, ins in kernels.items():
        for i, instr in enumerate(ins):
            m = re.match(r"global_load_(?:lds_)?dwordx4 .*s\[(\d+):(\d+)\]", instr)
            if not m:
                continue
            base = {int(m.group(1)), int(m.group(2))}
            ws = 0
            for j in range(i - 1, max(-1, i - 8), -1):
                w = re.match(r"v_(?:readlane|readfirstlane)_b32 s(\d+),", ins[j])
                assert not (w and int(w.group(1)) in base and ws < 5), (
                    f"{name}: '{ins[j]}' only {ws} wait states before '{instr}'")
                ws += _wait_states(ins[j])


def test_m0_write_is_one_wait_state_before_direct_lds_load(ffn_asm):
    n = 0
    for name, ins in _kernels(ffn_asm).items():
        for i, instr in enumerate(ins):
            if not instr.startswith("global_load_lds_dwordx4"):
                continue
            n += 1
            j = i - 1
            ws = 0
            while j >= 0 and not ins[j].startswith("s_mov_b32 m0"):
                ws += _wait_states(ins[j])
                j -= 1
                assert i - j < 6, f"{name}: no M0 write just before '{instr}'"
            assert ws >= 1, f"{name}: M0 written immediately before '{instr}'"
    assert n > 0


def test_asm_load_kernels_do_not_spill(ffn_asm):
    n = 0
    for m in re.finditer(r"\.amdhsa_kernel (\S+)\n(.*?)\.end_amdhsa_kernel", ffn_asm, re.S):
        if "lds_kernel" not in m.group(1):
            continue
        n += 1
        size = int(re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", m.group(2)).group(1))
        assert size == 0, f"{m.group(1)} spills {size} bytes per lane"
    assert n > 0
