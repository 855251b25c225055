"""Checks on the generated gfx950 code of the FFN kernels and of the attention
projections, which share the streaming building block (no GPU needed).

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
    asynchronous load has not landed yet);
  * no move, spill or LDS write reads the destination of such a load between the load
    and the explicit wait that covers it (the compiler believes the value is there as
    soon as the asm statement has been issued and could copy it, e.g. on a loop back edge).
"""
import os
import re

import pytest

from paper_2602_00879_amd import build as B


@pytest.fixture(scope="module", params=["des_ffn.hip", "des_attention.hip"])
def ffn_asm(request, tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / (request.param + ".s"))
    B.device_asm(request.param, out)
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


def _regs(operand):
    """Vector registers named by one operand: v7 -> {7}, v[4:7] -> {4..7}."""
    m = re.fullmatch(r"v(\d+)", operand)
    if m:
        return {int(m.group(1))}
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


_TRACKED = [0]  # hand-written loads seen by the scan (the check must not be vacuous)


def _scan_pending_reads(name, ins, pending, errors, prev=""):
    """Walks instructions in text order keeping the vector-memory operations that may
    still be outstanding (they complete in order, so a wait for at most n outstanding
    leaves the last n); an instruction that reads a destination still pending is an error."""
    for instr in ins:
        op, _, rest = instr.partition(" ")
        ops = [o.strip() for o in rest.split(",")] if rest else []
        w = re.search(r"vmcnt\((\d+)\)", instr) if op == "s_waitcnt" else None
        if w:
            n = int(w.group(1))
            pending[:] = pending[-n:] if n > 0 else []
            prev = instr
            continue
        is_vmem = op.startswith(("global_load", "global_store", "global_atomic", "buffer_", "flat_", "scratch_"))
        srcs = ops if op.startswith("global_store") else ops[1:]
        src_regs = set().union(*[_regs(re.sub(r"\s.*", "", o)) for o in srcs]) if srcs else set()
        busy = set().union(*[d for d in pending if d]) if pending else set()
        # what the compiler might do with a value it believes present: copy it (a move at a
        # loop back edge, a move to an accumulation register), spill it or store it.
        # Arithmetic is not flagged: a text-order scan cannot tell that the loop's last
        # trip issued no loads, and the epilogue reuses those registers legitimately.
        copies = op.startswith(("v_mov_b", "v_accvgpr", "v_pk_mov", "scratch_store", "ds_write", "v_swap"))
        if copies and src_regs & busy:
            errors.append(f"{name}: '{instr}' reads v{sorted(src_regs & busy)} before the wait that covers its load")
        if is_vmem:
            # the hand-written loads are the 16-byte non-temporal ones issued right after
            # their own `s_nop 4`; the compiler waits for its own loads itself
            mine = op == "global_load_dwordx4" and instr.endswith(" nt") and prev == "s_nop 4"
            pending.append(_regs(ops[0]) if mine else set())
            _TRACKED[0] += 1 if mine else 0
        prev = instr
    return prev


def test_no_read_of_an_asynchronously_loaded_register_before_its_wait(ffn_asm):
    """Only the loads of the long-block kernels are asynchronous in this sense; their
    kernels are scanned in text order and every loop body (a label followed later by a
    backward branch to it) a second time with the state at the branch, which covers a
    copy on the back edge."""
    errors = []
    n = 0
    _TRACKED[0] = 0
    for m in re.finditer(r"\n(_ZN3des\w*lds_kernel\w+):[^\n]*\n(.*?)\n\s*s_endpgm", ffn_asm, re.S):
        n += 1
        lines = [l.split(";")[0].strip() for l in m.group(2).split("\n")]
        lines = [l for l in lines if l and not l.startswith(".")]
        label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
        pending = []
        prev = ""
        for i, l in enumerate(lines):
            if l.endswith(":"):
                continue
            prev = _scan_pending_reads(m.group(1), [l], pending, errors, prev)
            b = re.match(r"s_cbranch\w+ (\S+)|s_branch (\S+)", l)
            tgt = (b.group(1) or b.group(2)) if b else None
            if tgt in label_at and label_at[tgt] < i:  # a back edge: once more round the loop
                body = [x for x in lines[label_at[tgt]:i + 1] if not x.endswith(":")]
                _scan_pending_reads(m.group(1), body, list(pending), errors)
    assert n > 0 and _TRACKED[0] > 40
    assert not errors, "\n".join(errors[:10])

