"""What the fast GEMM kernel relies on in the generated code, checked on the gfx950 assembly.

Its MFMAs are inline asm, so the compiler knows neither their latency nor the wait states an
accumulator read needs after one.  The kernel is only correct if nothing but an MFMA touches an
accumulator register between the first MFMA and the wait states that follow the last one:
no spill, no copy, no early read.  (No GPU needed: hipcc cross-compiles.)
"""
import re

import pytest

from paper_2602_20656_amd import build as lb

KERNELS = tuple("gemm_bf16_%s_kernelILb%dE" % (k, o) for k in ("nk", "kn", "nk_tail", "kn_tail") for o in (1, 0))
SMALL = tuple("gemm_bf16_%s128%s_kernelILb%dE" % (k, t, o) for k in ("nk", "kn") for t in ("", "_tail") for o in (1, 0))   # 128 x 128 tiles, 64 accumulators
MEDIUM = tuple("gemm_bf16_%s256x128%s_kernelILb%dE" % (k, t, o) for k in ("nk", "kn") for t in ("", "_tail") for o in (1, 0))   # 256 x 128 tiles, 128 accumulators
ACCS = {**{k: 256 for k in KERNELS}, **{k: 64 for k in SMALL}, **{k: 128 for k in MEDIUM}}
AGPR = re.compile(r"\ba(\[\d+:\d+\]|\d+)\b")


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    path = lb.device_assembly("gemm.hip", str(tmp_path_factory.mktemp("asm")))
    return open(path).read()


def _body(text, name):
    m = re.search(r"^(\S*%s\S*):.*\n" % re.escape(name), text, re.M)
    assert m, name
    end = text.index("s_endpgm", m.end())
    return m.group(1), [l.split(";")[0].strip() for l in text[m.end():end].splitlines()]


def _metadata(text, sym):
    """The amdhsa.kernels entry of one kernel as a dict of its scalar fields."""
    kernels = text[text.index("amdhsa.kernels:"):]
    for entry in re.split(r"\n  - (?=\.)", kernels):
        if re.search(r"\.name:\s+%s\b" % re.escape(sym), entry):
            return dict(re.findall(r"\.(\w+):\s+(\S+)", entry))
    raise AssertionError(sym)


@pytest.mark.parametrize("name", KERNELS + SMALL + MEDIUM)
def test_no_spills_and_all_agprs_for_accumulators(assembly, name):
    sym, _ = _body(assembly, name)
    meta = _metadata(assembly, sym)
    assert meta["vgpr_spill_count"] == "0" and meta["sgpr_spill_count"] == "0", meta
    assert meta["agpr_count"] == str(ACCS[name]), meta
    assert meta["private_segment_fixed_size"] == "0", meta


def _blocks(lines):
    """Basic blocks in text order: (falls_in, [instructions]); falls_in is False after an unconditional branch."""
    blocks, cur, falls_in = [], [], True
    for l in lines:
        if not l:
            continue
        if l.endswith(":") and not l.startswith("s_") and not l.startswith("v_"):
            prev = cur[-1] if cur else ""
            blocks.append((falls_in, cur))
            falls_in, cur = not prev.startswith("s_branch"), []
        else:
            cur.append(l)
    blocks.append((falls_in, cur))
    return blocks


@pytest.mark.parametrize("name", KERNELS + SMALL + MEDIUM)
def test_only_mfmas_touch_accumulators_until_the_wait_states(assembly, name):
    _, lines = _body(assembly, name)
    mfma = [i for i, l in enumerate(lines) if l.startswith("v_mfma_f32_16x16x32_bf16")]
    assert len(mfma) >= 3 * ACCS[name] // 2        # the steady-state step and at least two peeled steps
    nop = next(i for i in range(mfma[-1], len(lines)) if lines[i].startswith("s_nop 7"))
    assert lines[nop + 1].startswith("s_nop 7") and lines[nop + 2].startswith("s_nop 7")
    for falls_in, block in _blocks(lines[mfma[0]:nop]):
        has_mfma = any(l.startswith("v_mfma") for l in block)
        for l in block:
            if l.startswith("v_mfma_f32_16x16x32_bf16"):
                continue
            assert not l.startswith("scratch_"), l
            if AGPR.search(l):
                # the one exception: the zero fill of the accumulators on the path that skips the
                # steady-state loop, a block of its own that is only jumped to and holds no MFMA
                assert not has_mfma and not falls_in and l.startswith(("v_accvgpr_mov_b32", "v_accvgpr_write_b32")), l


@pytest.mark.parametrize("name", KERNELS)
def test_steady_state_step_is_branch_free_with_one_side_instruction_per_mfma(assembly, name):
    _, lines = _body(assembly, name)
    lines = [l for l in lines if l]
    # the loop: from its label to the first backward scalar branch behind the first MFMA
    first = next(i for i, l in enumerate(lines) if l.startswith("v_mfma"))
    back = next(i for i in range(first, len(lines)) if lines[i].startswith("s_cbranch"))
    label = lines[back].split()[-1] + ":"
    head = max(i for i in range(first) if lines[i].startswith(label))
    body = [l for l in lines[head + 1:back] if not l.endswith(":")]
    assert sum(l.startswith("v_mfma") for l in body) == 128
    assert sum(l.startswith("global_load_lds_dwordx4") for l in body) == 16
    if "_nk_" in name:
        assert sum(l.startswith("ds_read_b128") for l in body) == 32
    else:   # B stored [K,N]: 16 reads of A, 2 x 16 transposing reads of B
        assert sum(l.startswith("ds_read_b128") for l in body) == 16
        assert sum(l.startswith("ds_read_b64_tr_b16") for l in body) == 32
        assert not any(l.startswith(("v_mov_b32", "v_perm_b32")) for l in body)   # fragment halves land in place
    assert sum(l.startswith("s_barrier") for l in body) == 1
    run, worst, lead = 0, 0, None
    for l in body:      # side instructions between two MFMAs
        if l.startswith("v_mfma"):
            if lead is None:
                lead = run          # in front of the first MFMA: the loop's own bookkeeping
            else:
                worst = max(worst, run)
            run = 0
        elif not l.startswith(("s_waitcnt", "s_barrier")):
            run += 1
    assert worst <= 2, worst        # an M0 write, a load or a fragment read; nothing longer
    # slot rotation, two running pointers, the counter ([K,N]: and the slot's base added to 8 fragment addresses)
    assert lead + run <= 24, (lead, run)


@pytest.mark.parametrize("name", SMALL + MEDIUM)
def test_small_tile_step_has_one_side_instruction_per_mfma(assembly, name):
    ni = 4 if name in SMALL else 8          # A fragments per wavefront and k-slice; 4 B fragments
    _, lines = _body(assembly, name)
    lines = [l for l in lines if l]
    first = next(i for i, l in enumerate(lines) if l.startswith("v_mfma"))
    back = next(i for i in range(first, len(lines)) if lines[i].startswith("s_cbranch"))
    label = lines[back].split()[-1] + ":"
    head = max(i for i in range(first) if lines[i].startswith(label))
    body = [l for l in lines[head + 1:back] if not l.endswith(":")]
    assert sum(l.startswith("v_mfma") for l in body) == 2 * ni * 4
    assert sum(l.startswith("global_load_lds_dwordx4") for l in body) == ni + 4
    assert sum(l.startswith("s_barrier") for l in body) == 1
    if "_nk" in name:
        assert sum(l.startswith("ds_read_b128") for l in body) == 2 * (ni + 4)
    else:   # B stored [K,N]: reads of A, 2 x 8 transposing reads of B
        assert sum(l.startswith("ds_read_b128") for l in body) == 2 * ni
        assert sum(l.startswith("ds_read_b64_tr_b16") for l in body) == 16
    run, worst, seen = 0, 0, False
    for l in body:
        if l.startswith("v_mfma"):
            if seen:
                worst = max(worst, run)
            seen, run = True, 0
        elif not l.startswith(("s_waitcnt", "s_barrier")):
            run += 1
    assert worst <= 4, worst   # an address add or two with a read; an offset add with an M0 write
