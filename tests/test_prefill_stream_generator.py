"""Host-side checks of the generator that writes the instruction stream of the pipelined pre-fill
kernel (no GPU): it runs for both dtypes, its own hazard check accepts the stream it emits and
rejects a planted violation, and the LDS geometry it assumes is conflict-free by construction."""
import importlib.util
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load():
    spec = importlib.util.spec_from_file_location(
        "gen_prefill_pipe", os.path.join(ROOT, "paper_2604_22782_amd", "csrc", "gen_prefill_pipe.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


MOD = _load()
GEN = {(nq, paged): MOD.generator(nq, bool(paged)) for nq in (2,) for paged in (0, 1)}   # the shape the library builds
G = GEN[(2, 0)]


@pytest.mark.parametrize("paged", [0, 1])
@pytest.mark.parametrize("nq", [2])
@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_stream_is_generated_and_self_consistent(dt, nq, paged):
    G = GEN[(nq, paged)]
    assert G.PAGED == bool(paged)
    assert (G.NQ, G.WAVES * G.NQ, G.THREADS) == (nq, 8, 512 // nq)
    lines = [l for l in G.generate(dt) if not l.startswith("//")]
    text = "\n".join(lines)
    n_mfma = sum(l.startswith("v_mfma") for l in lines)
    # per row block: prologue 8 + loop bodies of 32 (bf16: fast; general; masked) + the last O update 8
    n_bodies = 3 if dt == "bf16" else 2
    # bf16: five half tiles of scores are formed again where a wave leaves the fast bodies (8 each)
    assert n_mfma == nq * (8 + n_bodies * 32 + 8 + (5 * 8 if dt == "bf16" else 0))
    assert f"v_mfma_f32_32x32x16_{dt}" in text
    # every branch target exists exactly once
    labels = re.findall(r"^(L_\w+_%=):$", text, flags=re.M)
    assert len(labels) == len(set(labels))
    for tgt in re.findall(r"s_c?branch\w* (L_\w+_%=)", text):
        assert tgt in labels, tgt
    # one barrier in the prologue, one per loop body variant (the computing ones, one staging-only)
    assert sum(l == "s_barrier" for l in lines) == 2 + n_bodies
    if dt == "bf16":
        # the fast stream has no maximum and no subtraction: per score one exponential, one addition, half a packing
        i, j = lines.index("L_FAST_%=:"), lines.index("L_FAST_END_%=:")
        ops = [l.split()[0] for l in lines[i:j] if not l.endswith(":")]
        per_tile = 64 * 32 * nq // 64
        assert ops.count("v_exp_f32_e32") == per_tile and ops.count("v_cvt_pk_bf16_f32") == per_tile // 2
        assert not any(o.startswith(("v_max", "v_fma", "v_sub_f32", "v_mul_f32")) for o in ops)
        # both half steps end with the range check of the row sums, and each has its way out
        assert sum(l.startswith("s_cbranch_vccnz L_FALL_f") for l in lines[i:j]) == 2
        assert "L_ENTRY_g1_%=:" in lines and "L_TAIL_g_%=:" in lines
    # every register the stream names lies in the ranges the asm statement declares as clobbered
    for m in re.finditer(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]", text):
        lo = int(m.group(1) or m.group(2))
        hi = int(m.group(1) or m.group(3))
        assert G.FIRST_V <= lo <= hi <= G.LAST_V
    for m in re.finditer(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]", text):
        hi = int(m.group(1) or m.group(3))
        assert hi < 128 * nq
    assert G.LAST_V < 256      # one wave per SIMD: 256 vector and 256 accumulator registers per lane
    for m in re.finditer(r"\bs(\d+)\b|\bs\[(\d+):(\d+)\]", text):
        lo = int(m.group(1) or m.group(2))
        hi = int(m.group(1) or m.group(3))
        assert G.FIRST_S <= lo <= hi <= G.LAST_S


@pytest.mark.parametrize("nq,paged", [(2, 0), (2, 1)])
def test_hazard_check_accepts_the_stream_and_rejects_a_planted_read(nq, paged):
    G = GEN[(nq, paged)]
    lines = G.generate("bf16")
    G.check_mfma_results(lines)                      # the real stream: fine
    i = next(k for k, l in enumerate(lines) if l.startswith("v_mfma") and " v[" in l.split(",")[0])
    dst = int(re.match(r"v_mfma\w+ v\[(\d+):", lines[i]).group(1))
    planted = lines[:i + 1] + [f"v_add_f32_e32 v200, v200, v{dst}"] + lines[i + 1:]
    with pytest.raises(AssertionError):
        G.check_mfma_results(planted)
    # eleven instructions later the same read is allowed
    ok = lines[:i + 1] + ["s_nop 7", "s_nop 2", f"v_add_f32_e32 v200, v200, v{dst}"]
    G.check_mfma_results(ok)


def _piece_offset(piece, row):
    """Byte offset inside a 1 KiB chunk of the 16-byte piece `piece` (0..15) of row `row` (0..3)."""
    return 256 * (piece >> 2) + 64 * row + 16 * (piece & 3)


def test_lds_layout_is_bank_conflict_free():
    """64 banks x 4 bytes.  A load writes lane L's 16 bytes at 16 L of its chunk: the lane-to-(row,
    piece) map of the layout must fill the chunk exactly, with four neighbouring lanes on one row's
    64 contiguous bytes.  K operand: a pass of 16 lanes reads 16 bytes each of rows c = 0..15, same
    piece; V operand: a pass of 16 lanes reads 8 bytes each (4 rows x 4 x 8 bytes).  Every pass must
    touch each bank at most once."""
    chunk = G.CHUNK
    assert chunk == 1040
    for lane in range(64):
        row, piece = (lane >> 2) & 3, 4 * (lane >> 4) + (lane & 3)
        assert _piece_offset(piece, row) == 16 * lane
    for quad in range(16):
        rows = {(lane >> 2) & 3 for lane in range(4 * quad, 4 * quad + 4)}
        pieces = sorted(4 * (lane >> 4) + (lane & 3) for lane in range(4 * quad, 4 * quad + 4))
        assert len(rows) == 1 and pieces == list(range(pieces[0], pieces[0] + 4)) and pieces[0] % 4 == 0

    def banks(addr, nbytes):
        return [((addr + b) // 4) % 64 for b in range(0, nbytes, 4)]
    for hh in range(2):
        for s in range(8):
            for base_c in (0, 16):
                used = []
                for c in range(base_c, base_c + 16):
                    used += banks((c >> 2) * chunk + _piece_offset(2 * s + hh, c & 3), 16)
                assert len(used) == len(set(used)) == 64
    for hh in range(2):
        for a in range(2):
            for db in range(4):
                used = []
                for sl in range(16):   # key row 4 hh + sl / 4, d offset 32 db + 16 a + 4 (sl % 4): 8 bytes
                    d_byte = 2 * (32 * db + 16 * a + 4 * (sl & 3))
                    used += banks(hh * chunk + _piece_offset(d_byte // 16, sl >> 2) + d_byte % 16, 8)
                assert len(used) == len(set(used)) == 32
    # the ring fits the 160 KiB of LDS of a compute unit
    assert G.LDS_BYTES <= 160 * 1024
