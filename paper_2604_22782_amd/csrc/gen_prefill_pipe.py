#!/usr/bin/env python3
"""Writes the hand-scheduled gfx950 instruction stream of the pipelined pre-fill attention kernel
(prefill_pipe.hip includes the generated header).

Why a generated stream: the kernel keeps one wave per SIMD busy with 64 query rows, and its inner
loop only reaches the matrix-core rate if every MFMA is followed by a handful of independent
vector instructions (softmax of the previous 32 keys), LDS operand reads two operands ahead and
now and then a memory instruction of the tile three tiles ahead.  A lone wave issues in order:
a burst of slow instructions (transcendentals, memory) anywhere starves the matrix cores, so the
order of the ~450 instructions per 64-key tile and the ~400 registers per lane are fixed here.

What is computed (paper Eq. (3.1), pre-fill phase of Sec. 3.1.1): for a wave's 64 query rows
(two blocks of 32, "nq" = 0, 1) and the keys 0..position of each row,
  S^T = K Q^T (v_mfma_f32_32x32x16), online softmax down the columns, O^T += V^T P^T.
Keys are walked in half tiles of 32 ("u"); a half step runs, interleaved,
  matrix cores:  S^T(u+1)  and  O^T += V^T(u-1) P^T(u-1)
  vector ALU:    max / exp2 / row sums / 16-bit weights of S^T(u)
so the three stages of three consecutive half tiles are in flight at once.

K/V tiles (64 keys) go from HBM straight into LDS (buffer_load ... lds, no registers): lane L of
such a load writes 16 bytes at M0 + 16 L, so one instruction fills a 1 KiB chunk = 4 rows.  Inside
a chunk the 16-byte piece p of row r sits at 256 (p / 4) + 64 r + 16 (p % 4), so that four
neighbouring lanes fetch the 64 contiguous bytes of one row (the vector cache handles them as one
access), and chunks are 1040 bytes apart: both the 128-bit K operand reads (16 lanes = 16
consecutive rows, one piece) and the transposing 64-bit V reads (4 rows x 32 bytes per 16 lanes)
then touch every bank exactly once.
Four tile stages form a ring.  Tile t+3 is requested in the second half of tile t (its stage held
tile t-1, last read in the first half); one barrier per tile, placed after every wave has waited
for its own loads of tile t+1 and for its last reads of tile t-1, publishes the former and
releases the latter.  A load is in flight for about 1.75 tiles before anybody waits for it.

Boundaries of a row tile (a work group walks several, see prefill_pipe.hip).  What a wave pays there is
time at the memory pipeline, not arithmetic, so their shape follows the pipeline: Q is requested first and
tile 0 right behind it, tiles 1 and 2 only between the steps of the scaled copy (they are needed a tile
step later each); the output rows do not leave as the lanes hold them (16-byte pieces of 32 rows per
instruction) but through a private LDS region per wave behind the ring, 16 rows at a time, as whole rows
(4 rows of 256 contiguous bytes per store instruction); and a wave whose work group has no tile left
ends with its stores in flight.

bf16 only: tiles entirely below a wave's diagonal run a FAST copy of the loop body first.  It
multiplies K with a second copy of Q^T that carries scale x log2(e) (rounded to bf16 once more), so
the accumulators hold the exponents of the weights, and takes weight = 2^score without a running
maximum (bf16 weights have the exponent range of fp32): per score one v_exp, one v_add and half a
v_cvt_pk instead of v_max3 / v_fma / v_exp / v_add / v_cvt_pk.  After every half tile each lane's
sum of the half tile is checked against [2^-40, 2^9]; outside it the wave leaves, out of line, for
the general stream, which forms the scores again from the caller's Q and scales them in fp32 (so
nothing a result depends on was computed from the twice-rounded copy outside the checked range).

Register map (per lane):
  a[0:127]    O^T accumulators  [nq][d block of 32][16]
  a[128:191]  Q^T as MFMA B operand [nq][k step of 16][4]
  a[192:255]  bf16: Q^T x scale x log2(e), rounded to bf16 again (operand of the fast bodies)
  v[32:63], v[64:95]    S^T of even / odd half tiles [nq][16]
  v[96:111], v[112:127] P^T (16-bit pairs) of even / odd half tiles [nq][k step of 16 keys][4]
  v[128:...]  rings of K / V^T operands read from LDS, then softmax state, lane constants, addresses
  v[0:23], s[0:39] are left to the compiler for the operands of the asm statement.

generator(nq, paged) fixes the wave shape (nq row blocks of 32 per wave; the library builds nq = 2)
and whether the stream is the one for caches addressed through a block table (one block id per wave
and tile, see PAGED below).

Hazards the hardware does not interlock (MFMA result read by the vector ALU, transcendental
result read by the next instruction, lane-swap operands, M0 written right before a load to LDS)
are kept apart by construction or by s_nop; see the comments at the emit sites.
"""
from __future__ import annotations

import re
import sys
import types

def generator(nq: int = 2, paged: bool = False):
    """Everything that depends on the wave shape (nq row blocks of 32 per wave) and on the cache
    addressing (contiguous, or paged through a block table): register map, emitters, generate()."""
    # Layout of a 1 KiB chunk (4 rows x 16 pieces of 16 bytes): lane L = 16 (p / 4) + 4 r + p % 4, so
    # four neighbouring lanes fetch the 64 contiguous bytes of one row (one access of the vector cache
    # per four lanes); chunks are 1040 bytes apart.
    CHUNK = 1040              # 4 rows x 256 bytes + padding that turns the bank groups from chunk to chunk
    T_BYTES = 16 * CHUNK      # one tensor (K or V) of a 64-key tile
    STAGE = 2 * T_BYTES       # K then V
    N_STAGE = 4
    LDS_RING = N_STAGE * STAGE
    # Output rows leave through a private region per wave behind the ring (NQ = 2 only): 16 rows of 256 bytes,
    # 272 bytes apart, so that the 64-bit writes of 16 rows x 2 lane halves and the 128-bit reads of 4 rows x
    # 16 pieces each touch every bank once.
    OUT_ROW = 272
    OUT_REGION = 16 * OUT_ROW

    # ---- shape ------------------------------------------------------------------------------------------
    # NQ = row blocks of 32 per wave.  NQ = 2: 4 waves per work group, one per SIMD, ~400 registers per
    # lane, every LDS operand feeds two MFMAs.  NQ = 1: 8 waves per work group, two per SIMD, < 256
    # registers per lane, so the second wave can issue while the first waits.
    NQ = nq
    assert NQ in (1, 2)
    # PAGED = K/V rows are found through a block table (blocks of 2^shift >= 16 positions).  The 16 (or,
    # with 8 waves, 8) rows a wave stages per tile lie inside one block, so a wave needs ONE block id
    # per tile; it is loaded one tile ahead with a vector load (the same counter as the tile loads,
    # which complete in order) and moved to a scalar register.
    PAGED = bool(paged)
    WAVES = 8 // NQ                       # waves per work group (256 query rows)
    THREADS = 64 * WAVES
    CPW = 16 // WAVES                     # 1 KiB chunks per wave, tile and tensor
    LDS_BYTES = LDS_RING + (WAVES * OUT_REGION if NQ == 2 else 0)
    NEL = 16 * NQ                         # scores per lane and half tile

    # ---- register names ---------------------------------------------------------------------------
    PD = 2      # operand groups fetched ahead of the MFMAs that use them
    RING = 4    # operand buffers per ring (> PD)

    FIRST_V = 24 if NQ == 2 else 8        # v[0:FIRST_V) are left to the compiler
    _next = [32 if NQ == 2 else 8]


    def _alloc(n=1, align=1):
        base = (_next[0] + align - 1) // align * align
        _next[0] = base + n
        return base


    SA, SB = _alloc(16 * NQ, 4), _alloc(16 * NQ, 4)      # S^T of even / odd half tiles [nq][16]
    PA, PB = _alloc(8 * NQ, 4), _alloc(8 * NQ, 4)        # P^T of even / odd half tiles [nq][2][4]
    KO = _alloc(4 * RING, 4)
    VO = _alloc(4 * RING, 4)
    _per_q = lambda: tuple(_alloc() for _ in range(NQ))
    T_MAX, T_MAX2, M_NEW, M_RUN, NEG_MC, L_SUM, ALPHA, LIM, DIFF = (_per_q() for _ in range(9))
    LANE, COL, HH = _alloc(), _alloc(), _alloc()
    KL, VL = _alloc(), _alloc()            # lane parts of the K / V^T read addresses (LDS base included)
    KA_CUR, KA_NXT = _alloc(), _alloc()    # K read address of tile t / t+1
    VA_PRV, VA_CUR = _alloc(), _alloc()    # V^T read address of tile t-1 / t
    ROWB, PIECE = _alloc(), _alloc()       # staging: first row of this lane in a tile, byte offset of its piece
    VOFF = tuple(_alloc() for _ in range(CPW))   # byte offsets of this lane's rows of the tile being fetched
    VBO = tuple(_alloc() for _ in range(CPW))    # ... in tile 0 (constants)
    LIMV = _alloc()                        # byte offset of the lane's piece in the last needed row
    V_BLK, V_TOFF, V_T, V_L4 = _alloc(), _alloc(), _alloc(), _alloc()   # paged: block id, table offset, temp, lane % 4
    NEG_INF = _alloc()
    STG = _alloc()
    Q_OFF, O_OFF, ROW = _per_q(), _per_q(), _per_q()
    TMP = tuple(range(_alloc(16, 2), _next[0]))   # scratch; TMP[4:6] and TMP[12:14] are 64-bit store operands
    NT = 8                                 # weights of the fast stream on their way from v_exp to row sum and packing
    EXPT = tuple(_alloc() for _ in range(NT))
    P_SUM = _per_q()                       # fast stream: row sums of the half tile
    LAST_V = (_next[0] + 7) // 8 * 8 - 1
    assert LAST_V < 256 and PD < RING and TMP[4] % 2 == 0 and TMP[12] % 2 == 0

    A_O, A_Q = 0, 64 * NQ
    FAST_SPAN = (9 + 40) << 23      # bit pattern of 2^9 minus that of 2^-40: the range of lane sums the fast stream keeps
    A_QS = 96 * NQ            # bf16: a second copy of Q^T, multiplied by scale x log2(e) (operand of the fast stream)
    # softmax software pipeline: element i gets its fma at step i, its exponential EXP_LAG steps later,
    # and is first read (row sum, 16-bit packing) USE_LAG steps later
    EXP_LAG = 2
    USE_LAG = 4
    # first gap of a half step that takes softmax instructions.  The vector ALU may read an MFMA result
    # only 11 issued instructions after the MFMA (no hardware interlock); check_mfma_results() verifies it.
    FIRST_GAP = 0

    S_T, S_TMP, S_STW, S_J0, S_FLAG = 40, 41, 42, 43, 44
    S_CMP = 46                     # pair
    S_ST_NXT, S_ST_CUR = 48, 49    # LDS offsets of the stages of tiles t+1, t
    S_ONES, S_NCS, S_WBASE = 50, 51, 52
    S_ST_PRV = 53                  # ... of tile t-1 (the stage tile t+3 goes to)
    S_EXEC = 54                    # pair
    S_NK1 = 56
    S_SOFF, S_NKM63 = 57, 58       # scalar byte offset of the tile being requested; last needed key - 63

    TBL = 1 if PAGED else 0         # extra loads per tile in the queue of the tile loads (the block id)
    S_BLK, S_R0, S_R0W, S_LASTIDX, S_T2 = 60, 61, 62, 63, 64   # paged: block id, first row of the wave's part, ...

    FIRST_S, LAST_S = 40, 64 if PAGED else 59


    class Asm:
        def __init__(self, dt: str):
            self.dt = dt              # "bf16" or "f16"
            self.lines: list[str] = []
            self.lds: list[object] = []   # LDS operations in program order (tags)
            self.waited = -1              # index of the newest operation known to be complete
            self.uid = 0

        def e(self, s: str):
            self.lines.extend(s.split("\n"))

        def c(self, s: str):
            self.lines.append("// " + s)

        def fresh(self) -> int:
            self.uid += 1
            return self.uid

        # LDS operations complete in order; lgkmcnt(n) waits until at most n are outstanding.
        def lds_op(self, text: str, tag):
            self.e(text)
            self.lds.append(tag)

        def wait_lds(self, tag):
            idx = max(i for i, t in enumerate(self.lds) if t == tag)
            if idx <= self.waited:
                return
            n = len(self.lds) - 1 - idx
            self.e(f"s_waitcnt lgkmcnt({min(n, 15)})")
            self.waited = len(self.lds) - 1 - min(n, 15)

        def reset_lds(self, pending):
            self.lds = list(pending)
            self.waited = -1


    def vr(b, n=1):
        return f"v{b}" if n == 1 else f"v[{b}:{b + n - 1}]"


    def ar(b, n=1):
        return f"a{b}" if n == 1 else f"a[{b}:{b + n - 1}]"


    def sr(b, n=1):
        return f"s{b}" if n == 1 else f"s[{b}:{b + n - 1}]"


    # ---- softmax of one half tile (vector ALU stream) ------------------------------------------------
    def fast_stream(A: Asm, s_cur: int, p_cur: int):
        """The softmax of a half tile without a running maximum (bf16 weights, tiles below the
        diagonal): weight = 2^score, straight from the accumulators.  The fast bodies multiply K with
        the copy of Q that was multiplied by scale x log2(e) and rounded to bf16 again, so the
        accumulators hold the exponents; bf16 weights have the exponent range of fp32, so no
        reference point is needed for moderate scores.  half_step() checks after every half tile
        that each lane's sum of the half tile lies in [2^-40, 2^9] (scores between about -40 and
        +8 in log2 units; the second rounding of Q moves a score by up to 2^-9 of its size, which is why
        the upper end is where it is and not at the 2^14 that overflow alone would allow) and
        otherwise leaves for the general stream, which recomputes the scores from the caller's Q and
        scales them in fp32.  Per score: v_exp, v_add, half a v_cvt_pk -- the maximum (v_max3 per two
        scores) and the multiply-subtract (one per score) of the general stream are gone."""
        assert A.dt == "bf16"
        o = []
        S = [[s_cur + 16 * q + r for r in range(16)] for q in range(NQ)]
        elems = [(i % NQ, i // NQ) for i in range(NEL)]
        lag = 4
        assert NT > lag + NQ
        for i in range(NEL + lag):
            if i < NEL:
                q, r = elems[i]
                o.append(f"v_exp_f32_e32 {vr(EXPT[i % NT])}, {vr(S[q][r])}")
            if i >= lag:
                j = i - lag
                q, r = elems[j]
                if r == 0:
                    o.append(f"v_mov_b32_e32 {vr(P_SUM[q])}, {vr(EXPT[j % NT])}")
                else:
                    o.append(f"v_add_f32_e32 {vr(P_SUM[q])}, {vr(P_SUM[q])}, {vr(EXPT[j % NT])}")
                if r % 2 == 1:      # its partner (q, r - 1) was element j - NQ
                    o.append(f"v_cvt_pk_bf16_f32 {vr(p_cur + 8 * q + r // 2)}, {vr(EXPT[(j - NQ) % NT])}, {vr(EXPT[j % NT])}")
        return o

    def softmax_stream(A: Asm, s_cur: int, p_cur: int, masked: bool, tagid: str):
        """Returns a list of instruction strings.  s_cur: 32 registers [nq][16], element r of a block is
        key 8 (r / 4) + 4 hh + (r % 4) of the half tile.  p_cur: 16 registers [nq][2][4]."""
        o = []
        S = [[s_cur + 16 * q + r for r in range(16)] for q in range(NQ)]
        if masked:
            # key offset inside the half tile vs. (row position - first key of the half tile - 4 hh)
            for r in range(16):
                for q in range(NQ):
                    kk = 8 * (r // 4) + (r % 4)
                    o.append(f"v_cmp_lt_i32_e64 vcc, {vr(LIM[q])}, {kk}")
                    o.append(f"v_cndmask_b32_e32 {vr(S[q][r])}, {vr(S[q][r])}, {vr(NEG_INF)}, vcc")
        for q in range(NQ):
            o.append(f"v_max3_f32 {vr(T_MAX[q])}, {vr(S[q][0])}, {vr(S[q][1])}, {vr(S[q][2])}")
        for k in range(6):
            for q in range(NQ):
                o.append(f"v_max3_f32 {vr(T_MAX[q])}, {vr(T_MAX[q])}, {vr(S[q][3 + 2 * k])}, {vr(S[q][4 + 2 * k])}")
        for q in range(NQ):
            o.append(f"v_max_f32_e32 {vr(T_MAX[q])}, {vr(T_MAX[q])}, {vr(S[q][15])}")
        for q in range(NQ):
            o.append(f"v_mov_b32_e32 {vr(T_MAX2[q])}, {vr(T_MAX[q])}")
        # the lane swap must not follow a vector write of its operands within two issue slots
        o.append("s_nop 1")
        for q in range(NQ):
            # lanes 32-63 of the first operand <-> lanes 0-31 of the second: afterwards the first holds
            # the lower half's value in both halves, the second the upper half's
            o.append(f"v_permlane32_swap_b32_e32 {vr(T_MAX[q])}, {vr(T_MAX2[q])}")
        o.append("s_nop 1")
        for q in range(NQ):
            o.append(f"v_max3_f32 {vr(M_NEW[q])}, {vr(T_MAX[q])}, {vr(T_MAX2[q])}, {vr(M_RUN[q])}")
        for q in range(NQ):
            o.append(f"v_sub_f32_e32 {vr(DIFF[q])}, {vr(M_NEW[q])}, {vr(M_RUN[q])}")
        # rescale only when some row's maximum grew by more than 2^8 in weight (threshold in raw scores)
        if NQ == 2:
            o.append(f"v_cmp_lt_f32_e64 {sr(S_CMP, 2)}, %[thr], {vr(DIFF[0])}")
            o.append(f"v_cmp_lt_f32_e32 vcc, %[thr], {vr(DIFF[1])}")
            o.append(f"s_or_b64 vcc, vcc, {sr(S_CMP, 2)}")
        else:
            o.append(f"v_cmp_lt_f32_e32 vcc, %[thr], {vr(DIFF[0])}")
        # one entry: nothing may be scheduled between the branch and the label its target returns to
        o.append(f"s_cbranch_vccnz L_RESC_{tagid}_%=\nL_RET_{tagid}_%=:")
        # weights 2^(cs s - cs m), their row sums and their 16-bit form, software-pipelined element by
        # element so that the slow transcendental instructions are spread evenly between the MFMAs
        # (a run of them would leave the matrix cores waiting for the in-order instruction stream).
        # A v_exp result is first read two instructions later; v_dot2 would sum the rounded pairs in one
        # instruction but runs on the matrix pipeline and does not overlap with MFMAs.
        elems = [(i % NQ, i // NQ) for i in range(NEL)]  # (q, r), alternating row blocks

        def pack(q, j):
            d = p_cur + 8 * q + j
            if A.dt == "bf16":
                return [f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(S[q][2 * j])}, {vr(S[q][2 * j + 1])}"]
            return [f"v_cvt_f16_f32_e32 {vr(S[q][2 * j])}, {vr(S[q][2 * j])}",
                    f"v_cvt_f16_f32_e32 {vr(S[q][2 * j + 1])}, {vr(S[q][2 * j + 1])}",
                    f"v_pack_b32_f16 {vr(d)}, {vr(S[q][2 * j])}, {vr(S[q][2 * j + 1])}"]

        for i in range(NEL + USE_LAG):
            if i < NEL:
                q, r = elems[i]
                o.append(f"v_fma_f32 {vr(S[q][r])}, {vr(S[q][r])}, %[cs], {vr(NEG_MC[q])}")
            if EXP_LAG <= i < NEL + EXP_LAG:
                q, r = elems[i - EXP_LAG]
                o.append(f"v_exp_f32_e32 {vr(S[q][r])}, {vr(S[q][r])}")
            if USE_LAG <= i < NEL + USE_LAG:
                q, r = elems[i - USE_LAG]
                o.append(f"v_add_f32_e32 {vr(L_SUM[q])}, {vr(L_SUM[q])}, {vr(S[q][r])}")
                if r % 2 == 1:  # both elements of register pair (q, r / 2) are final
                    o += pack(q, r // 2)
        if masked:
            for q in range(NQ):
                o.append(f"v_subrev_u32_e32 {vr(LIM[q])}, 32, {vr(LIM[q])}")
        return o


    def rescale_blocks(A: Asm, tagid: str):
        """Out-of-line code of one half step: new running maximum, and the deferred O rescale."""
        A.e(f"L_RESC_{tagid}_%=:")
        for q in range(NQ):
            A.e(f"v_sub_f32_e32 {vr(ALPHA[q])}, {vr(M_RUN[q])}, {vr(M_NEW[q])}")
        for q in range(NQ):
            A.e(f"v_mul_f32_e32 {vr(ALPHA[q])}, %[cs], {vr(ALPHA[q])}")
        for q in range(NQ):
            A.e(f"v_exp_f32_e32 {vr(ALPHA[q])}, {vr(ALPHA[q])}")
        for q in range(NQ):
            A.e(f"v_mov_b32_e32 {vr(M_RUN[q])}, {vr(M_NEW[q])}")
        for q in range(NQ):
            A.e(f"v_mul_f32_e32 {vr(NEG_MC[q])}, {sr(S_NCS)}, {vr(M_NEW[q])}")
        for q in range(NQ):  # >= 4 instructions after the exponentials
            A.e(f"v_mul_f32_e32 {vr(L_SUM[q])}, {vr(L_SUM[q])}, {vr(ALPHA[q])}")
        A.e(f"s_mov_b32 {sr(S_FLAG)}, 1")
        A.e(f"s_branch L_RET_{tagid}_%=")

        A.e(f"L_RESO_{tagid}_%=:")
        # the accumulators were last written by MFMAs issued a few instructions ago: let them retire
        for _ in range(3):
            A.e("s_nop 7")
        for q in range(NQ):
            for i in range(0, 64, 8):
                for k in range(8):
                    A.e(f"v_accvgpr_read_b32 {vr(TMP[k])}, {ar(A_O + 64 * q + i + k)}")
                for k in range(8):
                    A.e(f"v_mul_f32_e32 {vr(TMP[k])}, {vr(TMP[k])}, {vr(ALPHA[q])}")
                for k in range(8):
                    A.e(f"v_accvgpr_write_b32 {ar(A_O + 64 * q + i + k)}, {vr(TMP[k])}")
        A.e("s_nop 7")
        A.e(f"s_mov_b32 {sr(S_FLAG)}, 0")
        A.e(f"s_branch L_RESO_RET_{tagid}_%=")


    # ---- operand reads -----------------------------------------------------------------------------
    def k_read(A: Asm, addr: int, kb: int, g: int, tag):
        dst = KO + 4 * (g % RING)
        step = 256 * (g // 2) + 32 * (g % 2)     # pieces 2 g, 2 g + 1 of the row
        A.lds_op(f"ds_read_b128 {vr(dst, 4)}, {vr(addr)} offset:{kb * 8 * CHUNK + step}", tag)


    def v_read(A: Asm, addr: int, kb: int, g: int, tag_lo, tag_hi):
        x, db = g // 4, g % 4
        dst = VO + 4 * (g % RING)
        off = (kb * 8 + 4 * x) * CHUNK + db * 256
        A.lds_op(f"ds_read_b64_tr_b16 {vr(dst, 2)}, {vr(addr)} offset:{off}", tag_lo)
        A.lds_op(f"ds_read_b64_tr_b16 {vr(dst + 2, 2)}, {vr(addr)} offset:{off + 2 * CHUNK}", tag_hi)


    def half_step(A: Asm, hs: int, qk, pv, sm, nxt, extra, tagid: str, cold=False, publish=False):
        """One half step.
        qk  = (K address register, key block, S destination base[, scaled]) or None; scaled: multiply with
              the copy of Q^T that carries scale x log2(e) (fast bodies)
        pv  = (V address register, key block, P source base) or None
        sm  = (S source base, P destination base, masked[, fast]) or None; fast: the stream without a
              running maximum (fast_stream), followed by the range check of the row sums
        nxt = ((K address register, key block) or None, (V address register, key block) or None):
              operands of the next half step's first PD groups, fetched at the end of this one
        extra = ({gap: [instructions issued first]}, {gap: [instructions issued last]}) (staging)
        publish: before it requests the first operands of the next half step (the first reads of the
              newly published tile) the wave waits for its loads of that tile and for its own
              outstanding operand reads, then meets the other waves at the barrier.
        hs  = serial number of the half step inside the emitted code (tags of its operand reads)."""
        fast = bool(sm) and len(sm) > 3 and sm[3]
        valu = [] if not sm else fast_stream(A, sm[0], sm[1]) if fast else softmax_stream(A, sm[0], sm[1], sm[2], tagid)
        # MFMAs of the half step in issue order; a "gap" of other instructions follows each of them
        slots = []
        for g in range(8):
            for q in range(NQ):
                if qk:
                    slots.append(("qk", g, q))
                if pv:
                    slots.append(("pv", g, q))
        n = len(slots)
        gaps = [[] for _ in range(n)]
        head, tail = extra or ({}, {})
        for gi, lst in head.items():   # positions given on a scale of 32
            gaps[gi * n // 32].extend(lst)
        # An in-order wave reaches the next MFMA only after issuing everything before it: time per
        # MFMA is max(32 clocks of the matrix pipe, issue time of its gap).  Spread the vector stream
        # by issue cost (a transcendental costs about three plain instructions).
        def cost(ins):
            return 0 if ins.endswith(":") else 3 if ins.startswith("v_exp") else 1
        total = sum(cost(i) for i in valu)
        ngap = n - FIRST_GAP
        done, gi = 0, 0
        for ins in valu:
            while gi < ngap - 1 and done >= total * (gi + 1) / ngap:
                gi += 1
            gaps[FIRST_GAP + gi].append(ins)
            done += cost(ins)
        for gi, lst in tail.items():
            assert len(gaps[gi * n // 32]) >= 2   # something is issued between an M0 write and its load
            gaps[gi * n // 32].extend(lst)

        def fetch(hs_id, g, kcfg, vcfg):
            if kcfg:
                k_read(A, kcfg[0], kcfg[1], g, ("K", hs_id, g))
            if vcfg:
                v_read(A, vcfg[0], vcfg[1], g, ("Vl", hs_id, g), ("Vh", hs_id, g))

        kcfg = (qk[0], qk[1]) if qk else None
        vcfg = (pv[0], pv[1]) if pv else None
        if cold:
            for g in range(PD):
                fetch(hs, g, kcfg, vcfg)
        cur_g = -1
        for si, (kind, g, q) in enumerate(slots):
            if g != cur_g:   # first MFMA of operand group g
                cur_g = g
                if publish and g + PD == 8:
                    # every operand of this half step has been requested: wait for the last one (reads
                    # return in order), for this wave's loads of the tile after next, then meet the others
                    A.wait_lds(("Vh", hs, 7))
                    A.e(f"s_waitcnt vmcnt({2 * CPW + TBL})")  # all but the newest loads (the tile requested last) landed
                    A.e("s_barrier")
                if g + PD < 8:
                    fetch(hs, g + PD, kcfg, vcfg)
                elif nxt is not None:
                    fetch(hs + 1, g + PD - 8, nxt[0], nxt[1])
                # one wait per group: the V^T pair was requested after the K operand and returns after it
                A.wait_lds(("Vh", hs, g) if pv else ("K", hs, g))
            ko, vo = KO + 4 * (g % RING), VO + 4 * (g % RING)
            if kind == "qk":
                s_dst = qk[2] + 16 * q
                c_in = "0" if g == 0 else vr(s_dst, 16)
                a_q = A_QS if (len(qk) > 3 and qk[3]) else A_Q
                A.e(f"v_mfma_f32_32x32x16_{A.dt} {vr(s_dst, 16)}, {vr(ko, 4)}, {ar(a_q + 32 * q + 4 * g, 4)}, {c_in}")
            else:
                x, db = g // 4, g % 4
                p_src = pv[2] + 8 * q + 4 * x
                acc = A_O + 64 * q + 16 * db
                A.e(f"v_mfma_f32_32x32x16_{A.dt} {ar(acc, 16)}, {vr(vo, 4)}, {vr(p_src, 4)}, {ar(acc, 16)}")
            for ins in gaps[si]:
                A.e(ins)
        if fast:
            # every lane's sum of the half tile inside [2^-40, 2^9]?  One unsigned compare per row block:
            # the bit pattern of a positive float minus that of 2^-40 is at most that of 2^9 minus that of
            # 2^-40 exactly then (smaller sums wrap around, infinities and NaNs are above).  Otherwise the
            # wave leaves for the general stream (out of line, never returns); else the sums join the
            # running row sums.
            for q in range(NQ):
                A.e(f"v_subrev_u32_e32 {vr(TMP[q])}, 0x2b800000, {vr(P_SUM[q])}")
            A.e(f"v_cmp_lt_u32_e32 vcc, 0x{FAST_SPAN:08x}, {vr(TMP[0])}")
            for q in range(1, NQ):
                A.e(f"s_mov_b64 {sr(S_CMP, 2)}, vcc")
                A.e(f"v_cmp_lt_u32_e32 vcc, 0x{FAST_SPAN:08x}, {vr(TMP[q])}")
                A.e(f"s_or_b64 vcc, vcc, {sr(S_CMP, 2)}")
            A.e(f"s_cbranch_vccnz L_FALL_{tagid}_%=")
            for q in range(NQ):
                A.e(f"v_add_f32_e32 {vr(L_SUM[q])}, {vr(L_SUM[q])}, {vr(P_SUM[q])}")
        elif sm:
            A.e(f"s_cmp_lg_u32 {sr(S_FLAG)}, 0")
            A.e(f"s_cbranch_scc1 L_RESO_{tagid}_%=")
            A.e(f"L_RESO_RET_{tagid}_%=:")


    def pending_reads(hs, with_k=True, with_v=True):
        out = []
        for g in range(PD):
            if with_k:
                out.append(("K", hs, g))
            if with_v:
                out += [("Vl", hs, g), ("Vh", hs, g)]
        return out


    # ---- staging (HBM -> LDS) -------------------------------------------------------------------------
    def clamped_offsets():
        """Byte offsets of the lane's four rows of the tile whose first row is at byte S_SOFF, rows
        past the last needed key repeating it (finite, and masked wherever they are not the real
        key); the scalar offset then is zero.  Paged: S_SOFF is the byte offset of the wave's first row
        (S_R0 its position), and a row is past the end by position, not by offset."""
        o = []
        for i in range(CPW):
            if PAGED:
                o.append(f"s_add_u32 {sr(S_T2)}, {sr(S_R0)}, {4 * i}")
                o.append(f"v_add_u32_e32 {vr(V_T)}, {sr(S_T2)}, {vr(V_L4)}")
                o.append(f"v_cmp_lt_u32_e32 vcc, {sr(S_NK1)}, {vr(V_T)}")
                o.append(f"v_add_u32_e32 {vr(VOFF[i])}, {sr(S_SOFF)}, {vr(VBO[i])}")
                o.append(f"v_cndmask_b32_e32 {vr(VOFF[i])}, {vr(VOFF[i])}, {vr(LIMV)}, vcc")
            else:
                o.append(f"v_add_u32_e32 {vr(VOFF[i])}, {sr(S_SOFF)}, {vr(VBO[i])}")
                o.append(f"v_min_u32_e32 {vr(VOFF[i])}, {vr(LIMV)}, {vr(VOFF[i])}")
        o.append(f"s_mov_b32 {sr(S_SOFF)}, 0")
        return o


    def paged_tile_offset(tagid: str):
        """Paged: S_J0 = first position of the tile.  The block id of the wave's part of it has landed in
        V_BLK; S_SOFF = byte offset of the wave's first row.  Then the id of the next tile is requested."""
        return [f"s_waitcnt vmcnt({2 * CPW})",                       # the id was requested before the previous tile's loads
                f"v_readfirstlane_b32 {sr(S_BLK)}, {vr(V_BLK)}",
                f"s_cmp_lt_u32 {sr(S_BLK)}, %[nblk]",
                f"s_cbranch_scc0 L_BADBLK_{tagid}_%=\nL_BADRET_{tagid}_%=:",
                f"s_add_u32 {sr(S_R0)}, {sr(S_J0)}, {sr(S_R0W)}",
                f"s_and_b32 {sr(S_T2)}, {sr(S_R0)}, %[bsm1]",
                f"s_lshl_b32 {sr(S_SOFF)}, {sr(S_BLK)}, %[shift]",
                f"s_add_u32 {sr(S_SOFF)}, {sr(S_SOFF)}, {sr(S_T2)}",
                f"s_mul_i32 {sr(S_SOFF)}, {sr(S_SOFF)}, %[krb]"] + paged_request_id(64)


    def paged_request_id(ahead: int):
        """Requests the block id of the wave's part of the tile `ahead` positions after S_R0's tile (the
        table index is clamped to the last block the work group needs: tiles past the end repeat it)."""
        return [f"s_add_u32 {sr(S_T2)}, {sr(S_R0)}, {ahead}",
                f"s_lshr_b32 {sr(S_T2)}, {sr(S_T2)}, %[shift]",
                f"s_min_u32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_LASTIDX)}",
                f"s_lshl_b32 {sr(S_T2)}, {sr(S_T2)}, 2",
                f"v_mov_b32_e32 {vr(V_TOFF)}, {sr(S_T2)}",
                f"global_load_dword {vr(V_BLK)}, {vr(V_TOFF)}, %[tbl]"]


    def bad_block_paths(A: Asm, tags):
        """Out of line: a block id outside the pool raises the fault word; the rows are read as zeros
        (an offset past the end of the buffer descriptor)."""
        for tagid in tags:
            A.e(f"L_BADBLK_{tagid}_%=:")
            A.e(f"v_mov_b32_e32 {vr(V_T)}, 2")                        # SKV_FAULT_BLOCK_ID
            A.e(f"v_mov_b32_e32 {vr(V_TOFF)}, 0")
            A.e(f"global_atomic_or {vr(V_TOFF)}, {vr(V_T)}, %[flt]")
            A.e("s_waitcnt vmcnt(0)")                                   # keeps the in-order accounting of the loads simple
            A.e(f"s_mov_b32 {sr(S_BLK)}, %[nblk]")
            A.e(f"s_branch L_BADRET_{tagid}_%=")


    def tile_load(which: str, i: int, base_sreg: int):
        """Chunk 4 w + i of K or V: lane L fetches its piece of its row of the chunk (see CHUNK).  Returns
        (M0 write, load): another instruction must be issued between the two."""
        srd, off = ("%[srdk]", 0) if which == "k" else ("%[srdv]", T_BYTES)
        return (f"s_add_u32 m0, {sr(base_sreg)}, {off + i * CHUNK}",
                f"buffer_load_dwordx4 {vr(VOFF[i])}, {srd}, {sr(S_SOFF)} offen lds")


    def staging_ops(tagid: str):
        """Requests tile t+3 (second half step of tile t) into the stage tile t-1 just left.  Returns
        ({gap: [instructions issued first in the gap]}, {gap: [instructions issued last]}).  While
        the whole tile lies before the last needed key its row offsets are the constants of tile 0
        plus a scalar offset; only the tail tiles pay for the clamp.  The memory instructions are kept
        three gaps apart: a burst of them would hold up the in-order stream."""
        head = {0: [f"s_add_u32 {sr(S_STW)}, {sr(S_ST_PRV)}, {sr(S_WBASE)}",
                    f"s_lshl_b32 {sr(S_J0)}, {sr(S_T)}, 6",
                    f"s_add_u32 {sr(S_J0)}, {sr(S_J0)}, 192"] +
                   (paged_tile_offset(tagid) if PAGED else [f"s_mul_i32 {sr(S_SOFF)}, {sr(S_J0)}, %[krb]"]) +
                   [f"s_cmp_le_i32 {sr(S_J0)}, {sr(S_NKM63)}",
                    "\n".join([f"s_cbranch_scc1 L_INRANGE_{tagid}_%="] + clamped_offsets() + [f"L_INRANGE_{tagid}_%=:"])]}
        tail = {}
        n = 0
        for i in range(CPW):
            for which in ("k", "v"):
                m0w, ld = tile_load(which, i, S_STW)
                head[2 + (12 // CPW) * n] = [m0w]
                tail[2 + (12 // CPW) * n] = [ld]
                n += 1
        return head, tail


    def rotate_addresses(A: Asm, vector=True):
        """Top of tile t: stage offsets and operand addresses move on by one tile."""
        if vector:
            A.e(f"v_mov_b32_e32 {vr(KA_CUR)}, {vr(KA_NXT)}")
            A.e(f"v_mov_b32_e32 {vr(VA_PRV)}, {vr(VA_CUR)}")
        A.e(f"s_mov_b32 {sr(S_ST_PRV)}, {sr(S_ST_CUR)}")
        A.e(f"s_mov_b32 {sr(S_ST_CUR)}, {sr(S_ST_NXT)}")
        A.e(f"s_add_u32 {sr(S_ST_NXT)}, {sr(S_ST_NXT)}, {STAGE}")
        A.e(f"s_cmp_lt_u32 {sr(S_ST_NXT)}, {N_STAGE * STAGE}")
        A.e(f"s_cselect_b32 {sr(S_ST_NXT)}, {sr(S_ST_NXT)}, 0")
        if vector:
            A.e(f"v_add_u32_e32 {vr(KA_NXT)}, {sr(S_ST_NXT)}, {vr(KL)}")
            A.e(f"v_add_u32_e32 {vr(VA_CUR)}, {sr(S_ST_CUR)}, {vr(VL)}")


    def body(A: Asm, masked: bool, name: str, fast=False, entries=False):
        """Tile t for a computing wave: half steps u = 2t and 2t + 1.  entries: labels at the start of
        the second half step and behind it, where a wave that left the fast stream joins this body
        (the matrix-core, LDS and staging instructions of all bodies are the same, so the counters of
        outstanding LDS reads and loads agree at these points)."""
        A.reset_lds(pending_reads(0))
        rotate_addresses(A)
        half_step(A, 0, qk=(KA_CUR, 1, SB, fast), pv=(VA_PRV, 1, PB), sm=(SA, PA, masked, fast),
                  nxt=((KA_NXT, 0), (VA_CUR, 0)), extra=None, tagid=name + "0", publish=True)
        if entries:
            A.e(f"L_ENTRY_{name}1_%=:")
        half_step(A, 1, qk=(KA_NXT, 0, SA, fast), pv=(VA_CUR, 0, PA), sm=(SB, PB, masked, fast),
                  nxt=((KA_NXT, 1), (VA_CUR, 1)), extra=staging_ops(name), tagid=name + "1")
        if entries:
            A.e(f"L_TAIL_{name}_%=:")
        assert A.lds[-3 * PD:] == pending_reads(2), A.lds[-6:]


    def recompute_scores(A: Asm, addr: int, kb: int, s_dst: int):
        """S^T of key block kb of the tile at LDS address `addr` once more, from the caller's Q^T (the
        fast bodies multiply with its scaled copy).  Used where a wave passes from the fast bodies to
        the general ones; the operands go through TMP, not through the rings, which already hold
        operands of the next half step.  The reads are not entered in the generator's count of LDS
        operations: they are complete when the block ends, so every later wait still covers what it
        is meant to cover."""
        for g in range(8):
            t = TMP[4 * (g % 2)]
            step = 256 * (g // 2) + 32 * (g % 2)
            A.e(f"ds_read_b128 {vr(t, 4)}, {vr(addr)} offset:{kb * 8 * CHUNK + step}")
            A.e("s_waitcnt lgkmcnt(0)")
            for q in range(NQ):
                dst = s_dst + 16 * q
                c_in = "0" if g == 0 else vr(dst, 16)
                A.e(f"v_mfma_f32_32x32x16_{A.dt} {vr(dst, 16)}, {vr(t, 4)}, {ar(A_Q + 32 * q + 4 * g, 4)}, {c_in}")
        for _ in range(3):                    # the results are read by the vector ALU next
            A.e("s_nop 7")


    def fallback_block(A: Asm, tagid: str, cur, nxt, p_cur: int, resume: str):
        """Out of line, reached from the range check of the fast stream's half step `tagid`: the weights
        of the half tile left the range in which the fast stream is used.  cur, nxt = (K address
        register, key block, S base) of this half tile and of the next one, whose scores the half step
        has just formed with the scaled Q: both are formed again from the caller's Q.  The rows get a
        running maximum (0, the reference point the fast stream used, if the row already has weight;
        none yet otherwise), the softmax of the half tile is redone with the general stream (the row
        sums do not contain this half tile yet) and the wave continues in the general loop at `resume`."""
        x = "x" + tagid[-1]
        A.e(f"L_FALL_{tagid}_%=:")
        A.e("s_nop 7")                        # the MFMAs issued last retire before anything below
        A.e("s_nop 7")
        for q in range(NQ):
            A.e(f"v_mov_b32_e32 {vr(T_MAX[q])}, {vr(L_SUM[q])}")
            A.e(f"v_mov_b32_e32 {vr(T_MAX2[q])}, {vr(L_SUM[q])}")
        A.e("s_nop 1")
        for q in range(NQ):
            A.e(f"v_permlane32_swap_b32_e32 {vr(T_MAX[q])}, {vr(T_MAX2[q])}")
        A.e("s_nop 1")
        for q in range(NQ):                   # the row's sum over both lane halves
            A.e(f"v_add_f32_e32 {vr(T_MAX[q])}, {vr(T_MAX[q])}, {vr(T_MAX2[q])}")
        for q in range(NQ):
            A.e(f"v_cmp_eq_f32_e32 vcc, 0, {vr(T_MAX[q])}")
            A.e(f"v_cndmask_b32_e32 {vr(M_RUN[q])}, 0, {vr(NEG_INF)}, vcc")
        recompute_scores(A, *cur)
        recompute_scores(A, *nxt)
        for ins in softmax_stream(A, cur[2], p_cur, False, x):
            A.e(ins)
        A.e(f"s_cmp_lg_u32 {sr(S_FLAG)}, 0")
        A.e(f"s_cbranch_scc1 L_RESO_{x}_%=")
        A.e(f"L_RESO_RET_{x}_%=:")
        A.e(f"s_branch {resume}")


    def store_rows_through_lds(A: Asm):
        """O^T / l, rounded, to memory.  A lane holds, of ITS row, 4 consecutive features per (d block, group
        of 8): stored as they lie, an instruction would write 16-byte pieces of 32 rows, and the memory
        pipeline takes such an instruction piece by piece (4-6 us per pass for the 32 instructions of a
        wave, with the four waves of the work group queueing at it).  So 16 rows at a time go through the
        wave's private LDS region and leave as whole rows: a lane reads 16 bytes, 16 lanes a row, one
        instruction writes 4 rows of 256 contiguous bytes.  Nothing of the ring is touched, so the other
        waves may still be reading it.  Scratch: S^T and P^T registers (dead by now), TMP[8:15]."""
        e, dt = A.e, A.dt
        W_ADDR, R_ADDR, G_OFF, L16, T_ROW, T_ADR = TMP[8], TMP[9], TMP[10], TMP[11], TMP[12], TMP[13]
        OB = (SA, SB)            # rounded output of row block q: 2 registers per (d block, group of 8)
        RB = PA                  # 16 registers: the four 128-bit reads of a round
        e(f"s_mov_b64 {sr(S_EXEC, 2)}, exec")
        e(f"s_mul_i32 {sr(S_TMP)}, %[wv], {OUT_REGION}")
        e(f"s_add_u32 {sr(S_TMP)}, {sr(S_TMP)}, %[lds]")
        e(f"s_add_u32 {sr(S_TMP)}, {sr(S_TMP)}, {LDS_RING}")
        # write address: row c % 16 of the region, 8 hh (+ 64 db + 16 g4 per instruction)
        e(f"v_and_b32_e32 {vr(TMP[0])}, 15, {vr(COL)}")
        e(f"v_mul_u32_u24_e32 {vr(TMP[0])}, {OUT_ROW}, {vr(TMP[0])}")
        e(f"v_lshl_add_u32 {vr(TMP[0])}, {vr(HH)}, 3, {vr(TMP[0])}")
        e(f"v_add_u32_e32 {vr(W_ADDR)}, {sr(S_TMP)}, {vr(TMP[0])}")
        # read address: row L / 16 (+ 4 i per instruction), piece L % 16; the same split addresses memory
        e(f"v_lshrrev_b32_e32 {vr(L16)}, 4, {vr(LANE)}")
        e(f"v_and_b32_e32 {vr(TMP[1])}, 15, {vr(LANE)}")
        e(f"v_mul_u32_u24_e32 {vr(TMP[0])}, {OUT_ROW}, {vr(L16)}")
        e(f"v_lshl_add_u32 {vr(TMP[0])}, {vr(TMP[1])}, 4, {vr(TMP[0])}")
        e(f"v_add_u32_e32 {vr(R_ADDR)}, {sr(S_TMP)}, {vr(TMP[0])}")
        e(f"v_mul_u32_u24_e32 {vr(TMP[0])}, %[qrs], {vr(L16)}")
        e(f"v_lshl_add_u32 {vr(G_OFF)}, {vr(TMP[1])}, 4, {vr(TMP[0])}")
        e(f"v_cmp_gt_u32_e32 vcc, 16, {vr(COL)}")              # lanes of the first 16 rows of a row block
        e(f"s_mov_b64 {sr(S_CMP, 2)}, vcc")
        for q in range(NQ):
            for db in range(4):
                for g4 in range(4):
                    t = TMP[0:4]
                    base = A_O + 64 * q + 16 * db + 4 * g4
                    o = OB[q] + 2 * (4 * db + g4)
                    for k in range(4):
                        e(f"v_accvgpr_read_b32 {vr(t[k])}, {ar(base + k)}")
                    for k in range(4):
                        e(f"v_mul_f32_e32 {vr(t[k])}, {vr(t[k])}, {vr(L_SUM[q])}")
                    if dt == "bf16":
                        e(f"v_cvt_pk_bf16_f32 {vr(o)}, {vr(t[0])}, {vr(t[1])}")
                        e(f"v_cvt_pk_bf16_f32 {vr(o + 1)}, {vr(t[2])}, {vr(t[3])}")
                    else:
                        for k in range(4):
                            e(f"v_cvt_f16_f32_e32 {vr(t[k])}, {vr(t[k])}")
                        e(f"v_pack_b32_f16 {vr(o)}, {vr(t[0])}, {vr(t[1])}")
                        e(f"v_pack_b32_f16 {vr(o + 1)}, {vr(t[2])}, {vr(t[3])}")
            for h in range(2):
                if h == 0:
                    e(f"s_mov_b64 exec, {sr(S_CMP, 2)}")
                else:
                    e(f"s_andn2_b64 exec, {sr(S_EXEC, 2)}, {sr(S_CMP, 2)}")
                for db in range(4):
                    for g4 in range(4):
                        o = OB[q] + 2 * (4 * db + g4)
                        e(f"ds_write_b64 {vr(W_ADDR)}, {vr(o, 2)} offset:{64 * db + 16 * g4}")
                e(f"s_mov_b64 exec, {sr(S_EXEC, 2)}")
                e("s_waitcnt lgkmcnt(0)")
                for i in range(4):
                    e(f"ds_read_b128 {vr(RB + 4 * i, 4)}, {vr(R_ADDR)} offset:{4 * OUT_ROW * i}")
                e("s_waitcnt lgkmcnt(0)")          # also: the region is free for the next round's writes
                for i in range(4):
                    r0 = 32 * q + 16 * h + 4 * i
                    e(f"v_add_u32_e32 {vr(T_ROW)}, {r0}, {vr(L16)}")
                    e(f"s_mul_i32 {sr(S_J0)}, %[qrs], {r0}")
                    e(f"v_cmp_gt_i32_e32 vcc, %[rvs], {vr(T_ROW)}")
                    e(f"v_add_u32_e32 {vr(T_ADR)}, {sr(S_J0)}, {vr(G_OFF)}")
                    e("s_and_b64 exec, exec, vcc")
                    e(f"global_store_dwordx4 {vr(T_ADR)}, {vr(RB + 4 * i, 4)}, %[op]")
                    e(f"s_mov_b64 exec, {sr(S_EXEC, 2)}")


    def body_stage_only(A: Asm):
        rotate_addresses(A, vector=False)
        A.e(f"s_waitcnt vmcnt({2 * CPW + TBL})")
        A.e("s_barrier")
        head, tail = staging_ops("s")
        for gi in sorted(head):
            for ins in head[gi]:
                A.e(ins)
            if gi in tail:
                A.e("s_nop 0")  # M0 must not be written by the instruction right before the load
                for ins in tail[gi]:
                    A.e(ins)


    # ---- hazard check ---------------------------------------------------------------------------------

    _MFMA_V = re.compile(r"^v_mfma\w+ ([va])\[(\d+):(\d+)\]")
    _VREG = re.compile(r"\b([va])(\d+)\b|\b([va])\[(\d+):(\d+)\]")


    def check_mfma_results(lines, need=11):
        """No instruction other than an MFMA may touch a VGPR block within `need` issued instructions
        after the MFMA that writes it (vector reads of matrix results are not interlocked)."""
        recent = []  # (file, lo, hi, age)
        for ln in lines:
            if ln.endswith(":") or ln.startswith("//"):
                continue
            m = _MFMA_V.match(ln)
            if not ln.startswith("v_mfma"):
                regs = set()
                for r in _VREG.finditer(ln):
                    if r.group(1):
                        regs.add((r.group(1), int(r.group(2))))
                    else:
                        regs.update((r.group(3), x) for x in range(int(r.group(4)), int(r.group(5)) + 1))
                for f, lo, hi, age in recent:
                    assert not any(rf == f and lo <= x <= hi for rf, x in regs), (ln, f, lo, hi, age)
            step = int(ln.split()[1]) + 1 if ln.startswith("s_nop") else 1
            recent = [(f, lo, hi, age + step) for f, lo, hi, age in recent if age + step < need]
            if m:
                recent.append((m.group(1), int(m.group(2)), int(m.group(3)), 0))


    # ---- the whole stream ---------------------------------------------------------------------------
    def generate(dt: str) -> list[str]:
        A = Asm(dt)
        e = A.e
        ones = 0x3F803F80 if dt == "bf16" else 0x3C003C00

        A.c("lane constants")
        e(f"s_mov_b32 {sr(S_ONES)}, 0x{ones:08x}")
        e(f"s_xor_b32 {sr(S_NCS)}, %[cs], 0x80000000")
        e(f"s_mov_b32 {sr(S_NK1)}, %[nk1]")
        e(f"v_and_b32_e32 {vr(LANE)}, 63, %[tid]")
        e(f"v_and_b32_e32 {vr(COL)}, 31, {vr(LANE)}")
        e(f"v_lshrrev_b32_e32 {vr(HH)}, 5, {vr(LANE)}")
        # K operand: row c of the key block (chunk c / 4, row c % 4 of it), piece 2 s + hh of k step s
        e(f"v_lshrrev_b32_e32 {vr(TMP[0])}, 2, {vr(COL)}")
        e(f"v_mul_u32_u24_e32 {vr(TMP[0])}, {CHUNK}, {vr(TMP[0])}")
        e(f"v_and_b32_e32 {vr(TMP[1])}, 3, {vr(COL)}")
        # 64 r + 16 hh (+ 256 (s / 2) + 32 (s % 2) per k step)
        e(f"v_lshlrev_b32_e32 {vr(TMP[1])}, 6, {vr(TMP[1])}")
        e(f"v_lshl_add_u32 {vr(TMP[1])}, {vr(HH)}, 4, {vr(TMP[1])}")
        e(f"v_add3_u32 {vr(KL)}, {vr(TMP[0])}, {vr(TMP[1])}, %[lds]")
        # V^T operand through the transposing read: lane (sl = lane % 16, a = (lane / 16) % 2, hh) reads
        # 8 bytes of key row 4 hh + sl / 4 (chunk hh, row sl / 4), d offset 16 a + 4 (sl % 4) of the d
        # block: piece 2 a + (sl % 4) / 2, half sl % 2
        e(f"v_and_b32_e32 {vr(TMP[0])}, 15, {vr(LANE)}")
        e(f"v_bfe_u32 {vr(TMP[1])}, {vr(LANE)}, 4, 1")
        e(f"v_mul_u32_u24_e32 {vr(TMP[2])}, {CHUNK}, {vr(HH)}")
        # byte offset in the chunk: 64 row + 32 a + 16 (piece % 2)
        e(f"v_lshl_add_u32 {vr(TMP[2])}, {vr(TMP[1])}, 5, {vr(TMP[2])}")
        e(f"v_bfe_u32 {vr(TMP[3])}, {vr(TMP[0])}, 1, 1")
        e(f"v_lshl_add_u32 {vr(TMP[2])}, {vr(TMP[3])}, 4, {vr(TMP[2])}")
        e(f"v_lshrrev_b32_e32 {vr(TMP[3])}, 2, {vr(TMP[0])}")
        e(f"v_lshl_add_u32 {vr(TMP[2])}, {vr(TMP[3])}, 6, {vr(TMP[2])}")
        e(f"v_and_b32_e32 {vr(TMP[3])}, 1, {vr(TMP[0])}")
        e(f"v_lshl_add_u32 {vr(TMP[2])}, {vr(TMP[3])}, 3, {vr(TMP[2])}")
        e(f"s_add_u32 {sr(S_TMP)}, %[lds], {T_BYTES}")
        e(f"v_add_u32_e32 {vr(VL)}, {sr(S_TMP)}, {vr(TMP[2])}")
        # staging: wave w fills chunks 4 w .. 4 w + 3 of each tensor
        e(f"s_lshl_b32 {sr(S_TMP)}, %[wv], {2 + CPW.bit_length() - 1}")
        # row (L / 4) % 4, piece 4 (L / 16) + L % 4
        e(f"v_bfe_u32 {vr(TMP[0])}, {vr(LANE)}, 2, 2")
        e(f"v_add_u32_e32 {vr(ROWB)}, {sr(S_TMP)}, {vr(TMP[0])}")
        e(f"v_lshrrev_b32_e32 {vr(TMP[0])}, 4, {vr(LANE)}")
        e(f"v_and_b32_e32 {vr(TMP[1])}, 3, {vr(LANE)}")
        e(f"v_lshl_add_u32 {vr(TMP[0])}, {vr(TMP[0])}, 2, {vr(TMP[1])}")
        e(f"v_lshlrev_b32_e32 {vr(PIECE)}, 4, {vr(TMP[0])}")
        e(f"s_mul_i32 {sr(S_WBASE)}, %[wv], {CPW * CHUNK}")
        e(f"s_add_u32 {sr(S_WBASE)}, {sr(S_WBASE)}, %[lds]")
        if PAGED:
            # rows are addressed inside the wave's block: constants (4 i + L % 4) rows + piece; the
            # block's offset is the scalar part, from the table
            e(f"s_mov_b32 {sr(S_R0W)}, {sr(S_TMP)}")                  # first row of the wave's part of a tile
            e(f"v_bfe_u32 {vr(V_L4)}, {vr(LANE)}, 2, 2")
            for i in range(CPW):
                e(f"v_add_u32_e32 {vr(TMP[0])}, {4 * i}, {vr(V_L4)}")
                e(f"v_mad_u32_u24 {vr(VBO[i])}, {vr(TMP[0])}, %[krb], {vr(PIECE)}")
            # block ids of the last needed key and of the wave's parts of tiles 0, 1, 2: four loads, one wait
            e(f"s_lshr_b32 {sr(S_LASTIDX)}, {sr(S_NK1)}, %[shift]")
            e(f"s_lshl_b32 {sr(S_T2)}, {sr(S_LASTIDX)}, 2")
            e(f"v_mov_b32_e32 {vr(TMP[4])}, {sr(S_T2)}")
            e(f"global_load_dword {vr(TMP[8])}, {vr(TMP[4])}, %[tbl]")
            for x in range(3):
                e(f"s_add_u32 {sr(S_T2)}, {sr(S_R0W)}, {64 * x}")
                e(f"s_lshr_b32 {sr(S_T2)}, {sr(S_T2)}, %[shift]")
                e(f"s_min_u32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_LASTIDX)}")
                e(f"s_lshl_b32 {sr(S_T2)}, {sr(S_T2)}, 2")
                e(f"v_mov_b32_e32 {vr(TMP[5 + x])}, {sr(S_T2)}")
                e(f"global_load_dword {vr(TMP[9 + x])}, {vr(TMP[5 + x])}, %[tbl]")
            e("s_waitcnt vmcnt(0)")
            e(f"v_readfirstlane_b32 {sr(S_BLK)}, {vr(TMP[8])}")
            e(f"s_cmp_lt_u32 {sr(S_BLK)}, %[nblk]")
            e("s_cbranch_scc0 L_BADBLK_last_%=\nL_BADRET_last_%=:")
            e(f"s_and_b32 {sr(S_T2)}, {sr(S_NK1)}, %[bsm1]")
            e(f"s_lshl_b32 {sr(S_TMP)}, {sr(S_BLK)}, %[shift]")
            e(f"s_add_u32 {sr(S_TMP)}, {sr(S_TMP)}, {sr(S_T2)}")       # physical row of the last needed key
            e(f"v_mov_b32_e32 {vr(TMP[0])}, {sr(S_TMP)}")
            e(f"v_mad_u32_u24 {vr(LIMV)}, {vr(TMP[0])}, %[krb], {vr(PIECE)}")
        else:
            for i in range(CPW):
                e(f"v_add_u32_e32 {vr(TMP[0])}, {4 * i}, {vr(ROWB)}")
                e(f"v_mad_u32_u24 {vr(VBO[i])}, {vr(TMP[0])}, %[krb], {vr(PIECE)}")
            e(f"v_mov_b32_e32 {vr(TMP[0])}, {sr(S_NK1)}")
            e(f"v_mad_u32_u24 {vr(LIMV)}, {vr(TMP[0])}, %[krb], {vr(PIECE)}")
        e(f"s_sub_i32 {sr(S_NKM63)}, {sr(S_NK1)}, 63")

        A.c("Q^T into AGPRs: lane (row c, k group hh) holds Q[row][16 s + 8 hh, +8); rows past the last valid one repeat it")
        e(f"s_sub_u32 {sr(S_TMP)}, %[rv], 1")
        e(f"v_lshlrev_b32_e32 {vr(TMP[2])}, 4, {vr(HH)}")
        for q in range(NQ):
            e(f"v_add_u32_e32 {vr(ROW[q])}, {32 * q}, {vr(COL)}")
            e(f"v_min_u32_e32 {vr(TMP[0])}, {sr(S_TMP)}, {vr(ROW[q])}")
            e(f"v_mad_u32_u24 {vr(Q_OFF[q])}, {vr(TMP[0])}, %[qrs], {vr(TMP[2])}")
        for q in range(NQ):
            for s in range(8):
                e(f"global_load_dwordx4 {ar(A_Q + 32 * q + 4 * s, 4)}, {vr(Q_OFF[q])}, %[qp] offset:{32 * s}")
        # output: element r of d block db is d = 32 db + 8 (r / 4) + 4 hh + (r % 4)
        if NQ != 2:     # NQ = 2 stores whole rows through LDS (store_rows_through_lds) and needs no lane offsets
            e(f"v_lshlrev_b32_e32 {vr(TMP[2])}, 3, {vr(HH)}")
            for q in range(NQ):
                e(f"v_mad_u32_u24 {vr(O_OFF[q])}, {vr(ROW[q])}, %[qrs], {vr(TMP[2])}")

        def tile_request(x):
            """Request of tile x (0, 1, 2) as chunks of instructions, one load each (the first with the set-up)."""
            pre = []
            if PAGED:
                if x == 2:   # the id of tile 3 joins the queue before the loads of tile 2, as in the loop
                    pre.append(f"s_add_u32 {sr(S_R0)}, {sr(S_R0W)}, 128")
                    pre += paged_request_id(64)
                pre += [f"v_readfirstlane_b32 {sr(S_BLK)}, {vr(TMP[9 + x])}",
                        f"s_cmp_lt_u32 {sr(S_BLK)}, %[nblk]",
                        f"s_cbranch_scc0 L_BADBLK_p{x}_%=", f"L_BADRET_p{x}_%=:",
                        f"s_add_u32 {sr(S_R0)}, {sr(S_R0W)}, {64 * x}",
                        f"s_and_b32 {sr(S_T2)}, {sr(S_R0)}, %[bsm1]",
                        f"s_lshl_b32 {sr(S_SOFF)}, {sr(S_BLK)}, %[shift]",
                        f"s_add_u32 {sr(S_SOFF)}, {sr(S_SOFF)}, {sr(S_T2)}",
                        f"s_mul_i32 {sr(S_SOFF)}, {sr(S_SOFF)}, %[krb]"]
            else:
                pre.append(f"s_mul_i32 {sr(S_SOFF)}, %[krb], {64 * x}")
            pre += clamped_offsets()
            pre.append(f"s_add_u32 {sr(S_STW)}, {sr(S_WBASE)}, {x * STAGE}")
            chunks = []
            for i in range(CPW):
                for which in ("k", "v"):
                    m0w, ld = tile_load(which, i, S_STW)
                    chunks.append(pre + [m0w, "s_nop 0", ld])
                    pre = []
            return chunks

        A.c("tile 0 requested right behind Q: both are needed first.  Tiles 1 and 2 follow once Q has landed")
        A.c("(a compute unit moves a burst of this size at about 45 bytes per clock: 64 KiB of Q and 96 KiB of")
        A.c("tiles in one go keep every wave at the memory pipeline for 4 us; tiles 1, 2 are not needed before")
        A.c("the second and third tile step)")
        for chunk in tile_request(0):
            for ins in chunk:
                e(ins)

        A.c("state")
        for i in range(64 * NQ):
            e(f"v_accvgpr_write_b32 {ar(A_O + i)}, 0")
        for i in range(8 * NQ):
            e(f"v_mov_b32_e32 {vr(PB + i)}, 0")
        e(f"v_mov_b32_e32 {vr(NEG_INF)}, 0xff800000")
        for q in range(NQ):
            e(f"v_mov_b32_e32 {vr(M_RUN[q])}, 0xff800000")
            e(f"v_mov_b32_e32 {vr(L_SUM[q])}, 0")
            e(f"v_mov_b32_e32 {vr(NEG_MC[q])}, 0")
        e(f"s_mov_b32 {sr(S_FLAG)}, 0")
        e(f"s_mov_b32 {sr(S_T)}, 0")
        A.c("stage offsets before the first rotation: tile -1 in stage 3, tile 0 in stage 0")
        e(f"s_mov_b32 {sr(S_ST_CUR)}, {3 * STAGE}")
        e(f"s_mov_b32 {sr(S_ST_NXT)}, 0")
        A.c("the first half step multiplies zero weights with the V part of stage 3: make it finite")
        full = T_BYTES // (16 * THREADS)          # passes in which every thread writes 16 bytes
        rest = T_BYTES - full * 16 * THREADS      # bytes left for the last, partial pass
        e(f"v_lshlrev_b32_e32 {vr(TMP[0])}, 4, %[tid]")
        e(f"v_min_u32_e32 {vr(TMP[1])}, {rest - 16}, {vr(TMP[0])}")
        e(f"s_add_u32 {sr(S_TMP)}, %[lds], {3 * STAGE + T_BYTES}")
        e(f"v_add_u32_e32 {vr(TMP[0])}, {sr(S_TMP)}, {vr(TMP[0])}")
        e(f"v_add_u32_e32 {vr(TMP[1])}, {sr(S_TMP)}, {vr(TMP[1])}")
        for i in range(full):
            e(f"ds_write_b128 {vr(TMP[0])}, {vr(PB, 4)} offset:{16 * THREADS * i}")
        e(f"ds_write_b128 {vr(TMP[1])}, {vr(PB, 4)} offset:{16 * THREADS * full}")

        late = tile_request(1) + tile_request(2)
        if dt == "bf16":
            A.c("Q has landed once only tile 0's loads are outstanding: a second copy, multiplied by scale x log2(e)")
            A.c("and rounded to bf16 again, for the fast bodies; the requests of tiles 1 and 2 go out between its steps")
            e(f"s_waitcnt vmcnt({2 * CPW})")
            steps = list(range(0, 32 * NQ, 4))
            for it, base in enumerate(steps):
                for k in range(4):
                    e(f"v_accvgpr_read_b32 {vr(TMP[k])}, {ar(A_Q + base + k)}")
                for k in range(4):
                    e(f"v_lshlrev_b32_e32 {vr(TMP[4 + k])}, 16, {vr(TMP[k])}")
                for k in range(4):
                    e(f"v_and_b32_e32 {vr(TMP[k])}, 0xffff0000, {vr(TMP[k])}")
                for k in range(8):
                    e(f"v_mul_f32_e32 {vr(TMP[k])}, %[cs], {vr(TMP[k])}")
                for k in range(4):
                    e(f"v_cvt_pk_bf16_f32 {vr(TMP[k])}, {vr(TMP[4 + k])}, {vr(TMP[k])}")
                for k in range(4):
                    e(f"v_accvgpr_write_b32 {ar(A_QS + base + k)}, {vr(TMP[k])}")
                for chunk in late[it * len(late) // len(steps):(it + 1) * len(late) // len(steps)]:
                    for ins in chunk:
                        e(ins)
        else:
            A.c("tiles 1, 2 requested")
            for chunk in late:
                for ins in chunk:
                    e(ins)
        for i in range(CPW):   # the loop adds a scalar offset to these as long as whole tiles are in range
            e(f"v_mov_b32_e32 {vr(VOFF[i])}, {vr(VBO[i])}")
        A.c("tile 0 has landed once at most the newest loads (tiles 1, 2) are outstanding")
        e(f"s_waitcnt vmcnt({4 * CPW + TBL}) lgkmcnt(0)")
        e("s_barrier")
        e(f"v_mov_b32_e32 {vr(KA_NXT)}, {vr(KL)}")
        e(f"v_add_u32_e32 {vr(VA_CUR)}, {3 * STAGE}, {vr(VL)}")

        A.c("S^T of half tile 0")
        A.reset_lds([])
        half_step(A, -1, qk=(KA_NXT, 0, SA, dt == "bf16"), pv=None, sm=None, nxt=((KA_NXT, 1), (VA_CUR, 1)), extra=[],
                  tagid="pro", cold=True)

        n_pro = len(A.lines)
        fast = dt == "bf16"
        if fast:
            A.c("tiles entirely below the wave's diagonal, bf16: weights without a running maximum.  Not when the")
            A.c("log-sum-exp is asked for (the training forward): it is the scores themselves, and the twice-rounded Q")
            A.c("moves it by up to 4e-3; those calls take the general stream for every tile")
            e("s_cmp_lg_u64 %[lsep], 0")
            e("s_cbranch_scc1 L_FAST_END_%=")
            e("L_FAST_%=:")
            e(f"s_cmp_ge_i32 {sr(S_T)}, %[tms]")
            e("s_cbranch_scc1 L_FAST_END_%=")
            n0 = len(A.lines)
            body(A, False, "f", fast=True)
            check_mfma_results(A.lines[:n0] + A.lines[n0:] * 2)   # after the prologue, and around the loop
            e(f"s_add_u32 {sr(S_T)}, {sr(S_T)}, 1")
            e("s_branch L_FAST_%=")
            e("L_FAST_END_%=:")
            A.c("the scores of the next half tile were formed with the scaled Q: once more from the caller's")
            for _ in range(2):
                e("s_nop 7")
            recompute_scores(A, KA_NXT, 0, SA)
            A.c("rows that went through the fast stream have weight relative to the reference point 0; a wave that")
            A.c("has not run a fast tile goes on in the general loop (which ends at once unless the fast one was skipped)")
            e(f"s_cmp_eq_u32 {sr(S_T)}, 0")
            e("s_cbranch_scc1 L_FULL_%=")
            for q in range(NQ):
                e(f"v_mov_b32_e32 {vr(M_RUN[q])}, 0")
            e("s_branch L_FULL_END_%=")

        A.c("tiles entirely below the wave's diagonal, general stream (fp16; bf16 after leaving the fast stream)")
        e("L_FULL_%=:")
        e(f"s_cmp_ge_i32 {sr(S_T)}, %[tms]")
        e("s_cbranch_scc1 L_FULL_END_%=")
        n0 = len(A.lines)
        body(A, False, "g", entries=fast)
        check_mfma_results(A.lines[:n_pro] + A.lines[n0:] * 2)   # after the prologue, and around the loop
        e(f"s_add_u32 {sr(S_T)}, {sr(S_T)}, 1")
        e("s_branch L_FULL_%=")
        e("L_FULL_END_%=:")

        A.c("tiles that touch the diagonal: lim = row position - first key of the half tile - 4 hh")
        e(f"s_lshl_b32 {sr(S_TMP)}, {sr(S_T)}, 6")
        e(f"s_sub_i32 {sr(S_TMP)}, %[p0], {sr(S_TMP)}")
        e(f"v_lshlrev_b32_e32 {vr(TMP[0])}, 2, {vr(HH)}")
        for q in range(NQ):
            e(f"v_sub_u32_e32 {vr(LIM[q])}, {vr(ROW[q])}, {vr(TMP[0])}")
            e(f"v_add_u32_e32 {vr(LIM[q])}, {sr(S_TMP)}, {vr(LIM[q])}")
        e("L_MASK_%=:")
        e(f"s_cmp_gt_i32 {sr(S_T)}, %[twl]")
        e("s_cbranch_scc1 L_MASK_END_%=")
        n1 = len(A.lines)
        body(A, True, "m")
        check_mfma_results(A.lines[n0:n1] + A.lines[n1:] * 2)  # unmasked -> masked, masked -> masked
        check_mfma_results(A.lines[:n_pro] + A.lines[n1:])     # prologue -> masked
        if fast:
            check_mfma_results(A.lines[n_pro:n0] + A.lines[n1:])   # fast -> masked
        e(f"s_add_u32 {sr(S_T)}, {sr(S_T)}, 1")
        e("s_branch L_MASK_%=")
        e("L_MASK_END_%=:")

        A.c("a wave without rows only helps with the staging")
        e("s_cmp_lt_i32 %[twl], 0")
        e("s_cbranch_scc1 L_STAGE_%=")

        A.c("last O^T += V^T P^T")
        A.reset_lds(pending_reads(0))
        half_step(A, 0, qk=None, pv=(VA_CUR, 1, PB), sm=None, nxt=None, extra=[], tagid="dr")
        for _ in range(3):  # the accumulators are read by the vector ALU next
            e("s_nop 7")
        # Every K/V request of this wave has landed before its first output store is issued: loads and
        # stores may retire out of order, so afterwards only "everything" could be waited for, and the
        # stores' trip to memory would be spent idle.  With the loads out of the way a wave whose work
        # group has no tile left leaves the statement with its stores in flight (nothing reads them,
        # and waits of a later pass only become longer by stores that are older than its loads).
        e("s_waitcnt vmcnt(0)")

        A.c("row sums of both lane halves, normalise, store")
        for q in range(NQ):
            e(f"v_mov_b32_e32 {vr(T_MAX2[q])}, {vr(L_SUM[q])}")
        e("s_nop 1")
        for q in range(NQ):
            e(f"v_permlane32_swap_b32_e32 {vr(L_SUM[q])}, {vr(T_MAX2[q])}")
        e("s_nop 1")
        for q in range(NQ):
            e(f"v_add_f32_e32 {vr(L_SUM[q])}, {vr(L_SUM[q])}, {vr(T_MAX2[q])}")
        A.c("optional log-sum-exp of the scaled scores (natural log): ln 2 (log2 l + cs m), one float per row")
        e("s_cmp_eq_u64 %[lsep], 0")
        e("s_cbranch_scc1 L_NOLSE_%=")
        for q in range(NQ):
            e(f"v_log_f32_e32 {vr(M_NEW[q])}, {vr(L_SUM[q])}")
        e(f"v_cmp_eq_u32_e64 {sr(S_CMP, 2)}, 0, {vr(HH)}")     # both lane halves hold the row: the low one stores
        for q in range(NQ):
            e(f"v_sub_f32_e32 {vr(M_NEW[q])}, {vr(M_NEW[q])}, {vr(NEG_MC[q])}")
        for q in range(NQ):
            e(f"v_mul_f32_e32 {vr(M_NEW[q])}, 0x3f317218, {vr(M_NEW[q])}")
        for q in range(NQ):
            e(f"v_cmp_gt_i32_e32 vcc, %[rvs], {vr(ROW[q])}")
            e(f"s_and_b64 vcc, vcc, {sr(S_CMP, 2)}")
            e(f"s_and_saveexec_b64 {sr(S_EXEC, 2)}, vcc")
            e(f"v_lshlrev_b32_e32 {vr(TMP[0])}, 2, {vr(ROW[q])}")
            e(f"global_store_dword {vr(TMP[0])}, {vr(M_NEW[q])}, %[lsep]")
            e(f"s_mov_b64 exec, {sr(S_EXEC, 2)}")
        e("L_NOLSE_%=:")
        for q in range(NQ):
            e(f"v_rcp_f32_e32 {vr(L_SUM[q])}, {vr(L_SUM[q])}")
        e("s_nop 1")
        if NQ == 2:
            store_rows_through_lds(A)
        for q in range(NQ if NQ != 2 else 0):
            e(f"v_cmp_gt_i32_e32 vcc, %[rvs], {vr(ROW[q])}")
            e(f"s_and_saveexec_b64 {sr(S_EXEC, 2)}, vcc")
            n = 0
            for db in range(4):
                for g4 in range(4):
                    t = TMP[(n % 2) * 8:(n % 2) * 8 + 8]
                    n += 1
                    base = A_O + 64 * q + 16 * db + 4 * g4
                    for k in range(4):
                        e(f"v_accvgpr_read_b32 {vr(t[k])}, {ar(base + k)}")
                    for k in range(4):
                        e(f"v_mul_f32_e32 {vr(t[k])}, {vr(t[k])}, {vr(L_SUM[q])}")
                    if dt == "bf16":
                        e(f"v_cvt_pk_bf16_f32 {vr(t[4])}, {vr(t[0])}, {vr(t[1])}")
                        e(f"v_cvt_pk_bf16_f32 {vr(t[5])}, {vr(t[2])}, {vr(t[3])}")
                    else:
                        for k in range(4):
                            e(f"v_cvt_f16_f32_e32 {vr(t[k])}, {vr(t[k])}")
                        e(f"v_pack_b32_f16 {vr(t[4])}, {vr(t[0])}, {vr(t[1])}")
                        e(f"v_pack_b32_f16 {vr(t[5])}, {vr(t[2])}, {vr(t[3])}")
                    e(f"global_store_dwordx2 {vr(O_OFF[q])}, {vr(t[4], 2)}, %[op] offset:{64 * db + 16 * g4}")
            e(f"s_mov_b64 exec, {sr(S_EXEC, 2)}")

        e("s_waitcnt lgkmcnt(0)")
        e(f"s_cmp_ge_i32 {sr(S_T)}, %[nt]")
        e("s_cbranch_scc1 L_DONE_%=")       # the usual case: the waves of a work group end in the same tile

        A.c("remaining tiles of the work group: staging and barriers only")
        e("L_STAGE_%=:")
        e("s_waitcnt vmcnt(0) lgkmcnt(0)")  # also the output stores: loads and stores may retire out of order
        e("L_STAGE_LOOP_%=:")
        e(f"s_cmp_ge_i32 {sr(S_T)}, %[nt]")
        e("s_cbranch_scc1 L_END_%=")
        body_stage_only(A)
        e(f"s_add_u32 {sr(S_T)}, {sr(S_T)}, 1")
        e("s_branch L_STAGE_LOOP_%=")

        A.c("out-of-line: running maximum moved")
        for name in ("g0", "g1", "m0", "m1") + (("x0", "x1") if fast else ()):
            rescale_blocks(A, name)
        if fast:
            A.c("out-of-line: a row sum of the fast stream left its range")
            fallback_block(A, "f0", (KA_CUR, 0, SA), (KA_CUR, 1, SB), PA, "L_ENTRY_g1_%=")
            fallback_block(A, "f1", (KA_CUR, 1, SB), (KA_NXT, 0, SA), PB, "L_TAIL_g_%=")
            A.e("s_branch L_END_%=")
        if PAGED:
            A.e("s_branch L_END_%=")
            bad_block_paths(A, ["last", "p0", "p1", "p2", "g", "m", "s"] + (["f"] if fast else []))
        e("L_END_%=:")
        e("s_waitcnt vmcnt(0) lgkmcnt(0)")
        e("L_DONE_%=:")
        return A.lines


    def clobbers() -> str:
        n_acc = 128 * NQ
        regs = [f"v{i}" for i in range(FIRST_V, LAST_V + 1)] + [f"a{i}" for i in range(n_acc)]
        regs += [f"s{i}" for i in range(FIRST_S, LAST_S + 1)]
        regs += ["vcc", "scc", "memory"]  # m0 is written too; nothing follows the statement
        return ", ".join(f'"{r}"' for r in regs)


    return types.SimpleNamespace(**locals())


def main(out_path: str, nq: int, paged: bool):
    G = generator(nq, paged)
    with open(out_path, "w") as f:
        f.write("// Generated by gen_prefill_pipe.py -- do not edit.\n")
        tag = f"{nq}P" if paged else f"{nq}"
        f.write(f"#define SKV_PIPE{tag}_LDS_BYTES {G.LDS_BYTES}\n")
        f.write(f"#define SKV_PIPE{tag}_THREADS {G.THREADS}\n")
        for dt in ("bf16", "f16"):
            f.write(f"#define SKV_PIPE{tag}_ASM_{dt.upper()} \\\n")
            for line in G.generate(dt):
                if line.startswith("//"):
                    continue
                f.write(f'    "{line}\\n" \\\n')
            f.write('    ""\n')
        f.write(f"#define SKV_PIPE{tag}_CLOBBERS {G.clobbers()}\n")


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("out")
    ap.add_argument("--nq", type=int, default=2)
    ap.add_argument("--paged", type=int, default=0)
    a = ap.parse_args()
    main(a.out, a.nq, bool(a.paged))
