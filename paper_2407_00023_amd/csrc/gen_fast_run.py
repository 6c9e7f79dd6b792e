#!/usr/bin/env python3
"""Writes fast_run_d128.inc: the tiles of the bf16 extend-attention kernel as gfx950 assembly.

One inline-assembly statement per kernel instance holds every kind of tile, for head dimension 128 and 32 packed query
rows per wave, with every register chosen here.  (Left to the compiler's register allocator the 64 output accumulators
are split around the phases of a tile and copied every tile, and spill reloads inside the loop serialise the
global -> LDS loads behind them; and several statements, each with its fixed registers, made the compiler spill
everything it held around them.)  A mode operand picks the kind: runs of consecutive unmasked tiles that issue the
next tile's loads themselves (its rows in the pool through slot ids, 32-bit or 64-bit addresses, as codes of the fp8
pool, or in the extend tokens), and single tiles, plain or with keys hidden from rows, whose loads the caller issues.

A tile is 32 slots of one MFMA each; what follows an MFMA in the stream runs in its shadow:
    phase A  S0 = K(block 0) Q^T     | addresses + issue of the next tile's global -> LDS loads
    phase B  S1 = K(block 1) Q^T     | probabilities 2^(c S0 - m), their sum; slot ids of the tile after next
    (leave with status 1 if a lane's sum exceeds the limit: block 0 outgrew the running maximum m)
    phase C  O += V(block 0) P0      | probabilities 2^(c S1 - m), their sum
    (leave with status 2)
    phase D  O += V(block 1) P1      | -
    wait for this wave's loads (fp8 pool: turn the rows that landed into bfloat16), workgroup barrier, next tile

Every instruction costs its wave an issue slot of about four cycles whatever unit executes it, so the schedule is
written for few instructions: row sums deferred by one piece, one address for the four slot-id loads where the tile
after next lies wholly in the prefix, M0 written ahead of the address arithmetic that then serves as its wait state,
LDS reads awaited two fragments at a time by counting them (they return in order).  Wait states the hardware does not
interlock are written out, other work standing in them where there is any: the last MFMA of a score block and the
first ALU read of it (eleven slots), a dot-product instruction and any other kind of ALU instruction that reads its
result (three), a transcendental and a use of its result (one), a write of M0 and the load that uses it (one).  The
loop is written out for both ring slots, so that every LDS offset is an immediate and no address register changes
between tiles.

Run:  python gen_fast_run.py  (the build does)."""
import os

KS, NB = 8, 4            # k-slices of QK^T, head-dim blocks of O^T
ROWB, TILEB, STAGEB = 256, 16384, 32768
UPW, RPB = 4, 4          # 1 KB load blocks per wave and tensor, rows per block

NFR = 8                  # fragment buffers (K and V^T fragments share them: the two kinds are read in different phases)
PD = 5                   # LDS fragments in flight ahead of their MFMA
PAIRWAIT, DEFER_SUM, M0_FIRST, FAST_SLOTS, SETTLE = True, True, True, True, False   # (switches for experiments)

# ---- vector registers (everything from v44 up belongs to the assembly) ----
ACC = [192 + 16 * b for b in range(NB)]
Q = [160 + 4 * s for s in range(KS)]
SC0, SC1 = 144, 128
PB0, PB1 = 120, 112
FR = [80 + 4 * i for i in range(NFR)]
KRD = [72 + s for s in range(8)]
VRD = [64 + i for i in range(8)]   # index b * 2 + h2
SLN = [60, 61, 62, 63]
L, NEGM, KOFF0, VOFF0, ROWI, KRD0, VRD0 = 59, 58, 57, 56, 55, 54, 53
T = [46, 47, 48, 49, 50, 51, 52]
LSUM, ROWOFF = 45, 44
LIM0, LIM1, NEGINF = T[0], T[1], T[6]   # masked single tiles (they issue no loads: the T registers are free)
MASKS = [72, 74]                        # ... and two scalar register pairs for their comparisons
FIRST_V = 44
# ---- scalar registers ----
P0, RING, STATUS, PEND = 40, 41, 42, 43
SLOTS, BASE_K, BASE_V = 44, 46, 48     # 64-bit pairs: slot ids; K rows (pool or k_ext); V rows (pool + K->V distance, or v_ext)
C = 52                                  # s[52:59]: see the operand list in emit()
C2 = 60                                 # s[60:63]
S_T = [68, 69, 70, 71]                  # scratch scalars
C_SHIFT, C_MASK, C_PSTRIDE, C_NSLOT1, C_P1, C_XSTRIDE, C_EXTMAX, C_LDSW = range(C, C + 8)
C_128, C_192, C_P, C_SCALE = range(C2, C2 + 4)
# the fp8 pool's runs (kind pool8) take other values in four of the operands, and one operand more:
C_EXPPAGE, C_EXPV = C_XSTRIDE, C_EXTMAX   # bytes from one page's row exponents to the next page's; from a K row's exponent to its V row's
EXP_BASE = C_128                          # s[60:61]: the row exponents of this KV head
EXST = 51                                 # LDS address of this wave's staging area for row exponents
DEC_RAW, DEC_EXP, DEC_OUT = 80, 96, 128   # decode at the end of a tile: codes (16 registers), exponents (8), bfloat16 (32)
LIMIT = "0x53800000"   # 2^40: a lane's probabilities of one key block may sum to this much before the run is left
ONES = "0x3f803f80"    # bf16 (1, 1)


def v(i, n=1):
    return f"v{i}" if n == 1 else f"v[{i}:{i + n - 1}]"


def s(i, n=1):
    return f"s{i}" if n == 1 else f"s[{i}:{i + n - 1}]"


class Stream:
    def __init__(self):
        self.lines = []
        self.lds = []      # ids of LDS reads in flight, oldest first
        self.next_id = 0
        self.tail = []     # code placed behind the loop (rarely taken paths)

    def emit(self, text):
        self.lines.append(text)

    def lds_read(self, text):
        self.emit(text)
        self.lds.append(self.next_id)
        self.next_id += 1
        return self.next_id - 1

    def wait_lds(self, op_id):
        """Wait until LDS read op_id (and every older one) has returned."""
        if op_id not in self.lds:
            return
        after = len(self.lds) - 1 - self.lds.index(op_id)
        self.emit(f"s_waitcnt lgkmcnt({after})")
        self.lds = self.lds[len(self.lds) - after:] if after else []


def tile(st, kind, ring, uid, upw):
    """One tile that sits in ring slot `ring`; the next tile is loaded into the other slot.

    Every instruction costs its wave an issue slot (four cycles, more for a few), whatever unit executes it, and a
    wave runs two of its four phases at that limit: the schedule below is written for few instructions.  LDS
    reads are awaited two fragments at a time; where the hardware wants wait states between two instructions (a write
    of M0 and the load that uses it, a transcendental and the use of its result, the last MFMA of a score block and
    the first ALU read of it - eleven issue slots) other work stands there instead of s_nop."""
    e = st.emit
    ext, wide, raw8 = kind == "ext", kind == "pool64", kind == "pool8"
    noload, masked = kind in ("plain", "masked"), kind == "masked"   # (single tiles: the kernel issues the next tile's loads itself)
    here, there = ring * STAGEB, (ring ^ 1) * STAGEB
    last = {}   # fragment number (0..15 K, 16..31 V) -> id of its last LDS read

    def read_frag(f):
        if f >= 32:
            return
        buf = FR[f % NFR]
        if f < 16:   # K fragment: key block f // 8, k-slice f % 8
            blk, sl = divmod(f, 8)
            off = here + blk * 32 * ROWB
            o = f" offset:{off}" if off else ""
            last[f] = st.lds_read(f"ds_read_b128 {v(buf, 4)}, {v(KRD[sl])}{o}")
        else:        # V^T fragment: key block g // 8, 16-key group (g % 8) // 4, head-dim block g % 4
            g = f - 16
            blk, j = divmod(g, 8)
            cs, b = divmod(j, NB)
            off = here + blk * 32 * ROWB + cs * 16 * ROWB
            o = f" offset:{off}" if off else ""
            st.lds_read(f"ds_read_b64_tr_b16 {v(buf, 2)}, {v(VRD[2 * b])}{o}")
            last[f] = st.lds_read(f"ds_read_b64_tr_b16 {v(buf + 2, 2)}, {v(VRD[2 * b + 1])}{o}")

    def wait_pair(f):
        """Before the MFMA of an even fragment: it and the next one have arrived."""
        if not PAIRWAIT:
            st.wait_lds(last[f])
        elif f % 2 == 0:
            st.wait_lds(last[f + 1])

    def mfma(dst, a, b, c):
        e(f"v_mfma_f32_32x32x16_bf16 {dst}, {a}, {b}, {c}")

    def load_piece(u, which):
        m0 = there + u * 1024 + (TILEB if which else 0)
        # (M0 first: the address arithmetic that follows is the wait state the load needs after it)
        if M0_FIRST:
            e(f"s_add_u32 m0, {s(C_LDSW)}, {m0}" if m0 else f"s_mov_b32 m0, {s(C_LDSW)}")
        if which == 0:
            if ext:
                # position of the row in the extend tokens, clamped to the last valid key; times the token stride
                e(f"s_add_u32 {s(S_T[2])}, {s(P0)}, {64 + RPB * u}")
                e(f"s_sub_u32 {s(S_T[2])}, {s(S_T[2])}, {s(C_P)}")
                e(f"v_add_u32 {v(T[0])}, {s(S_T[2])}, {v(ROWI)}")
                e(f"v_min_i32 {v(T[0])}, {s(C_EXTMAX)}, {v(T[0])}")
                e(f"v_mul_u32_u24 {v(ROWOFF)}, {s(C_XSTRIDE)}, {v(T[0])}")
            elif wide:
                # slot id (never outside the pool) -> page, offset in the page -> number of the K row from the head's
                # first, in rows of 256 bytes, then in units of 16 bytes (the 64-bit shift-and-add shifts by 4 at most;
                # below 2^32 for pools of up to 64 GB).  (T[0], T[1]) = (that number, 0) is its 64-bit operand.
                e(f"v_med3_i32 {v(T[0])}, {v(SLN[u])}, 0, {s(C_NSLOT1)}")
                e(f"v_lshrrev_b32 {v(T[6])}, {s(C_SHIFT)}, {v(T[0])}")
                e(f"v_and_b32 {v(T[0])}, {s(C_MASK)}, {v(T[0])}")
                e(f"v_mad_u32_u24 {v(T[0])}, {v(T[6])}, {s(C_PSTRIDE)}, {v(T[0])}")
                e(f"v_lshlrev_b32 {v(T[0])}, 4, {v(T[0])}")
            else:
                # slot id (never outside the pool) -> page, offset in the page -> byte offset of the K row
                e(f"v_med3_i32 {v(T[0])}, {v(SLN[u])}, 0, {s(C_NSLOT1)}")
                e(f"v_lshrrev_b32 {v(T[1])}, {s(C_SHIFT)}, {v(T[0])}")
                e(f"v_and_b32 {v(T[0])}, {s(C_MASK)}, {v(T[0])}")
                e(f"v_lshlrev_b32 {v(T[0])}, 8, {v(T[0])}")
                e(f"v_mad_u32_u24 {v(ROWOFF)}, {v(T[1])}, {s(C_PSTRIDE)}, {v(T[0])}")
            x = [0, 64, s(C_128), s(C_192)][u]
            if wide:
                # (the bases are 256-byte aligned: adding the offset inside the row never carries)
                e(f"v_lshl_add_u64 {v(T[2], 2)}, {v(T[0], 2)}, 4, {s(BASE_K, 2)}")
                e(f"v_xad_u32 {v(T[2])}, {v(KOFF0)}, {x}, {v(T[2])}")
            else:
                e(f"v_xad_u32 {v(T[2])}, {v(KOFF0)}, {x}, {v(ROWOFF)}")
            addr, base = T[2], BASE_K
        else:
            if wide:
                e(f"v_lshl_add_u64 {v(T[4], 2)}, {v(T[0], 2)}, 4, {s(BASE_V, 2)}")
                e(f"v_xad_u32 {v(T[4])}, {v(VOFF0)}, {16 * u}, {v(T[4])}")
                addr, base = T[4], BASE_V
            else:
                e(f"v_xad_u32 {v(T[3])}, {v(VOFF0)}, {16 * u}, {v(ROWOFF)}")
                addr, base = T[3], BASE_V
        if not M0_FIRST:
            e(f"s_add_u32 m0, {s(C_LDSW)}, {m0}" if m0 else f"s_mov_b32 m0, {s(C_LDSW)}")
            e("s_nop 0")
        if wide:
            e(f"global_load_lds_dwordx4 {v(addr, 2)}, off")
        else:
            e(f"global_load_lds_dwordx4 {v(addr)}, {s(base, 2)}")

    def load_piece8(u, half):
        """fp8 pool: the next tile's rows as codes.  A row's 128 codes go to the first half of the 256 LDS bytes its
        bfloat16 form will take (the lanes that would fetch the second half are switched off), its two exponents (K, V)
        as one byte each to the wave's staging area (one lane per row).  T[6] = 16 (lane % 16)."""
        if half == 0:
            e(f"s_add_u32 m0, {s(C_LDSW)}, {there + u * 1024}")
            e(f"v_med3_i32 {v(T[0])}, {v(SLN[u])}, 0, {s(C_NSLOT1)}")
            e(f"v_lshrrev_b32 {v(T[1])}, {s(C_SHIFT)}, {v(T[0])}")
            e(f"v_and_b32 {v(T[0])}, {s(C_MASK)}, {v(T[0])}")
            e(f"v_mad_u32_u24 {v(T[2])}, {v(T[1])}, {s(C_PSTRIDE)}, {v(T[6])}")
            e(f"v_lshl_add_u32 {v(T[2])}, {v(T[0])}, 7, {v(T[2])}")
            e(f"v_mad_u32_u24 {v(T[3])}, {v(T[1])}, {s(C_EXPPAGE)}, {v(T[0])}")
            e(f"s_mov_b64 exec, {s(MASKS[0], 2)}")
            e(f"global_load_lds_dwordx4 {v(T[2])}, {s(BASE_K, 2)}")
            e(f"s_add_u32 m0, {s(C_LDSW)}, {there + TILEB + u * 1024}")
            e("s_nop 0")
            e(f"global_load_lds_dwordx4 {v(T[2])}, {s(BASE_V, 2)}")
            e("s_mov_b64 exec, -1")
        else:
            e(f"s_add_u32 m0, {s(EXST)}, {2 * u * 256}")
            e(f"v_add_u32 {v(T[2])}, {s(C_EXPV)}, {v(T[3])}")
            e(f"s_mov_b64 exec, {s(MASKS[1], 2)}")
            e(f"global_load_lds_ubyte {v(T[3])}, {s(EXP_BASE, 2)}")
            e(f"s_add_u32 m0, {s(EXST)}, {(2 * u + 1) * 256}")
            e("s_nop 0")
            e(f"global_load_lds_ubyte {v(T[2])}, {s(EXP_BASE, 2)}")
            e("s_mov_b64 exec, -1")

    def decode8():
        """fp8 pool, after this wave's loads have landed: its rows of the next tile from codes to bfloat16, in place.
        All sixteen lanes of a row read their 8 codes before any of them writes, and nobody else touches the row
        before the barrier.  The fragment and score registers are free here."""
        e(f"v_and_b32 {v(T[0])}, 15, {v(ROWI)}")                          # lane / 16
        e(f"v_lshl_add_u32 {v(T[1])}, {v(T[0])}, 8, {s(C_LDSW)}")          # this lane's row in load block 0, ring slot 0
        e(f"v_lshl_add_u32 {v(T[5])}, {v(T[0])}, 6, {s(EXST)}")            # the word that holds the row's exponent
        e(f"v_lshlrev_b32 {v(T[0])}, 4, {v(T[0])}")
        e(f"v_xor_b32 {v(T[6])}, {v(KOFF0)}, {v(T[0])}")                   # 16 (lane % 16)
        e(f"v_add_u32 {v(T[6])}, {v(T[1])}, {v(T[6])}")                    # where this lane's 16 bytes of a load block go
        e(f"v_lshrrev_b32 {v(T[2])}, 1, {v(KOFF0)}")
        e(f"v_lshrrev_b32 {v(T[3])}, 1, {v(VOFF0)}")
        for u in range(upw):
            if 32 * u <= 64:
                e(f"v_xad_u32 {v(T[4])}, {v(T[2])}, {32 * u}, {v(T[1])}")
            else:   # (not an inline constant)
                e(f"v_xor_b32 {v(T[4])}, {32 * u}, {v(T[2])}")
                e(f"v_add_u32 {v(T[4])}, {v(T[1])}, {v(T[4])}")
            st.lds_read(f"ds_read_b64 {v(DEC_RAW + 4 * u, 2)}, {v(T[4])} offset:{there + u * 1024}")
            e(f"v_xad_u32 {v(T[4])}, {v(T[3])}, {8 * u}, {v(T[1])}")
            st.lds_read(f"ds_read_b64 {v(DEC_RAW + 4 * u + 2, 2)}, {v(T[4])} offset:{there + TILEB + u * 1024}")
            st.lds_read(f"ds_read_b32 {v(DEC_EXP + 2 * u)}, {v(T[5])} offset:{2 * u * 256}")
            st.lds_read(f"ds_read_b32 {v(DEC_EXP + 2 * u + 1)}, {v(T[5])} offset:{(2 * u + 1) * 256}")
        for u in range(upw):
            for t in range(2):
                if u == 0 and t == 0:
                    e("s_waitcnt lgkmcnt(0)")
                    st.lds.clear()
                ex, raw, out = DEC_EXP + 2 * u + t, DEC_RAW + 4 * u + 2 * t, DEC_OUT + 4 * (2 * u + t)
                e(f"v_bfe_i32 {v(ex)}, {v(ex)}, 0, 8")
                e(f"v_lshl_add_u32 {v(ex)}, {v(ex)}, 23, 0x3f800000")       # 2^k as a float
                for h in range(2):
                    e(f"v_cvt_scalef32_pk_bf16_fp8 {v(out + 2 * h)}, {v(raw + h)}, {v(ex)}")
                    e(f"v_cvt_scalef32_pk_bf16_fp8 {v(out + 2 * h + 1)}, {v(raw + h)}, {v(ex)} op_sel:[1,0,0]")
                e(f"ds_write_b128 {v(T[6])}, {v(out, 4)} offset:{there + t * TILEB + u * 1024}")
        e("s_waitcnt lgkmcnt(0)")

    pending = []   # probability pair whose row-sum contribution is still to be added: [register]

    def flush_sum():
        if pending:
            e(f"v_dot2c_f32_bf16 {v(LSUM)}, {ONES}, {v(pending.pop())}")

    def exp_piece(sc, pb, idx, lim=None):
        """Probabilities of elements 2 idx, 2 idx + 1 of a score block.  The row-sum step of the piece before stands
        between the exponentials and the first use of their results.  Masked tiles: register i of a lane holds the key
        at offset 8 (i / 4) + i % 4 from the lane's first key of the block, visible if that is below the lane's limit;
        the exponent of a hidden key becomes -inf (two comparisons ahead of the two selections, so that their results
        have reached the scalar registers)."""
        if masked:
            for k, i in enumerate((2 * idx, 2 * idx + 1)):
                e(f"v_cmp_gt_i32 {s(MASKS[k], 2)}, {v(lim)}, {8 * (i // 4) + i % 4}")
        e(f"v_fma_f32 {v(T[4])}, {v(sc + 2 * idx)}, {s(C_SCALE)}, {v(NEGM)}")
        e(f"v_fma_f32 {v(T[5])}, {v(sc + 2 * idx + 1)}, {s(C_SCALE)}, {v(NEGM)}")
        if masked:
            e(f"v_cndmask_b32 {v(T[4])}, {v(NEGINF)}, {v(T[4])}, {s(MASKS[0], 2)}")
            e(f"v_cndmask_b32 {v(T[5])}, {v(NEGINF)}, {v(T[5])}, {s(MASKS[1], 2)}")
        e(f"v_exp_f32 {v(T[4])}, {v(T[4])}")
        e(f"v_exp_f32 {v(T[5])}, {v(T[5])}")
        if pending:
            flush_sum()
        else:
            e("s_nop 0")
        e(f"v_cvt_pk_bf16_f32 {v(pb + idx)}, {v(T[4])}, {v(T[5])}")
        pending.append(pb + idx)
        if not DEFER_SUM:
            flush_sum()

    def end_of_sums(f):
        """The last row-sum step of a key block, and then three instructions before anything but another such step
        reads the sum (the result of a dot-product instruction reaches other ALU instructions three issue slots
        late, and the hardware does not wait for it): the LDS reads this MFMA slot (fragment f) still owes and the
        wait that the next MFMA needs anyway."""
        flush_sum()
        n0 = len(st.lines)
        read_frag(f + PD)
        st.wait_lds(last[f + 2])
        while len(st.lines) - n0 < 3:
            e("s_nop 0")

    def slot_ids():
        """Slot ids of this lane's four rows in the tile after the next one (rows outside the prefix repeat the last
        prefix slot).  Usually that tile lies wholly in the prefix: one address, four loads at fixed distances."""
        e(f"s_add_u32 {s(S_T[3])}, {s(P0)}, 128")
        e(f"s_add_u32 {s(S_T[2])}, {s(P0)}, 191")
        e(f"s_cmp_le_i32 {s(S_T[2])}, {s(C_P1)}")
        e(f"s_cbranch_scc0 Lslow{ring}{uid}" if FAST_SLOTS else f"s_branch Lslow{ring}{uid}")
        e(f"v_add_lshl_u32 {v(T[6])}, {s(S_T[3])}, {v(ROWI)}, 2")
        for u in range(upw):
            o = f" offset:{4 * RPB * u}" if u else ""
            e(f"global_load_dword {v(SLN[u])}, {v(T[6])}, {s(SLOTS, 2)}{o}")
        e(f"Lback{ring}{uid}:")
        t = st.tail
        t.append(f"Lslow{ring}{uid}:")
        for u in range(upw):
            t.append(f"s_add_u32 {s(S_T[2])}, {s(S_T[3])}, {RPB * u}")
            t.append(f"v_add_u32 {v(T[6])}, {s(S_T[2])}, {v(ROWI)}")
            t.append(f"v_min_i32 {v(T[6])}, {s(C_P1)}, {v(T[6])}")
            t.append(f"v_lshlrev_b32 {v(T[6])}, 2, {v(T[6])}")
            t.append(f"global_load_dword {v(SLN[u])}, {v(T[6])}, {s(SLOTS, 2)}")
        t.append(f"s_branch Lback{ring}{uid}")

    for f in range(PD):
        read_frag(f)
    if wide:
        e(f"v_mov_b32 {v(T[1])}, 0")
    if raw8:
        e(f"v_and_b32 {v(T[6])}, 15, {v(ROWI)}")
        e(f"v_lshlrev_b32 {v(T[6])}, 4, {v(T[6])}")
        e(f"v_xor_b32 {v(T[6])}, {v(KOFF0)}, {v(T[6])}")   # 16 (lane % 16): load block 0 swizzles by the row, lane / 16
    # ---- phase A: S0 = K(block 0) Q^T | the next tile's loads ----
    for sl in range(KS):
        wait_pair(sl)
        mfma(v(SC0, 16), v(FR[sl % NFR], 4), v(Q[sl], 4), v(SC0, 16) if sl else "0")
        read_frag(sl + PD)
        if sl < 2 * upw and raw8:
            load_piece8(sl // 2, sl % 2)
        elif sl < 2 * upw and not noload:
            load_piece(sl // 2, sl % 2)
    # ---- phase B: S1 = K(block 1) Q^T | slot ids of the tile after next, probabilities of block 0 ----
    e(f"v_mov_b32 {v(LSUM)}, 0")
    for sl in range(KS):
        f = KS + sl
        wait_pair(f)
        mfma(v(SC1, 16), v(FR[f % NFR], 4), v(Q[sl], 4), v(SC1, 16) if sl else "0")
        if sl < KS - 1:
            read_frag(f + PD)
        if sl == 0 and not ext and not noload:
            slot_ids()   # (also the distance block 0's scores need from the MFMA that wrote them last)
        elif sl == 0:
            if masked:
                e(f"v_subrev_u32 {v(LIM1)}, 32, {v(LIM0)}")
                e(f"v_mov_b32 {v(NEGINF)}, 0xff800000")
            e("s_nop 7")
        if sl == 0 and SETTLE:
            e("s_nop 7")
            e("s_nop 3")
        exp_piece(SC0, PB0, sl, LIM0)
    end_of_sums(2 * KS - 1)
    e(f"v_cmp_lt_u32 vcc, {LIMIT}, {v(LSUM)}")
    e(f"s_cbranch_vccnz Lover1{st.kind_end}")
    e(f"v_add_f32 {v(L)}, {v(L)}, {v(LSUM)}")
    e(f"v_mov_b32 {v(LSUM)}, 0")
    # ---- phase C: O += V(block 0) P0 | probabilities of block 1 (its scores were last written thirteen issue slots ago) ----
    for j in range(8):
        f = 16 + j
        wait_pair(f)
        cs, b = divmod(j, NB)
        mfma(v(ACC[b], 16), v(FR[f % NFR], 4), v(PB0 + 4 * cs, 4), v(ACC[b], 16))
        if j < 7:
            read_frag(f + PD)
        if j == 0 and SETTLE:
            e("s_nop 7")
            e("s_nop 3")
        exp_piece(SC1, PB1, j, LIM1)
    end_of_sums(23)
    e(f"v_cmp_lt_u32 vcc, {LIMIT}, {v(LSUM)}")
    e(f"s_cbranch_vccnz Lover2{st.kind_end}")
    e(f"v_add_f32 {v(L)}, {v(L)}, {v(LSUM)}")
    # ---- phase D: O += V(block 1) P1 ----
    for j in range(8):
        f = 24 + j
        wait_pair(f)
        cs, b = divmod(j, NB)
        mfma(v(ACC[b], 16), v(FR[f % NFR], 4), v(PB1 + 4 * cs, 4), v(ACC[b], 16))
        read_frag(f + PD)
    assert not st.lds, st.lds
    # ---- this wave's part of the next tile has landed, and so has everyone else's ----
    e("s_waitcnt vmcnt(0)")
    if raw8:
        decode8()
    if kind not in st.no_barrier:
        e("s_barrier")
    e(f"s_add_u32 {s(P0)}, {s(P0)}, 64")
    e(f"s_mov_b32 {s(RING)}, {ring ^ 1}")
    e(f"s_cmp_lt_i32 {s(P0)}, {s(PEND)}")


KINDS = ["pool", "ext", "pool64", "plain", "masked", "pool8"]   # mode operand = 1 + index
MODE = 50                                                # scalar register of the mode operand


def gen(upw, kinds=KINDS, no_barrier=()):
    """All kinds of run in one statement (one set of register constraints for the compiler to meet), chosen by the mode
    operand.  Labels of a kind carry its name; Lover1 / Lover2 / Ldone are common.  A tile of a kind in no_barrier ends
    once this wave's loads have landed, and the caller brings the workgroup together (it has work to do on what landed)."""
    st = Stream()
    st.no_barrier = no_barrier
    e = st.emit
    end = "%="
    # ---- entry: LDS read addresses in ring slot 0 (the operands give those of the slot that holds the tile at P0) ----
    e(f"s_lshl_b32 {s(S_T[0])}, {s(RING)}, 15")
    e(f"v_subrev_u32 {v(KRD[0])}, {s(S_T[0])}, {v(KRD0)}")
    e(f"v_subrev_u32 {v(VRD[0])}, {s(S_T[0])}, {v(VRD0)}")
    for k in range(1, 8):
        e(f"v_xor_b32 {v(KRD[k])}, {32 * k}, {v(KRD[0])}")
    for b in range(1, NB):
        e(f"v_xor_b32 {v(VRD[2 * b])}, {64 * b}, {v(VRD[0])}")
    for b in range(NB):
        e(f"v_xor_b32 {v(VRD[2 * b + 1])}, 32, {v(VRD[2 * b])}")
        e(f"v_add_u32 {v(VRD[2 * b + 1])}, 0x800, {v(VRD[2 * b + 1])}")
    e(f"s_mov_b32 {s(STATUS)}, 0")
    for kind in kinds[1:]:
        e(f"s_cmp_eq_u32 {s(MODE)}, {KINDS.index(kind) + 1}")
        e(f"s_cbranch_scc1 Lkind_{kind}{end}")
    for kind in kinds:
        uid = f"_{kind}{end}"
        e(f"Lkind{uid}:")
        if kind == "pool8":
            # lanes that fetch the codes of a row (the first eight of every sixteen); the lane that fetches its exponents
            e(f"s_mov_b32 {s(MASKS[0])}, 0x00ff00ff")
            e(f"s_mov_b32 {s(MASKS[0] + 1)}, 0x00ff00ff")
            e(f"s_mov_b32 {s(MASKS[1])}, 0x00010001")
            e(f"s_mov_b32 {s(MASKS[1] + 1)}, 0x00010001")
        e(f"s_cmp_eq_u32 {s(RING)}, 0")
        e(f"s_cbranch_scc0 Lring1{uid}")
        # the loop body is written out for both ring slots: every LDS offset is an immediate
        e(f"Lring0{uid}:")
        st.kind_end = end
        tile(st, kind, 0, uid, upw)
        e(f"s_cbranch_scc0 Ldone{end}")
        e(f"Lring1{uid}:")
        tile(st, kind, 1, uid, upw)
        e(f"s_cbranch_scc1 Lring0{uid}")
        e(f"s_branch Ldone{end}")
    for ln in st.tail:
        e(ln)
    e(f"Lover1{end}:")
    e(f"s_mov_b32 {s(STATUS)}, 1")
    e(f"s_branch Ldone{end}")
    e(f"Lover2{end}:")
    e(f"s_mov_b32 {s(STATUS)}, 2")               # the sum of block 0 is in L already
    e(f"Ldone{end}:")
    e("s_waitcnt vmcnt(0) lgkmcnt(0)")           # prefetched fragments and slot ids of a run that was left early
    return st.lines


def emit(name, upw, kinds=KINDS[:5], no_barrier=()):
    lines = gen(upw, kinds, no_barrier)
    kv8 = "pool8" in kinds
    body = "\n".join(f'        "{ln}\\n\\t"' for ln in lines)
    clob = ([f"v{i}" for i in range(FIRST_V, 53) if i != LIM0] + [f"v{i}" for i in range(64, 160)] + [f"s{i}" for i in S_T] +
            [f"s{i}" for i in range(MASKS[0], MASKS[1] + 2)] + ["vcc", "scc", "memory"] + (["exec"] if kv8 else []))
    clobbers = ", ".join(f'"{c}"' for c in clob)
    sln = ", ".join(f'"+{{v{SLN[u]}}}"(sl_next[{u}])' for u in range(upw))
    return f'''
// a wave loads {upw} blocks of a tile
__device__ __forceinline__ void {name}(int mode, f32x16& acc0, f32x16& acc1, f32x16& acc2, f32x16& acc3, const bf16x32& q_lo,
                                       const bf16x32& q_hi, float& l_run, float neg_m, int32_t (&sl_next)[{upw}],
                                       unsigned k_rd0, unsigned v_rd0, unsigned ld_koff0, unsigned ld_voff0, int row_in_tile,
                                       int& p0, int& ring, int& status, int p_end, const void* slots, const void* base_k,
                                       const void* base_v, int lim, const i32x8& c, const i32x4& c2{", unsigned exp_stage" if kv8 else ""}) {{
    asm volatile(
{body}
        : "+{{v[192:207]}}"(acc0), "+{{v[208:223]}}"(acc1), "+{{v[224:239]}}"(acc2), "+{{v[240:255]}}"(acc3), "+{{v59}}"(l_run),
          {sln}, "+{{s40}}"(p0),
          "+{{s41}}"(ring), "={{s42}}"(status), "+{{v{LIM0}}}"(lim)
        : "{{v[160:175]}}"(q_lo), "{{v[176:191]}}"(q_hi), "{{v58}}"(neg_m), "{{v54}}"(k_rd0), "{{v53}}"(v_rd0), "{{v57}}"(ld_koff0),
          "{{v56}}"(ld_voff0), "{{v55}}"(row_in_tile), "{{s43}}"(p_end), "{{s[44:45]}}"(slots), "{{s[46:47]}}"(base_k),
          "{{s[48:49]}}"(base_v), "{{s[52:59]}}"(c), "{{s[60:63]}}"(c2), "{{s{MODE}}}"(mode){f', "{{s{EXST}}}"(exp_stage)' if kv8 else ""}
        : {clobbers});
}}
'''


HEADER = '''// GENERATED by gen_fast_run.py - do not edit.  Tiles of extend_bf16_kernel<128, 4, 1> (a wave loads four 1 KB blocks of
// a K or V tile) and extend_bf16_kernel<128, 8, 1> (_w8: two blocks) as gfx950 assembly with fixed registers; the
// generator describes the schedule.  One statement per kernel holds every kind of tile, so that the compiler meets one
// set of register constraints; the mode operand chooses:
//   1  a run of tiles, the NEXT tile of each wholly in the prefix (its rows come from the pool through slot ids)
//   2  a run of tiles, the next tile wholly in the extend tokens
//   3  as 1 for pools of 4 GB and more (pool rows addressed in 64 bits; base_k / base_v 256-byte aligned)
//   4  one tile, arithmetic only (the caller has issued the next tile's loads)
//   5  as 4 with keys hidden from rows: lim = how many keys of the tile, counted from the lane's first, its row sees
// (_kv8, for the fp8 pool: modes 2, 4, 5 and
//   6  a run of tiles, the next tile of each wholly in the prefix: its rows arrive as codes and row exponents and are
//      turned into bfloat16 in LDS once they have landed; base_k / base_v then point at the codes, c[2] is the page
//      stride of the codes in bytes, c[5] the page stride of the row exponents, c[6] the distance from a K row's
//      exponent to its V row's, c2[0..1] the address of the KV head's row exponents, exp_stage the LDS address of the
//      wave's staging area for them;
// a single tile (4, 5) ends without the workgroup barrier - the caller decodes the pool rows that have landed first.)
//
// Operands: acc0..3 output accumulators (head-dim blocks 0..3); q_lo / q_hi the eight query fragments (k-slices 0..3,
// 4..7); l_run this lane's share of the row sum; neg_m minus the running maximum; sl_next the pool
// slots of the rows this lane loads for the next tile (updated to those of the tile after the last one done);
// k_rd0 / v_rd0 LDS read addresses (k-slice 0; head-dim block 0, first half) in the ring slot of the tile at p0;
// ld_koff0 / ld_voff0 byte offsets inside a K / V row of this lane's 16 bytes of load block 0; row_in_tile the row of
// the tile this lane loads in block 0; p0 first key of the tile (advanced by 64 per tile done); ring its ring slot;
// status 0 = ran to p_end, 1 / 2 = the tile at p0 outgrew the running maximum in key block 0 / 1 (see the kernel);
// slots the request's slot ids; base_k / base_v where K / V rows are fetched from; lim see mode 5 (scratch otherwise);
// c = {page shift, page mask, page stride in bytes (mode 3: in rows of 256 bytes), num_slots - 1, P - 1, extend token
// stride in bytes, kv_hi - 1 - P, LDS address of this wave's load block 0 in ring slot 0}; c2 = {128, 192, P, bits of
// scale * log2(e)}.
'''


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    text = (HEADER + emit("fast_tiles_d128", 4) + emit("fast_tiles_d128_w8", 2) +
            emit("fast_tiles_d128_kv8", 4, ["pool8", "ext", "plain", "masked"], no_barrier=("plain", "masked")))
    path = os.path.join(here, "fast_run_d128.inc")
    old = open(path).read() if os.path.exists(path) else None
    if old != text:
        open(path, "w").write(text)
    return path


if __name__ == "__main__":
    print(main())
