#!/usr/bin/env python3
"""Writes fast_run_d128.inc: the runs of steady-state tiles of the bf16 extend-attention kernel as gfx950 assembly.

One inline-assembly statement holds the whole loop over a run of tiles that need no mask, for head dimension 128,
32 packed query rows per wave, with every register chosen here.  (Left to the compiler's register allocator the 64
output accumulators are split around the phases of a tile and copied every tile, and spill reloads inside the loop
serialise the global -> LDS loads behind them.)  Two variants: the NEXT tile lies wholly in the prefix (its rows come
from the pool through slot ids) or wholly in the extend tokens.

A tile is 32 slots of one MFMA each; what follows an MFMA in the stream runs in its shadow:
    phase A  S0 = K(block 0) Q^T     | addresses + issue of the next tile's global -> LDS loads (8 pieces)
    phase B  S1 = K(block 1) Q^T     | probabilities 2^(c S0 - m), their sum; slot ids of the tile after next
    (leave with status 1 if a lane's sum exceeds the limit: block 0 outgrew the running maximum m)
    phase C  O += V(block 0) P0      | probabilities 2^(c S1 - m), their sum
    (leave with status 2)
    phase D  O += V(block 1) P1      | LDS read addresses move to the other ring slot
    wait for this wave's loads, workgroup barrier, next tile

Wait states the hardware does not interlock are written out: an s_nop block between the last MFMA that writes a score
block and the first ALU read of it, one instruction between a transcendental and a use of its result, one s_nop after
a write of M0.  LDS reads are awaited by counting them (they return in order).

Run:  python gen_fast_run.py  (the build does)."""
import os

KS, NB = 8, 4            # k-slices of QK^T, head-dim blocks of O^T
ROWB, TILEB, STAGEB = 256, 16384, 32768
UPW, RPB = 4, 4          # 1 KB load blocks per wave and tensor, rows per block

# ---- vector registers (everything from v52 up belongs to the assembly) ----
ACC = [192 + 16 * b for b in range(NB)]
Q = [160 + 4 * s for s in range(KS)]
SC0, SC1 = 144, 128
PB0, PB1 = 120, 112
KF = [100, 104, 108]
VF = [88, 92, 96]
KRD = [80 + s for s in range(8)]
VRD = [72 + i for i in range(8)]   # index b * 2 + h2
SLN = [68, 69, 70, 71]
L, NEGM, KOFF0, VOFF0, ROWI, KRD0, VRD0 = 67, 66, 65, 64, 63, 62, 61
T = [54, 55, 56, 57, 58, 59, 60]
LSUM, ROWOFF = 53, 52
# ---- scalar registers ----
P0, RING, STATUS, PEND = 40, 41, 42, 43
SLOTS, BASE_K, BASE_V = 44, 46, 48     # 64-bit pairs: slot ids; K rows (pool or k_ext); V rows (pool + K->V distance, or v_ext)
C = 52                                  # s[52:59]: see the operand list in emit()
C2 = 60                                 # s[60:63]
S_T = [68, 69, 70, 71, 72, 73]          # scratch scalars
C_SHIFT, C_MASK, C_PSTRIDE, C_NSLOT1, C_P1, C_XSTRIDE, C_EXTMAX, C_LDSW = range(C, C + 8)
C_128, C_192, C_P, C_SCALE = range(C2, C2 + 4)
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


def gen(ext):
    st = Stream()
    e = st.emit
    uid = "%="
    # ---- entry: LDS read addresses of the ring slot that holds the tile at P0 ----
    for k in range(8):
        e(f"v_xor_b32 {v(KRD[k])}, {32 * k}, {v(KRD0)}" if k else f"v_mov_b32 {v(KRD[0])}, {v(KRD0)}")
    for b in range(NB):
        e(f"v_xor_b32 {v(VRD[2 * b])}, {64 * b}, {v(VRD0)}" if b else f"v_mov_b32 {v(VRD[0])}, {v(VRD0)}")
    for b in range(NB):
        e(f"v_xor_b32 {v(VRD[2 * b + 1])}, 32, {v(VRD[2 * b])}")
        e(f"v_add_u32 {v(VRD[2 * b + 1])}, 0x800, {v(VRD[2 * b + 1])}")
    e(f"s_mov_b32 {s(STATUS)}, 0")
    e(f"Ltile{uid}:")
    # per-tile scalars: LDS base of this wave's pieces in the OTHER ring slot; step of the read addresses to it
    e(f"s_xor_b32 {s(S_T[0])}, {s(RING)}, 1")
    e(f"s_lshl_b32 {s(S_T[0])}, {s(S_T[0])}, 15")                 # (ring ^ 1) * STAGEB
    e(f"s_add_u32 {s(S_T[0])}, {s(S_T[0])}, {s(C_LDSW)}")          # + smem + wave * UPW * 1024
    e(f"s_lshl_b32 {s(S_T[1])}, {s(RING)}, 16")
    e(f"s_sub_u32 {s(S_T[1])}, 0x8000, {s(S_T[1])}")               # + STAGEB from slot 0, - STAGEB from slot 1

    kfrag, vfrag = {}, {}   # fragment number -> id of its (last) LDS read

    def read_k(g):  # K fragment g: key block g // 8, k-slice g % 8
        blk, sl = divmod(g, 8)
        off = f" offset:{blk * 32 * ROWB}" if blk else ""
        kfrag[g] = st.lds_read(f"ds_read_b128 {v(KF[g % 3], 4)}, {v(KRD[sl])}{off}")

    def read_v(g):  # V^T fragment g: key block g // 8, 16-key group (g % 8) // 4, head-dim block g % 4
        blk, j = divmod(g, 8)
        cs, b = divmod(j, NB)
        off = blk * 32 * ROWB + cs * 16 * ROWB
        o = f" offset:{off}" if off else ""
        st.lds_read(f"ds_read_b64_tr_b16 {v(VF[g % 3], 2)}, {v(VRD[2 * b])}{o}")
        vfrag[g] = st.lds_read(f"ds_read_b64_tr_b16 {v(VF[g % 3] + 2, 2)}, {v(VRD[2 * b + 1])}{o}")

    def load_piece(u, which):
        m0 = u * 1024 + (TILEB if which else 0)
        if which == 0:
            if ext:
                # position of the row in the extend tokens, clamped to the last valid key; times the token stride
                e(f"s_add_u32 {s(S_T[2])}, {s(P0)}, {64 + RPB * u}")
                e(f"s_sub_u32 {s(S_T[2])}, {s(S_T[2])}, {s(C_P)}")
                e(f"v_add_u32 {v(T[0])}, {s(S_T[2])}, {v(ROWI)}")
                e(f"v_min_i32 {v(T[0])}, {s(C_EXTMAX)}, {v(T[0])}")
                e(f"v_mul_u32_u24 {v(ROWOFF)}, {s(C_XSTRIDE)}, {v(T[0])}")
            else:
                # slot id (never outside the pool) -> page, offset in the page -> byte offset of the K row
                e(f"v_med3_i32 {v(T[0])}, {v(SLN[u])}, 0, {s(C_NSLOT1)}")
                e(f"v_lshrrev_b32 {v(T[1])}, {s(C_SHIFT)}, {v(T[0])}")
                e(f"v_and_b32 {v(T[0])}, {s(C_MASK)}, {v(T[0])}")
                e(f"v_lshlrev_b32 {v(T[0])}, 8, {v(T[0])}")
                e(f"v_mad_u32_u24 {v(ROWOFF)}, {v(T[1])}, {s(C_PSTRIDE)}, {v(T[0])}")
            x = [0, 64, s(C_128), s(C_192)][u]
            e(f"v_xad_u32 {v(T[2])}, {v(KOFF0)}, {x}, {v(ROWOFF)}")
            addr, base = T[2], BASE_K
        else:
            e(f"v_xad_u32 {v(T[3])}, {v(VOFF0)}, {16 * u}, {v(ROWOFF)}")
            addr, base = T[3], BASE_V
        e(f"s_add_u32 m0, {s(S_T[0])}, {m0}" if m0 else f"s_mov_b32 m0, {s(S_T[0])}")
        e("s_nop 0")
        e(f"global_load_lds_dwordx4 {v(addr)}, {s(base, 2)}")

    def exp_piece(sc, pb, idx, gap):
        """Probabilities of elements 2 idx, 2 idx + 1 of a score block; gap() emits what separates the
        exponentials from the first use of their results."""
        e(f"v_fma_f32 {v(T[4])}, {v(sc + 2 * idx)}, {s(C_SCALE)}, {v(NEGM)}")
        e(f"v_fma_f32 {v(T[5])}, {v(sc + 2 * idx + 1)}, {s(C_SCALE)}, {v(NEGM)}")
        e(f"v_exp_f32 {v(T[4])}, {v(T[4])}")
        e(f"v_exp_f32 {v(T[5])}, {v(T[5])}")
        if not gap():
            e("s_nop 0")
        e(f"v_cvt_pk_bf16_f32 {v(pb + idx)}, {v(T[4])}, {v(T[5])}")
        e(f"v_dot2c_f32_bf16 {v(LSUM)}, {ONES}, {v(pb + idx)}")

    def settle():
        e("s_nop 7")
        e("s_nop 3")

    # ---- phase A ----
    read_k(0)
    read_k(1)
    for sl in range(KS):
        st.wait_lds(kfrag[sl])
        c = v(SC0, 16) if sl else "0"
        e(f"v_mfma_f32_32x32x16_bf16 {v(SC0, 16)}, {v(KF[sl % 3], 4)}, {v(Q[sl], 4)}, {c}")
        read_k(sl + 2)
        load_piece(sl // 2, sl % 2)
    # ---- phase B ----
    e(f"v_mov_b32 {v(LSUM)}, 0")
    for sl in range(KS):
        g = KS + sl
        st.wait_lds(kfrag[g])
        c = v(SC1, 16) if sl else "0"
        e(f"v_mfma_f32_32x32x16_bf16 {v(SC1, 16)}, {v(KF[g % 3], 4)}, {v(Q[sl], 4)}, {c}")
        if not ext and sl < UPW:
            # slot id of this lane's row in the tile after the next one (rows outside the prefix repeat the last prefix slot)
            e(f"s_add_u32 {s(S_T[3])}, {s(P0)}, {128 + RPB * sl}")
            e(f"v_add_u32 {v(T[6])}, {s(S_T[3])}, {v(ROWI)}")
            e(f"v_min_i32 {v(T[6])}, {s(C_P1)}, {v(T[6])}")
            e(f"v_lshlrev_b32 {v(T[6])}, 2, {v(T[6])}")
            e(f"global_load_dword {v(SLN[sl])}, {v(T[6])}, {s(SLOTS, 2)}")
        if sl == 0:
            settle()   # S0 was last written by the MFMA before this slot's

        def gap(sl=sl):
            if sl + 2 < KS:
                read_k(KS + sl + 2)
            else:
                read_v(sl + 2 - KS)
            return True
        exp_piece(SC0, PB0, sl, gap)
    e(f"v_cmp_lt_u32 vcc, {LIMIT}, {v(LSUM)}")
    e(f"s_cbranch_vccnz Lover1{uid}")
    e(f"v_add_f32 {v(L)}, {v(L)}, {v(LSUM)}")
    e(f"v_mov_b32 {v(LSUM)}, 0")
    # ---- phase C ----
    for j in range(8):
        st.wait_lds(vfrag[j])
        cs, b = divmod(j, NB)
        e(f"v_mfma_f32_32x32x16_bf16 {v(ACC[b], 16)}, {v(VF[j % 3], 4)}, {v(PB0 + 4 * cs, 4)}, {v(ACC[b], 16)}")
        if j == 0:
            settle()   # S1 was last written by the MFMA before this slot's

        def gap(j=j):
            read_v(j + 2)
            return True
        exp_piece(SC1, PB1, j, gap)
    e(f"v_cmp_lt_u32 vcc, {LIMIT}, {v(LSUM)}")
    e(f"s_cbranch_vccnz Lover2{uid}")
    e(f"v_add_f32 {v(L)}, {v(L)}, {v(LSUM)}")
    # ---- phase D ----
    for j in range(8):
        g = 8 + j
        st.wait_lds(vfrag[g])
        cs, b = divmod(j, NB)
        e(f"v_mfma_f32_32x32x16_bf16 {v(ACC[b], 16)}, {v(VF[g % 3], 4)}, {v(PB1 + 4 * cs, 4)}, {v(ACC[b], 16)}")
        if g + 2 < 16:
            read_v(g + 2)
        if j < 4:   # K read addresses are done with this tile
            e(f"v_add_u32 {v(KRD[2 * j])}, {s(S_T[1])}, {v(KRD[2 * j])}")
            e(f"v_add_u32 {v(KRD[2 * j + 1])}, {s(S_T[1])}, {v(KRD[2 * j + 1])}")
        if j >= 6:  # the last V read was issued in slot 5
            for i in range(4 * (j - 6), 4 * (j - 6) + 4):
                e(f"v_add_u32 {v(VRD[i])}, {s(S_T[1])}, {v(VRD[i])}")
    assert not st.lds, st.lds
    # ---- this wave's part of the next tile has landed, and so has everyone else's ----
    e("s_waitcnt vmcnt(0)")
    e("s_barrier")
    e(f"s_add_u32 {s(P0)}, {s(P0)}, 64")
    e(f"s_xor_b32 {s(RING)}, {s(RING)}, 1")
    e(f"s_cmp_lt_i32 {s(P0)}, {s(PEND)}")
    e(f"s_cbranch_scc1 Ltile{uid}")
    e(f"s_branch Ldone{uid}")
    e(f"Lover1{uid}:")
    e(f"s_mov_b32 {s(STATUS)}, 1")
    e(f"s_branch Ldone{uid}")
    e(f"Lover2{uid}:")
    e(f"s_mov_b32 {s(STATUS)}, 2")               # the sum of block 0 is in L already
    e(f"Ldone{uid}:")
    e("s_waitcnt vmcnt(0) lgkmcnt(0)")           # prefetched fragments and slot ids of a run that was left early
    return st.lines


def emit(name, ext):
    lines = gen(ext)
    body = "\n".join(f'        "{ln}\\n\\t"' for ln in lines)
    clob = [f"v{i}" for i in range(52, 61)] + [f"v{i}" for i in range(72, 160)] + [f"s{i}" for i in S_T] + ["vcc", "scc", "memory"]
    clobbers = ", ".join(f'"{c}"' for c in clob)
    return f'''
// {'next tile in the extend tokens' if ext else 'next tile in the prefix (pool rows through slot ids)'}
__device__ __forceinline__ void {name}(f32x16& acc0, f32x16& acc1, f32x16& acc2, f32x16& acc3, const bf16x32& q_lo,
                                       const bf16x32& q_hi, float& l_run, float neg_m, int32_t (&sl_next)[4],
                                       unsigned k_rd0, unsigned v_rd0, unsigned ld_koff0, unsigned ld_voff0, int row_in_tile,
                                       int& p0, int& ring, int& status, int p_end, const void* slots, const void* base_k,
                                       const void* base_v, const i32x8& c, const i32x4& c2) {{
    asm volatile(
{body}
        : "+{{v[192:207]}}"(acc0), "+{{v[208:223]}}"(acc1), "+{{v[224:239]}}"(acc2), "+{{v[240:255]}}"(acc3), "+{{v67}}"(l_run),
          "+{{v68}}"(sl_next[0]), "+{{v69}}"(sl_next[1]), "+{{v70}}"(sl_next[2]), "+{{v71}}"(sl_next[3]), "+{{s40}}"(p0),
          "+{{s41}}"(ring), "={{s42}}"(status)
        : "{{v[160:175]}}"(q_lo), "{{v[176:191]}}"(q_hi), "{{v66}}"(neg_m), "{{v62}}"(k_rd0), "{{v61}}"(v_rd0), "{{v65}}"(ld_koff0),
          "{{v64}}"(ld_voff0), "{{v63}}"(row_in_tile), "{{s43}}"(p_end), "{{s[44:45]}}"(slots), "{{s[46:47]}}"(base_k),
          "{{s[48:49]}}"(base_v), "{{s[52:59]}}"(c), "{{s[60:63]}}"(c2)
        : {clobbers});
}}
'''


HEADER = '''// GENERATED by gen_fast_run.py - do not edit.  Runs of steady-state tiles of extend_bf16_kernel<128, 4, 1> as
// gfx950 assembly with fixed registers; the generator describes the schedule.
//
// Operands: acc0..3 output accumulators (head-dim blocks 0..3); q_lo / q_hi the eight query fragments (k-slices 0..3,
// 4..7); l_run this lane's share of the row sum; neg_m minus the running maximum; sl_next the pool
// slots of the rows this lane loads for the next tile (updated to those of the tile after the last one done);
// k_rd0 / v_rd0 LDS read addresses (k-slice 0; head-dim block 0, first half) in the ring slot of the tile at p0;
// ld_koff0 / ld_voff0 byte offsets inside a K / V row of this lane's 16 bytes of load block 0; row_in_tile the row of
// the tile this lane loads in block 0; p0 first key of the tile (advanced by 64 per tile done); ring its ring slot;
// status 0 = ran to p_end, 1 / 2 = the tile at p0 outgrew the running maximum in key block 0 / 1 (see the kernel);
// slots the request's slot ids; base_k / base_v where K / V rows are fetched from; c = {page shift, page mask, page
// stride in bytes, num_slots - 1, P - 1, extend token stride in bytes, kv_hi - 1 - P, LDS address of this wave's load
// block 0 in ring slot 0}; c2 = {128, 192, P, bits of scale * log2(e)}.
'''


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    text = HEADER + emit("fast_run_pool_d128", False) + emit("fast_run_ext_d128", True)
    path = os.path.join(here, "fast_run_d128.inc")
    old = open(path).read() if os.path.exists(path) else None
    if old != text:
        open(path, "w").write(text)
    return path


if __name__ == "__main__":
    print(main())
