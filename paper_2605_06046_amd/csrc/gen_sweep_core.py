#!/usr/bin/env python3
"""Writes fea_sweep_core.inc: the hand-scheduled gfx950 instruction sequences with which the
waves of one workgroup sweep a piece of a shared run together.
Run it after changing the schedule:  python3 gen_sweep_core.py > fea_sweep_core.inc

A piece of a shared run (one KV head x a range of whole 32-token tiles) is swept for several row
tiles of up to 64 query rows (requests x group heads).  The row tiles read the same KV bytes, so
the planner puts them on neighbouring waves of one workgroup - a team of 2 or of 4 - and the
team fetches every tile once: each wave requests its part of the tile (global -> LDS), the
tiles sit in a ring all team members read, and one workgroup barrier per tile says both "every
part of the next tile has landed" and "everybody is done with the slot about to be refilled".
What a wave computes for its own row tile is what sweep_item computes - per query row the
triple (m, l, acc[128]) of an online softmax over the piece, the reference exponent m raised
(and O^T, l rescaled) only when a score exceeds it by more than 2^24.

Why by hand: a wave has no second wave on its SIMD, so the matrix core only stays busy if the
products of tile t+1 are in flight while the vector unit turns tile t's scores into weights,
and the 144 accumulation registers must stay put for the whole sweep.  The compiler does
neither for this loop (it moves or spills the accumulators), so the registers are assigned
here and the instruction streams - matrix core, vector unit, scalar unit with the memory
requests - are interleaved in program order.

Team of T waves (T = 2, 4), ring of D = 2 T tiles: K ring (D slots of two 4 KB blocks), then V
ring.  Rank r requests, per tile, T = 4: one block (K b0, K b1, V b0, V b1 for r = 0..3, 4
loads); T = 2: both blocks of K (r = 0) or of V (r = 1), 8 loads.  Tiles 0 .. D-1 are requested
up front.  Iteration t: first phase (S of tile t+1, weights of tile t, V transposes) on fragments
read from LDS during the iteration before; then, tile t being read out, the barrier, tile t+D
requested into its slot and the LDS reads of iteration t+1 requested (K of tile t+2, V of tile
t+1), whose latency the second phase (O^T += V^T P^T) covers.  A wave's own requests complete
in order, so "my part of tile t+2 has landed" is vmcnt(loads x min(D-3, n-3-t)).

Register map (fixed, listed as clobbers so that the compiler keeps its own values elsewhere):
  a[0:127]    O^T accumulators   O(nt, i) = a[(8 nt + i) 4 ..]      nt: row tile of 16, i: dim 8 n + i
  a[128:143]  row sums           L(nt)
  a[144:175]  S^T buffer A, a[176:207] S^T buffer B    S(nt, mt): tokens 16 mt + 4 kg + jj, row 16 nt + n
  v[32:35] / v[36:39] LDS addresses of this iteration's K / V fragments
  v[40:103]   Q^T fragments      Q(nt, ks)
  v[104:135]  K fragments of the next tile   KA(mt, ks)
  v[136:167]  V rows of this tile            VR(j)
  v[168:199]  V transposed                   VA(i)
  v[200:207]  weights (two sets)             P(set)
  v[208:223]  temporaries, v[224:227] ones, v[228:231] -m per row tile,
  v[232:235] / v[236:239] LDS addresses of the K / V fragments in slot 0, v[240:243] lane offsets of the loads,
  v[244:247] scratch (table address, block ids), v[248:249] lane addresses of the two cross-lane
  maxima, v[250:253] raw score maximum of the coming tile per row tile, v[254:255] scratch.
  s[64:79]    counters, selectors, block ids, addresses, the "raise" mask.
"""

SLOT = 8192           # two blocks of K (or V): one ring slot


def Q(nt, ks): b = 40 + (nt * 4 + ks) * 4; return f"v[{b}:{b + 3}]"
def KA(mt, ks): b = 104 + (mt * 4 + ks) * 4; return f"v[{b}:{b + 3}]"
def VR(j): b = 136 + 4 * j; return f"v[{b}:{b + 3}]"
def VRe(j, c): return f"v{136 + 4 * j + c}"
def VA(i): b = 168 + 4 * i; return f"v[{b}:{b + 3}]"
def VAe(i, w): return f"v{168 + 4 * i + w}"
def P(s): b = 200 + 4 * s; return f"v[{b}:{b + 3}]"
def Pe(s, c): return f"v{200 + 4 * s + c}"
def T(x): return f"v{208 + x}"
ONES = "v[224:227]"
def NEGM(nt): return f"v{228 + nt}"
def KB(ks): return f"v{232 + ks}"      # slot 0
def VB(i): return f"v{236 + i}"
def KBT(ks): return f"v{32 + ks}"      # this iteration's slot
def VBT(i): return f"v{36 + i}"
def DOFF(i): return f"v{240 + i}"
VTAB, VID = "v244", "v[246:247]"
A16, A32 = "v248", "v249"
def TM(nt): return f"v{250 + nt}"
def O(nt, i): b = (nt * 8 + i) * 4; return f"a[{b}:{b + 3}]"
def Oe(nt, i, jj): return f"a{(nt * 8 + i) * 4 + jj}"
def LACC(nt): b = 128 + 4 * nt; return f"a[{b}:{b + 3}]"
def S(buf, nt, mt): b = 144 + 32 * buf + (nt * 2 + mt) * 4; return f"a[{b}:{b + 3}]"
def Se(buf, nt, mt, jj): return f"a{144 + 32 * buf + (nt * 2 + mt) * 4 + jj}"

ST, SSEL0, SSEL1, SB0, SB1, SLO, SHI, SSLOT, STMP, STMP2, SJ = "s64", "s66", "s67", "s68", "s69", "s70", "s71", "s72", "s73", "s74", "s75"
SADDR = "s[70:71]"
SEXEC, SRAISE = "s[76:77]", "s[78:79]"


class Lds:
    """Counts LDS operations in flight so that waits name the right number."""
    def __init__(self): self.n = 0
    def issue(self): self.n += 1; return self.n - 1
    def wait_for(self, idx): return f"s_waitcnt lgkmcnt({self.n - 1 - idx})"


class Gen:
    def __init__(self, team):
        self.T = team
        self.D = 2 * team
        self.L = 4 if team == 4 else 8       # loads per tile part
        self.out = []
        self.uid = 0

    def emit(self, s): self.out.append(s)

    def label(self, stem):
        self.uid += 1
        return f"{stem}{self.uid}_%="

    # ---- memory side
    def issue_own(self):
        """Requests this wave's part of tile SJ (the caller has checked SJ < ntiles)."""
        e = self.emit
        e(f"s_lshl_b32 {STMP}, {SJ}, 3")
        e(f"s_add_u32 {STMP}, {STMP}, %[tab]")
        e(f"s_add_u32 {STMP}, {STMP}, %[tabsel]")
        e(f"v_mov_b32 {VTAB}, {STMP}")
        e(f"ds_read_b32 v246, {VTAB}" if self.T == 4 else f"ds_read_b64 {VID}, {VTAB}")
        e("s_waitcnt lgkmcnt(0)")
        e(f"v_readfirstlane_b32 {SB0}, v246")
        if self.T == 2:
            e(f"v_readfirstlane_b32 {SB1}, v247")
        e("s_nop 3")
        e(f"s_max_i32 {SB0}, {SB0}, 0")
        if self.T == 2:
            e(f"s_max_i32 {SB1}, {SB1}, 0")
        e(f"s_and_b32 {SSLOT}, {SJ}, {self.D - 1}")
        e(f"s_lshl_b32 {SSLOT}, {SSLOT}, 13")
        e(f"s_add_u32 {SSLOT}, {SSLOT}, %[team]")
        e(f"s_add_u32 {SSLOT}, {SSLOT}, %[own_ring]")
        for blk, sb in enumerate((SB0, SB1)[: (1 if self.T == 4 else 2)]):
            e(f"s_mul_i32 {STMP}, {sb}, %[hkv]")
            e(f"s_add_u32 {STMP}, {STMP}, %[g]")
            e(f"s_lshr_b32 {SHI}, {STMP}, 20")
            e(f"s_lshl_b32 {SLO}, {STMP}, 12")
            e(f"s_add_u32 {SLO}, {SLO}, %[own_lo]")
            e(f"s_addc_u32 {SHI}, {SHI}, %[own_hi]")
            for q in range(4):
                e(f"s_add_u32 m0, {SSLOT}, {blk * 4096 + q * 1024}")
                e("s_nop 0")
                e(f"global_load_lds_dwordx4 {DOFF(q)}, {SADDR}")

    def wait_younger(self, sreg, kmax):
        """Waits until at most min(kmax, sreg) of this wave's tile parts are still on their way."""
        e = self.emit
        end = self.label("WE")
        labs = {}
        for k in range(kmax, 0, -1):
            labs[k] = self.label("W")
            e(f"s_cmp_ge_i32 {sreg}, {k}")
            e(f"s_cbranch_scc1 {labs[k]}")
        e("s_waitcnt vmcnt(0)")
        e(f"s_branch {end}")
        for k in range(kmax, 0, -1):
            e(f"{labs[k]}:")
            e(f"s_waitcnt vmcnt({k * self.L})")
            if k > 1:
                e(f"s_branch {end}")
        e(f"{end}:")

    # ---- instruction streams of one tile
    def scores(self, buf, kb, lds):
        """S(buf) = K Q^T for the tile whose K fragments are addressed by kb(ks).
        Returns (LDS read lines, [(mfma line, index of the LDS read it needs or None)])."""
        reads, mf, idx = [], [], {}
        for mt in range(2):
            for ks in range(4):
                reads.append(f"ds_read_b128 {KA(mt, ks)}, {kb(ks)} offset:{mt * 4096}")
                idx[(mt, ks)] = lds.issue()
        for mt in range(2):
            for ks in range(4):
                for nt in range(4):
                    c = "0" if ks == 0 else S(buf, nt, mt)
                    mf.append((f"v_mfma_f32_16x16x32_bf16 {S(buf, nt, mt)}, {KA(mt, ks)}, {Q(nt, ks)}, {c}",
                               idx[(mt, ks)] if nt == 0 else None))
        return reads, mf

    @staticmethod
    def weights_chain(buf, nt, pset):
        """P(pset) = bf16(exp2(S(buf, nt) * scale - m)) for this lane's 8 tokens."""
        v = []
        for mt in range(2):
            for jj in range(4):
                v.append(f"v_accvgpr_read_b32 {T(mt * 4 + jj)}, {Se(buf, nt, mt, jj)}")
        for x in range(8):
            v.append(f"v_fma_f32 {T(x)}, {T(x)}, %[scale], {NEGM(nt)}")
        for x in range(8):
            v.append(f"v_exp_f32 {T(x)}, {T(x)}")
        for c in range(4):
            v.append(f"v_cvt_pk_bf16_f32 {Pe(pset, c)}, {T(2 * c)}, {T(2 * c + 1)}")
        return v

    @staticmethod
    def perms():
        """8x8 transposes of 16-bit values, VA(i)[w] from VR(2w), VR(2w+1); ordered by w so that the first
        ones only need the first V rows."""
        v = []
        for w in range(4):
            for i in range(8):
                sel = SSEL1 if (i & 1) else SSEL0
                v.append((f"v_perm_b32 {VAe(i, w)}, {VRe(2 * w + 1, i >> 1)}, {VRe(2 * w, i >> 1)}, {sel}", 2 * w + 1))
        return v

    @staticmethod
    def pv(nt, pset):
        m = [f"v_mfma_f32_16x16x32_bf16 {LACC(nt)}, {ONES}, {P(pset)}, {LACC(nt)}"]
        for i in range(8):
            m.append(f"v_mfma_f32_16x16x32_bf16 {O(nt, i)}, {VA(i)}, {P(pset)}, {O(nt, i)}")
        return m

    def frag_reads(self, with_k):
        """Requests the LDS reads an iteration's first phase consumes: K fragments of the tile after it (unless it is
        the last) and the V rows of its own tile - all but the last V row, so that at most 15 reads are in flight.
        The address registers must have been set.  Returns the Lds counter and the read indices the waits refer to."""
        e = self.emit
        lds = Lds()
        kidx = {}
        if with_k:
            for mt in range(2):
                for ks in range(4):
                    e(f"ds_read_b128 {KA(mt, ks)}, {KBT(ks)} offset:{mt * 4096}")
                    kidx[(mt, ks)] = lds.issue()
        vidx = []
        for j in range(7 if with_k else 8):
            e(f"ds_read_b128 {VR(j)}, {VBT(j & 3)} offset:{(j >> 2) * 4096}")
            vidx.append(lds.issue())
        return lds, kidx, vidx

    def set_addresses(self, k_tile_plus, v_tile_plus, with_k):
        """LDS addresses of the fragments of K(t + k_tile_plus) and of the rows of V(t + v_tile_plus)."""
        e = self.emit
        D = self.D
        if with_k:
            e(f"s_add_u32 {STMP}, {ST}, {k_tile_plus}")
            e(f"s_and_b32 {STMP}, {STMP}, {D - 1}")
            e(f"s_lshl_b32 {STMP}, {STMP}, 13")
            for ks in range(4):
                e(f"v_add_u32 {KBT(ks)}, {STMP}, {KB(ks)}")
        e(f"s_add_u32 {STMP}, {ST}, {v_tile_plus}")
        e(f"s_and_b32 {STMP}, {STMP}, {D - 1}")
        e(f"s_lshl_b32 {STMP}, {STMP}, 13")
        for i in range(4):
            e(f"v_add_u32 {VBT(i)}, {STMP}, {VB(i)}")

    def tile(self, cur, last, name):
        """Iteration t: weights of tile t from S(cur), O^T += V(t)^T P^T and, unless `last`, S(1-cur) = K(t+1) Q^T.
        The LDS reads of the first phase were requested by the iteration before (or the prologue)."""
        e = self.emit
        nxt = 1 - cur
        D = self.D
        e(f"; ---- {name}")
        # the reads in flight, in the order frag_reads requested them
        lds = Lds()
        mf = []
        if not last:
            _, mf = self.scores(nxt, KBT, lds)          # (only its bookkeeping: the reads themselves are already on their way)
        vidx = [lds.issue() for _ in range(8 if last else 7)]
        vread7 = f"ds_read_b128 {VR(7)}, {VBT(3)} offset:4096"
        # ---- phase 1: S MFMAs with the first weights and the transposes on the vector unit (the weights need
        # nothing from LDS, so they go first and the V rows have landed by the time of the transposes)
        valu = [("plain", x) for x in self.weights_chain(cur, 0, 0)]
        valu += [("plain", x) for x in self.weights_chain(cur, 1, 1)]
        valu += [("perm", x) for x in self.perms()]
        state = {"vi": 0, "pending": not last}

        def late_read():
            if state["pending"]:
                e(vread7); vidx.append(lds.issue()); state["pending"] = False

        def push_valu(k):
            for _ in range(k):
                if state["vi"] >= len(valu):
                    return
                kind, x = valu[state["vi"]]
                if kind == "perm":
                    line, need = x
                    if need == 7:
                        late_read()               # (at most 15 LDS reads in flight)
                    e(lds.wait_for(vidx[need]))
                    e(line)
                else:
                    e(x)
                state["vi"] += 1
        for k, (line, need) in enumerate(mf):
            if need is not None:
                e(lds.wait_for(need))
            e(line)
            if k == 3:
                late_read()
            push_valu(3)
        push_valu(len(valu))
        e("s_waitcnt lgkmcnt(0)")
        if not last:
            # ---- tile t is read out by me.  My part of tile t+2 has landed; after the barrier everybody's has, and
            # everybody is done with tile t: refill its slot with tile t+D, and request the reads of iteration t+1.
            e(f"s_sub_i32 {STMP}, %[ntiles], {ST}")
            e(f"s_sub_i32 {STMP}, {STMP}, 3")
            self.wait_younger(STMP, D - 3)
            e("s_barrier")
            no = self.label("NI")
            e(f"s_add_u32 {SJ}, {ST}, {D}")
            e(f"s_cmp_lt_i32 {SJ}, %[ntiles]")
            e(f"s_cbranch_scc0 {no}")
            self.issue_own()
            e(f"{no}:")
            nolast, done = self.label("RK"), self.label("RD")
            e(f"s_add_u32 {STMP2}, {ST}, 2")
            e(f"s_cmp_lt_i32 {STMP2}, %[ntiles]")
            e(f"s_cbranch_scc1 {nolast}")
            self.set_addresses(2, 1, False)             # iteration t+1 is the last: only V(t+1)
            self.frag_reads(False)
            e(f"s_branch {done}")
            e(f"{nolast}:")
            self.set_addresses(2, 1, True)
            self.frag_reads(True)
            e(f"{done}:")
        # ---- phase 2: O^T += V^T P^T for row tiles 0, 1 with the weights of row tiles 2, 3 on the vector unit
        e("s_nop 1")
        valu2 = self.weights_chain(cur, 2, 0)
        m2 = self.pv(0, 0) + self.pv(1, 1)
        k2 = 0
        for k, line in enumerate(m2):     # P(0) is rewritten for row tile 2 only after the products of row tile 0 are issued
            e(line)
            if k >= 9:
                for _ in range(4):
                    if k2 < len(valu2): e(valu2[k2]); k2 += 1
        while k2 < len(valu2): e(valu2[k2]); k2 += 1
        e("s_nop 1")
        valu3 = self.weights_chain(cur, 3, 1)
        n_chain = len(valu3)
        if not last:
            # while the last products run: does a score of tile t+1 outgrow its row's reference?
            e(f"s_mov_b64 {SRAISE}, 0")
            for nt in range(4):
                for mt in range(2):
                    for jj in range(4):
                        valu3.append(f"v_accvgpr_read_b32 {T(8 + mt * 4 + jj)}, {Se(nxt, nt, mt, jj)}")
                valu3.append(f"v_max3_f32 {T(8)}, {T(8)}, {T(9)}, {T(10)}")
                valu3.append(f"v_max3_f32 {T(11)}, {T(11)}, {T(12)}, {T(13)}")
                valu3.append(f"v_max3_f32 {T(8)}, {T(8)}, {T(11)}, {T(14)}")
                valu3.append(f"v_max_f32 {TM(nt)}, {T(8)}, {T(15)}")
                valu3.append(f"v_fma_f32 {T(9)}, {TM(nt)}, %[scale], {NEGM(nt)}")
                valu3.append(f"v_cmp_lt_f32 vcc, 0x41c00000, {T(9)}")
                valu3.append(f"s_or_b64 {SRAISE}, {SRAISE}, vcc")
        k3 = 0
        for line in self.pv(2, 0):
            e(line)
            for _ in range(4):
                if k3 < n_chain: e(valu3[k3]); k3 += 1
        while k3 < n_chain: e(valu3[k3]); k3 += 1
        e("s_nop 1")
        for line in self.pv(3, 1):
            e(line)
            for _ in range(5):
                if k3 < len(valu3): e(valu3[k3]); k3 += 1
        while k3 < len(valu3): e(valu3[k3]); k3 += 1
        if not last:
            no = self.label("NR")
            e(f"s_cmp_eq_u64 {SRAISE}, 0")
            e(f"s_cbranch_scc1 {no}")
            self.raise_refs()
            e(f"{no}:")

    def raise_refs(self):
        """Rare: every row's reference becomes max(old reference, row maximum of the coming tile); O^T and the
        row sums are scaled by 2^(old - new) (1 where nothing changed)."""
        e = self.emit
        e("s_nop 7")
        e("s_nop 7")
        e("s_nop 3")
        for nt in range(4):
            e(f"ds_bpermute_b32 {T(8)}, {A16}, {TM(nt)}")
            e("s_waitcnt lgkmcnt(0)")
            e(f"v_max_f32 {T(9)}, {TM(nt)}, {T(8)}")
            e("s_nop 1")
            e(f"ds_bpermute_b32 {T(8)}, {A32}, {T(9)}")
            e("s_waitcnt lgkmcnt(0)")
            e(f"v_max_f32 {T(9)}, {T(9)}, {T(8)}")
            e(f"v_mul_f32 {T(9)}, %[scale], {T(9)}")
            e(f"v_xor_b32 {T(10)}, 0x80000000, {NEGM(nt)}")
            e(f"v_max_f32 {T(9)}, {T(9)}, {T(10)}")
            e(f"v_sub_f32 {T(10)}, {T(10)}, {T(9)}")
            e(f"v_exp_f32 {T(10)}, {T(10)}")
            e(f"v_xor_b32 {NEGM(nt)}, 0x80000000, {T(9)}")
            e("s_nop 1")
            regs = [f"a{(nt * 8 + i) * 4 + jj}" for i in range(8) for jj in range(4)] + [f"a{128 + 4 * nt + jj}" for jj in range(4)]
            for k in range(0, len(regs), 4):
                grp = regs[k:k + 4]
                for x, r in enumerate(grp): e(f"v_accvgpr_read_b32 {T(11 + x)}, {r}")
                for x, r in enumerate(grp): e(f"v_mul_f32 {T(11 + x)}, {T(10)}, {T(11 + x)}")
                for x, r in enumerate(grp): e(f"v_accvgpr_write_b32 {r}, {T(11 + x)}")
        e("s_nop 7")

    def build(self):
        e = self.emit
        D = self.D
        vring = D * SLOT
        e(f"; ---- team of {self.T}: setup (selectors, ones, per-lane addresses)")
        e(f"s_mov_b32 {SSEL0}, 0x05040100")
        e(f"s_mov_b32 {SSEL1}, 0x07060302")
        for k in range(4):
            e(f"v_mov_b32 v{224 + k}, 0x3f803f80")
        e(f"v_add_u32 {KB(0)}, %[team], %[koff0]")
        for ks in range(1, 4):
            e(f"v_xor_b32 {KB(ks)}, {64 * ks}, %[koff0]")
            e(f"v_add_u32 {KB(ks)}, %[team], {KB(ks)}")
        e(f"v_add_u32 {VB(0)}, %[team], %[voff0]")
        e(f"v_add_u32 {VB(0)}, {vring}, {VB(0)}")
        for i in range(1, 4):
            e(f"v_xor_b32 {VB(i)}, {16 * i}, %[voff0]")
            e(f"v_add_u32 {VB(i)}, {256 * i + vring}, {VB(i)}")
            e(f"v_add_u32 {VB(i)}, %[team], {VB(i)}")
        e(f"v_mov_b32 {DOFF(0)}, %[doff0]")
        for i in range(1, 4):
            e(f"v_xor_b32 {DOFF(i)}, {64 * i}, %[doff0]")
            e(f"v_add_u32 {DOFF(i)}, {1024 * i}, {DOFF(i)}")
        e("; ---- query rows (rows past the end repeat a valid one), then my parts of the first D-1 tiles")
        for nt in range(4):
            for ks in range(4):
                e(f"global_load_dwordx4 {Q(nt, ks)}, %[q{nt}], %[qbase] offset:{64 * ks}")
        for j in range(D):
            no = self.label("NP")
            e(f"s_mov_b32 {SJ}, {j}")
            if j >= 4:
                e(f"s_cmp_lt_i32 {SJ}, %[ntiles]")
                e(f"s_cbranch_scc0 {no}")
            self.issue_own()
            e(f"{no}:")
        for k in range(144):
            e(f"v_accvgpr_write_b32 a{k}, 0")
        e("; ---- S(A) = K(0) Q^T, reference exponent = row maximum of the first tile")
        e(f"s_sub_i32 {STMP}, %[ntiles], 2")       # my parts of tiles 0 and 1
        self.wait_younger(STMP, D - 2)
        e("s_barrier")
        lds = Lds()
        kreads, mf = self.scores(0, KB, lds)
        for r in kreads: e(r)
        for line, need in mf:
            if need is not None: e(lds.wait_for(need))
            e(line)
        e("s_waitcnt lgkmcnt(0)")
        e("s_nop 7")
        e("s_nop 7")
        e(f"v_xor_b32 {A16}, 64, %[lane4]")       # lane ^ 16
        e(f"v_xor_b32 {A32}, 128, %[lane4]")      # lane ^ 32
        for nt in range(4):
            for mt in range(2):
                for jj in range(4):
                    e(f"v_accvgpr_read_b32 {T(mt * 4 + jj)}, {Se(0, nt, mt, jj)}")
            e(f"v_max3_f32 {T(8)}, {T(0)}, {T(1)}, {T(2)}")
            e(f"v_max3_f32 {T(9)}, {T(3)}, {T(4)}, {T(5)}")
            e(f"v_max3_f32 {T(8)}, {T(8)}, {T(6)}, {T(7)}")
            e(f"v_max_f32 {T(8)}, {T(8)}, {T(9)}")
            e(f"ds_bpermute_b32 {T(10)}, {A16}, {T(8)}")
            e("s_waitcnt lgkmcnt(0)")
            e(f"v_max_f32 {T(8)}, {T(8)}, {T(10)}")
            e("s_nop 1")
            e(f"ds_bpermute_b32 {T(10)}, {A32}, {T(8)}")
            e("s_waitcnt lgkmcnt(0)")
            e(f"v_max_f32 {T(8)}, {T(8)}, {T(10)}")
            e(f"v_mul_f32 {T(8)}, %[scale], {T(8)}")
            e(f"v_xor_b32 {NEGM(nt)}, 0x80000000, {T(8)}")
        e(f"s_mov_b32 {ST}, 0")
        self.set_addresses(1, 0, True)             # the reads of iteration 0: K(1) and V(0)
        self.frag_reads(True)
        e("LOOP_%=:")
        e(f"s_add_u32 {STMP}, {ST}, 1")
        e(f"s_cmp_eq_u32 {STMP}, %[ntiles]")
        e("s_cbranch_scc1 LASTA_%=")
        self.tile(0, False, "TA")
        e(f"s_add_u32 {ST}, {ST}, 1")
        e(f"s_add_u32 {STMP}, {ST}, 1")
        e(f"s_cmp_eq_u32 {STMP}, %[ntiles]")
        e("s_cbranch_scc1 LASTB_%=")
        self.tile(1, False, "TB")
        e(f"s_add_u32 {ST}, {ST}, 1")
        e("s_branch LOOP_%=")
        e("LASTA_%=:")
        self.tile(0, True, "LA")
        e("s_branch DONE_%=")
        e("LASTB_%=:")
        self.tile(1, True, "LB")
        e("DONE_%=:")
        e("; ---- partial rows: acc[128] per row as the other sweeps lay them out, then (m, l)")
        e("s_nop 7")
        e("s_nop 7")
        e("s_nop 3")
        e(f"s_mov_b64 {SEXEC}, exec")
        e(f"v_lshlrev_b32 {TM(0)}, 3, %[nrow]")         # (m, l) offset of row n: 8 n
        for nt in range(4):
            e(f"s_mov_b64 exec, {SEXEC}")               # (the (m, l) store of the row tile before narrowed it)
            e(f"v_add_u32 v244, {16 * nt}, %[nrow]")
            e(f"v_cmp_gt_i32 vcc, %[nrows], v244")
            e(f"s_and_b64 exec, {SEXEC}, vcc")
            e(f"v_add_u32 v245, {16 * nt * 512}, %[dst0]")
            k = 0
            for jj in range(4):
                for half in range(2):
                    base = 4 * (k & 3)
                    for x in range(4):
                        e(f"v_accvgpr_read_b32 {T(base + x)}, {Oe(nt, 4 * half + x, jj)}")
                    e("s_nop 0")
                    e(f"global_store_dwordx4 v245, v[{208 + base}:{208 + base + 3}], %[accbase] offset:{jj * 32 + half * 16}")
                    k += 1
            e(f"v_xor_b32 v254, 0x80000000, {NEGM(nt)}")
            e(f"v_accvgpr_read_b32 v255, a{128 + 4 * nt}")
            e(f"v_cmp_gt_u32 vcc, 64, %[lane4]")          # (m, l): lanes of the first lane group only
            e(f"s_and_b64 exec, exec, vcc")
            e(f"v_add_u32 {TM(1)}, {16 * nt * 8}, {TM(0)}")
            e("s_nop 0")
            e(f"global_store_dwordx2 {TM(1)}, v[254:255], %[mlbase]")
            e("s_nop 1")
        e(f"s_mov_b64 exec, {SEXEC}")
        e("s_waitcnt vmcnt(0)")
        return self.out


def main():
    print("// Generated by gen_sweep_core.py - do not edit by hand.")
    for team in (2, 4):
        lines = Gen(team).build()
        print(f"#define FEA_TEAM{team}_CORE_ASM \\")
        print(" \\\n".join(f'    "{line}\\n\\t"' for line in lines))
        print()
    vregs = ", ".join(f'"v{k}"' for k in range(32, 256))
    aregs = ", ".join(f'"a{k}"' for k in range(0, 208))
    sregs = ", ".join(f'"s{k}"' for k in range(64, 80))
    print(f"#define FEA_TEAM_CORE_CLOBBERS {vregs}, {aregs}, {sregs}, \"vcc\", \"scc\", \"m0\", \"memory\"")


if __name__ == "__main__":
    main()
