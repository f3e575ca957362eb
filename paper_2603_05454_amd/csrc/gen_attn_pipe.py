#!/usr/bin/env python3
"""Generator of lsp_attn_pipe_loop.inc: the hand-scheduled block loop of the
long-suffix bf16 attention kernel (head_dim 128) as one inline-asm statement,
and of lsp_attn_pipe_idle_loop.inc, the loader-only loop that waves without an
active query run beside it (generate_idle below).

Why generated assembly: with compiler scheduling a wave issues the products of a
32-key block as one burst (waiting on every LDS fragment read just before its
matrix instruction) and the soft-max as another, and the two waves of a SIMD do
not fill each other's gaps well enough (measured: the matrix pipe ran ~45 % of
the time).  Here the issue order of a block is fixed by hand:

  * one-block software pipeline per wave: while the matrix pipe runs S(j+1) =
    K(j+1).Q^T (8 dependent v_mfma_f32_32x32x16_bf16), the vector ALU turns
    S(j) into bf16 probabilities, two scores per matrix instruction, in three
    staggered stages (fma, exp2 one slot later, pack + row sum one slot after
    that) so that no instruction waits for its operand; then O^T += V(j)^T.P(j)^T
    (8 instructions on 4 independent accumulators) covers the block maximum of
    S(j+1) and the LDS reads of the K fragments of block j+2;
  * every LDS fragment is requested at least half a block before it is used; the
    s_waitcnt values are computed by this script from the issue order;
  * the reference m of the online soft-max moves on a cold, wave-uniform branch
    taken at the top of a block when its maximum exceeds m by 8 octaves.

Register map (VGPRs; the kernel runs two waves per SIMD, 256 registers each):
  v0-15 / v16-31   score blocks S (ping-pong: current / next)
  v32-63           Q fragments (B operand of the first product), 8 x 4
  v64-95           K fragments of the next block, 8 x 4
  v96-127          V^T fragments of the current block, 8 x 4 (f = 4*k2 + db)
  v128-135         packed probabilities (B operand of the second product)
  v136-151         soft-max temporaries (one pair per packed word)
  v152-159         LDS addresses of the K fragments (stage 0), v160-163 of V^T
  v164/165         lane offsets of this wave's K / V rows in a block (bytes)
  v166/167         the same for suffix rows (copied to v164/165 at the switch)
  v168 -m, v169 row sum l, v170 block maximum, v171 block sum, v172-175 scratch
  v176-239         O^T accumulators, 4 x 16
  v240-255         not touched (left to the compiler)
SGPRs s64-s79 are scratch; every other scalar is an asm operand.

Blocks: the loop only sees FULL 32-row blocks: first the nc blocks of the cache,
then the blocks of the suffix rows; ragged ends are handled by the caller.
Ring: NS = 8 stages of 8 KB K + 8 KB V; block i lives in stage i % 8; iteration j
requests block j + 6 (into the stage block j - 2 left), reads V(j) and K(j+2);
the workgroup meets at a barrier after every odd iteration, before which each
wave waits until all but its newest 4 loads (2 blocks) have landed.
"""
import os

NS, LA, TILE = 8, 6, 32 * 256
VBASE = NS * TILE

S = [list(range(0, 16)), list(range(16, 32))]
QF = [32 + 4 * k for k in range(8)]
KF = [64 + 4 * k for k in range(8)]
VF = [96 + 4 * f for f in range(8)]
PF = list(range(128, 136))
T = list(range(136, 152))
KADDR = list(range(152, 160))
VADDR = list(range(160, 164))
KOFF, VOFF, KOFF_S, VOFF_S = 164, 165, 166, 167
NM, LSUM, BM, BSUM, X0, X1, X2, X3 = 168, 169, 170, 171, 172, 173, 174, 175
O = [176 + 16 * d for d in range(4)]

# scratch SGPRs
SG = dict(m0save=64, kp=66, vp=68, step=70, li=71, jn=72, sw=73, t=74)


def vr(a, n=1):
    return f"v{a}" if n == 1 else f"v[{a}:{a + n - 1}]"


class Emitter:
    def __init__(self):
        self.lines = []
        self.lds_issued = 0      # LDS reads issued so far (they return in order)
        self.lds_seq = {}        # register base -> sequence number of the read that fills it

    def e(self, s):
        self.lines.append(s)

    def lds_read(self, kind, dst, n, addr, offset):
        self.e(f"{kind} {vr(dst, n)}, v{addr} offset:{offset}")
        self.lds_seq[dst] = self.lds_issued
        self.lds_issued += 1

    def need(self, *dsts):
        """Wait until the LDS reads that fill these registers have returned."""
        seqs = [self.lds_seq[d] for d in dsts if d in self.lds_seq]
        if not seqs:
            return
        allowed = self.lds_issued - max(seqs) - 1      # reads issued after the newest one needed
        self.e(f"s_waitcnt lgkmcnt({min(allowed, 15)})")
        for d in [d for d, q in self.lds_seq.items() if q <= max(seqs)]:
            del self.lds_seq[d]


def switch_to_suffix(E):
    E.e(f"s_mov_b64 s[{SG['kp']}:{SG['kp'] + 1}], %[ks]")
    E.e(f"s_mov_b64 s[{SG['vp']}:{SG['vp'] + 1}], %[vs]")
    E.e(f"s_mov_b32 s{SG['step']}, %[sstep]")
    E.e(f"v_mov_b32 v{KOFF}, v{KOFF_S}")
    E.e(f"v_mov_b32 v{VOFF}, v{VOFF_S}")


def load_block(E, stage, tag):
    """Request the next block of the key stream into `stage` (2 wave-wide loads: this
    wave's 4 K rows and 4 V rows); beyond the last block the pointers stay, so the last
    block is requested again (into a stage nobody reads) and the number of loads in
    flight is fixed.  The switch from cache rows to suffix rows is out of line."""
    li, kp, vp, step, t = SG["li"], SG["kp"], SG["vp"], SG["step"], SG["t"]
    E.e(f"s_cmp_eq_u32 s{li}, s{SG['sw']}")
    E.e(f"s_cbranch_scc1 .Lswitch_{tag}_%=")
    E.e(f".Lissue_{tag}_%=:")
    E.e(f"s_add_u32 m0, %[ldsk], {stage * TILE}")
    E.e(f"s_add_u32 s{li}, s{li}, 1")
    E.e(f"global_load_lds_dwordx4 v{KOFF}, s[{kp}:{kp + 1}]")
    E.e(f"s_add_u32 m0, %[ldsk], {VBASE + stage * TILE}")
    E.e(f"s_cmp_lt_u32 s{li}, %[nb]")
    E.e(f"global_load_lds_dwordx4 v{VOFF}, s[{vp}:{vp + 1}]")
    E.e(f"s_cselect_b32 s{t}, s{step}, 0")
    E.e(f"s_add_u32 s{kp}, s{kp}, s{t}")
    E.e(f"s_addc_u32 s{kp + 1}, s{kp + 1}, 0")
    E.e(f"s_add_u32 s{vp}, s{vp}, s{t}")
    E.e(f"s_addc_u32 s{vp + 1}, s{vp + 1}, 0")


def switch_code(E, tag):
    E.e(f".Lswitch_{tag}_%=:")
    switch_to_suffix(E)
    E.e(f"s_branch .Lissue_{tag}_%=")


def read_k_frags(E, stage, ks):
    for kk in ks:
        E.lds_read("ds_read_b128", KF[kk], 4, KADDR[kk], stage * TILE)


def block_max(E, sn, part):
    """Maximum of this lane's 16 scores of register block sn (raw, unscaled), in three parts.
    The fold over the two lanes of a query happens on the cold path only."""
    if part == 0:
        E.e(f"v_max_f32 v{BM}, v{sn[0]}, v{sn[1]}")
        E.e(f"v_max3_f32 v{BM}, v{BM}, v{sn[2]}, v{sn[3]}")
    else:
        for r in range(4 + 6 * (part - 1), 10 + 6 * (part - 1), 2):
            E.e(f"v_max3_f32 v{BM}, v{BM}, v{sn[r]}, v{sn[r + 1]}")


def iteration(E, u):
    """Block j = 8n + u: soft-max of S(j) under S(j+1) = K(j+1).Q^T, then O += V(j)^T.P(j)^T."""
    cur, nxt = S[u & 1], S[(u + 1) & 1]
    # reference check on the maximum of S(j) (computed while the previous block's second product ran)
    # (any lane's own half-column above the reference by 8 octaves sends the wave to the cold path)
    E.e(f"v_fma_f32 v{X0}, v{BM}, %[sc], v{NM}")
    E.e(f"v_cmp_lt_f32 vcc, 0x41000000, v{X0}")
    E.e(f"s_cbranch_vccnz .Lresc_{u}_%=")
    E.e(f".Lafter_{u}_%=:")
    load_block(E, (u + LA) % NS, f"i{u}")

    def stage_f(i):
        for e in (2 * i, 2 * i + 1):
            E.e(f"v_fma_f32 v{T[e]}, v{cur[e]}, %[sc], v{NM}")

    def stage_e(i):
        for e in (2 * i, 2 * i + 1):
            E.e(f"v_exp_f32 v{T[e]}, v{T[e]}")

    def stage_c(i):
        E.e(f"v_cvt_pk_bf16_f32 v{PF[i]}, v{T[2 * i]}, v{T[2 * i + 1]}")
        E.e(f"v_dot2c_f32_bf16 v{LSUM}, 0x3f803f80, v{PF[i]}")

    # first product of the NEXT block, soft-max of this one, V^T fragment reads of this one;
    # the wave in this half of its iteration goes first when the two waves of a SIMD both have
    # an instruction ready, the one in the second product yields: its eight independent matrix
    # instructions fill whatever the other leaves (measured: 2.5 % faster than equal priorities;
    # raising the priority anywhere inside the second product loses all of it again)
    E.e("s_setprio 1")
    for kk in range(8):
        if kk % 4 == 0:
            E.need(*KF[kk:kk + 4])
        c = vr(nxt[0], 16) if kk else "0"
        E.e(f"v_mfma_f32_32x32x16_bf16 {vr(nxt[0], 16)}, {vr(KF[kk], 4)}, {vr(QF[kk], 4)}, {c}")
        k2, db = kk // 4, kk % 4
        E.lds_read("ds_read_b64_tr_b16", VF[kk], 2, VADDR[db], VBASE * 0 + u * TILE + 4096 * k2)
        E.lds_read("ds_read_b64_tr_b16", VF[kk] + 2, 2, VADDR[db], u * TILE + 4096 * k2 + 2048)
        stage_f(kk)
        if kk >= 1:
            stage_e(kk - 1)
        if kk >= 2:
            stage_c(kk - 2)
    # second product of this block
    E.e("s_setprio 0")
    for m in range(8):
        k2, db = m // 4, m % 4
        f = 4 * k2 + db
        if m % 4 == 0:
            E.need(*[VF[f + d] + h for d in range(4) for h in (0, 2)])
        E.e(f"v_mfma_f32_32x32x16_bf16 {vr(O[db], 16)}, {vr(VF[f], 4)}, {vr(PF[4 * k2], 4)}, {vr(O[db], 16)}")
        if m == 0:
            stage_e(7)
            stage_c(6)
        elif m == 1:
            stage_c(7)
        elif m == 2:
            read_k_frags(E, (u + 2) % NS, (0, 1))
        elif m == 3:
            read_k_frags(E, (u + 2) % NS, (2, 3))
        elif m == 4:
            read_k_frags(E, (u + 2) % NS, (4, 5))
            block_max(E, nxt, 0)
        elif m == 5:
            read_k_frags(E, (u + 2) % NS, (6, 7))
            block_max(E, nxt, 1)
        elif m == 6:
            block_max(E, nxt, 2)
    E.e(f"s_add_u32 s{SG['jn']}, s{SG['jn']}, 1")
    E.e(f"s_cmp_lt_u32 s{SG['jn']}, %[nb]")
    E.e("s_cbranch_scc0 .Lexit_%=")
    if u & 1:
        E.e(f"s_waitcnt vmcnt({2 * (LA - 4)})")
        E.e("s_barrier")


def rescale(E, u):
    """Cold path: lanes whose block maximum exceeds the reference by more than 8 octaves
    take it as the new reference; sums and accumulators are scaled by 2^(old - new)."""
    E.e(f".Lresc_{u}_%=:")
    E.e("s_nop 15")                                        # the accumulators were written by matrix instructions
    E.e(f"v_mov_b32 v{X1}, v{BM}")                         # fold the two lanes of a query: both get the column maximum
    E.e("s_nop 1")
    E.e(f"v_permlane32_swap_b32 v{BM}, v{X1}")
    E.e("s_nop 1")
    E.e(f"v_max_f32 v{BM}, v{BM}, v{X1}")
    E.e(f"v_mul_f32 v{BM}, %[sc], v{BM}")                  # log2 domain
    E.e(f"v_add_f32 v{X0}, v{BM}, v{NM}")
    E.e(f"v_cmp_lt_f32 vcc, 0x41000000, v{X0}")            # per query now (the same in both of its lanes)
    E.e(f"v_xor_b32 v{X1}, 0x80000000, v{NM}")             # old reference
    E.e("s_nop 1")
    E.e(f"v_cndmask_b32 v{X2}, v{X1}, v{BM}, vcc")         # new reference: the block maximum where vcc, else the old one
    E.e(f"v_sub_f32 v{X3}, v{X1}, v{X2}")
    E.e("s_nop 0")
    E.e(f"v_exp_f32 v{X3}, v{X3}")                         # 2^(old - new): 1 where unchanged, 0 on the first block (old = -inf)
    E.e(f"v_xor_b32 v{NM}, 0x80000000, v{X2}")
    E.e("s_nop 1")
    E.e(f"v_mul_f32 v{LSUM}, v{LSUM}, v{X3}")
    for r in range(O[0], O[0] + 64):
        E.e(f"v_mul_f32 v{r}, v{r}, v{X3}")
    E.e("s_nop 4")
    E.e(f"s_branch .Lafter_{u}_%=")


def generate():
    E = Emitter()
    li, kp, vp, step, jn = SG["li"], SG["kp"], SG["vp"], SG["step"], SG["jn"]
    E.e(f"s_mov_b32 s{SG['m0save']}, m0")
    E.e(f"s_mov_b64 s[{kp}:{kp + 1}], %[kc]")
    E.e(f"s_mov_b64 s[{vp}:{vp + 1}], %[vc]")
    E.e(f"s_mov_b32 s{step}, %[cstep]")
    E.e(f"s_mov_b32 s{li}, 0")
    E.e(f"s_mov_b32 s{jn}, 0")
    # index of the block at which the stream switches from cache rows to suffix rows (none: never)
    E.e("s_cmp_lt_u32 %[nc], %[nb]")
    E.e(f"s_cselect_b32 s{SG['sw']}, %[nc], -1")
    for t in range(LA):
        load_block(E, t, f"p{t}")
    # blocks 0..3 have landed everywhere
    E.e(f"s_waitcnt vmcnt({2 * (LA - 4)})")
    E.e("s_barrier")
    # S(0) = K(0).Q^T, its maximum, and the K fragments of block 1
    read_k_frags(E, 0, range(8))
    for kk in range(8):
        E.need(KF[kk])
        c = vr(S[0][0], 16) if kk else "0"
        E.e(f"v_mfma_f32_32x32x16_bf16 {vr(S[0][0], 16)}, {vr(KF[kk], 4)}, {vr(QF[kk], 4)}, {c}")
    E.e("s_nop 7")
    read_k_frags(E, 1, range(8))
    E.e("s_nop 7")
    for part in range(3):
        block_max(E, S[0], part)
    E.e(".Lloop_%=:")
    for u in range(NS):
        iteration(E, u)
    E.e("s_branch .Lloop_%=")
    E.e(".Lexit_%=:")
    E.e("s_waitcnt vmcnt(0) lgkmcnt(0)")
    E.e(f"s_mov_b32 m0, s{SG['m0save']}")
    E.e("s_nop 15")
    E.e("s_branch .Lend_%=")
    for u in range(NS):
        rescale(E, u)
        switch_code(E, f"i{u}")
    for t in range(LA):
        switch_code(E, f"p{t}")
    E.e(".Lend_%=:")
    return E.lines


def generate_idle():
    """The loop of a wave none of whose 32 queries is active (the last tile of a suffix that
    is not a multiple of 256 rows): its share of every block's loads, the waits and the
    barriers of the loop above in the same order, and nothing else - the matrix pipe and the
    vector ALU of its SIMD are left to the other wave."""
    E = Emitter()
    li, kp, vp, step, jn = SG["li"], SG["kp"], SG["vp"], SG["step"], SG["jn"]
    E.e(f"s_mov_b32 s{SG['m0save']}, m0")
    E.e(f"s_mov_b64 s[{kp}:{kp + 1}], %[kc]")
    E.e(f"s_mov_b64 s[{vp}:{vp + 1}], %[vc]")
    E.e(f"s_mov_b32 s{step}, %[cstep]")
    E.e(f"s_mov_b32 s{li}, 0")
    E.e(f"s_mov_b32 s{jn}, 0")
    E.e("s_cmp_lt_u32 %[nc], %[nb]")
    E.e(f"s_cselect_b32 s{SG['sw']}, %[nc], -1")
    for t in range(LA):
        load_block(E, t, f"p{t}")
    E.e(f"s_waitcnt vmcnt({2 * (LA - 4)})")
    E.e("s_barrier")
    E.e(".Lloop_%=:")
    for u in range(NS):
        load_block(E, (u + LA) % NS, f"i{u}")
        E.e(f"s_add_u32 s{jn}, s{jn}, 1")
        E.e(f"s_cmp_lt_u32 s{jn}, %[nb]")
        E.e("s_cbranch_scc0 .Lexit_%=")
        if u & 1:
            E.e(f"s_waitcnt vmcnt({2 * (LA - 4)})")
            E.e("s_barrier")
    E.e("s_branch .Lloop_%=")
    E.e(".Lexit_%=:")
    E.e("s_waitcnt vmcnt(0)")
    E.e(f"s_mov_b32 m0, s{SG['m0save']}")
    E.e("s_branch .Lend_%=")
    for u in range(NS):
        switch_code(E, f"i{u}")
    for t in range(LA):
        switch_code(E, f"p{t}")
    E.e(".Lend_%=:")
    return E.lines


HEADER = """// GENERATED by gen_attn_pipe.py - do not edit; the register map, the pipeline and the
// synchronisation protocol are described in that script.
// Expects in scope: f32x16 oacc[4]; float nm, lsum; u32x16 qf_lo, qf_hi, addr;
// uint64_t kc_base, vc_base, ks_base, vs_base; uint32_t cstep, sstep, nc, nb, ldsk; float sc.
"""


def main():
    lines = generate()
    body = "\n".join(f'    "{l}\\n"' for l in lines)
    clob = [f"v{i}" for i in list(range(0, 32)) + list(range(64, 152)) + list(range(170, 176))]
    clob += [f"s{i}" for i in range(64, 80)] + ["vcc", "scc", "memory"]
    text = HEADER + "asm volatile(\n" + body + "\n"
    text += ('    : "+{v[176:191]}"(oacc[0]), "+{v[192:207]}"(oacc[1]), "+{v[208:223]}"(oacc[2]), "+{v[224:239]}"(oacc[3]),\n'
             '      "+{v168}"(nm), "+{v169}"(lsum), "+{v[152:167]}"(addr)\n'
             '    : "{v[32:47]}"(qf_lo), "{v[48:63]}"(qf_hi),\n'
             '      [kc] "s"(kc_base), [vc] "s"(vc_base), [ks] "s"(ks_base), [vs] "s"(vs_base),\n'
             '      [cstep] "s"(cstep), [sstep] "s"(sstep), [nc] "s"(nc), [nb] "s"(nb), [ldsk] "s"(ldsk), [sc] "s"(sc)\n')
    text += "    : " + ", ".join(f'"{c}"' for c in clob) + ");\n"
    here = os.path.dirname(os.path.abspath(__file__))
    out = os.path.join(here, "lsp_attn_pipe_loop.inc")
    with open(out, "w") as f:
        f.write(text)
    with open(os.path.join(here, "lsp_attn_pipe_idle_loop.inc"), "w") as f:
        f.write(idle_text())
    return out


IDLE_HEADER = """// GENERATED by gen_attn_pipe.py - do not edit: the block loop of a wave without an active query
// (loads, waits and barriers of lsp_attn_pipe_loop.inc in the same order, nothing else).
// Expects in scope: u32x16 addr; uint64_t kc_base, vc_base, ks_base, vs_base;
// uint32_t cstep, sstep, nc, nb, ldsk.
"""


def idle_text():
    body = "\n".join(f'    "{l}\\n"' for l in generate_idle())
    clob = [f"s{i}" for i in range(64, 80)] + ["scc", "memory"]
    text = IDLE_HEADER + "asm volatile(\n" + body + "\n"
    text += ('    : "+{v[152:167]}"(addr)\n'
             '    : [kc] "s"(kc_base), [vc] "s"(vc_base), [ks] "s"(ks_base), [vs] "s"(vs_base),\n'
             '      [cstep] "s"(cstep), [sstep] "s"(sstep), [nc] "s"(nc), [nb] "s"(nb), [ldsk] "s"(ldsk)\n')
    text += "    : " + ", ".join(f'"{c}"' for c in clob) + ");\n"
    return text


if __name__ == "__main__":
    print(main())
