#!/usr/bin/env python3
"""Writes ta_sp_block.inc: the per-tile blocks of the 256-row KV-pass kernel as single inline-asm statements.

    python gen_sp_block.py > ta_sp_block.inc

One block of tile i holds up to three streams, merged into one in-order instruction sequence so that a wave keeps
the matrix pipe and the vector ALU busy at the same time:

  PV   O^T += V^T(i-1) . P^T(i-1)        16 MFMAs (kb = r/4, db = r%4), A fragments by transposing LDS reads from
                                         the row-major V tile (two ds_read_b64_tr_b16 per fragment)
  S    S^T(i+1) = K(i+1) . Q^T           16 MFMAs (kk = r/2, tb = r%2), A fragments from the swizzled K tile
  SM   running softmax of S^T(i) -> P(i) about 150 vector instructions

The large operands live in fixed physical VGPRs that the compiler never sees: the kernel is compiled with
amdgpu_num_vgpr(16), which confines the register allocator to v0..v31 (the attribute counts in units of two on
this target), and everything from v32 up belongs to these blocks from the first to the last of a walk.  (The
softmax addresses single registers of the score and probability tuples, which asm operands cannot express.)

  v[48:111] O (4 x 16)   v[112:143] score buffer A   v[144:175] score buffer B   v[176:191] P   v[192:223] Q
  v[224:247] ring of 6 LDS fragments   v[248:255] softmax temporaries
  v[38:41] V fragment addresses of the current block (one per head-dim block)   v[46:47] page-lookup temporaries
  v34 v35 v37 v42 v43 further softmax temporaries
  v[32:33] lane constants: LDS offsets of the lane's V fragments and K fragments   v36 K fragment address of the
  current block

V fragments.  The V tile lies in LDS as it lies in the cache, one 256-byte row per token, with the 32-byte blocks of
a row XOR-placed by (token & 7).  ds_read_b64_tr_b16 works on groups of 16 lanes: lane j names 8 bytes (four
elements E_j[0..3]) and lane i receives E_{4k + i/4}[i % 4] for k = 0..3.  With lanes 4k..4k+3 of a group on the four
8-byte pieces of one 32-byte block of token k, lane i receives head-dim column (16 * block + i) of four tokens: the
A operand of the second product (rows = head-dim columns, contraction = tokens) without any re-layout.  The token
sets (16kb + 4hf + {0..3}, then + 8) follow the contraction slots the probabilities occupy after the first product.

Small helpers move values between the two worlds: sp_zero_o, sp_load_q, sp_set_bases, sp_scale_o, sp_mask_A/B,
sp_put_q15.

S^T(i) and S^T(i+1) alternate between buffers A and B, so every block exists in an "A current" and a "B current"
flavour.  P has one buffer: the PV MFMAs, which read P(i-1), come first in program order and the conversion that
overwrites a quarter of P is emitted only after the last MFMA reading that quarter (MFMA reads its A/B operands
when it issues).  Each MFMA consumes one 16-byte LDS fragment read issued DIST steps earlier.

Running softmax in base 2 with a lazily moved reference M (scaled units): M changes only when the tile maximum
exceeds M + 4, so P <= 16 and the rescaling of O (done by the caller when alpha != 1) is rare.  Two row sums are
kept: l of the fp32 probabilities (for the log-sum-exp) and l2 of their bf16 roundings, which are the weights the PV
product actually applies -- normalising O by l2 makes the output an exact weighted mean of V rows.  (With l alone
the output of a row that sees two or three keys is off by the rounding of their weights, up to 0.4 % of a value.)
"""
O, SA, SB, P, Q, FR, TMP = 48, 112, 144, 176, 192, 224, 248
NF = 6
DIST = NF - 1
TM_A, TM_B, T_SWAP, T_MC, T_THR, T_TK, PS0, PS1 = (TMP + i for i in range(8))
NTMP = 8

X0, X1, X2, X3, X4 = 34, 35, 37, 42, 43   # more softmax temporaries: a dependent vector instruction issues 9 clocks after
                           # its producer, an independent one after 5, so maxima and sums run as four chains
RL = 38                    # v[38:41]: the four V fragment addresses of the current block (head-dim blocks 0..3)
PT0, PT1 = 46, 47          # page lookup of the fast blocks: LDS address of the page id, the id itself
VA_BASE, KA_BASE, KADDR = 32, 33, 36   # lane constants and the K fragment address of the current block
S_CMP = 90                 # s[90:91]: lane mask of "the reference moves" (a select on an SGPR mask is a plain
                           # vector instruction; the same select on VCC costs four times as much on this chip)


def v(n):
    return "v%d" % n


def vr(n, k):
    return "v[%d:%d]" % (n, n + k - 1)


def frag(r):
    return FR + 4 * (r % NF)


def softmax_ops(sc):
    """(instruction, index of the PV MFMA that must already be issued or -1) in program order."""
    s = lambda t: v(sc + t)
    ops = []
    add = lambda ins, need=-1: ops.append((ins, need))
    mx = (TM_A, TM_B, X0, X1)                                # four chains of maxima, eight scores each
    for q in range(4):
        add("v_max_f32 %s, %s, %s" % (v(mx[q]), s(8 * q), s(8 * q + 1)))
    for j in range(1, 4):
        for q in range(4):
            add("v_max3_f32 %s, %s, %s, %s" % (v(mx[q]), v(mx[q]), s(8 * q + 2 * j), s(8 * q + 2 * j + 1)))
    add("v_max_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(TM_B)))
    add("v_max3_f32 %s, %s, %s, %s" % (v(TM_A), v(TM_A), v(X0), v(X1)))
    add("v_mov_b32 %s, %s" % (v(T_SWAP), v(TM_A)))
    add("s_nop 1")                                           # VALU write -> permlane swap read
    add("v_permlane32_swap_b32 %s, %s" % (v(TM_A), v(T_SWAP)))  # both halves of a row see both maxima
    add("s_nop 1")
    add("v_max_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(T_SWAP)))
    add("v_mul_f32 %s, %%[c], %s" % (v(T_MC), v(TM_A)))      # tile maximum in scaled units
    add("v_add_f32 %s, 4.0, %%[m]" % v(T_THR))
    add("v_cmp_gt_f32 s[%d:%d], %s, %s" % (S_CMP, S_CMP + 1, v(T_MC), v(T_THR)))
    add("s_nop 1")                                           # a lane mask written by a vector compare needs two
                                                             # wait states before a vector instruction reads it
    add("v_cndmask_b32 %s, %%[m], %s, s[%d:%d]" % (v(T_THR), v(T_MC), S_CMP, S_CMP + 1))   # new reference
    add("v_sub_f32 %%[al], %%[m], %s" % v(T_THR))
    add("v_exp_f32 %[al], %[al]")                            # alpha = 2^(M_old - M_new); 1 when unchanged
    add("v_mov_b32 %%[m], %s" % v(T_THR))
    add("v_mov_b32 %s, 0x3f803f80" % v(T_SWAP))              # bf16 (1, 1): the maxima are done with this register

    def stage_a(g):                                          # x = 2^(s*c - M) for scores 4g..4g+3, in place
        xs = [sc + 4 * g + k for k in range(4)]
        for k in range(4):
            add("v_fma_f32 %s, %s, %%[c], -%%[m]" % (v(xs[k]), s(4 * g + k)))
        for k in range(4):
            add("v_exp_f32 %s, %s" % (v(xs[k]), v(xs[k])))

    ps = (PS0, PS1, X2, X3)                                  # four chains of the row sum
    d2 = (TM_A, TM_B, X0, X1)                                # four chains of the sum of the rounded values

    def stage_b(g):                                          # row sums and the two packed P registers
        xs = [sc + 4 * g + k for k in range(4)]
        need = 4 * (g // 2) + 3                              # last PV MFMA reading P quarter g/2
        if g == 0:
            for k in range(4):
                add("v_mov_b32 %s, %s" % (v(ps[k]), v(xs[k])))
        else:
            for k in range(4):
                add("v_add_f32 %s, %s, %s" % (v(ps[k]), v(ps[k]), v(xs[k])))
        add("v_cvt_pk_bf16_f32 %s, %s, %s" % (v(P + 2 * g), v(xs[0]), v(xs[1])), need)
        add("v_cvt_pk_bf16_f32 %s, %s, %s" % (v(P + 2 * g + 1), v(xs[2]), v(xs[3])), need)
        # second row sum, of the rounded values: what the PV product really weighs V with
        for h in range(2):
            c = d2[2 * (g & 1) + h]
            add("v_dot2_f32_bf16 %s, %s, %s, %s" % (v(c), v(P + 2 * g + h), v(T_SWAP), "0" if g < 2 else v(c)), need)

    stage_a(0)
    for g in range(1, 8):
        stage_a(g)
        stage_b(g - 1)
    stage_b(7)
    add("v_add_f32 %s, %s, %s" % (v(PS0), v(PS0), v(PS1)))
    add("v_add_f32 %s, %s, %s" % (v(X2), v(X2), v(X3)))
    add("v_add_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(TM_B)))   # (the dot results are more than 3 wait states old)
    add("v_add_f32 %s, %s, %s" % (v(X0), v(X0), v(X1)))
    add("v_add_f32 %s, %s, %s" % (v(PS0), v(PS0), v(X2)))
    add("v_add_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(X0)))
    add("v_fma_f32 %%[l], %%[l], %%[al], %s" % v(PS0))
    add("v_fma_f32 %%[l2], %%[l2], %%[al], %s" % v(TM_A))
    return ops


def address_setup(has_pv, has_s):
    """Fragment addresses of this block: lane constants plus the ring slots' byte offsets (SGPR operands)."""
    out = []
    if has_pv:
        out.append("v_add_u32 %s, %%[sva], %s" % (v(RL), v(VA_BASE)))
        for db in range(1, 4):
            out.append("v_xor_b32 %s, %d, %s" % (v(RL + db), 64 * db, v(RL)))      # head-dim block db: see V tile layout
    if has_s:
        out.append("v_add_u32 %s, %%[ska], %s" % (v(KADDR), v(KA_BASE)))
    return out


def mfma_steps(has_pv, has_s, sn):
    """Per MFMA: (instructions that fetch its A fragment -- LDS reads carry a tag --, mfma line)."""
    steps = []
    if has_pv:
        for r in range(16):
            kb, db = r >> 2, r & 3
            f = frag(len(steps))
            rd = [("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(f, 2), v(RL + db), kb * 4096), True),
                  ("ds_read_b64_tr_b16 %s, %s offset:%d" % (vr(f + 2, 2), v(RL + db), kb * 4096 + 2048), True)]
            mf = "v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (vr(O + 16 * db, 16), vr(f, 4), vr(P + 4 * kb, 4),
                                                              vr(O + 16 * db, 16))
            steps.append((rd, mf))
    if has_s:
        for r in range(16):
            kk, tb = r >> 1, r & 1
            f = frag(len(steps))
            rd = []
            if tb == 0 and kk > 0:
                rd.append(("v_xor_b32 %s, %d, %s" % (v(T_TK), kk * 32, v(KADDR)), False))
            rd.append(("ds_read_b128 %s, %s offset:%d" % (vr(f, 4), v(KADDR) if kk == 0 else v(T_TK), tb * 8192), True))
            dst = vr(sn + 16 * tb, 16)
            mf = "v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (dst, vr(f, 4), vr(Q + 4 * kk, 4), "0" if kk == 0 else dst)
            steps.append((rd, mf))
    return steps


def weave(steps, aux, pre):
    """One in-order sequence: the fragment fetches run DIST MFMAs ahead, `pre` items of `aux` hide the latency of the
    first fetches, the rest of `aux` is spread evenly between the MFMAs.  An aux item with mf = k may not come before
    MFMA k (it overwrites what that MFMA reads).  Items are dicts: t (text), lds (tag of an LDS operation it starts),
    needs (tags whose data it uses)."""
    n = len(steps)
    seq = []

    def put_reads(r):
        for text, is_lds in steps[r][0]:
            seq.append(dict(t=text, lds=("f", r, len(seq)) if is_lds else None))

    def tags(r):
        return [x["lds"] for x in seq if x.get("lds") and x["lds"][:2] == ("f", r)]

    for r in range(min(DIST, n)):
        put_reads(r)
    vi = 0
    pre = min(pre, len(aux))
    while vi < pre and aux[vi].get("mf", -1) < 0:
        seq.append(aux[vi])
        vi += 1
    pre = vi
    for r in range(n):
        if r + DIST < n:
            put_reads(r + DIST)
        seq.append(dict(t=steps[r][1], needs=tags(r)))
        target = pre + (len(aux) - pre) * (r + 1) // n
        while vi < len(aux) and vi < target:
            need = aux[vi].get("mf", -1)
            if need >= 0 and need >= r and r < n - 1:
                break                                 # this P quarter is still being read
            seq.append(aux[vi])
            vi += 1
    seq += aux[vi:]
    return seq


def with_waits(seq):
    """Instruction lines of a sequence, with an exact `s_waitcnt lgkmcnt` in front of every item that uses the data of
    an LDS operation (LDS operations return in order: waiting until k younger ones are outstanding is enough)."""
    lines, issued, done = [], [], -1
    for it in seq:
        needs = it.get("needs")
        if needs:
            pos = max(issued.index(x) for x in needs)
            if pos > done:
                lines.append("s_waitcnt lgkmcnt(%d)" % (len(issued) - 1 - pos))
                done = pos
        lines.append(it["t"])
        if it.get("lds"):
            issued.append(it["lds"])
            assert len(issued) - 1 - done <= 15, "more LDS operations in flight than the counter can hold"
        if it.get("flush"):
            issued, done = [], -1
    return lines


def block(name, cur, has_pv, has_s, has_sm):
    sc, sn = (SA, SB) if cur == "A" else (SB, SA)
    steps = mfma_steps(has_pv, has_s, sn)
    ops = softmax_ops(sc) if has_sm else []
    aux = [dict(t=t, mf=need) for t, need in ops]
    seq = [dict(t="s_nop 7")] + [dict(t=t) for t in address_setup(has_pv, has_s)]
    seq += weave(steps, aux, 10 if steps else len(aux))
    lines = with_waits(seq)
    if has_pv and not has_s:
        lines += ["s_nop 15", "s_nop 7"]              # O is read by ordinary code next
    outs, ins, sig = [], [], []
    if has_pv:
        ins += ['[sva] "s"(sva)']
        sig += ["uint32_t sva"]
    if has_sm:
        outs += ['[m] "+v"(m)', '[l] "+v"(l)', '[l2] "+v"(l2)', '[al] "=&v"(alpha)']
        sig += ["float &m", "float &l", "float &l2", "float &alpha"]
        ins += ['[c] "s"(c)']
        sig += ["float c"]
    if has_s:
        ins += ['[ska] "s"(ska)']
        sig += ["uint32_t ska"]
    clob = ['"memory"', '"vcc"'] + (['"s%d"' % S_CMP, '"s%d"' % (S_CMP + 1)] if has_sm else [])
    return emit(name, sig, lines, outs, ins, clob)


# Scalar registers of the fast loop (clobbers): constants copied from the operands once, and temporaries.
S_KG, S_VG = 60, 62                     # s[60:61], s[62:63]: cache base of this KV head (K, V)
S_KSP, S_VSP, S_KSS, S_VSS = 64, 65, 66, 67      # page and slot strides in bytes
S_PSHIFT, S_PMASK, S_PCADJ, S_C = 68, 69, 70, 71  # page shift/mask, LDS address of the page-id cache, softmax scale
S_KDST, S_VDST = 72, 73                 # LDS targets of this wave's loads
ST = 80                                 # s80..s85 temporaries, s[86:87] K tile base, s[88:89] V tile base


def sg(n):
    return "s%d" % n


def fast_step_items(cur, label, helper=False):
    """One tile of the steady state as a list of items (no waits yet): the full block (PV, S, softmax) plus
    everything else the tile needs -- page lookup and addresses of tile i+3, its four cache loads, ring bookkeeping,
    the (rare) rescaling of O, and the closing barrier.
    helper=True leaves the block itself out: a wave without query rows still moves its share of the tiles."""
    sc, sn = (SA, SB) if cur == "A" else (SB, SA)
    steps = [] if helper else mfma_steps(True, True, sn)
    sm = [] if helper else [(t.replace("%[c]", sg(S_C)), need) for t, need in softmax_ops(sc)]
    page_a = [  # page id of the tile to load: LDS read now, used a few MFMAs later; slot part of the addresses
        dict(t="s_lshr_b32 %s, %%[pos], %s" % (sg(ST), sg(S_PSHIFT))),
        dict(t="s_lshl_b32 %s, %s, 2" % (sg(ST), sg(ST))),
        dict(t="s_add_u32 %s, %s, %s" % (sg(ST), sg(ST), sg(S_PCADJ))),
        dict(t="v_mov_b32 %s, %s" % (v(PT0), sg(ST))),
        dict(t="ds_read_b32 %s, %s" % (v(PT1), v(PT0)), lds=("p", 0)),
        dict(t="s_and_b32 %s, %%[pos], %s" % (sg(ST + 1), sg(S_PMASK))),
        dict(t="s_mul_i32 %s, %s, %s" % (sg(ST + 2), sg(ST + 1), sg(S_KSS))),
        dict(t="s_mul_hi_u32 %s, %s, %s" % (sg(ST + 3), sg(ST + 1), sg(S_KSS))),
        dict(t="s_mul_i32 %s, %s, %s" % (sg(ST + 4), sg(ST + 1), sg(S_VSS))),
        dict(t="s_mul_hi_u32 %s, %s, %s" % (sg(ST + 5), sg(ST + 1), sg(S_VSS))),
    ]
    page_b = [
        dict(t="v_readfirstlane_b32 %s, %s" % (sg(ST), v(PT1)), needs=[("p", 0)]),
        dict(t="s_nop 3"),
    ] + [dict(t=x) for x in [
        "s_mul_i32 s86, %s, %s" % (sg(ST), sg(S_KSP)), "s_mul_hi_u32 s87, %s, %s" % (sg(ST), sg(S_KSP)),
        "s_add_u32 s86, s86, %s" % sg(ST + 2), "s_addc_u32 s87, s87, %s" % sg(ST + 3),
        "s_add_u32 s86, s86, %s" % sg(S_KG), "s_addc_u32 s87, s87, %s" % sg(S_KG + 1),
        "s_mul_i32 s88, %s, %s" % (sg(ST), sg(S_VSP)), "s_mul_hi_u32 s89, %s, %s" % (sg(ST), sg(S_VSP)),
        "s_add_u32 s88, s88, %s" % sg(ST + 4), "s_addc_u32 s89, s89, %s" % sg(ST + 5),
        "s_add_u32 s88, s88, %s" % sg(S_VG), "s_addc_u32 s89, s89, %s" % sg(S_VG + 1),
    ]]
    dma = [["s_add_u32 m0, %s, %%[ik]" % sg(S_KDST), "s_nop 0", "global_load_lds_dwordx4 %[koff0], s[86:87] nt"],
           ["s_add_u32 m0, m0, 0x400", "s_nop 0", "global_load_lds_dwordx4 %[koff1], s[86:87] nt"],
           ["s_add_u32 m0, %s, %%[iv]" % sg(S_VDST), "s_nop 0", "global_load_lds_dwordx4 %[voff0], s[88:89] nt"],
           ["s_add_u32 m0, m0, 0x400", "s_nop 0", "global_load_lds_dwordx4 %[voff1], s[88:89] nt"]]

    def ring(reg, wrap):
        return ["s_add_u32 %s, %s, 0x4000" % (reg, reg), "s_cmp_eq_u32 %s, 0x%x" % (reg, wrap),
                "s_cselect_b32 %s, 0, %s" % (reg, reg)]
    rings = ring("%[ik]", 0xc000) + ring("%[iv]", 0x14000) + ring("%[kn]", 0xc000) + ring("%[vp]", 0x14000) + \
        ["s_add_u32 %[pos], %[pos], 64"]

    aux = list(page_a)
    aux += [dict(t=t, mf=need) for t, need in sm[:12]]
    aux += page_b
    rest = sm[12:]
    # Loads of tile i+3: late in the block, one every 10 softmax instructions from the 90th on (they are not needed
    # before the end of the next block; issued early they cost the 256-row shapes 1.4 %, spread evenly 1 %).
    di, dma_end = 0, 0
    if helper:
        for x in dma:
            aux += [dict(t=y) for y in x]
        di = 4
    for j, (t, need) in enumerate(rest):
        aux.append(dict(t=t, mf=need))
        if j >= 90 and (j - 90) % 10 == 0 and di < 4:
            aux += [dict(t=x) for x in dma[di]]
            di += 1
            dma_end = len(aux)                     # the loads read the ring positions ik and iv
    assert di == 4
    if helper:
        aux += [dict(t=x) for x in rings]
    else:
        # ring bookkeeping: behind the last load, one scalar instruction after every fourth other one (a compare and
        # the select that reads its SCC stay neighbours: other scalar work writes SCC too)
        k, i = dma_end, 0
        while i < len(rings):
            grp = rings[i:i + 2] if rings[i].startswith("s_cmp") else rings[i:i + 1]
            at = min(k, len(aux))
            for x in reversed(grp):
                aux.insert(at, dict(t=x))
            i += len(grp)
            k += 4 + len(grp)

    seq = [] if helper else [dict(t="s_nop 3")] + [dict(t=t.replace("%[sva]", "%[vp]").replace("%[ska]", "%[kn]"))
                                                   for t in address_setup(True, True)]
    seq += weave(steps, aux, 16)
    if not helper:
        # O still holds sums relative to the old reference when it moved (rare): rescale, then close the tile
        seq += [dict(t="v_cmp_neq_f32 vcc, 1.0, %[al]"), dict(t="s_cbranch_vccz %df" % label), dict(t="s_nop 15"),
                dict(t="s_nop 7")]
        seq += [dict(t="v_mul_f32 %s, %%[al], %s" % (v(O + k), v(O + k))) for k in range(64)]
        seq += [dict(t="s_nop 3"), dict(t="%d:" % label)]
    seq += [dict(t="s_waitcnt vmcnt(4)"), dict(t="s_waitcnt lgkmcnt(0)", flush=True), dict(t="s_barrier")]
    return seq


def fast_loop(name, helper=False):
    """`cnt` pairs of steady-state tiles (buffer A current, then buffer B) as one asm statement with its own loop,
    so that the scalar bookkeeping of a tile is issued in the shadow of its matrix and vector work.
    Ring positions (byte offsets): ik, iv = slots the next loads go to; kn = K slot of tile i+1; vp = V slot of
    tile i-1."""
    head = ["s_mov_b64 s[%d:%d], %%[kg]" % (S_KG, S_KG + 1), "s_mov_b64 s[%d:%d], %%[vg]" % (S_VG, S_VG + 1),
            "s_mov_b64 s[%d:%d], %%[sp]" % (S_KSP, S_VSP), "s_mov_b64 s[%d:%d], %%[ss]" % (S_KSS, S_VSS),
            "s_mov_b64 s[%d:%d], %%[pp]" % (S_PSHIFT, S_PMASK), "s_mov_b64 s[%d:%d], %%[pc]" % (S_PCADJ, S_C),
            "s_mov_b64 s[%d:%d], %%[dst]" % (S_KDST, S_VDST), "1:"]
    seq = [dict(t=t) for t in head] + fast_step_items("A", 2, helper) + fast_step_items("B", 3, helper)
    seq += [dict(t="s_sub_u32 %[cnt], %[cnt], 1"), dict(t="s_cmp_lg_u32 %[cnt], 0"), dict(t="s_cbranch_scc1 1b")]
    lines = with_waits(seq)
    sig = ([] if helper else ["float &m", "float &l", "float &l2"]) + ["uint32_t &ik", "uint32_t &iv", "uint32_t &kn", "uint32_t &vp",
           "uint32_t &pos", "uint32_t &cnt", "uint64_t kg", "uint64_t vg", "uint64_t sp", "uint64_t ss", "uint64_t pp",
           "uint64_t pc", "uint64_t dst", "uint32_t koff0", "uint32_t koff1", "uint32_t voff0", "uint32_t voff1"]
    outs = ([] if helper else ['[m] "+v"(m)', '[l] "+v"(l)', '[l2] "+v"(l2)', '[al] "=&v"(alpha)']) + \
           ['[%s] "+s"(%s)' % (x, x) for x in ("ik", "iv", "kn", "vp", "pos", "cnt")]
    ins = ['[%s] "s"(%s)' % (x, x) for x in ("kg", "vg", "sp", "ss", "pp", "pc", "dst")] + \
          ['[%s] "v"(%s)' % (x, x) for x in ("koff0", "koff1", "voff0", "voff1")]
    clob = ['"memory"', '"vcc"', '"scc"'] + ['"s%d"' % i for i in list(range(60, 74)) + list(range(80, 92))]
    return emit(name, sig, lines, outs, ins, clob, pre=None if helper else "    float alpha;")


def emit(name, sig, lines, outs, ins, clob, pre=None):
    code = ["__device__ __forceinline__ void %s(%s)" % (name, ", ".join(sig)), "{"] + ([pre] if pre else []) + ["    asm volatile("]
    for ln in lines:
        code.append('        "%s\\n\\t"' % ln)
    code.append("        : " + ", ".join(outs))
    code.append("        : " + ", ".join(ins))
    code.append("        : " + ", ".join(clob) + ");")
    code.append("}")
    return "\n".join(code)


def helpers():
    out = []
    # O = 0.  Naming v255 as clobbered makes the compiler size the kernel's register file for all 256 VGPRs.
    out.append(emit("sp_zero_o", [], ["v_mov_b32 %s, 0" % v(O + k) for k in range(64)], [], [], ['"memory"', '"v255"']))
    # Q of the lane's row straight from global memory into its registers: eight 16-byte pieces, 32 bytes apart.
    # Nothing waits here; the caller's next wait on the vector-memory counter covers these loads.
    lines = ["global_load_dwordx4 %s, %%[qp], off offset:%d" % (vr(Q + 4 * k, 4), 32 * k) for k in range(8)]
    out.append(emit("sp_load_q", ["const void *qp"], lines, [], ['[qp] "v"(qp)'], ['"memory"']))
    out.append(emit("sp_set_bases", ["uint32_t va", "uint32_t ka"],
                    ["v_mov_b32 %s, %%%d" % (v(r), k) for k, r in enumerate((VA_BASE, KA_BASE))], [],
                    ['"v"(va)', '"v"(ka)'], ['"memory"']))
    lines = ["s_nop 15", "s_nop 7"] + ["v_mul_f32 %s, %%[al], %s" % (v(O + k), v(O + k)) for k in range(64)] + ["s_nop 3"]
    out.append(emit("sp_scale_o", ["float alpha"], lines, [], ['[al] "v"(alpha)'], ['"memory"']))
    for cur, base in (("A", SA), ("B", SB)):
        lines = ["s_nop 15", "s_nop 7", "v_mov_b32 %s, 0xff800000" % v(TMP)]
        for tb in range(2):
            for i in range(16):
                bit = 8 * (i // 4) + (i % 4)
                lines.append("v_and_b32 %s, 0x%x, %%[%s]" % (v(TMP + 1), 1 << bit, "lo" if tb == 0 else "hi"))
                lines.append("v_cmp_eq_u32 vcc, 0, %s" % v(TMP + 1))
                lines.append("v_cndmask_b32 %s, %s, %s, vcc" % (v(base + 16 * tb + i), v(base + 16 * tb + i), v(TMP)))
        out.append(emit("sp_mask_" + cur, ["uint32_t lo", "uint32_t hi"], lines, [], ['[lo] "v"(lo)', '[hi] "v"(hi)'],
                        ['"memory"', '"vcc"']))
    # Epilogue: the lane's 64 values of O (its half of a query row) become 16-bit fixed point with one scale for the
    # row -- value = scale * int16, scale = inv * (largest magnitude of the row) / 32767 -- and go to the row-major
    # staging block in LDS, 256 bytes per row: the lane's piece c (four values, 8 bytes) lives at byte address
    # a0 ^ (c << 4) (the caller folds row, lane half and chunk swizzle into a0).  The rounding to int16 is the
    # "add 1.5 * 2^23" trick: the low 16 bits of the sum are the rounded value in two's complement.
    # scale comes back NaN when the row holds a NaN (the sum of its values is one then).
    T0, T1, T2, T3, AM, SU, XS = (TMP + i for i in range(7))
    lines = ["s_nop 15", "s_nop 7"]
    lines += ["v_max3_f32 %s, |%s|, |%s|, |%s|" % (v(AM), v(O), v(O + 1), v(O + 2)),
              "v_max3_f32 %s, |%s|, |%s|, |%s|" % (v(T0), v(O + 3), v(O + 4), v(O + 5)),
              "v_add_f32 %s, %s, %s" % (v(SU), v(O), v(O + 1)), "v_add_f32 %s, %s, %s" % (v(T1), v(O + 2), v(O + 3))]
    for k in range(6, 64, 4):                                # two chains of maxima, two chains of sums
        lines.append("v_max3_f32 %s, %s, |%s|, |%s|" % (v(AM), v(AM), v(O + k), v(O + k + 1)))
        if k + 3 < 64:
            lines.append("v_max3_f32 %s, %s, |%s|, |%s|" % (v(T0), v(T0), v(O + k + 2), v(O + k + 3)))
    for k in range(4, 64, 2):
        lines.append("v_add_f32 %s, %s, %s" % (v(SU) if (k // 2) % 2 == 0 else v(T1), v(SU) if (k // 2) % 2 == 0 else v(T1), v(O + k)))
        lines.append("v_add_f32 %s, %s, %s" % (v(T1) if (k // 2) % 2 == 0 else v(SU), v(T1) if (k // 2) % 2 == 0 else v(SU), v(O + k + 1)))
    lines += ["v_max_f32 %s, %s, %s" % (v(AM), v(AM), v(T0)), "v_add_f32 %s, %s, %s" % (v(SU), v(SU), v(T1)),
              "v_mov_b32 %s, %s" % (v(XS), v(AM)), "s_nop 1", "v_permlane32_swap_b32 %s, %s" % (v(AM), v(XS)), "s_nop 1",
              "v_max_f32 %s, %s, %s" % (v(AM), v(AM), v(XS)),             # both halves of a row see the row's maximum
              "v_mov_b32 %s, %s" % (v(XS), v(SU)), "s_nop 1", "v_permlane32_swap_b32 %s, %s" % (v(SU), v(XS)), "s_nop 1",
              "v_add_f32 %s, %s, %s" % (v(SU), v(SU), v(XS)),
              "v_mul_f32 %s, %%[inv], %s" % (v(T0), v(AM)),
              "v_mul_f32 %%[sc], 0x38000100, %s" % v(T0),                   # * 1/32767
              "v_cmp_u_f32 vcc, %s, %s" % (v(SU), v(SU)),
              "v_mov_b32 %s, 0x7fc00000" % v(T1),
              "v_cndmask_b32 %%[sc], %%[sc], %s, vcc" % v(T1),
              "v_rcp_f32 %s, %s" % (v(T2), v(AM)),
              "v_cmp_gt_f32 vcc, %s, 0" % v(AM),
              "s_nop 0",
              "v_mul_f32 %s, 0x46fffe00, %s" % (v(T2), v(T2)),              # 32767 / max
              "v_cndmask_b32 %s, 0, %s, vcc" % (v(AM), v(T2)),               # an all-zero row: every value stays 0
              "v_mov_b32 %s, 0x4b400000" % v(SU),                            # 1.5 * 2^23
              "v_mov_b32 %s, 0x05040100" % v(XS)]                            # byte selector: low halves of two registers
    for c in range(16):
        for j in range(4):
            lines.append("v_fma_f32 %s, %s, %s, %s" % (v(T0 + j), v(O + 4 * c + j), v(AM), v(SU)))
        lines.append("v_perm_b32 %s, %s, %s, %s" % (v(O + 2 * c), v(T1), v(T0), v(XS)))
        lines.append("v_perm_b32 %s, %s, %s, %s" % (v(O + 2 * c + 1), v(T3), v(T2), v(XS)))
        lines.append("v_xor_b32 %s, 0x%x, %%[a0]" % (v(T0), c << 4))
        lines.append("ds_write_b64 %s, v[%d:%d]" % (v(T0), O + 2 * c, O + 2 * c + 1))
    lines.append("s_waitcnt lgkmcnt(0)")
    out.append(emit("sp_put_q15", ["float inv", "uint32_t a0", "float &sc"], lines, ['[sc] "=&v"(sc)'],
                    ['[inv] "v"(inv)', '[a0] "v"(a0)'], ['"memory"', '"vcc"']))
    return "\n\n".join(out)


def generate():
    """The whole text of ta_sp_block.inc."""
    import contextlib
    import io
    buf = io.StringIO()
    with contextlib.redirect_stdout(buf):
        print("// Generated by gen_sp_block.py -- do not edit.")
        print(block("sp_s_first", "B", False, True, False))          # S^T(0) into buffer A ("current" B is unused)
        for cur in "AB":
            print()
            print(block("sp_full_" + cur, cur, True, True, True))
            print()
            print(block("sp_last_" + cur, cur, True, False, True))    # no tile after this one
        print()
        print(block("sp_head_A", "A", False, True, True))            # tile 0 when a tile 1 follows
        print()
        print(block("sp_only_A", "A", False, False, True))           # tile 0 of a one-tile walk
        print()
        print(block("sp_pv", "A", True, False, False))               # drain: the last tile's P . V
        print()
        print(fast_loop("sp_fast_loop"))
        print()
        print(fast_loop("sp_fast_loop_helper", helper=True))
        print()
        print(helpers())

    return buf.getvalue()


if __name__ == "__main__":
    import sys
    sys.stdout.write(generate())
