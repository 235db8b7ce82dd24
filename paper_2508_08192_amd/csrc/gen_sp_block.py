#!/usr/bin/env python3
"""Writes ta_sp_block.inc: the per-tile blocks of the 256-row KV-pass kernel as single inline-asm statements.

    python gen_sp_block.py > ta_sp_block.inc

One block of tile i holds up to three streams, merged into one in-order instruction sequence so that a wave keeps
the matrix pipe and the vector ALU busy at the same time:

  PV   O^T += V^T(i-1) . P^T(i-1)        16 MFMAs (kb = r/4, db = r%4), A fragments from the token-minor V tile
  S    S^T(i+1) = K(i+1) . Q^T           16 MFMAs (kk = r/2, tb = r%2), A fragments from the swizzled K tile
  SM   running softmax of S^T(i) -> P(i) about 140 vector instructions

The large operands live in fixed physical VGPRs that the compiler never sees: the kernel is compiled with
amdgpu_num_vgpr(16), which confines the register allocator to v0..v31 (the attribute counts in units of two on
this target), and everything from v32 up belongs to these blocks from the first to the last of a walk.  (The
softmax addresses single registers of the score and probability tuples, which asm operands cannot express.)

  v[48:111] O (4 x 16)   v[112:143] score buffer A   v[144:175] score buffer B   v[176:191] P   v[192:223] Q
  v[224:247] ring of 6 LDS fragments   v[248:255] softmax temporaries   v[38:47] re-layout temporaries
  v[32:35] lane constants: LDS offsets of the lane's V fragments, K fragments, re-layout reads and writes
  v[36:37] K fragment address and re-layout write address of the current block

Small helpers move values between the two worlds: sp_zero_o, sp_load_q, sp_set_bases, sp_get_rl, sp_scale_o,
sp_mask_A/B, sp_put_o.

S^T(i) and S^T(i+1) alternate between buffers A and B, so every block exists in an "A current" and a "B current"
flavour.  P has one buffer: the PV MFMAs, which read P(i-1), come first in program order and the conversion that
overwrites a quarter of P is emitted only after the last MFMA reading that quarter (MFMA reads its A/B operands
when it issues).  Each MFMA consumes one 16-byte LDS fragment read issued DIST steps earlier.

Running softmax in base 2 with a lazily moved reference M (scaled units): M changes only when the tile maximum
exceeds M + 4, so P <= 16 and the rescaling of O (done by the caller when alpha != 1) is rare.  Two row sums are
kept: l of the fp32 probabilities (for the log-sum-exp) and l2 of their bf16 roundings, which are the weights the PV
product actually applies -- normalising O by l2 makes the output an exact weighted mean of V rows.
"""
O, SA, SB, P, Q, FR, TMP = 48, 112, 144, 176, 192, 224, 248
NF = 6
DIST = NF - 1
TM_A, TM_B, T_SWAP, T_MC, T_THR, T_TK, PS0, PS1 = (TMP + i for i in range(8))
NTMP = 8


RL = 38                    # v[38:47]: re-layout temporaries of the fast blocks (four 8-byte rows, two outputs);
                           # v[38:41] double as the four V fragment addresses while the PV reads are being issued
VA_BASE, KA_BASE, RD_BASE, WR_BASE, KADDR, WRT = 32, 33, 34, 35, 36, 37   # lane constants and per-block addresses



def v(n):
    return "v%d" % n


def vr(n, k):
    return "v[%d:%d]" % (n, n + k - 1)


def frag(r):
    return vr(FR + 4 * (r % NF), 4)


def softmax_ops(sc):
    """(instruction, index of the PV MFMA that must already be issued or -1) in program order."""
    s = lambda t: v(sc + t)
    ops = []
    add = lambda ins, need=-1: ops.append((ins, need))
    add("v_max_f32 %s, %s, %s" % (v(TM_A), s(0), s(1)))
    add("v_max_f32 %s, %s, %s" % (v(TM_B), s(16), s(17)))
    for j in range(1, 8):
        add("v_max3_f32 %s, %s, %s, %s" % (v(TM_A), v(TM_A), s(2 * j), s(2 * j + 1)))
        add("v_max3_f32 %s, %s, %s, %s" % (v(TM_B), v(TM_B), s(16 + 2 * j), s(17 + 2 * j)))
    add("v_max_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(TM_B)))
    add("v_mov_b32 %s, %s" % (v(T_SWAP), v(TM_A)))
    add("s_nop 1")                                           # VALU write -> permlane swap read
    add("v_permlane32_swap_b32 %s, %s" % (v(TM_A), v(T_SWAP)))  # both halves of a row see both maxima
    add("s_nop 1")
    add("v_max_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(T_SWAP)))
    add("v_mul_f32 %s, %%[c], %s" % (v(T_MC), v(TM_A)))      # tile maximum in scaled units
    add("v_add_f32 %s, 4.0, %%[m]" % v(T_THR))
    add("v_cmp_gt_f32 vcc, %s, %s" % (v(T_MC), v(T_THR)))
    add("v_cndmask_b32 %s, %%[m], %s, vcc" % (v(T_THR), v(T_MC)))   # new reference
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

    def stage_b(g):                                          # row sum (unrounded) and the two packed P registers
        xs = [sc + 4 * g + k for k in range(4)]
        need = 4 * (g // 2) + 3                              # last PV MFMA reading P quarter g/2
        if g == 0:
            add("v_add_f32 %s, %s, %s" % (v(PS0), v(xs[0]), v(xs[1])))
            add("v_add_f32 %s, %s, %s" % (v(PS1), v(xs[2]), v(xs[3])))
        else:
            add("v_add_f32 %s, %s, %s" % (v(PS0), v(PS0), v(xs[0])))
            add("v_add_f32 %s, %s, %s" % (v(PS1), v(PS1), v(xs[1])))
            add("v_add_f32 %s, %s, %s" % (v(PS0), v(PS0), v(xs[2])))
            add("v_add_f32 %s, %s, %s" % (v(PS1), v(PS1), v(xs[3])))
        add("v_cvt_pk_bf16_f32 %s, %s, %s" % (v(P + 2 * g), v(xs[0]), v(xs[1])), need)
        add("v_cvt_pk_bf16_f32 %s, %s, %s" % (v(P + 2 * g + 1), v(xs[2]), v(xs[3])), need)
        # second row sum, of the rounded values: what the PV product really weighs V with
        add("v_dot2_f32_bf16 %s, %s, %s, %s" % (v(TM_A), v(P + 2 * g), v(T_SWAP), "0" if g == 0 else v(TM_A)), need)
        add("v_dot2_f32_bf16 %s, %s, %s, %s" % (v(TM_B), v(P + 2 * g + 1), v(T_SWAP), "0" if g == 0 else v(TM_B)), need)

    stage_a(0)
    for g in range(1, 8):
        stage_a(g)
        stage_b(g - 1)
    stage_b(7)
    add("v_add_f32 %s, %s, %s" % (v(PS0), v(PS0), v(PS1)))
    add("v_fma_f32 %%[l], %%[l], %%[al], %s" % v(PS0))
    add("s_nop 1")                                           # a dot result needs 3 wait states before another VALU reads it
    add("v_add_f32 %s, %s, %s" % (v(TM_A), v(TM_A), v(TM_B)))
    add("v_fma_f32 %%[l2], %%[l2], %%[al], %s" % v(TM_A))
    return ops


def address_setup(has_pv, has_s):
    """Fragment addresses of this block: lane constants plus the ring slots' byte offsets (SGPR operands)."""
    out = []
    if has_pv:
        out.append("v_add_u32 %s, %%[sva], %s" % (v(RL), v(VA_BASE)))
        for db in range(1, 4):
            out.append("v_xor_b32 %s, %d, %s" % (v(RL + db), 32 * db, v(RL)))      # head-dim block db: see V tile layout
    if has_s:
        out.append("v_add_u32 %s, %%[ska], %s" % (v(KADDR), v(KA_BASE)))
    return out


def mfma_steps(has_pv, has_s, sn):
    """Per MFMA: (LDS read lines, mfma line, is_pv)."""
    steps = []
    if has_pv:
        for r in range(16):
            kb, db = r >> 2, r & 3
            rd = ["ds_read_b128 {f}, %s offset:%d" % (v(RL + db), kb * 4096 + 512 * db)]
            mf = "v_mfma_f32_32x32x16_bf16 %s, {f}, %s, %s" % (vr(O + 16 * db, 16), vr(P + 4 * kb, 4), vr(O + 16 * db, 16))
            steps.append((rd, mf, True))
    if has_s:
        for r in range(16):
            kk, tb = r >> 1, r & 1
            rd = []
            if tb == 0 and kk > 0:
                rd.append("v_xor_b32 %s, %d, %s" % (v(T_TK), kk * 32, v(KADDR)))
            rd.append("ds_read_b128 {f}, %s offset:%d" % (v(KADDR) if kk == 0 else v(T_TK), tb * 8192))
            dst = vr(sn + 16 * tb, 16)
            mf = "v_mfma_f32_32x32x16_bf16 %s, {f}, %s, %s" % (dst, vr(Q + 4 * kk, 4), "0" if kk == 0 else dst)
            steps.append((rd, mf, False))
    return steps


def block(name, cur, has_pv, has_s, has_sm):
    sc, sn = (SA, SB) if cur == "A" else (SB, SA)
    steps = mfma_steps(has_pv, has_s, sn)
    ops = softmax_ops(sc) if has_sm else []
    n = len(steps)
    lines = ["s_nop 7"] + address_setup(has_pv, has_s)
    reads = lambda r: [x.replace("{f}", frag(r)) for x in steps[r][0]]
    for r in range(min(DIST, n)):
        lines += reads(r)
    vi = 0
    pre = 10 if n else len(ops)                      # vector work that hides the latency of the first fragments
    while vi < min(pre, len(ops)) and ops[vi][1] < 0:
        lines.append(ops[vi][0])
        vi += 1
    n_pv = 16 if has_pv else 0
    for r in range(n):
        if r + DIST < n:
            lines += reads(r + DIST)
        lines.append("s_waitcnt lgkmcnt(%d)" % min(DIST, n - 1 - r))
        lines.append(steps[r][1].replace("{f}", frag(r)))
        target = pre + (len(ops) - pre) * (r + 1) // n
        while vi < len(ops) and vi < target:
            need = ops[vi][1]
            if has_pv and need >= 0 and need >= r and r < n - 1:
                break                                 # this P quarter is still being read
            lines.append(ops[vi][0])
            vi += 1
    while vi < len(ops):
        lines.append(ops[vi][0])
        vi += 1
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
    return emit(name, sig, lines, outs, ins, ['"memory"', '"vcc"'])


# Scalar registers of the fast loop (clobbers): constants copied from the operands once, and temporaries.
S_KG, S_VG = 60, 62                     # s[60:61], s[62:63]: cache base of this KV head (K, V)
S_KSP, S_VSP, S_KSS, S_VSS = 64, 65, 66, 67      # page and slot strides in bytes
S_PSHIFT, S_PMASK, S_PCADJ, S_C = 68, 69, 70, 71  # page shift/mask, LDS address of the page-id cache, softmax scale
S_KDST, S_VDST, S_LO, S_HI = 72, 73, 74, 75       # LDS targets of this wave's loads; v_perm selectors
ST = 80                                 # s80..s85 temporaries, s[86:87] K tile base, s[88:89] V tile base


def sg(n):
    return "s%d" % n


def fast_step_items(cur, label, helper=False):
    """One tile of the steady state as a list of instructions (no waits yet): the full block (PV, S, softmax)
    plus everything else the tile needs -- page lookup and addresses of tile i+3, its four cache loads, the
    in-place re-layout of V(i), ring bookkeeping, the (rare) rescaling of O, and the closing barrier.
    helper=True leaves the block itself out: a wave without query rows still moves its share of the tiles."""
    sc, sn = (SA, SB) if cur == "A" else (SB, SA)
    steps = [] if helper else mfma_steps(True, True, sn)
    n = len(steps)
    sm = [] if helper else [(t.replace("%[c]", sg(S_C)), need) for t, need in softmax_ops(sc)]
    rx = lambda k: RL + 2 * k          # row k, columns 0..1 (dword x)
    ry = lambda k: RL + 2 * k + 1      # row k, columns 2..3 (dword y)
    t0, t1 = RL + 8, RL + 9
    page_a = [  # page id of the tile to load: LDS read now, used a few MFMAs later; slot part of the addresses
        "s_lshr_b32 %s, %%[pos], %s" % (sg(ST), sg(S_PSHIFT)),
        "s_lshl_b32 %s, %s, 2" % (sg(ST), sg(ST)),
        "s_add_u32 %s, %s, %s" % (sg(ST), sg(ST), sg(S_PCADJ)),
        "v_mov_b32 %s, %s" % (v(t0), sg(ST)),
        ("ds_read_b32 %s, %s" % (v(t1), v(t0)), ("p", 0)),
        "s_and_b32 %s, %%[pos], %s" % (sg(ST + 1), sg(S_PMASK)),
        "s_mul_i32 %s, %s, %s" % (sg(ST + 2), sg(ST + 1), sg(S_KSS)),
        "s_mul_hi_u32 %s, %s, %s" % (sg(ST + 3), sg(ST + 1), sg(S_KSS)),
        "s_mul_i32 %s, %s, %s" % (sg(ST + 4), sg(ST + 1), sg(S_VSS)),
        "s_mul_hi_u32 %s, %s, %s" % (sg(ST + 5), sg(ST + 1), sg(S_VSS)),
    ]
    page_b = [
        ("v_readfirstlane_b32 %s, %s" % (sg(ST), v(t1)), None, [("p", 0)]),
        "s_nop 3",
        "s_mul_i32 s86, %s, %s" % (sg(ST), sg(S_KSP)), "s_mul_hi_u32 s87, %s, %s" % (sg(ST), sg(S_KSP)),
        "s_add_u32 s86, s86, %s" % sg(ST + 2), "s_addc_u32 s87, s87, %s" % sg(ST + 3),
        "s_add_u32 s86, s86, %s" % sg(S_KG), "s_addc_u32 s87, s87, %s" % sg(S_KG + 1),
        "s_mul_i32 s88, %s, %s" % (sg(ST), sg(S_VSP)), "s_mul_hi_u32 s89, %s, %s" % (sg(ST), sg(S_VSP)),
        "s_add_u32 s88, s88, %s" % sg(ST + 4), "s_addc_u32 s89, s89, %s" % sg(ST + 5),
        "s_add_u32 s88, s88, %s" % sg(S_VG), "s_addc_u32 s89, s89, %s" % sg(S_VG + 1),
    ]
    dma = [["s_add_u32 m0, %s, %%[ik]" % sg(S_KDST), "s_nop 0", "global_load_lds_dwordx4 %[koff0], s[86:87] nt"],
           ["s_add_u32 m0, m0, 0x400", "s_nop 0", "global_load_lds_dwordx4 %[koff1], s[86:87] nt"],
           ["s_add_u32 m0, %s, %%[iv]" % sg(S_VDST), "s_nop 0", "global_load_lds_dwordx4 %[voff0], s[88:89] nt"],
           ["s_add_u32 m0, m0, 0x400", "s_nop 0", "global_load_lds_dwordx4 %[voff1], s[88:89] nt"]]
    def ring(reg, wrap):
        return ["s_add_u32 %s, %s, 0x4000" % (reg, reg), "s_cmp_eq_u32 %s, 0x%x" % (reg, wrap),
                "s_cselect_b32 %s, 0, %s" % (reg, reg)]
    rings = ring("%[ik]", 0xc000) + ring("%[iv]", 0x14000) + ring("%[kn]", 0xc000) + ["s_mov_b32 %[vp], %[vc]"] + \
            ring("%[vc]", 0x14000) + ["s_add_u32 %[pos], %[pos], 64"]

    def item(x, mf=-1):
        if isinstance(x, tuple):
            d = dict(t=x[0], mf=mf)
            if x[1]:
                d["lds"] = x[1]
            if len(x) > 2:
                d["needs"] = x[2]
            return d
        return dict(t=x, mf=mf)

    aux = [item(x) for x in page_a]
    for t, need in sm[:12]:
        aux.append(dict(t=t, mf=need))
    aux += [item(x) for x in page_b]
    rl_reads = [dict(t="v_add_u32 %s, %%[vc], %s" % (v(t1), v(RD_BASE))),
                dict(t="v_add_u32 %s, %%[vc], %s" % (v(WRT), v(WR_BASE)))]
    for k in range(4):
        rl_reads.append(dict(t="ds_read_b64 %s, %s offset:%d" % (vr(rx(k), 2), v(t1), 256 * k), lds=("r", k)))
    slo, shi = sg(S_LO), sg(S_HI)
    relay = [
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(t0), v(rx(1)), v(rx(0)), slo), needs=[("r", 0), ("r", 1)]),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(t1), v(rx(3)), v(rx(2)), slo), needs=[("r", 2), ("r", 3)]),
        dict(t="ds_write2_b32 %s, %s, %s offset1:1" % (v(WRT), v(t0), v(t1)), lds=("w", 0)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(rx(0)), v(rx(1)), v(rx(0)), shi)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(rx(2)), v(rx(3)), v(rx(2)), shi)),
        dict(t="v_xor_b32 %s, 16, %s" % (v(rx(1)), v(WRT))),
        dict(t="ds_write2_b32 %s, %s, %s offset1:1" % (v(rx(1)), v(rx(0)), v(rx(2))), lds=("w", 1)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(t0), v(ry(1)), v(ry(0)), slo)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(t1), v(ry(3)), v(ry(2)), slo)),
        dict(t="v_xor_b32 %s, 32, %s" % (v(rx(3)), v(WRT))),
        dict(t="ds_write2_b32 %s, %s, %s offset1:1" % (v(rx(3)), v(t0), v(t1)), lds=("w", 2)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(ry(0)), v(ry(1)), v(ry(0)), shi)),
        dict(t="v_perm_b32 %s, %s, %s, %s" % (v(ry(2)), v(ry(3)), v(ry(2)), shi)),
        dict(t="v_xor_b32 %s, 48, %s" % (v(ry(1)), v(WRT))),
        dict(t="ds_write2_b32 %s, %s, %s offset1:1" % (v(ry(1)), v(ry(0)), v(ry(2))), lds=("w", 3)),
    ]
    rest = sm[12:]
    # Loads of tile i+3: late in the block, one every 10 softmax instructions from the 90th on (they are not needed
    # before the end of the next block; issued early they cost the 256-row shapes 1.4 %, spread evenly 1 %).  The
    # re-layout shares v[38:47] with the V fragment addresses and the page lookup, so it starts once the last PV read
    # is out (MFMA 11).
    ri, started, di, ring_at, dma_end = 0, False, 0, 0, 0
    if helper:
        for x in dma:
            aux += [dict(t=y) for y in x]
        aux += rl_reads
        started, di = True, 4
    for j, (t, need) in enumerate(rest):
        aux.append(dict(t=t, mf=need))
        if j >= 90 and (j - 90) % 10 == 0 and di < 4:
            aux += [dict(t=x) for x in dma[di]]
            di += 1
            dma_end = len(aux)                     # the loads read the ring positions ik and iv
        if j >= 50 and not started:
            for it in rl_reads:
                aux.append(dict(it, mf=11))
            started = True
            ring_at = len(aux) + 24                # ring bookkeeping: after the last use of every ring position
        elif started and (j - 50) % 4 == 0 and ri < len(relay):
            aux.append(dict(relay[ri], mf=11))
            ri += 1
    assert started and di == 4
    for it in relay[ri:]:
        aux.append(dict(it, mf=11))
    if helper:
        aux += [dict(t=x) for x in rings]
    else:
        # spread through the second half of the block, one scalar instruction after every fourth other one
        # (a compare and the select that reads its SCC stay neighbours: other scalar work writes SCC too)
        k, i = max(ring_at, dma_end), 0
        while i < len(rings):
            grp = rings[i:i + 2] if rings[i].startswith("s_cmp") else rings[i:i + 1]
            at = min(k, len(aux))
            for x in reversed(grp):
                aux.insert(at, dict(t=x))
            i += len(grp)
            k += 4 + len(grp)

    seq = [] if helper else [dict(t="s_nop 3")] + [dict(t=t.replace("%[sva]", "%[vp]").replace("%[ska]", "%[kn]"))
                                                   for t in address_setup(True, True)]
    def put_reads(r):
        for x in steps[r][0]:
            seq.append(dict(t=x.replace("{f}", frag(r)), lds=("f", r) if x.startswith("ds_read") else None))
    for r in range(min(DIST, n)):
        put_reads(r)
    vi = 0
    pre = min(16, len(aux))
    while vi < pre:
        seq.append(aux[vi])
        vi += 1
    for r in range(n):
        if r + DIST < n:
            put_reads(r + DIST)
        seq.append(dict(t=steps[r][1].replace("{f}", frag(r)), needs=[("f", r)]))
        target = pre + (len(aux) - pre) * (r + 1) // n
        while vi < len(aux) and vi < target:
            need = aux[vi].get("mf", -1)
            if need >= 0 and need >= r and r < n - 1:
                break
            seq.append(aux[vi])
            vi += 1
    seq += aux[vi:]
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
    so that the scalar bookkeeping of a tile is issued in the shadow of its matrix and vector work."""
    head = ["s_mov_b64 s[%d:%d], %%[kg]" % (S_KG, S_KG + 1), "s_mov_b64 s[%d:%d], %%[vg]" % (S_VG, S_VG + 1),
            "s_mov_b64 s[%d:%d], %%[sp]" % (S_KSP, S_VSP), "s_mov_b64 s[%d:%d], %%[ss]" % (S_KSS, S_VSS),
            "s_mov_b64 s[%d:%d], %%[pp]" % (S_PSHIFT, S_PMASK), "s_mov_b64 s[%d:%d], %%[pc]" % (S_PCADJ, S_C),
            "s_mov_b64 s[%d:%d], %%[dst]" % (S_KDST, S_VDST), "s_mov_b32 %s, 0x05040100" % sg(S_LO),
            "s_mov_b32 %s, 0x07060302" % sg(S_HI), "1:"]
    seq = [dict(t=t) for t in head] + fast_step_items("A", 2, helper) + fast_step_items("B", 3, helper)
    seq += [dict(t="s_sub_u32 %[cnt], %[cnt], 1"), dict(t="s_cmp_lg_u32 %[cnt], 0"), dict(t="s_cbranch_scc1 1b")]
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
        if it.get("flush"):
            issued, done = [], -1
    sig = ([] if helper else ["float &m", "float &l", "float &l2"]) + ["uint32_t &ik", "uint32_t &iv", "uint32_t &kn", "uint32_t &vp", "uint32_t &vc",
           "uint32_t &pos", "uint32_t &cnt", "uint64_t kg", "uint64_t vg", "uint64_t sp", "uint64_t ss", "uint64_t pp",
           "uint64_t pc", "uint64_t dst", "uint32_t koff0", "uint32_t koff1", "uint32_t voff0", "uint32_t voff1"]
    outs = ([] if helper else ['[m] "+v"(m)', '[l] "+v"(l)', '[l2] "+v"(l2)', '[al] "=&v"(alpha)']) + \
           ['[%s] "+s"(%s)' % (x, x) for x in ("ik", "iv", "kn", "vp", "vc", "pos", "cnt")]
    ins = ['[%s] "s"(%s)' % (x, x) for x in ("kg", "vg", "sp", "ss", "pp", "pc", "dst")] + \
          ['[%s] "v"(%s)' % (x, x) for x in ("koff0", "koff1", "voff0", "voff1")]
    clob = ['"memory"', '"vcc"', '"scc"'] + ['"s%d"' % i for i in list(range(60, 76)) + list(range(80, 90))]
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
    out.append(emit("sp_set_bases", ["uint32_t va", "uint32_t ka", "uint32_t rd", "uint32_t wr"],
                    ["v_mov_b32 %s, %%%d" % (v(r), k) for k, r in enumerate((VA_BASE, KA_BASE, RD_BASE, WR_BASE))], [],
                    ['"v"(va)', '"v"(ka)', '"v"(rd)', '"v"(wr)'], ['"memory"']))
    out.append(emit("sp_get_rl", ["uint32_t &rd", "uint32_t &wr"],
                    ["v_mov_b32 %%0, %s" % v(RD_BASE), "v_mov_b32 %%1, %s" % v(WR_BASE)], ['"=v"(rd)', '"=v"(wr)'], [],
                    ['"memory"']))
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
    # Epilogue: O *= inv in place, then each lane's sixteen 16-byte pieces go to the row-major staging block in LDS;
    # piece c of the lane lives at byte address a0 ^ (c << 5) (the caller folds the row, the lane half and the
    # chunk swizzle into a0).
    lines = ["s_nop 15", "s_nop 7"] + ["v_mul_f32 %s, %%[inv], %s" % (v(O + k), v(O + k)) for k in range(64)]
    for c in range(16):
        t = v(TMP + (c & 3))
        lines.append("v_xor_b32 %s, 0x%x, %%[a0]" % (t, c << 5))
        lines.append("ds_write_b128 %s, v[%d:%d]" % (t, O + 4 * c, O + 4 * c + 3))
    lines.append("s_waitcnt lgkmcnt(0)")
    out.append(emit("sp_put_o", ["float inv", "uint32_t a0"], lines, [], ['[inv] "v"(inv)', '[a0] "v"(a0)'], ['"memory"']))
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
