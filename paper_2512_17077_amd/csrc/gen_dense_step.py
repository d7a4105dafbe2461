#!/usr/bin/env python3
"""Writes attend_dense_step.inc: the instruction stream of one 32-key step of the dense Refresh kernel
(attend_dense_bf16.hip) as inline-assembly text with a fixed register map.

Why text and not builtins: with one wave per SIMD the kernel has 512 registers, but only the lower 256
(v0..v255) can feed vector instructions; the upper 256 (a0..a255) can only feed the matrix cores.  The
compiler, once it uses the upper half at all, puts every MFMA result there, the scores included, and
then copies them down one register at a time for the softmax: +60 % vector instructions.  Here the
output accumulators and the queries live in a-registers, the scores, probabilities and LDS operands in
v-registers, and the order of issue is exactly the order written: one MFMA, then the few vector and
LDS instructions that fit under it, and so on.

Run `python3 gen_dense_step.py` in this folder after changing the schedule; the .inc file is committed.

One step (iteration j) at D = 128, NQB = 2 blocks of 32 queries per wave:
    slots  0..15   S^T(j+1) = K(j+1) Q^T         MFMA(t, qb), K operand t shared by the two blocks
    slots 16..31   O^T += V(j-1)^T P(j-1)^T      MFMA(u, db, qb), V^T operand (u, db) shared likewise
    slots 32..35   l += ones P(j-1)^T             row sums of the same probabilities, MFMA(u, qb)
    all slots      P(j) = exp2(S(j) z - m z)      on the scores of the previous step: per pair of scores
                                                   2 fma, 2 exp, 1 cvt_pk (-> bf16 x 2)
    slots 20..31   row maxima of S(j+1)           16 max / max3
    LDS            16 transposing reads (V^T operands, four slots ahead of their MFMAs),
                   8 ds_read_b128 (K operands of step j+2, after the S chain has consumed the old ones)
Matrix results are read by vector instructions no sooner than four MFMAs after they were issued (the
hardware does not interlock that; 12 wait states are required), and a transcendental's result is not
read by the next instruction.
"""
import os
import sys

# timing experiments only (wrong results): leave out the vector work or the LDS operand fetches
NO_VALU = "--no-valu" in sys.argv
NO_DS = "--no-ds" in sys.argv
NO_KREAD = "--no-kread" in sys.argv   # keep the waits, drop the reads themselves
NO_VREAD = "--no-vread" in sys.argv
NO_LOADS = "--no-loads" in sys.argv   # keep the barrier, drop the global_load_lds (LDS keeps what the prologue loaded)

# ---- register map (v-registers; a-registers are numbered separately)
ST_A, ST_B = 96, 128          # scores, [qb][16]
PB_A, PB_B = 160, 176         # packed probabilities, [qb][u][4]
KOP = 192                     # K operands [t][4]
VOP = 224                     # V^T operand buffers [NBUF][4]
TMP = 76                      # [2][2] logits / probabilities in flight
SM = 70                       # lsum0, lsum1, nmz0, nmz1, mx0, mx1
ADDR = 80                     # ka[8], va[2][4]
NBUF = int(os.environ.get("DLLM_GEN_NBUF", "8"))
ACC = 0                       # a: acc[qb][db][16]
ONES = "0x3f803f80"           # bf16 (1, 1)


def vr(base, n=1):
    return f"v{base}" if n == 1 else f"v[{base}:{base + n - 1}]"


def ar(base, n=1):
    return f"a{base}" if n == 1 else f"a[{base}:{base + n - 1}]"


def gen_step(D, cur, nxt, pnew, pold, with_scores=True, with_softmax=True, with_loads=False):
    """Instruction list of one step.  with_scores/with_softmax False: the closing P V product only."""
    NT, NDB = D // 16, D // 32
    QR = 16 * 2 * NDB                      # a: q[qb][t][4] after the accumulators
    ROWB = 2 * D
    n_s = NT * 2 if with_scores else 0     # score MFMAs
    n_pv = 2 * NDB * 2                     # P V MFMAs
    n_ls = 4                               # row-sum MFMAs
    nslots = n_s + n_pv + n_ls
    LS = QR + 4 * NT * 2                   # a: ls[qb][16] after the queries

    # ---- MFMAs per slot
    mfma = []
    if with_scores:
        for t in range(NT):
            for qb in range(2):
                c = "0" if t == 0 else vr(nxt + 16 * qb, 16)
                mfma.append((f"v_mfma_f32_32x32x16_bf16 {vr(nxt + 16 * qb, 16)}, {vr(KOP + 4 * t, 4)}, "
                             f"{ar(QR + 4 * (NT * qb + t), 4)}, {c}", None))
    for u in range(2):
        for db in range(NDB):
            p = u * NDB + db
            for qb in range(2):
                a = ACC + 16 * (NDB * qb + db)
                mfma.append((f"v_mfma_f32_32x32x16_bf16 {ar(a, 16)}, {vr(VOP + 4 * (p % NBUF), 4)}, "
                             f"{vr(pold + 4 * (2 * qb + u), 4)}, {ar(a, 16)}", ("v", p) if qb == 0 else None))
    # row sums: row 0 of ones * P^T, accumulated like the outputs (the a-register blocks after the queries)
    for u in range(2):
        for qb in range(2):
            a = LS + 16 * qb
            mfma.append((f"v_mfma_f32_32x32x16_bf16 {ar(a, 16)}, %[ones], {vr(pold + 4 * (2 * qb + u), 4)}, {ar(a, 16)}", None))

    # ---- LDS reads per slot: (text, tag)
    ds = [[] for _ in range(nslots)]
    npairs = 2 * NDB

    def vread(p, rd):
        u, db = divmod(p, NDB)
        return (f"ds_read_b64_tr_b16 {vr(VOP + 4 * (p % NBUF) + 2 * rd, 2)}, {vr(ADDR + 8 + NDB * rd + db)} "
                f"offset:%[voff{u}]", ("v", p))

    # the first NBUF operand pairs are fetched ahead of the P V phase, the others as their buffer frees up
    first = min(NBUF, npairs)
    if with_scores:
        lead = n_s - 2 * first
        for p in range(first):
            ds[lead + 2 * p].append(vread(p, 0))
            ds[lead + 2 * p + 1].append(vread(p, 1))
    else:
        for p in range(first):   # nothing to hide behind: all at once, in front
            ds[0].append(vread(p, 0))
            ds[0].append(vread(p, 1))
    for p in range(first, npairs):
        s0 = n_s + 2 * (p - NBUF) + 2   # after both MFMAs that read this buffer have been issued
        ds[s0].append(vread(p, 0))
        ds[s0 + 1].append(vread(p, 1))
    if with_scores:
        free = [s for s in range(n_s, n_s + n_pv) if not ds[s]]
        assert len(free) >= NT, (len(free), NT)
        for t in range(NT):
            ds[free[t]].append((f"ds_read_b128 {vr(KOP + 4 * t, 4)}, {vr(ADDR + t)} offset:%[koff]", ("k", t)))

    # ---- vector work
    valu = [[] for _ in range(nslots)]
    if with_softmax:
        ops = []
        pairs = [(qb, u, jj) for qb in range(2) for u in range(2) for jj in range(4)]

        # Row sums: the four extra MFMAs above add up the probabilities as rounded to bf16, the values the
        # matrix cores multiply with V, so the vector units only convert.
        def finish(i):
            qb, u, jj = pairs[i]
            t0 = TMP + 2 * (i % 2)
            w = pnew + 4 * (2 * qb + u) + jj
            return [f"v_cvt_pk_bf16_f32 {vr(w)}, {vr(t0)}, {vr(t0 + 1)}"], [], []

        for i, (qb, u, jj) in enumerate(pairs):
            t0 = TMP + 2 * (i % 2)
            s0 = cur + 16 * qb + 8 * u + 2 * jj
            cvt, add0, add1 = finish(i - 1) if i > 0 else ([], [], [])
            ops += [f"v_fma_f32 {vr(t0)}, {vr(s0)}, %[zs], {vr(SM + 2 + qb)}",
                    f"v_fma_f32 {vr(t0 + 1)}, {vr(s0 + 1)}, %[zs], {vr(SM + 2 + qb)}"]
            ops += [f"v_exp_f32_e32 {vr(t0)}, {vr(t0)}", f"v_exp_f32_e32 {vr(t0 + 1)}, {vr(t0 + 1)}"]
            ops += cvt + add0 + add1
        cvt, add0, add1 = finish(len(pairs) - 1)
        ops += ["s_nop 0"] + cvt + add0 + add1      # the nop keeps the last exp's result from being read at once
        for s in range(nslots):   # evenly: about three per MFMA at D = 128
            valu[s] += ops[s * len(ops) // nslots:(s + 1) * len(ops) // nslots]
        # row maxima of the new scores, well after the S chain
        mops = []
        for i in range(8):
            for qb in range(2):
                s0 = nxt + 16 * qb + 2 * i
                m = vr(SM + 4 + qb)
                mops.append(f"v_max_f32_e32 {m}, {vr(s0)}, {vr(s0 + 1)}" if i == 0 else
                            f"v_max3_f32 {m}, {m}, {vr(s0)}, {vr(s0 + 1)}")
        start = n_s + 4
        span = nslots - start
        for i, op in enumerate(mops):
            valu[start + i * span // len(mops)].append(op)

    # ---- tile loads (first step of a tile only): K then V rows of the tile two ahead, global memory
    # straight into LDS, one load every other MFMA so that their issue (about 50 cycles each when issued
    # back to back) hides under the matrix work.  m0 holds the LDS destination of the wave's slice.
    loads = [[] for _ in range(nslots)]
    if with_loads:
        nld = 64 * (D // 8) // 256
        seq = [("%[kt]", "%[lk]", i) for i in range(nld)] + [("%[vt]", "%[lv]", i) for i in range(nld)]
        for n, (base, lds, i) in enumerate(seq):
            loads[2 + 2 * n] = [f"s_add_u32 m0, %[wl], {lds}+{i * 256 * 16}",
                                f"global_load_lds_dwordx4 %[lo{i}], {base}"]

    # ---- emit, with the waits for LDS data: reads return in order, so a consumer waits until no more
    # reads are outstanding than were issued after the one it needs (steady state: the previous step's
    # tail is the same as this step's)
    order = []   # DS tags in issue order over this step
    for s in range(nslots):
        for _, tag in ds[s]:
            order.append(tag)
    lines = []
    issued = []   # tags issued so far in this step

    def wait_for(tag_pred, from_prev):
        if from_prev:
            # needed read was issued in the previous step: everything after it there, plus all issued here
            idx = max(i for i, t in enumerate(order) if tag_pred(t))
            n = (len(order) - 1 - idx) + len(issued)
        else:
            idx = max(i for i, t in enumerate(issued) if tag_pred(t))
            n = len(issued) - 1 - idx
        return n

    if not with_scores:   # the closing product: its first operand fetches come before its first MFMA
        for dtext, tag in ds[0]:
            lines.append(dtext)
            issued.append(tag)
        ds[0] = []
    if NO_VALU:
        valu = [[] for _ in range(nslots)]
    for s in range(nslots):
        text, need = mfma[s]
        if NO_DS:
            lines.append(text)
            lines += valu[s]
            continue
        if with_scores and s < n_s and s % 2 == 0:
            t = s // 2
            n = wait_for(lambda tag: tag == ("k", t), True)
            lines.append(f"s_waitcnt lgkmcnt({min(n, 15)})")
        if need is not None:
            p = need[1]
            n = wait_for(lambda tag: tag == ("v", p), False)
            lines.append(f"s_waitcnt lgkmcnt({min(n, 15)})")
        lines.append(text)
        if with_loads and s == 1:
            # Tile boundary: the loads issued a tile ago (the next tile) have landed in every wave, and every
            # wave is done with the tile before last, whose ring slots the loads below refill.  Two MFMAs
            # are in the pipe while the waves meet.
            lines += ["s_waitcnt vmcnt(0)", "s_barrier"]
        if loads[s] and not NO_LOADS:
            lines.append(loads[s][0])
        for dtext, tag in ds[s]:
            if not ((NO_KREAD and tag[0] == "k") or (NO_VREAD and tag[0] == "v")):
                lines.append(dtext)
            issued.append(tag)
        lines += valu[s][:1]
        if loads[s] and not NO_LOADS:
            lines.append(loads[s][1])
        lines += valu[s][1:]
    if with_softmax:
        # does any new score exceed its running maximum by more than the lazy step?  (lanes as a mask)
        lines += [f"v_fma_f32 {vr(TMP)}, {vr(SM + 4)}, %[zs], {vr(SM + 2)}",
                  f"v_fma_f32 {vr(TMP + 1)}, {vr(SM + 5)}, %[zs], {vr(SM + 3)}",
                  f"v_max_f32_e32 {vr(TMP)}, {vr(TMP)}, {vr(TMP + 1)}",
                  f"v_cmp_gt_f32_e64 %[grow], {vr(TMP)}, %[lazy]"]
    return lines


def as_macro(name, lines):
    body = " \\\n".join(f'  "{l}\\n\\t"' for l in lines)
    return f"#define {name} \\\n{body}\n"


def gen_score0(D):
    """S^T(0) into st_a from the K operands in kop, then enough wait states for any reader"""
    NT, NDB = D // 16, D // 32
    QR = 16 * 2 * NDB
    lines = []
    for t in range(NT):
        for qb in range(2):
            c = "0" if t == 0 else vr(ST_A + 16 * qb, 16)
            lines.append(f"v_mfma_f32_32x32x16_bf16 {vr(ST_A + 16 * qb, 16)}, {vr(KOP + 4 * t, 4)}, "
                         f"{ar(QR + 4 * (NT * qb + t), 4)}, {c}")
    return lines + ["s_nop 15", "s_nop 15"]


def gen_acc_init(D):
    regs = list(range(16 * 2 * (D // 32)))
    ls = 16 * 2 * (D // 32) + 4 * (D // 16) * 2
    regs += list(range(ls, ls + 32))        # the row-sum blocks behind the queries
    return [f"v_accvgpr_write_b32 a{i}, 0" for i in regs]


def gen_acc_scale(D):
    """acc[qb] *= %[al<qb>] for both blocks, well after the last MFMA and before the next one."""
    n = 16 * (D // 32)
    lines = ["s_nop 15", "s_nop 15"]
    for qb in range(2):
        for i in range(0, n, 4):
            regs = [qb * n + i + c for c in range(4)]
            lines += [f"v_accvgpr_read_b32 {vr(TMP + c)}, a{r}" for c, r in enumerate(regs)]
            lines += [f"v_mul_f32_e32 {vr(TMP + c)}, %[al{qb}], {vr(TMP + c)}" for c in range(4)]
            lines += [f"v_accvgpr_write_b32 a{r}, {vr(TMP + c)}" for c, r in enumerate(regs)]
    ls = 2 * n + 4 * (D // 16) * 2   # the row sums: only row 0 of each block is ever non-zero
    for qb in range(2):
        lines += [f"v_accvgpr_read_b32 {vr(TMP)}, a{ls + 16 * qb}", f"v_mul_f32_e32 {vr(TMP)}, %[al{qb}], {vr(TMP)}",
                  f"v_accvgpr_write_b32 a{ls + 16 * qb}, {vr(TMP)}"]
    lines += ["s_nop 7"]
    return lines


def gen_acc_read(k):
    """sixteen accumulator registers a[16k .. 16k+15] into operands %0 .. %15"""
    return [f"v_accvgpr_read_b32 %{i}, a{16 * k + i}" for i in range(16)]


def main():
    out = ["// Generated by gen_dense_step.py -- do not edit by hand.  One 32-key step of the dense Refresh kernel as",
           "// inline-assembly text over a fixed register map; see the generator for the schedule and the map.",
           "// Named operands: %[ones] (four v-registers: the A operand whose first row is bf16 ones), %[zs] (softmax_scale * log2 e, scalar), %[koff] (byte offset of the K rows fetched",
           "// for step j+2), %[voff0], %[voff1] (byte offsets of the V rows of step j-1, keys 0..15 and 16..31),",
           "// %[grow] (out, scalar pair: lanes whose newest scores outgrew the running maximum by more than %[lazy]);",
           "// in the _AB text (the first step of a tile) also %[kt], %[vt] (scalar pairs: first K / V row of the tile",
           "// to load), %[lo0..] (per-lane byte offsets of the 16-byte chunks), %[wl] (LDS address of the wave's",
           "// slice of a load round), %[lk], %[lv] (byte offsets of the K / V ring slots to fill).",
           ""]
    for D in (128, 64):
        out.append(as_macro(f"DLLM_DENSE_STEP_{D}_AB", gen_step(D, ST_A, ST_B, PB_A, PB_B, with_loads=True)))
        out.append(as_macro(f"DLLM_DENSE_STEP_{D}_BA", gen_step(D, ST_B, ST_A, PB_B, PB_A)))
        out.append(as_macro(f"DLLM_DENSE_TAIL_{D}_A", gen_step(D, 0, 0, 0, PB_A, False, False)))
        out.append(as_macro(f"DLLM_DENSE_TAIL_{D}_B", gen_step(D, 0, 0, 0, PB_B, False, False)))
        out.append(as_macro(f"DLLM_DENSE_SCORE0_{D}", gen_score0(D)))
        out.append(as_macro(f"DLLM_DENSE_ACC_INIT_{D}", gen_acc_init(D)))
        out.append(as_macro(f"DLLM_DENSE_ACC_SCALE_{D}", gen_acc_scale(D)))
    for k in range(8):
        out.append(as_macro(f"DLLM_DENSE_ACC_READ_{k}", gen_acc_read(k)))
    outdir = os.path.dirname(os.path.abspath(__file__))
    for a in sys.argv[1:]:
        if a.startswith("--out="):
            outdir = a[6:]
    path = os.path.join(outdir, "attend_dense_step.inc")
    with open(path, "w") as f:
        f.write("\n".join(out))
    print("wrote", path)


if __name__ == "__main__":
    main()
