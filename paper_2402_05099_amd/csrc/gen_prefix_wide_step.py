#!/usr/bin/env python3
"""Writes prefix_wide_step.inc (D = 128) and prefix_wide_step_d64.inc (D = 64): the body of one pipeline step of the
256-row shared-block attention kernel (prefix_wide_impl.h) as straight-line C++.

A step is 16 MFMAs in a fixed order (8 for the scores of the next stage, 8 for P*V of the current stage; a stage is
32 keys at D = 128 and 64 keys, two score tiles, at D = 64).  Between them go, in fixed places: the step's vector-ALU
work (exponentials of the current scores, packing to bf16, fp32 row sums, row maxima of the next scores), its two
HBM->LDS copy instructions (addressed by the kernel's copy cursor `cur`, which runs NS-1 stages ahead of the piece
`pc` being computed) and its 24 LDS fragment reads.  Every gap ends in a scheduling barrier so that the compiler keeps
this order: a wavefront then always has a matrix instruction in flight while it issues vector-ALU instructions,
instead of running the two kinds back to back.  At D = 64 a step has twice the softmax work for the same 16 MFMAs:
the vector ALU, not the matrix pipe, sets its length.

usage: gen_prefix_wide_step.py [D [out.inc [vector-ALU cycles per gap]]]     (no arguments: both files)
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_OUT = {128: os.path.join(HERE, "prefix_wide_step.inc"), 64: os.path.join(HERE, "prefix_wide_step_d64.inc")}
DEFAULT_CAP = {128: 28.0, 64: 52.0}     # a 32x32x16 MFMA occupies the matrix pipe for 32 cycles
MAX_FROM = 10       # first gap that may hold row-maximum work (the score MFMAs end at gap 7)
XYZW = "xyzw"
# measured issue cost of one wave64 instruction, cycles
C_FMA, C_EXP, C_CVT, C_ADD, C_MAX, C_HALF = 5.2, 8.8, 5.2, 4.9, 5.2, 19.0


def build(D=128, CAP=None):
    CAP = DEFAULT_CAP[D] if CAP is None else CAP
    wide = D == 128
    # score tile(s) of a stage as the kernel names them
    cur_t = ["Scur"] if wide else ["Scur.a", "Scur.b"]
    nxt_t = ["Snext"] if wide else ["Snext.a", "Snext.b"]
    mf = []         # (MFMA statement, statements before the gap's ALU work, statements after it)
    # Only half a stage of K and of V fragments is held in registers (two wavefronts share a SIMD's register file):
    # each fragment register is reloaded twice per step, four gaps before its next use.  Fragment f of a stage's K is
    # (score tile f / KS, k-step f % KS); V fragments are (16-key group tt, 32-column block db).
    KS = D // 16
    for q in range(8):
        tile, ks = (0, q) if wide else (q // 4, q % 4)
        f = "mfma_first" if ks == 0 else "mfma_acc"
        if q < 4:    # second half of the K fragments of stage j+1
            post = [f"kf[{q}] = lds_k(slot1, {q + 4});"]
        else:        # first half of the K fragments of stage j+2, for the next step
            post = [f"kf[{q - 4}] = lds_k(slot2, {q - 4});"]
        mf.append((f"{f}({nxt_t[tile]}, kf[{q & 3}], qf[{ks}]);", [], post))
    DB = D // 32
    for i in range(8):
        tt, db = i // DB, i % DB
        if i < 4:    # second half of the V fragments of stage j
            post = [f"vf[{i}] = lds_v(slot, {(i + 4) // DB}, {db});"]
        else:        # first half of the V fragments of stage j+1, for the next step
            post = [f"vf[{i - 4}] = lds_v(slot1, {(i - 4) // DB}, {db});"]
        mf.append((f"mfma_acc(Oacc[{db}], vf[{i & 3}], pb[{tt}]);", [], post))
    # the copy that keeps the ring NS-1 stages ahead (the copy cursor may already be in a later piece): scalar address
    # arithmetic in gap 0, the two copy instructions in gaps 1 and 3
    mf[0][1].extend(["const int64_t cp_off = (int64_t)min(cur.ks + cur.t * KT, cur.kwin) * rstride_b;",
                     "const unsigned cp_dst = ldsw + (unsigned)((slot + NS - 1) & (NS - 1)) * STB;"])
    mf[1][1].append("copy16(cur.Kg + cp_off, cur.voffK, cp_dst);")
    mf[3][1].append("copy16(cur.Vg + cp_off, cur.voffV, cp_dst + VRING);")

    crit, late = [], []     # (cycles, statement, earliest gap, deadline gap)
    n = 0
    NPB = (32 if wide else 64) // 16        # packed operands pb[h]: the exponentials of keys 16 h .. 16 h + 15 of the stage
    for h in range(NPB):
        dl = 8 + (8 // NPB) * h             # the gap of the first MFMA that reads pb[h]
        src = cur_t[h // 2]
        ids = list(range(n, n + 4))
        # all multiply-adds of a block of 8 scores, then its exponentials, then the packs: no instruction uses the
        # result of the one just before it
        for p, k in enumerate(ids):
            i0 = 8 * (h % 2) + 2 * p
            crit.append((C_FMA, f"const float xa{k} = fmaf({src}[{i0}], c2, -mc);", 0, dl))
            crit.append((C_FMA, f"const float xb{k} = fmaf({src}[{i0 + 1}], c2, -mc);", 0, dl))
        for p, k in enumerate(ids):
            crit.append((C_EXP, f"const float ea{k} = __builtin_amdgcn_exp2f(xa{k});", 0, dl))
            crit.append((C_EXP, f"const float eb{k} = __builtin_amdgcn_exp2f(xb{k});", 0, dl))
        for p, k in enumerate(ids):
            crit.append((C_CVT, f"pb[{h}].{XYZW[p]} = pack_bf16_pair(ea{k}, eb{k});", 0, dl))
        # the row sums: at D = 128 they fill what the gaps have left at the end of the step; at D = 64 (twice the
        # exponentials, and the vector ALU sets the pace anyway) they follow their block so that its 8 exponentials die
        for p, k in enumerate(ids):
            (late if wide else crit).append((C_ADD, f"lsum[0] += ea{k};", 0, 99))
            (late if wide else crit).append((C_ADD, f"lsum[1] += eb{k};", 0, 99))
        n += 4
    # row maximum of the new scores: two chains per score tile, interleaved
    chains = []
    for t, S in enumerate(nxt_t):
        a, b = f"ma{t}", f"mb{t}"
        chains.append([f"float {a} = max3f({S}[0], {S}[1], {S}[2]);", f"{a} = max3f({a}, {S}[3], {S}[4]);",
                       f"{a} = max3f({a}, {S}[5], {S}[6]);", f"{a} = max3f({a}, {S}[7], {S}[15]);"])
        chains.append([f"float {b} = max3f({S}[8], {S}[9], {S}[10]);", f"{b} = max3f({b}, {S}[11], {S}[12]);",
                       f"{b} = max3f({b}, {S}[13], {S}[14]);"])
    mx = []
    for i in range(4):
        for ch in chains:
            if i < len(ch):
                mx.append((C_MAX, ch[i], MAX_FROM, 99))
    if wide:
        mx.append((C_MAX, "tmax = max2f(ma0, mb0);", MAX_FROM, 99))
    else:
        mx.append((C_MAX, "tmax = max3f(ma0, mb0, ma1);", MAX_FROM, 99))
        mx.append((C_MAX, "tmax = max2f(tmax, mb1);", MAX_FROM, 99))
    mx.append((C_HALF, "tmax = half_max_swap(tmax);", MAX_FROM, 99))
    out = []
    ci = mi = li = 0
    first_max = True
    for g, (stmt, pre, post) in enumerate(mf):
        out.append(f"// gap {g}")
        out.append(stmt)
        out.extend(pre)
        used = 0.0
        while used < CAP:
            if ci < len(crit):
                s = crit[ci]; ci += 1
            elif g >= MAX_FROM and mi < len(mx):
                if first_max:
                    out.append("if (kMasked) mask_stage(Snext, j + 1);")
                    first_max = False
                s = mx[mi]; mi += 1
            elif li < len(late):
                s = late[li]; li += 1
            else:
                break
            assert g < s[3], ("deadline missed", g, s)
            out.append(s[1]); used += s[0]
        out.extend(post)
        out.append("__builtin_amdgcn_sched_barrier(0);")
    assert ci == len(crit) and mi == len(mx) and li == len(late), ("work left over", ci, len(crit), mi, len(mx), li, len(late))
    return "\n".join("        " + l for l in out) + "\n"


def write(D, out=None, cap=None):
    with open(out or DEFAULT_OUT[D], "w") as f:
        f.write(f"// Generated by gen_prefix_wide_step.py (one pipeline step of prefix_wide_impl.h, D = {D}); do not edit by hand.\n" + build(D, cap))


if __name__ == "__main__":
    if len(sys.argv) > 1:
        write(int(sys.argv[1]), sys.argv[2] if len(sys.argv) > 2 else None, float(sys.argv[3]) if len(sys.argv) > 3 else None)
    else:
        write(128)
        write(64)
