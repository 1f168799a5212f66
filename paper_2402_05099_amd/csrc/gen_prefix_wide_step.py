#!/usr/bin/env python3
"""Writes prefix_wide_step.inc: the body of one pipeline step of the 256-row shared-block attention kernel
(prefix_wide.hip) as straight-line C++.

A step is 16 MFMAs in a fixed order (8 for the scores of the next 32 keys, 8 for P*V of the current 32 keys).
Between them go, in fixed places: the step's vector-ALU work (exponentials of the current scores, packing to bf16,
fp32 row sums, row maxima of the next scores), its two HBM->LDS copy instructions (addressed by the kernel's copy
cursor `cur`, which runs NS-1 stages ahead of the piece `pc` being computed) and its 24 LDS fragment reads.  Every
gap ends in a scheduling barrier so that the compiler keeps this order: a wavefront then always has a matrix
instruction in flight while it issues vector-ALU instructions, instead of running the two kinds back to back.

usage: gen_prefix_wide_step.py [out.inc] [vector-ALU cycles per gap]
"""
import os
import sys

OUT = sys.argv[1] if len(sys.argv) > 1 else os.path.join(os.path.dirname(os.path.abspath(__file__)), "prefix_wide_step.inc")
CAP = float(sys.argv[2]) if len(sys.argv) > 2 else 28.0   # a 32x32x16 MFMA occupies the matrix pipe for 32 cycles
MAX_FROM = 10       # first gap that may hold row-maximum work (the score MFMAs end at gap 7)
XYZW = "xyzw"
# measured issue cost of one wave64 instruction, cycles
C_FMA, C_EXP, C_CVT, C_ADD, C_MAX, C_HALF = 5.2, 8.8, 5.2, 4.9, 5.2, 19.0


def build():
    mf = []         # (MFMA statement, statements before the gap's ALU work, statements after it)
    # Only half a stage of K and of V fragments is held in registers (two wavefronts share a SIMD's register file):
    # each fragment register is reloaded twice per step, four gaps before its next use.
    for q in range(8):
        f = "mfma_first" if q == 0 else "mfma_acc"
        if q < 4:    # second half of the K rows of stage j+1
            post = [f"kf[{q}] = lds_k(slot1, {q + 4});"]
        else:        # first half of the K rows of stage j+2, for the next step
            post = [f"kf[{q - 4}] = lds_k(slot2, {q - 4});"]
        mf.append((f"{f}(Snext, kf[{q & 3}], qf[{q}]);", [], post))
    for tt in range(2):
        for db in range(4):
            if tt == 0:  # keys 16..31 of stage j
                post = [f"vf[{db}] = lds_v(slot, 1, {db});"]
            else:        # keys 0..15 of stage j+1, for the next step
                post = [f"vf[{db}] = lds_v(slot1, 0, {db});"]
            mf.append((f"mfma_acc(Oacc[{db}], vf[{db}], pb[{tt}]);", [], post))
    # the copy that keeps the ring NS-1 stages ahead (the copy cursor may already be in a later piece): scalar address
    # arithmetic in gap 0, the two copy instructions in gaps 1 and 3
    mf[0][1].extend(["const int64_t cp_off = (int64_t)min(cur.ks + cur.t * KT, cur.kwin) * rstride_b;",
                     "const unsigned cp_dst = ldsw + (unsigned)((slot + NS - 1) & (NS - 1)) * STB;"])
    mf[1][1].append("copy16(cur.Kg + cp_off, cur.voffK, cp_dst);")
    mf[3][1].append("copy16(cur.Vg + cp_off, cur.voffV, cp_dst + VRING);")

    crit, late = [], []     # (cycles, statement, earliest gap, deadline gap)
    n = 0
    for h in range(2):
        dl = 8 if h == 0 else 12
        ids = list(range(n, n + 4))
        # all multiply-adds of a block of 8 scores, then its exponentials, then the packs: no instruction uses the
        # result of the one just before it
        for p, k in enumerate(ids):
            i0 = 8 * h + 2 * p
            crit.append((C_FMA, f"const float xa{k} = fmaf(Scur[{i0}], c2, -mc);", 0, dl))
            crit.append((C_FMA, f"const float xb{k} = fmaf(Scur[{i0 + 1}], c2, -mc);", 0, dl))
        for p, k in enumerate(ids):
            crit.append((C_EXP, f"const float ea{k} = __builtin_amdgcn_exp2f(xa{k});", 0, dl))
            crit.append((C_EXP, f"const float eb{k} = __builtin_amdgcn_exp2f(xb{k});", 0, dl))
        for p, k in enumerate(ids):
            crit.append((C_CVT, f"pb[{h}].{XYZW[p]} = pack_bf16_pair(ea{k}, eb{k});", 0, dl))
            late.append((C_ADD, f"lsum[0] += ea{k};", 0, 99))
            late.append((C_ADD, f"lsum[1] += eb{k};", 0, 99))
        n += 4
    # row maximum of the new scores: two chains, interleaved
    S = "Snext"
    cha = [f"float ma = max3f({S}[0], {S}[1], {S}[2]);", f"ma = max3f(ma, {S}[3], {S}[4]);",
           f"ma = max3f(ma, {S}[5], {S}[6]);", f"ma = max3f(ma, {S}[7], {S}[15]);"]
    chb = [f"float mb = max3f({S}[8], {S}[9], {S}[10]);", f"mb = max3f(mb, {S}[11], {S}[12]);",
           f"mb = max3f(mb, {S}[13], {S}[14]);"]
    mx = []
    for i in range(4):
        mx.append((C_MAX, cha[i], MAX_FROM, 99))
        if i < len(chb):
            mx.append((C_MAX, chb[i], MAX_FROM, 99))
    mx.append((C_MAX, "tmax = max2f(ma, mb);", MAX_FROM, 99))
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


if __name__ == "__main__":
    with open(OUT, "w") as f:
        f.write("// Generated by gen_prefix_wide_step.py (one pipeline step of prefix_wide.hip); do not edit by hand.\n" + build())
