#!/usr/bin/env python3
"""Generates gemm_16_kloop.inc: the hand-scheduled K loop of the 256x256x64 GEMM tile.

Run from the build (python gen_gemm_kloop.py > gemm_16_kloop.inc); the output is committed too.

Workgroup: 4 wavefronts (one per SIMD, so each owns 512 registers), wave grid 2x2, wave tile 128x128 =
4x4 accumulator tiles of v_mfma_f32_32x32x16 kept in 256 AGPRs.  A slice is 64 deep: 4 steps of 16 MFMAs.

Software pipeline (t = slice):
  * global memory -> registers two slices ahead: the 16 loads of slice t+2 are issued during steps 0-1 of
    slice t into register set P[t % 2]; a slice of MFMA work is shorter than an HBM round trip, and LDS
    (160 KB) cannot hold more than two 64 KB stages, so the extra slice in flight lives in registers;
  * registers -> LDS: set P[(t+1) % 2] (slice t+1, in flight for more than one slice) is written to LDS stage
    (t+1) % 2 during steps 2-3 of slice t, after s_waitcnt vmcnt(16) (everything but the 16 youngest loads);
  * LDS -> fragments one step ahead, one read behind each of the first 8 MFMAs of a step;
  * one barrier per slice, placed after MFMA 12 of the last step: behind it the first fragments of the next
    slice are read while MFMAs 13-16 keep the matrix pipe busy.
Near the end of K the loads re-read the last slice (in bounds) and the last LDS write is never read, which keeps
the slice bodies free of branches.

The W fragment is the first MFMA operand, so accumulator tiles come out transposed (a lane owns one row of A).
"""
import os
import sys

EXP = os.environ.get("PRISM_KLOOP_EXPERIMENT", "")   # timing experiments only: "noadvance", "noloads", "nowrites"

# ---- register plan (all clobbered) ----
GA = [20 + j for j in range(8)]         # global byte offsets of this thread's 8 A chunks
GB = [28 + j for j in range(8)]
AA = [36 + k for k in range(4)]         # LDS address of the lane's first A fragment row, step k (stage 0)
AB = [40 + k for k in range(4)]
WA, WB = 44, 45                         # LDS write address of this thread's first A / B chunk (stage 0)
P = [{"A": [64 + 4 * j for j in range(8)], "B": [96 + 4 * j for j in range(8)]},
     {"A": [192 + 4 * j for j in range(8)], "B": [224 + 4 * j for j in range(8)]}]
F = [{"A": [128 + 4 * i for i in range(4)], "B": [144 + 4 * j for j in range(4)]},
     {"A": [160 + 4 * i for i in range(4)], "B": [176 + 4 * j for j in range(4)]}]
CLOBBER_V = list(range(20, 46)) + list(range(64, 256))
CLOBBER_S = [20, 21, 22, 23, 24, 25, 26, 27, 28]

STAGE = 32768                           # bytes per LDS stage of one operand
A_FRAG_OFF = [0, 4096, 8192, 12288]     # 32 rows x 128 B apart


def v4(r):
    return f"v[{r}:{r + 3}]"


def reads(fs, k, stage, b_off):
    """The 8 fragment reads of step k from `stage` into fragment set fs, in the order a0,b0,b1,b2,b3,a1,a2,a3."""
    ra = lambda i: f"ds_read_b128 {v4(F[fs]['A'][i])}, v{AA[k]} offset:{stage * STAGE + A_FRAG_OFF[i]}"
    rb = lambda j: f"ds_read_b128 {v4(F[fs]['B'][j])}, v{AB[k]} offset:{stage * STAGE + b_off[j]}"
    return [ra(0), rb(0), rb(1), rb(2), rb(3), ra(1), ra(2), ra(3)]


def mfma(mn, fs, i, j):
    acc = f"%{i * 4 + j}"
    return f"{mn} {acc}, {v4(F[fs]['B'][j])}, {v4(F[fs]['A'][i])}, {acc}"


def loads(pset, which):
    if EXP in ("noloads", "noloadswrites"):
        return ["s_nop 0"] * 8
    base = "s[20:21]" if which == "A" else "s[22:23]"
    off = GA if which == "A" else GB
    return [f"global_load_dwordx4 {v4(P[pset][which][j])}, v{off[j]}, {base}" for j in range(8)]


def writes(pset, which, stage):
    if EXP in ("nowrites", "noloadswrites") and stage >= 0:
        return ["s_nop 0"] * 8
    w = WA if which == "A" else WB
    return [f"ds_write_b128 v{w}, {v4(P[pset][which][j])} offset:{stage * STAGE + j * 4096}" for j in range(8)]


ADVANCE = [  # bases move to the next slice only while that stays inside the operand (s25 = slice index, s26 = last)
    "s_cmp_lt_u32 s25, s26", "s_cselect_b32 s27, 128, 0", "s_cselect_b32 s28, 1, 0",
    "s_add_u32 s20, s20, s27", "s_addc_u32 s21, s21, 0", "s_add_u32 s22, s22, s27", "s_addc_u32 s23, s23, 0",
    "s_add_u32 s25, s25, s28"]
if EXP == "noadvance":
    ADVANCE = ["s_nop 0"]


def slice_body(mn, cur, b_off):
    """Slice whose operands sit in LDS stage `cur`.  Loads go to P[cur], writes come from P[1-cur] into stage 1-cur."""
    nxt = 1 - cur
    out = []
    order = [(i, j) for i in range(4) for j in range(4)]
    waits_read = {1: 6, 2: 6, 3: 6, 4: 6, 5: 6, 9: 9, 13: 8}
    for k in range(4):
        fs = k & 1
        if k < 3:
            behind_first = reads(1 - fs, k + 1, cur, b_off)            # one behind each of MFMAs 1..8
        else:
            behind_first = writes(nxt, "B", nxt)
        if k == 0:
            behind_last = loads(cur, "A")
        elif k == 1:
            behind_last = loads(cur, "B")
        elif k == 2:
            behind_last = writes(nxt, "A", nxt)
        else:
            behind_last = []
        if k == 2:
            w = dict(waits_read); w[13] = 12                              # 8 reads + 4 writes younger than a3
        elif k == 3:
            w = {1: 14, 2: 14, 3: 14, 4: 14, 5: 14, 9: 15, 13: None}      # the queue also holds the 16 LDS writes
        else:
            w = waits_read
        for m, (i, j) in enumerate(order, start=1):
            if k == 3 and m == 13:
                out += ["s_waitcnt lgkmcnt(0)", "s_barrier"]
                out += reads(0, 0, nxt, b_off)                            # first fragments of the next slice
            elif w.get(m) is not None:
                out.append(f"s_waitcnt lgkmcnt({w[m]})")
            if k == 2 and m == 9:
                out.append("s_waitcnt vmcnt(16)")                         # slice t+1 has landed in P[nxt]
            out.append(mfma(mn, fs, i, j))
            if m <= 8:
                out.append(behind_first[m - 1])
            elif behind_last:
                out.append(behind_last[m - 9])
        if k == 1:
            out += ADVANCE
    return out


def kloop(mn, b_off):
    s = []
    # ---- setup: step addresses differ only in the swizzled chunk bits; chunk rows are 32 apart
    s += [f"v_mov_b32 v{AA[0]}, %16", f"v_xor_b32 v{AA[1]}, 32, %16", f"v_xor_b32 v{AA[2]}, 64, %16", f"v_xor_b32 v{AA[3]}, 96, %16"]
    s += [f"v_mov_b32 v{AB[0]}, %17", f"v_xor_b32 v{AB[1]}, 32, %17", f"v_xor_b32 v{AB[2]}, 64, %17", f"v_xor_b32 v{AB[3]}, 96, %17"]
    s += [f"v_mov_b32 v{WA}, %18", f"v_mov_b32 v{WB}, %19", f"v_mov_b32 v{GA[0]}, %20", f"v_mov_b32 v{GB[0]}, %21"]
    for j in range(1, 8):
        s += [f"v_add_u32 v{GA[j]}, %22, v{GA[j - 1]}", f"v_add_u32 v{GB[j]}, %22, v{GB[j - 1]}"]
        if j == 4:
            s += [f"v_add_u32 v{GB[4]}, %26, v{GB[4]}"]   # SwiGLU: chunk rows 128.. of the B tile are the up rows, F rows further in W
    s += ["s_mov_b64 s[20:21], %23", "s_mov_b64 s[22:23], %24", "s_mov_b32 s24, %25", "s_sub_u32 s26, %25, 1", "s_mov_b32 s25, 0"]
    # ---- prologue: slice 0 -> P0 -> LDS stage 0, slice 1 -> P1 (in flight), first fragments
    s += loads(0, "A") + loads(0, "B") + ADVANCE + loads(1, "A") + loads(1, "B") + ADVANCE
    s += ["s_waitcnt vmcnt(16)"] + writes(0, "A", 0) + writes(0, "B", 0) + ["s_waitcnt lgkmcnt(0)", "s_barrier"]
    s += reads(0, 0, 0, b_off)
    s += ["L_loop_%=:"] + slice_body(mn, 0, b_off)
    s += ["s_sub_u32 s24, s24, 1", "s_cmp_eq_u32 s24, 0", "s_cbranch_scc1 L_done_%="]
    s += slice_body(mn, 1, b_off)
    s += ["s_sub_u32 s24, s24, 1", "s_cmp_lg_u32 s24, 0", "s_cbranch_scc1 L_loop_%="]
    s += ["L_done_%=:", "s_waitcnt vmcnt(0) lgkmcnt(0)", "s_nop 15", "s_nop 15"]   # MFMA results settle before the epilogue reads them
    return s


def emit(name, lines):
    print(f"#define {name} \\")
    for l in lines:
        print(f'  "{l}\\n" \\')
    print('  ""')
    print()


def main():
    print("// Generated by gen_gemm_kloop.py - do not edit.  See that file for the schedule.")
    print("// Operands: %0..%15 accumulators acc[i][j] (operand i*4+j, AGPRs); %16 / %17 LDS byte address of the lane's first")
    print("// A / B fragment row (step 0, stage 0); %18 / %19 LDS byte address this thread writes its first A / B chunk to;")
    print("// %20 / %21 byte offset of that chunk in A / W; %22 bytes between chunk rows (32 rows); %23 / %24 base of A / W;")
    print("// %25 number of 64-deep slices; %26 extra byte offset of B chunk rows 128..255 (0, or the gate->up distance for SwiGLU).")
    print()
    plain = [0, 4096, 8192, 12288]                 # B fragments: 4 consecutive 32-row blocks
    swiglu = [0, 4096, 16384, 20480]               # 2 gate blocks, then the 2 matching up blocks 128 rows further
    for tname, mn in (("F16", "v_mfma_f32_32x32x16_f16"), ("BF16", "v_mfma_f32_32x32x16_bf16")):
        emit(f"PRISM_KLOOP4_{tname}_PLAIN", kloop(mn, plain))
        emit(f"PRISM_KLOOP4_{tname}_SWIGLU", kloop(mn, swiglu))
    regs = ", ".join(f'"v{r}"' for r in CLOBBER_V) + ", " + ", ".join(f'"s{r}"' for r in CLOBBER_S)
    print(f"#define PRISM_KLOOP4_CLOBBERS {regs}, \"scc\", \"memory\"")


if __name__ == "__main__":
    main()
