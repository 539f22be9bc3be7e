#!/usr/bin/env python3
"""Generates gemm_16_kloop.inc: the hand-scheduled K loop of the 256x256x64 GEMM tile.

    python gen_gemm_kloop.py > gemm_16_kloop.inc        (the output is committed too)

Workgroup: 4 wavefronts (one per SIMD, so each owns 512 registers), wave grid 2x2, wave tile 128x128 =
4x4 accumulator tiles of v_mfma_f32_32x32x16 kept in 256 AGPRs: the largest wave tile the register file
allows, i.e. the fewest LDS bytes per MFMA (the kernel is power-limited on MI355X, so bytes moved per flop,
not latency, set its speed).  A slice is 64 deep: 4 steps of 16 MFMAs.

Pipeline (t = slice):
  * global memory -> LDS directly (global_load_lds_dwordx4, no staging registers): the 16 loads of slice t+1
    are issued behind the even MFMAs of steps 0 and 1 of slice t into LDS stage (t+1) % 2.  Each instruction
    fills 8 tile rows (1 KiB); the XOR swizzle is applied on the source side (lane l fetches the chunk that
    belongs in slot l % 8 of row l / 8);
  * LDS -> fragments one step ahead, one read behind every odd MFMA of a step (an even stream, no bursts);
  * one barrier per slice, after MFMA 8 of the last step (preceded by s_waitcnt vmcnt(0): this wave's share of
    slice t+1 has landed); behind it the first fragments of slice t+1 are read while MFMAs 9-16 keep the
    matrix pipe busy.
Near the end of K the loads re-read the last slice (in bounds, into the stage nobody reads), which keeps the
slice bodies free of branches.

The W fragment is the first MFMA operand, so accumulator tiles come out transposed (a lane owns one row of A).
"""
# ---- register plan (all clobbered) ----
GA = [20 + j for j in range(8)]         # byte offset into A of the chunk this lane fetches in load instruction j
GB = [28 + j for j in range(8)]
AA = [36 + k for k in range(4)]         # LDS address of the lane's first A fragment row, step k (stage 0)
AB = [40 + k for k in range(4)]
F = [{"A": [64 + 4 * i for i in range(4)], "B": [80 + 4 * j for j in range(4)]},
     {"A": [96 + 4 * i for i in range(4)], "B": [112 + 4 * j for j in range(4)]}]
CLOBBER_V = list(range(20, 44)) + list(range(64, 128))
CLOBBER_S = [20, 21, 22, 23, 24, 25, 26, 27, 28, 29]

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


def loads(which, stage):
    """8 direct-to-LDS loads of this wave for one operand: M0 = LDS destination (wave base %20 / %21 + 1 KiB per
    instruction + stage), source = running base s[20:21] / s[22:23] + the lane's byte offset."""
    base, lds, off = ("s[20:21]", "%20", GA) if which == "A" else ("s[22:23]", "%21", GB)
    return [f"s_add_u32 m0, {lds}, {stage * STAGE + j * 1024}\\n s_nop 0\\n global_load_lds_dwordx4 v{off[j]}, {base}"
            for j in range(8)]


def advance(which):
    """Moves one operand's base to the next slice while that stays inside the operand (s25 / s29 = index of the slice the
    base points at, s26 = last slice)."""
    idx, lo, hi = ("s25", "s20", "s21") if which == "A" else ("s29", "s22", "s23")
    return [f"s_cmp_lt_u32 {idx}, s26", "s_cselect_b32 s27, 128, 0", "s_cselect_b32 s28, 1, 0",
            f"s_add_u32 {lo}, {lo}, s27", f"s_addc_u32 {hi}, {hi}, 0", f"s_add_u32 {idx}, {idx}, s28"]


# LDS reads return in order, so lgkmcnt(n) = "all but the n youngest have landed".  The 8 reads of a step's operands
# (a0,b0,b1,b2,b3,a1,a2,a3) are issued during the step before, one behind every odd MFMA (1,3,..,15), so that LDS sees an
# even stream instead of bursts.  Before MFMA m the queue holds what is left of those 8 plus the younger reads already
# issued in this step: MFMA 1 needs a0,b0 -> b1..a3 = 6 may be pending; MFMA 2 needs b1 -> 5 older + 1 younger = 6;
# MFMA 3 needs b2 -> 4 + 1 = 5; MFMA 4 needs b3 -> 3 + 2 = 5; MFMA 5 needs a1 -> 2 + 2 = 4; MFMA 9 needs a2 -> 1 + 4 = 5;
# MFMA 13 needs a3 -> 0 + 6 = 6.
WAITS = {1: 6, 2: 6, 3: 5, 4: 5, 5: 4, 9: 5, 13: 6}
# last step of a slice: no reads of a next step; everything has landed before the barrier behind MFMA 8 (other waves
# overwrite this stage right after it)
WAITS_LAST = {1: 6, 2: 5, 3: 4, 4: 3, 5: 2}


def slice_body(mn, cur, b_off):
    """Slice t, whose operands sit in LDS stage `cur`.  Stage 1 - cur receives slice t+1: its A half was requested during
    the last step of slice t-1, its B half is requested here during step 0.  After this slice's barrier stage `cur` is
    free and the A half of slice t+2 is requested into it."""
    nxt = 1 - cur
    out = []
    # boustrophedon over the 4 x 4 accumulator tiles: consecutive matrix instructions differ in ONE operand fragment, also
    # where a row of tiles ends (fewer operand-bus toggles for the same arithmetic; the part runs at its power limit)
    order = [(i, j if i % 2 == 0 else 3 - j) for i in range(4) for j in range(4)]
    for k in range(4):
        fs = k & 1
        behind_odd = reads(1 - fs, k + 1, cur, b_off) if k < 3 else []          # behind MFMAs 1,3,..,15
        behind_even = loads("B", nxt) if k == 0 else []                         # behind MFMAs 2,4,..,16
        after_barrier = loads("A", cur) if k == 3 else []                       # behind MFMAs 9..16 of the last step
        waits = WAITS if k < 3 else WAITS_LAST
        for m, (i, j) in enumerate(order, start=1):
            if k == 3 and m == 9:
                out += ["s_waitcnt vmcnt(0) lgkmcnt(0)", "s_barrier"]
                out += reads(0, 0, nxt, b_off)                                  # first fragments of the next slice
            if waits.get(m) is not None:
                out.append(f"s_waitcnt lgkmcnt({waits[m]})")
            out.append(mfma(mn, fs, i, j))
            if m % 2 == 1 and behind_odd:
                out.append(behind_odd[m // 2])
            elif m % 2 == 0 and behind_even:
                out.append(behind_even[m // 2 - 1])
            if m >= 9 and after_barrier:
                out.append(after_barrier[m - 9])
        if k == 0:
            out += advance("B")
        if k == 3:
            out += advance("A")
    return out


def kloop(mn, b_off):
    s = []
    # ---- setup: step addresses differ only in the swizzled chunk bits; load instructions are 8 rows apart and
    #      alternate between the two swizzle phases (chunk ^ 4, i.e. byte offset ^ 64)
    s += [f"v_mov_b32 v{AA[0]}, %16", f"v_xor_b32 v{AA[1]}, 32, %16", f"v_xor_b32 v{AA[2]}, 64, %16", f"v_xor_b32 v{AA[3]}, 96, %16"]
    s += [f"v_mov_b32 v{AB[0]}, %17", f"v_xor_b32 v{AB[1]}, 32, %17", f"v_xor_b32 v{AB[2]}, 64, %17", f"v_xor_b32 v{AB[3]}, 96, %17"]
    s += [f"v_mov_b32 v{GA[0]}, %18", f"v_mov_b32 v{GB[0]}, %19"]
    for j in range(1, 8):
        s += [f"v_add_u32 v{GA[j]}, %22, v{GA[j - 1]}", f"v_add_u32 v{GB[j]}, %22, v{GB[j - 1]}",
              f"v_xor_b32 v{GA[j]}, 64, v{GA[j]}", f"v_xor_b32 v{GB[j]}, 64, v{GB[j]}"]
    s += ["s_mov_b64 s[20:21], %23", "s_mov_b64 s[22:23], %24", "s_mov_b32 s24, %25", "s_sub_u32 s26, %25, 1", "s_mov_b32 s25, 0", "s_mov_b32 s29, 0"]
    # ---- prologue: slice 0 -> LDS stage 0, first fragments
    s += loads("A", 0) + loads("B", 0) + advance("A") + advance("B")
    s += ["s_waitcnt vmcnt(0)", "s_barrier"] + reads(0, 0, 0, b_off)
    s += loads("A", 1) + advance("A")                                           # A half of slice 1
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
    print("// A / B fragment row (step 0, stage 0); %18 / %19 byte offset into A / W of the chunk this lane fetches in its wave's")
    print("// first load instruction; %20 / %21 LDS byte address of the first row that instruction fills (stage 0, uniform);")
    print("// %22 bytes between the rows of consecutive load instructions (8 rows); %23 / %24 base of A / W; %25 number of slices.")
    print()
    plain = [0, 4096, 8192, 12288]                 # B fragments: 4 consecutive 32-row blocks
    swiglu = [0, 4096, 16384, 20480]               # 2 gate blocks, then the 2 matching up blocks 128 rows further
    for tname, mn in (("F16", "v_mfma_f32_32x32x16_f16"), ("BF16", "v_mfma_f32_32x32x16_bf16")):
        emit(f"PRISM_KLOOP4_{tname}_PLAIN", kloop(mn, plain))
        emit(f"PRISM_KLOOP4_{tname}_SWIGLU", kloop(mn, swiglu))
    regs = ", ".join(f'"v{r}"' for r in CLOBBER_V) + ", " + ", ".join(f'"s{r}"' for r in CLOBBER_S)
    # m0 (written before every direct-to-LDS load) is not listed: the compiler reserves it, sets it right before each of
    # its own uses and never keeps a value in it across a statement; hipcc diagnoses it in a clobber list
    print(f"#define PRISM_KLOOP4_CLOBBERS {regs}, \"scc\", \"memory\"")


if __name__ == "__main__":
    main()
