// Hand-scheduled K-slice (64 deep) of the 256x256 GEMM tile for one wavefront that owns a 128x64
// block: 4 A fragments x 2 B fragments per 16-deep step, 4 steps, 32 matrix instructions, 24 LDS
// reads.  The compiler's own schedule of this loop waits on every LDS read right before the MFMA
// that needs it; here the reads of step kk+1 are issued one behind each of the first six MFMAs of
// step kk and s_waitcnt only asks for what the next MFMA pair needs, so the MFMA pipe never waits
// on LDS inside a slice.
//
// Operands of the asm block: %0..%7 accumulators acc[i][j] (i = A fragment 0..3, j = B fragment 0..1,
// operand i*2+j); %8..%11 LDS byte address of this lane's A row for step 0..3 (the XOR swizzle makes it
// lane- and step-specific); %12..%15 the same for B.  Immediate offsets select fragment and stage.
// The accumulators live in AGPRs (128 of them), which leaves 128 architectural VGPRs at two waves per SIMD.
// Scratch registers (clobbered): A fragments v[72:87] / v[88:103] (two sets), B fragments
// v[104:111] / v[112:119] / v[120:127] (three sets).  A fragment set is overwritten only several MFMA
// issue slots after its last reader.
//
// LDS reads return in order, so lgkmcnt(n) = "all but the n youngest reads have landed".
#pragma once

#define PRISM_DSR(dst, addr, off) "ds_read_b128 " dst ", " addr " offset:" #off "\n"
// the W fragment (b) is the instruction's first operand: the accumulator tile comes out transposed, i.e. a lane
// holds ONE row of A (token) and runs of 4 consecutive output columns, which the epilogues store as vectors
#define PRISM_MM(mn, acc, a, b) mn " " acc ", " b ", " a ", " acc "\n"
#define PRISM_WAIT(n) "s_waitcnt lgkmcnt(" #n ")\n"

// fragment registers
#define A0_0 "v[72:75]"
#define A0_1 "v[76:79]"
#define A0_2 "v[80:83]"
#define A0_3 "v[84:87]"
#define A1_0 "v[88:91]"
#define A1_1 "v[92:95]"
#define A1_2 "v[96:99]"
#define A1_3 "v[100:103]"
#define B0_0 "v[104:107]"
#define B0_1 "v[108:111]"
#define B1_0 "v[112:115]"
#define B1_1 "v[116:119]"
#define B2_0 "v[120:123]"
#define B2_1 "v[124:127]"

// one 16-deep step: 8 MFMAs from (a0..a3, b0, b1), with the 6 reads of the next step interleaved
#define PRISM_STEP_WITH_READS(mn, a0, a1, a2, a3, b0, b1, na0, na1, na2, na3, nb0, nb1, nA, nB, oa0, oa1, oa2, oa3, ob0, ob1) \
  PRISM_WAIT(3)                                                                                                     \
  PRISM_MM(mn, "%0", a0, b0) PRISM_DSR(nb0, nB, ob0)                                                                \
  PRISM_MM(mn, "%1", a0, b1) PRISM_DSR(nb1, nB, ob1)                                                                \
  PRISM_WAIT(4)                                                                                                     \
  PRISM_MM(mn, "%2", a1, b0) PRISM_DSR(na0, nA, oa0)                                                                \
  PRISM_MM(mn, "%3", a1, b1) PRISM_DSR(na1, nA, oa1)                                                                \
  PRISM_WAIT(5)                                                                                                     \
  PRISM_MM(mn, "%4", a2, b0) PRISM_DSR(na2, nA, oa2)                                                                \
  PRISM_MM(mn, "%5", a2, b1) PRISM_DSR(na3, nA, oa3)                                                                \
  PRISM_WAIT(6)                                                                                                     \
  PRISM_MM(mn, "%6", a3, b0)                                                                                        \
  PRISM_MM(mn, "%7", a3, b1)

#define PRISM_STEP_LAST(mn, a0, a1, a2, a3, b0, b1) \
  PRISM_WAIT(3) PRISM_MM(mn, "%0", a0, b0) PRISM_MM(mn, "%1", a0, b1) \
  PRISM_WAIT(2) PRISM_MM(mn, "%2", a1, b0) PRISM_MM(mn, "%3", a1, b1) \
  PRISM_WAIT(1) PRISM_MM(mn, "%4", a2, b0) PRISM_MM(mn, "%5", a2, b1) \
  PRISM_WAIT(0) PRISM_MM(mn, "%6", a3, b0) PRISM_MM(mn, "%7", a3, b1)

// one slice.  oa0..oa3: byte offsets of the 4 A fragments (stage included); ob0, ob1: of the 2 B fragments.
// Step kk reads through the address registers aA[kk] = v[56+kk], aB[kk] = v[60+kk].
#define PRISM_KSLICE_TEXT(mn, oa0, oa1, oa2, oa3, ob0, ob1)                                                          \
  PRISM_DSR(B0_0, "v60", ob0) PRISM_DSR(B0_1, "v60", ob1)                                                            \
  PRISM_DSR(A0_0, "v56", oa0) PRISM_DSR(A0_1, "v56", oa1) PRISM_DSR(A0_2, "v56", oa2) PRISM_DSR(A0_3, "v56", oa3)    \
  PRISM_STEP_WITH_READS(mn, A0_0, A0_1, A0_2, A0_3, B0_0, B0_1, A1_0, A1_1, A1_2, A1_3, B1_0, B1_1, "v57", "v61",   \
                        oa0, oa1, oa2, oa3, ob0, ob1)                                                                \
  PRISM_STEP_WITH_READS(mn, A1_0, A1_1, A1_2, A1_3, B1_0, B1_1, A0_0, A0_1, A0_2, A0_3, B2_0, B2_1, "v58", "v62",   \
                        oa0, oa1, oa2, oa3, ob0, ob1)                                                                \
  PRISM_STEP_WITH_READS(mn, A0_0, A0_1, A0_2, A0_3, B2_0, B2_1, A1_0, A1_1, A1_2, A1_3, B0_0, B0_1, "v59", "v63",   \
                        oa0, oa1, oa2, oa3, ob0, ob1)                                                                \
  PRISM_STEP_LAST(mn, A1_0, A1_1, A1_2, A1_3, B0_0, B0_1)

// The 8 direct-to-LDS loads of one slice for this wave: M0 = LDS destination of the instruction (stage
// base of the wave + 1 KiB per instruction), source = uniform base s[20:21] / s[22:23] (advanced by one
// slice = 128 bytes afterwards) + the lane's byte offset v[64..67] (A) / v[68..71] (B).
// %16 / %17: LDS byte address of the wave's first destination row in stage 0 of A / B.
#define PRISM_LDSLOAD(m0src, imm, voff, sbase) \
  "s_add_u32 m0, " m0src ", " #imm "\n s_nop 0\n global_load_lds_dwordx4 " voff ", " sbase "\n"
#define PRISM_STAGE_LOADS(st)                                                                                        \
  PRISM_LDSLOAD("%16", st + 0, "v64", "s[20:21]") PRISM_LDSLOAD("%16", st + 1024, "v65", "s[20:21]")                 \
  PRISM_LDSLOAD("%16", st + 2048, "v66", "s[20:21]") PRISM_LDSLOAD("%16", st + 3072, "v67", "s[20:21]")              \
  PRISM_LDSLOAD("%17", st + 0, "v68", "s[22:23]") PRISM_LDSLOAD("%17", st + 1024, "v69", "s[22:23]")                 \
  PRISM_LDSLOAD("%17", st + 2048, "v70", "s[22:23]") PRISM_LDSLOAD("%17", st + 3072, "v71", "s[22:23]")              \
  "s_add_u32 s20, s20, 128\n s_addc_u32 s21, s21, 0\n s_add_u32 s22, s22, 128\n s_addc_u32 s23, s23, 0\n"            \
  ""

#define PRISM_VMWAIT "s_waitcnt vmcnt(0)\n"

// The whole K loop of the tile.  Operands: %0..%7 accumulators (AGPRs); %8 / %9 LDS byte address of this lane's
// first A / B fragment row for step 0, stage 0 (steps 1..3 are that address ^ 32, ^ 64, ^ 96: the XOR swizzle
// only touches the chunk bits); %10 / %11 the lane's byte offset into A / W for its first load instruction;
// %12 byte distance between the rows of consecutive load instructions (8 rows); %13 / %14 base address of
// A / W (64-bit SGPR pairs); %15 number of slices.  Scratch: v[56:63] fragment addresses, v[64:71] load offsets,
// s[20:23] running bases, s24 slices left.
#define PRISM_KLOOP_TEXT(mn, ob1_s0, ob1_s1)                                                                          \
  "v_mov_b32 v56, %8\n v_xor_b32 v57, 32, %8\n v_xor_b32 v58, 64, %8\n v_xor_b32 v59, 96, %8\n"                      \
  "v_mov_b32 v60, %9\n v_xor_b32 v61, 32, %9\n v_xor_b32 v62, 64, %9\n v_xor_b32 v63, 96, %9\n"                      \
  /* load offsets: instruction j reads rows 8 j .. 8 j + 7; odd j carry the other swizzle phase (chunk ^ 4) */        \
  "v_mov_b32 v64, %10\n v_add_u32 v65, %12, v64\n v_add_u32 v66, %12, v65\n v_add_u32 v67, %12, v66\n"               \
  "v_xor_b32 v65, 64, v65\n v_xor_b32 v67, 64, v67\n"                                                                \
  "v_mov_b32 v68, %11\n v_add_u32 v69, %12, v68\n v_add_u32 v70, %12, v69\n v_add_u32 v71, %12, v70\n"               \
  "v_xor_b32 v69, 64, v69\n v_xor_b32 v71, 64, v71\n"                                                                \
  "s_mov_b64 s[20:21], %13\n s_mov_b64 s[22:23], %14\n s_mov_b32 s24, %15\n"                                         \
  PRISM_STAGE_LOADS(0)                                                                                              \
  PRISM_VMWAIT "s_barrier\n"                                                                                 \
  "L_loop_%=:\n"                                                                                                     \
  "s_cmp_lt_u32 s24, 2\n s_cbranch_scc1 L_skip1_%=\n"                                                                \
  PRISM_STAGE_LOADS(32768)                                                                                          \
  "L_skip1_%=:\n"                                                                                                    \
  PRISM_KSLICE_TEXT(mn, 0, 4096, 8192, 12288, 0, ob1_s0)                                                             \
  PRISM_VMWAIT "s_barrier\n"                                                                                 \
  "s_sub_u32 s24, s24, 1\n s_cmp_eq_u32 s24, 0\n s_cbranch_scc1 L_done_%=\n"                                         \
  "s_cmp_lt_u32 s24, 2\n s_cbranch_scc1 L_skip0_%=\n"                                                                \
  PRISM_STAGE_LOADS(0)                                                                                              \
  "L_skip0_%=:\n"                                                                                                    \
  PRISM_KSLICE_TEXT(mn, 32768, 36864, 40960, 45056, 32768, ob1_s1)                                                   \
  PRISM_VMWAIT "s_barrier\n"                                                                                 \
  "s_sub_u32 s24, s24, 1\n s_cmp_lg_u32 s24, 0\n s_cbranch_scc1 L_loop_%=\n"                                         \
  "L_done_%=:\n"                                                                                                     \
  "s_waitcnt vmcnt(0)\n s_nop 15\n s_nop 15\n" /* the last MFMA results must not be read by the code that follows too early */

#define PRISM_KLOOP_CLOBBERS                                                                                          \
  "v56", "v57", "v58", "v59", "v60", "v61", "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71",    \
      "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", \
      "v88", "v89", "v90", "v91", "v92", "v93", "v94", "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102",     \
      "v103", "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", \
      "v117", "v118", "v119", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "s20", "s21", "s22",   \
      "s23", "s24", "scc", "memory"

#define PRISM_KLOOP(mn, acc, aA0, aB0, gA0, gB0, stride, baseA, baseB, nk, ldsA, ldsB, ob1_s0, ob1_s1)               \
  asm volatile(PRISM_KLOOP_TEXT(mn, ob1_s0, ob1_s1)                                                                  \
               : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[2][0]), "+a"(acc[2][1]), \
                 "+a"(acc[3][0]), "+a"(acc[3][1])                                                                    \
               : "v"(aA0), "v"(aB0), "v"(gA0), "v"(gB0), "s"(stride), "s"(baseA), "s"(baseB), "s"(nk), "s"(ldsA), "s"(ldsB)                                                                                \
               : PRISM_KLOOP_CLOBBERS)
