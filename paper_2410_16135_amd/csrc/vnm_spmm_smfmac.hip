// vnm_spmm on the 2:4 sparse matrix cores of gfx950 (V_SMFMAC_F32_32X32X32_F16).
//
// Computes Y^T = W' . X^T so that the compressed weight is the sparse A operand (rows = output
// channels) and the activations are the dense B operand (columns = tokens).  What makes V:N:M differ
// from plain 2:4 (Appendix A) is that the B rows a row block needs are the 4 kept input columns of
// each of its column blocks, and they differ from row block to row block.  Design:
//
//   * X is first re-laid by the staging pass (vnm_stage.hip) into per-(token tile, K step) images
//     [raw input column][token].  A workgroup owns WR row blocks x 128 tokens and streams the images
//     of its token tile through a ring of LDS buffers with asynchronous global->LDS copies
//     (global_load_lds_dwordx4: no registers, no VALU work, fully coalesced).
//   * The raw image (all M columns of every block) is shared by the WR row blocks of the
//     workgroup; the per-row-block gather happens when a wave reads its B operand: each
//     ds_read_b64_tr_b16 fetches, for 16 tokens, the 4 kept columns of one column block -- the rows
//     are chosen per lane from the packed column table -- and hands every lane the 4 K-consecutive
//     values of its token.  LDS read traffic is exactly the gathered operand; there is no select
//     arithmetic.
//   * A wave owns one row block (V rows = V/32 A tiles) x TW tokens (TW/32 B tiles).  Its A operand
//     (kept values in lane order + 2-bit positions) comes straight from the packed copy in global
//     memory, one 16-byte load per lane and tile; accumulators stay in registers for the whole K
//     loop.
//   * The K loop is written in assembly (see below), in two variants: one column table per
//     64-row block (V = 64, 128) or one per 32-row tile (V = 32).
#include <type_traits>
#include "vnm_internal.h"

namespace vnm {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
#define VNM_LDS(T) __attribute__((address_space(3))) T*
#define VNM_GLB(T) __attribute__((address_space(1))) T*

// ds_read_b64_tr_b16 (used by the loop below): 16 lanes x 8 bytes in, transposed out: lanes
// 4j..4j+3 of a 16-lane group address row j (16 consecutive fp16 of it), and lane i receives
// element i of each of the 4 rows.

// ---------------------------------------------------------------------------------------------
// Steady-state K loop for V = 64 (2 A tiles x 4 B tiles per wave), written in assembly.
//
// Why assembly: the loop keeps two kinds of vector-memory operations in flight at once -- the
// register loads of the A operand two steps ahead and the asynchronous global->LDS copies of the
// image NBUF-1 steps ahead -- and must wait for the older ones while the younger ones keep flying
// (vmcnt counts both, in issue order).  Compiled code drains everything (vmcnt(0)) at each use,
// which serialises the copies with the multiply.  Here every wait is explicit; the schedule of one
// step is described at VNM_ASM_STEP.
// The body is unrolled three times so that the three A register sets rotate by name.
// Fixed registers (declared clobbered):
//   v[186:189] B row addresses, v190 v191 scratch, v[192:223] B tiles 0..3,
//   A sets {values tile 0, values tile 1, index word, column table}:
//     set0 v[224:227] v[228:231] v232 v233, set1 v[234:237] v[238:241] v242 v243,
//     set2 v[244:247] v[248:251] v252 v253
//   s[80:81] A values ptr, s[82:83] index ptr, s[84:85] column table ptr, s[86:87] image ptr,
//   s[88:89] copy source
// The accumulators leave the loop in registers that the compiled epilogue reads with ordinary
// vector instructions.  The compiler cannot see the matrix instructions inside the assembly block,
// so it inserts none of the wait states the hardware requires between a matrix-core write of a
// register and a vector-ALU read of it (up to 18 for a 16-pass instruction): the block owns that
// hazard and ends with 24 idle states of its own, whatever else stands between the last
// v_smfmac and the exit.
// Validated with the HIP compiler of ROCm 7.2.0 (HIP 7.2.26015, AMD clang 22.0.0git roc-7.2.0); the loops name physical registers
// v178-v253 and s80-s89 and declare them clobbered, which needs the compiler to keep its own live
// values below them: a build that fails with "register allocation" errors here means a newer
// compiler needs more registers around the block.
#define VNM_ASM_MFMA_DRAIN "s_nop 15\n s_nop 7\n"
#define VNM_ASM_COPY(K4096)                                   \
  "s_add_u32 %[tci], %[woff], " #K4096 "\n"                   \
  "s_min_u32 %[tci], %[tci], %[clamp]\n"                      \
  "s_add_u32 s88, s86, %[tci]\n"                              \
  "s_addc_u32 s89, s87, 0\n"                                  \
  "s_add_u32 m0, %[wr], %[tci]\n"                             \
  "s_nop 0\n"                                                 \
  "global_load_lds_dwordx4 %[voff16], s[88:89]\n"
// Copies per wave and image, split in two groups issued under two different MFMAs.
// 4-wave workgroups: chunk stride 4 KiB; 8-wave workgroups: 8 KiB.
#define VNM_C4_3A VNM_ASM_COPY(0) VNM_ASM_COPY(4096)
#define VNM_C4_3B VNM_ASM_COPY(8192)
#define VNM_C4_4A VNM_ASM_COPY(0) VNM_ASM_COPY(4096)
#define VNM_C4_4B VNM_ASM_COPY(8192) VNM_ASM_COPY(12288)
#define VNM_C4_5A VNM_C4_4A VNM_ASM_COPY(8192)
#define VNM_C4_5B VNM_ASM_COPY(12288) VNM_ASM_COPY(16384)
#define VNM_C4_6A VNM_C4_5A
#define VNM_C4_6B VNM_C4_5B VNM_ASM_COPY(20480)
#define VNM_C4_7A VNM_C4_5A VNM_ASM_COPY(12288)
#define VNM_C4_7B VNM_ASM_COPY(16384) VNM_ASM_COPY(20480) VNM_ASM_COPY(24576)
#define VNM_C4_8A VNM_C4_7A
#define VNM_C4_8B VNM_C4_7B VNM_ASM_COPY(28672)
#define VNM_C4_9A VNM_C4_7A VNM_ASM_COPY(16384)
#define VNM_C4_9B VNM_ASM_COPY(20480) VNM_ASM_COPY(24576) VNM_ASM_COPY(28672) VNM_ASM_COPY(32768)
#define VNM_C4_10A VNM_C4_9A
#define VNM_C4_10B VNM_C4_9B VNM_ASM_COPY(36864)
#define VNM_C8_2A VNM_ASM_COPY(0)
#define VNM_C8_2B VNM_ASM_COPY(8192)
#define VNM_C8_3A VNM_ASM_COPY(0) VNM_ASM_COPY(8192)
#define VNM_C8_3B VNM_ASM_COPY(16384)
#define VNM_C8_4A VNM_C8_3A
#define VNM_C8_4B VNM_ASM_COPY(16384) VNM_ASM_COPY(24576)
#define VNM_C8_5A VNM_C8_3A VNM_ASM_COPY(16384)
#define VNM_C8_5B VNM_ASM_COPY(24576) VNM_ASM_COPY(32768)

// two of the four transposing reads of one B tile (rows A0, A1 -> register pairs R0, R1)
#define VNM_ASM_READ2(OFF, R0, A0, R1, A1)                                     \
  "ds_read_b64_tr_b16 v[" #R0 ":" #R0 "+1], v" #A0 " offset:" #OFF "\n"        \
  "ds_read_b64_tr_b16 v[" #R1 ":" #R1 "+1], v" #A1 " offset:" #OFF "\n"
#define VNM_ASM_READ4(OFF, R0, R1, R2, R3)                                     \
  VNM_ASM_READ2(OFF, R0, 186, R1, 187) VNM_ASM_READ2(OFF, R2, 188, R3, 189)

#define VNM_ASM_A_ADVANCE                                                      \
  "s_add_u32 s80, s80, 2048\n s_addc_u32 s81, s81, 0\n"                        \
  "s_add_u32 s82, s82, 256\n s_addc_u32 s83, s83, 0\n"                         \
  "s_add_u32 s84, s84, 32\n s_addc_u32 s85, s85, 0\n"
#define VNM_ASM_LOAD_A(W0, W1, IDX, PC)                                        \
  "global_load_dwordx4 v[" W0 "], %[voff16], s[80:81]\n"                       \
  "global_load_dwordx4 v[" W1 "], %[voff16], s[80:81] offset:1024\n"           \
  "global_load_dword v" IDX ", %[voffi], s[82:83]\n"                           \
  "global_load_dword v" PC ", %[voffp], s[84:85]\n"                            \
  VNM_ASM_A_ADVANCE

// B row addresses of a step from its column table register PC (4 x 8-bit row offsets) and ring slot
#define VNM_ASM_ADDR(PC)                                                                          \
      "v_add_u32 v190, %[rd], %[vtok]\n"                                                          \
      "v_and_b32 v191, 0xff, v" PC "\n"                                                           \
      "v_mad_u32_u24 v186, v191, %[pitch], v190\n"                                                \
      "v_bfe_u32 v191, v" PC ", 8, 8\n"                                                           \
      "v_mad_u32_u24 v187, v191, %[pitch], v190\n"                                                \
      "v_bfe_u32 v191, v" PC ", 16, 8\n"                                                          \
      "v_mad_u32_u24 v188, v191, %[pitch], v190\n"                                                \
      "v_lshrrev_b32 v191, 24, v" PC "\n"                                                         \
      "v_mad_u32_u24 v189, v191, %[pitch], v190\n"

// One K step.  CUR = A set of this step, NPC = column table register of the next step's set (landed
// by the time it is used), LOAD = set that receives A(s+2).
// The memory instructions are spread between the eight MFMAs, at most three after each, so that
// the LDS, the vector-memory path and the matrix pipe are all fed continuously instead of in
// bursts (in-order issue would otherwise let a full vector-memory queue hold back the LDS reads
// behind it).  B tiles are requested two tiles (four MFMAs) ahead of their use, across the step
// boundary; at every use exactly the four reads of the following tile may still be in flight, so
// every wait is lgkmcnt(4).  Order of one step:
//   tiles 0,1 multiplied | under them: A(s+2) requested, tiles 2,3 of this step requested, the
//       scalar pointer and ring updates
//   wait for A(s+1) and image s+1 (vmcnt), barrier -- every wave has left step s-1, its ring slot
//       is free
//   tiles 2,3 multiplied | under them: next step's row addresses, copies of the image NBUF-1
//       ahead, next step's tiles 0,1
// Nothing but the two waits stands between the fourth and the fifth MFMA: the barrier brings the
// two waves of a SIMD to the same point of the step, so whatever is issued next to it is issued by
// both while the matrix pipe has nothing queued (measured: 800 -> 775 clocks per step).
#define VNM_ASM_STEP(CW0, CW1, CIDX, NPC, LW0, LW1, LIDX, LPC, COPY_A, COPY_B, VMWSTR)             \
      "s_waitcnt lgkmcnt(4)\n s_nop 0\n"                                                          \
      "v_smfmac_f32_32x32x32_f16 %[a00], v[" CW0 "], v[192:199], v" CIDX "\n"                     \
      "global_load_dwordx4 v[" LW0 "], %[voff16], s[80:81]\n"                                     \
      VNM_ASM_READ2(128, 208, 186, 210, 187)                                                      \
      "v_smfmac_f32_32x32x32_f16 %[a10], v[" CW1 "], v[192:199], v" CIDX " abid:1\n"              \
      "global_load_dwordx4 v[" LW1 "], %[voff16], s[80:81] offset:1024\n"                         \
      VNM_ASM_READ2(128, 212, 188, 214, 189)                                                      \
      "s_waitcnt lgkmcnt(4)\n s_nop 0\n"                                                          \
      "v_smfmac_f32_32x32x32_f16 %[a01], v[" CW0 "], v[200:207], v" CIDX "\n"                     \
      "global_load_dword v" LIDX ", %[voffi], s[82:83]\n"                                         \
      VNM_ASM_READ2(192, 216, 186, 218, 187)                                                      \
      "s_add_u32 s80, s80, 2048\n s_addc_u32 s81, s81, 0\n"                                       \
      "s_add_u32 s82, s82, 256\n s_addc_u32 s83, s83, 0\n"                                        \
      "s_add_u32 %[rd], %[rd], %[img]\n s_cmp_eq_u32 %[rd], %[lend]\n s_cselect_b32 %[rd], %[lbeg], %[rd]\n" \
      "v_smfmac_f32_32x32x32_f16 %[a11], v[" CW1 "], v[200:207], v" CIDX " abid:1\n"              \
      "global_load_dword v" LPC ", %[voffp], s[84:85]\n"                                          \
      VNM_ASM_READ2(192, 220, 188, 222, 189)                                                      \
      "s_add_u32 s84, s84, 32\n s_addc_u32 s85, s85, 0\n"                                         \
      "s_waitcnt vmcnt(" VMWSTR ")\n"                                                             \
      "s_barrier\n"                                                                               \
      "s_waitcnt lgkmcnt(4)\n s_nop 0\n"                                                          \
      "v_smfmac_f32_32x32x32_f16 %[a02], v[" CW0 "], v[208:215], v" CIDX "\n"                     \
      VNM_ASM_ADDR(NPC)                                                                           \
      VNM_ASM_READ2(0, 192, 186, 194, 187)                                                        \
      COPY_A                                                                                      \
      "v_smfmac_f32_32x32x32_f16 %[a12], v[" CW1 "], v[208:215], v" CIDX " abid:1\n"              \
      VNM_ASM_READ2(0, 196, 188, 198, 189)                                                        \
      COPY_B                                                                                      \
      "s_add_u32 %[wr], %[wr], %[img]\n s_cmp_eq_u32 %[wr], %[lend]\n s_cselect_b32 %[wr], %[lbeg], %[wr]\n" \
      "s_add_u32 s86, s86, %[img]\n s_addc_u32 s87, s87, 0\n"                                     \
      "s_waitcnt lgkmcnt(4)\n s_nop 0\n"                                                          \
      "v_smfmac_f32_32x32x32_f16 %[a03], v[" CW0 "], v[216:223], v" CIDX "\n"                     \
      VNM_ASM_READ2(64, 200, 186, 202, 187)                                                       \
      "v_smfmac_f32_32x32x32_f16 %[a13], v[" CW1 "], v[216:223], v" CIDX " abid:1\n"              \
      VNM_ASM_READ2(64, 204, 188, 206, 189)                                                       \
      "s_sub_u32 %[n], %[n], 1\n"                                                                 \
      "s_cmp_eq_u32 %[n], 0\n"                                                                    \
      "s_cbranch_scc1 9f\n"

#define VNM_ASM_LOOP_V64(COPY_A, COPY_B, VMWSTR)                                                  \
  asm volatile(                                                                                   \
      "s_mov_b32 s80, %[pa_lo]\n s_mov_b32 s81, %[pa_hi]\n"                                       \
      "s_mov_b32 s82, %[pi_lo]\n s_mov_b32 s83, %[pi_hi]\n"                                       \
      "s_mov_b32 s84, %[pc_lo]\n s_mov_b32 s85, %[pc_hi]\n"                                       \
      "s_mov_b32 s86, %[xs_lo]\n s_mov_b32 s87, %[xs_hi]\n"                                       \
      VNM_ASM_LOAD_A("224:227", "228:231", "232", "233")                                          \
      VNM_ASM_LOAD_A("234:237", "238:241", "242", "243")                                          \
      "s_waitcnt vmcnt(0) lgkmcnt(0)\n"                                                           \
      "s_barrier\n"                                                                               \
      VNM_ASM_ADDR("233")                                                                         \
      VNM_ASM_READ4(0, 192, 194, 196, 198)                                                        \
      VNM_ASM_READ4(64, 200, 202, 204, 206)                                                       \
      "1:\n"                                                                                \
      VNM_ASM_STEP("224:227", "228:231", "232", "243", "244:247", "248:251", "252", "253", COPY_A, COPY_B, VMWSTR) \
      VNM_ASM_STEP("234:237", "238:241", "242", "253", "224:227", "228:231", "232", "233", COPY_A, COPY_B, VMWSTR) \
      VNM_ASM_STEP("244:247", "248:251", "252", "233", "234:237", "238:241", "242", "243", COPY_A, COPY_B, VMWSTR) \
      "s_branch 1b\n"                                                                             \
      "9:\n"                                                                                      \
      "s_waitcnt vmcnt(0) lgkmcnt(0)\n"                                                           \
      "s_barrier\n"                                                                               \
      VNM_ASM_MFMA_DRAIN                                                                          \
      : [a00] "+v"(acc[0][0]), [a01] "+v"(acc[0][1]), [a02] "+v"(acc[0][2]), [a03] "+v"(acc[0][3]), \
        [a10] "+v"(acc[1][0]), [a11] "+v"(acc[1][1]), [a12] "+v"(acc[1][2]), [a13] "+v"(acc[1][3]), \
        [rd] "+&s"(l_rd), [wr] "+&s"(l_wr), [n] "+&s"(l_n), [tci] "=&s"(l_tci)                    \
      : [pa_lo] "s"(l_pa_lo), [pa_hi] "s"(l_pa_hi), [pi_lo] "s"(l_pi_lo), [pi_hi] "s"(l_pi_hi),   \
        [pc_lo] "s"(l_pc_lo), [pc_hi] "s"(l_pc_hi), [xs_lo] "s"(l_xs_lo), [xs_hi] "s"(l_xs_hi),   \
        [voff16] "v"(l_voff16), [voffi] "v"(l_voffi), [voffp] "v"(l_voffp), [vtok] "v"(l_vtok),   \
        [woff] "s"(l_woff), [clamp] "s"(l_clamp), [pitch] "s"(l_pitch), [img] "s"(l_img),         \
        [lbeg] "s"(l_lbeg), [lend] "s"(l_lend)                                                    \
      : "memory", "scc", "m0",                                                                    \
        "v186", "v187", "v188", "v189", "v190", "v191",                                           \
        "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", "v200", "v201", "v202", "v203", \
        "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211", "v212", "v213", "v214", "v215", \
        "v216", "v217", "v218", "v219", "v220", "v221", "v222", "v223", "v224", "v225", "v226", "v227", \
        "v228", "v229", "v230", "v231", "v232", "v233", "v234", "v235", "v236", "v237", "v238", "v239", \
        "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", "v248", "v249", "v250", "v251", \
        "v252", "v253",                                                                           \
        "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89")

// ---------------------------------------------------------------------------------------------
// The same loop for packed row blocks that carry two column tables (V = 32: the two 32-row tiles of
// a wave belong to different row blocks of the pattern and gather different columns).  Every MFMA
// then has a B operand of its own: 8 operands of 4 reads per step, kept in a ring of four 8-register
// slots; operand i + 3 is requested right after MFMA i into the slot MFMA i - 1 has just used, so at
// every use the 8 reads of the two following operands may still be in flight (lgkmcnt(8)).
// Registers: v178 v179 scratch, v[180:183] row addresses of table 0, v[184:187] of table 1,
// slots v[188:195] v[196:203] v[204:211] v[212:219], A sets {values tile 0, values tile 1, index
// word, column tables 0 and 1} with even-aligned tuples: {v[220:223] v[224:227] v230 v[228:229]},
// {v[232:235] v[236:239] v242 v[240:241]}, {v[244:247] v[248:251] v243 v[252:253]}.
#define VNM_D_READ4(OFF, X, A0)                                                                   \
  "ds_read_b64_tr_b16 v[" #X ":" #X "+1], v[" #A0 "] offset:" #OFF "\n"                           \
  "ds_read_b64_tr_b16 v[" #X "+2:" #X "+3], v[" #A0 "+1] offset:" #OFF "\n"                       \
  "ds_read_b64_tr_b16 v[" #X "+4:" #X "+5], v[" #A0 "+2] offset:" #OFF "\n"                       \
  "ds_read_b64_tr_b16 v[" #X "+6:" #X "+7], v[" #A0 "+3] offset:" #OFF "\n"
#define VNM_D_A_ADVANCE                                                        \
  "s_add_u32 s80, s80, 2048\n s_addc_u32 s81, s81, 0\n"                        \
  "s_add_u32 s82, s82, 256\n s_addc_u32 s83, s83, 0\n"                         \
  "s_add_u32 s84, s84, 64\n s_addc_u32 s85, s85, 0\n"
#define VNM_D_LOAD_A(W0, W1, IDX, PC)                                          \
  "global_load_dwordx4 v[" W0 "], %[voff16], s[80:81]\n"                       \
  "global_load_dwordx4 v[" W1 "], %[voff16], s[80:81] offset:1024\n"           \
  "global_load_dword v" IDX ", %[voffi], s[82:83]\n"                           \
  "global_load_dwordx2 v[" PC "], %[voffp], s[84:85]\n"                        \
  VNM_D_A_ADVANCE
#define VNM_D_ADDR1(PC, A0, A1, A2, A3)                                                           \
      "v_and_b32 v179, 0xff, v" PC "\n"                                                           \
      "v_mad_u32_u24 v" #A0 ", v179, %[pitch], v178\n"                                            \
      "v_bfe_u32 v179, v" PC ", 8, 8\n"                                                           \
      "v_mad_u32_u24 v" #A1 ", v179, %[pitch], v178\n"                                            \
      "v_bfe_u32 v179, v" PC ", 16, 8\n"                                                          \
      "v_mad_u32_u24 v" #A2 ", v179, %[pitch], v178\n"                                            \
      "v_lshrrev_b32 v179, 24, v" PC "\n"                                                         \
      "v_mad_u32_u24 v" #A3 ", v179, %[pitch], v178\n"
#define VNM_D_ADDR(PC0, PC1)                                                                      \
      "v_add_u32 v178, %[rd], %[vtok]\n"                                                          \
      VNM_D_ADDR1(PC0, 180, 181, 182, 183) VNM_D_ADDR1(PC1, 184, 185, 186, 187)
#define VNM_D_W "s_waitcnt lgkmcnt(8)\n s_nop 0\n"
// CUR set = (CW0, CW1, CIDX); NPC0/NPC1 = column tables of the next step's set; LOAD set receives A(s+2)
#define VNM_D_STEP(CW0, CW1, CIDX, NPC0, NPC1, LW0, LW1, LIDX, LPC, COPY_A, COPY_B, VMWSTR)        \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a00], v[" CW0 "], v[188:195], v" CIDX "\n"                     \
      "global_load_dwordx4 v[" LW0 "], %[voff16], s[80:81]\n"                                     \
      VNM_D_READ4(64, 212, 184)                                                                   \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a10], v[" CW1 "], v[196:203], v" CIDX " abid:1\n"              \
      "global_load_dwordx4 v[" LW1 "], %[voff16], s[80:81] offset:1024\n"                         \
      VNM_D_READ4(128, 188, 180)                                                                  \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a01], v[" CW0 "], v[204:211], v" CIDX "\n"                     \
      "global_load_dword v" LIDX ", %[voffi], s[82:83]\n"                                         \
      VNM_D_READ4(128, 196, 184)                                                                  \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a11], v[" CW1 "], v[212:219], v" CIDX " abid:1\n"              \
      "global_load_dwordx2 v[" LPC "], %[voffp], s[84:85]\n"                                      \
      VNM_D_READ4(192, 204, 180)                                                                  \
      VNM_D_A_ADVANCE                                                                             \
      "s_add_u32 %[rd], %[rd], %[img]\n s_cmp_eq_u32 %[rd], %[lend]\n s_cselect_b32 %[rd], %[lbeg], %[rd]\n" \
      "s_waitcnt vmcnt(" VMWSTR ")\n"                                                             \
      "s_barrier\n"                                                                               \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a02], v[" CW0 "], v[188:195], v" CIDX "\n"                     \
      VNM_D_READ4(192, 212, 184)                                                                  \
      COPY_A                                                                                      \
      VNM_D_ADDR(NPC0, NPC1)                                                                      \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a12], v[" CW1 "], v[196:203], v" CIDX " abid:1\n"              \
      VNM_D_READ4(0, 188, 180)                                                                    \
      COPY_B                                                                                      \
      "s_add_u32 %[wr], %[wr], %[img]\n s_cmp_eq_u32 %[wr], %[lend]\n s_cselect_b32 %[wr], %[lbeg], %[wr]\n" \
      "s_add_u32 s86, s86, %[img]\n s_addc_u32 s87, s87, 0\n"                                     \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a03], v[" CW0 "], v[204:211], v" CIDX "\n"                     \
      VNM_D_READ4(0, 196, 184)                                                                    \
      VNM_D_W                                                                                     \
      "v_smfmac_f32_32x32x32_f16 %[a13], v[" CW1 "], v[212:219], v" CIDX " abid:1\n"              \
      VNM_D_READ4(64, 204, 180)                                                                   \
      "s_sub_u32 %[n], %[n], 1\n"                                                                 \
      "s_cmp_eq_u32 %[n], 0\n"                                                                    \
      "s_cbranch_scc1 9f\n"

#define VNM_ASM_LOOP_D(COPY_A, COPY_B, VMWSTR)                                                    \
  asm volatile(                                                                                   \
      "s_mov_b32 s80, %[pa_lo]\n s_mov_b32 s81, %[pa_hi]\n"                                       \
      "s_mov_b32 s82, %[pi_lo]\n s_mov_b32 s83, %[pi_hi]\n"                                       \
      "s_mov_b32 s84, %[pc_lo]\n s_mov_b32 s85, %[pc_hi]\n"                                       \
      "s_mov_b32 s86, %[xs_lo]\n s_mov_b32 s87, %[xs_hi]\n"                                       \
      VNM_D_LOAD_A("220:223", "224:227", "230", "228:229")                                        \
      VNM_D_LOAD_A("232:235", "236:239", "242", "240:241")                                        \
      "s_waitcnt vmcnt(0) lgkmcnt(0)\n"                                                           \
      "s_barrier\n"                                                                               \
      VNM_D_ADDR("228", "229")                                                                    \
      VNM_D_READ4(0, 188, 180)                                                                    \
      VNM_D_READ4(0, 196, 184)                                                                    \
      VNM_D_READ4(64, 204, 180)                                                                   \
      "1:\n"                                                                                \
      VNM_D_STEP("220:223", "224:227", "230", "240", "241", "244:247", "248:251", "243", "252:253", COPY_A, COPY_B, VMWSTR) \
      VNM_D_STEP("232:235", "236:239", "242", "252", "253", "220:223", "224:227", "230", "228:229", COPY_A, COPY_B, VMWSTR) \
      VNM_D_STEP("244:247", "248:251", "243", "228", "229", "232:235", "236:239", "242", "240:241", COPY_A, COPY_B, VMWSTR) \
      "s_branch 1b\n"                                                                             \
      "9:\n"                                                                                      \
      "s_waitcnt vmcnt(0) lgkmcnt(0)\n"                                                           \
      "s_barrier\n"                                                                               \
      VNM_ASM_MFMA_DRAIN                                                                          \
      : [a00] "+v"(acc[0][0]), [a01] "+v"(acc[0][1]), [a02] "+v"(acc[0][2]), [a03] "+v"(acc[0][3]), \
        [a10] "+v"(acc[1][0]), [a11] "+v"(acc[1][1]), [a12] "+v"(acc[1][2]), [a13] "+v"(acc[1][3]), \
        [rd] "+&s"(l_rd), [wr] "+&s"(l_wr), [n] "+&s"(l_n), [tci] "=&s"(l_tci)                    \
      : [pa_lo] "s"(l_pa_lo), [pa_hi] "s"(l_pa_hi), [pi_lo] "s"(l_pi_lo), [pi_hi] "s"(l_pi_hi),   \
        [pc_lo] "s"(l_pc_lo), [pc_hi] "s"(l_pc_hi), [xs_lo] "s"(l_xs_lo), [xs_hi] "s"(l_xs_hi),   \
        [voff16] "v"(l_voff16), [voffi] "v"(l_voffi), [voffp] "v"(l_voffp), [vtok] "v"(l_vtok),   \
        [woff] "s"(l_woff), [clamp] "s"(l_clamp), [pitch] "s"(l_pitch), [img] "s"(l_img),         \
        [lbeg] "s"(l_lbeg), [lend] "s"(l_lend)                                                    \
      : "memory", "scc", "m0",                                                                    \
        "v178", "v179", "v180", "v181", "v182", "v183", "v184", "v185",                           \
        "v186", "v187", "v188", "v189", "v190", "v191",                                           \
        "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", "v200", "v201", "v202", "v203", \
        "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211", "v212", "v213", "v214", "v215", \
        "v216", "v217", "v218", "v219", "v220", "v221", "v222", "v223", "v224", "v225", "v226", "v227", \
        "v228", "v229", "v230", "v231", "v232", "v233", "v234", "v235", "v236", "v237", "v238", "v239", \
        "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", "v248", "v249", "v250", "v251", \
        "v252", "v253",                                                                           \
        "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89")

struct SpmmArgs {
  const unsigned char* Xs; int64_t T;
  const uint4* pa; const unsigned short* pidx; const unsigned* pcol;
  int64_t out, R, S;
  int M;
  int image_bytes;   // multiple of 1024
  void* Y; int64_t ldy;
  int vec_store;     // Y and ldy allow 4-wide stores
  int wide_store;    // fp16 Y: 16-byte aligned base and ldy % 8 == 0 (LDS-transposed epilogue)
  int y_fp32;
  // split K: workgroup z handles K steps [z * ks_steps, min(S, (z + 1) * ks_steps)) and writes its
  // partial product to Y + z * z_stride elements (an fp32 scratch then, summed by a second kernel)
  int64_t ks_steps, z_stride;
  // fused epilogue (null = none): bias per weight row, destination channel per weight row
  const _Float16* bias; const int* perm_out;
};

// One K step = 8 column blocks = 8*M raw input columns = 32 compacted K = one staged image.
// NCW: wave-wide 1 KiB copies per wave and image (V = 64 assembly loop; 0 elsewhere).
// NBUF: depth of the LDS image ring.
// DUAL: the packed row blocks carry two column tables (V = 32 patterns), assembly loop only.
// FUSED: the epilogue looks at bias and perm_out (the plain instantiation ignores them and is exactly
// the kernel the benchmark times).
template <int V, int TW, int WR, int WT, int NCW, int NBUF, bool DUAL, bool FUSED>
__global__ void __launch_bounds__(64 * WR * WT)
spmm_smfmac_kernel(const SpmmArgs a) {
  constexpr int AT = V / 32, BT = TW / 32, NW = WR * WT;
  static_assert(WT * TW == kTokTile, "a workgroup spans one staged token tile");
  static_assert(BT <= 4 && AT <= 4, "tiling assumed by the step body");
  constexpr int P = kImagePitch;
  static_assert(V == 64 && TW == 128 && NCW > 0, "the K loop exists as the assembly loop for 64-row blocks only");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave / WT, wt = wave % WT;
  const int64_t r = (int64_t)blockIdx.y * WR + wr;
  const bool r_valid = r < a.R;
  const int64_t rr = r_valid ? r : a.R - 1;      // out-of-range waves compute a valid row block, store nothing
  const int64_t t0 = (int64_t)blockIdx.x * kTokTile;
  const int64_t s0 = (int64_t)blockIdx.z * a.ks_steps;
  const int64_t S = (a.S - s0) < a.ks_steps ? (a.S - s0) : a.ks_steps;   // steps of this workgroup
  const int64_t rs0 = rr * a.S + s0;                                      // its first (row block, step)
  const int img = a.image_bytes;
  const int n_ci = img / 1024;                   // wave-wide copies per image
  const int ncw = (n_ci + NW - 1) / NW;          // copies per wave and image

  f16v acc[AT][BT];
#pragma unroll
  for (int i = 0; i < AT; ++i)
#pragma unroll
    for (int j = 0; j < BT; ++j)
#pragma unroll
      for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.f;

  // B-operand lane roles
  const int hB = lane >> 5, tg = (lane >> 4) & 1, kq = (lane & 15) >> 2, q = lane & 3;
  const unsigned lds0 = (unsigned)(size_t)(VNM_LDS(unsigned char))smem;
  const unsigned tokoff = (unsigned)((wt * TW + tg * 16 + q * 4) * 2);

  const unsigned char* xs_tile = a.Xs + ((int64_t)blockIdx.x * a.S + s0) * img;
  // copy this wave's share of image s into ring slot `slot`; chunks beyond the image are clamped to
  // its last chunk (an idempotent duplicate) so that every wave issues the same number of copies
  auto copy_image = [&](int64_t s, int slot) {
    const unsigned char* src = xs_tile + s * img + lane * 16;
    for (int k = 0; k < ncw; ++k) {
      int ci = wave + k * NW;
      ci = ci < n_ci ? ci : n_ci - 1;
      __builtin_amdgcn_global_load_lds((VNM_GLB(void))(src + ci * 1024),
                                       (VNM_LDS(void))(smem + slot * img + ci * 1024), 16, 0, 0);
    }
  };

  // prologue: the first NBUF-1 images (the assembly loop waits for them together with its first
  // A operands, one memory latency instead of two)
  for (int k = 0; k < NBUF - 1 && k < S; ++k) copy_image(k, k);

  {
    // All S steps run in the assembly loop.  Every step requests the image NBUF-1 steps ahead and
    // the A operand 2 steps ahead without looking at S: near the end these requests reach past the
    // tile's images and past the row block's operands, into the next tile / row block or into the
    // slack that the staged buffer (3 images) and the packed weight (8 KiB) carry for this
    // purpose; what they fetch is never used.
    {
      const uint64_t pa_p = (uint64_t)(a.pa + rs0 * AT * 64);
      const uint64_t pi_p = (uint64_t)(a.pidx + rs0 * 64 * AT);
      const uint64_t pc_p = (uint64_t)(a.pcol + rs0 * (DUAL ? 16 : 8));
      const uint64_t xs_p = (uint64_t)(xs_tile + (int64_t)(NBUF - 1) * img);
      unsigned l_pa_lo = __builtin_amdgcn_readfirstlane((unsigned)pa_p), l_pa_hi = __builtin_amdgcn_readfirstlane((unsigned)(pa_p >> 32));
      unsigned l_pi_lo = __builtin_amdgcn_readfirstlane((unsigned)pi_p), l_pi_hi = __builtin_amdgcn_readfirstlane((unsigned)(pi_p >> 32));
      unsigned l_pc_lo = __builtin_amdgcn_readfirstlane((unsigned)pc_p), l_pc_hi = __builtin_amdgcn_readfirstlane((unsigned)(pc_p >> 32));
      unsigned l_xs_lo = __builtin_amdgcn_readfirstlane((unsigned)xs_p), l_xs_hi = __builtin_amdgcn_readfirstlane((unsigned)(xs_p >> 32));
      unsigned l_voff16 = lane * 16, l_voffi = lane * 4, l_voffp = (hB * 4 + kq) * (DUAL ? 8 : 4), l_vtok = tokoff;
      unsigned l_woff = wave * 1024, l_clamp = (n_ci - 1) * 1024, l_pitch = P, l_img = img;
      unsigned l_lbeg = __builtin_amdgcn_readfirstlane(lds0), l_lend = l_lbeg + NBUF * img;
      unsigned l_rd = l_lbeg, l_wr = l_lbeg + (NBUF - 1) * img, l_tci;
      const int64_t n_steady = S;
      unsigned l_n = (unsigned)n_steady;
      // VMW = operations that may stay in flight at a step's wait: the 4 loads of A(s+2) issued at
      // its start and, with a ring of 4, the NCW copies issued after the previous step's barrier
      // (with a ring of 3 those copies are image s+1 itself and must have landed)
#define VNM_GO(W, N, VM3, VM4)                                                    \
      if constexpr (NW == W && NCW == N && !DUAL) {                              \
        if constexpr (NBUF == 4) VNM_ASM_LOOP_V64(VNM_C##W##_##N##A, VNM_C##W##_##N##B, VM4);  \
        else VNM_ASM_LOOP_V64(VNM_C##W##_##N##A, VNM_C##W##_##N##B, VM3);         \
      }                                                                          \
      if constexpr (NW == W && NCW == N && DUAL) {                               \
        if constexpr (NBUF == 4) VNM_ASM_LOOP_D(VNM_C##W##_##N##A, VNM_C##W##_##N##B, VM4);    \
        else VNM_ASM_LOOP_D(VNM_C##W##_##N##A, VNM_C##W##_##N##B, VM3);           \
      }
      VNM_GO(4, 3, "4", "7") VNM_GO(4, 4, "4", "8") VNM_GO(4, 5, "4", "9") VNM_GO(4, 6, "4", "10")
      VNM_GO(4, 7, "4", "11") VNM_GO(4, 8, "4", "12") VNM_GO(4, 9, "4", "13") VNM_GO(4, 10, "4", "14")
      VNM_GO(8, 2, "4", "6") VNM_GO(8, 3, "4", "7") VNM_GO(8, 4, "4", "8") VNM_GO(8, 5, "4", "9")
#undef VNM_GO
    }
  }

  // ---- epilogue.  A lane holds, per (A tile, B tile, jq), 4 consecutive output channels of one
  // token -- 8 bytes of fp16 -- so storing straight from the accumulators would scatter 8-byte
  // pieces over 64 different rows per instruction.  For fp16 output the wave's tile is therefore
  // turned around in LDS (the ring is free after the last barrier): written as [token][V channels]
  // with a pitch of V*2+8 bytes (conflict-free 8-byte writes), read back 16 bytes per lane with
  // V/8 lanes per token, and stored as whole V*2-byte runs of each Y row.
  if (!r_valid) return;
  const int tokl = lane & 31;
  if constexpr (FUSED) {
    if (a.bias) {
      // bias of output channel r V + 32 i + 8 jq + 4 hB + e, the channel this lane holds in
      // accumulator element 4 jq + e of A tile i.  All loads are issued before the first use
      // (unconditional, index clamped: rows beyond `out` are never stored, whatever is added there).
      float bv[AT][16];
#pragma unroll
      for (int i = 0; i < AT; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int64_t o = r * V + i * 32 + 8 * (k >> 2) + 4 * hB + (k & 3);
          bv[i][k] = (float)a.bias[o < a.out ? o : a.out - 1];
        }
#pragma unroll
      for (int i = 0; i < AT; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k)
#pragma unroll
          for (int j = 0; j < BT; ++j) acc[i][j][k] += bv[i][k];
    }
  }
  if (!a.y_fp32 && a.wide_store && (!FUSED || !a.perm_out)) {
    constexpr int EP = V * 2 + 8;                         // bytes per token row in LDS
    unsigned char* ep = smem + (size_t)wave * TW * EP;    // this wave's private region
#pragma unroll
    for (int j = 0; j < BT; ++j)
#pragma unroll
      for (int i = 0; i < AT; ++i)
#pragma unroll
        for (int jq = 0; jq < 4; ++jq) {
          h4 pk = {(_Float16)acc[i][j][4 * jq], (_Float16)acc[i][j][4 * jq + 1],
                   (_Float16)acc[i][j][4 * jq + 2], (_Float16)acc[i][j][4 * jq + 3]};
          *(h4*)(ep + (size_t)(j * 32 + tokl) * EP + (i * 32 + 8 * jq + 4 * hB) * 2) = pk;
        }
    constexpr int LPT = V / 8;                            // lanes per token row (16 bytes each)
    constexpr int TPI = 64 / LPT;                         // token rows per wave-wide store
    const int ch = lane % LPT, tl = lane / LPT;
    _Float16* Yh = (_Float16*)a.Y + (int64_t)blockIdx.z * a.z_stride;
#pragma unroll
    for (int it = 0; it < TW / TPI; ++it) {
      const int tk = it * TPI + tl;
      const uint4 v = *(const uint4*)(ep + (size_t)tk * EP + ch * 16);
      const int64_t tok = t0 + wt * TW + tk;
      const int64_t o = r * V + ch * 8;
      // Y is written once and not read again here: non-temporal stores keep it from displacing the
      // operands other workgroups still stream through L2 (measured 5-10 % of the kernel)
      if (tok < a.T && o + 8 <= a.out) {
        u4v vv = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(vv, (u4v*)(Yh + tok * a.ldy + o));
      }
      else if (tok < a.T) {
        const _Float16* hv = (const _Float16*)&v;
        for (int e = 0; e < 8; ++e) if (o + e < a.out) Yh[tok * a.ldy + o + e] = hv[e];
      }
    }
    return;
  }
  const bool final_y = gridDim.z == 1;
  auto store4 = [&](auto* dst, int64_t o, float v0, float v1, float v2, float v3) {
    using OutT = std::remove_pointer_t<decltype(dst)>;
    if (a.vec_store && o + 3 < a.out) {
      // final results leave non-temporally; split-K partials are read back at once and stay cached
      if (sizeof(OutT) == 2) {
        h4 pk = {(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};
        if (final_y) __builtin_nontemporal_store(pk, (h4*)dst); else *(h4*)dst = pk;
      } else {
        f4 pk = {v0, v1, v2, v3};
        if (final_y) __builtin_nontemporal_store(pk, (f4*)dst); else *(f4*)dst = pk;
      }
    } else {
      if (o < a.out) dst[0] = (OutT)v0;
      if (o + 1 < a.out) dst[1] = (OutT)v1;
      if (o + 2 < a.out) dst[2] = (OutT)v2;
      if (o + 3 < a.out) dst[3] = (OutT)v3;
    }
  };
  if (FUSED && a.perm_out) {
    // Output permutation (Eq. 6, P_o^T): channel o of the weight's row order goes to column
    // perm_out[o] of Y, one 2- or 4-byte store per element (rows of Y are token-major, so a
    // permutation of the channels leaves nothing contiguous); split-K partials never come here.
#pragma unroll
    for (int i = 0; i < AT; ++i)
#pragma unroll
      for (int jq = 0; jq < 4; ++jq)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t o = r * V + i * 32 + 8 * jq + 4 * hB + e;
          const int64_t dst = o < a.out ? (int64_t)a.perm_out[o] : -1;
          if (dst < 0 || dst >= a.out) continue;
#pragma unroll
          for (int j = 0; j < BT; ++j) {
            const int64_t tok = t0 + wt * TW + j * 32 + tokl;
            if (tok >= a.T) continue;
            const float v = acc[i][j][4 * jq + e];
            if (a.y_fp32) ((float*)a.Y)[tok * a.ldy + dst] = v;
            else ((_Float16*)a.Y)[tok * a.ldy + dst] = (_Float16)v;
          }
        }
    return;
  }
#pragma unroll
  for (int j = 0; j < BT; ++j) {
    const int64_t tok = t0 + wt * TW + j * 32 + tokl;
    if (tok >= a.T) continue;
#pragma unroll
    for (int i = 0; i < AT; ++i) {
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const int64_t o = r * V + i * 32 + 8 * jq + 4 * hB;
        const float v0 = acc[i][j][4 * jq], v1 = acc[i][j][4 * jq + 1], v2 = acc[i][j][4 * jq + 2],
                    v3 = acc[i][j][4 * jq + 3];
        if (a.y_fp32) store4((float*)a.Y + (int64_t)blockIdx.z * a.z_stride + tok * a.ldy + o, o, v0, v1, v2, v3);
        else store4((_Float16*)a.Y + (int64_t)blockIdx.z * a.z_stride + tok * a.ldy + o, o, v0, v1, v2, v3);
      }
    }
  }
}

bool spmm_smfmac_applicable(const void* X, int64_t ldx, const Dims& d) {
  return has_packed(d.V, d.M) && d.in % 8 == 0 && ldx % 8 == 0 && ((uintptr_t)X & 15) == 0;
}

template <int V, int TW, int WR, int WT, int NCW, int NBUF, bool DUAL, bool FUSED>
static int launch_cfg2(const SpmmArgs& a, hipStream_t st) {
  size_t lds = (size_t)NBUF * a.image_bytes;
  const size_t ep = (size_t)WR * WT * TW * (V * 2 + 8);     // epilogue transposition, per wave [TW][V] fp16
  if (ep > lds) lds = ep;
  auto kern = spmm_smfmac_kernel<V, TW, WR, WT, NCW, NBUF, DUAL, FUSED>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_smfmac)")) return rc_lds;
  dim3 grid((unsigned)((a.T + kTokTile - 1) / kTokTile), (unsigned)((a.R + WR - 1) / WR),
            (unsigned)((a.S + a.ks_steps - 1) / a.ks_steps));
  hipLaunchKernelGGL(kern, grid, dim3(64 * WR * WT), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_smfmac_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

template <int V, int TW, int WR, int WT, int NCW, int NBUF, bool DUAL>
static int launch_cfg(const SpmmArgs& a, hipStream_t st) {
  if (a.bias || a.perm_out) return launch_cfg2<V, TW, WR, WT, NCW, NBUF, DUAL, true>(a, st);
  return launch_cfg2<V, TW, WR, WT, NCW, NBUF, DUAL, false>(a, st);
}

// V = 64: pick the assembly loop by workgroup size (4 or 8 row blocks), by copies per wave
// (NCW = ceil(image KiB / waves)) and by ring depth.
template <int NBUF, bool DUAL>
static int launch_v64_w4(const SpmmArgs& a, hipStream_t st) {
  const int ncw = (a.image_bytes / 1024 + 3) / 4;
  switch (ncw) {
    case 3: return launch_cfg<64, 128, 4, 1, 3, NBUF, DUAL>(a, st);
    case 4: return launch_cfg<64, 128, 4, 1, 4, NBUF, DUAL>(a, st);
    case 5: return launch_cfg<64, 128, 4, 1, 5, NBUF, DUAL>(a, st);
    case 6: return launch_cfg<64, 128, 4, 1, 6, NBUF, DUAL>(a, st);
    case 7: return launch_cfg<64, 128, 4, 1, 7, NBUF, DUAL>(a, st);
    case 8: return launch_cfg<64, 128, 4, 1, 8, NBUF, DUAL>(a, st);
    case 9: return launch_cfg<64, 128, 4, 1, 9, NBUF, DUAL>(a, st);
    case 10: return launch_cfg<64, 128, 4, 1, 10, NBUF, DUAL>(a, st);
  }
  return VNM_ERR_UNSUPPORTED;
}
template <int NBUF, bool DUAL>
static int launch_v64_w8(const SpmmArgs& a, hipStream_t st) {
  const int ncw = (a.image_bytes / 1024 + 7) / 8;
  switch (ncw) {
    case 2: return launch_cfg<64, 128, 8, 1, 2, NBUF, DUAL>(a, st);
    case 3: return launch_cfg<64, 128, 8, 1, 3, NBUF, DUAL>(a, st);
    case 4: return launch_cfg<64, 128, 8, 1, 4, NBUF, DUAL>(a, st);
    case 5: return launch_cfg<64, 128, 8, 1, 5, NBUF, DUAL>(a, st);
  }
  return VNM_ERR_UNSUPPORTED;
}

// Sum of the KS fp32 partial products [KS][T][out] into Y (fp16 or fp32, leading dimension ldy),
// plus the fused bias and output permutation if given.
template <typename OutT>
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ part, int KS, int64_t T, int64_t out, OutT* __restrict__ Y, int64_t ldy,
                     const _Float16* __restrict__ bias, const int* __restrict__ perm_out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * out) return;
  float acc = 0.f;
  const float* p = part + idx;
  const int64_t zs = T * out;
  int z = 0;
  for (; z + 4 <= KS; z += 4) {
    const float a0 = p[(int64_t)z * zs], a1 = p[(int64_t)(z + 1) * zs], a2 = p[(int64_t)(z + 2) * zs],
                a3 = p[(int64_t)(z + 3) * zs];
    acc += (a0 + a1) + (a2 + a3);
  }
  for (; z < KS; ++z) acc += p[(int64_t)z * zs];
  const int64_t t = idx / out, o = idx - t * out;
  if (bias) acc += (float)bias[o];
  const int64_t dst = perm_out ? (int64_t)perm_out[o] : o;
  if (dst >= 0 && dst < out) Y[t * ldy + dst] = (OutT)acc;
}

constexpr int64_t kSplitKMaxTokens = 2048;
constexpr int64_t kSplitKMaxBytes = 64ll << 20;

int64_t splitk_scratch_bytes(int64_t T, int64_t out) {
  if (T <= 0 || T > kSplitKMaxTokens) return 0;
  int64_t b = 16 * T * out * 4;
  if (b > kSplitKMaxBytes) b = kSplitKMaxBytes;
  return (b + 255) / 256 * 256;
}

int launch_spmm_smfmac(const void* Xs, int64_t T, const void* packed, const Dims& d,
                       void* Y, int64_t ldy, int y_dtype, void* scratch, int64_t scratch_bytes,
                       const Fused& f, hipStream_t st) {
  const PackedLayout pl = packed_layout(d);
  const char* p = (const char*)packed;
  SpmmArgs a{};
  a.bias = f.bias; a.perm_out = f.perm_out;
  a.Xs = (const unsigned char*)Xs; a.T = T;
  a.pa = (const uint4*)(p + pl.pa_off);
  a.pidx = (const unsigned short*)(p + pl.pidx_off);
  a.pcol = (const unsigned*)(p + pl.pcol_off);
  const bool dual = packed_tables(d.V) == 2;
  a.out = d.out; a.R = packed_row_blocks(d); a.S = d.S; a.M = d.M;  // 64-row blocks of the packed copy
  a.image_bytes = (int)image_bytes(d.M);
  a.Y = Y; a.ldy = ldy; a.y_fp32 = y_dtype;
  a.ks_steps = d.S; a.z_stride = 0;
  if ((T + kTokTile - 1) / kTokTile > 0x7FFFFFFF || (a.R + 1) / 2 > 65535) return VNM_ERR_UNSUPPORTED;
  const bool deep = 2 * 4 * (size_t)a.image_bytes <= 150 * 1024;
  // 8 row blocks per workgroup (one per CU) halve the image traffic per flop, 4 (two per CU) give
  // twice as many workgroups.  Pick by the number of rounds the grid needs on the 256 CUs: a round
  // costs the K loop (about 15 % slower per step with 4) plus a fixed prologue and store of about 12
  // K steps' worth, which dominates when K is short.
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  const int64_t rounds8 = (tiles * ((a.R + 7) / 8) + 255) / 256, rounds4 = (tiles * ((a.R + 3) / 4) + 511) / 512;
  const double cost8 = (double)rounds8 * ((double)d.S + 12.0), cost4 = (double)rounds4 * (1.15 * (double)d.S + 12.0);
  bool wide = a.R >= 8 && cost8 <= cost4;
  // Few tokens: too few (token tile, row group) pairs to occupy the 256 CUs, and the job is to
  // stream the compressed weight at HBM rate.  Split K over up to 16 workgroups per pair; each
  // writes an fp32 partial product to the scratch, a second kernel adds them up.
  int KS = 1;
  const int64_t base = tiles * ((a.R + 3) / 4);
  if (scratch && T <= kSplitKMaxTokens && base < 192) {
    // up to 256 tokens: about 200 workgroups measured best.  Beyond that the partial products (ks x T x
    // out floats written, then read by the reduction) weigh in: about 256 workgroups while fewer than
    // half the CUs would have one, and a split in two only where the K loop is long enough to pay
    // for the reduction (measured: 276 K steps gain 19 %, 103 steps lose 10 %)
    int64_t ks = 1;
    if (T <= 256) ks = (200 + base / 2) / base;
    else if (base < 128) ks = 256 / base;
    else if (d.S >= 192) ks = 2;
    if (ks > 16) ks = 16;
    if (ks > d.S / 4) ks = d.S / 4;                                   // at least 4 K steps each
    while (ks > 1 && ks * T * d.out * 4 > scratch_bytes) --ks;
    if (ks > 1) {
      a.ks_steps = (d.S + ks - 1) / ks;
      KS = (int)((d.S + a.ks_steps - 1) / a.ks_steps);
    }
  }
  if (KS > 1) {
    a.Y = scratch; a.ldy = d.out; a.y_fp32 = 1; a.z_stride = T * d.out;
    a.bias = nullptr; a.perm_out = nullptr;                           // applied by the reduction
    wide = false;
  }
  // Output permutation: rather than scattering 2-byte stores from the epilogue, Y is written in the
  // weight's row order (contiguous runs) and its rows are permuted in place by a second pass
  // through LDS while they are still in cache; rows too long for LDS take the scattering epilogue.
  const int y_elem = y_dtype == 0 ? 2 : 4;
  const bool post_permute = KS == 1 && f.perm_out && d.out * y_elem <= permute_rows_max_bytes();
  if (post_permute) a.perm_out = nullptr;
  a.wide_store = (a.y_fp32 == 0) && (a.ldy % 8 == 0) && (((uintptr_t)a.Y & 15) == 0);
  a.vec_store = (a.ldy % 4 == 0) && (((uintptr_t)a.Y & (a.y_fp32 == 0 ? 7 : 15)) == 0);
  int rc = VNM_ERR_UNSUPPORTED;
  const bool ring4 = 4 * (size_t)a.image_bytes <= 150 * 1024;
  if (!dual) {
    if (wide) rc = ring4 ? launch_v64_w8<4, false>(a, st) : launch_v64_w8<3, false>(a, st);
    else rc = deep ? launch_v64_w4<4, false>(a, st) : launch_v64_w4<3, false>(a, st);
  } else {
    if (wide) rc = ring4 ? launch_v64_w8<4, true>(a, st) : launch_v64_w8<3, true>(a, st);
    else rc = deep ? launch_v64_w4<4, true>(a, st) : launch_v64_w4<3, true>(a, st);
  }
  if (rc != VNM_OK) return rc;
  if (post_permute) return launch_permute_rows(Y, ldy, Y, ldy, T, d.out, y_elem, true, f.perm_out, st);
  if (KS == 1) return rc;
  return launch_splitk_reduce(scratch, KS, T, d.out, Y, ldy, y_dtype, f, st);
}

int launch_splitk_reduce(const void* part, int KS, int64_t T, int64_t out, void* Y, int64_t ldy,
                         int y_dtype, const Fused& f, hipStream_t st) {
  const int64_t n = T * out;
  if (y_dtype == 0)
    hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       (const float*)part, KS, T, out, (_Float16*)Y, ldy, f.bias, f.perm_out);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       (const float*)part, KS, T, out, (float*)Y, ldy, f.bias, f.perm_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "splitk_reduce_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
