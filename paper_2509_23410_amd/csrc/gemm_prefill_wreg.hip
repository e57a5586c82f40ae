// Prefill-shaped hybrid GEMM for tile = 128 with the weights loaded straight into registers (Section 4 /
// Appendix A of the paper: the product for the prefill input, dense and 2:4 tiles mixed inside one launch).
//
// Workgroup = 256 output features (two tile rows) x 256 rows of X, 4 wavefronts (one per SIMD).  Wavefront w owns
// 64 features (4 strips of tile row w / 2) x ALL 256 rows of X: its weight fragments are private, so they go
// global -> registers in the stored register order (layout.h) with no LDS traffic, no transposition and no barrier
// between producer and consumer, two 64-column steps ahead.  X is shared by the four wavefronts and goes
// global -> LDS directly (no registers) in whole 128-byte rows, three steps ahead, through a ring of four 32 KB
// stages.  Every row of X in a step is one full cache line: a 32-column step would use half of each line it
// pulls through the vector L1 and was measured to cost 1.5x the L1 <- L2 requests.
//
// A step is 16 "column blocks" (16 rows of X each).  Per column block and wavefront:
//   dense: 8 x v_mfma_f32_16x16x32_bf16   or   2:4: 4 x v_smfmac_f32_16x16x64_bf16
// plus the two LDS reads of the column block seven ahead (across step boundaries: the LDS pipeline never drains;
// a 2:4 column block lasts 64 cycles, and three blocks ahead did not cover the LDS latency)
// and at most one global load.  With one wavefront per SIMD nothing hides an instruction that is not a matrix
// instruction, and a taken branch is a bubble in the matrix pipe, so the dense / 2:4 decision is ONE scalar branch
// per step (a wavefront works on one tile at a time) around two branch-free instruction streams.
//
// Registers.  Everything that is loaded asynchronously or lives across that branch is addressed BY NAME in the asm
// statements and never seen by the compiler as a value:
//   a[0:255]     the 64 accumulator tiles (strip s, column block cb) at a[4 (16 s + cb) .. + 3]
//   v[128:223]   weights of three steps in rotation, 8 x 4 registers each (see PATCH_WR_VA)
//   v[64:127]    X operands of eight column blocks in rotation, 8 registers each
// As compiler values they would meet at the branch (and at the loop edge) as phi nodes, where the register
// allocator may insert copies - it did: it split the accumulators and spilled, and it copied X operands whose
// LDS reads were still in flight.  Every asm statement declares all of these registers clobbered, so the compiler
// keeps nothing of its own there; its own values fit below v64 and it uses no accumulation register, which
// tests/test_abi_host.py checks on the generated assembly.
// The loads are counted, not tracked: every step issues exactly 16 vector-memory loads per wavefront (8 for the
// weights whatever the tile type, 8 for X) and 32 LDS reads, so every s_waitcnt below is a compile-time constant.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epilogue.h"
#include "kernels.h"
#include "layout.h"

namespace patch {

typedef float wr_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWrBN = 256, kWrBM = 256;
constexpr int kWrStage = kWrBM * 128;   // 256 rows of X x 64 columns, swizzled
constexpr int kWrRing = 4 * kWrStage;   // 128 KB: the four X stages
constexpr int kWrOut = 4096;            // per wavefront: 16 rows x 64 features fp32 of the output stage
constexpr int kWrLds = kWrRing + 4 * kWrOut;   // 144 KB

typedef __attribute__((address_space(3))) void* wr_lptr_t;

// ---- register names (the assembler evaluates the index expressions)
// accumulator tile of strip S, column block CB
#define PATCH_WR_C(S, CB) "a[4*(16*" #S "+" #CB "):4*(16*" #S "+" #CB ")+3]"
// weight register I (0..7) of step buffer AB (0..2):
//   dense: I = 2 s + h: operand h of strip s;   2:4: I = s: values of strip s, I = 4 + s: position dword in its first register
#define PATCH_WR_VA(AB, I) "v[128+32*" #AB "+4*" #I ":128+32*" #AB "+4*" #I "+3]"
#define PATCH_WR_VI(AB, S) "v[128+32*" #AB "+16+4*" #S "]"
// X operand set SET (0..3): low / high half (the two dense operands) and the pair (the 2:4 operand)
#define PATCH_WR_VBL(SET) "v[64+8*" #SET ":64+8*" #SET "+3]"
#define PATCH_WR_VBH(SET) "v[68+8*" #SET ":68+8*" #SET "+3]"
#define PATCH_WR_VB(SET) "v[64+8*" #SET ":64+8*" #SET "+7]"
#define PATCH_WR_R8(r, p) r #p "0", r #p "1", r #p "2", r #p "3", r #p "4", r #p "5", r #p "6", r #p "7"
#define PATCH_WR_R10(r, p) PATCH_WR_R8(r, p), r #p "8", r #p "9"
#define PATCH_WR_CLOBBER                                                                                           \
    "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", PATCH_WR_R10("a", 1), PATCH_WR_R10("a", 2),          \
        PATCH_WR_R10("a", 3), PATCH_WR_R10("a", 4), PATCH_WR_R10("a", 5), PATCH_WR_R10("a", 6), PATCH_WR_R10("a", 7),  \
        PATCH_WR_R10("a", 8), PATCH_WR_R10("a", 9), PATCH_WR_R10("a", 10), PATCH_WR_R10("a", 11), PATCH_WR_R10("a", 12), \
        PATCH_WR_R10("a", 13), PATCH_WR_R10("a", 14), PATCH_WR_R10("a", 15), PATCH_WR_R10("a", 16),                  \
        PATCH_WR_R10("a", 17), PATCH_WR_R10("a", 18), PATCH_WR_R10("a", 19), PATCH_WR_R10("a", 20),                  \
        PATCH_WR_R10("a", 21), PATCH_WR_R10("a", 22), PATCH_WR_R10("a", 23), PATCH_WR_R10("a", 24), "a250", "a251",  \
        "a252", "a253", "a254", "a255", "v64", "v65", "v66", "v67", "v68", "v69", PATCH_WR_R10("v", 7), PATCH_WR_R10("v", 8), PATCH_WR_R10("v", 9),      \
        PATCH_WR_R10("v", 10), PATCH_WR_R10("v", 11), PATCH_WR_R10("v", 12), PATCH_WR_R10("v", 13), PATCH_WR_R10("v", 14),                \
        PATCH_WR_R10("v", 15), PATCH_WR_R10("v", 16), PATCH_WR_R10("v", 17), PATCH_WR_R10("v", 18),                  \
        PATCH_WR_R10("v", 19), PATCH_WR_R10("v", 20), PATCH_WR_R10("v", 21), "v220", "v221", "v222", "v223"

// ---- registers of the step loop.  The loop is ONE asm statement (no compiler-generated instruction inside it: with one
// wavefront per SIMD every instruction that is not issued in the shadow of a matrix instruction stalls the matrix pipe,
// and the code the compiler placed between the column blocks - the next step's addresses, the loop control, its
// hazard nops - cost about 300 cycles of a 2048-cycle dense step).  A lone wavefront issues about one instruction
// every five to six cycles, so a 2:4 step (64 matrix instructions in 1024 cycles) is bound by its instruction count:
// a global load is ONE instruction (lane offsets and bases prepared once per tile), and what changes only with the
// tile is computed in odd steps only.  Besides the accumulators, the weight buffers and the X operand sets the loop
// owns, by name:
//   s80       step index s
//   s[82:83]  X + 128 min(s + 3, S - 1): source of the X loads issued in step s
//   s[74:75]  address of the tile the weight loads fetch (the tile of steps s + 2 / s + 3), s76 its table entry,
//             s86 its type as a mask (0 dense, -1 2:4)
//   s[84:85]  base of weight-load slots 0-3 of this step: the tile + K-step (s % 2) of the dense operands or 2:4 values
//   s[96:97]  base of slots 4-7: the tile + K-step of the dense operands (the 2:4 position dwords hold both K-steps)
//   s87       type of the tile the NEXT step multiplies (0 dense, 1 2:4; 0 for a wavefront without a tile row)
//   s81, s88-s90, s[94:95] scratch     s91 LDS address of this wavefront's first 1 KB piece of stage (s + 3) % 4
//   s[92:93]  lane mask of the selects
//   v224 / v225  lane LDS addresses (low / high X operand) of the stage an EVEN step reads in column blocks 0-8 and an odd
//                step reads in column blocks 9-15; v226 / v227 the other way round
//   v228-v235    lane offsets of the eight weight-load slots for the type of the tile being loaded, selected from
//   v236-v243    ... those of a dense tile: slot I = operand I % 2 of strip I / 2: lane * 16 + (I / 2) 4096 + (I % 2) 1024
//   v244-v251    ... those of a 2:4 tile: slot I < 4 = values of strip I: lane * 16 + I 2048; slot 4 + s = 16 bytes starting
//                at the lane's position dword of strip s: lane * 4 + 16384 + s 256 (the first register is the dword, the
//                rest is ignored; the last lanes read up to 12 bytes into the next tile or the zeroed slack behind the payload)
//   (each plus the offset of the wavefront's four strips inside the tile)
// Every step updates them in "control slots": up to three light instructions per column block, each placed behind a
// matrix instruction (K1, K2, K3 below), so that they issue while the matrix pipe is busy.
//
// ---- weight load of slot I (0..7) of the step two ahead into buffer ABN: one instruction in column block I
#define PATCH_WR_WLOAD_03(ABN, I) "global_load_dwordx4 " PATCH_WR_VA(ABN, I) ", v[228+" #I "], s[84:85]\n\t"
#define PATCH_WR_WLOAD_47(ABN, I) "global_load_dwordx4 " PATCH_WR_VA(ABN, I) ", v[228+" #I "], s[96:97]\n\t"
// X load SLOT (0..7) of the step three ahead: 16 bytes per lane, global -> LDS at m0 + lane * 16
#define PATCH_WR_X3(SLOT) "s_add_u32 m0, s91, 4096*" #SLOT "\n\t"
#define PATCH_WR_X4(SLOT) "global_load_lds_dwordx4 %[xo" #SLOT "], s[82:83]\n\t"
// load parts of column block CB: LD3 (one matrix instruction before LD4: a write of m0 needs a wait state), LD4
#define PATCH_WR_LD3_0(ABN) ""
#define PATCH_WR_LD3_1(ABN) ""
#define PATCH_WR_LD3_2(ABN) ""
#define PATCH_WR_LD3_3(ABN) ""
#define PATCH_WR_LD3_4(ABN) ""
#define PATCH_WR_LD3_5(ABN) ""
#define PATCH_WR_LD3_6(ABN) ""
#define PATCH_WR_LD3_7(ABN) ""
#define PATCH_WR_LD3_8(ABN) PATCH_WR_X3(0)
#define PATCH_WR_LD3_9(ABN) PATCH_WR_X3(1)
#define PATCH_WR_LD3_10(ABN) PATCH_WR_X3(2)
#define PATCH_WR_LD3_11(ABN) PATCH_WR_X3(3)
#define PATCH_WR_LD3_12(ABN) PATCH_WR_X3(4)
#define PATCH_WR_LD3_13(ABN) PATCH_WR_X3(5)
#define PATCH_WR_LD3_14(ABN) PATCH_WR_X3(6)
#define PATCH_WR_LD3_15(ABN) PATCH_WR_X3(7)
#define PATCH_WR_LD4_0(ABN) PATCH_WR_WLOAD_03(ABN, 0)
#define PATCH_WR_LD4_1(ABN) PATCH_WR_WLOAD_03(ABN, 1)
#define PATCH_WR_LD4_2(ABN) PATCH_WR_WLOAD_03(ABN, 2)
#define PATCH_WR_LD4_3(ABN) PATCH_WR_WLOAD_03(ABN, 3)
#define PATCH_WR_LD4_4(ABN) PATCH_WR_WLOAD_47(ABN, 4)
#define PATCH_WR_LD4_5(ABN) PATCH_WR_WLOAD_47(ABN, 5)
#define PATCH_WR_LD4_6(ABN) PATCH_WR_WLOAD_47(ABN, 6)
#define PATCH_WR_LD4_7(ABN) PATCH_WR_WLOAD_47(ABN, 7)
#define PATCH_WR_LD4_8(ABN) PATCH_WR_X4(0)
#define PATCH_WR_LD4_9(ABN) PATCH_WR_X4(1)
#define PATCH_WR_LD4_10(ABN) PATCH_WR_X4(2)
#define PATCH_WR_LD4_11(ABN) PATCH_WR_X4(3)
#define PATCH_WR_LD4_12(ABN) PATCH_WR_X4(4)
#define PATCH_WR_LD4_13(ABN) PATCH_WR_X4(5)
#define PATCH_WR_LD4_14(ABN) PATCH_WR_X4(6)
#define PATCH_WR_LD4_15(ABN) PATCH_WR_X4(7)

// ---- lane LDS addresses by step parity PAR: column blocks 0-8 read ahead inside the step's own stage (address pair
// "cur"), column blocks 9-15 into the next stage ("nxt")
#define PATCH_WR_CURL_0 "v224"
#define PATCH_WR_CURH_0 "v225"
#define PATCH_WR_NXTL_0 "v226"
#define PATCH_WR_NXTH_0 "v227"
#define PATCH_WR_CURL_1 "v226"
#define PATCH_WR_CURH_1 "v227"
#define PATCH_WR_NXTL_1 "v224"
#define PATCH_WR_NXTH_1 "v225"

// ---- control slots: PATCH_WR_K<slot>_<column block>_<step parity>.  In order (s = this step):
//   blocks 0-2    s[82:83] = X + 128 min(s + 3, S - 1);  s91 = LDS address of stage (s + 3) % 4     (used by blocks 8-15)
//   blocks 9-10   "cur" lane addresses = stage (s + 2) % 4: the next step's "nxt" (last read in block 8)
//   block 15      s80 = s + 1
//   even steps (the next step is K-step 1 of the same tiles), blocks 10-12: the bases of its weight loads,
//                 s[84:85] = tile + (2:4 ? 1024 : 2048), s[96:97] = tile + (2:4 ? 0 : 2048)
//   odd steps (the next step starts new tiles): blocks 2-4 s87 = type of tile (s + 1) / 2, which the next step
//                 multiplies; blocks 4-6 s76 = table entry of tile (s + 3) / 2, which the next two steps' weight loads fetch;
//                 blocks 10-15, after this step's last weight load (block 7): its address s[74:75], its type s86, the
//                 eight lane offsets v228-v235 for that type, both bases = the tile (K-step 0)
// A scalar compare and the select that reads its result share a slot, and so do the two halves of a 64-bit add.
#define PATCH_WR_K1_0_0 "s_add_i32 s88, s80, 3\n\t"
#define PATCH_WR_K2_0_0 "s_min_i32 s89, s88, %[sm1]\n\t"
#define PATCH_WR_K3_0_0 "s_lshl_b32 s89, s89, 7\n\t"
#define PATCH_WR_K1_1_0 "s_add_u32 s82, %[xlo], s89\n\ts_addc_u32 s83, %[xhi], 0\n\t"
#define PATCH_WR_K2_1_0 "s_and_b32 s88, s88, 3\n\t"
#define PATCH_WR_K3_1_0 "s_lshl_b32 s88, s88, 15\n\t"
#define PATCH_WR_K1_2_0 "s_add_u32 s91, %[ldsw], s88\n\t"
#define PATCH_WR_K2_2_0 ""
#define PATCH_WR_K3_2_0 ""
#define PATCH_WR_K1_3_0 ""
#define PATCH_WR_K2_3_0 ""
#define PATCH_WR_K3_3_0 ""
#define PATCH_WR_K1_4_0 ""
#define PATCH_WR_K2_4_0 ""
#define PATCH_WR_K3_4_0 ""
#define PATCH_WR_K1_5_0 ""
#define PATCH_WR_K2_5_0 ""
#define PATCH_WR_K3_5_0 ""
#define PATCH_WR_K1_6_0 ""
#define PATCH_WR_K2_6_0 ""
#define PATCH_WR_K3_6_0 ""
#define PATCH_WR_K1_7_0 ""
#define PATCH_WR_K2_7_0 ""
#define PATCH_WR_K3_7_0 ""
#define PATCH_WR_K1_8_0 ""
#define PATCH_WR_K2_8_0 ""
#define PATCH_WR_K3_8_0 ""
#define PATCH_WR_K1_9_0 "s_add_i32 s88, s80, 2\n\t"
#define PATCH_WR_K2_9_0 "s_and_b32 s88, s88, 3\n\t"
#define PATCH_WR_K3_9_0 "s_lshl_b32 s88, s88, 15\n\t"
#define PATCH_WR_K1_10_0 "v_add_u32 v224, s88, %[bl0]\n\t"
#define PATCH_WR_K2_10_0 "v_add_u32 v225, s88, %[bh0]\n\t"
#define PATCH_WR_K3_10_0 "s_and_b32 s81, s86, -1024\n\t"
#define PATCH_WR_K1_11_0 "s_add_i32 s81, s81, 2048\n\t"
#define PATCH_WR_K2_11_0 "s_add_u32 s84, s74, s81\n\ts_addc_u32 s85, s75, 0\n\t"
#define PATCH_WR_K3_11_0 "s_andn2_b32 s81, 2048, s86\n\t"
#define PATCH_WR_K1_12_0 "s_add_u32 s96, s74, s81\n\ts_addc_u32 s97, s75, 0\n\t"
#define PATCH_WR_K2_12_0 ""
#define PATCH_WR_K3_12_0 ""
#define PATCH_WR_K1_13_0 ""
#define PATCH_WR_K2_13_0 ""
#define PATCH_WR_K3_13_0 ""
#define PATCH_WR_K1_14_0 ""
#define PATCH_WR_K2_14_0 ""
#define PATCH_WR_K3_14_0 ""
#define PATCH_WR_K1_15_0 ""
#define PATCH_WR_K2_15_0 ""
#define PATCH_WR_K3_15_0 "s_add_i32 s80, s80, 1\n\t"
#define PATCH_WR_K1_0_1 "s_add_i32 s88, s80, 3\n\t"
#define PATCH_WR_K2_0_1 "s_min_i32 s89, s88, %[sm1]\n\t"
#define PATCH_WR_K3_0_1 "s_lshl_b32 s89, s89, 7\n\t"
#define PATCH_WR_K1_1_1 "s_add_u32 s82, %[xlo], s89\n\ts_addc_u32 s83, %[xhi], 0\n\t"
#define PATCH_WR_K2_1_1 "s_and_b32 s88, s88, 3\n\t"
#define PATCH_WR_K3_1_1 "s_lshl_b32 s88, s88, 15\n\t"
#define PATCH_WR_K1_2_1 "s_add_u32 s91, %[ldsw], s88\n\t"
#define PATCH_WR_K2_2_1 "s_add_i32 s88, s80, 1\n\t"
#define PATCH_WR_K3_2_1 "s_lshr_b32 s88, s88, 1\n\t"
#define PATCH_WR_K1_3_1 "s_min_u32 s88, s88, %[tkm1]\n\t"
#define PATCH_WR_K2_3_1 "v_readlane_b32 s89, %[ent0], s88\n\t"
#define PATCH_WR_K3_3_1 "v_readlane_b32 s90, %[ent1], s88\n\t"
#define PATCH_WR_K1_4_1 "s_cmp_lt_u32 s88, 64\n\ts_cselect_b32 s89, s89, s90\n\t"
#define PATCH_WR_K2_4_1 "s_and_b32 s87, s89, %[live]\n\t"
#define PATCH_WR_K3_4_1 "s_add_i32 s88, s80, 3\n\t"
#define PATCH_WR_K1_5_1 "s_lshr_b32 s88, s88, 1\n\t"
#define PATCH_WR_K2_5_1 "s_min_u32 s88, s88, %[tkm1]\n\t"
#define PATCH_WR_K3_5_1 "v_readlane_b32 s76, %[ent0], s88\n\t"
#define PATCH_WR_K1_6_1 "v_readlane_b32 s90, %[ent1], s88\n\t"
#define PATCH_WR_K2_6_1 "s_cmp_lt_u32 s88, 64\n\ts_cselect_b32 s76, s76, s90\n\t"
#define PATCH_WR_K3_6_1 ""
#define PATCH_WR_K1_7_1 ""
#define PATCH_WR_K2_7_1 ""
#define PATCH_WR_K3_7_1 ""
#define PATCH_WR_K1_8_1 ""
#define PATCH_WR_K2_8_1 ""
#define PATCH_WR_K3_8_1 ""
#define PATCH_WR_K1_9_1 "s_add_i32 s88, s80, 2\n\t"
#define PATCH_WR_K2_9_1 "s_and_b32 s88, s88, 3\n\t"
#define PATCH_WR_K3_9_1 "s_lshl_b32 s88, s88, 15\n\t"
#define PATCH_WR_K1_10_1 "v_add_u32 v226, s88, %[bl0]\n\t"
#define PATCH_WR_K2_10_1 "v_add_u32 v227, s88, %[bh0]\n\t"
#define PATCH_WR_K3_10_1 "s_lshr_b32 s94, s76, 1\n\t"
#define PATCH_WR_K1_11_1 "s_mov_b32 s95, 0\n\t"
#define PATCH_WR_K2_11_1 "s_lshl_b64 s[94:95], s[94:95], 8\n\t"
#define PATCH_WR_K3_11_1 "s_add_u32 s74, %[plo], s94\n\ts_addc_u32 s75, %[phi], s95\n\t"
#define PATCH_WR_K1_12_1 "s_bitcmp1_b32 s76, 0\n\ts_cselect_b32 s86, -1, 0\n\t"
#define PATCH_WR_K2_12_1 "s_bitcmp1_b32 s76, 0\n\ts_cselect_b64 s[92:93], -1, 0\n\t"
#define PATCH_WR_K3_12_1 "v_cndmask_b32_e64 v228, v236, v244, s[92:93]\n\t"
#define PATCH_WR_K1_13_1 "v_cndmask_b32_e64 v229, v237, v245, s[92:93]\n\t"
#define PATCH_WR_K2_13_1 "v_cndmask_b32_e64 v230, v238, v246, s[92:93]\n\t"
#define PATCH_WR_K3_13_1 "v_cndmask_b32_e64 v231, v239, v247, s[92:93]\n\t"
#define PATCH_WR_K1_14_1 "v_cndmask_b32_e64 v232, v240, v248, s[92:93]\n\t"
#define PATCH_WR_K2_14_1 "v_cndmask_b32_e64 v233, v241, v249, s[92:93]\n\t"
#define PATCH_WR_K3_14_1 "v_cndmask_b32_e64 v234, v242, v250, s[92:93]\n\t"
#define PATCH_WR_K1_15_1 "v_cndmask_b32_e64 v235, v243, v251, s[92:93]\n\t"
#define PATCH_WR_K2_15_1 "s_mov_b64 s[84:85], s[74:75]\n\ts_mov_b64 s[96:97], s[74:75]\n\t"
#define PATCH_WR_K3_15_1 "s_add_i32 s80, s80, 1\n\t"
// block 8 starts with the step's barrier: this wavefront's share of X(s+1) has landed (the loads issued after it: A(s+1),
// X(s+2), A(s+2)); past the barrier all of X(s+1) is visible (first read in block 9) and every read of stage (s-1) % 4
// has completed, so the loads of X(s+3) (one per block 8-15) may overwrite it
#define PATCH_WR_PRE_0 ""
#define PATCH_WR_PRE_1 ""
#define PATCH_WR_PRE_2 ""
#define PATCH_WR_PRE_3 ""
#define PATCH_WR_PRE_4 ""
#define PATCH_WR_PRE_5 ""
#define PATCH_WR_PRE_6 ""
#define PATCH_WR_PRE_7 ""
#define PATCH_WR_PRE_8 "s_waitcnt vmcnt(24)\n\ts_barrier\n\t"
#define PATCH_WR_PRE_9 ""
#define PATCH_WR_PRE_10 ""
#define PATCH_WR_PRE_11 ""
#define PATCH_WR_PRE_12 ""
#define PATCH_WR_PRE_13 ""
#define PATCH_WR_PRE_14 ""
#define PATCH_WR_PRE_15 ""
// which address pair column block CB reads ahead with
#define PATCH_WR_RAL_0(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_1(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_2(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_3(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_4(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_5(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_6(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_7(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_8(PAR) PATCH_WR_CURL_##PAR
#define PATCH_WR_RAL_9(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_10(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_11(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_12(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_13(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_14(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAL_15(PAR) PATCH_WR_NXTL_##PAR
#define PATCH_WR_RAH_0(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_1(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_2(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_3(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_4(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_5(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_6(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_7(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_8(PAR) PATCH_WR_CURH_##PAR
#define PATCH_WR_RAH_9(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_10(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_11(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_12(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_13(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_14(PAR) PATCH_WR_NXTH_##PAR
#define PATCH_WR_RAH_15(PAR) PATCH_WR_NXTH_##PAR

// ---- one column block CB of X (operand set SET) against the wavefront's four strips (weights of step buffer AB),
// after waiting for its operands, plus the two LDS reads of the column block seven ahead into set NSET (LDS byte
// offset OFF from the lane addresses), one global load - blocks 0-7 a weight load of step s+2 (buffer ABN), blocks
// 8-15 an X load of step s+3 - and the block's control slots.  J = K-step inside the tile, PAR = parity of the step.
#define PATCH_WR_PIECE_DENSE(CB, SET, NSET, AB, ABN, J, PAR, OFF) PATCH_WR_PIECE_DENSE_(CB, SET, NSET, AB, ABN, J, PAR, OFF)
#define PATCH_WR_PIECE_DENSE_(CB, SET, NSET, AB, ABN, J, PAR, OFF)                                                 \
    PATCH_WR_PRE_##CB                                                                                              \
    "s_waitcnt lgkmcnt(12)\n\t"                                                                                    \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(0, CB) ", " PATCH_WR_VA(AB, 0) ", " PATCH_WR_VBL(SET) ", " PATCH_WR_C(0, CB) "\n\t" \
    "ds_read_b128 " PATCH_WR_VBL(NSET) ", " PATCH_WR_RAL_##CB(PAR) " offset:" #OFF "\n\t"                          \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(1, CB) ", " PATCH_WR_VA(AB, 2) ", " PATCH_WR_VBL(SET) ", " PATCH_WR_C(1, CB) "\n\t" \
    "ds_read_b128 " PATCH_WR_VBH(NSET) ", " PATCH_WR_RAH_##CB(PAR) " offset:" #OFF "\n\t"                          \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(2, CB) ", " PATCH_WR_VA(AB, 4) ", " PATCH_WR_VBL(SET) ", " PATCH_WR_C(2, CB) "\n\t" \
    PATCH_WR_LD3_##CB(ABN)                                                                                         \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(3, CB) ", " PATCH_WR_VA(AB, 6) ", " PATCH_WR_VBL(SET) ", " PATCH_WR_C(3, CB) "\n\t" \
    PATCH_WR_LD4_##CB(ABN)                                                                                         \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(0, CB) ", " PATCH_WR_VA(AB, 1) ", " PATCH_WR_VBH(SET) ", " PATCH_WR_C(0, CB) "\n\t" \
    PATCH_WR_K1_##CB##_##PAR                                                                                       \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(1, CB) ", " PATCH_WR_VA(AB, 3) ", " PATCH_WR_VBH(SET) ", " PATCH_WR_C(1, CB) "\n\t" \
    PATCH_WR_K2_##CB##_##PAR                                                                                       \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(2, CB) ", " PATCH_WR_VA(AB, 5) ", " PATCH_WR_VBH(SET) ", " PATCH_WR_C(2, CB) "\n\t" \
    PATCH_WR_K3_##CB##_##PAR                                                                                       \
    "v_mfma_f32_16x16x32_bf16 " PATCH_WR_C(3, CB) ", " PATCH_WR_VA(AB, 7) ", " PATCH_WR_VBH(SET) ", " PATCH_WR_C(3, CB) "\n\t"
#define PATCH_WR_PIECE_SPARSE(CB, SET, NSET, AB, ABN, J, PAR, OFF) PATCH_WR_PIECE_SPARSE_(CB, SET, NSET, AB, ABN, J, PAR, OFF)
#define PATCH_WR_PIECE_SPARSE_(CB, SET, NSET, AB, ABN, J, PAR, OFF)                                                \
    PATCH_WR_PRE_##CB                                                                                              \
    "s_waitcnt lgkmcnt(12)\n\t"                                                                                    \
    "v_smfmac_f32_16x16x64_bf16 " PATCH_WR_C(0, CB) ", " PATCH_WR_VA(AB, 0) ", " PATCH_WR_VB(SET) ", " PATCH_WR_VI(AB, 0) " abid:" #J "\n\t" \
    "ds_read_b128 " PATCH_WR_VBL(NSET) ", " PATCH_WR_RAL_##CB(PAR) " offset:" #OFF "\n\t"                          \
    "ds_read_b128 " PATCH_WR_VBH(NSET) ", " PATCH_WR_RAH_##CB(PAR) " offset:" #OFF "\n\t"                          \
    "v_smfmac_f32_16x16x64_bf16 " PATCH_WR_C(1, CB) ", " PATCH_WR_VA(AB, 1) ", " PATCH_WR_VB(SET) ", " PATCH_WR_VI(AB, 1) " abid:" #J "\n\t" \
    PATCH_WR_LD3_##CB(ABN)                                                                                         \
    PATCH_WR_K1_##CB##_##PAR                                                                                       \
    "v_smfmac_f32_16x16x64_bf16 " PATCH_WR_C(2, CB) ", " PATCH_WR_VA(AB, 2) ", " PATCH_WR_VB(SET) ", " PATCH_WR_VI(AB, 2) " abid:" #J "\n\t" \
    PATCH_WR_LD4_##CB(ABN)                                                                                         \
    PATCH_WR_K2_##CB##_##PAR                                                                                       \
    "v_smfmac_f32_16x16x64_bf16 " PATCH_WR_C(3, CB) ", " PATCH_WR_VA(AB, 3) ", " PATCH_WR_VB(SET) ", " PATCH_WR_VI(AB, 3) " abid:" #J "\n\t" \
    PATCH_WR_K3_##CB##_##PAR
// weight load I of a step into buffer AB: 16 bytes per lane, asynchronous
#define PATCH_WR_LOAD_A(AB, I, voff_, base_)                                                                       \
    asm volatile("global_load_dwordx4 " PATCH_WR_VA(AB, I) ", %0, %1" : : "v"(voff_), "s"(base_) : PATCH_WR_CLOBBER)
// first LDS reads of the kernel (column block CB of stage 0 into set CB)
#define PATCH_WR_LDS_FIRST(CB, al_, ah_)                                                                           \
    asm volatile("ds_read_b128 " PATCH_WR_VBL(CB) ", %0 offset:2048*" #CB "\n\t"                                   \
                 "ds_read_b128 " PATCH_WR_VBH(CB) ", %1 offset:2048*" #CB                                          \
                 :                                                                                                 \
                 : "v"(al_), "v"(ah_)                                                                              \
                 : PATCH_WR_CLOBBER)
// column blocks of a step with their operand sets: P(CB, SET, NSET)
#define PATCH_WR_16(P) P(0, 0, 7) P(1, 1, 0) P(2, 2, 1) P(3, 3, 2) P(4, 4, 3) P(5, 5, 4) P(6, 6, 5) P(7, 7, 6) P(8, 0, 7) P(9, 1, 0) P(10, 2, 1) P(11, 3, 2) P(12, 4, 3) P(13, 5, 4) P(14, 6, 5) P(15, 7, 6)


// Y = sum over the slices of the partial products, slice 0 first: a fixed order, so the result is reproducible.
// (Adding the partials to Y with fp32 atomics instead was 2-3x slower than this second launch.)
__global__ __launch_bounds__(256) void wr_reduce_kernel(const wr_f32x4* __restrict__ ws, size_t n4, int slices, float* __restrict__ Y, int ybf16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        wr_f32x4 acc = ws[i];
        for (int s = 1; s < slices; ++s) {
            const wr_f32x4 v = ws[(size_t)s * n4 + i];
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        store4(Y, (int64_t)(4 * i), acc, ybf16);
    }
}

// The same for a set of weights in one launch: blockIdx.y = weight; its slices lie one behind the other at ws[y].
struct WrReduceSet {
    const float* ws[kMaxMany];
    float* Y[kMaxMany];
    size_t n4[kMaxMany];
};
__global__ __launch_bounds__(256) void wr_reduce_set_kernel(const WrReduceSet set, int slices, int ybf16) {
    const int y = blockIdx.y;
    const wr_f32x4* ws = reinterpret_cast<const wr_f32x4*>(set.ws[0]);
    float* Y = set.Y[0];
    size_t n4 = set.n4[0];
#pragma unroll
    for (int i = 1; i < kMaxMany; ++i)
        if (y == i) { ws = reinterpret_cast<const wr_f32x4*>(set.ws[i]); Y = set.Y[i]; n4 = set.n4[i]; }
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        wr_f32x4 acc = ws[i];
        for (int s = 1; s < slices; ++s) {
            const wr_f32x4 v = ws[(size_t)s * n4 + i];
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        store4(Y, (int64_t)(4 * i), acc, ybf16);
    }
}

__device__ __forceinline__ uint64_t wr_uniform64(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// Tile t of the launch order -> feature block bn (256 features), row block bm (256 rows): groups of 4 row blocks x
// all feature blocks, so that the workgroups an XCD runs at a time cover about 8 feature blocks x 4 row blocks
// and share both operands in its L2.
__device__ __forceinline__ void wr_tile_of(int t, int tiles_n, int tiles_m, int& bn, int& bm) {
    constexpr int GM = 4;
    const int full = (tiles_m / GM) * GM * tiles_n;
    if (t < full) {
        const int g = t / (GM * tiles_n), rem = t % (GM * tiles_n);
        bn = rem / GM;
        bm = g * GM + rem % GM;
    } else {
        const int gm = tiles_m % GM, rem = t - full;
        bn = rem / gm;
        bm = (tiles_m / GM) * GM + rem % gm;
    }
}

// Sum of the partial tiles of a MODE 2 launch (slot (t - t0) * slices + y, 256 rows x 256 features each, slice 0
// first) into Y.  Block = 16 rows of one tile; thread = 4 x 4 features of one row.
__global__ __launch_bounds__(256) void wr_tail_reduce_kernel(const float* __restrict__ ws, int slices, int t0, int tiles_n, int tiles_m,
                                                             int64_t M, int Tk_all, const WeightSet set, int ybf16) {
    const int j = blockIdx.x >> 4, chunk = blockIdx.x & 15;
    int bn, bm;
    wr_tile_of(t0 + j, tiles_n, tiles_m, bn, bm);
    const uint32_t* table = set.table[0];
    float* Y = set.Y[0];
    int64_t N = set.N[0];
    int first = 0;
    for (int i = 1; i < set.count; ++i)
        if (bn >= set.first[i]) { table = set.table[i]; Y = set.Y[i]; N = set.N[i]; first = set.first[i]; }
    bn -= first;
    const int32_t* pairs = reinterpret_cast<const int32_t*>(table) + (N / 128) * (int64_t)Tk_all;
    const int r = 16 * chunk + (threadIdx.x >> 4);
    const int64_t m = (int64_t)bm * kWrBM + r;
    if (m >= M) return;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int f = (threadIdx.x & 15) * 4 + 64 * u;   // feature inside the 256-feature block
        const int row = pairs[2 * bn + (f >> 7)];
        if (row < 0) continue;                           // no second tile row
        const float* src = ws + (int64_t)j * slices * (kWrBM * kWrBN) + r * kWrBN + f;
        wr_f32x4 acc = *reinterpret_cast<const wr_f32x4*>(src);
        for (int y = 1; y < slices; ++y) {
            const wr_f32x4 v = *reinterpret_cast<const wr_f32x4*>(src + (int64_t)y * (kWrBM * kWrBN));
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        store4(Y, m * N + (int64_t)row * 128 + (f & 127), acc, ybf16);
    }
}

// The launch covers tiles t0 .. t0 + cnt - 1 of the order above.
// MODE 0: whole K, results to Y.
// MODE 1: K split over gridDim.y workgroups per output tile (a grid of tiles alone would leave most of the chip
//         idle); slice y writes its partial product to Y + y * M * N (a workspace), wr_reduce_kernel sums the slices.
// MODE 2: the same split for the last few tiles of a launch whose tile count is a little more than a multiple of the
//         CU count (a part-filled last round): slice y of tile t writes a 256 x 256 partial tile to slot
//         (t - t0) * gridDim.y + y of the workspace, wr_tail_reduce_kernel sums the slots into Y.
template <int MODE>
__global__ __launch_bounds__(256) void prefill_kernel_wreg(const uint16_t* __restrict__ X, int64_t M, int64_t K, int Tk_all, int tiles_n,
                                                           int tiles_m, int t0, int cnt, const WeightSet set, int ybf16) {
    constexpr bool SPLIT = MODE != 0;
    constexpr int TILE = 128;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tr = w >> 1, sh = w & 1;  // tile row of the block, half (4 strips) of the tile
    const int col = lane & 15, q = lane >> 4;

    // ---- block -> tile of the launch order.  Consecutive blocks go to different XCDs (hardware round-robin), each
    // with its own L2, so every XCD gets a contiguous run of this launch's part of the order.
    int bid = blockIdx.x;
    {
        const int per = (cnt + 7) / 8;
        const int x = bid & 7, i = bid >> 3;
        const int t = x * per + i;
        bid = (i < per && t < cnt) ? t0 + t : -1;
    }
    if (bid < 0) return;
    int bn, bm;
    wr_tile_of(bid, tiles_n, tiles_m, bn, bm);
    // which weight of the set the feature block belongs to: scalar selects, made explicitly uniform, so that the
    // weight addresses stay in scalar registers
    const uint8_t* __restrict__ payload = set.payload[0];
    const uint32_t* __restrict__ table = set.table[0];
    float* __restrict__ Y = set.Y[0];
    int64_t N = set.N[0];
    if (set.count > 1) {
        int first = 0;
#pragma unroll
        for (int i = 1; i < kMaxMany; ++i) {
            const bool here = i < set.count && bn >= set.first[i];
            payload = here ? set.payload[i] : payload;
            table = here ? set.table[i] : table;
            Y = here ? set.Y[i] : Y;
            N = here ? set.N[i] : N;
            first = here ? set.first[i] : first;
        }
        bn -= __builtin_amdgcn_readfirstlane(first);
    }
    payload = reinterpret_cast<const uint8_t*>(wr_uniform64(reinterpret_cast<uint64_t>(payload)));
    table = reinterpret_cast<const uint32_t*>(wr_uniform64(reinterpret_cast<uint64_t>(table)));
    Y = reinterpret_cast<float*>(wr_uniform64(reinterpret_cast<uint64_t>(Y)));
    N = (int64_t)wr_uniform64((uint64_t)N);
    const int64_t m0 = (int64_t)bm * kWrBM;
    // The two tile rows of feature block bn: rows pairs[2 bn], pairs[2 bn + 1] of the list behind the table, chosen
    // by the packer so that both are 2:4 in as many steps as possible (the wavefronts meet at a barrier every step:
    // a step with one dense and one 2:4 tile row lasts as long as a dense one).
    // With an odd number of tile rows the last block has no second row (-1): its wavefronts copy X and meet the
    // barriers like the others, read the first row's weights (valid addresses) and multiply nothing.
    // (read through the constant address space: a scalar load; the table pointer came out of scalar selects, after
    // which the compiler no longer knows its address space and would use flat vector loads)
    const __attribute__((address_space(4))) int32_t* pairs =
        reinterpret_cast<const __attribute__((address_space(4))) int32_t*>(reinterpret_cast<uintptr_t>(table)) + (N / TILE) * (int64_t)Tk_all;
    const int row0 = pairs[2 * bn], row1 = pairs[2 * bn + 1];
    const bool live = tr == 0 || row1 >= 0;
    const int64_t nrow = (int64_t)__builtin_amdgcn_readfirstlane((tr == 0 || row1 < 0) ? row0 : row1) * TILE;  // first feature of this wavefront's tile row
    // this workgroup's K slice, in tiles: to the rest of the kernel it is a product with a shorter K
    const int t_begin = SPLIT ? (int)((int64_t)blockIdx.y * Tk_all / gridDim.y) : 0;
    const int Tk = SPLIT ? (int)((int64_t)(blockIdx.y + 1) * Tk_all / gridDim.y) - t_begin : Tk_all;
    const __attribute__((address_space(1))) uint32_t* trow =
        reinterpret_cast<const __attribute__((address_space(1))) uint32_t*>(reinterpret_cast<uintptr_t>(table)) + (nrow / TILE) * Tk_all + t_begin;

    // ---- per-lane sources of the X copy: wavefront w copies the 1 KB pieces w, w+4, ..., w+28 of the 32 KB stage.
    // LDS chunk c (16 bytes) = row c / 8, physical chunk c % 8, which holds logical chunk (c % 8) ^ ((row / 2) % 8):
    // 16 consecutive rows reading the same logical chunk then hit 16 distinct 16-byte bank groups.
    // Byte offsets from X + step * 128 (a scalar base); the host keeps M * K * 2 below 4 GB for this kernel.
    uint32_t xoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = (w + 4 * i) * 64 + lane;
        const int m = c >> 3, pp = c & 7, pl = pp ^ ((m >> 1) & 7);
        int64_t row = m0 + m;
        if (row >= M) row = M - 1;  // rows past M: any valid row, their outputs are not stored
        xoff[i] = (uint32_t)((row * K + pl * 8) * 2);
    }
    const uint8_t* const xbase = reinterpret_cast<const uint8_t*>(X) + (size_t)t_begin * (TILE * 2);
    // ---- per-lane LDS read addresses of a column block's two operands (+ stage * 32 KB + block * 2 KB)
    const uint32_t lds0 = (uint32_t)(size_t)((wr_lptr_t)lds);
    const int swz = (col >> 1) & 7;
    const uint32_t bl0 = lds0 + col * 128 + ((q ^ swz) << 4);
    const uint32_t bh0 = lds0 + col * 128 + (((4 + q) ^ swz) << 4);
    // ---- weight loads of one step: 8 instructions ("slots") per wavefront whatever the tile type, each 16 bytes per
    // lane from a scalar address that is selected, not branched on:
    //   dense slot i    : operand i % 2 of strip i / 2 at K-step j
    //   2:4 slot i < 4  : values of strip i at K-step j
    //   2:4 slot 4 + s  : 16 bytes starting at the lane's position dword of strip s (the first register is the
    //                     dword, the rest is ignored; the last lanes read up to 12 bytes into the next tile or the
    //                     zeroed slack behind the payload)
    const uint32_t vlane16 = lane * 16, vlane4 = lane * 4;
    auto a_base = [&](int slot, int j, uint32_t e) -> const uint8_t* {
        const int cd = sh * 4 * 2 * kDenseFragBytes + (slot >> 1) * 2 * kDenseFragBytes + j * kDenseFragBytes + (slot & 1) * 1024;
        const int cs = slot < 4 ? sh * 4 * 2 * kSparseFragBytes + slot * 2 * kSparseFragBytes + j * kSparseFragBytes
                                : sparse_vals_bytes(TILE) + (4 * sh + slot - 4) * 64 * 4;
        return payload + entry_offset(e) + (entry_sparse(e) ? cs : cd);
    };
    auto a_voff = [&](int slot, uint32_t e) { return (slot >= 4 && entry_sparse(e)) ? vlane4 : vlane16; };
#define PATCH_WR_LOAD_STEP(AB, j_, e_)                                                                             \
    PATCH_WR_LOAD_A(AB, 0, a_voff(0, e_), a_base(0, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 1, a_voff(1, e_), a_base(1, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 2, a_voff(2, e_), a_base(2, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 3, a_voff(3, e_), a_base(3, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 4, a_voff(4, e_), a_base(4, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 5, a_voff(5, e_), a_base(5, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 6, a_voff(6, e_), a_base(6, j_, e_));                                                      \
    PATCH_WR_LOAD_A(AB, 7, a_voff(7, e_), a_base(7, j_, e_));
    // X loads of one step (8 instructions) into a ring stage: prologue only, the loop issues them from the
    // column-block statements.  m0 = LDS byte address of the wavefront's 1 KB piece.
    auto load_x_slot = [&](int slot, int s, int stage) {
        const uint8_t* xb = xbase + (size_t)s * 128;
        const uint32_t m0v = lds0 + stage * kWrStage + (w + 4 * slot) * 1024;
        // (one wait state between the write of m0 and the load that reads it as its LDS base)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(xoff[slot]), "s"(xb) : "memory");
    };

    const int S = 2 * Tk;  // 64-column steps
    // the tile row's table entries: lane l of ent[i] holds tile 64 i + l; the loop fetches them with v_readlane (a
    // scalar load in the loop would be waited for with lgkmcnt(0), i.e. together with every LDS read in flight).
    // Tk <= 128 (prefill_wreg_supports).
    uint32_t ent[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int t = 64 * i + lane;
        ent[i] = trow[t < Tk ? t : Tk - 1];
    }
    // a use right here: the compiler waits for these loads now
    asm volatile("" : "+v"(ent[0]), "+v"(ent[1]));

    // accumulators: zero
#define PATCH_WR_ZERO(CB, SET, NSET)                                                                               \
    asm volatile("v_accvgpr_write_b32 a[16*" #CB "+0], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+1], 0\n\t"            \
                 "v_accvgpr_write_b32 a[16*" #CB "+2], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+3], 0\n\t"            \
                 "v_accvgpr_write_b32 a[16*" #CB "+4], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+5], 0\n\t"            \
                 "v_accvgpr_write_b32 a[16*" #CB "+6], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+7], 0\n\t"            \
                 "v_accvgpr_write_b32 a[16*" #CB "+8], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+9], 0\n\t"            \
                 "v_accvgpr_write_b32 a[16*" #CB "+10], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+11], 0\n\t"          \
                 "v_accvgpr_write_b32 a[16*" #CB "+12], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+13], 0\n\t"          \
                 "v_accvgpr_write_b32 a[16*" #CB "+14], 0\n\tv_accvgpr_write_b32 a[16*" #CB "+15], 0" ::: PATCH_WR_CLOBBER);
    PATCH_WR_16(PATCH_WR_ZERO)
#undef PATCH_WR_ZERO

    // ---- prologue, in the order the steady state would have produced: X(0) | A(0) X(1) | A(1) X(2)
    {
        const uint32_t e0 = __builtin_amdgcn_readlane(ent[0], 0);   // tile 0: steps 0 and 1
        const int s1 = S > 1 ? 1 : 0, s2 = S > 2 ? 2 : S - 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) load_x_slot(i, 0, 0);
        asm volatile("" ::: "memory");
        PATCH_WR_LOAD_STEP(0, 0, e0)
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < 8; ++i) load_x_slot(i, s1, 1);
        asm volatile("" ::: "memory");
        PATCH_WR_LOAD_STEP(1, 1, e0)
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < 8; ++i) load_x_slot(i, s2, 2);
    }
    asm volatile("s_waitcnt vmcnt(24)" ::: "memory");  // X(0) (and A(0)) landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // X operands: column block cb lives in set cb % 8 and is requested seven blocks ahead.  Before block cb the
    // reads of blocks cb .. cb+6 (two each) are in flight; waiting until twelve are left completes block cb.
    PATCH_WR_LDS_FIRST(0, bl0, bh0);
    PATCH_WR_LDS_FIRST(1, bl0, bh0);
    PATCH_WR_LDS_FIRST(2, bl0, bh0);
    PATCH_WR_LDS_FIRST(3, bl0, bh0);
    PATCH_WR_LDS_FIRST(4, bl0, bh0);
    PATCH_WR_LDS_FIRST(5, bl0, bh0);
    PATCH_WR_LDS_FIRST(6, bl0, bh0);

    // lane offsets of the weight loads inside a tile: dense operands, 2:4 values, 2:4 position dwords
    const uint32_t vd = lane * 16 + sh * 4 * 2 * kDenseFragBytes, vs = lane * 16 + sh * 4 * 2 * kSparseFragBytes;
    const uint32_t vm = lane * 4 + sh * 4 * 64 * 4;
// LDS offset of the column block seven ahead
#define PATCH_WR_OFF_0 14336
#define PATCH_WR_OFF_1 16384
#define PATCH_WR_OFF_2 18432
#define PATCH_WR_OFF_3 20480
#define PATCH_WR_OFF_4 22528
#define PATCH_WR_OFF_5 24576
#define PATCH_WR_OFF_6 26624
#define PATCH_WR_OFF_7 28672
#define PATCH_WR_OFF_8 30720
#define PATCH_WR_OFF_9 0
#define PATCH_WR_OFF_10 2048
#define PATCH_WR_OFF_11 4096
#define PATCH_WR_OFF_12 6144
#define PATCH_WR_OFF_13 8192
#define PATCH_WR_OFF_14 10240
#define PATCH_WR_OFF_15 12288
// One step = 16 column blocks of one type.  SS = position in the round of six steps (three tiles: step buffer = SS % 3
// and K-step = SS % 2 are then compile-time constants), AB / ABN = weight buffers of steps s / s+2, J = K-step in the
// tile, PAR = SS % 2 = which lane address pair is "cur".
#define PATCH_WR_BODY_D_0(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 0, 2, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_D_1(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 1, 0, 1, 1, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_D_2(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 2, 1, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_D_3(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 0, 2, 1, 1, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_D_4(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 1, 0, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_D_5(CB, SET, NSET) PATCH_WR_PIECE_DENSE(CB, SET, NSET, 2, 1, 1, 1, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_0(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 0, 2, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_1(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 1, 0, 1, 1, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_2(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 2, 1, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_3(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 0, 2, 1, 1, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_4(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 1, 0, 0, 0, PATCH_WR_OFF_##CB)
#define PATCH_WR_BODY_S_5(CB, SET, NSET) PATCH_WR_PIECE_SPARSE(CB, SET, NSET, 2, 1, 1, 1, PATCH_WR_OFF_##CB)
// The dense steps of a round lie one behind the other, and so do the 2:4 steps: a step whose tile has the type of
// the one before is entered by falling through, and only a change of type (at most once per tile) takes a branch - a
// taken branch is a bubble in the matrix pipe.  Head of step SS in either chain: an even step ends the loop when
// s = S (S is even); A(s) has landed (the loads issued after it are X(s+1), A(s+1), X(s+2)); then the type check.
#define PATCH_WR_END_CHECK_0 "s_cmp_ge_i32 s80, %[S]\n\ts_cbranch_scc1 WR_END_%=\n\t"
#define PATCH_WR_END_CHECK_1 ""
#define PATCH_WR_STEP_D(SS, EVEN)                                                                                  \
    "WR_D" #SS "_%=:\n\t" PATCH_WR_END_CHECK_##EVEN "s_waitcnt vmcnt(24)\n\t"                                       \
    "s_cmp_lg_u32 s87, 0\n\ts_cbranch_scc1 WR_SB" #SS "_%=\n\t"                                                    \
    "WR_DB" #SS "_%=:\n\t" PATCH_WR_16(PATCH_WR_BODY_D_##SS)
#define PATCH_WR_STEP_S(SS, EVEN)                                                                                  \
    "WR_S" #SS "_%=:\n\t" PATCH_WR_END_CHECK_##EVEN "s_waitcnt vmcnt(24)\n\t"                                       \
    "s_cmp_eq_u32 s87, 0\n\ts_cbranch_scc1 WR_DB" #SS "_%=\n\t"                                                    \
    "WR_SB" #SS "_%=:\n\t" PATCH_WR_16(PATCH_WR_BODY_S_##SS)
    {
        const uint64_t xb64 = reinterpret_cast<uint64_t>(xbase), pl64 = reinterpret_cast<uint64_t>(payload);
        const uint32_t xlo = (uint32_t)xb64, xhi = (uint32_t)(xb64 >> 32), plo = (uint32_t)pl64, phi = (uint32_t)(pl64 >> 32);
        const uint32_t ldsw = lds0 + w * 1024;
        const int sm1 = S - 1, tkm1 = Tk - 1;
        const int live_i = __builtin_amdgcn_readfirstlane(live ? 1 : 0);
        asm volatile(
            // ---- lane offsets of the eight weight-load slots for either tile type
            "v_mov_b32 v236, %[vd]\n\tv_add_u32 v237, 1024, %[vd]\n\tv_add_u32 v238, 4096, %[vd]\n\tv_add_u32 v239, 5120, %[vd]\n\t"
            "v_add_u32 v240, 8192, %[vd]\n\tv_add_u32 v241, 9216, %[vd]\n\tv_add_u32 v242, 12288, %[vd]\n\tv_add_u32 v243, 13312, %[vd]\n\t"
            "v_mov_b32 v244, %[vs]\n\tv_add_u32 v245, 2048, %[vs]\n\tv_add_u32 v246, 4096, %[vs]\n\tv_add_u32 v247, 6144, %[vs]\n\t"
            "v_add_u32 v248, 16384, %[vm]\n\tv_add_u32 v249, 16640, %[vm]\n\tv_add_u32 v250, 16896, %[vm]\n\tv_add_u32 v251, 17152, %[vm]\n\t"
            // ---- state of step 0: stages 0 / 1, the weight loads fetch K-step 0 of tile min(1, Tk - 1), tile 0 is multiplied
            "s_mov_b32 s80, 0\n\t"
            "v_mov_b32 v224, %[bl0]\n\tv_mov_b32 v225, %[bh0]\n\t"
            "v_add_u32 v226, 0x8000, %[bl0]\n\tv_add_u32 v227, 0x8000, %[bh0]\n\t"
            "s_min_u32 s88, 1, %[tkm1]\n\t"
            "v_readlane_b32 s76, %[ent0], s88\n\t"
            "s_lshr_b32 s94, s76, 1\n\ts_mov_b32 s95, 0\n\ts_lshl_b64 s[94:95], s[94:95], 8\n\t"
            "s_add_u32 s74, %[plo], s94\n\ts_addc_u32 s75, %[phi], s95\n\t"
            "s_mov_b64 s[84:85], s[74:75]\n\ts_mov_b64 s[96:97], s[74:75]\n\t"
            "s_bitcmp1_b32 s76, 0\n\ts_cselect_b32 s86, -1, 0\n\ts_cselect_b64 s[92:93], -1, 0\n\t"
            "v_readlane_b32 s89, %[ent0], 0\n\t"
            "s_and_b32 s87, s89, %[live]\n\t"
            "v_cndmask_b32_e64 v228, v236, v244, s[92:93]\n\tv_cndmask_b32_e64 v229, v237, v245, s[92:93]\n\t"
            "v_cndmask_b32_e64 v230, v238, v246, s[92:93]\n\tv_cndmask_b32_e64 v231, v239, v247, s[92:93]\n\t"
            "v_cndmask_b32_e64 v232, v240, v248, s[92:93]\n\tv_cndmask_b32_e64 v233, v241, v249, s[92:93]\n\t"
            "v_cndmask_b32_e64 v234, v242, v250, s[92:93]\n\tv_cndmask_b32_e64 v235, v243, v251, s[92:93]\n\t"
            // ---- the loop: a round of six dense steps, a round of six 2:4 steps, entered at step 0 of the dense chain
            PATCH_WR_STEP_D(0, 0) PATCH_WR_STEP_D(1, 1) PATCH_WR_STEP_D(2, 0) PATCH_WR_STEP_D(3, 1) PATCH_WR_STEP_D(4, 0) PATCH_WR_STEP_D(5, 1)
            "s_branch WR_D0_%=\n\t"
            PATCH_WR_STEP_S(0, 0) PATCH_WR_STEP_S(1, 1) PATCH_WR_STEP_S(2, 0) PATCH_WR_STEP_S(3, 1) PATCH_WR_STEP_S(4, 0) PATCH_WR_STEP_S(5, 1)
            "s_branch WR_S0_%=\n\t"
            "WR_END_%=:"
            :
            : [S] "s"(S), [sm1] "s"(sm1), [tkm1] "s"(tkm1), [live] "s"(live_i), [xlo] "s"(xlo), [xhi] "s"(xhi), [plo] "s"(plo), [phi] "s"(phi),
              [ldsw] "s"(ldsw), [bl0] "v"(bl0), [bh0] "v"(bh0), [vd] "v"(vd), [vs] "v"(vs), [vm] "v"(vm), [ent0] "v"(ent[0]), [ent1] "v"(ent[1]),
              [xo0] "v"(xoff[0]), [xo1] "v"(xoff[1]), [xo2] "v"(xoff[2]), [xo3] "v"(xoff[3]), [xo4] "v"(xoff[4]), [xo5] "v"(xoff[5]),
              [xo6] "v"(xoff[6]), [xo7] "v"(xoff[7])
            : "memory", "scc", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", "v233", "v234", "v235", "v236", "v237",
              "v238", "v239", "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", "v248", "v249", "v250", "v251", "s74", "s75", "s76",
              "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95", "s96", "s97",
              PATCH_WR_CLOBBER);
    }
#undef PATCH_WR_STEP_D
#undef PATCH_WR_STEP_S

    // outstanding (re-fetched) loads and the reads requested for a step that does not exist must land before this
    // workgroup's LDS and registers can be handed on; the last matrix instructions may still be writing
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory", PATCH_WR_CLOBBER);

    // accumulator (s, cb), register r: feature nrow + 16 (4 sh + s) + 4 q + r, row m0 + 16 cb + col.
    // Stored from there, one instruction writes 16 rows x 64 bytes (half cache lines); a compute unit then takes about
    // 7 us for its 256 KB however idle the memory is, and a bf16 Y (quarter lines) is bound by the pattern, not by its
    // bytes (patch_probe_store_tiles runs both patterns on their own).  So every column block
    // (16 rows x this wavefront's 64 features) is turned through 4 KB of LDS of the wavefront's own, behind the X ring
    // (no barrier: a wavefront's LDS instructions execute in order): written as it lies in the registers, read back
    // as 4 rows x 256 contiguous bytes per instruction.  16-byte chunk c of row r sits at chunk c ^ r: the 16 lanes
    // that write one chunk column, and the 16 that read one row, each touch all 64 banks once.
    if (live) {
        uint8_t* const stg = lds + kWrRing + w * kWrOut;
        const int rr = lane >> 4, ch = lane & 15;   // as a reader: row rr of every four, chunk ch = features 4 ch .. 4 ch + 3
#define PATCH_WR_READ(S, CB)                                                                                       \
    asm volatile("v_accvgpr_read_b32 %0, a[4*(16*" #S "+" #CB ")+0]\n\tv_accvgpr_read_b32 %1, a[4*(16*" #S "+" #CB ")+1]\n\t" \
                 "v_accvgpr_read_b32 %2, a[4*(16*" #S "+" #CB ")+2]\n\tv_accvgpr_read_b32 %3, a[4*(16*" #S "+" #CB ")+3]"       \
                 : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3]))
#define PATCH_WR_STAGE(S, CB)                                                                                      \
    PATCH_WR_READ(S, CB);                                                                                          \
    *reinterpret_cast<wr_f32x4*>(stg + col * 256 + (((4 * S + q) ^ col) << 4)) = wr_f32x4{v[0], v[1], v[2], v[3]};
#define PATCH_WR_STORE(CB, SET, NSET)                                                                              \
    {                                                                                                              \
        float v[4];                                                                                                \
        PATCH_WR_STAGE(0, CB) PATCH_WR_STAGE(1, CB) PATCH_WR_STAGE(2, CB) PATCH_WR_STAGE(3, CB)                    \
        wr_f32x4 o[4];                                                                                             \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) { /* all four reads before the first store waits for one */  \
            const int r = 4 * j + rr;                                                                              \
            o[j] = *reinterpret_cast<const wr_f32x4*>(stg + r * 256 + ((ch ^ r) << 4));                            \
        }                                                                                                          \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                            \
            const int r = 4 * j + rr; /* row inside the column block */                                            \
            const int64_t m = m0 + 16 * CB + r;                                                                    \
            /* element offset of this lane's four features: a workspace slot (MODE 2), a workspace slice (MODE 1), Y */ \
            const int64_t ye = MODE == 2 ? ((int64_t)(bid - t0) * gridDim.y + blockIdx.y) * (kWrBM * kWrBN) + (16 * CB + r) * kWrBN + 128 * tr + 64 * sh + 4 * ch \
                                         : (MODE == 1 ? (int64_t)blockIdx.y * M * N : 0) + m * N + nrow + 64 * sh + 4 * ch;     \
            if (MODE == 2 || m < M) store4(Y, ye, o[j], PATCH_WR_YB);                                                       \
        }                                                                                                          \
    }
        // (the bf16 choice is taken once, not per store: MODE 1 / 2 write fp32 partial products, their sum is rounded by the reduction)
        if (MODE == 0 && ybf16) {
#define PATCH_WR_YB 1
            PATCH_WR_16(PATCH_WR_STORE)
#undef PATCH_WR_YB
        } else {
#define PATCH_WR_YB 0
            PATCH_WR_16(PATCH_WR_STORE)
#undef PATCH_WR_YB
        }
#undef PATCH_WR_STAGE
#undef PATCH_WR_STORE
#undef PATCH_WR_READ
    }
}

// Limits of the kernel: 32-bit lane offsets into X, two registers of table entries per tile row (128 tiles).
bool prefill_wreg_supports(const GemmArgs& a) {
    return a.tile == 128 && a.M > 0 && a.K <= 128 * 128 && (uint64_t)a.M * (uint64_t)a.K * 2 < (1ull << 32);
}

// K slices per output tile: as many as the workspace a.ws holds partial products for (M N fp32 each), at most
// `requested` if > 0, else as many as fill the chip when the tile grid covers less than about two thirds of it -
// each slice at least four tiles (eight steps) long, at most 8.  1 = no split (no workspace needed).
int prefill_wreg_split(const GemmArgs& a, int requested) {
    const int tiles = (int)(((a.N + kWrBN - 1) / kWrBN) * ((a.M + kWrBM - 1) / kWrBM));
    int s = requested;
    if (s <= 0) {
        s = 1;
        if (tiles < (a.n_cus * 2) / 3) {
            s = a.n_cus / tiles;
            if (s > a.Tk / 4) s = a.Tk / 4;
            if (s > 8) s = 8;
        }
    }
    if (s > a.Tk) s = a.Tk;
    const size_t per_slice = (size_t)a.M * (size_t)a.N * sizeof(float);
    const size_t fit = (a.ws && per_slice) ? a.ws_bytes / per_slice : 0;
    if ((size_t)s > fit) s = (int)fit;
    return s < 2 ? 1 : s;
}

// A launch whose tile count is a little more than a multiple of the CU count ends with a part-filled round that
// lasts as long as a full one.  With a workspace the last `tail` tiles (at most half a round) are cut into K slices
// that fill the chip once: returns the slice count (1 = no such split) and sets *tail.  It pays when the part of a
// round it saves outweighs writing and re-reading the partial tiles (an estimate from measured rates: 0.9 - 1.25 us
// per step depending on how full the chip is, 3 TB/s for the partials, 8 us for the two extra launches).
int prefill_wreg_tail(const GemmArgs& a, int* tail) {
    return prefill_wreg_tail_of((int)(((a.N + kWrBN - 1) / kWrBN) * ((a.M + kWrBM - 1) / kWrBM)), a, tail);
}

int prefill_wreg_tail_of(int tiles, const GemmArgs& a, int* tail) {
    const int t = tiles % a.n_cus;
    *tail = 0;
    if (!a.ws || tiles < a.n_cus || t == 0 || 2 * t > a.n_cus) return 1;
    int s = a.n_cus / t;
    if (s > 8) s = 8;
    if (s > a.Tk / 4) s = a.Tk / 4;
    const size_t per_slot = (size_t)kWrBM * kWrBN * sizeof(float);
    while (s >= 2 && (size_t)t * (size_t)s * per_slot > a.ws_bytes) --s;
    if (s < 2) return 1;
    // after more than three full rounds the workgroups are far out of step and a part-filled round costs much less
    // than a full one (gate + up in one launch, 5.4 rounds: splitting the last 96 tiles measured 4 % slower)
    // a K-step costs 0.9 us on a nearly empty chip and 1.25 us on a full one: the part-filled round is shorter than a
    // full round to begin with, and its slices run on a fuller chip
    const double fill = (double)t / a.n_cus, fill_s = (double)t * s / a.n_cus;
    const double round_us = 2.0 * a.Tk * (0.9 + 0.35 * fill) * (tiles / a.n_cus > 3 ? 0.4 : 1.0);
    const double gain_us = round_us - 2.0 * a.Tk / s * (0.9 + 0.35 * (fill_s < 1.0 ? fill_s : 1.0)) * (tiles / a.n_cus > 3 ? 0.4 : 1.0);
    const double cost_us = 2.0 * (double)t * s * per_slot / 3.0e6 + 8.0;
    if (gain_us <= cost_us) return 1;
    *tail = t;
    return s;
}

static void wr_grant_lds() {
    static const hipError_t granted0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_wreg<0>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kWrLds);
    static const hipError_t granted1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_wreg<1>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kWrLds);
    static const hipError_t granted2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel_wreg<2>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kWrLds);
    (void)granted0;
    (void)granted1;
    (void)granted2;
}

void wr_reduce(const float* ws, size_t n4, int slices, float* Y, int ybf16, hipStream_t stream) {
    const size_t blocks = (n4 + 255) / 256;
    hipLaunchKernelGGL(wr_reduce_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, stream,
                       reinterpret_cast<const wr_f32x4*>(ws), n4, slices, Y, ybf16);
}

void launch_prefill_wreg(const GemmArgs& a, int split_k, hipStream_t stream) {
    wr_grant_lds();
    const int tiles_n = (int)((a.N + kWrBN - 1) / kWrBN), tiles_m = (int)((a.M + kWrBM - 1) / kWrBM);
    const int nblk = tiles_n * tiles_m;
    const int grid = ((nblk + 7) / 8) * 8;
    const int split = prefill_wreg_split(a, split_k);
    WeightSet set = {};
    set.payload[0] = a.payload;
    set.table[0] = a.table;
    set.N[0] = a.N;
    set.count = 1;
    set.units = tiles_n;
    int tail = 0;
    const int tail_split = (split == 1 && split_k == 0) ? prefill_wreg_tail(a, &tail) : 1;
    if (split == 1 && tail_split > 1) {
        // all full rounds unsplit, then the part-filled round in K slices over the whole chip, then their sum
        const int body = nblk - tail;
        set.Y[0] = a.Y;
        hipLaunchKernelGGL(prefill_kernel_wreg<0>, dim3(((body + 7) / 8) * 8), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk, tiles_n,
                           tiles_m, 0, body, set, a.ybf16);
        set.Y[0] = a.ws;
        hipLaunchKernelGGL(prefill_kernel_wreg<2>, dim3(((tail + 7) / 8) * 8, tail_split), dim3(256), kWrLds, stream, a.X, a.M, a.K,
                           a.Tk, tiles_n, tiles_m, body, tail, set, 0);
        set.Y[0] = a.Y;
        hipLaunchKernelGGL(wr_tail_reduce_kernel, dim3(tail * 16), dim3(256), 0, stream, a.ws, tail_split, body, tiles_n, tiles_m, a.M,
                           a.Tk, set, a.ybf16);
    } else if (split == 1) {
        set.Y[0] = a.Y;
        hipLaunchKernelGGL(prefill_kernel_wreg<0>, dim3(grid), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk, tiles_n, tiles_m, 0, nblk,
                           set, a.ybf16);
    } else {
        set.Y[0] = a.ws;
        hipLaunchKernelGGL(prefill_kernel_wreg<1>, dim3(grid, split), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk, tiles_n,
                           tiles_m, 0, nblk, set, 0);
        wr_reduce(a.ws, (size_t)a.M * (size_t)a.N / 4, split, a.Y, a.ybf16, stream);
    }
}

void launch_prefill_wreg_set(const GemmArgs& a, const WeightSet& set, hipStream_t stream) {
    wr_grant_lds();
    const int tiles_m = (int)((a.M + kWrBM - 1) / kWrBM);
    const int nblk = set.units * tiles_m;
    // A set whose tile grid covers less than about two thirds of the chip (q / k / v of a 13B layer at M = 512: 120
    // tiles): K in slices over the whole set in ONE launch - slice y of weight i writes its partial product to the
    // workspace region of that weight - and one reduction launch over all weights.  (One split launch and one
    // reduction per weight took 126 us on that set.)
    if (a.ws && nblk < (a.n_cus * 2) / 3) {
        int64_t out_floats = 0;
        for (int i = 0; i < set.count; ++i) out_floats += a.M * set.N[i];
        int split = a.n_cus / nblk;
        if (split > a.Tk / 4) split = a.Tk / 4;
        if (split > 8) split = 8;
        const size_t fit = out_floats ? a.ws_bytes / ((size_t)out_floats * sizeof(float)) : 0;
        if ((size_t)split > fit) split = (int)fit;
        if (split >= 2) {
            WeightSet part = set;
            WrReduceSet red = {};
            size_t off = 0, n4_max = 0;
            for (int i = 0; i < set.count; ++i) {
                part.Y[i] = a.ws + off;
                red.ws[i] = a.ws + off;
                red.Y[i] = set.Y[i];
                red.n4[i] = (size_t)a.M * (size_t)set.N[i] / 4;
                if (red.n4[i] > n4_max) n4_max = red.n4[i];
                off += (size_t)split * (size_t)a.M * (size_t)set.N[i];
            }
            hipLaunchKernelGGL(prefill_kernel_wreg<1>, dim3(((nblk + 7) / 8) * 8, split), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk,
                               set.units, tiles_m, 0, nblk, part, 0);
            const size_t blocks = (n4_max + 255) / 256;
            hipLaunchKernelGGL(wr_reduce_set_kernel, dim3((unsigned)(blocks < 2048 ? blocks : 2048), (unsigned)set.count), dim3(256), 0, stream,
                               red, split, a.ybf16);
            return;
        }
    }
    int tail = 0;
    const int tail_split = prefill_wreg_tail_of(nblk, a, &tail);   // 1 without a.ws
    if (tail_split > 1) {
        const int body = nblk - tail;
        hipLaunchKernelGGL(prefill_kernel_wreg<0>, dim3(((body + 7) / 8) * 8), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk, set.units,
                           tiles_m, 0, body, set, a.ybf16);
        WeightSet part = set;
        for (int i = 0; i < kMaxMany; ++i) part.Y[i] = a.ws;   // partial tiles go to workspace slots, whatever the weight
        hipLaunchKernelGGL(prefill_kernel_wreg<2>, dim3(((tail + 7) / 8) * 8, tail_split), dim3(256), kWrLds, stream, a.X, a.M, a.K,
                           a.Tk, set.units, tiles_m, body, tail, part, 0);
        hipLaunchKernelGGL(wr_tail_reduce_kernel, dim3(tail * 16), dim3(256), 0, stream, a.ws, tail_split, body, set.units, tiles_m, a.M,
                           a.Tk, set, a.ybf16);
        return;
    }
    const int grid = ((nblk + 7) / 8) * 8;
    hipLaunchKernelGGL(prefill_kernel_wreg<0>, dim3(grid), dim3(256), kWrLds, stream, a.X, a.M, a.K, a.Tk, set.units, tiles_m, 0, nblk,
                       set, a.ybf16);
}

}  // namespace patch
