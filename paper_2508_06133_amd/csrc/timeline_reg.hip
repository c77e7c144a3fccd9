// Timeline kernel with the future-memory profile held in vector registers.
//
// Phase 2 of Algorithm 1 ("Scheduling Execution"), one wavefront per candidate order, same
// search as the LDS-ring kernel (see simulate.hip): the k-th request of the order starts at
// the smallest round t >= the previous start at which P(tau) + s + (tau - t) <= M for all
// tau in (t, t + o]  (Eq. 1), P being the memory already committed to round tau.
//
// Layout.  The profile of rounds b64 .. b64 + 64 NR - 1 lives in NR vector registers: register
// r of lane l belongs to round b64 + 64 r + l and holds Q = P + 64 r.  b64 is kept equal to
// 64 floor((t+1)/64), so the window (t, t+o] of the request being placed always starts in
// register 0 and, with NR = ceil(o_max/64) + 1, always ends inside the file.  When t crosses
// a multiple of 64 the file moves down by one register (NR subtract-64 moves per 64 rounds
// of simulated time) and an empty row enters at the top.  There is no LDS traffic, no
// address arithmetic and no memory wait in the hot loops:
//   check   per row:  y = Q_r + (s - M);  c = min(y, 64 r);  acc = max(acc, c)
//           c is the least admissible start that the row's round imposes, relative to the
//           lane's round in row 0.  Rounds at or before t yield at most their own index, i.e.
//           nothing above t, so the dead lanes in front of the window need no mask.
//   update  per row:  Q_r += s + (tau - t)
//   Only the last row of a window is lane-masked (rounds beyond t + o), by value.
//
// The row loops are hand-written gfx950 assembly over a fixed block of physical VGPRs (v28
// upward) that only these assembly blocks touch, and the whole placement of up to 64 consecutive
// requests is ONE assembly statement (place_block): the vector unit's issue slots are what bounds
// the kernel, and the code a compiler wraps around separate check / update statements (copies for
// loop-carried values, a compare and a select to keep a completion round, recomputed masks) cost
// a third of them.  A pass over rows 0..re is entered by one computed jump (s_getpc / s_setpc,
// 64-byte slots) to a stub that handles the masked last row `re` with constant register numbers
// and then branches into a descending chain of full rows re-1..0, which runs to its end without
// a single compare or branch.  Rows are paired (five vector instructions per two rows in the
// check, three in the update).
// The compiler-generated part of the kernel and the operands of the assembly statements need
// fewer than 28 VGPRs, so the block is never allocated (the build verifies that on the emitted
// assembly of every instantiation); the clobber lists keep the block, s72, s73 and vcc out of the
// compiler's hands across the assembly statements.
#include "kvsched_internal.h"
#include "device_util.h"

#include <limits.h>

namespace {

// First register of the profile block; the KVS_CLOB_* lists start there.  The compiler's own
// registers (and the operands it hands to the assembly statements) must stay below it: the build
// checks that on the emitted assembly of every instantiation.  (The lists below are generated text:
// registers v30.., row numbers 0..NR-1 ascending and NR-1..1 descending for each file size.)
#define KVS_PB "30"

#define KVS_CLOB_9 "v30", "v31", "v32", "v33", "v34", "v35", "v36", "v37", "v38"
#define KVS_CLOB_33 KVS_CLOB_9, "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", \
    "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57", "v58", "v59", "v60", "v61", "v62"
#define KVS_CLOB_65 KVS_CLOB_33, "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71", "v72", "v73", \
    "v74", "v75", "v76", "v77", "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", "v88", \
    "v89", "v90", "v91", "v92", "v93", "v94"
#define KVS_CLOB_129 KVS_CLOB_65, "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", \
    "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", \
    "v118", "v119", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "v128", "v129", "v130", \
    "v131", "v132", "v133", "v134", "v135", "v136", "v137", "v138", "v139", "v140", "v141", "v142", "v143", \
    "v144", "v145", "v146", "v147", "v148", "v149", "v150", "v151", "v152", "v153", "v154", "v155", "v156", \
    "v157", "v158"
#define KVS_CLOB_225 KVS_CLOB_129, "v159", "v160", "v161", "v162", "v163", "v164", "v165", "v166", "v167", \
    "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", "v176", "v177", "v178", "v179", "v180", \
    "v181", "v182", "v183", "v184", "v185", "v186", "v187", "v188", "v189", "v190", "v191", "v192", "v193", \
    "v194", "v195", "v196", "v197", "v198", "v199", "v200", "v201", "v202", "v203", "v204", "v205", "v206", \
    "v207", "v208", "v209", "v210", "v211", "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", \
    "v220", "v221", "v222", "v223", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", \
    "v233", "v234", "v235", "v236", "v237", "v238", "v239", "v240", "v241", "v242", "v243", "v244", "v245", \
    "v246", "v247", "v248", "v249", "v250", "v251", "v252", "v253", "v254"

// Scalar registers of place_block: the pair it jumps through and, for the 65-row file, the row offsets 192 k.
#define KVS_SCLOB_PLAIN "s66", "s67"
#define KVS_SCLOB_65 "s66", "s67", "s68", "s69", "s70", "s71", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", \
    "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", "s88"

// Row numbers as the assembler's .irp wants them: all rows ascending (one stub each), and the
// rows that can be the last row of a window with at least one full row below, descending.
#define KVS_ASC_9 "0,1,2,3,4,5,6,7,8"
#define KVS_DESC_9 "8,7,6,5,4,3,2,1"
#define KVS_ASC_33 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32"
#define KVS_DESC_33 "32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"
#define KVS_ASC_65 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32,33,34,35,36,37,38,39,40,41,42,43,44,45,46,47,48,49,50,51,52,53,54,55,56,57,58,59,60,61,62,63,64"
#define KVS_DESC_65 "64,63,62,61,60,59,58,57,56,55,54,53,52,51,50,49,48,47,46,45,44,43,42,41,40,39,38,37,36,35,34,33,32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"
#define KVS_ASC_129 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32,33,34,35,36,37,38,39,40,41,42,43,44,45,46,47,48,49,50,51,52,53,54,55,56,57,58,59,60,61,62,63,64,65,66,67,68,69,70,71,72,73,74,75,76,77,78,79,80,81,82,83,84,85,86,87,88,89,90,91,92,93,94,95,96,97,98,99,100,101,102,103,104,105,106,107,108,109,110,111,112,113,114,115,116,117,118,119,120,121,122,123,124,125,126,127,128"
#define KVS_DESC_129 "128,127,126,125,124,123,122,121,120,119,118,117,116,115,114,113,112,111,110,109,108,107,106,105,104,103,102,101,100,99,98,97,96,95,94,93,92,91,90,89,88,87,86,85,84,83,82,81,80,79,78,77,76,75,74,73,72,71,70,69,68,67,66,65,64,63,62,61,60,59,58,57,56,55,54,53,52,51,50,49,48,47,46,45,44,43,42,41,40,39,38,37,36,35,34,33,32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"
#define KVS_ASC_225 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32,33,34,35,36,37,38,39,40,41,42,43,44,45,46,47,48,49,50,51,52,53,54,55,56,57,58,59,60,61,62,63,64,65,66,67,68,69,70,71,72,73,74,75,76,77,78,79,80,81,82,83,84,85,86,87,88,89,90,91,92,93,94,95,96,97,98,99,100,101,102,103,104,105,106,107,108,109,110,111,112,113,114,115,116,117,118,119,120,121,122,123,124,125,126,127,128,129,130,131,132,133,134,135,136,137,138,139,140,141,142,143,144,145,146,147,148,149,150,151,152,153,154,155,156,157,158,159,160,161,162,163,164,165,166,167,168,169,170,171,172,173,174,175,176,177,178,179,180,181,182,183,184,185,186,187,188,189,190,191,192,193,194,195,196,197,198,199,200,201,202,203,204,205,206,207,208,209,210,211,212,213,214,215,216,217,218,219,220,221,222,223,224"
#define KVS_DESC_225 "224,223,222,221,220,219,218,217,216,215,214,213,212,211,210,209,208,207,206,205,204,203,202,201,200,199,198,197,196,195,194,193,192,191,190,189,188,187,186,185,184,183,182,181,180,179,178,177,176,175,174,173,172,171,170,169,168,167,166,165,164,163,162,161,160,159,158,157,156,155,154,153,152,151,150,149,148,147,146,145,144,143,142,141,140,139,138,137,136,135,134,133,132,131,130,129,128,127,126,125,124,123,122,121,120,119,118,117,116,115,114,113,112,111,110,109,108,107,106,105,104,103,102,101,100,99,98,97,96,95,94,93,92,91,90,89,88,87,86,85,84,83,82,81,80,79,78,77,76,75,74,73,72,71,70,69,68,67,66,65,64,63,62,61,60,59,58,57,56,55,54,53,52,51,50,49,48,47,46,45,44,43,42,41,40,39,38,37,36,35,34,33,32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"

// Expands STMT(clobber-list, rows ascending, rows descending, place_block's scalar clobbers) for the
// instantiated file size
// (NR - 1 must be even: the row chains process rows in pairs).
#define KVS_FOR_NR(STMT)                                                                         \
    do {                                                                                         \
        static_assert(NR == 9 || NR == 33 || NR == 65 || NR == 129 || NR == 225,                 \
                      "profile file sizes: 9, 33, 65, 129 or 225 rows");                         \
        if constexpr (NR == 9) {                                                                 \
            STMT(KVS_CLOB_9, KVS_ASC_9, KVS_DESC_9, KVS_SCLOB_PLAIN);                                             \
        } else if constexpr (NR == 33) {                                                         \
            STMT(KVS_CLOB_33, KVS_ASC_33, KVS_DESC_33, KVS_SCLOB_PLAIN);                                          \
        } else if constexpr (NR == 65) {                                                         \
            STMT(KVS_CLOB_65, KVS_ASC_65, KVS_DESC_65, KVS_SCLOB_65);                                          \
        } else if constexpr (NR == 129) {                                                        \
            STMT(KVS_CLOB_129, KVS_ASC_129, KVS_DESC_129, KVS_SCLOB_PLAIN);                                       \
        } else {                                                                                 \
            STMT(KVS_CLOB_225, KVS_ASC_225, KVS_DESC_225, KVS_SCLOB_PLAIN);                                       \
        }                                                                                        \
    } while (0)

// Q_r = 64 r for all rows: nothing committed.
template <int NR>
__device__ __forceinline__ void prof_init()
{
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                        \
    asm volatile(".set kvs_r, 0\n"                             \
                 ".rept %c[nr]\n"                              \
                 "  v_mov_b32 v[" KVS_PB "+kvs_r], 64*kvs_r\n" \
                 "  .set kvs_r, kvs_r+1\n"                     \
                 ".endr\n"                                     \
                 :                                             \
                 : [nr] "n"(NR)                                \
                 : CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

// The register file to / from memory (row r of lane l at word 64 r + l): a timeline that has
// placed a common prefix of the order is saved once and resumed by every candidate.
template <int NR>
__device__ __forceinline__ void prof_store(int32_t *rows, int lane)
{
    int voff = lane * 4;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                           \
    asm volatile(".set kvs_r, 0\n"                                                \
                 ".rept %c[nr]\n"                                                 \
                 "  global_store_dword %[voff], v[" KVS_PB "+kvs_r], %[base]\n"   \
                 "  v_add_u32 %[voff], 0x100, %[voff]\n"                          \
                 "  .set kvs_r, kvs_r+1\n"                                        \
                 ".endr\n"                                                        \
                 "s_waitcnt vmcnt(0)\n"                                           \
                 : [voff] "+v"(voff)                                              \
                 : [base] "s"(rows), [nr] "n"(NR)                                 \
                 : "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

template <int NR>
__device__ __forceinline__ void prof_load(const int32_t *rows, int lane)
{
    int voff = lane * 4;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                           \
    asm volatile(".set kvs_r, 0\n"                                                \
                 ".rept %c[nr]\n"                                                 \
                 "  global_load_dword v[" KVS_PB "+kvs_r], %[voff], %[base]\n"    \
                 "  v_add_u32 %[voff], 0x100, %[voff]\n"                          \
                 "  .set kvs_r, kvs_r+1\n"                                        \
                 ".endr\n"                                                        \
                 "s_waitcnt vmcnt(0)\n"                                           \
                 : [voff] "+v"(voff)                                              \
                 : [base] "s"(rows), [nr] "n"(NR)                                 \
                 : "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

// ---------------------------------------------------------------------------------------------
// Placing up to 64 consecutive requests of the order: ONE assembly statement.
//
// Lane j of vns / vo holds M - s and o of a request; the requests are taken from lane cnt - 1 down to
// lane 0 (the lane number is kept in M0 for v_readlane / v_writelane, and the loop ends when it
// borrows).  Round tau imposes the start bound min(P(tau) + s - M + tau, tau) on the
// request (from round tau on it no longer overlaps tau); with Q_r = P + 64 r that is, relative to the
// lane's round in row 0, min(Q_r + (s - M), 64 r).  For each request in turn:
//   blocked? rows 0..re of the profile (re = row of the window's last round t + o; the last row is
//            masked by value beyond that round: the lanes of mk).  A limit 64 r, r >= 1, exceeds
//            every admissible (t - b64) - lane, so whether the request is blocked does not depend
//            on those limits: acc = max(max over rows >= 1 of Q_r, min(Q_0, M - s)) - (M - s),
//            one v_max3 per two rows, and the request is blocked iff acc > (t - b64) - lane in some
//            lane.  Most requests are not, and are admitted after this pass alone;
//   bounds   if acc <= 64 in every lane no limit of a row >= 1 was reached and acc already holds
//            the exact bounds; otherwise a second pass takes the rows with their limits
//            (acc = max over rows of min(Q_r + (s - M), 64 r), five instructions per two rows);
//   move on  t becomes the largest bound (six DPP steps), the register file moves down so that row 0
//            holds round t + 1 again, and only the rounds that have entered the window since are
//            looked at: nearly always the window's last row alone (one computed jump to a stub of
//            that row), otherwise rows rs..re one by one (a computed jump per row: the row number is
//            not known at compile time and VGPR index mode is avoided); blocked again: repeat;
//   admit    rows 0..re get the ramp s + (tau - t) (by value zero beyond the window); the start
//            round t goes to the request's lane of cv.
// A pass over rows 0..re is entered by one computed jump (table base + 64 (re + 1), s_setpc) to a
// 64-byte stub that handles the masked last row with constant register numbers and branches into a
// descending chain of full rows re-1..0, which runs to its end without a compare or a branch.
//
// Both the vector unit (one instruction per cycle and compute unit) and the scalar unit (the same,
// shared by the four SIMDs) are close to saturated by this loop, so it is written to need few of
// either: the window mask is one scalar shift, the table addresses are computed once per block,
// EXEC is never touched.
//
// Wait states (gfx950 does not interlock these; the distances below are by construction):
//   a VALU instruction that reads an SGPR or VCC written by a VALU instruction (v_readlane, v_cmp)
//   needs two instructions in between: M - s is read by vector instructions only behind a computed
//   jump (at least five scalar instructions later); oj, vcc and the DPP result are read by scalar
//   instructions, which need none;
//   DPP reads of a VGPR written by the previous VALU instruction, and v_readlane of one: s_nop 1.
// The kernel has no other use of M0 (no LDS, no relative addressing).

// Maximum over the 64 lanes of %[y] into lane 63 (four DPP steps inside the 16-lane rows, two row
// broadcasts), read into %[tc].
#define KVS_WAVE_MAX                                                                            \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"           \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n"           \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] row_half_mirror row_mask:0xf bank_mask:0xf\n"               \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] row_mirror row_mask:0xf bank_mask:0xf\n"                    \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] row_bcast:15 row_mask:0xa bank_mask:0xf\n"                  \
    "s_nop 1\n"                                                                                 \
    "v_max_i32_dpp %[y], %[y], %[y] row_bcast:31 row_mask:0xc bank_mask:0xf\n"                  \
    "s_nop 1\n"                                                                                 \
    "v_readlane_b32 %[tc], %[y], 63\n"

// Pads the slot that began at the last label 7 to the given number of bytes (never executed: slots
// end in a branch).
#define KVS_SLOT_PAD(bytes) "  .fill (" #bytes "-(.-7b))/4, 4, 0xbf800000\n"

template <int NR>
__device__ __forceinline__ int place_block(int cnt, int vns, int vo, int lane, int vmin, int M, int &t, int &b64)
{
    int cv, acc, y, z, tl, vw;
    int ns, oj, x64, off, u64, w, rs, ta, tb, tc, ql, qh, cl, ch, ul, uh, rl, rh;
    long long mk;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                                       \
    asm volatile(                                                                                       \
        /* table addresses: slot of row r at base + 64 (r + 1) for the stubs of a whole pass, */       \
        /* whole passes and single rows alike */                                                    \
        "s_getpc_b64 s[66:67]\n"                                                                        \
        "60:\n"                                                                                         \
        "s_add_u32 %[ql], s66, 64f-60b-64\n"                                                            \
        "s_addc_u32 %[qh], s67, 0\n"                                                                    \
        "s_add_u32 %[cl], s66, 61f-60b-64\n"                                                            \
        "s_addc_u32 %[ch], s67, 0\n"                                                                    \
        "s_add_u32 %[ul], s66, 62f-60b-64\n"                                                            \
        "s_addc_u32 %[uh], s67, 0\n"                                                                    \
        "s_add_u32 %[rl], s66, 63f-60b-64\n"                                                            \
        "s_addc_u32 %[rh], s67, 0\n"                                                                    \
        "s_sub_u32 %[u64], %[t], %[b64]\n"                                                              \
        "v_sub_u32 %[tl], %[u64], %[lane]\n" /* (t - b64) - lane */                                     \
        "s_add_u32 %[u64], %[u64], 64\n"     /* x64 of a request is its decode length plus this */      \
        /* The 65-row file (long decodes, few wavefronts per SIMD) updates a row in one instruction: the */ \
        /* ramp of row r is that of row r mod 3 (three vectors) plus 192 floor(r / 3) from a scalar */    \
        /* register (s[67 + k] = 192 k); vw = M - (t - b64) + lane there, the ramp of row 0 is vw - (M - s). */ \
        /* The other files take rows in pairs from the ramp of the window's last row, */                  \
        /* vw + 64 (re + 1) - (M - s) with vw = M - 64 - (t - b64) + lane. */                             \
        ".if %c[nr] == 65\n"                                                                            \
        "  .set kvs_r, 1\n"                                                                             \
        "  .rept 21\n"                                                                                  \
        "    s_movk_i32 s[67+kvs_r], 192*kvs_r\n"                                                       \
        "    .set kvs_r, kvs_r+1\n"                                                                     \
        "  .endr\n"                                                                                     \
        "  s_mov_b32 %[w], %[M]\n"                                                                      \
        ".else\n"                                                                                       \
        "  s_sub_u32 %[w], %[M], 64\n"                                                                  \
        ".endif\n"                                                                                      \
        "v_sub_u32 %[vw], %[w], %[tl]\n"    /* ramp in lane l of the window's last row: vw + (s - M) + 64 (re + 1) */ \
        "v_mov_b32 %[cv], 0\n"                                                                          \
        "s_sub_u32 m0, %[cnt], 1\n"                                                                     \
        /* ---- next request (lane m0, counting down): is it blocked at all? */                         \
        "40:\n"                                                                                         \
        "v_readlane_b32 %[ns], %[vns], m0\n"                                                            \
        "v_readlane_b32 %[oj], %[vo], m0\n"                                                             \
        "s_add_u32 %[x64], %[oj], %[u64]\n" /* (t + o - b64) + 64: row and lane of the window's last round */ \
        "s_lshl_b64 %[mk], -2, %[x64]\n"    /* the lanes behind it (the shift uses x64 mod 64) */       \
        "s_andn2_b32 %[off], %[x64], 63\n"  /* 64 (re + 1) */                                           \
        "s_add_u32 s66, %[ql], %[off]\n"                                                                \
        "s_addc_u32 s67, %[qh], 0\n"                                                                    \
        "s_setpc_b64 s[66:67]\n"                                                                        \
        "64:\n"                                                                                         \
        ".irp r," ASC "\n"                                                                              \
        "7:\n"                                                                                          \
        "  .if \\r == 0\n"                                                                              \
        "    v_min_i32 %[y], %[ns], v[" KVS_PB "]\n"                                                    \
        "    v_cndmask_b32_e64 %[acc], %[y], %[vmin], %[mk]\n"                                          \
        "    s_branch 26f\n"                                                                            \
        "  .else\n"                                                                                     \
        "    v_cndmask_b32_e64 %[acc], v[" KVS_PB "+\\r], %[vmin], %[mk]\n"                             \
        "    .if \\r == 1\n"                                                                            \
        "      v_min_i32 %[y], %[ns], v[" KVS_PB "]\n"                                                  \
        "      v_max_i32 %[acc], %[acc], %[y]\n"                                                        \
        "      s_branch 26f\n"                                                                          \
        "    .else\n"                                                                                   \
        "      .if (\\r & 1) == 1\n"                                                                    \
        "        v_max_i32 %[acc], %[acc], v[" KVS_PB "+\\r-1]\n"                                       \
        "      .endif\n"                                                                                \
        "      s_branch 25\\r\\()f\n"                                                                   \
        "    .endif\n"                                                                                  \
        "  .endif\n" KVS_SLOT_PAD(64)                                                                   \
        ".endr\n"                                                                                       \
        /* entry 25r: the rows below those of stub r, two per instruction; y stands for row 0 */       \
        ".irp r," DESC "\n"                                                                             \
        "25\\r:\n"                                                                                      \
        "  .if (\\r & 1) == 0\n"                                                                        \
        "    .if \\r == 2\n"                                                                            \
        "      v_min_i32 %[y], %[ns], v[" KVS_PB "]\n"                                                  \
        "      v_max3_i32 %[acc], %[acc], v[" KVS_PB "+1], %[y]\n"                                      \
        "    .else\n"                                                                                   \
        "      v_max3_i32 %[acc], %[acc], v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-2]\n"                   \
        "    .endif\n"                                                                                  \
        "  .endif\n"                                                                                    \
        ".endr\n"                                                                                       \
        "26:\n"                                                                                         \
        "v_subrev_u32 %[acc], %[ns], %[acc]\n"                                                          \
        "41:\n"                                                                                         \
        "v_cmp_gt_i32 vcc, %[acc], %[tl]\n"                                                             \
        "s_cbranch_vccnz 52f\n"                                                                         \
        /* ---- admit at round t */                                                                     \
        "42:\n"                                                                                         \
        ".if %c[nr] != 65\n"                                                                            \
        "  s_sub_u32 %[rs], %[off], %[ns]\n"                                                            \
        ".endif\n"                                                                                      \
        "s_add_u32 s66, %[ul], %[off]\n"                                                                \
        "s_addc_u32 s67, %[uh], 0\n"                                                                    \
        "s_setpc_b64 s[66:67]\n"                                                                        \
        "62:\n"                                                                                         \
        ".irp r," ASC "\n"                                                                              \
        "7:\n"                                                                                          \
        "  .if %c[nr] == 65\n"                                                                          \
        /*   z, acc, y (once the masked row is done): the ramps of rows 0, 1, 2 */                      \
        "    v_subrev_u32 %[z], %[ns], %[vw]\n"                                                         \
        "    .if \\r == 0\n"                                                                            \
        "      v_cndmask_b32_e64 %[y], %[z], 0, %[mk]\n"                                                \
        "      v_add_u32 v[" KVS_PB "], %[y], v[" KVS_PB "]\n"                                          \
        "      s_branch 43f\n"                                                                          \
        "    .else\n"                                                                                   \
        "      v_add_u32 %[y], 64*\\r, %[z]\n"                                                          \
        "      v_cndmask_b32_e64 %[y], %[y], 0, %[mk]\n"                                                \
        "      v_add_u32 v[" KVS_PB "+\\r], %[y], v[" KVS_PB "+\\r]\n"                                  \
        "      .if \\r >= 2\n"                                                                          \
        "        v_add_u32 %[acc], 64, %[z]\n"                                                          \
        "      .endif\n"                                                                                \
        "      .if \\r >= 3\n"                                                                          \
        "        v_add_u32 %[y], 0x80, %[z]\n"                                                          \
        "      .endif\n"                                                                                \
        "      s_branch 30\\r\\()f\n"                                                                   \
        "    .endif\n"                                                                                  \
        "  .else\n"                                                                                     \
        "    v_add_u32 %[y], %[rs], %[vw]\n"                                                            \
        "    .if \\r == 0\n"                                                                            \
        "      v_cndmask_b32_e64 %[y], %[y], 0, %[mk]\n"                                                \
        "      v_add_u32 v[" KVS_PB "], %[y], v[" KVS_PB "]\n"                                          \
        "      s_branch 43f\n"                                                                          \
        "    .else\n"                                                                                   \
        /*     z: ramp of the even row of the pair that holds row r - 1 */                              \
        "      .if (\\r & 1) == 1\n"                                                                    \
        "        v_subrev_u32 %[z], 64, %[y]\n"                                                         \
        "      .else\n"                                                                                 \
        "        v_add_u32 %[z], 0xffffff80, %[y]\n"                                                    \
        "      .endif\n"                                                                                \
        "      v_cndmask_b32_e64 %[y], %[y], 0, %[mk]\n"                                                \
        "      v_add_u32 v[" KVS_PB "+\\r], %[y], v[" KVS_PB "+\\r]\n"                                  \
        "      s_branch 30\\r\\()f\n"                                                                   \
        "    .endif\n"                                                                                  \
        "  .endif\n" KVS_SLOT_PAD(64)                                                                   \
        ".endr\n"                                                                                       \
        ".irp r," DESC "\n"                                                                             \
        "30\\r:\n"                                                                                      \
        "  .if %c[nr] == 65\n"                                                                          \
        "    .if (\\r-1) == 0\n"                                                                        \
        "      v_add_u32 v[" KVS_PB "], %[z], v[" KVS_PB "]\n"                                          \
        "    .elseif (\\r-1) == 1\n"                                                                    \
        "      v_add_u32 v[" KVS_PB "+1], %[acc], v[" KVS_PB "+1]\n"                                    \
        "    .elseif (\\r-1) == 2\n"                                                                    \
        "      v_add_u32 v[" KVS_PB "+2], %[y], v[" KVS_PB "+2]\n"                                      \
        "    .elseif ((\\r-1) - 3*((\\r-1)/3)) == 0\n"                                                  \
        "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[z], s[67+(\\r-1)/3]\n"            \
        "    .elseif ((\\r-1) - 3*((\\r-1)/3)) == 1\n"                                                  \
        "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[acc], s[67+(\\r-1)/3]\n"          \
        "    .else\n"                                                                                   \
        "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[y], s[67+(\\r-1)/3]\n"            \
        "    .endif\n"                                                                                  \
        "  .else\n"                                                                                     \
        "    .if ((\\r-1) & 1) == 1\n"                                                                  \
        "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[z], 64\n"                         \
        "    .else\n"                                                                                   \
        "      v_add_u32 v[" KVS_PB "+\\r-1], %[z], v[" KVS_PB "+\\r-1]\n"                              \
        "      .if (\\r-1) >= 2\n"                                                                      \
        "        v_add_u32 %[z], 0xffffff80, %[z]\n"                                                    \
        "      .endif\n"                                                                                \
        "    .endif\n"                                                                                  \
        "  .endif\n"                                                                                    \
        ".endr\n"                                                                                       \
        "43:\n"                                                                                         \
        "v_writelane_b32 %[cv], %[t], m0\n"  /* the start round; the caller adds the lane's decode length */ \
        "s_sub_u32 m0, m0, 1\n"             /* borrows behind lane 0 */                                 \
        "s_cbranch_scc0 40b\n"                                                                          \
        "s_branch 50f\n"                                                                                \
        /* ---- blocked.  The bounds found are exact unless one exceeds 64 in some lane (only then */   \
        /* can a row's limit 64 r, r >= 1, have mattered): then the pass with the limits */             \
        "52:\n"                                                                                         \
        "v_cmp_lt_i32 vcc, 64, %[acc]\n"                                                                \
        "s_cbranch_vccz 44f\n"                                                                          \
        "s_add_u32 s66, %[cl], %[off]\n"                                                                \
        "s_addc_u32 s67, %[ch], 0\n"                                                                    \
        "s_setpc_b64 s[66:67]\n"                                                                        \
        "61:\n"                                                                                         \
        ".irp r," ASC "\n"                                                                              \
        "7:\n"                                                                                          \
        "  v_subrev_u32 %[y], %[ns], v[" KVS_PB "+\\r]\n"                                                  \
        "  v_min_i32 %[y], 64*\\r, %[y]\n"                                                              \
        "  v_cndmask_b32_e64 %[acc], %[y], %[vmin], %[mk]\n"                                            \
        "  .if \\r == 0\n"                                                                              \
        "    s_branch 44f\n"                                                                            \
        "  .else\n"                                                                                     \
        "    .if (\\r & 1) == 1\n"                                                                      \
        "      v_mov_b32 %[z], %[acc]\n"                                                                \
        "    .endif\n"                                                                                  \
        "    s_branch 20\\r\\()f\n"                                                                     \
        "  .endif\n" KVS_SLOT_PAD(64)                                                                   \
        ".endr\n"                                                                                       \
        ".irp r," DESC "\n"                                                                             \
        "20\\r:\n"                                                                                      \
        "  .if ((\\r-1) & 1) == 1\n"                                                                    \
        "    v_subrev_u32 %[z], %[ns], v[" KVS_PB "+\\r-1]\n"                                              \
        "    v_min_i32 %[z], 64*(\\r-1), %[z]\n"                                                        \
        "  .else\n"                                                                                     \
        "    v_subrev_u32 %[y], %[ns], v[" KVS_PB "+\\r-1]\n"                                              \
        "    v_min_i32 %[y], 64*(\\r-1), %[y]\n"                                                        \
        "    v_max3_i32 %[acc], %[acc], %[y], %[z]\n"                                                   \
        "  .endif\n"                                                                                    \
        ".endr\n"                                                                                       \
        /* ---- move t to the largest bound, the register file with it, look at what is new */          \
        "44:\n"                                                                                         \
        "v_add_u32 %[y], %[acc], %[lane]\n"                                                             \
        KVS_WAVE_MAX                                                                                    \
        "s_add_u32 %[t], %[tc], %[b64]\n"                                                               \
        "s_add_u32 %[ta], %[tc], 1\n"                                                                   \
        "s_andn2_b32 %[rs], %[ta], 63\n"     /* row 0 starts at 64 floor((t + 1) / 64): 64 x rows to move down */ \
        "s_add_u32 %[b64], %[b64], %[rs]\n"                                                             \
        "s_sub_u32 %[tb], %[x64], %[rs]\n"   /* the last round looked at, as x64 counts in the moved file */ \
        "s_sub_u32 %[u64], %[tc], %[rs]\n"                                                              \
        "v_sub_u32 %[tl], %[u64], %[lane]\n"                                                            \
        "s_add_u32 %[u64], %[u64], 64\n"                                                                \
        "v_sub_u32 %[vw], %[w], %[tl]\n"                                                                \
        "s_add_u32 %[x64], %[oj], %[u64]\n"                                                             \
        "s_lshl_b64 %[mk], -2, %[x64]\n"                                                                \
        "s_andn2_b32 %[off], %[x64], 63\n"                                                              \
        "s_lshr_b32 %[rs], %[rs], 6\n"       /* rows to move down; SCC: any */                          \
        "s_cbranch_scc0 46f\n"                                                                          \
        "s_cmp_ge_u32 %[rs], %c[nr]\n"                                                                  \
        "s_cbranch_scc1 47f\n"                                                                          \
        "45:\n"                                                                                         \
        ".set kvs_r, 0\n"                                                                               \
        ".rept %c[nr]-1\n"                                                                              \
        "  v_subrev_u32 v[" KVS_PB "+kvs_r], 64, v[" KVS_PB "+kvs_r+1]\n"                               \
        "  .set kvs_r, kvs_r+1\n"                                                                       \
        ".endr\n"                                                                                       \
        "v_mov_b32 v[" KVS_PB "+%c[nr]-1], 64*(%c[nr]-1)\n"                                             \
        "s_sub_u32 %[rs], %[rs], 1\n"                                                                   \
        "s_cmp_lg_u32 %[rs], 0\n"                                                                       \
        "s_cbranch_scc1 45b\n"                                                                          \
        "s_branch 46f\n"                                                                                \
        "47:\n"                                                                                         \
        ".set kvs_r, 0\n"                                                                               \
        ".rept %c[nr]\n"                                                                                \
        "  v_mov_b32 v[" KVS_PB "+kvs_r], 64*kvs_r\n"                                                   \
        "  .set kvs_r, kvs_r+1\n"                                                                       \
        ".endr\n"                                                                                       \
        "46:\n"                                                                                         \
        "s_cmp_ge_u32 %[tb], %[off]\n"       /* are all rounds not looked at yet in the window's last row? */ \
        "s_cbranch_scc0 48f\n"                                                                          \
        "s_add_u32 s66, %[rl], %[off]\n"                                                                \
        "s_addc_u32 s67, %[rh], 0\n"                                                                    \
        "s_setpc_b64 s[66:67]\n"                                                                        \
        "63:\n"                                                                                         \
        ".irp r," ASC "\n"                                                                              \
        "7:\n"                                                                                          \
        "  v_subrev_u32 %[y], %[ns], v[" KVS_PB "+\\r]\n"                                               \
        "  v_min_i32 %[y], 64*\\r, %[y]\n"                                                              \
        "  v_cndmask_b32_e64 %[acc], %[y], %[vmin], %[mk]\n"                                            \
        "  v_cmp_gt_i32 vcc, %[acc], %[tl]\n"                                                           \
        "  s_cbranch_vccz 42b\n"                                                                        \
        "  s_branch 44b\n" KVS_SLOT_PAD(64)                                                             \
        ".endr\n"                                                                                       \
        /* rows tb..tc, the last of them masked */                                                      \
        "48:\n"                                                                                         \
        "s_add_u32 %[tb], %[tb], 1\n"                                                                   \
        "s_lshr_b32 %[tb], %[tb], 6\n"                                                                  \
        "s_sub_u32 %[tb], %[tb], 1\n"                                                                   \
        "s_lshr_b32 %[tc], %[x64], 6\n"                                                                 \
        "s_sub_u32 %[tc], %[tc], 1\n"                                                                   \
        "v_mov_b32 %[acc], %[vmin]\n"                                                                   \
        "51:\n"                                                                                         \
        "s_cmp_eq_u32 %[tb], %[tc]\n"                                                                   \
        "s_cselect_b64 vcc, %[mk], 0\n"                                                                \
        "s_add_u32 %[ta], %[tb], 1\n"                                                                   \
        "s_lshl_b32 %[ta], %[ta], 4\n"       /* 16-byte slots, the first 16 bytes behind s_getpc's successor */ \
        "s_getpc_b64 s[66:67]\n"                                                                        \
        "s_add_u32 s66, s66, %[ta]\n"                                                                   \
        "s_addc_u32 s67, s67, 0\n"                                                                      \
        "s_setpc_b64 s[66:67]\n"                                                                        \
        ".fill 1, 4, 0xbf800000\n"                                                                      \
        ".irp r," ASC "\n"                                                                              \
        "7:\n"                                                                                          \
        "  v_subrev_u32 %[y], %[ns], v[" KVS_PB "+\\r]\n"                                                  \
        "  v_min_i32 %[y], 64*\\r, %[y]\n"                                                              \
        "  s_branch 49f\n" KVS_SLOT_PAD(16)                                                             \
        ".endr\n"                                                                                       \
        "49:\n"                                                                                         \
        "v_cndmask_b32_e32 %[y], %[y], %[vmin], vcc\n"                                                 \
        "v_max_i32 %[acc], %[acc], %[y]\n"                                                              \
        "s_add_u32 %[tb], %[tb], 1\n"                                                                   \
        "s_cmp_le_u32 %[tb], %[tc]\n"                                                                   \
        "s_cbranch_scc1 51b\n"                                                                          \
        /* ---- the new rounds' bounds (exact): admitted now, or blocked once more */                   \
        "53:\n"                                                                                         \
        "v_cmp_gt_i32 vcc, %[acc], %[tl]\n"                                                             \
        "s_cbranch_vccz 42b\n"                                                                          \
        "s_branch 44b\n"                                                                                \
        "50:\n"                                                                                         \
        : [cv] "=&v"(cv), [acc] "=&v"(acc), [y] "=&v"(y), [z] "=&v"(z), [tl] "=&v"(tl), [vw] "=&v"(vw), \
          [ns] "=&s"(ns), [oj] "=&s"(oj), [x64] "=&s"(x64), [off] "=&s"(off), [u64] "=&s"(u64),         \
          [w] "=&s"(w), [rs] "=&s"(rs), [ta] "=&s"(ta), [tb] "=&s"(tb), [tc] "=&s"(tc), [ql] "=&s"(ql), \
          [qh] "=&s"(qh), [cl] "=&s"(cl), [ch] "=&s"(ch), [ul] "=&s"(ul), [uh] "=&s"(uh), [rl] "=&s"(rl), \
          [rh] "=&s"(rh), [mk] "=&s"(mk), [t] "+s"(t), [b64] "+s"(b64)                  \
        : [cnt] "s"(cnt), [vns] "v"(vns), [vo] "v"(vo), [lane] "v"(lane), [vmin] "v"(vmin),             \
          [M] "s"(M), [nr] "n"(NR)                                                                      \
        : "scc", "vcc", SCLOB, CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return cv;
}

// One int32 read through the scalar unit (the address is the same for the whole wavefront).
__device__ __forceinline__ int scalar_read(const int32_t *base, int index)
{
    int v;
    asm volatile("s_load_dword %[v], %[base], %[off]\n"
                 "s_waitcnt lgkmcnt(0)\n"
                 : [v] "=s"(v)
                 : [base] "s"(base), [off] "s"(index * 4)
                 : "memory");
    return v;
}

// Head of a saved timeline state: words 0, 1 = b64, t (every lane stores the same two values), then
// the lanes' partial sums of completion rounds as 64 int64 at byte 256.  The profile rows follow
// at byte 768 (prof_store).  Written in assembly so that no temporary can land in the profile block.
template <int NR>
__device__ __forceinline__ void state_head_store(int32_t *snap, int b64, int t, long long tel_lane, int lane)
{
    int a, b, off;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                                        \
    asm volatile("v_mov_b32 %[a], %[b64]\n"                                                              \
                 "v_mov_b32 %[b], %[t]\n"                                                                \
                 "v_mov_b32 %[off], 0\n"                                                                 \
                 "global_store_dword %[off], %[a], %[base]\n"                                            \
                 "global_store_dword %[off], %[b], %[base] offset:4\n"                                   \
                 "v_lshlrev_b32 %[off], 3, %[lane]\n"                                                    \
                 "global_store_dwordx2 %[off], %[tel], %[base] offset:256\n"                             \
                 "s_waitcnt vmcnt(0)\n"                                                                  \
                 : [a] "=&v"(a), [b] "=&v"(b), [off] "=&v"(off)                                          \
                 : [base] "s"(snap), [b64] "s"(b64), [t] "s"(t), [tel] "v"(tel_lane), [lane] "v"(lane)   \
                 : "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

// Snapshots handed over inside one launch.  The wave that writes a snapshot and the waves that read
// it run on different compute units, in general under different L2 caches, so the hand-over follows
// the device-scope release / acquire sequences of the hardware's memory model, written out here
// because the snapshot itself is stored and loaded by assembly the compiler does not see into:
//   writer: all stores done -> write back the L2 -> done -> store the progress word at device scope;
//   reader: load the progress word at device scope -> invalidate stale cache lines -> load the snapshot.
// The progress word (zero at launch) holds the number j of snapshots published so far (they are taken
// in order), or ~j once the writer has stopped after j of them (a request that cannot be scheduled).
// It is kept in KVS_PROGRESS_COPIES copies, 64 bytes apart, written by one store of the writer's 64
// lanes; a reader polls the copy of its wave number: thousands of readers polling one address slow
// the writer down measurably.
// A reader that needs snapshot b polls the word about every 3 us until it is >= b; it gives up when
// the word says the writer has stopped, or has not moved for SimParams::snap_wait_polls polls (by
// default some 14 ms), and then starts from the latest snapshot there is, or from the beginning.
// The writer waits for nobody, so the word stops moving at the latest when the writer's wave ends,
// and every wait ends.

template <int NR>
__device__ __forceinline__ void snapshot_progress_set(int32_t *progress, int value, int lane)  // device-scope store
{
    static_assert(KVS_PROGRESS_COPIES == 64 && KVS_PROGRESS_STRIDE_WORDS == 16, "one copy per lane, 64 bytes apart");
    int off, v;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                       \
    asm volatile("v_lshlrev_b32 %[off], 6, %[lane]\n"                                   \
                 "v_mov_b32 %[v], %[val]\n"                                             \
                 "global_store_dword %[off], %[v], %[base] sc1\n"                       \
                 : [off] "=&v"(off), [v] "=&v"(v)                                       \
                 : [base] "s"(progress), [val] "s"(value), [lane] "v"(lane)             \
                 : "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

template <int NR>
__device__ __forceinline__ void snapshot_publish(int32_t *progress, int count, int lane)
{
    asm volatile("s_waitcnt vmcnt(0)\n"
                 "buffer_wbl2 sc1\n"
                 "s_waitcnt vmcnt(0)\n" ::: "memory");
    snapshot_progress_set<NR>(progress, count, lane);
}

// The reader's side as one scalar loop; returns the snapshot to start from (0: none).  rb = 0
// (nothing to wait for) passes through.  Written as a single block so that the compiler sees one
// scalar result, as from a scalar load.
template <int NR>
__device__ __forceinline__ int snapshot_wait(const int32_t *progress, int rb, int polls, int copy)
{
    int f, cnt, last, voff, v;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                                                 \
    asm volatile("s_cmp_eq_u32 %[rb], 0\n"                                                                        \
                 "s_cbranch_scc1 4f\n"                                                                            \
                 "s_max_i32 %[cnt], %[polls], 1\n"                                                                \
                 "s_mov_b32 %[last], -1\n"                                                                        \
                 "s_lshl_b32 %[f], %[copy], 6\n"                                                                  \
                 "v_mov_b32 %[voff], %[f]\n"                                                                      \
                 "1:\n"                                                                                           \
                 "global_load_dword %[v], %[voff], %[base] sc1\n"                                                 \
                 "s_waitcnt vmcnt(0)\n"                                                                           \
                 "v_readfirstlane_b32 %[f], %[v]\n"                                                               \
                 "s_cmp_lt_i32 %[f], 0\n"                                                                         \
                 "s_cbranch_scc1 3f\n" /* the writer has stopped */                                               \
                 "s_cmp_ge_i32 %[f], %[rb]\n"                                                                     \
                 "s_cbranch_scc1 4f\n" /* it is there */                                                          \
                 "s_cmp_eq_u32 %[f], %[last]\n"                                                                   \
                 "s_cbranch_scc1 2f\n"                                                                            \
                 "s_mov_b32 %[last], %[f]\n" /* the writer has moved: count anew */                               \
                 "s_max_i32 %[cnt], %[polls], 1\n"                                                                \
                 "s_branch 5f\n"                                                                                  \
                 "2:\n"                                                                                           \
                 "s_sub_u32 %[cnt], %[cnt], 1\n"                                                                  \
                 "s_cmp_eq_u32 %[cnt], 0\n"                                                                       \
                 "s_cbranch_scc0 5f\n"                                                                            \
                 "s_mov_b32 %[rb], %[f]\n" /* waited long enough: what there is (f < rb) */                       \
                 "s_branch 4f\n"                                                                                  \
                 "5:\n"                                                                                           \
                 "s_sleep 127\n"                                                                                  \
                 "s_branch 1b\n"                                                                                  \
                 "3:\n"                                                                                           \
                 "s_not_b32 %[f], %[f]\n" /* snapshots published before it stopped */                             \
                 "s_min_i32 %[rb], %[rb], %[f]\n"                                                                 \
                 "4:\n"                                                                                           \
                 "buffer_inv sc1\n"                                                                               \
                 : [rb] "+s"(rb), [f] "=&s"(f), [cnt] "=&s"(cnt), [last] "=&s"(last), [voff] "=&v"(voff),         \
                   [v] "=&v"(v)                                                                                   \
                 : [base] "s"(progress), [polls] "s"(polls), [copy] "s"(copy)                                     \
                 : "scc", "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return rb;
}

// The number of snapshots published so far, read once without waiting (the reader's side of the same
// hand-over: what the writer stored before publishing them may be loaded afterwards).
template <int NR>
__device__ __forceinline__ int progress_peek(const int32_t *progress, int copy)
{
    int f, voff, v;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                                                                                 \
    asm volatile("s_lshl_b32 %[f], %[copy], 6\n"                                                                  \
                 "v_mov_b32 %[voff], %[f]\n"                                                                      \
                 "global_load_dword %[v], %[voff], %[base] sc1\n"                                                 \
                 "s_waitcnt vmcnt(0)\n"                                                                           \
                 "v_readfirstlane_b32 %[f], %[v]\n"                                                               \
                 "s_cmp_lt_i32 %[f], 0\n"                                                                         \
                 "s_cbranch_scc0 1f\n"                                                                            \
                 "s_not_b32 %[f], %[f]\n" /* the writer has stopped: what it published before */                  \
                 "1:\n"                                                                                           \
                 "buffer_inv sc1\n"                                                                               \
                 : [f] "=&s"(f), [voff] "=&v"(voff), [v] "=&v"(v)                                                 \
                 : [base] "s"(progress), [copy] "s"(copy)                                                         \
                 : "scc", "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return f;
}

// One int32 of a snapshot's head through the vector unit (the scalar cache takes no part in the
// hand-over above).
template <int NR>
__device__ __forceinline__ int snapshot_word(const int32_t *snap, int index)
{
    int off, v;
#define KVS_STMT(CLOB, ASC, DESC, SCLOB)                              \
    asm volatile("v_mov_b32 %[off], %[idx]\n"                  \
                 "global_load_dword %[v], %[off], %[base]\n"   \
                 "s_waitcnt vmcnt(0)\n"                        \
                 : [off] "=&v"(off), [v] "=&v"(v)              \
                 : [base] "s"(snap), [idx] "s"(index * 4)      \
                 : "memory", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return __builtin_amdgcn_readfirstlane(v);
}

// RES: the launch runs the candidates named by p.cand_list; the wave of candidate 0 saves its
// state every 64 positions, candidates with a resume block start from such a snapshot.
// ONE (with RES): both in the same launch, handed over through p.snap_flags.
template <int NR, int WPB, bool MOVES, bool RES, bool ONE>
__global__ __launch_bounds__(WAVE *WPB) void timeline_reg_kernel(SimParams p)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave_no = __builtin_amdgcn_readfirstlane(blockIdx.x * WPB + (threadIdx.x >> 6));
    if (wave_no >= p.C) return;
    const int cand = RES ? scalar_read(p.cand_list, wave_no) : wave_no;
    if (p.skip && scalar_read(p.skip, cand) != INT_MAX) {  // known to be another candidate's timeline
        if (threadIdx.x % WAVE == 0 && p.tel_out) p.tel_out[cand] = 0;  // (relative to that one's, as for a row that stops early)
        return;
    }

    const int n_all = p.n;
    const int M = p.M;
    OrderReader<MOVES> rd;
    if (MOVES) {
        rd.row = p.src.base;
        rd.mt = KVSCHED_MOVE_SWAP;
        rd.mi = rd.mj = 0;
        if (cand < p.C - 1) {  // the last timeline is the base order itself
            rd.mt = p.src.moves[3 * (size_t)cand];
            rd.mi = min(max(p.src.moves[3 * (size_t)cand + 1], 0), n_all - 1);
            rd.mj = min(max(p.src.moves[3 * (size_t)cand + 2], 0), n_all - 1);
        }
    } else {
        rd.row = p.src.orders + (size_t)cand * (size_t)n_all;
        rd.mt = rd.mi = rd.mj = 0;
    }
    // the stretch of positions a move changes (through the scalar unit, like everything the rows' control flow uses)
    const int move_lo = MOVES ? __builtin_amdgcn_readfirstlane(min(rd.mi, rd.mj)) : 0;
    const int move_hi = MOVES ? __builtin_amdgcn_readfirstlane(max(rd.mi, rd.mj)) : 0;
    int32_t *crow = p.completion_out ? p.completion_out + (size_t)cand * (size_t)n_all : nullptr;

    // positions [k_first, n) of the order are placed; the state after the first k_first ones
    // (a prefix shared by all candidates) comes from memory when there is one
    int k_first = p.k_begin;
    const int32_t *state_in = p.state_in;
    if (p.resume_ok && scalar_read(p.resume_ok, 0) == 0) {  // what the state was computed from has changed since
        k_first = 0;
        state_in = nullptr;
    }
    const int n = p.k_end > 0 ? p.k_end : n_all;  // one past the last position placed here
    // Rejoining row 0.  A row that differs from row 0 only at positions i..j holds the same requests
    // there in another order.  If row 0 starts the requests of positions i - 1 .. j in one and the same
    // round (start rounds never decrease along the order, so the two ends tell; for i = 0: in round 0),
    // then so does this row: none of them can start before the request at position i - 1, and each fits
    // that round beside any part of the others, since all of them do.  From position j + 1 on the two
    // timelines are the same, and this row need not place what row 0 places anyway: it stops at the
    // 64-position boundary behind j (or does not start at all, when row 0 is already past it), reports
    // the boundary, and leaves its sum of completion rounds relative to row 0's; a later pass adds row
    // 0's sum and takes the completion rounds from there on from row 0.
    // (Among moves the stretch is the move's own, and row 0 stands for the base order.)
    int rejoin_k = -1;  // the boundary, as a position
    if (RES && p.rejoin_block) {
        if (lane == 0) p.rejoin_block[cand] = INT_MAX;
        if (cand != p.snap_cand && p.k_end == 0) {
            const int j = MOVES ? move_hi : scalar_read(p.diff_last, cand);
            if (j >= 0 && (j >> 6) + 1 <= p.rejoin_blocks) rejoin_k = 64 * ((j >> 6) + 1);
        }
    }
    const int peek_copy = wave_no & (KVS_PROGRESS_COPIES - 1);
    // (row 0 has published the boundary's snapshot, hence its start rounds before the boundary too)
    auto rest_is_row0 = [&](int boundary_block) __attribute__((always_inline)) -> bool {  // (a call would not know of the register block)
        const int avail = ONE ? progress_peek<NR>(p.snap_flags, peek_copy) : p.rejoin_blocks;
        if (avail < boundary_block) return false;
        const int i = MOVES ? move_lo : scalar_read(p.diff_first, cand);
        const int j = MOVES ? move_hi : scalar_read(p.diff_last, cand);
        const int at_j = snapshot_word<NR>(p.start0, j);
        const int before_i = i > 0 ? snapshot_word<NR>(p.start0, i - 1) : 0;
        return at_j == before_i;
    };
    if (rejoin_k >= 0 && rest_is_row0(rejoin_k >> 6)) {  // nothing to place at all
        if (lane == 0) {
            p.rejoin_block[cand] = 0;
            if (p.tel_out) p.tel_out[cand] = 0;
        }
        return;
    }
    if (RES && p.resume_block) {
        const int planned = scalar_read(p.resume_block, cand);
        // ONE: taken in this very launch: wait for it, within bounds
        const int rb = ONE ? snapshot_wait<NR>(p.snap_flags, planned, p.snap_wait_polls, wave_no & (KVS_PROGRESS_COPIES - 1)) : planned;
        if (ONE && rb != planned) p.resume_block[cand] = rb;  // (every lane, same value) the accounts show what was really skipped
        if (rb > 0) {
            k_first = 64 * rb;
            state_in = p.snapshots + (size_t)(rb - 1) * (size_t)p.snap_stride;
        }
    }
    const bool takes_snapshots = RES && p.snap_blocks > 0 && cand == p.snap_cand;
    int b64 = 0;             // round of lane 0 of register 0: 64 * floor((t + 1) / 64)
    int t = 0;               // start round of the previous request in the order
    long long tel_lane = 0;  // completion rounds summed per lane; added up over the lanes at the end
    if (state_in) {
        b64 = snapshot_word<NR>(state_in, 0);
        t = snapshot_word<NR>(state_in, 1);
        if (t < 0) {  // the shared prefix could not be scheduled
            if (lane == 0 && p.tel_out) p.tel_out[cand] = -1;
            return;
        }
        tel_lane = ((const long long *)(state_in + 64))[lane];
        prof_load<NR>(state_in + KVS_STATE_HEAD_WORDS, lane);
    } else {
        prof_init<NR>();
    }
    const int vmin = -(1 << 30);  // below every bound (s - M > -2^30), and s - M may still be added to it

    // 64 positions of the order at a time: ids read coalesced, lengths gathered; the next
    // block is fetched while the current one is being placed.  Within a block of cnt positions
    // lane cnt - 1 holds the first and lane 0 the last (place_block counts its lane number down).
    int rq_n = 0, sv_n = 1, ov_n = 1;
    {
        const int k = k_first + min(WAVE, n - k_first) - 1 - lane;
        if (k >= k_first) {
            rq_n = min(max(rd.at(k), 0), n_all - 1);
            sv_n = p.s[rq_n];
            ov_n = p.o[rq_n];
        }
    }
    int n_stop = n;  // (the loop has one way out: the kernel's assembly operands stay scalar that way)
    for (int k0 = k_first; k0 < n_stop; k0 += WAVE) {
        if (RES && k0 == rejoin_k && rest_is_row0(k0 >> 6)) {  // the state is row 0's after k0 positions
            const int32_t *snap = p.snapshots + (size_t)((k0 >> 6) - 1) * (size_t)p.snap_stride;
            tel_lane -= ((const long long *)(snap + 64))[lane];
            if (lane == 0) p.rejoin_block[cand] = k0 >> 6;
            n_stop = 0;
            continue;
        }
        if (takes_snapshots && k0 > 0 && (k0 >> 6) <= p.snap_blocks) {  // the state after k0 positions
            int32_t *snap = p.snapshots + (size_t)((k0 >> 6) - 1) * (size_t)p.snap_stride;
            state_head_store<NR>(snap, b64, t, tel_lane, lane);
            prof_store<NR>(snap + KVS_STATE_HEAD_WORDS, lane);
            if (ONE) snapshot_publish<NR>(p.snap_flags, k0 >> 6, lane);
        }
        const int cnt = __builtin_amdgcn_readfirstlane(min(WAVE, n - k0));
        const int k = k0 + cnt - 1 - lane;  // this lane's position (none if k < k0)
        const int rq = rq_n, sv = sv_n, ov = ov_n;
        rq_n = 0, sv_n = 1, ov_n = 1;
        {
            const int k1 = k0 + WAVE;
            const int kn = k1 + min(WAVE, n - k1) - 1 - lane;
            if (kn >= k1) {
                rq_n = min(max(rd.at(kn), 0), n_all - 1);
                sv_n = p.s[rq_n];
                ov_n = p.o[rq_n];
            }
        }
        const bool bad = (sv < 1) | (ov < 1) | (ov > p.o_bound) | ((long long)sv + (long long)ov > (long long)M);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // cannot be scheduled: report, do not loop forever
            if (lane == 0) {
                if (p.tel_out) p.tel_out[cand] = -1;
                if (p.state_out) p.state_out[1] = -1;  // poisons every timeline that resumes from it
            }
            if (ONE && takes_snapshots)  // nobody shall wait for the snapshots that will not come
                snapshot_progress_set<NR>(p.snap_flags, ~(k0 >> 6), lane);
            return;  // (snapshots not taken stay marked unusable, as the host left them)
        }
        // the up to 64 requests of this block, one after the other (place_block returns the lanes' start
        // rounds); cv: completion round of this lane's position
        const int pv = place_block<NR>(cnt, M - sv, ov, lane, vmin, M, t, b64);
        const int cv = (k >= k0 ? ov : 0) + pv;
        tel_lane += cv;
        if (crow && k >= k0) crow[p.completion_by_position ? k : rq] = cv;
        if ((RES ? takes_snapshots : p.C == 1) && p.start0 && k >= k0) p.start0[k] = pv;  // (published with the next snapshot)
    }
    if (p.state_out) {
        state_head_store<NR>(p.state_out, b64, t, tel_lane, lane);
        prof_store<NR>(p.state_out + KVS_STATE_HEAD_WORDS, lane);
    }
    for (int d = 32; d > 0; d >>= 1) tel_lane += __shfl_down(tel_lane, d);
    const long long tel = tel_lane;  // lane 0 holds the total
    if (lane == 0 && p.tel_out) p.tel_out[cand] = tel;
}

template <int NR, int WPB>
int launch_reg(const SimParams &p, hipStream_t st)
{
    const unsigned blocks = (unsigned)((p.C + WPB - 1) / WPB);
    // (Resumed timelines are of very different length and many stop early: a workgroup of one wavefront gives
    // its place to the next as soon as it ends.)
    if (p.src.moves && p.cand_list && p.snap_flags)  // moves against a base order, resumed from the base order's states
        hipLaunchKernelGGL((timeline_reg_kernel<NR, 1, true, true, true>), dim3((unsigned)p.C), dim3(WAVE), 0, st, p);
    else if (p.src.orders && p.cand_list && p.snap_flags)
        hipLaunchKernelGGL((timeline_reg_kernel<NR, 1, false, true, true>), dim3((unsigned)p.C), dim3(WAVE), 0, st, p);
    else if (p.src.orders && p.cand_list)
        hipLaunchKernelGGL((timeline_reg_kernel<NR, WPB, false, true, false>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    else if (p.src.orders)
        hipLaunchKernelGGL((timeline_reg_kernel<NR, WPB, false, false, false>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    else
        hipLaunchKernelGGL((timeline_reg_kernel<NR, WPB, true, false, false>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

}  // namespace

static int reg_rows_for(int32_t o_bound)
{
    const int rows = (o_bound + 63) / 64 + 1;
    return rows <= 9 ? 9 : rows <= 33 ? 33 : rows <= 65 ? 65 : rows <= 129 ? 129 : 225;
}

int32_t kvs_reg_state_words(int32_t o_bound) { return KVS_STATE_HEAD_WORDS + 64 * reg_rows_for(o_bound); }

// o_bound <= KVS_REG_MAX_O.  Rows needed: ceil(o_bound / 64) + 1.  Wavefronts per SIMD by file size
// (512 VGPRs per SIMD lane): 8 up to 33 rows, 5 at 65, 3 at 129, 2 at 225; a file cannot be larger
// than that, vector instructions address 256 registers.
int kvs_launch_simulate_reg(const SimParams &p, hipStream_t st)
{
    const int rows = (p.o_bound + 63) / 64 + 1;
    if (rows <= 9) return launch_reg<9, 4>(p, st);
    if (rows <= 33) return launch_reg<33, 4>(p, st);
    if (rows <= 65) return launch_reg<65, 4>(p, st);
    if (rows <= 129) return launch_reg<129, 4>(p, st);
    if (rows <= 225) return launch_reg<225, 4>(p, st);
    return KVSCHED_ERANGE;
}
