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
// The row loops are hand-written gfx950 assembly over a fixed block of physical VGPRs (v24
// upward) that only these assembly blocks touch.  The kernel is bound by the scalar unit (one per
// compute unit, shared by its four SIMDs: adding eight scalar instructions per request cost
// 11 % of the run time, eight vector instructions 1.6 %), so the loops are laid out to need
// almost no scalar work: a pass over rows 0..re is entered by one computed jump
// (s_getpc / s_setpc, 64-byte slots) to a stub that handles the masked last row `re` with
// constant register numbers and then branches into a descending chain of full rows re-1..0,
// which runs to its end without a single compare or branch.  Rows are paired (five vector
// instructions per two rows in the check, three in the update).  Only the rounds that enter
// the window after t has moved are reached through VGPR index mode.
// The compiler-generated part of the kernel needs fewer than 24 VGPRs, so it never allocates
// the block (the build verifies that); the clobber lists keep the block, s72, s73 and vcc out
// of its hands across the assembly statements.
#include "kvsched_internal.h"
#include "device_util.h"

#include <limits.h>

namespace {

// First register of the profile block; the KVS_CLOB_* lists start there.
#define KVS_PB "24"

#define KVS_CLOB_9 "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32"
#define KVS_CLOB_33                                                                                               \
    KVS_CLOB_9, "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", \
        "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56"
#define KVS_CLOB_65                                                                                                \
    KVS_CLOB_33, "v57", "v58", "v59", "v60", "v61", "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", \
        "v71", "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85",   \
        "v86", "v87", "v88"

// Row numbers as the assembler's .irp wants them: all rows ascending (one stub each), and the
// rows that can be the last row of a window with at least one full row below, descending.
#define KVS_ASC_9 "0,1,2,3,4,5,6,7,8"
#define KVS_DESC_9 "8,7,6,5,4,3,2,1"
#define KVS_ASC_33 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32"
#define KVS_DESC_33 "32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"
#define KVS_ASC_65 "0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,32,33,34,35,36,37,38,39,40,41,42,43,44,45,46,47,48,49,50,51,52,53,54,55,56,57,58,59,60,61,62,63,64"
#define KVS_DESC_65 "64,63,62,61,60,59,58,57,56,55,54,53,52,51,50,49,48,47,46,45,44,43,42,41,40,39,38,37,36,35,34,33,32,31,30,29,28,27,26,25,24,23,22,21,20,19,18,17,16,15,14,13,12,11,10,9,8,7,6,5,4,3,2,1"

// gfx950 needs a wait state between s_set_gpr_idx_on and the first VALU instruction that uses
// the index: issued back to back, about 0.3 % of the timelines of a fully occupied GPU came
// out wrong (never on a lightly loaded one); a single s_nop removed every mismatch.  Two wait
// states are inserted.
#define KVS_IDX_WAIT "s_nop 1\n"

// Expands STMT(clobber-list, rows ascending, rows descending) for the instantiated file size
// (NR - 1 must be even: the row chains process rows in pairs).
#define KVS_FOR_NR(STMT)                                                                            \
    do {                                                                                            \
        if constexpr (NR == 9) {                                                                    \
            STMT(KVS_CLOB_9, KVS_ASC_9, KVS_DESC_9);                                                \
        } else if constexpr (NR == 33) {                                                            \
            STMT(KVS_CLOB_33, KVS_ASC_33, KVS_DESC_33);                                             \
        } else {                                                                                    \
            static_assert(NR == 9 || NR == 33 || NR == 65, "profile file sizes: 9, 33 or 65 rows"); \
            STMT(KVS_CLOB_65, KVS_ASC_65, KVS_DESC_65);                                             \
        }                                                                                           \
    } while (0)

// Q_r = 64 r for all rows: nothing committed.
template <int NR>
__device__ __forceinline__ void prof_init()
{
#define KVS_STMT(CLOB, ASC, DESC)                                        \
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
#define KVS_STMT(CLOB, ASC, DESC)                                                           \
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
#define KVS_STMT(CLOB, ASC, DESC)                                                           \
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

// Rows move down by one: row r takes over the rounds of row r + 1 (whose offset was 64 more);
// the top row becomes empty.
template <int NR>
__device__ __forceinline__ void prof_rotate1()
{
#define KVS_STMT(CLOB, ASC, DESC)                                                            \
    asm volatile(".set kvs_r, 0\n"                                                 \
                 ".rept %c[nrm1]\n"                                                \
                 "  v_subrev_u32 v[" KVS_PB "+kvs_r], 64, v[" KVS_PB "+kvs_r+1]\n" \
                 "  .set kvs_r, kvs_r+1\n"                                         \
                 ".endr\n"                                                         \
                 "v_mov_b32 v[" KVS_PB "+%c[nrm1]], 64*%c[nrm1]\n"                 \
                 :                                                                 \
                 : [nrm1] "n"(NR - 1)                                              \
                 : CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

// Computed jump to the 64-byte slot of row re = x64/64 - 1: the slots start 64 bytes after the
// instruction that follows s_getpc_b64 (four 4-byte instructions, then padding).
#define KVS_DISPATCH                      \
    "s_getpc_b64 s[72:73]\n"              \
    "s_andn2_b32 %[t0], %[x64], 63\n"     \
    "s_add_u32 s72, s72, %[t0]\n"         \
    "s_addc_u32 s73, s73, 0\n"            \
    "s_setpc_b64 s[72:73]\n"              \
    ".fill 12, 4, 0xbf800000\n"

// Pads the slot that began at the last label 7 to 64 bytes (never executed: slots end in a branch).
#define KVS_SLOT_END "  .fill (64-(.-7b))/4, 4, 0xbf800000\n"

// Rows 0..re (row 0 holds round t + 1): per lane, the largest over its rounds of the least
// admissible start, relative to the lane's round in row 0.  x64 = (t + o - b64) + 64, so that
// re = x64/64 - 1 and the last round of the window sits in lane x64 & 63 of row re; sb = s - M;
// vmin = INT_MIN in every lane.
template <int NR>
__device__ __forceinline__ int prof_check_from0(int x64, int sb, int lane, int vmin)
{
    int acc, y, z, t0;
#define KVS_STMT(CLOB, ASC, DESC)                                                              \
    asm volatile("s_and_b32 %[t0], %[x64], 63\n"                                               \
                 "v_cmp_ge_u32 vcc, %[t0], %[lane]\n" KVS_DISPATCH                             \
                 ".irp r," ASC "\n"                                                            \
                 "7:\n"                                                                        \
                 "  v_add_u32 %[y], %[sb], v[" KVS_PB "+\\r]\n"                                \
                 "  v_min_i32 %[y], 64*\\r, %[y]\n"                                            \
                 "  v_cndmask_b32 %[acc], %[vmin], %[y], vcc\n"                                \
                 "  .if \\r == 0\n"                                                            \
                 "    s_branch 9f\n"                                                           \
                 "  .else\n"                                                                   \
                 "    .if (\\r & 1) == 1\n"                                                    \
                 "      v_mov_b32 %[z], %[acc]\n"                                              \
                 "    .endif\n"                                                                \
                 "    s_branch 20\\r\\()f\n"                                                   \
                 "  .endif\n" KVS_SLOT_END                                                     \
                 ".endr\n"                                                                     \
                 ".irp r," DESC "\n"                                                           \
                 "20\\r:\n"                                                                    \
                 "  .if ((\\r-1) & 1) == 1\n"                                                  \
                 "    v_add_u32 %[z], %[sb], v[" KVS_PB "+\\r-1]\n"                            \
                 "    v_min_i32 %[z], 64*(\\r-1), %[z]\n"                                      \
                 "  .else\n"                                                                   \
                 "    v_add_u32 %[y], %[sb], v[" KVS_PB "+\\r-1]\n"                            \
                 "    v_min_i32 %[y], 64*(\\r-1), %[y]\n"                                      \
                 "    v_max3_i32 %[acc], %[acc], %[y], %[z]\n"                                 \
                 "  .endif\n"                                                                  \
                 ".endr\n"                                                                     \
                 "9:\n"                                                                        \
                 : [acc] "=&v"(acc), [y] "=&v"(y), [z] "=&v"(z), [t0] "=&s"(t0)                \
                 : [x64] "s"(x64), [sb] "s"(sb), [lane] "v"(lane), [vmin] "v"(vmin)            \
                 : "scc", "vcc", "s72", "s73", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return acc;
}

// The same over rows rs..re with rs > 0 unknown at compile time (the rounds that entered the
// window after t moved): short scalar loop through VGPR index mode.
template <int NR>
__device__ __forceinline__ int prof_check_from(int rs, int x64, int sb, int lane, int vmin)
{
    int acc, y, t0, t1, re;
#define KVS_STMT(CLOB, ASC, DESC)                                                                 \
    asm volatile("v_mov_b32 %[acc], %[vmin]\n"                                                    \
                 "s_lshr_b32 %[re], %[x64], 6\n"                                                  \
                 "s_sub_u32 %[re], %[re], 1\n"                                                    \
                 "s_mov_b32 %[t1], %[rs]\n"                                                       \
                 "s_cmp_ge_u32 %[t1], %[re]\n"                                                    \
                 "s_cbranch_scc1 2f\n"                                                            \
                 "1:\n"                                                                           \
                 "s_set_gpr_idx_on %[t1], gpr_idx(SRC0)\n" KVS_IDX_WAIT                           \
                 "v_mov_b32 %[y], v[" KVS_PB "]\n"                                                \
                 "s_set_gpr_idx_off\n"                                                            \
                 "s_lshl_b32 %[t0], %[t1], 6\n"                                                   \
                 "v_add_u32 %[y], %[sb], %[y]\n"                                                  \
                 "v_min_i32 %[y], %[t0], %[y]\n"                                                  \
                 "v_max_i32 %[acc], %[acc], %[y]\n"                                               \
                 "s_add_u32 %[t1], %[t1], 1\n"                                                    \
                 "s_cmp_lt_u32 %[t1], %[re]\n"                                                    \
                 "s_cbranch_scc1 1b\n"                                                            \
                 "2:\n"                                                                           \
                 "s_set_gpr_idx_on %[re], gpr_idx(SRC0)\n" KVS_IDX_WAIT                           \
                 "v_mov_b32 %[y], v[" KVS_PB "]\n"                                                \
                 "s_set_gpr_idx_off\n"                                                            \
                 "s_lshl_b32 %[t0], %[re], 6\n"                                                   \
                 "v_add_u32 %[y], %[sb], %[y]\n"                                                  \
                 "v_min_i32 %[y], %[t0], %[y]\n"                                                  \
                 "s_and_b32 %[t0], %[x64], 63\n"                                                  \
                 "v_cmp_ge_u32 vcc, %[t0], %[lane]\n"                                             \
                 "v_cndmask_b32 %[y], %[vmin], %[y], vcc\n"                                       \
                 "v_max_i32 %[acc], %[acc], %[y]\n"                                               \
                 : [acc] "=&v"(acc), [y] "=&v"(y), [t0] "=&s"(t0), [t1] "=&s"(t1), [re] "=&s"(re) \
                 : [rs] "s"(rs), [x64] "s"(x64), [sb] "s"(sb), [lane] "v"(lane), [vmin] "v"(vmin) \
                 : "scc", "vcc", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
    return acc;
}

// Admit: rows 0..re get the request's ramp.  ramp = s + (tau - t) for the lane's round in row 0.
// The chain of full rows runs downwards with a running ramp `e` (the ramp of the even row of
// the current pair) that steps by -128 per pair; the lowest pair uses `ramp` itself.
template <int NR>
__device__ __forceinline__ void prof_update(int x64, int ramp, int lane)
{
    int y, e, t0;
#define KVS_STMT(CLOB, ASC, DESC)                                                              \
    asm volatile("s_and_b32 %[t0], %[x64], 63\n"                                               \
                 "v_cmp_ge_u32 vcc, %[t0], %[lane]\n" KVS_DISPATCH                             \
                 ".irp r," ASC "\n"                                                            \
                 "7:\n"                                                                        \
                 "  .if \\r == 0\n"                                                            \
                 "    v_cndmask_b32 %[y], 0, %[ramp], vcc\n"                                   \
                 "  .else\n"                                                                   \
                 "    v_add_u32 %[y], 64*\\r, %[ramp]\n"                                       \
                 "    v_cndmask_b32 %[y], 0, %[y], vcc\n"                                      \
                 "  .endif\n"                                                                  \
                 "  v_add_u32 v[" KVS_PB "+\\r], %[y], v[" KVS_PB "+\\r]\n"                    \
                 "  .if \\r >= 3\n"                                                            \
                 "    v_add_u32 %[e], 128*((\\r-1)/2), %[ramp]\n"                              \
                 "  .endif\n"                                                                  \
                 "  .if \\r == 0\n"                                                            \
                 "    s_branch 8f\n"                                                           \
                 "  .else\n"                                                                   \
                 "    s_branch 30\\r\\()f\n"                                                   \
                 "  .endif\n" KVS_SLOT_END                                                     \
                 ".endr\n"                                                                     \
                 ".irp r," DESC "\n"                                                           \
                 "30\\r:\n"                                                                    \
                 "  .if (\\r-1) >= 2\n"                                                        \
                 "    .if ((\\r-1) & 1) == 1\n"                                                \
                 "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[e], 64\n"       \
                 "    .else\n"                                                                 \
                 "      v_add_u32 v[" KVS_PB "+\\r-1], %[e], v[" KVS_PB "+\\r-1]\n"            \
                 "      v_add_u32 %[e], 0xffffff80, %[e]\n"                                    \
                 "    .endif\n"                                                                \
                 "  .else\n"                                                                   \
                 "    .if ((\\r-1) & 1) == 1\n"                                                \
                 "      v_add3_u32 v[" KVS_PB "+\\r-1], v[" KVS_PB "+\\r-1], %[ramp], 64\n"    \
                 "    .else\n"                                                                 \
                 "      v_add_u32 v[" KVS_PB "+\\r-1], %[ramp], v[" KVS_PB "+\\r-1]\n"         \
                 "    .endif\n"                                                                \
                 "  .endif\n"                                                                  \
                 ".endr\n"                                                                     \
                 "8:\n"                                                                        \
                 : [y] "=&v"(y), [e] "=&v"(e), [t0] "=&s"(t0)                                  \
                 : [x64] "s"(x64), [ramp] "v"(ramp), [lane] "v"(lane)                          \
                 : "scc", "vcc", "s72", "s73", CLOB)
    KVS_FOR_NR(KVS_STMT);
#undef KVS_STMT
}

// Maximum over the 64 lanes (all active).  Four DPP steps give every lane of a 16-lane row the
// row's maximum; two row broadcasts carry it to lane 63.  A DPP read of a register written by
// the previous instruction needs two wait states.
__device__ __forceinline__ int wave_max_dpp(int v)
{
    int out;
    asm volatile("s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] row_half_mirror row_mask:0xf bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] row_mirror row_mask:0xf bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] row_bcast:15 row_mask:0xa bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_max_i32_dpp %[v], %[v], %[v] row_bcast:31 row_mask:0xc bank_mask:0xf\n"
                 "s_nop 1\n"
                 "v_readlane_b32 %[out], %[v], 63\n"
                 : [v] "+v"(v), [out] "=s"(out));
    return out;
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
#define KVS_STMT(CLOB, ASC, DESC)                                                                        \
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
#define KVS_STMT(CLOB, ASC, DESC)                                                       \
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
__device__ __forceinline__ int snapshot_wait(const int32_t *progress, int rb, int polls, int copy)
{
    int f, cnt, last, voff, v;
    asm volatile("s_cmp_eq_u32 %[rb], 0\n"
                 "s_cbranch_scc1 4f\n"
                 "s_max_i32 %[cnt], %[polls], 1\n"
                 "s_mov_b32 %[last], -1\n"
                 "s_lshl_b32 %[f], %[copy], 6\n"
                 "v_mov_b32 %[voff], %[f]\n"
                 "1:\n"
                 "global_load_dword %[v], %[voff], %[base] sc1\n"
                 "s_waitcnt vmcnt(0)\n"
                 "v_readfirstlane_b32 %[f], %[v]\n"
                 "s_cmp_lt_i32 %[f], 0\n"
                 "s_cbranch_scc1 3f\n"  // the writer has stopped
                 "s_cmp_ge_i32 %[f], %[rb]\n"
                 "s_cbranch_scc1 4f\n"  // it is there
                 "s_cmp_eq_u32 %[f], %[last]\n"
                 "s_cbranch_scc1 2f\n"
                 "s_mov_b32 %[last], %[f]\n"  // the writer has moved: count anew
                 "s_max_i32 %[cnt], %[polls], 1\n"
                 "s_branch 5f\n"
                 "2:\n"
                 "s_sub_u32 %[cnt], %[cnt], 1\n"
                 "s_cmp_eq_u32 %[cnt], 0\n"
                 "s_cbranch_scc0 5f\n"
                 "s_mov_b32 %[rb], %[f]\n"  // waited long enough: what there is (f < rb)
                 "s_branch 4f\n"
                 "5:\n"
                 "s_sleep 127\n"
                 "s_branch 1b\n"
                 "3:\n"
                 "s_not_b32 %[f], %[f]\n"  // snapshots published before it stopped
                 "s_min_i32 %[rb], %[rb], %[f]\n"
                 "4:\n"
                 "buffer_inv sc1\n"
                 : [rb] "+s"(rb), [f] "=&s"(f), [cnt] "=&s"(cnt), [last] "=&s"(last), [voff] "=&v"(voff), [v] "=&v"(v)
                 : [base] "s"(progress), [polls] "s"(polls), [copy] "s"(copy)
                 : "scc", "memory");
    return rb;
}

// One int32 of a snapshot's head through the vector unit (the scalar cache takes no part in the
// hand-over above).
__device__ __forceinline__ int snapshot_word(const int32_t *snap, int index)
{
    int off, v;
    asm volatile("v_mov_b32 %[off], %[idx]\n"
                 "global_load_dword %[v], %[off], %[base]\n"
                 "s_waitcnt vmcnt(0)\n"
                 : [off] "=&v"(off), [v] "=&v"(v)
                 : [base] "s"(snap), [idx] "s"(index * 4)
                 : "memory");
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
    int32_t *crow = p.completion_out ? p.completion_out + (size_t)cand * (size_t)n_all : nullptr;

    // positions [k_first, n) of the order are placed; the state after the first k_first ones
    // (a prefix shared by all candidates) comes from memory when there is one
    int k_first = p.k_begin;
    const int32_t *state_in = p.state_in;
    if (RES && p.resume_block) {
        const int planned = scalar_read(p.resume_block, cand);
        // ONE: taken in this very launch: wait for it, within bounds
        const int rb = ONE ? snapshot_wait(p.snap_flags, planned, p.snap_wait_polls, wave_no & (KVS_PROGRESS_COPIES - 1)) : planned;
        if (ONE && rb != planned) p.resume_block[cand] = rb;  // (every lane, same value) the accounts show what was really skipped
        if (rb > 0) {
            k_first = 64 * rb;
            state_in = p.snapshots + (size_t)(rb - 1) * (size_t)p.snap_stride;
        }
    }
    const bool takes_snapshots = RES && p.snap_blocks > 0 && cand == p.snap_cand;
    const int n = p.k_end > 0 ? p.k_end : n_all;  // one past the last position placed here
    int b64 = 0;             // round of lane 0 of register 0: 64 * floor((t + 1) / 64)
    int t = 0;               // start round of the previous request in the order
    long long tel_lane = 0;  // completion rounds summed per lane; added up over the lanes at the end
    if (state_in) {
        b64 = snapshot_word(state_in, 0);
        t = snapshot_word(state_in, 1);
        if (t < 0) {  // the shared prefix could not be scheduled
            if (lane == 0 && p.tel_out) p.tel_out[cand] = -1;
            return;
        }
        tel_lane = ((const long long *)(state_in + 64))[lane];
        prof_load<NR>(state_in + KVS_STATE_HEAD_WORDS, lane);
    } else {
        prof_init<NR>();
    }
    int u64 = t - b64 + 64;  // x64 of a request is its decode length plus this
    const int vmin = INT_MIN;

    // 64 positions of the order at a time: ids read coalesced, lengths gathered; the next
    // block is fetched while the current one is being placed
    int rq_n = 0, sv_n = 1, ov_n = 1;
    if (k_first + lane < n) {
        rq_n = min(max(rd.at(k_first + lane), 0), n_all - 1);
        sv_n = p.s[rq_n];
        ov_n = p.o[rq_n];
    }
    for (int k0 = k_first; k0 < n; k0 += WAVE) {
        if (takes_snapshots && k0 > 0 && (k0 >> 6) <= p.snap_blocks) {  // the state after k0 positions
            int32_t *snap = p.snapshots + (size_t)((k0 >> 6) - 1) * (size_t)p.snap_stride;
            state_head_store<NR>(snap, b64, t, tel_lane, lane);
            prof_store<NR>(snap + KVS_STATE_HEAD_WORDS, lane);
            if (ONE) snapshot_publish<NR>(p.snap_flags, k0 >> 6, lane);
        }
        const int k = k0 + lane;
        const int rq = rq_n, sv = sv_n, ov = ov_n;
        rq_n = 0, sv_n = 1, ov_n = 1;
        if (k + WAVE < n) {
            rq_n = min(max(rd.at(k + WAVE), 0), n_all - 1);
            sv_n = p.s[rq_n];
            ov_n = p.o[rq_n];
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
        const int cnt = min(WAVE, n - k0);
        int cv = 0;  // completion round of position k0 + lane
        for (int j = 0; j < cnt; ++j) {
            const int sj = __builtin_amdgcn_readlane(sv, j);
            const int oj = __builtin_amdgcn_readlane(ov, j);
            const int sb = sj - M;
            int x64 = oj + u64;  // (t + oj - b64) + 64: row and lane of the window's last round
            int need = prof_check_from0<NR>(x64, sb, lane, vmin) + (lane + b64);  // least start the lane's rounds allow
            while (__builtin_amdgcn_ballot_w64(need > t) != 0) {
                t = wave_max_dpp(need);
                const int lo = x64 + b64 - 63;  // first round not looked at yet
                // keep register 0 on the row of round t + 1
                const int b64n = (t + 1) & ~63;
                int shift = (b64n - b64) >> 6;
                b64 = b64n;
                u64 = t - b64 + 64;
                x64 = oj + u64;
                if (shift >= NR) {
                    prof_init<NR>();
                } else {
                    for (; shift > 0; --shift) prof_rotate1<NR>();
                }
                need = prof_check_from<NR>((lo - b64) >> 6, x64, sb, lane, vmin) + (lane + b64);
            }
            // admitted at round t: holds sj + a tokens at round t + a, i.e. sj - t + b64 + l in lane l of row 0
            prof_update<NR>(x64, lane + (sj + 64 - u64), lane);
            const int hi = t + oj;
            cv = (lane == j) ? hi : cv;  // vector compare + select: the scalar unit is the scarce one
        }
        tel_lane += cv;
        if (crow && k < n) crow[p.completion_by_position ? k : rq] = cv;
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
    if (p.src.moves && p.cand_list && p.snap_flags)  // moves against a base order, resumed from the base order's states
        hipLaunchKernelGGL((timeline_reg_kernel<NR, WPB, true, true, true>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    else if (p.src.orders && p.cand_list && p.snap_flags)
        hipLaunchKernelGGL((timeline_reg_kernel<NR, WPB, false, true, true>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
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
    return rows <= 9 ? 9 : rows <= 33 ? 33 : 65;
}

int32_t kvs_reg_state_words(int32_t o_bound) { return KVS_STATE_HEAD_WORDS + 64 * reg_rows_for(o_bound); }

// o_bound <= KVS_REG_MAX_O.  Rows needed: ceil(o_bound / 64) + 1.
int kvs_launch_simulate_reg(const SimParams &p, hipStream_t st)
{
    const int rows = (p.o_bound + 63) / 64 + 1;
    if (rows <= 9) return launch_reg<9, 4>(p, st);
    if (rows <= 33) return launch_reg<33, 4>(p, st);
    if (rows <= 65) return launch_reg<65, 4>(p, st);
    return KVSCHED_ERANGE;
}
