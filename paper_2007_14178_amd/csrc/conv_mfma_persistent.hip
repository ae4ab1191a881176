// XNOR convolution on the matrix cores, persistent form (Sec. III-A steps 1b-1d and 3, Eq. 11).
//
// Same arithmetic and operand layouts as conv_mfma.hip (FP4 +-1/0 operands of
// v_mfma_f32_32x32x64_f8f6f4, filters = rows, pixels = columns, fp32 accumulators that hold the
// integer dot products exactly); what differs is how the work is scheduled on a compute unit:
//
//   * One workgroup of 8 waves per compute unit, as two independent groups of 4 waves.  A group is
//     what a workgroup is in conv_mfma.hip (2x2 waves, 128 filters x one band of up to 256 output
//     pixels, its own half of the LDS) and walks through several (band, filter tile) items.  Each
//     SIMD holds one wave of either group.
//   * The groups run half an item apart (the second group starts when the first is half-way through
//     its first contraction), so that one group's set-up, staging and output stores run beside the
//     other group's MFMA loop instead of beside its set-up, staging and stores.
//   * The contraction of an item is ONE flat loop over all (chunk, tap, 64-channel step) with no
//     padding steps between chunks; the filter-operand ring and the pixel-operand reads run across
//     chunk boundaries.  The hand-over of an LDS chunk buffer is two counters in LDS per group
//     ("chunk c is complete in its buffer", "this wave has read the last of chunk c") instead of a
//     drain and a workgroup barrier: a wave counts up when it has done its part and looks at the
//     count a few steps before it needs the other waves' part, which by then has long happened.
//     (The LDS executes one wave's operations in issue order, so a count-up issued after a wave's
//     writes is seen after them, and reads issued after a successful look see the writes.)
//
// Every wait on a counter is bounded: a wave that has waited kSpinLimit looks goes on (a logic
// error would show as wrong numbers, never as a hang).
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "conv_mfma_common.hpp"

namespace xnor {
namespace {

constexpr int kSpinLimit = 1 << 16;
constexpr int kGroupThreads = 256;

struct PParams {
    const uint32_t *Ipk;
    const uint4 *Wx;
    const float *K, *alpha;
    const float *A;  // if not null: K is not given but formed here from A (second half of Eq. 10)
    float *out;
    int32_t *dot;
    uint32_t *Opk;   // chained form: packed signs of the output [N][OH][OW][Cwn] ...
    float *P;        // ... and per (pixel, 32-filter tile) sums of |out| [N*OH*OW][4*f_tiles]
    int Cwn, f_tiles;
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int TH;          // output rows (of the whole batch) per band
    int total_rows;  // N*OH
    int Wp;          // staged columns per input row  = (OW-1)*sw + kw
    int RHfull;      // staged rows of a whole image  = (OH-1)*sh + kh
    int S2;          // k-steps (64 channels) per tap over all channels
    int CH;          // packed words per LDS channel chunk (even)
    int nchunks;
    int pitch16;     // LDS slot pitch in 16-byte units (CH + 1, odd)
    int buf16;       // distance between a group's two chunk buffers in 16-byte units (0: one buffer)
    int ka16;        // start of the two K / alpha copies inside a group's region (16-byte units)
    int dump16;      // the 64-byte slot behind the first chunk buffer (and, buf16 on, behind the second)
                     // that takes the loop's writes of threads without a live item
    int grp16;       // size of one group's LDS region (16-byte units)
    int shared16;    // start of what both groups share: the counters, then the step table
    int tab_len;     // entries of the step table (4 * nturns + 4)
    int chunk_steps; // steps of a whole chunk: taps * CH / 2
    int nturns;      // ring turns (4 steps) per item
    int ragged;      // the last chunk has fewer than CH words
    int near_out;    // a band's outputs lie within 2^31 bytes of its first image's first filter plane of a tile
    int tile_steps;  // k-steps the workspace holds per 32-filter tile
    FastDiv dCHV, dWp, dRH;
    FastDiv dOW, dOH;
    int nbands, bands_per_xcd, items_per_xcd, wgs_per_xcd;
    int whole_items;   // the first whole_items items of an XCD are taken whole, each of the rest as two
                       // half items (one 64-filter half of the tile each), so that the last round of
                       // work is spread over twice as many groups
    int work_per_xcd;  // whole_items + 2 * (items_per_xcd - whole_items)
    int start_turn;  // the first group lets the second one start at this turn of its first item
    int prio_mask;   // the second group raises its issue priority in the turns t with (t & prio_mask) != 0
    int stagger;     // the odd workgroups of an XCD start this many times 1024 cycles late (0: all at once)
    int scr16;       // start of the eight waves' 2 KB store scratch (16-byte units), if quad is set
    int quad;        // the fp32 outputs leave as 16-byte stores of four consecutive pixels (through scr16)
#ifdef XNOR_TS_BUILD
    unsigned long long *ts;   // (measurement build) [workgroup][group][item < 8][8] shader-clock stamps
    int dbg;                  // (measurement build) 1: no output stores, 2: second groups idle
#endif
};

#ifdef XNOR_TS_BUILD
#define XNOR_STAMP_K(k, i)                                                                          \
    do {                                                                                            \
        if (p.ts && wave == 0 && (tid8 & 63) == 0 && (k) >= 0 && (k) < 8)                                  \
            p.ts[(((size_t)blockIdx.x * 2 + grp) * 8 + (k)) * 8 + (i)] = __builtin_readcyclecounter(); \
    } while (0)
#else
#define XNOR_STAMP_K(k, i) do { } while (0)
#endif

// counters (uint32) at the start of the shared area
enum { kCtrReady0 = 0, kCtrReady1 = 1, kCtrDone0 = 2, kCtrDone1 = 3, kCtrStart = 4, kCtrWords = 8 };

// One lane counts up.  Ordered behind this wave's earlier LDS operations by the LDS itself.
__device__ __forceinline__ void count_up(uint32_t lds_addr, int lane)
{
    if (lane == 0) asm volatile("ds_add_u32 %0, %1" : : "v"(lds_addr), "v"(1u) : "memory");
    asm volatile("" ::: "memory");
}

// Wait until the counter has reached `target` (counters only grow; compared as a difference so
// that a wrap would not matter).
__device__ __forceinline__ bool wait_count(uint32_t lds_addr, uint32_t target)
{
    bool ok = false;
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        uint32_t v;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr) : "memory");
        if ((int32_t)((uint32_t)__builtin_amdgcn_readfirstlane((int)v) - target) >= 0) {
            ok = true;
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    asm volatile("" ::: "memory");
    return ok;
}

// ------------------------------------------------------------------------------------------------
// The contraction of one item as ONE asm statement: nothing the compiler emits can sit between a
// load issued here and the wait that covers it, and every register that is written by a load in
// flight is a fixed register that only this statement names (v168..v255, listed as clobbers).
//
//   filter-operand ring  A[u][i]  u = 0..3 (step mod 4), i = 0..1   v[168+8u+4i .. +3]
//   pixel operands       B[p][j]  p = step mod 2, j = 0..3          v[200+16p+4j .. +3]
//   table entries boff[0..1] v232 v233;  addresses tmp[0..3] v234..v237;  counter value v238;  v239
//   staged words sv[0..1] v[240:243] v[244:247];  expanded words v[248:251] v[252:255]
//   (register tuples start at even registers)
//
// Per 64-channel step and wave: 8 MFMAs; between them the 4 pixel-operand reads for the NEXT step,
// the table entry two steps ahead, and the 2 filter-operand loads for the step THREE ahead.
//   LDS queue order per step:  T, B0, B1, B2, B3   (returns are in order: lgkmcnt(3) before the
//                              MFMA on Bj leaves the three younger requests in flight)
//   VMEM order per step:       A0, A1 of step s+3  (vmcnt(5) before the first use of A0(s),
//                              vmcnt(4) before A1(s))
// Anything else in the queues (staged words, counter operations) is older than the requests such a
// count leaves in flight, so it can only make a wait stricter.
//
// Chunk hand-over, at ring turns only.  While the loop is in chunk hc:
//   h1  at the chunk's first whole turn t1: the wave has read the last of chunk hc-1 -> count up
//   h2  one turn later: wait until every wave has (chunk hc+1 takes that buffer); this turn's steps
//       carry the expansion of the words fetched a chunk ago into it in the gaps between their
//       MFMAs; then count up "complete" and fetch the words of chunk hc+2
//   h3  at t3, the turn that holds the last step of chunk hc (whose reads ahead touch chunk
//       hc+1): wait until every wave has counted chunk hc+1 complete
// The in-loop staging takes 16-byte items (four channel words of one slot), at most two per
// thread, and whole chunks; the host only hands such layers (or single-chunk ones) to this kernel.
// ------------------------------------------------------------------------------------------------
#define RA00 "v[168:171]"
#define RA01 "v[172:175]"
#define RA10 "v[176:179]"
#define RA11 "v[180:183]"
#define RA20 "v[184:187]"
#define RA21 "v[188:191]"
#define RA30 "v[192:195]"
#define RA31 "v[196:199]"
#define RB00 "v[200:203]"
#define RB01 "v[204:207]"
#define RB02 "v[208:211]"
#define RB03 "v[212:215]"
#define RB10 "v[216:219]"
#define RB11 "v[220:223]"
#define RB12 "v[224:227]"
#define RB13 "v[228:231]"
#define RBOFF0 "v232"
#define RBOFF1 "v233"
#define RTMP0 "v234"
#define RTMPQ "v[234:237]"
#define RTMP1 "v235"
#define RTMP2 "v236"
#define RTMP3 "v237"
#define RPV "v238"
#define RSV0 "v[240:243]"
#define RSV1 "v[244:247]"
#define REA "v[248:251]"
#define REB "v[252:255]"
#define RT "v239"

#define PX_MFMA(ACC, A, B) "v_mfma_f32_32x32x64_f8f6f4 %[" #ACC "], " A ", " B ", %[" #ACC "] cbsz:4 blgp:4\n\t"
// an accumulator set to zero by the matrix pipe (0 x 0 + 0; RTMP0..3 hold zeros): eight of these take
// the pipe 256 cycles while the wave goes on, where 128 v_mov would take the wave 512
#define PX_ZERO(ACC) "v_mfma_f32_32x32x64_f8f6f4 %[" #ACC "], " RTMPQ ", " RTMPQ ", 0 cbsz:4 blgp:4\n\t"

// One step s: filter operands (a0, a1) from ring slot s % 4, pixel operands x0..x3 from operand
// buffer s % 2.  Everything a step fetches is for later steps:
//   * the pixel operands of step s + 2 go into this step's own buffer, each register one matrix
//     instruction after its last use (x0 after the instruction behind acc10, ..., x3 at the head of
//     step s + 1, from the address left in RTMP3): an LDS read has two steps to arrive, and a
//     16-byte read of 8 waves at once needs more than one;
//   * their table entry E(s + 2) sits in `bo_x`, read one and a half steps before; the entry
//     E(s + 3) is read into `bo_y` once y3's address has been formed from E(s + 1) there;
//   * the filter operands of step s + 3 go into ring slot (l0, l1), free since step s - 1.
// LDS operations complete in order; in flight at the head are, oldest first, R0 R1 R2 (step s - 2),
// R3 (s - 2), T (s - 1), R0 R1 R2 (s - 1): the counts below follow from that list.
// (G2 .. G7: further instructions for the gaps behind the third to eighth matrix instruction; the
//  last step of a turn carries the loop's bookkeeping there, where it costs no issue time)
#define PX_STEP_HEAD(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, G2, G3)                \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t"                                                                 \
    PX_MFMA(acc00, a0, x0)                                                                              \
    "ds_read_b128 " y3 ", " RTMP3 "\n\t"                                                                \
    "ds_read_b32 " bo_y ", %[tab] offset:" toff "\n\t"                                                  \
    "global_load_dwordx4 " l0 ", %[aoff], %[Ab0] offset:" goff "\n\t"                                   \
    "s_waitcnt lgkmcnt(8)\n\t"                                                                          \
    PX_MFMA(acc01, a0, x1)                                                                              \
    "global_load_dwordx4 " l1 ", %[aoff], %[Ab1] offset:" goff "\n\t"                                   \
    "s_waitcnt lgkmcnt(7)\n\t"                                                                          \
    PX_MFMA(acc02, a0, x2)                                                                              \
    G2                                                                                                  \
    "s_waitcnt lgkmcnt(6)\n\t"                                                                          \
    PX_MFMA(acc03, a0, x3)                                                                              \
    G3                                                                                                  \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t"
#define PX_STEPG(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, G2, G3, G4, G5, G6, G7)    \
    PX_STEP_HEAD(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, G2, G3)                    \
    PX_MFMA(acc10, a1, x0)                                                                              \
    "v_add_u32 " RTMP0 ", %[bB0], " bo_x "\n\t"                                                         \
    G4                                                                                                  \
    PX_MFMA(acc11, a1, x1)                                                                              \
    "ds_read_b128 " x0 ", " RTMP0 "\n\t"                                                                \
    "v_add_u32 " RTMP1 ", %[bB1], " bo_x "\n\t"                                                         \
    G5                                                                                                  \
    PX_MFMA(acc12, a1, x2)                                                                              \
    "ds_read_b128 " x1 ", " RTMP1 "\n\t"                                                                \
    "v_add_u32 " RTMP2 ", %[bB2], " bo_x "\n\t"                                                         \
    G6                                                                                                  \
    PX_MFMA(acc13, a1, x3)                                                                              \
    "ds_read_b128 " x2 ", " RTMP2 "\n\t"                                                                \
    "v_add_u32 " RTMP3 ", %[bB3], " bo_x "\n\t"                                                         \
    G7
#define PX_STEP(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff)                             \
    PX_STEPG(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, "", "", "", "", "", "")
// the step of an item that covers only one 32-filter tile per wave (a half item): without the second
// tile's MFMAs; the loads stay, so the counts do
#define PX_STEP_HALFG(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, G2, G3, G4, G5, G6, G7) \
    PX_STEP_HEAD(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, G2, G3)                    \
    "v_add_u32 " RTMP0 ", %[bB0], " bo_x "\n\t"                                                         \
    "ds_read_b128 " x0 ", " RTMP0 "\n\t"                                                                \
    "v_add_u32 " RTMP1 ", %[bB1], " bo_x "\n\t"                                                         \
    G4                                                                                                  \
    "ds_read_b128 " x1 ", " RTMP1 "\n\t"                                                                \
    "v_add_u32 " RTMP2 ", %[bB2], " bo_x "\n\t"                                                         \
    G5                                                                                                  \
    "ds_read_b128 " x2 ", " RTMP2 "\n\t"                                                                \
    "v_add_u32 " RTMP3 ", %[bB3], " bo_x "\n\t"                                                         \
    G6 G7
#define PX_STEP_HALF(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff)                        \
    PX_STEP_HALFG(a0, a1, x0, x1, x2, x3, y3, bo_x, bo_y, toff, l0, l1, goff, "", "", "", "", "", "")

// The bookkeeping of a turn, laid into the gaps of its last step: the ring and table offsets move on
// (behind the step's own last uses of them), the turn counter goes up, and `ev` says whether the next
// turn has anything to do before it starts (a hook of the chunk hand-over, the release of the second
// group, a change of issue priority); if not, the turn's end branches straight back to its start.
// The step also reads the group's two hand-over counters into RPV (ready) and RT (done): issued
// here, ahead of the step's last three operand reads, they have arrived when a hook at the next
// turn's start has waited for lgkmcnt(3), and in the common case (the other waves are within a turn
// of this one) they already show the count the hook waits for, which then costs no drain of the LDS
// queue.  `pv` says that the two registers hold such a reading (the turns that expand a chunk use
// them for other things).
#define PX_CTL2 "v_add_u32 %[aoff], " PX_AINC ", %[aoff]\n\t" "v_add_u32 %[tab], " PX_TINC ", %[tab]\n\t" \
                "s_add_u32 %[gi], %[gi], 1\n\t"
#define PX_CTL3 "ds_read_b32 " RPV ", %[ready]\n\t" "ds_read_b32 " RT ", %[done]\n\t" "s_mov_b32 %[pv], 1\n\t" \
                "s_cmp_eq_u32 %[gi], %[t1]\n\t" "s_cselect_b32 %[ev], 1, 0\n\t" "s_cmp_eq_u32 %[gi], %[t2]\n\t"
#define PX_CTL4 "s_cselect_b32 %[st2], 1, 0\n\t" "s_or_b32 %[ev], %[ev], %[st2]\n\t" "s_cmp_eq_u32 %[gi], %[t3]\n\t"
#define PX_CTL5 "s_cselect_b32 %[st2], 1, 0\n\t" "s_or_b32 %[ev], %[ev], %[st2]\n\t" "s_cmp_eq_u32 %[gi], %[sturn]\n\t"
#define PX_CTL6 "s_cselect_b32 %[st2], 1, 0\n\t" "s_or_b32 %[ev], %[ev], %[st2]\n\t" "s_and_b32 %[st2], %[gi], %[pmask]\n\t"
#define PX_CTL7 "s_cmp_lt_u32 %[st2], 2\n\t" "s_cselect_b32 %[st2], %[pmask], 0\n\t" "s_or_b32 %[ev], %[ev], %[st2]\n\t"

// one lane adds 1 to the counter at LDS address ADDR (ordered behind the wave's earlier LDS operations)
#define PX_SIGNAL(ADDR)                  \
    "s_mov_b64 exec, 1\n\t"              \
    "v_mov_b32 " RT ", 1\n\t"            \
    "ds_add_u32 %[" #ADDR "], " RT "\n\t" \
    "s_mov_b64 exec, -1\n\t"

// wait until the counter at ADDR has reached %[tg] (bounded: goes on after 65536 looks)
#define PX_WAIT(ADDR, TAG)                        \
    "s_mov_b32 %[sp], 0x10000\n\t"                \
    "Lw" TAG "%=:\n\t"                            \
    "ds_read_b32 " RPV ", %[" #ADDR "]\n\t"       \
    "s_waitcnt lgkmcnt(0)\n\t"                    \
    "v_readfirstlane_b32 %[st2], " RPV "\n\t"     \
    "s_sub_u32 %[st2], %[st2], %[tg]\n\t"         \
    "s_cmp_ge_i32 %[st2], 0\n\t"                  \
    "s_cbranch_scc1 Lwd" TAG "%=\n\t"             \
    "s_sleep 2\n\t"                               \
    "s_sub_u32 %[sp], %[sp], 1\n\t"               \
    "s_cmp_lg_u32 %[sp], 0\n\t"                   \
    "s_cbranch_scc1 Lw" TAG "%=\n\t"              \
    "Lwd" TAG "%=:\n\t"

// fetch this thread's two items of the chunk whose first word lies %[st] bytes into a slot (a thread
// without a live item fetches the band's first words and will expand them into the dump slot)
#define PX_ISSUE                                              \
    "v_add_u32 " RT ", %[st], %[soff0]\n\t"                   \
    "global_load_dwordx4 " RSV0 ", " RT ", %[band]\n\t"       \
    "v_add_u32 " RPV ", %[st], %[soff1]\n\t"                  \
    "global_load_dwordx4 " RSV1 ", " RPV ", %[band]\n\t"

// One ring turn that also expands the thread's two fetched items (8 packed words, the arithmetic of
// expand_word(): and / shift / four-entry byte table through v_perm_b32) into the chunk buffer that
// starts %[st] bytes behind buffer 0: the ~100 instructions sit in the gaps between the MFMAs, which
// a wave that issues 8 MFMAs per 256 cycles otherwise leaves empty.  The LDS writes in the queue are
// younger than the pixel-operand reads the steps' counts wait for, so the counts stay right (stricter).
// (generated by a script that lays the instructions of the expansion into the gaps of four steps;
//  the second form is the turn of a half item, without the second filter tile's MFMAs)
#define PX_TURN_COMMIT \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA00, RB00) \
    "ds_read_b128 " RB13 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF1 ", %[tab] offset:0\n\t" \
    "global_load_dwordx4 " RA30 ", %[aoff], %[Ab0] offset:0\n\t" \
    "s_waitcnt vmcnt(8)\n\t" \
    "v_add_u32 " RPV ", %[st], %[sdst0]\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA00, RB01) \
    "global_load_dwordx4 " RA31 ", %[aoff], %[Ab1] offset:0\n\t" \
    "v_and_b32 " RT ", %[m03], v240\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA00, RB02) \
    "v_lshrrev_b32 " RT ", 2, v240\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA00, RB03) \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v240\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    PX_MFMA(acc10, RA01, RB00) \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v240\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    PX_MFMA(acc11, RA01, RB01) \
    "ds_read_b128 " RB00 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF0 "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REA "\n\t" \
    "v_and_b32 " RT ", %[m03], v241\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    PX_MFMA(acc12, RA01, RB02) \
    "ds_read_b128 " RB01 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF0 "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v241\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v241\n\t" \
    PX_MFMA(acc13, RA01, RB03) \
    "ds_read_b128 " RB02 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v241\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA10, RB10) \
    "ds_read_b128 " RB03 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF0 ", %[tab] offset:4\n\t" \
    "global_load_dwordx4 " RA00 ", %[aoff], %[Ab0] offset:1024\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:16\n\t" \
    "v_and_b32 " RT ", %[m03], v242\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA10, RB11) \
    "global_load_dwordx4 " RA01 ", %[aoff], %[Ab1] offset:1024\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v242\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA10, RB12) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA10, RB13) \
    "v_lshrrev_b32 " RT ", 4, v242\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    PX_MFMA(acc10, RA11, RB10) \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF1 "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v242\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    PX_MFMA(acc11, RA11, RB11) \
    "ds_read_b128 " RB10 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF1 "\n\t" \
    "ds_write_b128 " RPV ", " REA " offset:32\n\t" \
    "v_and_b32 " RT ", %[m03], v243\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v243\n\t" \
    PX_MFMA(acc12, RA11, RB12) \
    "ds_read_b128 " RB11 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF1 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v243\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    PX_MFMA(acc13, RA11, RB13) \
    "ds_read_b128 " RB12 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF1 "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v243\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:48\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA20, RB00) \
    "ds_read_b128 " RB13 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF1 ", %[tab] offset:8\n\t" \
    "global_load_dwordx4 " RA10 ", %[aoff], %[Ab0] offset:2048\n\t" \
    "v_add_u32 " RPV ", %[st], %[sdst1]\n\t" \
    "v_and_b32 " RT ", %[m03], v244\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA20, RB01) \
    "global_load_dwordx4 " RA11 ", %[aoff], %[Ab1] offset:2048\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v244\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA20, RB02) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA20, RB03) \
    "v_lshrrev_b32 " RT ", 4, v244\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    PX_MFMA(acc10, RA21, RB00) \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF0 "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v244\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    PX_MFMA(acc11, RA21, RB01) \
    "ds_read_b128 " RB00 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF0 "\n\t" \
    "ds_write_b128 " RPV ", " REA "\n\t" \
    "v_and_b32 " RT ", %[m03], v245\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v245\n\t" \
    PX_MFMA(acc12, RA21, RB02) \
    "ds_read_b128 " RB01 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v245\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    PX_MFMA(acc13, RA21, RB03) \
    "ds_read_b128 " RB02 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF0 "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v245\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:16\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA30, RB10) \
    "ds_read_b128 " RB03 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF0 ", %[tab] offset:12\n\t" \
    "global_load_dwordx4 " RA20 ", %[aoff], %[Ab0] offset:3072\n\t" \
    "v_and_b32 " RT ", %[m03], v246\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA30, RB11) \
    "global_load_dwordx4 " RA21 ", %[aoff], %[Ab1] offset:3072\n\t" \
    "v_lshrrev_b32 " RT ", 2, v246\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA30, RB12) \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v246\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA30, RB13) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    PX_MFMA(acc10, RA31, RB10) \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF1 "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v246\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REA " offset:32\n\t" \
    PX_MFMA(acc11, RA31, RB11) \
    "ds_read_b128 " RB10 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF1 "\n\t" \
    "v_and_b32 " RT ", %[m03], v247\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    PX_MFMA(acc12, RA31, RB12) \
    "ds_read_b128 " RB11 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF1 "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    PX_MFMA(acc13, RA31, RB13) \
    "ds_read_b128 " RB12 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF1 "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:48\n\t"

#define PX_TURN_COMMIT_HALF \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA00, RB00) \
    "ds_read_b128 " RB13 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF1 ", %[tab] offset:0\n\t" \
    "global_load_dwordx4 " RA30 ", %[aoff], %[Ab0] offset:0\n\t" \
    "s_waitcnt vmcnt(8)\n\t" \
    "v_add_u32 " RPV ", %[st], %[sdst0]\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA00, RB01) \
    "global_load_dwordx4 " RA31 ", %[aoff], %[Ab1] offset:0\n\t" \
    "v_and_b32 " RT ", %[m03], v240\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA00, RB02) \
    "v_lshrrev_b32 " RT ", 2, v240\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA00, RB03) \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v240\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v240\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "ds_read_b128 " RB00 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF0 "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REA "\n\t" \
    "v_and_b32 " RT ", %[m03], v241\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "ds_read_b128 " RB01 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF0 "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v241\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v241\n\t" \
    "ds_read_b128 " RB02 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v241\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA10, RB10) \
    "ds_read_b128 " RB03 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF0 ", %[tab] offset:4\n\t" \
    "global_load_dwordx4 " RA00 ", %[aoff], %[Ab0] offset:1024\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:16\n\t" \
    "v_and_b32 " RT ", %[m03], v242\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA10, RB11) \
    "global_load_dwordx4 " RA01 ", %[aoff], %[Ab1] offset:1024\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v242\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA10, RB12) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA10, RB13) \
    "v_lshrrev_b32 " RT ", 4, v242\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF1 "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v242\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_read_b128 " RB10 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF1 "\n\t" \
    "ds_write_b128 " RPV ", " REA " offset:32\n\t" \
    "v_and_b32 " RT ", %[m03], v243\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v243\n\t" \
    "ds_read_b128 " RB11 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF1 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v243\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "ds_read_b128 " RB12 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF1 "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v243\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:48\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA20, RB00) \
    "ds_read_b128 " RB13 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF1 ", %[tab] offset:8\n\t" \
    "global_load_dwordx4 " RA10 ", %[aoff], %[Ab0] offset:2048\n\t" \
    "v_add_u32 " RPV ", %[st], %[sdst1]\n\t" \
    "v_and_b32 " RT ", %[m03], v244\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA20, RB01) \
    "global_load_dwordx4 " RA11 ", %[aoff], %[Ab1] offset:2048\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v244\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA20, RB02) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA20, RB03) \
    "v_lshrrev_b32 " RT ", 4, v244\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF0 "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v244\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_read_b128 " RB00 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF0 "\n\t" \
    "ds_write_b128 " RPV ", " REA "\n\t" \
    "v_and_b32 " RT ", %[m03], v245\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v245\n\t" \
    "ds_read_b128 " RB01 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF0 "\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v245\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "ds_read_b128 " RB02 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF0 "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v245\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:16\n\t" \
    "s_waitcnt vmcnt(5) lgkmcnt(7)\n\t" \
    PX_MFMA(acc00, RA30, RB10) \
    "ds_read_b128 " RB03 ", " RTMP3 "\n\t" \
    "ds_read_b32 " RBOFF0 ", %[tab] offset:12\n\t" \
    "global_load_dwordx4 " RA20 ", %[aoff], %[Ab0] offset:3072\n\t" \
    "v_and_b32 " RT ", %[m03], v246\n\t" \
    "v_perm_b32 v248, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt lgkmcnt(8)\n\t" \
    PX_MFMA(acc01, RA30, RB11) \
    "global_load_dwordx4 " RA21 ", %[aoff], %[Ab1] offset:3072\n\t" \
    "v_lshrrev_b32 " RT ", 2, v246\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "s_waitcnt lgkmcnt(7)\n\t" \
    PX_MFMA(acc02, RA30, RB12) \
    "v_perm_b32 v249, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v246\n\t" \
    "s_waitcnt lgkmcnt(6)\n\t" \
    PX_MFMA(acc03, RA30, RB13) \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v250, 0, %[tbl], " RT "\n\t" \
    "s_waitcnt vmcnt(6) lgkmcnt(5)\n\t" \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF1 "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v246\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v251, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REA " offset:32\n\t" \
    "ds_read_b128 " RB10 ", " RTMP0 "\n\t" \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF1 "\n\t" \
    "v_and_b32 " RT ", %[m03], v247\n\t" \
    "v_perm_b32 v252, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 2, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "ds_read_b128 " RB11 ", " RTMP1 "\n\t" \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF1 "\n\t" \
    "v_perm_b32 v253, 0, %[tbl], " RT "\n\t" \
    "v_lshrrev_b32 " RT ", 4, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v254, 0, %[tbl], " RT "\n\t" \
    "ds_read_b128 " RB12 ", " RTMP2 "\n\t" \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF1 "\n\t" \
    "v_lshrrev_b32 " RT ", 6, v247\n\t" \
    "v_and_b32 " RT ", %[m03], " RT "\n\t" \
    "v_perm_b32 v255, 0, %[tbl], " RT "\n\t" \
    "ds_write_b128 " RPV ", " REB " offset:48\n\t"

#define PX_AINC "0x1000"
#define PX_TINC "16"

#define PX_LOOP_ASM                                                                                      \
    /* scalar state */                                                                                   \
    "s_mov_b32 %[gi], 0\n\t"                                                                             \
    "s_mov_b32 %[pv], 0\n\t"                                                                             \
    "s_mov_b32 %[hc], 0\n\t"                                                                             \
    "s_mov_b32 %[t1], 0\n\t"                                                                             \
    "s_mov_b32 %[t2], 1\n\t"                                                                             \
    "s_add_u32 %[t3], %[csteps], -1\n\t"                                                                 \
    "s_lshr_b32 %[t3], %[t3], 2\n\t"                                                                     \
    /* the words of chunk 1 */                                                                           \
    "s_cmp_lt_u32 1, %[nchunks]\n\t"                                                                     \
    "s_cbranch_scc0 Lpre%=\n\t"                                                                          \
    "s_mov_b32 %[st], %[csrc]\n\t"                                                                       \
    PX_ISSUE                                                                                             \
    "Lpre%=:\n\t"                                                                                        \
    /* ring fill: filter operands of steps 0..2 */                                                       \
    "global_load_dwordx4 " RA00 ", %[aoff], %[Ab0]\n\t"                                                  \
    "global_load_dwordx4 " RA01 ", %[aoff], %[Ab1]\n\t"                                                  \
    "global_load_dwordx4 " RA10 ", %[aoff], %[Ab0] offset:1024\n\t"                                      \
    "global_load_dwordx4 " RA11 ", %[aoff], %[Ab1] offset:1024\n\t"                                      \
    "global_load_dwordx4 " RA20 ", %[aoff], %[Ab0] offset:2048\n\t"                                      \
    "global_load_dwordx4 " RA21 ", %[aoff], %[Ab1] offset:2048\n\t"                                      \
    "v_add_u32 %[aoff], 0xc00, %[aoff]\n\t"                                                              \
    /* the accumulators start at zero */                                                                 \
    "v_mov_b32 " RTMP0 ", 0\n\t"                                                                         \
    "v_mov_b32 " RTMP1 ", 0\n\t"                                                                         \
    "v_mov_b32 " RTMP2 ", 0\n\t"                                                                         \
    "v_mov_b32 " RTMP3 ", 0\n\t"                                                                         \
    "s_nop 4\n\t"                                                                                        \
    PX_ZERO(acc00) PX_ZERO(acc01) PX_ZERO(acc02) PX_ZERO(acc03)                                          \
    PX_ZERO(acc10) PX_ZERO(acc11) PX_ZERO(acc12) PX_ZERO(acc13)                                          \
    /* chunk 0 is complete in its buffer (all four waves have committed their part): waited for  */ \
    /* here, with the ring's first operands on their way                                          */ \
    "s_add_u32 %[tg], %[cbase], 4\n\t"                                                                   \
    PX_WAIT(ready, "p")                                                                                  \
    /* table entries 0 and 1; the pixel operands of step 0, entry 2, the first three operands of   */ \
    /* step 1 and the address of the fourth: the order in which the steps will issue them          */ \
    "ds_read_b32 " RBOFF0 ", %[tab]\n\t"                                                                 \
    "ds_read_b32 " RBOFF1 ", %[tab] offset:4\n\t"                                                        \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                           \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF0 "\n\t"                                                        \
    "ds_read_b128 " RB00 ", " RTMP0 "\n\t"                                                               \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF0 "\n\t"                                                        \
    "ds_read_b128 " RB01 ", " RTMP1 "\n\t"                                                               \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF0 "\n\t"                                                        \
    "ds_read_b128 " RB02 ", " RTMP2 "\n\t"                                                               \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF0 "\n\t"                                                        \
    "ds_read_b128 " RB03 ", " RTMP3 "\n\t"                                                               \
    "ds_read_b32 " RBOFF0 ", %[tab] offset:8\n\t"                                                        \
    "v_add_u32 %[tab], 12, %[tab]\n\t"                                                                   \
    "v_add_u32 " RTMP0 ", %[bB0], " RBOFF1 "\n\t"                                                        \
    "ds_read_b128 " RB10 ", " RTMP0 "\n\t"                                                               \
    "v_add_u32 " RTMP1 ", %[bB1], " RBOFF1 "\n\t"                                                        \
    "ds_read_b128 " RB11 ", " RTMP1 "\n\t"                                                               \
    "v_add_u32 " RTMP2 ", %[bB2], " RBOFF1 "\n\t"                                                        \
    "ds_read_b128 " RB12 ", " RTMP2 "\n\t"                                                               \
    "v_add_u32 " RTMP3 ", %[bB3], " RBOFF1 "\n\t"                                                        \
    /* ---- the loop over ring turns ---- */                                                             \
    "Ltop%=:\n\t"                                                                                        \
    /* (the counter readings of the turn before have landed: the hooks use their registers) */           \
    "s_waitcnt lgkmcnt(3)\n\t"                                                                           \
    "s_cmp_eq_u32 %[gi], %[sturn]\n\t"                                                                   \
    "s_cbranch_scc1 Lhs%=\n\t"                                                                           \
    "Lhk%=:\n\t"                                                                                         \
    "s_cmp_eq_u32 %[gi], %[t1]\n\t"                                                                      \
    "s_cbranch_scc1 Lh1%=\n\t"                                                                           \
    "s_cmp_eq_u32 %[gi], %[t2]\n\t"                                                                      \
    "s_cbranch_scc1 Lh2%=\n\t"                                                                           \
    "s_cmp_eq_u32 %[gi], %[t3]\n\t"                                                                      \
    "s_cbranch_scc1 Lh3%=\n\t"                                                                           \
    "Lturn%=:\n\t"                                                                                       \
    /* issue priority of this turn (second groups only: pmask != 0), see the kernel's comment */         \
    "s_cmp_eq_u32 %[pmask], 0\n\t"                                                                       \
    "s_cbranch_scc1 Lpd%=\n\t"                                                                           \
    "s_and_b32 %[st2], %[gi], %[pmask]\n\t"                                                              \
    "s_cmp_eq_u32 %[st2], 0\n\t"                                                                         \
    "s_cbranch_scc1 Lpl%=\n\t"                                                                           \
    "s_setprio 2\n\t"                                                                                    \
    "s_branch Lpd%=\n\t"                                                                                 \
    "Lpl%=:\n\t"                                                                                         \
    "s_setprio 0\n\t"                                                                                    \
    "Lpd%=:\n\t"                                                                                         \
    "s_cmp_eq_u32 %[onetile], 0\n\t"                                                                     \
    "s_cbranch_scc0 LturnH%=\n\t"                                                                        \
    "LturnW%=:\n\t"                                                                                      \
    PX_STEP(RA00, RA01, RB00, RB01, RB02, RB03, RB13, RBOFF0, RBOFF1, "0", RA30, RA31, "0")      \
    PX_STEP(RA10, RA11, RB10, RB11, RB12, RB13, RB03, RBOFF1, RBOFF0, "4", RA00, RA01, "1024")   \
    PX_STEP(RA20, RA21, RB00, RB01, RB02, RB03, RB13, RBOFF0, RBOFF1, "8", RA10, RA11, "2048")   \
    PX_STEPG(RA30, RA31, RB10, RB11, RB12, RB13, RB03, RBOFF1, RBOFF0, "12", RA20, RA21, "3072", \
             PX_CTL2, PX_CTL3, PX_CTL4, PX_CTL5, PX_CTL6, PX_CTL7)                               \
    "s_cmp_lt_u32 %[gi], %[nturns]\n\t"                                                                  \
    "s_cbranch_scc0 Lexit%=\n\t"                                                                         \
    "s_cmp_eq_u32 %[ev], 0\n\t"                                                                          \
    "s_cbranch_scc1 LturnW%=\n\t"                                                                        \
    "s_branch Ltop%=\n\t"                                                                                \
    /* the end of a turn that kept its bookkeeping for here (the turns that expand a chunk) */           \
    "Ltail%=:\n\t"                                                                                       \
    "s_mov_b32 %[pv], 0\n\t"                                                                             \
    "v_add_u32 %[aoff], " PX_AINC ", %[aoff]\n\t"                                                        \
    "v_add_u32 %[tab], " PX_TINC ", %[tab]\n\t"                                                          \
    "s_add_u32 %[gi], %[gi], 1\n\t"                                                                      \
    "s_cmp_lt_u32 %[gi], %[nturns]\n\t"                                                                  \
    "s_cbranch_scc1 Ltop%=\n\t"                                                                          \
    "Lexit%=:\n\t"                                                                                       \
    /* the reads ahead of the item's end have landed; this wave has read the last of the last chunk */   \
    "s_waitcnt vmcnt(0) lgkmcnt(0)\n\t"                                                                  \
    "s_setprio 0\n\t"                                                                                    \
    PX_SIGNAL(done)                                                                                      \
    "s_nop 15\n\t"                                                                                       \
    "s_nop 15\n\t"                                                                                       \
    "s_branch Lend%=\n\t"                                                                                \
    /* ---- the turn of a half item ---- */                                                              \
    "LturnH%=:\n\t"                                                                                      \
    PX_STEP_HALF(RA00, RA01, RB00, RB01, RB02, RB03, RB13, RBOFF0, RBOFF1, "0", RA30, RA31, "0")      \
    PX_STEP_HALF(RA10, RA11, RB10, RB11, RB12, RB13, RB03, RBOFF1, RBOFF0, "4", RA00, RA01, "1024")   \
    PX_STEP_HALF(RA20, RA21, RB00, RB01, RB02, RB03, RB13, RBOFF0, RBOFF1, "8", RA10, RA11, "2048")   \
    PX_STEP_HALFG(RA30, RA31, RB10, RB11, RB12, RB13, RB03, RBOFF1, RBOFF0, "12", RA20, RA21, "3072", \
                  PX_CTL2, PX_CTL3, PX_CTL4, PX_CTL5, PX_CTL6, PX_CTL7)                               \
    "s_cmp_lt_u32 %[gi], %[nturns]\n\t"                                                                  \
    "s_cbranch_scc0 Lexit%=\n\t"                                                                         \
    "s_cmp_eq_u32 %[ev], 0\n\t"                                                                          \
    "s_cbranch_scc1 LturnH%=\n\t"                                                                        \
    "s_branch Ltop%=\n\t"                                                                                \
    /* ---- h1 ---- */                                                                                   \
    "Lh1%=:\n\t"                                                                                         \
    "s_cmp_eq_u32 %[hc], 0\n\t"                                                                          \
    "s_cbranch_scc1 Lturn%=\n\t"                                                                         \
    PX_SIGNAL(done)                                                                                      \
    "s_branch Lturn%=\n\t"                                                                               \
    /* ---- h2: this turn also expands the next chunk ---- */                                            \
    "Lh2%=:\n\t"                                                                                         \
    "s_add_u32 %[st], %[hc], 1\n\t"                                                                      \
    "s_cmp_lt_u32 %[st], %[nchunks]\n\t"                                                                 \
    "s_cbranch_scc0 Lturn%=\n\t"                                                                         \
    "s_lshl_b32 %[tg], %[hc], 2\n\t"                                                                     \
    "s_add_u32 %[tg], %[tg], %[cbase]\n\t"                                                               \
    "s_cmp_eq_u32 %[pv], 0\n\t"                                                                          \
    "s_cbranch_scc1 Lh2s%=\n\t"                                                                          \
    "v_readfirstlane_b32 %[st2], " RT "\n\t"                                                             \
    "s_sub_u32 %[st2], %[st2], %[tg]\n\t"                                                                \
    "s_cmp_ge_i32 %[st2], 0\n\t"                                                                         \
    "s_cbranch_scc1 Lh2d%=\n\t"                                                                          \
    "Lh2s%=:\n\t"                                                                                        \
    PX_WAIT(done, "a")                                                                                   \
    "Lh2d%=:\n\t"                                                                                        \
    "s_and_b32 %[st], %[st], 1\n\t"                                                                      \
    "s_mul_i32 %[st], %[st], %[bufb]\n\t"                                                                \
    "s_cmp_eq_u32 %[onetile], 0\n\t"                                                                     \
    "s_cbranch_scc0 LcomH%=\n\t"                                                                         \
    PX_TURN_COMMIT                                                                                       \
    "Lcom2%=:\n\t"                                                                                       \
    PX_SIGNAL(ready)                                                                                     \
    "s_add_u32 %[st], %[hc], 2\n\t"                                                                      \
    "s_cmp_lt_u32 %[st], %[nchunks]\n\t"                                                                 \
    "s_cbranch_scc0 Ltail%=\n\t"                                                                         \
    "s_mul_i32 %[st], %[st], %[csrc]\n\t"                                                                \
    PX_ISSUE                                                                                             \
    "s_branch Ltail%=\n\t"                                                                               \
    "LcomH%=:\n\t"                                                                                       \
    PX_TURN_COMMIT_HALF                                                                                  \
    "s_branch Lcom2%=\n\t"                                                                               \
    /* ---- h3 ---- */                                                                                   \
    "Lh3%=:\n\t"                                                                                         \
    "s_add_u32 %[st], %[hc], 1\n\t"                                                                      \
    "s_cmp_lt_u32 %[st], %[nchunks]\n\t"                                                                 \
    "s_cbranch_scc0 Lturn%=\n\t"                                                                         \
    "s_add_u32 %[tg], %[hc], 2\n\t"                                                                      \
    "s_lshl_b32 %[tg], %[tg], 2\n\t"                                                                     \
    "s_add_u32 %[tg], %[tg], %[cbase]\n\t"                                                               \
    "s_cmp_eq_u32 %[pv], 0\n\t"                                                                          \
    "s_cbranch_scc1 Lh3s%=\n\t"                                                                          \
    "v_readfirstlane_b32 %[st2], " RPV "\n\t"                                                            \
    "s_sub_u32 %[st2], %[st2], %[tg]\n\t"                                                                \
    "s_cmp_ge_i32 %[st2], 0\n\t"                                                                         \
    "s_cbranch_scc1 Lh3d%=\n\t"                                                                          \
    "Lh3s%=:\n\t"                                                                                        \
    PX_WAIT(ready, "b")                                                                                  \
    "Lh3d%=:\n\t"                                                                                        \
    "s_mov_b32 %[hc], %[st]\n\t"                                                                         \
    "s_add_u32 %[t1], %[t3], 1\n\t"                                                                      \
    "s_add_u32 %[t2], %[t3], 2\n\t"                                                                      \
    "s_add_u32 %[st], %[hc], 1\n\t"                                                                      \
    "s_mul_i32 %[st], %[st], %[csteps]\n\t"                                                              \
    "s_add_u32 %[st], %[st], -1\n\t"                                                                     \
    "s_lshr_b32 %[t3], %[st], 2\n\t"                                                                     \
    "s_branch Lturn%=\n\t"                                                                               \
    /* ---- the first group lets the second one start ---- */                                            \
    "Lhs%=:\n\t"                                                                                         \
    PX_SIGNAL(start)                                                                                     \
    "s_mov_b32 %[sturn], -1\n\t"                                                                         \
    "s_branch Lhk%=\n\t"                                                                                 \
    "Lend%=:\n\t"

// The lane's index within its wave, produced anew (volatile: the compiler cannot carry values
// derived from it from one phase of the item loop to the next, where registers are scarce).
__device__ __forceinline__ int fresh_lane()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

template <int VW, bool CHAIN>
__global__ __launch_bounds__(512) void conv_mfma_persistent_kernel(PParams p)
{
    extern __shared__ uint4 lds[];
    const int tid8 = threadIdx.x;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid8 >> 6);   // wave-uniform, kept in an SGPR
    const int grp = wave8 >> 2, wave = wave8 & 3;
    const int wm = wave >> 1, wn = wave & 1;
    const int OHW = p.OH * p.OW;
    const int taps = p.kh * p.kw;
    const int Cw2 = 2 * p.S2;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)lds;

    // ---- shared by both groups: counters and the step table ----
    // The pixel operand of step t sits at (chunk buffer, tap(t), step-in-tap(t)) from the lane's
    // slot.  That offset is the same for every lane of either group, so it is tabulated once per
    // workgroup (one entry per step of an item in workspace order, in bytes); the entries past the
    // last step (what the reads ahead of the loop's end touch) point at tap 0 of buffer 0.
    uint32_t *const ctr = reinterpret_cast<uint32_t *>(lds + p.shared16);
    uint32_t *const table = ctr + kCtrWords;
    for (int tt = tid8; tt < p.tab_len; tt += 512) {
        const int c = min(tt / p.chunk_steps, p.nchunks - 1), t = tt - c * p.chunk_steps;
        const int steps_c = min(p.CH, Cw2 - c * p.CH) >> 1;
        uint32_t off = 0;
        if (t < taps * steps_c) {
            const int tap = t / steps_c, s = t - tap * steps_c;
            const int ky = tap / p.kw, kx = tap - ky * p.kw;
            off = (uint32_t)((c & 1) * p.buf16 + (ky * p.Wp + kx) * p.pitch16 + 2 * s);
        }
        table[tt] = off * 16u;
    }
    if (tid8 < kCtrWords) ctr[tid8] = 0;
    __syncthreads();   // the only workgroup barrier: from here on the groups go their own ways

    const uint32_t ctr_addr = lds_base + (uint32_t)p.shared16 * 16u;
    const uint32_t ready_addr = ctr_addr + 4u * (uint32_t)(kCtrReady0 + grp);
    const uint32_t done_addr = ctr_addr + 4u * (uint32_t)(kCtrDone0 + grp);
    const uint32_t start_addr = ctr_addr + 4u * (uint32_t)kCtrStart;
    const uint32_t tab_base = ctr_addr + 4u * (uint32_t)kCtrWords;
    uint4 *const glds = lds + grp * p.grp16;                       // this group's region
    const uint32_t glds_base = lds_base + (uint32_t)(grp * p.grp16) * 16u;
    char *const lds_bytes = reinterpret_cast<char *>(glds);

    // ---- which items: workgroups are handed to the 8 XCDs round-robin by their id, and each XCD
    // has its own L2.  XCD x takes a contiguous range of bands and runs through them once per filter
    // tile (item = filter tile * bands_per_xcd + band); its groups take the items round-robin, the
    // first groups of all its workgroups before the second ones, so that at any time the XCD works
    // on a window of consecutive bands of one filter tile and few compute units get the odd item.
    const int xcd = blockIdx.x & (kXcds - 1);
    const int wi = blockIdx.x >> kXcdShift;
    // (the even workgroups of an XCD come first)
    const int n_even = (p.wgs_per_xcd + 1) >> 1;
    const int slot = ((wi & 1) ? n_even + (wi >> 1) : (wi >> 1)) + grp * p.wgs_per_xcd;
#ifdef XNOR_TS_BUILD
    const int nslot = (p.dbg & 2) ? p.wgs_per_xcd : 2 * p.wgs_per_xcd;
    if ((p.dbg & 2) && grp == 1) return;
#else
    const int nslot = 2 * p.wgs_per_xcd;
#endif

    // Every group stores an item's outputs in one burst, and groups that start together stay
    // together: the workgroups without a unit of the last, partial round (the odd ones of an XCD)
    // start a quarter of an item's time late, so that the chip sees four bursts of stores per item
    // time instead of two (their second groups wait for the first ones anyway).
    if (grp == 0 && (wi & 1))
        for (int i = 0; i < p.stagger; ++i) __builtin_amdgcn_s_sleep(16);
    // the first group releases the second one at turn `sturn` of its first item (-1: not, or done);
    // with start_turn < 0 both start at once
    int sturn = grp == 0 ? p.start_turn : -1;
    if (grp == 1 && p.start_turn >= 0) wait_count(start_addr, 1u);

    typedef typename WordVec<VW>::type wvec;
    const int CHV = p.CH / VW;
    constexpr int UP = 2;                    // items per thread kept in registers

    // ---- the scalars of one item (a band x a filter tile) ----
    struct Item {
        int seq, ftile, R0, npix, n_first, oy0, r0, tile0, my_nt, items;
        int half;   // -1: the whole 128-filter tile; 0 / 1: its lower / upper 64 filters only
    };
    // work unit -> item: the whole items first, then the halves of the remaining ones
    auto item_of = [&](int seq, int &half) -> int {
        if (seq < p.whole_items) { half = -1; return seq; }
        const int h = seq - p.whole_items;
        half = h & 1;
        return p.whole_items + (h >> 1);
    };
    // the first item of this group at or after `seq` whose band exists (the last XCD's range is
    // padded), or -1.  (A division by a run-time value goes through the vector ALU: bring the
    // wave-uniform quotient back into a scalar register.)
    auto next_item = [&](int seq) -> int {
        for (; seq < p.work_per_xcd; seq += nslot) {
            int half;
            const int item = item_of(seq, half);
            const int ft = __builtin_amdgcn_readfirstlane(item / p.bands_per_xcd);
            // an upper half without filters has nothing to write (the chained form's per-tile sums
            // are read for every 32-filter tile, so there it writes its zeros)
            if (!CHAIN && half == 1 && ft * kFilterTile + kFilterTile / 2 >= p.F) continue;
            if (xcd * p.bands_per_xcd + (item - ft * p.bands_per_xcd) < p.nbands) return seq;
        }
        return -1;
    };
    auto decode = [&](int seq, Item &it) {
        it.seq = seq;
        int half_v;
        const int item = item_of(seq, half_v);
        it.half = __builtin_amdgcn_readfirstlane(half_v);
        it.ftile = __builtin_amdgcn_readfirstlane(item / p.bands_per_xcd);
        const int band = xcd * p.bands_per_xcd + (item - it.ftile * p.bands_per_xcd);
        // the band: TH rows of the batch's output rows, numbered R = n*OH + oy
        it.R0 = band * p.TH;
        const int rows = min(p.TH, p.total_rows - it.R0);
        it.npix = rows * p.OW;
        it.n_first = __builtin_amdgcn_readfirstlane(it.R0 / p.OH);
        it.oy0 = it.R0 - it.n_first * p.OH;
        it.r0 = (p.OH - 1 - it.oy0) * p.sh + p.kh;   // staged rows of the first image if it runs to its end
        const int dn_last = __builtin_amdgcn_readfirstlane((int)fdiv((uint32_t)(it.oy0 + rows - 1), p.dOH));
        const int n_last = it.n_first + dn_last, oy_last = it.oy0 + rows - 1 - dn_last * p.OH;
        const int srows = (n_last == it.n_first) ? (oy_last - it.oy0) * p.sh + p.kh
                                                 : it.r0 + (n_last - it.n_first - 1) * p.RHfull + oy_last * p.sh + p.kh;
        it.items = srows * p.Wp * CHV;           // one staging item = VW consecutive words of one slot
        // this wave's pixel tiles; the band's tiles are split evenly over the two wave columns
        const int NT = (it.npix + 31) >> 5;
        const int nt0 = (NT + 1) >> 1;
        it.tile0 = wn ? nt0 : 0;
        it.my_nt = wn ? NT - nt0 : nt0;
    };

    // ---- step 3 of the item whose dot products sit in the accumulators: out = float(dot) * K * alpha.
    // The stores are issued in eight pieces (two filter tiles x four groups of four accumulator
    // registers), after the loads of the group's NEXT item have been requested: a wave's 128 stores
    // take the compute unit's store path several thousand cycles, and a load queued behind them
    // waits that long.
    Item cur{};
    bool pending = false;   // cur's outputs are still in the accumulators
    v16f acc[kWM][kWN];
    float kvs[kWN];
    long long lane_b[kWN];
    bool lane_ok[kWN];
    int nfull = 0;
    int kitem = 0;          // contractions this group has completed
    // the 32-filter tile (of the whole layer) that this wave's accumulator row i holds
    auto tile32_of = [&](const Item &it, int i) -> int {
        return it.ftile * (2 * kWM) + (it.half < 0 ? wm * kWM + i : it.half * kWM + wm);
    };
    auto k_alpha_copy = [&](int k) -> float * {
        return reinterpret_cast<float *>(glds + p.ka16) + (k & 1) * (kBandPixels + kFilterTile);
    };
    // lane-derived indices of this phase are formed from a copy of the lane id that the compiler
    // cannot see through, or it computes them at kernel start and holds them across the loop
    auto epilogue_begin = [&]() {
        const int lane_e = fresh_lane();
        const int l32e = lane_e & 31, kge = lane_e >> 5;
        const float *Kl = k_alpha_copy(kitem - 1);
        // Per pixel tile of the wave: the lane's byte offset from (the band's first image, a filter
        // tile's first plane) to (its image, its 4*kg-th plane, its pixel), and its K.
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            const int q = (cur.tile0 + j) * 32 + l32e;                // pixel within the band
            lane_ok[j] = j < cur.my_nt && q < cur.npix;
            const int qq = lane_ok[j] ? q : 0;
            const int Rl = (int)fdiv((uint32_t)qq, p.dOW), ox = qq - Rl * p.OW;
            const int dn = (int)fdiv((uint32_t)(cur.oy0 + Rl), p.dOH);
            const int oy = cur.oy0 + Rl - dn * p.OH;
            kvs[j] = Kl[qq];
            lane_b[j] = (((long long)dn * p.F + 4 * kge) * OHW + oy * p.OW + ox) * 4;
        }
        // tiles of this wave whose 32 pixels all exist (uniform): only the band's last tile can be ragged
        nfull = max(0, min(cur.my_nt, (cur.npix - cur.tile0 * 32) >> 5));
    };
    // One filter tile (32 planes) of the wave's pixel tiles: one store instruction writes 32
    // consecutive pixels of two filter planes (two 128-byte runs).  While a band's outputs lie within
    // 2 GiB (p.near_out, decided on the host) a store is "scalar base + 32-bit lane offset": the walk
    // over the planes is scalar arithmetic and the vector ALU only multiplies.  The whole tiles go
    // plane by plane, the wave's tiles of one plane back to back: they are consecutive pixels, so
    // the cache lines that two tiles share are completed by consecutive stores.  Ragged tiles,
    // partial filter tiles and far outputs take one 64-bit vector add per store.
    auto store_filter_tile = [&](auto *tile_base, int nfilt, auto value) {
        typedef typename std::remove_pointer<decltype(tile_base)>::type elem_t;
        typedef __attribute__((address_space(1))) elem_t *ptr_t;
        const int kge = fresh_lane() >> 5;
        const long long plane1 = (long long)OHW * 4, plane5 = 5 * plane1;   // bytes between filter planes
        const bool all = nfilt >= 32;
        int first_slow = 0;
        if (p.near_out && all) {
            uint32_t v32[kWN];
#pragma unroll
            for (int j = 0; j < kWN; ++j) {
                v32[j] = (uint32_t)lane_b[j];
                asm volatile("" : "+v"(v32[j]));
            }
            // (one copy of the 16 x NF stores per count of whole tiles: a test of `j < nfull` around
            //  every store costs the wave two scalar instructions and a branch per store)
            auto planes = [&](auto nf) {
                constexpr int NF = decltype(nf)::value;
                const char *ub = reinterpret_cast<const char *>(tile_base);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
#pragma unroll
                    for (int j = 0; j < NF; ++j) *(ptr_t)(ub + v32[j]) = value(j, r);
                    ub += (r & 3) == 3 ? plane5 : plane1;
                }
            };
            switch (nfull) {
                case 4: planes(std::integral_constant<int, 4>{}); break;
                case 3: planes(std::integral_constant<int, 3>{}); break;
                case 2: planes(std::integral_constant<int, 2>{}); break;
                case 1: planes(std::integral_constant<int, 1>{}); break;
                default: break;
            }
            static_assert(kWN == 4, "one case per count of whole tiles");
            first_slow = nfull;
        }
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            if (j < first_slow || !lane_ok[j]) continue;
            char *pr = const_cast<char *>(reinterpret_cast<const char *>(tile_base)) + lane_b[j];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (all || 4 * kge + 8 * (r >> 2) + (r & 3) < nfilt) *(ptr_t)pr = value(j, r);
                pr += (r & 3) == 3 ? plane5 : plane1;
                asm volatile("" : "+v"(pr));   // (keeps the walk: one add per store)
            }
        }
    };
    // The same filter tile as 16-byte stores: a wave cannot have more than 64 vector-memory
    // operations in flight, so 128 dword stores per item hold it until the first ones are
    // acknowledged; 32 stores of 16 bytes it issues and leaves behind.  The accumulators go through
    // a 2 KB LDS scratch of the wave's own (no other wave touches it, LDS operations of a wave
    // execute in order): a stage is two registers of all four pixel tiles written as they lie (2
    // registers x 2 planes x 128 pixels), read back as four consecutive pixels per lane (32 lanes per
    // plane) and stored, plane by plane as above.
    auto store_filter_tile_quads = [&](float *tile_base, auto value) {
        typedef float __attribute__((may_alias)) fa_t;
        typedef float __attribute__((ext_vector_type(4), may_alias)) f4a_t;
        typedef float __attribute__((ext_vector_type(4))) f4_t;
        typedef __attribute__((address_space(1))) f4_t *ptr4_t;
        const int lane_s = fresh_lane();
        const int l32s = lane_s & 31, kgs = lane_s >> 5;
        // The lane as a writer of four consecutive pixels of its half-wave's plane (the host has
        // checked that such a quad never straddles two images and is 16-byte aligned).  Where the
        // wave's last tile is ragged the lanes past the last quad store that last quad once more
        // (the same bytes to the same place): no store is predicated.  (Formed here, per filter
        // tile, rather than kept in registers from the start of the phase.)
        const int nq = min(8 * cur.my_nt, (cur.npix - cur.tile0 * 32) >> 2);   // quads of the wave's own tiles (uniform, > 0)
        const int ql = min(l32s, nq - 1);
        const int q4 = cur.tile0 * 32 + 4 * ql;
        const int Rl = (int)fdiv((uint32_t)q4, p.dOW), ox = q4 - Rl * p.OW;
        const int dn = (int)fdiv((uint32_t)(cur.oy0 + Rl), p.dOH);
        const int oy = cur.oy0 + Rl - dn * p.OH;
        uint32_t vq = (uint32_t)((((long long)dn * p.F + 4 * kgs) * OHW + oy * p.OW + ox) * 4);
        float *const scr = reinterpret_cast<float *>(lds + p.scr16) + wave8 * 512;
        fa_t *const wr = scr + kgs * 128 + l32s;
        const f4a_t *const rd = reinterpret_cast<const f4a_t *>(scr + kgs * 128 + 4 * ql);
        const long long plane1 = (long long)OHW * 4, plane5 = 5 * plane1;
        asm volatile("" : "+v"(vq));
        const char *ub = reinterpret_cast<const char *>(tile_base);
        // software-pipelined by one stage: stage s+1 is written and read back (behind stage s's reads
        // in the LDS's queue, so nothing is overwritten early) before stage s's values are stored,
        // and a stage's LDS round trip runs under the previous stage's stores
        auto put = [&](int sgi) {
#ifdef XNOR_TS_BUILD
            if (p.dbg & 8) {     // (timing only) the values formed, nothing written
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int j = 0; j < kWN; ++j) { float t = value(j, 2 * sgi + e); asm volatile("" :: "v"(t)); }
                return;
            }
#endif
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int j = 0; j < kWN; ++j) wr[e * 256 + 32 * j] = value(j, 2 * sgi + e);
        };
        auto get = [&](f4_t (&v)[2]) {
#ifdef XNOR_TS_BUILD
            if (p.dbg & 8) { v[0] = f4_t{0, 0, 0, 0}; v[1] = v[0]; return; }
#endif
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const f4a_t va = rd[(e * 256) / 4];
                v[e] = f4_t{va[0], va[1], va[2], va[3]};
            }
        };
        f4_t cur_v[2], nxt_v[2];
        put(0);
        get(cur_v);
#pragma unroll
        for (int sgi = 0; sgi < 8; ++sgi) {
            if (sgi < 7) {
                put(sgi + 1);
                get(nxt_v);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int r = 2 * sgi + e;
#ifdef XNOR_TS_BUILD
                if (p.dbg & 12) { asm volatile("" :: "v"(cur_v[e])); } else   // (timing only) no global store
#endif
                *(ptr4_t)(ub + vq) = cur_v[e];
                ub += (r & 3) == 3 ? plane5 : plane1;
            }
            cur_v[0] = nxt_v[0];
            cur_v[1] = nxt_v[1];
        }
    };
    auto store_outputs = [&]() {
#pragma unroll
        for (int i = 0; i < kWM; ++i) {
            if (i > 0 && cur.half >= 0) break;                                // (a half item has one tile per wave)
            const int t32 = tile32_of(cur, i);
            const int ft = t32 * 32;                                         // the tile's first filter (uniform)
            const int nfilt = p.F - ft;                                      // how many of its 32 exist
            const long long tile_el = ((long long)cur.n_first * p.F + ft) * OHW;   // (uniform)
            // the lane's sixteen alphas of this tile: filters 8*(r/4) + 4*kg + r%4
            const float *Al = k_alpha_copy(kitem - 1) + kBandPixels + (t32 - cur.ftile * (2 * kWM)) * 32 + 4 * (fresh_lane() >> 5);
            float al[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) al[r] = Al[8 * (r >> 2) + (r & 3)];
            if (p.quad && nfilt >= 32) {
                if (cur.my_nt > 0 && cur.npix > cur.tile0 * 32)
                    store_filter_tile_quads(p.out + tile_el,
                                        [&](int j, int r) -> float { return acc[i][j][r] * (kvs[j] * al[r]); });
                continue;      // (p.quad is not set when dot is wanted)
            }
            store_filter_tile(p.out + tile_el, nfilt,
                              [&](int j, int r) -> float { return acc[i][j][r] * (kvs[j] * al[r]); });
            if (p.dot)
                store_filter_tile(p.dot + tile_el, nfilt,
                                  [&](int j, int r) -> int32_t { return (int32_t)acc[i][j][r]; });
        }
    };
    // Chained form (the paper's closing proposal, Sec. V): the next layer needs of this output O only
    // sign(O) packed along its channels (= these filters) and the channel mean of |O| (Eq. 10).  Both
    // come straight from the accumulators: lane l holds pixel l%32 of a tile and, in register r,
    // filter 8*(r/4) + 4*(l/32) + r%4, so a lane builds half of a 32-filter word, its partner lane
    // l^32 the other half.  o = float(dot) * (K * alpha) is formed exactly as in the fp32 output, the
    // bit is (o >= 0) and |o| is summed in double; a wave writes the sums over each of its 32-filter
    // tiles (the small kernel that follows adds the parts of all tiles and divides by F).
    auto chain_store = [&]() {
        const int lane_e = fresh_lane();
        const int l32e = lane_e & 31, kge = lane_e >> 5;
        const float *Alc = k_alpha_copy(kitem - 1) + kBandPixels;
        // the lane's sixteen alphas of each of the wave's filter tiles (0 for filters that do not exist)
        float al[kWM][16];
        int t32s[kWM];
#pragma unroll
        for (int i = 0; i < kWM; ++i) {
            t32s[i] = tile32_of(cur, cur.half >= 0 ? 0 : i);
            const float *Alt = Alc + (t32s[i] - cur.ftile * (2 * kWM)) * 32;
#pragma unroll
            for (int r = 0; r < 16; ++r) al[i][r] = Alt[8 * (r >> 2) + 4 * kge + (r & 3)];
        }
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            if (j >= cur.my_nt) break;
            const int q = (cur.tile0 + j) * 32 + l32e;
            const bool valid = q < cur.npix;
            const float kv = kvs[j];
            const long long pix = (long long)cur.R0 * p.OW + q;      // pixels of a band are consecutive
#pragma unroll
            for (int i = 0; i < kWM; ++i) {
                if (i > 0 && cur.half >= 0) break;
                const int t32 = t32s[i];
                uint32_t w = 0;
                // |o| of the lane's 16 filters summed in fp32 (positive terms: within 16 * 2^-24 of
                // their sum), the two half-words' sums added in double
                float asum32 = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * kge + (r & 3);
                    const float o = acc[i][j][r] * (kv * al[i][r]);
                    if (t32 * 32 + row < p.F) {              // bits and sums of filters that exist only
                        w |= (o >= 0.0f ? 1u : 0u) << row;
                        asum32 += fabsf(o);
                    }
                }
                w |= (uint32_t)__shfl_xor((int)w, 32);
                double asum = (double)asum32;
                asum += __shfl_xor(asum, 32);
                if (valid && kge == 0) {
                    if (t32 < p.Cwn) p.Opk[pix * p.Cwn + t32] = w;
                    p.P[pix * (4 * p.f_tiles) + t32] = (float)asum;
                }
            }
        }
    };
    // the outputs of the item in the accumulators, if there is one
    auto finish_item = [&]() {
        if (!pending) return;
        epilogue_begin();
        if constexpr (CHAIN) chain_store();
        else store_outputs();
        XNOR_STAMP_K(kitem - 1, 5);
        pending = false;
    };

    int seq = next_item(slot);
    while (true) {
        if (seq < 0) {           // no further item: the last one's outputs, if any, and out
            finish_item();
            break;
        }
        Item it;
        decode(seq, it);
        XNOR_STAMP_K(kitem, 0);
        const int ftile = it.ftile, R0 = it.R0, npix = it.npix, n_first = it.n_first, oy0 = it.oy0, r0 = it.r0;
        const int tile0 = it.tile0, my_nt = it.my_nt, items = it.items;

        // ---- staging: packed input words of the band's rows -> FP4 in LDS, zeros outside the image ----
        // all offsets into Ipk are taken from the band's first image (32 bits are enough, see the plan)
        const uint32_t *const band_base = p.Ipk + (long long)n_first * p.H * p.W * p.Cw;

        // where item `it` of chunk 0 comes from (word offset from band_base) and goes to
        auto locate = [&](int it, int &dst, bool &live) -> uint32_t {
            const bool in_range = it < items;
            const uint32_t itc = in_range ? (uint32_t)it : 0u;
            const uint32_t slt = fdiv(itc, p.dCHV);
            const int wq = (int)(itc - slt * CHV);
            const uint32_t rowg = fdiv(slt, p.dWp);
            const int col = (int)(slt - rowg * p.Wp);
            int n, iy;
            if ((int)rowg < r0) {
                n = n_first;
                iy = oy0 * p.sh - p.ph + (int)rowg;
            } else {
                const uint32_t tt = rowg - (uint32_t)r0;
                const uint32_t sg = fdiv(tt, p.dRH);
                n = n_first + 1 + (int)sg;
                iy = (int)(tt - sg * p.RHfull) - p.ph;
            }
            const int ix = col - p.pw;
            const int w = wq * VW;
            live = in_range && n < p.N && iy >= 0 && iy < p.H && ix >= 0 && ix < p.W && w < p.Cw;
            dst = in_range ? (int)(slt * p.pitch16 + wq * VW) : -1;
            return live ? (uint32_t)((((n - n_first) * p.H + iy) * p.W + ix) * p.Cw + w) : 0u;
        };
        // one item's words -> FP4 at byte offset `dst_b` of the group's region; a dead item is FP4
        // zeros (outside the image, or past the last channel word, the +-1 tensor is 0.0, not -1.0)
        auto put = [&](uint32_t dst_b, bool live, const wvec &v) {
            uint32_t words[VW];
            if constexpr (VW == 1) { words[0] = v; }
            if constexpr (VW == 2) { words[0] = v.x; words[1] = v.y; }
            if constexpr (VW == 4) { words[0] = v.x; words[1] = v.y; words[2] = v.z; words[3] = v.w; }
            uint4 *dst = reinterpret_cast<uint4 *>(lds_bytes + dst_b);
            if (live) {
#pragma unroll
                for (int k = 0; k < VW; ++k) dst[k] = expand_word(words[k], 32);
            } else {
#pragma unroll
                for (int k = 0; k < VW; ++k) dst[k] = make_uint4(0, 0, 0, 0);
            }
        };
        // A thread's first UP items: fetched here (ordinary loads: nothing of the MFMA loop is in
        // flight), expanded further down.  The same slots hold the thread's items of every later
        // chunk, a chunk only shifts the source by its first word: the loop takes the byte offset of
        // the words in chunk 0 and the LDS address of the slot in the first chunk buffer (a slot
        // outside every image, or no such item: offset 0 and the group's dump slot; such slots hold
        // zeros from the item's first fill and the loop must not write them).
        wvec sv[UP];
        uint32_t soff[UP], sdst[UP];
        int sdst_b[UP];
        bool slive[UP];
        const int tid_a = wave * 64 + fresh_lane();   // the thread within its group
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            const int itn = u * kGroupThreads + tid_a;
            int dst;
            bool live0;
            const uint32_t off = locate(itn, dst, live0);
            slive[u] = live0;
            soff[u] = live0 ? off * 4u : 0u;
            sdst_b[u] = dst < 0 ? -1 : dst * 16;
            sdst[u] = glds_base + (live0 ? (uint32_t)dst * 16u : (uint32_t)p.dump16 * 16u);
            wvec z = {};
            sv[u] = live0 ? *reinterpret_cast<const wvec *>(reinterpret_cast<const char *>(band_base) + off * 4u) : z;
        }
        // K of this band's pixel `tid`: given, or from the channel mean A with the same sum, order and
        // rounding as the stand-alone box filter (double accumulation over the in-image taps, one
        // divide).  No branches around the loads (out-of-image taps read a clamped address and add
        // 0), so that the unrolled loop has all its loads in flight at once.
        float k_mine = 0.0f, a_mine = 0.0f;
        if (tid_a < npix) {
            if (p.A) {
                const int Rl = (int)fdiv((uint32_t)tid_a, p.dOW), ox = tid_a - Rl * p.OW;
                const int dn = (int)fdiv((uint32_t)(oy0 + Rl), p.dOH);
                const int n = n_first + dn, oy = oy0 + Rl - dn * p.OH;
                const float *a = p.A + (long long)n * p.H * p.W;
                double sum = 0.0;
                const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
                int ky = 0, kx = 0;
#pragma unroll 9
                for (int t = 0; t < taps; ++t) {
                    const int iy = iy0 + ky, ix = ix0 + kx;
                    const bool in = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
                    const float v = a[in ? iy * p.W + ix : 0];
                    sum += in ? (double)v : 0.0;
                    if (++kx == p.kw) { kx = 0; ++ky; }
                }
                k_mine = (float)(sum / (double)taps);
            } else {
                k_mine = p.K[(long long)R0 * p.OW + tid_a];
            }
        }
        if (tid_a < kFilterTile && ftile * kFilterTile + tid_a < p.F) a_mine = p.alpha[ftile * kFilterTile + tid_a];
        asm volatile("" ::: "memory");
        XNOR_STAMP_K(kitem, 6);
        // the previous item's outputs: stored here, behind the loads just issued (a load issued
        // behind the stores would wait in the same queue until they have drained)
        finish_item();

        uint32_t bB[kWN];   // LDS byte address of the lane's pixel, tap (0,0), k-group kg
        const int lane_b2 = fresh_lane();
        const int l32 = lane_b2 & 31, kg = lane_b2 >> 5;
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            const int q = (tile0 + j) * 32 + l32;
            const int qq = (j < my_nt && q < npix) ? q : 0;   // idle lanes read pixel 0 and store nothing
            const int Rl = (int)fdiv((uint32_t)qq, p.dOW), ox = qq - Rl * p.OW;
            const int dn = (int)fdiv((uint32_t)(oy0 + Rl), p.dOH);
            const int n = n_first + dn, oy = oy0 + Rl - dn * p.OH;
            const int srow = (n == n_first) ? (oy - oy0) * p.sh
                                            : r0 + (n - n_first - 1) * p.RHfull + oy * p.sh;
            bB[j] = glds_base + (uint32_t)((srow * p.Wp + ox * p.sw) * p.pitch16 + kg) * 16u;
        }
        const uint4 *Abase[kWM];   // filter operands of this wave's tiles, step 0 (wave-uniform)
#pragma unroll
        for (int i = 0; i < kWM; ++i) {
            const int tile = __builtin_amdgcn_readfirstlane(tile32_of(it, it.half < 0 ? i : 0));   // (a half item: one tile, loaded twice)
            Abase[i] = p.Wx + ((long long)tile * p.tile_steps) * 64;
        }
        asm volatile("" ::: "memory");

        asm volatile("" ::: "memory");
        XNOR_STAMP_K(kitem, 7);

        // every wave of the group has left the previous item's contraction: its buffers are free
        const uint32_t cbase = (uint32_t)(4 * p.nchunks * kitem);   // both counters at this item's start
        if (kitem > 0) wait_count(done_addr, cbase);
        XNOR_STAMP_K(kitem, 1);
        // chunk 0 into the first buffer, every slot (zeros where the image ends); where there is a
        // second buffer its slots outside the image are zeroed once per item, no chunk writes them
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            if (sdst_b[u] < 0) continue;
            const bool live = slive[u];
            put((uint32_t)sdst_b[u], live, sv[u]);
            if (p.nchunks > 1 && !live) put((uint32_t)p.buf16 * 16u + (uint32_t)sdst_b[u], false, sv[u]);
        }
        const int lane_d = fresh_lane();
        const int tid_d = wave * 64 + lane_d;
        for (int itn = UP * kGroupThreads + tid_d; itn < items; itn += kGroupThreads) {   // (single-chunk layers only)
            int dst;
            bool live;
            const uint32_t off = locate(itn, dst, live);
            wvec z = {};
            const wvec v = live ? *reinterpret_cast<const wvec *>(reinterpret_cast<const char *>(band_base) + off * 4u) : z;
            put((uint32_t)dst * 16u, live, v);
        }
        // the band's K values and this group's 128 alphas go to LDS for the item's last phase (two
        // copies, taken in turn: waves may still be reading the previous item's)
        {
            float *const Kl = k_alpha_copy(kitem);
            Kl[tid_d] = k_mine;
            if (tid_d < kFilterTile) Kl[kBandPixels + tid_d] = a_mine;
        }
        count_up(ready_addr, lane_d);
        XNOR_STAMP_K(kitem, 2);

        // ---- the item becomes the current one ----
        cur = it;
        XNOR_STAMP_K(kitem, 3);

        // ---- contract ----
        {
            uint32_t a_off = (uint32_t)fresh_lane() * 16u;   // byte offset of this lane's filter operand, step 0
            uint32_t tab_addr = tab_base;
            int gi, hc, t1, t2, t3, st, st2, sp, tg, ev, pv;
            unsigned long long sx;
            asm volatile(PX_LOOP_ASM
                         : [acc00] "=&v"(acc[0][0]), [acc01] "=&v"(acc[0][1]), [acc02] "=&v"(acc[0][2]),
                           [acc03] "=&v"(acc[0][3]), [acc10] "=&v"(acc[1][0]), [acc11] "=&v"(acc[1][1]),
                           [acc12] "=&v"(acc[1][2]), [acc13] "=&v"(acc[1][3]), [aoff] "+v"(a_off),
                           [tab] "+v"(tab_addr), [sturn] "+s"(sturn), [gi] "=&s"(gi), [hc] "=&s"(hc),
                           [t1] "=&s"(t1), [t2] "=&s"(t2), [t3] "=&s"(t3), [st] "=&s"(st), [st2] "=&s"(st2),
                           [sp] "=&s"(sp), [tg] "=&s"(tg), [sx] "=&s"(sx), [ev] "=&s"(ev), [pv] "=&s"(pv)
                         : [bB0] "v"(bB[0]), [bB1] "v"(bB[1]), [bB2] "v"(bB[2]), [bB3] "v"(bB[3]),
                           [soff0] "v"(soff[0]), [soff1] "v"(soff[1]), [sdst0] "v"(sdst[0]), [sdst1] "v"(sdst[1]),
                           [ready] "v"(ready_addr), [done] "v"(done_addr), [start] "v"(start_addr),
                           [Ab0] "s"(Abase[0]), [Ab1] "s"(Abase[1]), [band] "s"(band_base),
                           [nturns] "s"(p.nturns), [nchunks] "s"(p.nchunks), [csteps] "s"(p.chunk_steps),
                           [cbase] "s"(cbase), [csrc] "s"(p.CH * 4), [bufb] "s"(p.buf16 * 16),
                           [pmask] "s"(grp == 1 ? p.prio_mask : 0), [onetile] "s"(__builtin_amdgcn_readfirstlane(it.half < 0 ? 0 : 1)),
                           [m03] "s"(0x03030303u), [tbl] "s"(0x222AA2AAu)
                         : "memory", "vcc", "scc",
                           "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", "v176", "v177", "v178",
                           "v179", "v180", "v181", "v182", "v183", "v184", "v185", "v186", "v187", "v188", "v189",
                           "v190", "v191", "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", "v200",
                           "v201", "v202", "v203", "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211",
                           "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", "v220", "v221", "v222",
                           "v223", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", "v233",
                           "v234", "v235", "v236", "v237", "v238", "v239", "v240", "v241", "v242", "v243", "v244",
                           "v245", "v246", "v247", "v248", "v249", "v250", "v251", "v252", "v253", "v254", "v255");
        }
        XNOR_STAMP_K(kitem, 4);
#ifdef XNOR_TS_BUILD
        pending = !(p.dbg & 1);
#else
        pending = true;
#endif
        ++kitem;
        seq = next_item(seq + nslot);
    }
    // a first group that never reached the releasing turn (no items, or too few turns) lets go now
    if (grp == 0 && sturn != -1) count_up(start_addr, fresh_lane());
}

// Tiling chosen on the host for one layer.
struct PPlan {
    bool ok;
    int TH, Wp, RHfull, S2, CH, nchunks, pitch16, buf16, ka16, dump16, grp16, shared16, tab_len, vw;
    int chunk_steps, T, nturns, tile_steps, f_tiles;
    int scr16;       // start of the waves' store scratch (16-byte units), 0 if the LDS has no room for it
    size_t lds_bytes, ws_bytes;
};

PPlan make_pplan(const Geom &g, const void *Ipk)
{
    PPlan pl{};
    pl.ok = false;
    if (g.OW > kBandPixels) return pl;   // a band is at least one whole output row
    const long long total_rows = (long long)g.N * g.OH;
    pl.TH = (int)std::min<long long>(total_rows, kBandPixels / g.OW);
    const long long wp = (long long)(g.OW - 1) * g.sw + g.kw, rh = (long long)(g.OH - 1) * g.sh + g.kh;
    if (wp > 4096 || rh > 4096) return pl;   // keeps the staging index math inside the fast-division range
    pl.Wp = (int)wp;
    pl.RHfull = (int)rh;
    const int Cw2 = (g.Cw + 1) & ~1;
    pl.S2 = Cw2 / 2;
    // most staged rows any band can need: try every starting row of an image
    long long max_rows = 0;
    for (int oy0 = 0; oy0 < g.OH; ++oy0) {
        const long long r0 = (long long)(g.OH - 1 - oy0) * g.sh + g.kh;
        const long long last = (long long)oy0 + std::min<long long>(pl.TH, total_rows) - 1;
        const long long n_last = last / g.OH, oy_last = last % g.OH;
        const long long sr = n_last == 0 ? (oy_last - oy0) * g.sh + g.kh
                                         : r0 + (n_last - 1) * rh + oy_last * g.sh + g.kh;
        max_rows = std::max(max_rows, sr);
    }
    const long long slots = max_rows * wp;
    if (slots > (1 << 16)) return pl;
    const int taps = g.kh * g.kw;
    // Channel chunks: one chunk in one buffer if the whole band fits a group's half of the LDS,
    // else the fewest chunks whose two buffers fit.  A chunk that is handed over inside the loop
    // must span three ring turns (fetch, expand, look).
    bool found = false;
    for (int nch = 1; nch <= pl.S2 && !found; ++nch) {
        const int CH = 2 * ((pl.S2 + nch - 1) / nch);
        const int nchunks = (Cw2 + CH - 1) / CH;
        const size_t one = (size_t)slots * (CH + 1) * 16;
        const int chunk_steps = taps * (CH / 2);
        const int T = (nchunks - 1) * chunk_steps + taps * ((Cw2 - (nchunks - 1) * CH) / 2);
        const int nturns = (T + kRing - 1) / kRing;
        const int tab_len = kRing * nturns + kRing;
        const size_t shared = (((size_t)kCtrWords + tab_len) * sizeof(uint32_t) + 15) & ~(size_t)15;
        // a chunk buffer is followed by a 64-byte dump slot: the loop's staging writes the (unused)
        // expansion of a thread without a live item there, at the same offset in either buffer
        const size_t data = nchunks > 1 ? 2 * (one + 64) : one;
        const size_t group = data + 2 * kKAlphaBytes;
        if (2 * group + shared > kLdsMax) continue;
        if (nchunks > 1 && chunk_steps < 3 * kRing) return pl;   // (more chunks would only be shorter)
        pl.CH = CH;
        pl.nchunks = nchunks;
        pl.pitch16 = CH + 1;
        pl.buf16 = nchunks > 1 ? (int)((one + 64) / 16) : 0;
        pl.ka16 = (int)(data / 16);
        pl.dump16 = (int)(one / 16);
        pl.grp16 = (int)(group / 16);
        pl.shared16 = 2 * pl.grp16;
        pl.tab_len = tab_len;
        pl.chunk_steps = chunk_steps;
        pl.T = T;
        pl.nturns = nturns;
        pl.lds_bytes = 2 * group + shared;
        // 2 KB per wave for the 16-byte output stores, where there is room
        pl.scr16 = 0;
        if (pl.lds_bytes + 8 * 2048 <= kLdsMax) {
            pl.scr16 = (int)(pl.lds_bytes / 16);
            pl.lds_bytes += 8 * 2048;
        }
        found = true;
    }
    if (!found) return pl;
    if ((long long)slots * pl.CH >= (1 << 20)) return pl;   // fast-division range
    if (((long long)slots * pl.pitch16 + pl.pitch16) * 16 >= (1 << 18)) return pl;   // 18-bit LDS offsets
    // staging addresses are 32-bit byte offsets from the band's first image
    if ((long long)(pl.TH / g.OH + 2) * g.H * g.W * g.Cw >= (1LL << 30)) return pl;
    const uintptr_t ip = reinterpret_cast<uintptr_t>(Ipk);
    pl.vw = (g.Cw % 4 == 0 && pl.CH % 4 == 0 && (ip & 15) == 0) ? 4
          : (g.Cw % 2 == 0 && (ip & 7) == 0)                    ? 2 : 1;
    if (pl.nchunks > 1) {
        // what the loop's own staging takes: whole chunks of 16-byte items, at most two per thread
        // (16-byte loads from addresses that are only 4-byte aligned are fine on this target)
        if (g.Cw % pl.CH != 0 || pl.CH % 4 != 0 || slots * (pl.CH / 4) > 2 * kGroupThreads) return pl;
        pl.vw = 4;
    }
    pl.f_tiles = ceil_div(g.F, kFilterTile);
    // the workspace holds the steps of a tile in loop order, then zero steps up to a whole ring and
    // one more ring (the filter-operand loads run three steps ahead of the last step)
    pl.tile_steps = kRing * pl.nturns + kRing;
    pl.ws_bytes = (size_t)pl.f_tiles * (kFilterTile / 32) * pl.tile_steps * 64 * sizeof(uint4);
    if ((ceil_div(total_rows, pl.TH) + 8) * (long long)pl.f_tiles > (1LL << 30)) return pl;
    pl.ok = true;
    return pl;
}

int compute_units(int dev)
{
    static std::atomic<int> cached[64];
    if (dev < 0 || dev >= 64) return 256;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cached[dev].store(v, std::memory_order_relaxed);
    return v;
}

template <int VW, bool CHAIN>
hipError_t raise_lds_once(int dev)
{
    // raise the kernel's dynamic-LDS limit to the hardware maximum once per device and kernel (the
    // call is slow on the host)
    static std::atomic<unsigned long long> raised{0};
    const unsigned long long bit = 1ull << (dev & 63);
    if (raised.load(std::memory_order_acquire) & bit) return hipSuccess;
    const hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(conv_mfma_persistent_kernel<VW, CHAIN>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
    if (err == hipSuccess) raised.fetch_or(bit, std::memory_order_release);
    return err;
}

template <int VW, bool CHAIN>
hipError_t launch_one(const PParams &p, int dev, unsigned grid, size_t lds_bytes, hipStream_t st)
{
    const hipError_t err = raise_lds_once<VW, CHAIN>(dev);
    if (err != hipSuccess) return err;
    conv_mfma_persistent_kernel<VW, CHAIN><<<dim3(grid), dim3(512), lds_bytes, st>>>(p);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_persistent_supports(const Geom &g)
{
    return make_pplan(g, nullptr).ok;
}

bool conv_mfma_persistent_preferred(const Geom &g)
{
    // Items come in rounds of one per wave group (two groups per compute unit).  Up to one round the
    // kernel's length is that of one (half) item; from three rounds on the uneven last round is a
    // small part of the whole.  In between (measured at 1.5 rounds) one workgroup per band, handed
    // out by the hardware as compute units fall free, ends sooner.
    const PPlan pl = make_pplan(g, nullptr);
    if (!pl.ok) return false;
    int dev = 0;
    const int cus = hipGetDevice(&dev) == hipSuccess ? compute_units(dev) : 256;
    const long long bands = ceil_div((long long)g.N * g.OH, pl.TH);
    const long long items_per_xcd = ceil_div(bands, kXcds) * pl.f_tiles;
    const long long nslot = 2LL * std::max(1, cus / kXcds);
    return items_per_xcd <= nslot || items_per_xcd >= 3 * nslot;
}

ExpandLayout conv_mfma_persistent_expand_layout(const Geom &g)
{
    const PPlan pl = make_pplan(g, nullptr);   // the workspace layout does not depend on alignment
    ExpandLayout L{};
    L.ok = pl.ok ? 1 : 0;
    L.CH = pl.CH; L.nchunks = pl.nchunks; L.chunk_pad = pl.chunk_steps; L.tile_steps = pl.tile_steps;
    L.Cw2 = 2 * pl.S2; L.ws_bytes = pl.ws_bytes;
    return L;
}

int conv_mfma_persistent_sum_parts(const Geom &g)
{
    const PPlan pl = make_pplan(g, nullptr);
    return pl.ok ? 4 * pl.f_tiles : 0;
}

hipError_t launch_conv_mfma_persistent(const uint32_t *Ipk, const float *K, const float *A, const float *alpha,
                                       const Geom &g, float *out, int32_t *dot, uint32_t *Opk, float *P,
                                       const void *workspace, hipStream_t st)
{
    const PPlan pl = make_pplan(g, Ipk);
    if (!pl.ok) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;

    PParams p{};
    p.Ipk = Ipk; p.Wx = static_cast<const uint4 *>(workspace); p.K = K; p.A = A; p.alpha = alpha;
    p.out = out; p.dot = dot; p.Opk = Opk; p.P = P; p.Cwn = (g.F + 31) / 32; p.f_tiles = pl.f_tiles;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.TH = pl.TH;
    p.total_rows = g.N * g.OH;
    p.Wp = pl.Wp; p.RHfull = pl.RHfull; p.S2 = pl.S2; p.CH = pl.CH; p.nchunks = pl.nchunks;
    p.pitch16 = pl.pitch16; p.buf16 = pl.buf16; p.ka16 = pl.ka16; p.dump16 = pl.dump16; p.grp16 = pl.grp16;
    p.shared16 = pl.shared16; p.tab_len = pl.tab_len; p.chunk_steps = pl.chunk_steps; p.nturns = pl.nturns;
    p.ragged = g.Cw % pl.CH != 0;
    // a band touches at most TH/OH + 2 images; a lane's offset also spans the tile's 32 planes
    p.near_out = ((long long)(pl.TH / g.OH + 2) * g.F + 32) * g.OH * g.OW * 4 < (1LL << 31);
    p.tile_steps = pl.tile_steps;
    // 16-byte output stores: four consecutive pixels of the batch's (n, oy, ox) order must be four
    // consecutive, 16-byte aligned floats of one plane: images and bands are whole quads
    p.scr16 = pl.scr16;
    p.quad = pl.scr16 > 0 && p.near_out && !dot && !Opk && out &&
             (reinterpret_cast<uintptr_t>(out) & 15) == 0 &&
             ((long long)g.OH * g.OW) % 4 == 0 && ((long long)pl.TH * g.OW) % 4 == 0;
    p.dCHV = make_fastdiv(pl.CH / pl.vw);
    p.dWp = make_fastdiv(pl.Wp);
    p.dRH = make_fastdiv(pl.RHfull);
    p.dOW = make_fastdiv(g.OW);
    p.dOH = make_fastdiv(g.OH);
    p.nbands = ceil_div(p.total_rows, pl.TH);
    p.bands_per_xcd = ceil_div(p.nbands, kXcds);
    p.items_per_xcd = p.bands_per_xcd * pl.f_tiles;
    p.stagger = 0;
    // One workgroup per compute unit, two groups each: 2 * CUs slots per XCD.
    const int cus_per_xcd = std::max(1, compute_units(dev) / kXcds);
    if (p.items_per_xcd < 2 * cus_per_xcd) {
        // A layer that does not give every group an item: as many items as the slots allow go out
        // as two half items, spread over the compute units first and over their second groups
        // after that, and all groups start at once (the kernel's length is that of one unit).
        p.whole_items = std::max(0, 2 * p.items_per_xcd - 2 * cus_per_xcd);
        p.work_per_xcd = p.whole_items + 2 * (p.items_per_xcd - p.whole_items);
        p.wgs_per_xcd = std::min(cus_per_xcd, p.work_per_xcd);
        p.start_turn = -1;
        // (all groups store at once at the end and no matrix loop runs beside the stores: the
        //  one-pixel stores are as fast there, without the pass through the LDS)
        p.quad = 0;
    } else {
        // Several rounds: the items beyond the last whole round go out as half items when that
        // spreads them over more groups (the kernel's length is that of its busiest compute
        // unit), and the second groups start half an item late, so that one group's epilogue
        // and set-up fall into the other's matrix loop.
        p.wgs_per_xcd = cus_per_xcd;
        const int nslot = 2 * p.wgs_per_xcd, rem = p.items_per_xcd % nslot;
        p.whole_items = (rem > 0 && 2 * rem <= nslot) ? p.items_per_xcd - rem : p.items_per_xcd;
        p.work_per_xcd = p.whole_items + 2 * (p.items_per_xcd - p.whole_items);
        p.start_turn = pl.nturns / 2;
        // (an item's time is about 2.5 times its matrix instructions': 8 x 32 cycles per step; the
        //  late workgroups have the time: they are the ones without a half item at the end)
        if (p.whole_items < p.items_per_xcd && p.work_per_xcd - p.whole_items <= p.wgs_per_xcd)
            p.stagger = (int)(0.625 * pl.nturns * 4 * 256 / 1024);
    }
    p.prio_mask = 7;
#ifdef XNOR_TS_BUILD
    {
        const char *e = getenv("XNOR_TS");
        p.ts = e ? reinterpret_cast<unsigned long long *>(strtoull(e, nullptr, 0)) : nullptr;
        const char *d = getenv("XNOR_DBG");
        p.dbg = d ? atoi(d) : 0;
        const char *st = getenv("XNOR_START_TURN");
        if (st) p.start_turn = atoi(st);
        const char *pm = getenv("XNOR_PMASK");
        if (pm) p.prio_mask = atoi(pm);
        const char *sg = getenv("XNOR_STAGGER");
        if (sg) p.stagger = atoi(sg);
        const char *qd = getenv("XNOR_NOQUAD");
        if (qd && atoi(qd)) p.quad = 0;
        const char *wg = getenv("XNOR_WGS");
        if (wg) p.wgs_per_xcd = std::min(p.wgs_per_xcd, atoi(wg));
    }
#endif
    const unsigned grid = (unsigned)(kXcds * p.wgs_per_xcd);

    if (Opk) {
        switch (pl.vw) {
            case 4: return launch_one<4, true>(p, dev, grid, pl.lds_bytes, st);
            case 2: return launch_one<2, true>(p, dev, grid, pl.lds_bytes, st);
            default: return launch_one<1, true>(p, dev, grid, pl.lds_bytes, st);
        }
    }
    switch (pl.vw) {
        case 4: return launch_one<4, false>(p, dev, grid, pl.lds_bytes, st);
        case 2: return launch_one<2, false>(p, dev, grid, pl.lds_bytes, st);
        default: return launch_one<1, false>(p, dev, grid, pl.lds_bytes, st);
    }
}

}  // namespace xnor
