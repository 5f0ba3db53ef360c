// The chained stage schedule of the 256-row GEMM tiles, as data.
//
// The kernel (gemm4_tile in mom_gemm.hip.inc, stage_c) asks these functions what to do behind each
// MFMA; a host program (tests/stage_schedule_check.cpp, run by the CPU tests) walks the same
// functions over many stages and checks what no compiler checks: every index in range, every
// fragment read behind a barrier that covers the loads of its data, every ring slot overwritten only
// behind a barrier that follows its last read, every MFMA operand register holding the fragment of
// the stage being multiplied.  Plain C++17, no HIP types.
//
// Vocabulary.  A stage is 64 K-elements of both operand tiles.  Ring entry 2T is the token tile of
// stage T, entry 2T+1 its weight tile; entry e lives in LDS slot e % 5.  P = 2T % 5 is the slot of
// the token tile of the stage being multiplied, and slots below are relative to P (mod 5).
// Stage T is MB rows (one per 16-row token block mb) of NB MFMA pairs (one per 16-row weight block
// nb: K-half 0, then K-half 1 into the same accumulator block).  Position A of a pair is between
// its two MFMAs, position B behind the second.  A wavefront moves MB 1-KiB blocks of a token tile
// and WL <= MB of a weight tile ("index" below).
#ifndef MOM_GEMM_SCHEDULE_H
#define MOM_GEMM_SCHEDULE_H

#if defined(__HIPCC__)
#define MOM_SCHED_FN __host__ __device__ constexpr
#else
#define MOM_SCHED_FN constexpr
#endif

namespace momk {
namespace chain {

constexpr int kSlots = 5;
enum Operand { NONE = 0, TOK = 1, WGT = 2 };

struct FragRead {     // LDS -> fragment register
    int operand;      // NONE: nothing at this position
    int khalf;        // 0, 1
    int block;        // mb (TOK) or nb (WGT)
    int ahead;        // the data belongs to stage T + ahead
    int slot;         // ring slot relative to P
};
struct RingLoad {     // global -> LDS
    int operand;
    int index;        // which of the wavefront's 1-KiB blocks of the tile
    int ahead;
    int slot;
};

// The stage barrier (s_waitcnt for the own ring loads and LDS reads, then s_barrier) sits in front of this row.
MOM_SCHED_FN int barrier_row() { return 1; }
// ... and lets this many of the youngest ring loads of the wavefront stay in flight.
MOM_SCHED_FN int barrier_loads_in_flight(int MB) { return MB; }
// Behind the barrier the weight pointers move to stage T + 2; in front of this row the token pointer moves to T + 3.
MOM_SCHED_FN int weight_pointer_ahead() { return 2; }
MOM_SCHED_FN int token_pointer_row(int MB) { return MB - 3; }
MOM_SCHED_FN int token_pointer_ahead() { return 3; }

// Position A of pair (mb, 0): the two token fragments (K-half `khalf`) that row mb - 1 has just freed take
// block mb - 1 of stage T + 1; row 0 takes the last block of stage T itself.
MOM_SCHED_FN FragRead token_read(int MB, int mb, int nb, int khalf) {
    if (nb != 0) return {NONE, 0, 0, 0, 0};
    if (mb == 0) return {TOK, khalf, MB - 1, 0, 0};
    return {TOK, khalf, mb - 1, 1, 2};
}

// Position A of pair (mb, nb): the 2 NB weight fragments of stage T + 1 (into the other fragment buffer) over
// rows 1 .. MB-1, three per row in rows 1 and 2, two per row later, behind the first MFMAs of pairs 1, 2 (, 3).
MOM_SCHED_FN FragRead weight_read(int NB, int mb, int nb) {
    if (mb < 1) return {NONE, 0, 0, 0, 0};
    const int first = (mb <= 2) ? 3 * (mb - 1) : 6 + 2 * (mb - 3);
    const int count = (mb <= 2) ? 3 : 2;
    const int k = nb - 1;
    if (k < 0 || k >= count) return {NONE, 0, 0, 0, 0};
    const int q = first + k;                 // q-th weight fragment: K-half q % 2 of block q / 2
    if ((q >> 1) >= NB) return {NONE, 0, 0, 0, 0};
    return {WGT, q & 1, q >> 1, 1, 3};
}

// Position B of pair (mb, nb): two ring loads per row.  Row 0: the last two token loads of stage T + 2 (slot P+4);
// rows 1 .. MB/2: the weights of stage T + 2 into slot P (the token tile of stage T, free since the barrier);
// the rows behind: all but the last two token loads of stage T + 3 into slot P+1 (the weight tile of stage T).
MOM_SCHED_FN RingLoad ring_load(int MB, int NB, int mb, int nb) {
    const int first = NB / 4, second = NB / 4 + NB / 2;
    if (nb != first && nb != second) return {NONE, 0, 0, 0};
    const int h = (nb == second);
    if (mb == 0) return {TOK, MB - 2 + h, 2, 4};
    if (mb <= MB / 2) return {WGT, 2 * (mb - 1) + h, 2, 0};
    return {TOK, 2 * (mb - MB / 2 - 1) + h, 3, 1};
}

// Prologue: loads of whole tiles in this order, then all but the last two token loads of stage 2; the wait that
// follows lets the loads behind stage 0 stay in flight.  Then stage 0 goes into registers but for the last
// token block (which every stage reads in its row 0).
struct PrologueTile { int operand, stage, slot, count; };
MOM_SCHED_FN PrologueTile prologue_tile(int MB, int WL, int i) {
    return i == 0 ? PrologueTile{TOK, 0, 0, MB} : i == 1 ? PrologueTile{WGT, 0, 1, WL} : i == 2 ? PrologueTile{TOK, 1, 2, MB}
         : i == 3 ? PrologueTile{WGT, 1, 3, WL} : PrologueTile{TOK, 2, 4, MB - 2};
}
MOM_SCHED_FN int prologue_tiles() { return 5; }
MOM_SCHED_FN int prologue_loads_in_flight(int MB, int WL) { return MB + WL + MB - 2; }
MOM_SCHED_FN bool prologue_reads_token_block(int MB, int mb) { return mb < MB - 1; }

}  // namespace chain
}  // namespace momk

#endif  // MOM_GEMM_SCHEDULE_H
