// Host-side check of the chained stage schedule of the 256-row GEMM tiles.
//
// Walks the very functions the kernel asks (paper_2504_12526_amd/csrc/mom_gemm_schedule.h) over a prologue
// and many stages, as one wavefront would execute them, and checks what the kernel relies on:
//   1. every ring load index is one of the wavefront's blocks and every tile's loads are issued exactly
//      once, into the slot its ring entry lives in, with the operand pointer standing at the tile's stage;
//   2. a fragment is read from LDS only behind a barrier whose s_waitcnt covered every load of its tile
//      (ring loads complete in order; the wait lets the youngest N stay in flight);
//   3. a ring slot is overwritten only behind a barrier that follows the last read of its previous tile;
//   4. at every MFMA both operand registers hold fragments of the stage being multiplied
//      (a register is never refilled before its last use, never used before it is refilled).
// Exit status 0 and one "ok" line per tile width, else a message and status 1.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <tuple>
#include <vector>

#include "mom_gemm_schedule.h"

namespace ch = momk::chain;

struct Load { int seq, operand, index, stage, slot; double time; };
struct Read { double time; int operand, khalf, block, slot, stage, buffer; };
struct Use { double time; int operand, khalf, block, buffer, stage; };

static int fail(const char* what, int NB, int a = 0, int b = 0, int c = 0) {
    std::printf("NB=%d: %s (%d, %d, %d)\n", NB, what, a, b, c);
    return 1;
}

static int check(int MB, int NB, int WL, int stages) {
    const int NS = ch::kSlots;
    std::vector<Load> loads;
    std::vector<Read> reads;
    std::vector<Use> uses;
    std::map<int, double> barrier_time;            // barrier id (-1 = prologue, T = barrier of stage T) -> time
    std::map<int, int> landed_upto;                // barrier id -> loads with seq < this have landed
    int tok_ptr = 0, wgt_ptr = 0;                  // the stage the operand pointers stand at
    auto issue = [&](int operand, int index, int stage, int slot, double t) -> int {
        if (index < 0 || index >= MB) return fail("ring load index out of range", NB, operand, index, (int)t);
        if (operand == ch::WGT && index >= WL) return 0;              // a narrow weight tile has fewer blocks
        const int ptr = operand == ch::TOK ? tok_ptr : wgt_ptr;
        if (ptr != stage) return fail("operand pointer stands at another stage than the load's tile", NB, operand, ptr, stage);
        loads.push_back({(int)loads.size(), operand, index, stage, slot, t});
        return 0;
    };
    // ---- prologue
    for (int i = 0; i < ch::prologue_tiles(); ++i) {
        const ch::PrologueTile pt = ch::prologue_tile(MB, WL, i);
        tok_ptr = wgt_ptr = pt.stage;
        for (int k = 0; k < MB; ++k)
            if (k < pt.count && issue(pt.operand, k, pt.stage, pt.slot, -10 + i)) return 1;
    }
    barrier_time[-1] = -5;
    landed_upto[-1] = (int)loads.size() - ch::prologue_loads_in_flight(MB, WL);
    for (int nb = 0; nb < NB; ++nb)
        for (int kh = 0; kh < 2; ++kh) reads.push_back({-4, ch::WGT, kh, nb, 1, 0, 0});
    for (int mb = 0; mb < MB; ++mb)
        if (ch::prologue_reads_token_block(MB, mb))
            for (int kh = 0; kh < 2; ++kh) reads.push_back({-4, ch::TOK, kh, mb, 0, 0, -1});
    // ---- stages
    auto when = [&](int T, int mb, int nb, int sub) { return (double)(((T * MB + mb) * NB + nb) * 4 + sub); };
    for (int T = 0; T < stages; ++T) {
        const int P = (2 * T) % NS, B = T % 2;
        for (int mb = 0; mb < MB; ++mb) {
            if (mb == ch::barrier_row()) {
                barrier_time[T] = when(T, mb, 0, 0) - 0.5;
                landed_upto[T] = (int)loads.size() - ch::barrier_loads_in_flight(MB);
                wgt_ptr = T + ch::weight_pointer_ahead();
            }
            if (mb == ch::token_pointer_row(MB)) tok_ptr = T + ch::token_pointer_ahead();
            for (int nb = 0; nb < NB; ++nb) {
                uses.push_back({when(T, mb, nb, 0), ch::WGT, 0, nb, B, T});
                uses.push_back({when(T, mb, nb, 0), ch::TOK, 0, mb, -1, T});
                for (int kh = 0; kh < 2; ++kh) {
                    const ch::FragRead f = ch::token_read(MB, mb, nb, kh);
                    if (f.operand == ch::TOK) {
                        if (f.block < 0 || f.block >= MB) return fail("token fragment block out of range", NB, f.block);
                        reads.push_back({when(T, mb, nb, 1), ch::TOK, f.khalf, f.block, (P + f.slot) % NS, T + f.ahead, -1});
                    }
                }
                const ch::FragRead f = ch::weight_read(NB, mb, nb);
                if (f.operand == ch::WGT) {
                    if (f.block < 0 || f.block >= NB) return fail("weight fragment block out of range", NB, f.block);
                    reads.push_back({when(T, mb, nb, 1), ch::WGT, f.khalf, f.block, (P + f.slot) % NS, T + f.ahead, B ^ 1});
                }
                uses.push_back({when(T, mb, nb, 2), ch::WGT, 1, nb, B, T});
                uses.push_back({when(T, mb, nb, 2), ch::TOK, 1, mb, -1, T});
                const ch::RingLoad l = ch::ring_load(MB, NB, mb, nb);
                if (l.operand != ch::NONE && issue(l.operand, l.index, T + l.ahead, (P + l.slot) % NS, when(T, mb, nb, 3))) return 1;
            }
        }
    }
    const int checked = stages - 4;               // the last stages' successors were never completed
    // 1. every tile: its loads once each, in the slot of its ring entry
    for (int T = 0; T < checked; ++T)
        for (int operand : {ch::TOK, ch::WGT}) {
            const int n = operand == ch::TOK ? MB : WL, slot = (2 * T + (operand == ch::WGT)) % NS;
            std::vector<int> seen(n, 0);
            for (const Load& l : loads)
                if (l.operand == operand && l.stage == T) {
                    if (l.slot != slot) return fail("ring load into the wrong slot", NB, T, l.slot, slot);
                    ++seen[l.index];
                }
            for (int i = 0; i < n; ++i)
                if (seen[i] != 1) return fail("tile load issued 0 or 2 times", NB, T, operand, i);
        }
    auto barrier_before = [&](double t) {
        int best = -2; double bt = -1e30;
        for (auto& kv : barrier_time) if (kv.second < t && kv.second > bt) { bt = kv.second; best = kv.first; }
        return best;
    };
    // 2. reads behind a barrier that covered the tile's loads, from the slot of the tile's ring entry
    std::map<int, double> last_read;               // ring entry -> time of its last read
    for (const Read& r : reads) {
        const int entry = 2 * r.stage + (r.operand == ch::WGT);
        if (last_read.find(entry) == last_read.end() || last_read[entry] < r.time) last_read[entry] = r.time;
        if (r.stage >= checked) continue;
        if (r.slot != entry % NS) return fail("fragment read from the wrong slot", NB, r.stage, r.slot, entry % NS);
        const int b = barrier_before(r.time);
        if (b == -2) return fail("fragment read before any barrier", NB, r.stage);
        for (const Load& l : loads)
            if (l.operand == r.operand && l.stage == r.stage && l.seq >= landed_upto[b])
                return fail("fragment read before its tile's loads were waited for", NB, r.stage, l.seq, landed_upto[b]);
    }
    // 3. slot reuse
    for (const Load& l : loads) {
        const int entry = 2 * l.stage + (l.operand == ch::WGT), prev = entry - NS;
        if (prev < 0 || l.stage >= checked) continue;
        if (last_read.find(prev) == last_read.end()) return fail("previous tile of a slot never read", NB, prev);
        bool ok = false;
        for (auto& kv : barrier_time) ok = ok || (last_read[prev] < kv.second && kv.second < l.time);
        if (!ok) return fail("ring load overwrites a tile with no barrier behind its last read", NB, entry, prev);
    }
    // 4. operand registers
    std::map<std::tuple<int, int, int, int>, int> holds;            // (operand, khalf, block, buffer) -> stage
    size_t ri = 0, ui = 0;
    // reads and uses are each in time order already; merge (a use at time t comes before a read at time t)
    while (ui < uses.size()) {
        while (ri < reads.size() && reads[ri].time < uses[ui].time) {
            const Read& r = reads[ri++];
            holds[std::make_tuple(r.operand, r.khalf, r.block, r.buffer)] = r.stage;
        }
        const Use& u = uses[ui++];
        if (u.stage >= checked) continue;
        auto it = holds.find(std::make_tuple(u.operand, u.khalf, u.block, u.buffer));
        if (it == holds.end() || it->second != u.stage)
            return fail("MFMA operand register does not hold the stage being multiplied", NB, u.stage, u.operand, u.block);
    }
    std::printf("NB=%d WL=%d: ok (%zu ring loads, %zu fragment reads, %zu operand uses over %d stages)\n", NB, WL, loads.size(),
                reads.size(), uses.size(), stages);
    return 0;
}

int main() {
    // the widths the kernels are built with: 256, 224, 192, 160, 128 staged weight rows = 8 .. 4 blocks per wavefront
    for (int nb : {8, 7, 6, 5, 4})
        if (check(8, nb, nb, 24)) return 1;
    return 0;
}
