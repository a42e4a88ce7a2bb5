// Host simulation of the LDS ring hand-over of the streaming attention kernel (RingPlan in csrc/lds_plan.h).
// Several waves run the kernel's sequence of loads, waits, barriers and reads under random interleavings; loads land
// at random later times unless a wait forces them.  A read of a stage fragment is a violation unless the youngest
// load issued to that fragment has landed and carries the kblock the reader expects (anything else is a race: data
// not there yet, or possibly overwritten already).  Exit status 0 = no violation in any run.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2509_22622_amd/csrc/lds_plan.h"

using ll::RingPlan;

enum Kind { LOAD, WAIT, BARRIER, READ };
struct Op { Kind kind; int a; };   // LOAD: kblock; WAIT: kblocks of own loads that may stay in flight; READ: kblock

// program of one wave for a segment of n steps (the waves differ only in which fragments they load)
static std::vector<Op> program(int n) {
    std::vector<Op> p;
    auto clamp = [&](int v) { return v < n - 1 ? v : n - 1; };          // past the end the last kblock is fetched again
    (void)clamp;
    for (int j = 0; j < RingPlan::AHEAD; ++j) p.push_back({LOAD, j});
    p.push_back({WAIT, RingPlan::AHEAD - RingPlan::LANDED});
    p.push_back({BARRIER, 0});
    p.push_back({READ, 0});                                             // K of kblock 0, then of kblock 1
    p.push_back({READ, 1});
    for (int i = 0; i < n; ++i) {
        p.push_back({READ, i});                                         // V^T of kblock i (first slots)
        p.push_back({LOAD, i + RingPlan::AHEAD});
        p.push_back({READ, i + 2});                                     // K of kblock i + 2 (later slots)
        if (RingPlan::barrier_after(i)) {
            p.push_back({WAIT, RingPlan::AHEAD - RingPlan::LANDED});
            p.push_back({BARRIER, 0});
        }
    }
    return p;
}

struct Flight { int wave, kblock; bool landed; };

static int simulate(int waves, int n, unsigned seed) {
    std::srand(seed);
    const std::vector<Op> prog = program(n);
    std::vector<size_t> pc(waves, 0);
    std::vector<int> at_barrier(waves, 0);
    std::vector<std::vector<Flight>> own(waves);                         // each wave's loads, in issue order
    // youngest load issued to (stage, fragment owner = wave)
    std::vector<std::vector<int>> youngest(RingPlan::STAGES, std::vector<int>(waves, -1));   // index into own[wave]
    auto land_some = [&]() {
        for (int w = 0; w < waves; ++w)
            for (Flight& f : own[w]) {
                if (f.landed) continue;                                  // loads of a wave land in issue order
                if (std::rand() % 4 == 0) f.landed = true; else break;
            }
    };
    for (;;) {
        bool all_done = true, all_waiting = true;
        for (int w = 0; w < waves; ++w) {
            if (pc[w] < prog.size()) all_done = false;
            if (pc[w] < prog.size() && !at_barrier[w]) all_waiting = false;
        }
        if (all_done) return 0;
        if (all_waiting) {                                               // everybody arrived: release
            for (int w = 0; w < waves; ++w) if (pc[w] < prog.size()) { at_barrier[w] = 0; ++pc[w]; }
            continue;
        }
        const int w = std::rand() % waves;
        if (pc[w] >= prog.size() || at_barrier[w]) continue;
        land_some();
        const Op op = prog[pc[w]];
        switch (op.kind) {
            case LOAD:
                own[w].push_back({w, op.a, false});
                youngest[op.a % RingPlan::STAGES][w] = int(own[w].size()) - 1;
                ++pc[w];
                break;
            case WAIT: {
                const int keep = op.a;                                   // kblocks' worth of loads (one load per kblock here)
                for (size_t i = 0; i + keep < own[w].size(); ++i) own[w][i].landed = true;
                ++pc[w];
                break;
            }
            case BARRIER:
                at_barrier[w] = 1;
                break;
            case READ:
                for (int o = 0; o < waves; ++o) {                        // a read takes fragments loaded by every wave
                    const int idx = youngest[op.a % RingPlan::STAGES][o];
                    if (idx < 0 || !own[o][idx].landed || own[o][idx].kblock != op.a) {
                        std::printf("seed %u: wave %d reads kblock %d, fragment of wave %d holds %s kblock %d\n", seed, w, op.a, o,
                                    idx < 0 ? "no" : (own[o][idx].landed ? "landed" : "in-flight"), idx < 0 ? -1 : own[o][idx].kblock);
                        return 1;
                    }
                }
                ++pc[w];
                break;
        }
    }
}

int main() {
    static_assert((RingPlan::STAGES & (RingPlan::STAGES - 1)) == 0, "stage = kblock & (STAGES - 1)");
    for (int n : {1, 2, 3, 4, 5, 8, 13, 40})
        for (unsigned seed = 1; seed <= 300; ++seed)
            if (simulate(3, n, seed * 7919u + n)) return 1;
    std::printf("ring plan ok\n");
    return 0;
}
