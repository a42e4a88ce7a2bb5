// Host replay of the LDS read plan of the streaming attention kernel (csrc/lds_plan.h): simulates the in-order
// LDS queue over several steps and checks, at every MFMA that consumes a fragment, that the wait count used there
// guarantees the fragment has arrived, is not stricter than needed, fits the 4-bit counter, and that no register
// is overwritten before its last use.  Exit status 0 = all good; prints the first violation otherwise.
#include <cstdio>
#include <deque>

#include "../paper_2509_22622_amd/csrc/lds_plan.h"

template <int D>
int check() {
    using P = ll::LdsPlan<D>;
    constexpr int KS = P::KS, NV = P::NV, NSLOT = KS + NV;
    // read id: step * 100 + kind * 50 + fragment (kind 0 = V^T of that step's kblock, 1 = K of the next kblock)
    std::deque<int> issued;                       // all reads so far, oldest first
    auto position_from_youngest = [&](int id) {   // 0 = youngest; -1 = never issued
        for (int i = int(issued.size()) - 1, n = 0; i >= 0; --i, ++n)
            if (issued[i] == id) return n;
        return -1;
    };
    for (int step = 0; step < 6; ++step) {
        for (int k = 0; k < NSLOT; ++k) {
            // the slot's MFMA first
            if (step > 0) {                        // step 0 stands for the prologue's reads (waited for separately)
                int need, count;
                if (k < KS) { need = (step - 1) * 100 + 50 + k; count = P::wait_k(k); }
                else        { need = step * 100 + (k - KS);     count = P::wait_v(k - KS); }
                const int pos = position_from_youngest(need);
                if (pos < 0) { std::printf("D=%d step %d slot %d: fragment %d was never read\n", D, step, k, need); return 1; }
                if (count > 15) { std::printf("D=%d slot %d: count %d does not fit the counter\n", D, k, count); return 1; }
                // waiting for "at most count outstanding" completes everything but the `count` youngest reads
                if (pos < count) { std::printf("D=%d step %d slot %d: wait %d too weak, fragment is %d from the youngest\n", D, step, k, count, pos); return 1; }
                if (pos != count) { std::printf("D=%d step %d slot %d: wait %d stricter than needed (%d)\n", D, step, k, count, pos); return 1; }
            }
            // then its reads: V^T before K, each in fragment order
            for (int f = 0; f < NV; ++f)
                if (P::vslot(f) == k) {
                    if (!(k < KS + f)) { std::printf("D=%d: V^T fragment %d read in slot %d, after its use\n", D, f, k); return 1; }
                    issued.push_back(step * 100 + f);     // register last used in slot KS + f of the step before: earlier
                }
            for (int f = 0; f < KS; ++f)
                if (P::kslot(f) == k) {
                    if (!(k > f)) { std::printf("D=%d: K fragment %d read in slot %d, before its register is free\n", D, f, k); return 1; }
                    issued.push_back(step * 100 + 50 + f);
                }
        }
    }
    // every fragment is read exactly once per step
    int nv = 0, nk = 0;
    for (int k = 0; k < NSLOT; ++k) {
        for (int f = 0; f < NV; ++f) nv += P::vslot(f) == k;
        for (int f = 0; f < KS; ++f) nk += P::kslot(f) == k;
    }
    if (nv != NV || nk != KS) { std::printf("D=%d: %d V^T and %d K reads per step\n", D, nv, nk); return 1; }
    return 0;
}

int main() {
    if (check<64>() || check<128>()) return 1;
    std::printf("lds plan ok\n");
    return 0;
}
