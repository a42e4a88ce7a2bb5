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

// The same replay for the plan of the 16x16x32 form (LdsPlan16): slot k < KS consumes K fragment k; slot KS + j
// (j < NV / 2) consumes V^T fragments 2 j and 2 j + 1 under ONE wait placed on the younger of the two; slot
// KS + NV / 2 + j uses the same two again without a wait.
template <int D, bool SPREAD>
int check16() {
    using P = ll::LdsPlan16<D, SPREAD>;
    constexpr int KS = P::KS, NV = P::NV, NSLOT = KS + NV, HV = NV / 2;
    std::deque<int> issued;
    auto position_from_youngest = [&](int id) {
        for (int i = int(issued.size()) - 1, n = 0; i >= 0; --i, ++n)
            if (issued[i] == id) return n;
        return -1;
    };
    for (int step = 0; step < 6; ++step) {
        for (int k = 0; k < NSLOT; ++k) {
            if (step > 0 && (k < KS || k < KS + HV)) {
                int need_old, need_young, count;
                if (k < KS) { need_old = need_young = (step - 1) * 100 + 50 + k; count = P::wait_k(k); }
                else        { need_old = step * 100 + 2 * (k - KS); need_young = need_old + 1; count = P::wait_v(k - KS); }
                const int pos_young = position_from_youngest(need_young), pos_old = position_from_youngest(need_old);
                if (pos_young < 0 || pos_old < 0) { std::printf("16: D=%d step %d slot %d: a fragment was never read\n", D, step, k); return 1; }
                if (count > 15) { std::printf("16: D=%d slot %d: count %d does not fit the counter\n", D, k, count); return 1; }
                if (pos_young < count || pos_old < count) { std::printf("16: D=%d step %d slot %d: wait %d too weak\n", D, step, k, count); return 1; }
                if (pos_young != count) { std::printf("16: D=%d step %d slot %d: wait %d stricter than needed (%d)\n", D, step, k, count, pos_young); return 1; }
            }
            if (k >= KS + HV) {   // second use: the fragments must be the ones of this step, untouched since
                for (int e = 0; e < 2; ++e) {
                    const int f = 2 * (k - KS - HV) + e;
                    if (P::last_use_v(f) != k || P::first_use_v(f) != k - HV) { std::printf("16: D=%d: use slots of V^T fragment %d\n", D, f); return 1; }
                }
            }
            for (int f = 0; f < NV; ++f)
                if (P::vslot(f) == k) {
                    // the register was last used in slot last_use_v(f) of the step before, and is first needed in first_use_v(f)
                    if (!(k < P::first_use_v(f))) { std::printf("16: D=%d: V^T fragment %d read in slot %d, after its use\n", D, f, k); return 1; }
                    if (!(P::last_use_v(f) < NSLOT)) return 1;
                    issued.push_back(step * 100 + f);
                }
            for (int f = 0; f < KS; ++f)
                if (P::kslot(f) == k) {
                    if (!(k > f)) { std::printf("16: D=%d: K fragment %d read in slot %d, before its register is free\n", D, f, k); return 1; }
                    issued.push_back(step * 100 + 50 + f);
                }
        }
    }
    int nv = 0, nk = 0;
    for (int k = 0; k < NSLOT; ++k) {
        for (int f = 0; f < NV; ++f) nv += P::vslot(f) == k;
        for (int f = 0; f < KS; ++f) nk += P::kslot(f) == k;
    }
    if (nv != NV || nk != KS) { std::printf("16: D=%d: %d V^T and %d K reads per step\n", D, nv, nk); return 1; }
    return 0;
}

int main() {
    if (check<64>() || check<128>()) return 1;
    if (check16<64, false>() || check16<128, false>() || check16<64, true>() || check16<128, true>()) return 1;
    std::printf("lds plan ok\n");
    return 0;
}
