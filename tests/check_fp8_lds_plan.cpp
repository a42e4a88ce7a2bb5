// Host replay of the LDS read plan of the 8-bit attention kernel (Fp8LdsPlan in csrc/lds_plan.h): simulates the
// in-order LDS queue over several steps exactly as the kernel issues it (per slot: wait, MFMA, then the two reads of
// the fragment AHEAD_SLOTS slots later into that slot's buffer) and checks at every MFMA that the wait count
// guarantees its fragment has arrived and is not stricter than needed, that the fragment in the buffer is the one
// the slot wants, and that no buffer is rewritten sooner than two slots after the MFMA that used it was issued (the
// margin the kernel relies on: by then another MFMA of the same wave has entered the matrix pipe behind it, so the
// first one has finished reading its operands).
#include <cstdio>
#include <deque>

#include "../paper_2509_22622_amd/csrc/lds_plan.h"

template <int D>
int check() {
    using P = ll::Fp8LdsPlan<D>;
    constexpr int NSLOT = P::NSLOT;
    std::deque<int> issued;                          // read ids, oldest first; id = 2 * (global slot) + piece
    int held[P::BUFFERS], last_use[P::BUFFERS];      // fragment (global slot) in each buffer, slot of its last MFMA
    for (int b = 0; b < P::BUFFERS; ++b) held[b] = last_use[b] = -1000;
    auto read_fragment = [&](int gslot, int now) {
        const int b = P::buffer(gslot % NSLOT);
        constexpr int MIN_REUSE_SLOTS = 2;
        if (now - last_use[b] < MIN_REUSE_SLOTS && last_use[b] >= 0) {
            std::printf("D=%d: buffer %d rewritten in slot %d, %d slots after its MFMA\n", D, b, now, now - last_use[b]);
            return 1;
        }
        held[b] = gslot;
        for (int piece = 0; piece < P::READS_PER_FRAGMENT; ++piece) issued.push_back(2 * gslot + piece);
        return 0;
    };
    // prologue: the fragments of the first AHEAD_SLOTS slots
    for (int j = 0; j < P::AHEAD_SLOTS; ++j)
        if (read_fragment(j, -1)) return 1;
    for (int g = 0; g < 5 * NSLOT; ++g) {            // global slot index over five steps
        const int b = P::buffer(g % NSLOT);
        if (held[b] != g) { std::printf("D=%d slot %d: buffer %d holds fragment %d\n", D, g, b, held[b]); return 1; }
        // position of the fragment's last read, counted from the youngest read
        int pos = -1;
        for (int i = int(issued.size()) - 1, n = 0; i >= 0; --i, ++n)
            if (issued[i] == 2 * g + P::READS_PER_FRAGMENT - 1) { pos = n; break; }
        if (pos < 0) { std::printf("D=%d slot %d: fragment never read\n", D, g); return 1; }
        if (P::wait() > 15) { std::printf("count does not fit the counter\n"); return 1; }
        if (pos < P::wait()) { std::printf("D=%d slot %d: wait %d too weak (fragment %d from the youngest)\n", D, g, P::wait(), pos); return 1; }
        if (pos != P::wait()) { std::printf("D=%d slot %d: wait %d stricter than needed (%d)\n", D, g, P::wait(), pos); return 1; }
        last_use[b] = g;                             // the MFMA
        if (read_fragment(g + P::AHEAD_SLOTS, g)) return 1;
    }
    return 0;
}

int main() {
    if (check<64>() || check<128>()) return 1;
    std::printf("fp8 lds plan ok\n");
    return 0;
}
