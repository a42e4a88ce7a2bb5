// Issue plan of the LDS fragment reads of one kblock step of the streaming attention kernel, and the
// s_waitcnt counts that go with it.  Plain constexpr C++ so that a host test can replay the plan.
//
// A step has KS + NV slots (KS = D/16 MFMAs of S^T = K Q^T for the next kblock, then NV = D/16 MFMAs of
// O^T += V^T P^T for this one).  Each slot issues its MFMA first, then its reads, V^T reads before K reads, each
// kind in fragment order.  The LDS returns data in issue order, so "at most N reads outstanding" means that every
// read but the N youngest has arrived.
#pragma once

namespace ll {

template <int D>
struct LdsPlan {
    static constexpr int KS = D / 16;    // K fragments per kblock = slots of the first MFMA group
    static constexpr int NV = D / 16;    // V^T fragments per kblock = slots of the second MFMA group
    // V^T fragment f of this step's kblock is read in slot f / 2: before slot KS + f needs it, after the step
    // before has used the register (its slot KS + f).
    static constexpr int vslot(int f) { return f / 2; }
    // K fragment f of the next kblock is read in slot KS + f / 2: after slot f of this step has used the register.
    static constexpr int kslot(int f) { return KS + f / 2; }
    // Reads issued after V^T fragment g when slot KS + g starts (its MFMA consumes the fragment): the later V^T
    // reads and the K reads of earlier slots.
    static constexpr int wait_v(int g) {
        int c = 0;
        for (int f = 0; f < NV; ++f) c += vslot(f) > vslot(g) || (vslot(f) == vslot(g) && f > g);
        for (int f = 0; f < KS; ++f) c += kslot(f) < KS + g;
        return c;
    }
    // Reads issued after K fragment ks (read in the step before) when slot ks starts: the later K reads of that
    // step and the V^T reads of this step's earlier slots.
    static constexpr int wait_k(int ks) {
        int c = 0;
        for (int f = 0; f < KS; ++f) c += kslot(f) > kslot(ks) || (kslot(f) == kslot(ks) && f > ks);
        for (int f = 0; f < NV; ++f) c += vslot(f) < ks;
        return c;
    }
};

// The plan of the same kernel built on 16x16x32 MFMAs (attn_stream16.hip).  A step has the same KS + NV slots, each
// now opened by the two MFMAs that share a fragment: slot k < KS takes K fragment k; the O^T slots run over the
// V^T fragments twice, slot KS + j taking fragments 2 j and 2 j + 1 for the first query block (j < NV / 2) and slot
// KS + NV / 2 + j the same two for the second.  Reads are issued as above (V^T fragment f in slot f / 2, K fragment
// f of the next kblock in slot KS + f / 2, after the slot's MFMAs, V^T before K, in fragment order).  A fragment is
// waited for at its first use only; the younger of a slot's two V^T fragments carries the wait for both.
// SPREAD: one read per slot instead (V^T fragment f in slot f, K fragment f in slot KS + f).
template <int D, bool SPREAD = false>
struct LdsPlan16 {
    static constexpr int KS = D / 16;
    static constexpr int NV = D / 16;
    static constexpr int vslot(int f) { return SPREAD ? f : f / 2; }
    static constexpr int kslot(int f) { return SPREAD ? KS + f : KS + f / 2; }
    static constexpr int first_use_v(int f) { return KS + f / 2; }            // slot of the first query block
    static constexpr int last_use_v(int f) { return KS + NV / 2 + f / 2; }    // slot of the second query block
    // Reads issued after V^T fragment 2 j + 1 when slot KS + j starts.
    static constexpr int wait_v(int j) {
        const int g = 2 * j + 1;
        int c = 0;
        for (int f = 0; f < NV; ++f) c += vslot(f) > vslot(g) || (vslot(f) == vslot(g) && f > g);
        for (int f = 0; f < KS; ++f) c += kslot(f) < KS + j;
        return c;
    }
    // Reads issued after K fragment k (read in the step before) when slot k starts.
    static constexpr int wait_k(int k) {
        int c = 0;
        for (int f = 0; f < KS; ++f) c += kslot(f) > kslot(k) || (kslot(f) == kslot(k) && f > k);
        for (int f = 0; f < NV; ++f) c += vslot(f) < k;
        return c;
    }
};

// The same for the kernel of the 8-bit cache.  A step has NK = 2 * D/64 slots of S^T MFMAs (for the next kblock)
// and DB = D/32 slots of O^T MFMAs (for this one); every MFMA consumes one operand fragment, read with two 16-byte
// LDS reads.  Slot k issues its MFMA first and then the two reads of the fragment that slot k + AHEAD_SLOTS needs
// (slots past the end of the step are the first slots of the next step), into register buffer
// (k + AHEAD_SLOTS) % BUFFERS.  So exactly (AHEAD_SLOTS - 1) fragments are issued between a fragment's reads and
// its use, and one wait count serves every slot.  A buffer is rewritten BUFFERS - AHEAD_SLOTS slots after the MFMA
// that used it was issued: two slots, i.e. after one more MFMA of the same wave has entered the matrix pipe behind it.
template <int D>
struct Fp8LdsPlan {
    static constexpr int NK = 2 * (D / 64);
    static constexpr int DB = D / 32;
    static constexpr int NSLOT = NK + DB;
    static constexpr int AHEAD_SLOTS = 2;
    static constexpr int BUFFERS = 4;
    static constexpr int READS_PER_FRAGMENT = 2;
    static constexpr int buffer(int slot) { return slot % BUFFERS; }
    // reads issued after a fragment's own when its slot starts
    static constexpr int wait() { return (AHEAD_SLOTS - 1) * READS_PER_FRAGMENT; }
    static_assert(NSLOT % BUFFERS == 0, "the buffer of a slot must not depend on the step");
    static_assert(AHEAD_SLOTS < BUFFERS, "a fragment would be read into a buffer still in use");
};

// The ring of K/V stages in LDS and its hand-over between the waves of a workgroup.
//   Kblock v lives in stage v % STAGES.  The prologue issues the loads of the first AHEAD kblocks; step i issues
//   those of kblock i + AHEAD, and reads kblock i (V^T) and kblock i + 2 (K for the scores of the step after next;
//   the prologue reads kblocks 0 and 1).  Every wave loads its own fragments of a stage.  Before each barrier a wave
//   waits until all but its youngest (AHEAD - LANDED) kblocks of loads have arrived; barriers stand after the
//   prologue's loads and after every step with an odd index.
struct RingPlan {
    static constexpr int STAGES = 8;   // a power of two
    static constexpr int AHEAD = 6;    // kblocks the loads run ahead of the step that issues them
    static constexpr int LANDED = 4;   // kblocks, counted from the next step, that have arrived at a barrier
    static constexpr bool barrier_after(int step) { return step & 1; }
};

}  // namespace ll
