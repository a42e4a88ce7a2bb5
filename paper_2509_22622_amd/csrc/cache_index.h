// Host-side bookkeeping of one layer's rolling KV cache: which frames are held,
// where each frame sits in the per-head key order, and which token-slot ranges a
// staged chunk attends to.  Pure C++ (no HIP), exact integer arithmetic.
//
// Key-set rule (paper Sec. 3.3, "Frame Sink" and "Short-window Attention"): a chunk
// starting at frame f0 attends to the sink frames [0, S), to the last W non-sink
// frames before f0, and to itself.  Stage/commit rule (Appendix Alg. 2): a chunk may
// be appended several times at the same start frame, the last version stays.
#pragma once
#include <cstdint>
#include <vector>

namespace ll {

struct Geometry {
    int P = 0;   // tokens per frame
    int S = 0;   // sink frames
    int W = 0;   // window frames (past, non-sink)
    int C = 0;   // chunk frames
    int ring() const { return W + C; }                       // ring capacity in frames
    int64_t slots() const { return int64_t(S + W + C) * P; } // token slots per head
};

struct SlotRange { int64_t begin, end; };   // half-open, in token slots

struct LayerIndex {
    // Frames held: sink frames [0, sink_have) and non-sink frames [lo, hi).
    int64_t sink_have = 0;
    int64_t lo = 0, hi = 0;
    // Staged chunk (start frame, length); staged_n == 0 means nothing is staged.
    int64_t staged_f0 = -1;
    int staged_n = 0;
};

enum class AppendKind { Invalid, First, Overwrite, Advance };

// First token slot of frame f in the per-head key order.
int64_t slot_of_frame(const Geometry& g, int64_t f);

// Classify an append at f0 against the layer's state.
AppendKind classify_append(const LayerIndex& L, int64_t f0);

// Apply an append of [f0, f0+n) (after classify_append said it is valid).
void apply_append(const Geometry& g, LayerIndex& L, int64_t f0, int n);

// State at the start of a re-prefill: non-sink frames dropped, nothing staged.
void begin_prefill(const Geometry& g, LayerIndex& L, bool include_sink, int64_t win_start);

// Stage [f0, f0+n) during a re-prefill (f0 may jump from the sink to win_start).
void prefill_stage(const Geometry& g, LayerIndex& L, int64_t f0, int n);

bool frame_held(const Geometry& g, const LayerIndex& L, int64_t f);

// Frames the staged chunk attends to, ascending.
std::vector<int64_t> live_frames(const Geometry& g, const LayerIndex& L);

// The same set as merged token-slot ranges, ascending (at most 3).
std::vector<SlotRange> live_ranges(const Geometry& g, const LayerIndex& L);

// Chunks of a re-prefill in order: the sink cut into chunks of C, then the window.
struct ChunkSpan { int64_t f0; int n; };
std::vector<ChunkSpan> prefill_chunks(const Geometry& g, bool include_sink, int64_t win_start, int n_win);

}  // namespace ll
