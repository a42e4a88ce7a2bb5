#include "cache_index.h"

#include <algorithm>

namespace ll {

int64_t slot_of_frame(const Geometry& g, int64_t f) {
    if (f < g.S) return f * g.P;
    return (int64_t(g.S) + (f - g.S) % g.ring()) * g.P;
}

AppendKind classify_append(const LayerIndex& L, int64_t f0) {
    if (L.staged_n == 0) return f0 == 0 ? AppendKind::First : AppendKind::Invalid;
    if (f0 == L.staged_f0) return AppendKind::Overwrite;
    if (f0 == L.staged_f0 + L.staged_n) return AppendKind::Advance;
    return AppendKind::Invalid;
}

static void stage(const Geometry& g, LayerIndex& L, int64_t f0, int n) {
    L.staged_f0 = f0;
    L.staged_n = n;
    const int64_t end = f0 + n;
    if (f0 < g.S) L.sink_have = std::min<int64_t>(g.S, end);
    if (end > g.S) {
        if (L.hi <= L.lo) L.lo = std::max<int64_t>(g.S, f0);   // first non-sink frame ever held
        L.hi = end;
    } else {
        L.hi = L.lo;                                             // only sink frames so far
    }
}

void apply_append(const Geometry& g, LayerIndex& L, int64_t f0, int n) { stage(g, L, f0, n); }

void begin_prefill(const Geometry& g, LayerIndex& L, bool include_sink, int64_t win_start) {
    if (include_sink) L.sink_have = 0;
    L.lo = L.hi = std::max<int64_t>(g.S, win_start);
    L.staged_f0 = -1;
    L.staged_n = 0;
}

void prefill_stage(const Geometry& g, LayerIndex& L, int64_t f0, int n) { stage(g, L, f0, n); }

bool frame_held(const Geometry& g, const LayerIndex& L, int64_t f) {
    if (f < 0) return false;
    if (f < g.S) return f < L.sink_have;
    // the ring keeps at most W + C frames below hi
    return f >= L.lo && f < L.hi && f >= L.hi - g.ring();
}

std::vector<int64_t> live_frames(const Geometry& g, const LayerIndex& L) {
    std::vector<int64_t> out;
    if (L.staged_n == 0) return out;
    const int64_t f0 = L.staged_f0, end = f0 + L.staged_n;
    for (int64_t f = 0; f < std::min<int64_t>(L.sink_have, g.S); ++f) out.push_back(f);
    const int64_t from = std::max<int64_t>(std::max<int64_t>(g.S, f0 - g.W), L.lo);
    for (int64_t f = from; f < end; ++f) out.push_back(f);
    return out;
}

std::vector<SlotRange> live_ranges(const Geometry& g, const LayerIndex& L) {
    std::vector<SlotRange> r;
    for (int64_t f : live_frames(g, L)) {
        const int64_t s = slot_of_frame(g, f);
        r.push_back({s, s + g.P});
    }
    std::sort(r.begin(), r.end(), [](const SlotRange& a, const SlotRange& b) { return a.begin < b.begin; });
    std::vector<SlotRange> m;
    for (const SlotRange& x : r) {
        if (!m.empty() && m.back().end == x.begin) m.back().end = x.end;
        else m.push_back(x);
    }
    return m;
}

std::vector<ChunkSpan> prefill_chunks(const Geometry& g, bool include_sink, int64_t win_start, int n_win) {
    std::vector<ChunkSpan> out;
    if (include_sink)
        for (int a = 0; a < g.S; a += g.C) out.push_back({a, std::min(g.C, g.S - a)});
    for (int a = 0; a < n_win; a += g.C) out.push_back({win_start + a, std::min(g.C, n_win - a)});
    return out;
}

}  // namespace ll
