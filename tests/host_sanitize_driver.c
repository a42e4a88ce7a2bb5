/* Host-side walk through the library's bookkeeping on index-only handles (no GPU), meant to run with the library's
 * host code built under AddressSanitizer and UndefinedBehaviorSanitizer: random streams of appends (repeated passes,
 * short chunks), re-prefills with and without the sink, resets, the introspection calls with small and large
 * buffers, and the prompt and train-time handles.  Checks what must hold at every step (return codes, at most three
 * ascending disjoint ranges that cover exactly the live frames' slots); a sanitizer report or a failed check ends the
 * program with a non-zero status.  Prints "host walk ok". */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/longlive.h"
#include "../include/longlive_diag.h"

static unsigned long long rng = 88172645463325252ULL;
static unsigned rnd(unsigned n) { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (unsigned)(rng % n); }
#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s (%s)\n", __LINE__, #c, ll_last_error()); return 1; } } while (0)

static int check_ranges(ll_cache* c, int layer, int P, int S, int W, int C) {
    int64_t frames[256], ranges[8], slot;
    int nf = 0, nr = 0, i, j;
    int64_t covered = 0, prev_end = -1;
    CHECK(ll_cache_live_frames(c, layer, frames, 256, &nf) == LL_OK);
    CHECK(nf <= S + W + C);
    CHECK(ll_cache_live_ranges(c, layer, ranges, 4, &nr) == LL_OK);
    CHECK(nr <= 3 && (nf == 0) == (nr == 0));
    for (i = 0; i < nr; ++i) {
        CHECK(ranges[2 * i] < ranges[2 * i + 1] && ranges[2 * i] > prev_end);
        prev_end = ranges[2 * i + 1];
        covered += ranges[2 * i + 1] - ranges[2 * i];
    }
    CHECK(covered == (int64_t)nf * P);
    for (i = 0; i < nf; ++i) {
        int inside = 0;
        CHECK(ll_cache_slot_of_frame(c, layer, frames[i], &slot) == LL_OK);
        for (j = 0; j < nr; ++j) inside |= slot >= ranges[2 * j] && slot + P <= ranges[2 * j + 1];
        CHECK(inside);
        if (i) CHECK(frames[i] > frames[i - 1]);
    }
    if (nf > 1) {   /* too small a buffer is an error that still reports the count */
        int n2 = 0;
        CHECK(ll_cache_live_frames(c, layer, frames, 1, &n2) == LL_ERR_BUFFER_TOO_SMALL && n2 == nf);
    }
    return 0;
}

int main(void) {
    int trial;
    for (trial = 0; trial < 300; ++trial) {
        const int C = 1 + (int)rnd(4), S = (int)rnd(6), W = (int)rnd(10), gh = 1 + (int)rnd(5), gw = 1 + (int)rnd(40);
        const int P = gh * gw, layers = 1 + (int)rnd(3), D = rnd(2) ? 64 : 128, fp8 = (int)rnd(4) == 0;
        ll_cache* c = NULL;
        int64_t f0 = 0;
        int step, staged = 0;
        if (fp8) CHECK(ll_cache_create_fp8(layers, 1 + (int)rnd(3), D, P, S, W, C, gh, gw, 10000.0f, (int)rnd(5) - 2, 0, NULL, 0, &c) == LL_OK);
        else CHECK(ll_cache_create(layers, 1 + (int)rnd(3), D, P, S, W, C, gh, gw, 10000.0f, NULL, 0, &c) == LL_OK);
        if (!fp8 && rnd(2)) CHECK(ll_cache_set_sink_relative(c, 1) == LL_OK);
        for (step = 0; step < 60; ++step) {
            const int layer = (int)rnd((unsigned)layers) * 0;      /* one layer carries the stream, the others stay empty */
            const unsigned what = rnd(20);
            if (what == 0 && staged) {                              /* re-prefill of what the ring may hold */
                const int n_win = (int)rnd((unsigned)(W + C + 1));
                const int with_sink = (int)rnd(2);
                const int64_t ws = n_win == 0 ? S : S + (int64_t)rnd(50);
                ll_status st = ll_recache_prefill(c, layer, with_sink, ws, n_win, NULL, NULL, NULL, NULL, NULL);
                if ((with_sink ? S : 0) + n_win == 0) { CHECK(st == LL_ERR_INVALID_ARG); continue; }
                if (st == LL_ERR_STATE) { CHECK(!with_sink); continue; }   /* sink not complete yet */
                CHECK(st == LL_OK);
                f0 = ws + n_win;
                if (n_win == 0) f0 = S;
                staged = 1;
                if (check_ranges(c, layer, P, S, W, C)) return 1;
                /* the staged chunk may be repeated; the stream goes on behind it */
                continue;
            }
            if (what == 1) {                                        /* out-of-order append: refused, nothing changes */
                CHECK(ll_chunk_append(c, layer, f0 + 1 + (int64_t)rnd(5), 1, NULL, NULL, NULL, NULL, NULL) == LL_ERR_STATE || !staged);
                if (!staged) { CHECK(ll_cache_reset(c, layer) == LL_OK); f0 = 0; }
                continue;
            }
            if (what == 2) { CHECK(ll_cache_reset(c, -1) == LL_OK); f0 = 0; staged = 0; continue; }
            {
                const int n = 1 + (int)rnd((unsigned)C), passes = 1 + (int)rnd(3);
                int p;
                for (p = 0; p < passes; ++p) CHECK(ll_chunk_append(c, layer, f0, n, NULL, NULL, NULL, NULL, NULL) == LL_OK);
                staged = 1;
                if (check_ranges(c, layer, P, S, W, C)) return 1;
                f0 += n;
            }
        }
        CHECK(ll_cache_destroy(c) == LL_OK);
    }
    {   /* the prompt side and the train-time handle */
        ll_prompt* pr = NULL;
        ll_clip* cl = NULL;
        int64_t ranges[4];
        int n = 0, i;
        CHECK(ll_prompt_create(3, 2, 64, 100, NULL, 0, &pr) == LL_OK);
        for (i = 0; i < 50; ++i) {
            const int layer = (int)rnd(3), tokens = 1 + (int)rnd(100);
            CHECK(ll_prompt_recache(pr, layer, NULL, NULL, tokens, NULL) == LL_OK);
            CHECK(ll_prompt_tokens(pr, layer, &n) == LL_OK && n == tokens);
            CHECK(ll_cross_attn(pr, layer, NULL, 1 + (int)rnd(5000), NULL, NULL) == LL_OK);
            CHECK(ll_cross_attn_out(pr, layer, NULL, 1 + (int)rnd(5000), NULL, NULL, NULL, NULL) == LL_OK);
        }
        CHECK(ll_prompt_recache(pr, 0, NULL, NULL, 101, NULL) == LL_ERR_INVALID_ARG);
        CHECK(ll_prompt_destroy(pr) == LL_OK);
        CHECK(ll_clip_create(2, 64, 60, 3, 6, 9, 3, 6, 10, 10000.0f, NULL, 0, &cl) == LL_OK);
        for (i = 0; i < 50; ++i) {
            const int n_ctx = (int)rnd(7), n_clip = 1 + (int)rnd(9), chunk = (int)rnd(3);
            const int64_t ctx_start = 3 + (int64_t)rnd(100);
            CHECK(ll_clip_forward(cl, ctx_start, n_ctx, n_clip, NULL, NULL, NULL, NULL, NULL) == LL_OK);
            if (chunk < (n_clip + 2) / 3) CHECK(ll_clip_chunk_key_ranges(cl, chunk, ranges, 2, &n) == LL_OK && n >= 1 && n <= 2);
            CHECK(ll_clip_backward(cl, NULL, NULL, NULL, NULL, NULL) == LL_OK);
        }
        CHECK(ll_clip_destroy(cl) == LL_OK);
        CHECK(ll_set_attn_variant(99) == LL_ERR_INVALID_ARG && ll_set_attn_variant(0) == LL_OK);
        CHECK(ll_attn_variant_name(99) == NULL);
    }
    printf("host walk ok\n");
    return 0;
}
