/* Plain C99 user of the library: the header must compile as C, the symbols must link with C linkage, and the
 * index-only handle must answer without a GPU.  Prints "c abi ok" and returns 0 on success. */
#include <stdio.h>
#include <string.h>

#include "../include/longlive.h"

int main(void) {
    ll_cache* c = NULL;
    int64_t frames[32], ranges[16], slot = -1;
    int n = 0, i;
    if (ll_cache_bytes(1, 2, 64, 60, 3, 6, 3) == 0) return 1;
    if (ll_cache_bytes(1, 2, 96, 60, 3, 6, 3) != 0) return 2;              /* head_dim must be 64 or 128 */
    if (ll_cache_create(1, 2, 64, 60, 3, 6, 3, 6, 10, 10000.0f, NULL, 0, &c) != LL_OK) return 3;
    for (i = 0; i < 6; ++i)                                                  /* six chunks of three frames */
        if (ll_chunk_append(c, 0, 3 * i, 3, NULL, NULL, NULL, NULL, NULL) != LL_OK) return 4;
    if (ll_cache_live_frames(c, 0, frames, 32, &n) != LL_OK || n != 12) return 5;   /* sink 3 + window 6 + chunk 3 */
    if (frames[0] != 0 || frames[2] != 2 || frames[3] != 9 || frames[11] != 17) return 6;
    if (ll_cache_slot_of_frame(c, 0, 17, &slot) != LL_OK || slot != (3 + (17 - 3) % 9) * 60) return 7;
    if (ll_cache_live_ranges(c, 0, ranges, 8, &n) != LL_OK || n < 1 || n > 3) return 8;
    if (ll_chunk_append(c, 0, 40, 3, NULL, NULL, NULL, NULL, NULL) != LL_ERR_STATE) return 9;
    if (strlen(ll_last_error()) == 0 || strcmp(ll_status_string(LL_ERR_STATE), "LL_ERR_STATE") != 0) return 10;
    if (ll_sink_window_attn(c, 0, NULL, NULL, NULL) != LL_ERR_INVALID_ARG) return 11;   /* no device cache */
    if (ll_cache_destroy(c) != LL_OK) return 12;
    {                                                                        /* the prompt side, index-only */
        ll_prompt* pr = NULL;
        if (ll_prompt_bytes(2, 2, 64, 77) == 0 || ll_prompt_bytes(2, 2, 64, 0) != 0) return 13;
        if (ll_prompt_create(2, 2, 64, 77, NULL, 0, &pr) != LL_OK) return 14;
        if (ll_cross_attn(pr, 1, NULL, 10, NULL, NULL) != LL_ERR_STATE) return 15;
        if (ll_prompt_recache(pr, 1, NULL, NULL, 40, NULL) != LL_OK) return 16;
        if (ll_prompt_tokens(pr, 1, &n) != LL_OK || n != 40) return 17;
        if (ll_cross_attn(pr, 1, NULL, 10, NULL, NULL) != LL_OK) return 18;
        if (ll_prompt_destroy(pr) != LL_OK) return 19;
    }
    {                                                                        /* the train-time rule, index-only */
        ll_clip* cl = NULL;
        if (ll_clip_bytes(2, 64, 60, 3, 6, 9, 3) == 0 || ll_clip_bytes(2, 96, 60, 3, 6, 9, 3) != 0) return 20;
        if (ll_clip_create(2, 64, 60, 3, 6, 9, 3, 6, 10, 10000.0f, NULL, 0, &cl) != LL_OK) return 21;
        if (ll_clip_backward(cl, NULL, NULL, NULL, NULL, NULL) != LL_ERR_STATE) return 22;
        if (ll_clip_forward(cl, 9, 6, 9, NULL, NULL, NULL, NULL, NULL) != LL_OK) return 23;
        if (ll_clip_backward(cl, NULL, NULL, NULL, NULL, NULL) != LL_OK) return 24;
        if (ll_clip_destroy(cl) != LL_OK) return 25;
    }
    printf("c abi ok\n");
    return 0;
}
