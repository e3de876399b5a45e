// Device-side control blocks shared by the kernels and the host driver of the library.
#pragma once
#include <stdint.h>

#define KS_MAX_ROWS 16
#define KS_NWG 256      // workgroups of every tuned kernel: one 1024-thread workgroup per compute unit

// What one forward pass works on. Lives in device memory so that a pass can be
// enqueued before the host knows its contents (the previous kernels fill it in).
struct PassCtl {
    int32_t active;     // 0: every kernel of the pass returns at once
    int32_t n_rows;     // rows carried by this pass (1 for a draft step)
    int32_t start;      // position of row 0; row r sits at start + r
    int32_t head_from;  // LM head / arg-max only for rows >= head_from
    int32_t tok[KS_MAX_ROWS];
};

// Result of the LM-head arg-max for each row of the last pass.
struct HeadResult {
    int32_t tok[KS_MAX_ROWS];
    float prob[KS_MAX_ROWS];   // softmax probability of tok at temperature 1
};

// State of one generation (Sec. 4.2 draft / verify rounds), advanced on the device.
struct GenState {
    int32_t cache_len;   // valid KV positions
    int32_t x_last;      // last emitted token = input of the next round
    int32_t emitted;     // tokens emitted so far (the prefill's token included)
    int32_t max_new;
    int32_t max_draft;
    float conf_thr;
    int32_t kmax;        // draft cap of the current round
    int32_t k;           // drafts made in the current round
    int32_t done;
    int32_t n_accepted;  // j of the last verification
    int32_t drafts[KS_MAX_ROWS];
    float draft_p[KS_MAX_ROWS];
    int64_t rounds, drafted, accepted, draft_passes;
};

struct KnnResult {
    int32_t idx;         // arg-max anchor
    int32_t label;       // its domain
    int32_t degenerate;  // 1: zero-norm / non-finite query or anchor met
    float score;         // its cosine similarity times |query| (the query norm is a common factor)
};
