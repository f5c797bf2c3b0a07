// Declarations shared by the translation units of the paged-cache reader.
#pragma once
#include "alora_internal.h"
#include "alora_attention.h"

namespace alora {

struct AttnArgs {
    const void *q, *kc, *vc;
    const int32_t *bt, *seq, *pos;
    void *out;
    int T, Hq, Hkv, n_seqs, max_blocks, bs, bs_shift;
    long long n_slots;
    float scale_log2e;   // scale * log2(e): the softmax runs on powers of two
    int splits;          // parts a row's context is cut into (one workgroup each); > 1: partials go to `part`
    float *part;         // [T][Hq][splits][D + 2]: running maximum, sum of weights, unnormalised weighted V
};

// Row-block kernel (bf16, head_dim 128): rows of one sequence that follow each other in the batch share
// the loads of their context.  Returns the hipError_t of its launch.
int launch_attention_blocks(const AttnArgs &a, int G, hipStream_t stream);

}  // namespace alora
