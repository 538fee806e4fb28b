// The model-derived bigram drafter the paper compares against (Related Work; Results, "TASC-spec": a bigram model
// that assigns each token its most probable next token under the given model, obtained from the model's conditional
// distribution for every vocabulary element; used alone and mixed with the context drafter).
//
// next(x) = greedy next token after the one-token sequence [x]: the vocabulary is pushed through the ordinary
// prefill path, `batch` single-token prompts at a time, so the forward kernels are the ones every other call uses.
// As a draft source it is the point mass on next(x): the order-2 table with C(x, next(x)) = 1, T(x) = 1 and no
// higher orders, built by the ordinary table builder from the V two-token outputs [x, next(x)].
#include <vector>

#include "tasc_internal.h"

namespace {
__global__ void k_bigram_prompts(int32_t* prompts, int first, int vocab, int B) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) prompts[i] = min(first + i, vocab - 1);       // the last chunk repeats the last token; not collected
}
// the token prefill committed after prompt position 0 of sequence i
__global__ void k_bigram_collect(const int32_t* __restrict__ tokens, int max_len, int first, int vocab, int B, int32_t* next_tok) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B && first + i < vocab) next_tok[first + i] = tokens[(size_t)i * max_len + 1];
}
__global__ void k_bigram_pairs(const int32_t* __restrict__ next_tok, int vocab, int32_t* pairs) {
    const int x = blockIdx.x * blockDim.x + threadIdx.x;
    if (x < vocab) { pairs[2 * x] = x; pairs[2 * x + 1] = next_tok[x]; }
}
struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
};
}  // namespace

extern "C" tasc_status tasc_model_bigram(const tasc_model* m, tasc_session* s, int32_t* next_tok, void* stream) {
    TASC_REQUIRE(m && s && next_tok, "model_bigram: null argument");
    TASC_REQUIRE(s->model == m, "model_bigram: session belongs to another model");
    hipStream_t st = (hipStream_t)stream;
    const int B = s->batch, V = m->desc.vocab;
    DevBuf prompts;
    TASC_HIP(hipMalloc(&prompts.p, (size_t)B * sizeof(int32_t)));
    std::vector<int64_t> offs(B + 1);
    for (int b = 0; b <= B; ++b) offs[b] = b;
    for (int first = 0; first < V; first += B) {
        k_bigram_prompts<<<dim3((B + 255) / 256), dim3(256), 0, st>>>((int32_t*)prompts.p, first, V, B);
        TASC_LAUNCH_CHECK();
        tasc_status rc = tasc_session_prefill(m, s, (const int32_t*)prompts.p, offs.data(), TASC_MEM_DEVICE, 1, stream);
        if (rc != TASC_OK) return rc;
        k_bigram_collect<<<dim3((B + 255) / 256), dim3(256), 0, st>>>(s->d.tokens, s->max_len, first, V, B, next_tok);
        TASC_LAUNCH_CHECK();
    }
    TASC_HIP(hipStreamSynchronize(st));
    s->prefilled = 0;                          // the sequences hold the last chunk of vocabulary tokens, not a caller's prompts
    return TASC_OK;
}

extern "C" tasc_status tasc_ngram_from_bigram(const int32_t* next_tok, tasc_mem where, int32_t vocab, int32_t n_max, void* stream,
                                              tasc_ngram** out) {
    TASC_REQUIRE(next_tok && out, "ngram_from_bigram: null argument");
    TASC_REQUIRE(vocab >= 1, "ngram_from_bigram: vocab %d", vocab);
    TASC_REQUIRE(where == TASC_MEM_HOST || where == TASC_MEM_DEVICE, "ngram_from_bigram: bad memory kind");
    hipStream_t st = (hipStream_t)stream;
    DevBuf staged, pairs;
    const int32_t* d_next = next_tok;
    if (where == TASC_MEM_HOST) {
        TASC_HIP(hipMalloc(&staged.p, (size_t)vocab * sizeof(int32_t)));
        TASC_HIP(hipMemcpyAsync(staged.p, next_tok, (size_t)vocab * sizeof(int32_t), hipMemcpyHostToDevice, st));
        d_next = (const int32_t*)staged.p;
    }
    TASC_HIP(hipMalloc(&pairs.p, (size_t)vocab * 2 * sizeof(int32_t)));
    k_bigram_pairs<<<dim3((vocab + 255) / 256), dim3(256), 0, st>>>(d_next, vocab, (int32_t*)pairs.p);
    TASC_LAUNCH_CHECK();
    std::vector<int64_t> offs((size_t)vocab + 1);
    for (int64_t x = 0; x <= vocab; ++x) offs[x] = 2 * x;
    // the ordinary builder: every two-token output holds one bigram window and no longer one; it rejects successors
    // outside [0, vocab)
    tasc_status rc = tasc_ngram_build((const int32_t*)pairs.p, offs.data(), vocab, vocab, n_max, 1, TASC_MEM_DEVICE, stream, out);
    (void)hipStreamSynchronize(st);            // before the staging buffers go
    return rc;
}
