// CPU oracle for paged GQA decode attention (and its causal, several-queries-per-request form,
// chunked prefill, at the end of this file).  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain, fp64 statement of what one decode step of
// attention over a paged KV cache computes.  It exists so that the GPU library
// can be checked against something that is obviously the definition; it is not
// part of the product, shares no code with the GPU path, and must only be
// reached from tests, the smoke check and the benchmark's CPU-baseline leg.
//
// What is computed (paper section 2, "Phases of LLM inference": a decode step
// takes the last generated token and the KV cache, i.e. one query vector per
// head attends over every cached key/value of its request; the attention
// itself is the scaled-dot-product definition the paper cites there.  Section
// 5.2, "KV cache transmission", fixes only that the cache lives in fixed-size
// blocks; block size, layout and table format are this build's choices and are
// passed here as explicit strides so the oracle bakes in no layout):
//
//   for request b, query head h, kv head j = floor(h / (Hq/Hkv)), L = context_lens[b]
//     k_t = K[block_table[b][t / page]][j][t % page][:]        t = 0..L-1   (v_t alike)
//     s_t = scale * sum_d q[b][h][d] * k_t[d]
//     M   = max_t s_t ;  w_t = exp(s_t - M) ;  Z = sum_t w_t
//     out[b][h][d] = (sum_t w_t * v_t[d]) / Z
//     lse[b][h]    = M + log(Z)                                  (optional output)
//
// Two-pass softmax (max first, then sums), sequential token order, every
// operation in double.  bf16 inputs are widened exactly.  `scale` arrives as
// the fp32 value the GPU uses and is widened, so both sides multiply by the
// same number.  Slots t >= L of the last page, and pages the block table does
// not name, are never read.
//
// Pins (tests/test_oracle_pins.py): length-1 context returns v_0 bit-exactly;
// identical keys / q = 0 / scale = 0 give the mean of V; constant V is
// returned unchanged; physical page permutation under a consistent block table
// is bit-invariant; duplicating the sequence leaves the output unchanged; a
// dominant key selects its value row; an independent dense (unpaged) numpy
// softmax(QK^T*scale)V agrees to 1e-12 on tiny inputs; merging per-part
// results by their log-sum-exp reproduces the unsplit result; poisoning unread
// slots with NaN changes nothing.  The prefill form is pinned by: one query per request
// reproduces the decode oracle bit for bit; every query row equals the decode oracle on the
// context cut after its own position; an independent dense masked softmax in numpy long doubles;
// the first token of a whole prompt returns v_0; changing a later token changes no earlier row.
// No part of this oracle is unpinned.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

inline double bf16_to_double(uint16_t bits) {
    uint32_t u = static_cast<uint32_t>(bits) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

struct Layout {
    int64_t q_stride_b, q_stride_h;                 // elements; dim stride is 1
    int64_t kv_stride_page, kv_stride_head, kv_stride_tok;  // elements; dim stride is 1
    int64_t bt_stride;                              // block_table row stride (entries)
};

// One query row (q_row: head_dim bf16 values) of request b over its first L cached tokens.
// Returns 0, or a negative code on a bad table entry.
int attend_row(const uint16_t* q_row, const uint16_t* k_pool, const uint16_t* v_pool,
               const int32_t* block_table, const Layout& lay, int64_t num_pool_pages,
               int b, int kv_head, int L, int head_dim, int page_size,
               double scale, double* out_row, double* lse_out) {
    std::vector<double> s(static_cast<size_t>(L));

    // pass 1: scores and their maximum
    double M = -INFINITY;
    for (int t = 0; t < L; ++t) {
        int32_t page = block_table[b * lay.bt_stride + t / page_size];
        if (page < 0 || page >= num_pool_pages) return -1;
        const uint16_t* k_row = k_pool + page * lay.kv_stride_page + kv_head * lay.kv_stride_head +
                                (t % page_size) * lay.kv_stride_tok;
        double dot = 0.0;
        for (int d = 0; d < head_dim; ++d) dot += bf16_to_double(q_row[d]) * bf16_to_double(k_row[d]);
        s[t] = scale * dot;
        if (s[t] > M) M = s[t];
    }

    // pass 2: weights, normaliser, weighted sum of value rows
    std::vector<double> acc(static_cast<size_t>(head_dim), 0.0);
    double Z = 0.0;
    for (int t = 0; t < L; ++t) {
        double w = std::exp(s[t] - M);
        Z += w;
        int32_t page = block_table[b * lay.bt_stride + t / page_size];
        const uint16_t* v_row = v_pool + page * lay.kv_stride_page + kv_head * lay.kv_stride_head +
                                (t % page_size) * lay.kv_stride_tok;
        for (int d = 0; d < head_dim; ++d) acc[d] += w * bf16_to_double(v_row[d]);
    }
    for (int d = 0; d < head_dim; ++d) out_row[d] = acc[d] / Z;
    if (lse_out) *lse_out = M + std::log(Z);
    return 0;
}

}  // namespace

extern "C" {

// Whole batch.  out: double [batch, num_q_heads, head_dim] contiguous;
// lse: double [batch, num_q_heads] or null.  Returns 0 on success, 1 for a bad
// shape, 2 for a context length < 1, 3 for a block-table entry outside the pool.
int oserve_oracle_paged_decode_attn(
        const uint16_t* q, int64_t q_stride_b, int64_t q_stride_h,
        const uint16_t* k_pool, const uint16_t* v_pool, int64_t num_pool_pages,
        int64_t kv_stride_page, int64_t kv_stride_head, int64_t kv_stride_tok,
        const int32_t* block_table, int64_t bt_stride, const int32_t* context_lens,
        int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
        int32_t page_size, float scale, double* out, double* lse) {
    if (batch < 0 || num_q_heads < 1 || num_kv_heads < 1 || head_dim < 1 || page_size < 1) return 1;
    if (num_q_heads % num_kv_heads != 0) return 1;
    const int group = num_q_heads / num_kv_heads;
    const Layout lay{q_stride_b, q_stride_h, kv_stride_page, kv_stride_head, kv_stride_tok, bt_stride};
    for (int b = 0; b < batch; ++b) {
        const int L = context_lens[b];
        if (L < 1) return 2;
        for (int h = 0; h < num_q_heads; ++h) {
            double* out_row = out + (static_cast<int64_t>(b) * num_q_heads + h) * head_dim;
            double* lse_p = lse ? lse + static_cast<int64_t>(b) * num_q_heads + h : nullptr;
            const uint16_t* q_row = q + b * lay.q_stride_b + h * lay.q_stride_h;
            int rc = attend_row(q_row, k_pool, v_pool, block_table, lay, num_pool_pages, b, h / group, L,
                                head_dim, page_size, static_cast<double>(scale), out_row, lse_p);
            if (rc != 0) return 3;
        }
    }
    return 0;
}

// One (request, query head) of the same batch: out_row is double [head_dim].
int oserve_oracle_one_head(
        const uint16_t* q, int64_t q_stride_b, int64_t q_stride_h,
        const uint16_t* k_pool, const uint16_t* v_pool, int64_t num_pool_pages,
        int64_t kv_stride_page, int64_t kv_stride_head, int64_t kv_stride_tok,
        const int32_t* block_table, int64_t bt_stride, const int32_t* context_lens,
        int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim, int32_t page_size,
        float scale, int32_t b, int32_t h, double* out_row, double* lse) {
    if (num_q_heads < 1 || num_kv_heads < 1 || head_dim < 1 || page_size < 1) return 1;
    if (num_q_heads % num_kv_heads != 0 || h < 0 || h >= num_q_heads || b < 0) return 1;
    const int L = context_lens[b];
    if (L < 1) return 2;
    const Layout lay{q_stride_b, q_stride_h, kv_stride_page, kv_stride_head, kv_stride_tok, bt_stride};
    int rc = attend_row(q + b * lay.q_stride_b + h * lay.q_stride_h, k_pool, v_pool, block_table, lay,
                        num_pool_pages, b, h / (num_q_heads / num_kv_heads), L, head_dim, page_size,
                        static_cast<double>(scale), out_row, lse);
    return rc != 0 ? 3 : 0;
}

// Chunked prefill over the same paged cache (paper section 2: the prefill phase processes the
// prompt's tokens in parallel and is compute-bound; a chunk of it, or a whole prompt, attends
// causally).  Request b brings n = q_lens[b] new query tokens whose keys and values are already
// the last n of its L = context_lens[b] cached tokens.  Query token i (0 <= i < n) sits at
// position p = L - n + i and attends to the cached tokens 0..p, nothing later:
//
//     out[q_start_b + i][h][:] = sum_{t <= p} softmax_{t <= p}(scale * <q_i, k_t>) * v_t
//
// with q_start_b = q_lens[0] + ... + q_lens[b-1] (queries of all requests packed one after the
// other).  n = 1 is the decode step above.  q: bf16 [sum n, num_q_heads, head_dim] by strides;
// out: double [sum n, num_q_heads, head_dim] contiguous.  Returns 0; 1 bad shape; 2 a length < 1 or
// n > L; 3 block-table entry outside the pool.
int oserve_oracle_paged_prefill_attn(
        const uint16_t* q, int64_t q_stride_tok, int64_t q_stride_h,
        const uint16_t* k_pool, const uint16_t* v_pool, int64_t num_pool_pages,
        int64_t kv_stride_page, int64_t kv_stride_head, int64_t kv_stride_tok,
        const int32_t* block_table, int64_t bt_stride, const int32_t* context_lens,
        const int32_t* q_lens, int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
        int32_t head_dim, int32_t page_size, float scale, double* out) {
    if (batch < 0 || num_q_heads < 1 || num_kv_heads < 1 || head_dim < 1 || page_size < 1) return 1;
    if (num_q_heads % num_kv_heads != 0) return 1;
    const int group = num_q_heads / num_kv_heads;
    const Layout lay{q_stride_tok, q_stride_h, kv_stride_page, kv_stride_head, kv_stride_tok, bt_stride};
    int64_t row = 0;
    for (int b = 0; b < batch; ++b) {
        const int L = context_lens[b];
        const int n = q_lens[b];
        if (L < 1 || n < 1 || n > L) return 2;
        for (int i = 0; i < n; ++i, ++row) {
            const int visible = L - n + i + 1;   // tokens 0..p
            for (int h = 0; h < num_q_heads; ++h) {
                const uint16_t* q_row = q + row * lay.q_stride_b + h * lay.q_stride_h;
                double* out_row = out + (row * num_q_heads + h) * head_dim;
                int rc = attend_row(q_row, k_pool, v_pool, block_table, lay, num_pool_pages, b, h / group,
                                    visible, head_dim, page_size, static_cast<double>(scale), out_row, nullptr);
                if (rc != 0) return 3;
            }
        }
    }
    return 0;
}

}  // extern "C"
