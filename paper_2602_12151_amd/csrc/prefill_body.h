// gfx950 device code: causal chunked-prefill attention over the paged KV cache.
//
// What is computed: the prefill side of paper section 2 ("Phases of LLM inference": the prompt's
// tokens are processed in parallel, compute-bound), in the form a serving engine runs it next to
// decode steps: request b brings n_b new query tokens whose keys/values are already the last n_b
// of its L_b cached tokens; query token i sits at position p = L_b - n_b + i and attends to the
// cached tokens 0..p.  n_b = 1 is a decode step.
//
// How, on CDNA4: one workgroup of four wavefronts, one per SIMD, per (request, kv head, block of
// query tokens); registers and LDS are budgeted for two workgroups per compute unit, so that every
// SIMD holds two wavefronts of different workgroups, whose phases drift apart: one's MFMAs then
// overlap the other's softmax arithmetic.  (Measured against one workgroup of eight wavefronts in
// which every second wavefront ran its softmax and value phases a macro step late: the same speed on
// long contexts, 5 % faster on whole prompts, less LDS and no third V buffer.)  Every wavefront owns
// 32 score columns = (32 / G) query tokens x the G heads of the GQA group, so the workgroup's 128
// columns share each K/V tile.  Keys advance kMacroKeys at a time:
//   * the wavefronts bring K and V tiles of kMacroKeys keys from the page pool straight into LDS
//     (buffer loads with the LDS flag, 16 bytes per lane, no staging registers).  A load instruction
//     fills 1 KB of LDS contiguously, so rows cannot be padded; instead the 16-byte chunks of a key's
//     row are stored XOR-swizzled.  A 16-byte-per-lane LDS read is served 16 lanes at a time
//     (measured: lanes 0-3, 12-15, 20-23, 24-27 together, 4-11, 16-19, 28-31 together, the same in the
//     upper half), and those 16 must hit 16 different chunk positions of the 256-byte bank row: K
//     chunks are XOR-ed with the key index (lane l fetches chunk (l % 16) ^ key).  V is read with the
//     transposing 8-byte read, 32 lanes served together: V chunks are XOR-ed with 2 (key % 8).  One
//     barrier per kMacroKeys keys; the loads of the next macro step are in flight during the current
//     one;
//   * S^T[key][col] = K_tile * Q^T with 16x16x32 bf16 MFMA (K from LDS as the A operand, Q held in
//     registers as the B operand for the whole item);
//   * online softmax in the log2 domain, one update per column and macro step, per-column state
//     lane-local; the running "maximum" is only a reference point: the common path computes no
//     maximum, it takes the weights against the reference point it has, and only when a column's sum
//     of weights over a macro step passes 2^20 are the true maxima found (and exchanged across lanes), the reference
//     point moved and the accumulators rescaled; the causal mask is a select and is applied only on
//     the macro steps that straddle a wavefront's diagonal;
//   * O^T[dim][col] += V_tile^T * P^T with 16x16x32 bf16 MFMA over all 32 keys of the step: the
//     score layout (lane holds keys 4g..4g+3 of each 16-key half) is used as the contraction order,
//     and the transposing LDS read (ds_read_b64_tr_b16) delivers V^T in exactly that order.
//   * the column sums of the weights (the softmax normaliser) come from the matrix cores as well: a
//     product of the rounded weights with an operand of ones.
// Accumulation is fp32; P is rounded to bf16 for the second product, and the normaliser is the sum
// of those rounded weights, so an output row is an exact convex combination of value rows.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <type_traits>

#include "kernels.h"

namespace oserve {
namespace prefill_detail {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float xor_f32(float v, int mask) { return __shfl_xor(v, mask, 64); }

constexpr int kPrefillThreads = 64 * kPrefillWaves;
constexpr int kColTiles = kPrefillColTiles;
constexpr int kStepKeys = 32;
constexpr int kMacroKeys = kPrefillMacroKeys;
constexpr float kSumLimit = 1048576.f;   // a column's sum of weights over a macro step beyond this moves the reference point of the softmax

// One work item: the whole workgroup (kPrefillThreads threads: four wavefronts, one per SIMD) must
// call this with the same `ip`.  `lds` points to prefill_lds_bytes<D>() bytes of LDS;
// `sync()` is a barrier among these threads; `wave` is the wavefront's index among them.
typedef __attribute__((address_space(3))) unsigned char lds_byte;

template <int D>
constexpr int prefill_lds_bytes() { return 4 * kPrefillMacroKeys * D * 2; }   // K and V tiles, both double-buffered

struct WorkgroupBarrier {
    __device__ __forceinline__ void operator()() const { __syncthreads(); }
};

template <int D, class Sync>
__device__ __forceinline__ void prefill_item_body(const PrefillParams& p, const PrefillItem* ip, lds_byte* lds,
                                                  const Sync& sync, const int wave) {
    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    constexpr int KK = D / 32;           // 16-byte K fragments per lane per 16-key half = score MFMAs per column tile
    constexpr int EV = D / 16;           // V elements per lane per key = value MFMA row tiles
    constexpr int ROW = D * 2;           // bytes of one key's row in LDS; chunk c of key k sits at slot c ^ (k % CH) (K) or c ^ 2 (k % (CH / 2)) (V)
    constexpr int TILE = kMacroKeys * ROW;
    constexpr int SUB = kMacroKeys / kStepKeys;   // 32-key steps per macro step
    constexpr int CT = kColTiles;
    lds_byte* const lds_k = lds;              // K tiles: double-buffered
    lds_byte* const lds_v = lds + 2 * TILE;   // V tiles: likewise

    const int lane = threadIdx.x & 63;
    const int i16 = lane & 15;
    const int g4 = lane >> 4;

    // ---- the item: read by every lane from pinned host memory, then made wave-uniform ----
    const int b = __builtin_amdgcn_readfirstlane(ip->request);
    const int kvh = __builtin_amdgcn_readfirstlane(ip->kv_head);
    const int q_begin = __builtin_amdgcn_readfirstlane(ip->q_begin);
    const int q_row0 = __builtin_amdgcn_readfirstlane(ip->q_row0);   // packed row of the request's query 0
    const int L = __builtin_amdgcn_readfirstlane(ip->context_len);
    const int n = __builtin_amdgcn_readfirstlane(ip->q_len);

    // pinned to a scalar register for the whole item (it is an operand of every exponent)
    const float scale_log2e = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale_log2e)));
    const int gshift = p.group_shift;
    const int rt = (16 * CT) >> gshift;               // query tokens per wavefront
    const int tok0 = q_begin + wave * rt;             // this wavefront's first query token
    const int first_pos = L - n;                      // position of the request's query 0
    // columns c = 16*ct + i16  ->  token tok0 + (c >> gshift), head c & (2^gshift - 1), where 2^gshift
    // is the group size rounded up to a power of two; tokens past the request's last one and heads
    // past the group's last one are computed as copies of the last one and not stored
    int tok[CT], pos[CT];
    bf16x8 qf[CT][KK];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int c = 16 * ct + i16;
        tok[ct] = tok0 + (c >> gshift);
        const int t_eff = min(tok[ct], n - 1);
        pos[ct] = first_pos + t_eff;
        const int head = kvh * p.group + min(c & ((1 << gshift) - 1), p.group - 1);
        const uint16_t* qrow = p.q + (static_cast<int64_t>(q_row0 + t_eff) * p.num_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[ct][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow + (4 * kk + g4) * 8));
    }
    const int pos_min = first_pos + min(tok0, n - 1);             // wave-uniform
    const int pos_max = first_pos + min(tok0 + rt - 1, n - 1);
    const int blk_last = min(q_begin + kPrefillWaves * rt, n) - 1;   // last query token of the block
    const int num_steps = (first_pos + blk_last) / kStepKeys + 1; // keys 0..pos of that token

    // ---- where the 16-token tiles live (same walk as the decode kernel) ----
    const int32_t* bt_row = p.block_table + static_cast<int64_t>(b) * p.max_pages_per_seq;
    const int last_tile = (L - 1) >> 4;
    const int tile_mask = (1 << p.tile_shift) - 1;
    const int64_t page_elems = (static_cast<int64_t>(p.num_kv_heads) * 16 * D) << p.tile_shift;
    const int64_t head_off = (static_cast<int64_t>(kvh) * 16 * D) << p.tile_shift;

    // ---- staging: per macro step the workgroup brings kMacroKeys / 16 K tiles and as many V tiles
    // (16 keys each) into LDS: wavefront w fetches tile w of K and tile w of V (two staging slots).
    // A load instruction brings 1 KB = KPL keys (four at head_dim 128, eight at 64); a key's row has
    // CH 16-byte chunks; lane l fetches key KPL q + l / CH, and of it the chunk that belongs at slot
    // l % CH of the row: chunk (l % CH) ^ (key % CH) for K and (l % CH) ^ 2 (key % (CH / 2)) for V. ----
    constexpr int CH = D / 8;              // 16-byte chunks of a row
    constexpr int KPL = 64 / CH;           // keys per load instruction
    constexpr int LOADS = 16 / KPL;        // load instructions per tile
    constexpr int TILES = kMacroKeys / 16;
    static_assert(TILES == kPrefillWaves, "one K tile and one V tile per wavefront");
    constexpr int NS = 2;                  // staging slots of a wavefront: its K tile, its V tile
    const int st_tile = wave;              // the same tile index for both slots: one page id serves them
    bool st_is_v[NS];
    int st_lane_off[NS][LOADS];            // byte offset of this lane's chunk within the tile, per load
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
        st_is_v[sl] = sl == 1;
#pragma unroll
        for (int q = 0; q < LOADS; ++q) {
            const int key = KPL * q + lane / CH;
            st_lane_off[sl][q] = (key * D + (((lane % CH) ^ (st_is_v[sl] ? 2 * (key % (CH / 2)) : key % CH)) * 8)) * 2;
        }
    }
    // V is read back with the transposing 8-byte LDS read: in each group of 16 lanes, lane s supplies
    // the address of four consecutive dims (4 (s % 4) ..) of key 4 g4 + s / 4, and lane i receives dim i
    // of the four keys.  The 16-byte chunks of a V row are stored XOR-ed with 2 (key % (CH / 2)), which at
    // head_dim 128 spreads the 32 lanes served together over all banks.
    int v_off[EV];
    {
        const int key = 4 * g4 + (i16 >> 2);
        const int t = ((i16 & 3) >> 1) ^ (2 * (key % (CH / 2)));
#pragma unroll
        for (int e = 0; e < EV; ++e) v_off[e] = key * ROW + ((2 * e) ^ t) * 16 + (i16 & 1) * 8;
    }
    // The page id of a tile is loaded one macro step before the tile loads that need it and is only
    // looked at (made wave-uniform) right before them, after the barrier in between has waited for
    // it anyway: no wait for it of its own.
    int next_pid, next_in_page;
    auto fetch_base = [&](int macro) {   // clamped: never reads a table entry the request does not own
        const int t = min(TILES * macro + st_tile, last_tile);
        next_pid = bt_row[t >> p.tile_shift];
        next_in_page = (t & tile_mask) * (16 * D);
    };
    auto stage_of = [&](int sl, int macro) -> lds_byte* {   // where this wavefront's tile of macro step `macro` goes
        return (st_is_v[sl] ? lds_v : lds_k) + (macro & 1) * TILE + st_tile * 16 * ROW;
    };
    auto pool_of = [&](int sl) -> const uint16_t* { return st_is_v[sl] ? p.v_pages : p.k_pages; };
    // loads of the macro step whose page id was fetched last
    auto prefetch = [&](int sl, lds_byte* dst, const uint16_t* pool) __attribute__((always_inline)) {
        const int64_t next_base = static_cast<int64_t>(__builtin_amdgcn_readfirstlane(next_pid)) * page_elems +
                                  head_off + next_in_page;
        // The tile is addressed through a buffer descriptor of its own (base = the tile, 4 KB long): a
        // buffer load into LDS counts only in the vector-memory counter, whereas the compiler treats a
        // global load into LDS as outstanding in the LDS counter as well and then makes every wait for
        // an LDS read a wait for all of them.
        const uintptr_t tile = reinterpret_cast<uintptr_t>(pool + next_base);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(tile));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(tile >> 32));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            reinterpret_cast<void*>((static_cast<uintptr_t>(hi) << 32) | lo), 0, 16 * ROW, 0x00020000);
#pragma unroll
        for (int q = 0; q < LOADS; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(dst + q * KPL * ROW),
                                                     16, st_lane_off[sl][q], 0, 0, 0);
    };

    f32x4 acc[EV][CT];
#pragma unroll
    for (int e = 0; e < EV; ++e)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[e][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m[CT], l[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) { m[ct] = -INFINITY; l[ct] = 0.f; }
    // eight bf16 ones: the A operand that turns a product with the weights into their column sums
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));

    // One macro step for this wavefront's 16*CT columns runs in three phases, so that the MFMAs of a
    // phase are issued back to back: (1) all scores of the kMacroKeys keys, (2) one online-softmax
    // update per column over all of them, (3) the value products.
    f32x4 s[SUB][CT][2];     // scores; lane (i16, g4) holds, for column i16 of tile ct, keys 32*sub + 16*h + 4*g4 + r
    auto scores = [&](const lds_byte* kt) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                bf16x8 kf[KK];
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    kf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) uint4*>(
                        kt + (32 * sub + 16 * h + i16) * ROW + (((4 * kk + g4) ^ (i16 % CH)) * 16)));
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk], qf[ct][kk], a, 0, 0, 0);
                    s[sub][ct][h] = a;
                }
            }
        // order of this block's K reads and MFMAs: the fragments of two 16-key halves in flight, then
        // per half its MFMAs followed by the reads of the half after the next
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * KK, 0);
#pragma unroll
        for (int i = 0; i < 2 * SUB - 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, CT * KK, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, KK, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * CT * KK, 0);
    };
    auto softmax_and_values = [&](int macro, const lds_byte* vt, auto masked) __attribute__((always_inline)) {
        bf16x8 pb[SUB][CT];
        if constexpr (decltype(masked)::value) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int key = kMacroKeys * macro + 32 * sub + 16 * h + 4 * g4 + r;
                            s[sub][ct][h][r] = key <= pos[ct] ? s[sub][ct][h][r] : -INFINITY;
                        }
        }
        // weights of column tile ct against the reference point mref (scaled, log2 units), rounded to bf16
        auto weights = [&](int ct, float mref) __attribute__((always_inline)) {
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub) {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x2 pp;
                    pp[0] = __builtin_amdgcn_exp2f(fmaf(s[sub][ct][j >> 1][2 * (j & 1)], scale_log2e, -mref));
                    pp[1] = __builtin_amdgcn_exp2f(fmaf(s[sub][ct][j >> 1][2 * (j & 1) + 1], scale_log2e, -mref));
                    w[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2));
                }
                pb[sub][ct] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
            }
        };
        // The sum of a column's weights over the macro step comes from the matrix cores, not from
        // adds: a product of the weights with an operand of ones gives every lane the sum over all
        // the step's keys of its column (already combined across the four lanes that share the
        // column), and it is the sum of the ROUNDED weights, the ones the value product uses, so that
        // the output is an exact convex combination of value rows.
        auto column_sums = [&](int ct) __attribute__((always_inline)) -> float {
            f32x4 t = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub) t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[sub][ct], t, 0, 0, 0);
            return t[0];
        };
        // The reference point of the online softmax need not be the maximum: the result does not
        // depend on it as long as nothing overflows.  The common path therefore computes no maximum at
        // all; it takes the weights against the reference point it has and looks at their sums.  Only
        // when a column's sum is beyond kSumLimit (a weight above 2^20; on the first step, where the
        // reference point is -inf, every weight is +inf or NaN) are the true maxima computed, the
        // reference points moved, the accumulators rescaled and the weights taken again.
        float sum[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) weights(ct, m[ct]);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) sum[ct] = column_sums(ct);
        bool beyond = false;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) beyond = beyond || !(sum[ct] <= kSumLimit);
        if (__builtin_amdgcn_ballot_w64(beyond) != 0) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                float mx = -INFINITY;
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[sub][ct][h][r]);
                // the scale is positive, so raw scores order like scaled ones
                mx *= scale_log2e;
                mx = fmaxf(mx, xor_f32(mx, 16));
                mx = fmaxf(mx, xor_f32(mx, 32));
                const float m_new = fmaxf(m[ct], mx);
                const float alpha = m_new == m[ct] ? 1.f : __builtin_amdgcn_exp2f(m[ct] - m_new);
                l[ct] *= alpha;
#pragma unroll
                for (int e = 0; e < EV; ++e) acc[e][ct] *= alpha;
                m[ct] = m_new;
                weights(ct, m_new);
                sum[ct] = column_sums(ct);
            }
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) l[ct] += sum[ct];
        // value products: contraction index 8*g4 + j  <->  key 32*sub + 16*(j/4) + 4*g4 + j%4.  One
        // transposing read hands lane (i16, g4) the values of dim 16*e + i16 at keys 4*g4 .. 4*g4+3 of
        // one 16-key half: half of the A operand of tile e, no permutes.
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub) {
#pragma unroll
            for (int e = 0; e < EV; ++e) {
                s16x4 half[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    half[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(vt + (32 * sub + 16 * h) * ROW + v_off[e]));
                    if constexpr (decltype(masked)::value) {
                        // keys at or beyond the context may hold anything; their probabilities are zero, but a
                        // NaN would survive the product, so their values are zeroed
                        const int key0 = kMacroKeys * macro + 32 * sub + 16 * h + 4 * g4;
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (key0 + r >= L) half[h][r] = 0;
                    }
                }
                const bf16x8 av = __builtin_bit_cast(bf16x8, __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[e][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[sub][ct], acc[e][ct], 0, 0, 0);
            }
        }
        if constexpr (!decltype(masked)::value) {
            // Order of this block's LDS reads and MFMAs: kAhead reads in flight, then two MFMAs (one row
            // tile, both column tiles) per two reads, so that a read is waited for only after the MFMAs
            // of several earlier tiles have been issued, not right after its own issue.
            constexpr int kReads = 2 * EV * SUB, kAhead = 8;
            __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
            for (int i = 0; i < (kReads - kAhead) / 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, CT, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, CT * kAhead / 2, 0);
        }
    };
    using Plain = std::integral_constant<bool, false>;
    using Masked = std::integral_constant<bool, true>;
    // phases 2 and 3 of macro step `macro`, if any of its keys is visible to this wavefront
    auto finish = [&](int macro, const lds_byte* vt) __attribute__((always_inline)) {
        const int first_key = kMacroKeys * macro;
        if (first_key + kMacroKeys - 1 > pos_min) softmax_and_values(macro, vt, Masked{});
        else softmax_and_values(macro, vt, Plain{});
    };

    // ---- main loop: one barrier per macro step.  A compute unit holds two workgroups; the two
    // wavefronts that then share a SIMD belong to different workgroups and drift apart, so that one's
    // softmax arithmetic overlaps the other's MFMA phases.
    const int num_macro = (num_steps + SUB - 1) / SUB;
    // macro steps with a key visible to this wavefront: 0 .. my_macros-1
    const int my_macros = min(num_macro, pos_max / kMacroKeys + 1);
    // One macro step.  The tile loads it issues land in buffers that nobody reads before the next
    // barrier; the pointers are declared non-overlapping so that the LDS reads of this step are not
    // made to wait for those loads.
    auto step = [&](int macro, lds_byte* __restrict__ dst0, const uint16_t* __restrict__ pool0,
                    lds_byte* __restrict__ dst1, const uint16_t* __restrict__ pool1,
                    const lds_byte* __restrict__ kt, const lds_byte* __restrict__ vt)
                    __attribute__((always_inline)) {
        if (macro + 1 < num_macro) {
            prefetch(0, dst0, pool0);
            prefetch(1, dst1, pool1);
            fetch_base(macro + 2);     // clamped to the request's last tile
        }
        if (macro < my_macros) { scores(kt); finish(macro, vt); }
    };
    // A wavefront's tile loads into LDS must have landed before the barrier lets the others read
    // them: the wait for its outstanding vector-memory loads is written out, not left to the compiler.
    fetch_base(0);
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) prefetch(sl, stage_of(sl, 0), pool_of(sl));
    fetch_base(1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    sync();
    for (int macro = 0; macro < num_macro; ++macro) {
        step(macro, stage_of(0, macro + 1), pool_of(0), stage_of(1, macro + 1), pool_of(1), lds_k + (macro & 1) * TILE,
             lds_v + (macro & 1) * TILE);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        sync();
    }

    // ---- write out: lane holds column i16 of each tile, dims 16*e + 4*g4 + r ----
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const float l_tot = l[ct];   // every lane holds its column's whole sum
        const int c = 16 * ct + i16;
        const int head_in_group = c & ((1 << gshift) - 1);
        if (tok[ct] < n && head_in_group < p.group) {
            const int head = kvh * p.group + head_in_group;
            float* dst = p.out + (static_cast<int64_t>(q_row0 + tok[ct]) * p.num_q_heads + head) * D + 4 * g4;
            const float inv = 1.f / l_tot;
#pragma unroll
            for (int e = 0; e < EV; ++e) {
                float4 o;
                o.x = acc[e][ct][0] * inv;
                o.y = acc[e][ct][1] * inv;
                o.z = acc[e][ct][2] * inv;
                o.w = acc[e][ct][3] * inv;
                *reinterpret_cast<float4*>(dst + 16 * e) = o;
            }
        }
    }
}

}  // namespace prefill_detail
}  // namespace oserve
