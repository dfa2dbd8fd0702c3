// gfx950 device code: one work item of split-sequence paged GQA decode attention.
//
// What is computed is the decode-phase attention of paper section 2 ("Phases
// of LLM inference": one query vector per head over the whole KV cache of the
// request; memory-bandwidth-bound) over a cache held in fixed-size blocks
// (section 5.2).  How it is computed is this library's design for CDNA4:
//
//  * one wavefront per work item (request, kv head, sequence split); all
//    query heads of the GQA group ride in one MFMA tile, so every K/V byte is
//    fetched once per group;
//  * K and V pages (16 tokens) go from HBM straight into the register layout
//    the bf16 MFMA wants, 16 bytes per lane per load, no LDS staging:
//      S^T[token][head] = K_page[16 x D] * Q^T[D x 16]      (16x16x32 MFMA, D/32 per page)
//      O^T[dim][head]  += V_page^T[D x 16] * P^T[16 x head]  (16x16x16 MFMA, D/16 per page)
//    The result layout of the first product (lane = head + 16*(token/4), four
//    tokens per lane) is exactly the operand layout of the second, so the
//    probabilities never cross lanes, and every per-head softmax quantity
//    (running max, normaliser, rescale factor) is lane-local in both;
//  * P is fed to the MFMA as hi + lo bf16 halves (two accumulations) so the
//    product keeps ~16 mantissa bits of P; accumulation is fp32;
//  * NBUF pages of K and V are in flight per wavefront (register ring),
//    physical page ids come from scalar loads one step ahead.
//
// MFMA operand layouts used (wave64, lane = 16*g + i, i = lane % 16):
//   16x16x32 bf16: A[i][8g..8g+7], B[8g..8g+7][i] as 8 bf16 per lane; D[4g+r][i] as 4 floats.
//   16x16x16 bf16: A[i][4g..4g+3], B[4g..4g+3][i] as 4 bf16 per lane; D[4g+r][i] as 4 floats.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <type_traits>

#include "kernels.h"

namespace oserve {
namespace decode_detail {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// K and V are read exactly once per decode step, so their loads carry the non-temporal hint: the
// lines are not retained in the L2 / last-level cache.  Measured on MI355X, a plain streaming read
// reaches 6.9 TB/s with the hint against 6.1 TB/s without.
__device__ __forceinline__ uint4 load16_stream(const uint16_t* p) {
    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ uint2 load8_stream(const uint16_t* p) {
    const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    return make_uint2(w[0], w[1]);
}

__device__ __forceinline__ float wave_xor_f32(float v, int mask) { return __shfl_xor(v, mask, 64); }

// One work item, computed by the calling wavefront (all 64 lanes active; `lane` = lane index).
// kPacked: the request's rows of q and out are found through the request table (a batch in which
// requests bring different numbers of query rows); otherwise row = request index.
template <int D, int NBUF, bool kPacked>
__device__ __forceinline__ void decode_item_body(const SplitParams& p, const int item, const int lane) {
    constexpr int KK = D / 32;  // K fragments (16 B) per lane per page = QK MFMAs per page
    constexpr int EV = D / 16;  // V elements per lane per token = PV MFMA tiles per page
    constexpr int VW = EV / 2;  // 32-bit words of V per lane per token
    constexpr int PAGE = 16;

    const int i16 = lane & 15;  // MFMA row/column index: token (K operand), head (results), dim slot (V operand)
    const int g4 = lane >> 4;   // MFMA k-group

    // ---- this wavefront's item: one wave-uniform 16-byte descriptor ----
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 desc = *reinterpret_cast<const __attribute__((address_space(4))) i32x4*>(
        reinterpret_cast<uintptr_t>(p.items + item));
    const int b = desc[0] & ((1 << kKvHeadShift) - 1);
    const int kvh = desc[0] >> kKvHeadShift;
    const int pbeg = desc[1];
    const int pend = desc[2];
    const int row_group = desc[3];
    int q_row = b;       // row of the request's query in q and out
    if constexpr (kPacked) q_row = __builtin_amdgcn_readfirstlane(p.req_info[b].q_row);
    int L = 0;           // valid tokens of the request, clamped into this item's last page (set below)
    int ragged_page = -1;  // the one page that may need masking
    // ---- Q as the B operand of the score MFMA: column = head i16, k-slots = dims ----
    bf16x8 qf[KK];
    {
        const bool head_ok = i16 < p.group;
        const uint16_t* qrow = p.q + (static_cast<int64_t>(q_row) * p.num_q_heads + kvh * p.group + (head_ok ? i16 : 0)) * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            uint4 w = *reinterpret_cast<const uint4*>(qrow + (4 * kk + g4) * 8);
            if (!head_ok) w = make_uint4(0u, 0u, 0u, 0u);
            qf[kk] = __builtin_bit_cast(bf16x8, w);
        }
    }

    // ---- where each 16-token tile lives: wave-uniform (scalar) block-table loads, fetched one step
    // before they are needed.  A page holds 1 << tile_shift tiles, one after the other.
    const int32_t* bt_row = p.block_table + static_cast<int64_t>(b) * p.max_pages_per_seq;
    const int last_page = pend - 1;
    const int tile_mask = (1 << p.tile_shift) - 1;
    const int64_t page_elems = (static_cast<int64_t>(p.num_kv_heads) * PAGE * D) << p.tile_shift;
    const int64_t head_off = (static_cast<int64_t>(kvh) * PAGE * D) << p.tile_shift;
    auto tile_base_of = [&](int pg) -> int64_t {  // clamped: never reads a table entry the request does not own
        const int t = min(pg, last_page);
        const int pid = __builtin_amdgcn_readfirstlane(bt_row[t >> p.tile_shift]);
        return static_cast<int64_t>(pid) * page_elems + head_off + (t & tile_mask) * (PAGE * D);
    };

    const int k_lane_off = i16 * D + g4 * 8;         // + 32*kk elements
    const int v_lane_off = (4 * g4) * D + EV * i16;  // + c*D elements

    uint4 kbuf[NBUF][KK];
    uint32_t vbuf[NBUF][4][VW];

    auto issue = [&](int slot, int64_t base) {
        const uint16_t* kp = p.k_pages + base + k_lane_off;
        const uint16_t* vp = p.v_pages + base + v_lane_off;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kbuf[slot][kk] = load16_stream(kp + 32 * kk);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if constexpr (VW == 4) {
                const uint4 w = load16_stream(vp + c * D);
                vbuf[slot][c][0] = w.x; vbuf[slot][c][1] = w.y; vbuf[slot][c][2] = w.z; vbuf[slot][c][3] = w.w;
            } else {
                const uint2 w = load8_stream(vp + c * D);
                vbuf[slot][c][0] = w.x; vbuf[slot][c][1] = w.y;
            }
        }
    };

    f32x4 acc[EV];
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY;  // running max of (score * scale * log2 e) for head i16
    float l = 0.f;        // this lane's share of the normaliser (its 4 tokens per page)

    // One page: scores, online-softmax update, PV accumulate.  `masked` (compile-time) is set only
    // for a request's ragged last page.
    auto consume = [&](int slot, int pg, auto masked) {
        // scores: S^T[token 4*g4+r][head i16]
        f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kbuf[slot][kk]), qf[kk], s, 0, 0, 0);
        float x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = s[r] * p.scale_log2e;

        uint32_t vw[4][VW];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int w = 0; w < VW; ++w) vw[c][w] = vbuf[slot][c][w];
        if constexpr (decltype(masked)::value) {
            // mask by select: the slots past the context may hold anything, NaN included
            const int valid = L - pg * PAGE;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = 4 * g4 + r < valid;
                x[r] = ok ? x[r] : -INFINITY;
#pragma unroll
                for (int w = 0; w < VW; ++w) vw[r][w] = ok ? vw[r][w] : 0u;
            }
        }

        // The running max m is kept equal in the four lanes that share a head.  Lanes exchange
        // maxima only when some lane's own tokens beat m (rare after the first pages).
        const float mx_own = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
        if (__builtin_amdgcn_ballot_w64(mx_own > m) != 0) {
            float mx = fmaxf(mx_own, wave_xor_f32(mx_own, 16));
            mx = fmaxf(mx, wave_xor_f32(mx, 32));
            const float m_new = fmaxf(m, mx);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            l *= alpha;
#pragma unroll
            for (int e = 0; e < EV; ++e) acc[e] *= alpha;
            m = m_new;
        }
        f32x2 p01, p23;
        p01[0] = __builtin_amdgcn_exp2f(x[0] - m);
        p01[1] = __builtin_amdgcn_exp2f(x[1] - m);
        p23[0] = __builtin_amdgcn_exp2f(x[2] - m);
        p23[1] = __builtin_amdgcn_exp2f(x[3] - m);
        l += (p01[0] + p01[1]) + (p23[0] + p23[1]);

        // P^T as the B operand (k = token 4*g4+r, column = head): hi and lo bf16 halves, p = hi + lo + O(2^-17 p)
        const uint32_t h01 = __builtin_bit_cast(uint32_t, __builtin_convertvector(p01, bf16x2));
        const uint32_t h23 = __builtin_bit_cast(uint32_t, __builtin_convertvector(p23, bf16x2));
        f32x2 r01, r23;
        r01[0] = p01[0] - __uint_as_float(h01 << 16);
        r01[1] = p01[1] - __uint_as_float(h01 & 0xFFFF0000u);
        r23[0] = p23[0] - __uint_as_float(h23 << 16);
        r23[1] = p23[1] - __uint_as_float(h23 & 0xFFFF0000u);
        const uint32_t l01 = __builtin_bit_cast(uint32_t, __builtin_convertvector(r01, bf16x2));
        const uint32_t l23 = __builtin_bit_cast(uint32_t, __builtin_convertvector(r23, bf16x2));
        const short4v p_hi = __builtin_bit_cast(short4v, make_uint2(h01, h23));
        const short4v p_lo = __builtin_bit_cast(short4v, make_uint2(l01, l23));

        // V^T as the A operand: row = dim slot i16 (dim EV*i16+e), k = token 4*g4+c
#pragma unroll
        for (int e = 0; e < EV; ++e) {
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
            const uint2 vt = make_uint2(__builtin_amdgcn_perm(vw[1][e >> 1], vw[0][e >> 1], sel),
                                        __builtin_amdgcn_perm(vw[3][e >> 1], vw[2][e >> 1], sel));
            const short4v a = __builtin_bit_cast(short4v, vt);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, p_hi, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, p_lo, acc[e], 0, 0, 0);
        }
    };
    using Full = std::integral_constant<bool, false>;
    using Ragged = std::integral_constant<bool, true>;

    // ---- pipeline: NBUF-1 pages in flight ahead of the one being consumed ----
    // Steady state issues the loads of page pg+NBUF-1 unconditionally before consuming page pg, so
    // the only wait is for the oldest page; the last NBUF-1 pages are drained without new loads.
    // An item shorter than NBUF-1 pages re-loads its last page in the prologue (harmless).
    int64_t base_ring[NBUF];
#pragma unroll
    for (int u = 0; u < NBUF; ++u) base_ring[u] = tile_base_of(pbeg + u);
#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) issue(u, base_ring[u]);
    int64_t next_base = base_ring[NBUF - 1];

    // The device copy of the length only decides how much of the page it falls in counts: a value
    // that disagrees with the plan is clamped into the last page this item owns.  It is fetched
    // here, after the first pages are on their way, because nothing needs it before the item's end.
    __builtin_amdgcn_sched_barrier(0);
    L = __builtin_amdgcn_readfirstlane(p.context_lens[b]);
    L = min(max(L, (pend - 1) * PAGE + 1), pend * PAGE);
    ragged_page = (L & (PAGE - 1)) ? pend - 1 : -1;

    auto drain = [&](int slot, int pg) {
#pragma unroll
        for (int k = 0; k < NBUF - 1; ++k)
            if (pg + k < pend) {
                if (pg + k == ragged_page) consume((slot + k) % NBUF, pg + k, Ragged{});
                else consume((slot + k) % NBUF, pg + k, Full{});
            }
    };

    const int main_end = pend - (NBUF - 1);
    int pg = pbeg;
    bool more = true;
    while (more) {
#pragma unroll
        for (int u = 0; u < NBUF; ++u) {
            if (more) {
                if (pg < main_end) {
                    issue((u + NBUF - 1) % NBUF, next_base);
                    next_base = tile_base_of(pg + NBUF);
                    consume(u, pg, Full{});  // the ragged page, if any, is the item's last: never here
                    ++pg;
                } else {
                    drain(u, pg);
                    more = false;
                }
            }
        }
    }

    // ---- write out: lane holds head i16, dims [4*EV*g4, 4*EV*(g4+1)) ----
    float l_tot = l + wave_xor_f32(l, 16);
    l_tot += wave_xor_f32(l_tot, 32);
    if (i16 < p.group) {
        const int h = kvh * p.group + i16;
        float* dst;
        float mul = 1.f;
        if (row_group < 0) {
            dst = p.out + (static_cast<int64_t>(q_row) * p.num_q_heads + h) * D;
            mul = 1.f / l_tot;
        } else {
            const int64_t row = static_cast<int64_t>(row_group) * p.num_q_heads + h;
            dst = p.partial_o + row * D;
            if (g4 == 0) {
                p.partial_ml[row * 2] = m;
                p.partial_ml[row * 2 + 1] = l_tot;
            }
        }
        dst += 4 * EV * g4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
            for (int e4 = 0; e4 < EV / 4; ++e4) {
                float4 o;
                o.x = acc[4 * e4 + 0][r] * mul;
                o.y = acc[4 * e4 + 1][r] * mul;
                o.z = acc[4 * e4 + 2][r] * mul;
                o.w = acc[4 * e4 + 3][r] * mul;
                *reinterpret_cast<float4*>(dst + r * EV + 4 * e4) = o;
            }
        }
    }
}

}  // namespace decode_detail
}  // namespace oserve
