// GQA attention over the paged KV cache on the gfx950 matrix cores.
//
// Page layout (per layer, page, kv head): K (16 tokens x hd) followed by V (hd x 16 tokens), 16-bit,
// each stored in MFMA operand order (see PageFrag) so that the operands come straight from HBM:
//   S^T[token][row] = sum_d K[token][d] * Q[row][d]     v_mfma_f32_16x16x32_bf16, A = K page (a lane
//                     reads 8 consecutive d of one token), B = the 16 query rows held in registers;
//   O^T[d][row]    += sum_token V^T[d][token] * P^T[token][row]   v_mfma_f32_16x16x16_bf16, A = V page
//                     (a lane reads 4 consecutive tokens of one d), B = P^T, which is exactly the
//                     register layout S^T came out in, so probabilities never leave the lane.
// A tile has 16 query rows.  Decode: the rows are the G = Hq/Hkv query heads that share one kv
// head (padded to 16), so K and V are read once per group.  Prefill: the rows are 16 consecutive
// positions of one query head, each with its own causal limit.
//
// Decode (attn_stream_kernel): the ordered stream of all (row, kv head, page) units of the batch is cut into equal
// ranges, one per workgroup; inside a range the four waves take pages round-robin, each with a private online
// softmax (running max m, sum l, unnormalised O), merged through LDS at the end of every (row, kv head) segment;
// a second small kernel merges the partial (m, l, O) of a pair that spans workgroups.
// Prefill (attn_prefill_kernel): one wave = one tile over all its pages, four heads per workgroup.
// Softmax is evaluated in base 2: scores are scaled by log2(e)/sqrt(hd) and v_exp_f32 is 2^x.
#include "spiral_internal.h"

namespace spiral {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kNegBig = -1.0e30f;

// Decode reads every K/V byte once: non-temporal loads keep the stream from displacing q, the block
// tables and the partial results in L2 (measured: 13 us less per launch at C3, -7 % step time).
// Prefill re-reads pages across heads and position tiles and keeps ordinary cached loads.
#ifndef ATTN_NT
#define ATTN_NT 1
#endif
#if ATTN_NT
#define KVLOAD(p) __builtin_nontemporal_load(p)
#else
#define KVLOAD(p) (*(p))
#endif

// q, the cached K/V and the probabilities share the 16-bit activation format (IEEE half by default:
// with bf16's 8 significant bits the attention output alone carries ~0.4 % error per layer)
__device__ __forceinline__ f32x4 mma_qk(const u32x4& k, const u32x4& q, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, k), __builtin_bit_cast(f16x8, q), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma_pv(const u32x2& v, const u32x2& p, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, v), __builtin_bit_cast(f16x4, p), c, 0, 0, 0);
}

// One (page, kv head) holds K then V, each 16 tokens x HD elements, stored in the order the MFMA
// operand registers want them, so that every wave-wide 16-byte load reads 1 KB of consecutive memory:
//   K element (token t, d):  (d/32)*512 + (((d%32)/8)*16 + t)*8 + d%8
//   V element (d, token t):  (d/32)*512 + ((t/4)*16 + d%16)*8 + ((d/16)%2)*4 + t%4
template <int HD>
struct PageFrag {
    u32x4 k[HD / 32];     // K: lane = (d%32)/8 * 16 + token, 8 consecutive d
    u32x4 v[HD / 32];     // V: lane = (t/4)*16 + d%16; .xy = 4 tokens of d-tile 2m, .zw = of d-tile 2m+1
};

template <int HD, bool NT = true>
__device__ __forceinline__ void load_page(PageFrag<HD>& f, const uint16_t* kp, int lane, bool real) {
    // !real: every lane reads the first 16 bytes of the page (a valid address, one cache line)
    const uint16_t* vp = kp + kPageTokens * HD;
    const int off = real ? lane * 8 : 0;
    const int step = real ? 512 : 0;
#pragma unroll
    for (int ks = 0; ks < HD / 32; ++ks) f.k[ks] = NT ? KVLOAD((const u32x4*)(kp + ks * step + off)) : *(const u32x4*)(kp + ks * step + off);
#pragma unroll
    for (int mp = 0; mp < HD / 32; ++mp) f.v[mp] = NT ? KVLOAD((const u32x4*)((real ? vp : kp) + mp * step + off)) : *(const u32x4*)((real ? vp : kp) + mp * step + off);
}

// ---------------------------------------------------------------------------------------------
// Causal prefill attention.  A tile is 16 consecutive positions of one query head, each row with its own
// causal limit; a workgroup holds four tiles, the same 16 positions of four adjacent heads, one per wave.
// Every wave walks all pages of its tile alone (no merge between waves); with G = 4 the four waves share
// a kv head and read the same pages at the same time, so K/V come from HBM/L2 once per workgroup.
// ---------------------------------------------------------------------------------------------
template <int HD, bool ACT32>
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnArgs a) {
    constexpr int KS = HD / 32, MT = HD / 16;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int G = a.n_q_heads / a.n_kv_heads;
    const int b = blockIdx.z, qb = blockIdx.x;
    const int h = blockIdx.y * 4 + wave;
    const int r_first = a.cu_rows[b];
    const int n_in_seq = a.cu_rows[b + 1] - r_first;
    if (qb * 16 >= n_in_seq || h >= a.n_q_heads) return;          // no barriers below: waves are independent
    const int n_valid_rows = min(16, n_in_seq - qb * 16);
    const int row0 = r_first + qb * 16;
    const int kvh = h / G;
    const int seq = a.row_seq[row0];
    const int pos0 = a.row_pos[row0];
    const int limit = li < n_valid_rows ? pos0 + li : -1;
    const int p_end = (pos0 + n_valid_rows - 1) / kPageTokens + 1;

    u32x4 qf[KS];
    {
        const uint16_t* qptr = a.q + ((size_t)(row0 + (li < n_valid_rows ? li : 0)) * a.n_q_heads + h) * HD + lg * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = *(const u32x4*)(qptr + ks * 32);
            qf[ks] = li < n_valid_rows ? v : u32x4{0u, 0u, 0u, 0u};
        }
    }
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;

    const int32_t* bt = a.block_table + (size_t)seq * a.max_blocks;
    const size_t page_elems = (size_t)a.n_kv_heads * (2 * kPageTokens * HD);
    const size_t head_off = (size_t)kvh * (2 * kPageTokens * HD);
    auto step = [&](const PageFrag<HD>& f, int pi) {
#include "attn_page_step.inc"
    };
    {
        // the next page is in flight while one is consumed; the prefetch is unconditional (past the end it re-reads
        // one valid 16-byte spot) so that the compiler's wait counts let it stay in flight during the arithmetic
        PageFrag<HD> cur, nxt;
        int pi = 0;
        load_page<HD, false>(cur, a.pages + (size_t)bt[0] * page_elems + head_off, lane, true);
        while (true) {
            const int pn = pi + 1;
            const bool more = pn < p_end;
            load_page<HD, false>(nxt, a.pages + (size_t)bt[more ? pn : pi] * page_elems + head_off, lane, more);
            step(cur, pi);
            if (!more) break;
            cur = nxt;
            pi = pn;
        }
    }

    // O^T[d][row]: lane (li, lg) holds d = mt * 16 + lg * 4 .. + 3 of row li; l is spread over the four lane groups
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (li < n_valid_rows) {
        const float inv = 1.0f / l_run;
        const size_t o_idx = ((size_t)(row0 + li) * a.n_q_heads + h) * HD + lg * 4;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            ActStore<ACT32>::put(a.out, o_idx + mt * 16 + 0, acc[mt].x * inv);
            ActStore<ACT32>::put(a.out, o_idx + mt * 16 + 1, acc[mt].y * inv);
            ActStore<ACT32>::put(a.out, o_idx + mt * 16 + 2, acc[mt].z * inv);
            ActStore<ACT32>::put(a.out, o_idx + mt * 16 + 3, acc[mt].w * inv);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Decode attention as one balanced stream over all (row, kv head, page) units of the batch.
//
// The units are ordered by (row, kv head, page); row_page_start[] is the prefix sum of the rows'
// page counts, so unit u of row r is u - row_page_start[r] * Hkv = kvh * pages(r) + page.  Workgroup
// w owns units [w * U, (w + 1) * U): every workgroup streams the same number of pages whatever the
// mix of sequence lengths, and a workgroup's range is cut into segments at (row, kv head)
// boundaries.  Within a segment the four waves take pages round-robin; at the end
// of a segment they merge through LDS and write one partial (m, l, O) into slot
// (row, kv head, w - first workgroup of that pair).  While a wave finishes a segment its first page of
// the next segment is already in flight and the next query rows are loaded under the merge, so the
// page stream does not stop at segment boundaries (a workgroup per chunk pays a start-up and a
// drain for every 16 pages: 5.2 vs 5.9 TB/s measured).
// ---------------------------------------------------------------------------------------------
template <int HD, bool ACT32>
__global__ __launch_bounds__(256) void attn_stream_kernel(AttnArgs a) {
    constexpr int KS = HD / 32, MT = HD / 16, OSTRIDE = HD + 4;
    extern __shared__ float lds_f[];
    const int G = a.n_q_heads / a.n_kv_heads;
    const int Hkv = a.n_kv_heads;
    float* s_o = lds_f;                         // [4][G][OSTRIDE]
    float* s_m = s_o + 4 * G * OSTRIDE;         // [4][16]
    float* s_l = s_m + 64;                      // [4][16]

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, lg = lane >> 4;
    const int U = a.units_per_wg;
    const int32_t* rps = a.row_page_start;
    const int T = rps[a.n_rows] * Hkv;
    int u = blockIdx.x * U;
    if (u >= T) return;
    const int u_end = min(u + U, T);

    // the row that holds unit u: the largest r with row_page_start[r] * Hkv <= u.  The prefix sums
    // increase strictly, so r + 1 is the number of entries that satisfy it: the lanes test 64 entries
    // at a time (one round of independent loads instead of a chain of dependent ones).
    int below = 0;
    for (int base = 0; base < a.n_rows; base += 64) {
        const int j = min(base + lane, a.n_rows - 1);
        const bool hit = base + lane < a.n_rows && rps[j] * Hkv <= u;
        below += __builtin_popcountll(__builtin_amdgcn_ballot_w64(hit));
    }
    const int lo = __builtin_amdgcn_readfirstlane(below) - 1;
    struct Seg { int r, kvh, p0, p1, np, rs, pos; const int32_t* bt; };
    Seg cur;
    cur.r = lo;
    cur.rs = rps[lo];
    cur.np = rps[lo + 1] - cur.rs;
    cur.kvh = (u - cur.rs * Hkv) / cur.np;
    cur.p0 = (u - cur.rs * Hkv) % cur.np;
    cur.p1 = min(cur.np, cur.p0 + (u_end - u));
    cur.pos = a.row_pos[lo];
    cur.bt = a.block_table + (size_t)a.row_seq[lo] * a.max_blocks;

    const size_t page_elems = (size_t)Hkv * (2 * kPageTokens * HD);
    constexpr int head_elems = 2 * kPageTokens * HD;

    u32x4 qf[KS];
    f32x4 acc[MT];
    float m_run, l_run;
    int limit;
    auto load_q = [&](const Seg& sg) {
        // rows >= G of the tile are padding: they read row 0's vector and are zeroed
        const uint16_t* qp = a.q + ((size_t)sg.r * a.n_q_heads + sg.kvh * G + (li < G ? li : 0)) * HD + lg * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = *(const u32x4*)(qp + ks * 32);
            qf[ks] = li < G ? v : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto reset = [&](const Seg& sg) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = kNegBig; l_run = 0.f; limit = sg.pos;
    };
    auto step = [&](const PageFrag<HD>& f, int pi) {
#include "attn_page_step.inc"
    };


    PageFrag<HD> cur_f, nxt_f;
    bool have = cur.p0 + wave < cur.p1;         // cur_f holds (or is being loaded with) this wave's first page of `cur`
    load_page<HD>(cur_f, a.pages + (size_t)cur.bt[have ? cur.p0 + wave : cur.p0] * page_elems + (size_t)cur.kvh * head_elems,
                  lane, have);
    load_q(cur);
    reset(cur);

    while (true) {
        // ---- where the next segment starts (if this workgroup has one)
        const int u_next = u + (cur.p1 - cur.p0);
        const bool has_next = u_next < u_end;
        Seg nxt = cur;
        if (has_next) {                          // cur ended at the last page of its pair
            if (cur.kvh + 1 < Hkv) {
                nxt.kvh = cur.kvh + 1;
            } else {
                nxt.r = cur.r + 1;
                nxt.kvh = 0;
                nxt.rs = cur.rs + cur.np;
                nxt.np = rps[nxt.r + 1] - nxt.rs;
                nxt.pos = a.row_pos[nxt.r];
                nxt.bt = a.block_table + (size_t)a.row_seq[nxt.r] * a.max_blocks;
            }
            nxt.p0 = 0;
            nxt.p1 = min(nxt.np, u_end - u_next);
        }
        const int pn0 = nxt.p0 + wave;
        const bool cross = has_next && pn0 < nxt.p1;

        // ---- this wave's pages of the segment, the following page always in flight
        if (have) {
            int pi = cur.p0 + wave;
            while (true) {
                const int pn = pi + 4;
                const bool more = pn < cur.p1;
                const bool real = more || cross;
                const int32_t* btp = more ? cur.bt : nxt.bt;
                const int idx = more ? pn : (cross ? pn0 : nxt.p0);      // nxt.p0 is a valid entry (nxt = cur without a successor)
                const int kv = more ? cur.kvh : nxt.kvh;
                load_page<HD>(nxt_f, a.pages + (size_t)btp[idx] * page_elems + (size_t)kv * head_elems, lane, real);
                step(cur_f, pi);
                cur_f = nxt_f;
                if (!more) break;
                pi = pn;
            }
        } else if (cross) {
            load_page<HD>(cur_f, a.pages + (size_t)nxt.bt[pn0] * page_elems + (size_t)nxt.kvh * head_elems, lane, true);
        }

        // ---- merge the four waves and write this segment's partial result
        l_run += __shfl_xor(l_run, 16, 64);
        l_run += __shfl_xor(l_run, 32, 64);
        const float m_fin = m_run, l_fin = l_run;
        f32x4 o_fin[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) o_fin[mt] = acc[mt];
        if (has_next) { load_q(nxt); reset(nxt); }     // the query rows of the next segment arrive under the merge

        __syncthreads();                               // the previous segment's merge has been read
        if (lg == 0) { s_m[wave * 16 + li] = m_fin; s_l[wave * 16 + li] = l_fin; }
        if (li < G) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                *(float4*)&s_o[(wave * G + li) * OSTRIDE + mt * 16 + lg * 4] =
                    make_float4(o_fin[mt].x, o_fin[mt].y, o_fin[mt].z, o_fin[mt].w);
        }
        __syncthreads();
        {
            const int pair_start = cur.rs * Hkv + cur.kvh * cur.np;
            const int slot = blockIdx.x - pair_start / U;
            float* dst0 = a.part + (((size_t)cur.r * Hkv + cur.kvh) * a.n_chunks + slot) * G * (HD + 2);
            for (int e = threadIdx.x; e < G * HD; e += 256) {
                const int j = e / HD, i = e % HD;
                const float M = fmaxf(fmaxf(s_m[j], s_m[16 + j]), fmaxf(s_m[32 + j], s_m[48 + j]));
                float L = 0.f, O = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float sc = __builtin_amdgcn_exp2f(s_m[w * 16 + j] - M);
                    L += s_l[w * 16 + j] * sc;
                    O += s_o[(w * G + j) * OSTRIDE + i] * sc;
                }
                float* dst = dst0 + (size_t)j * (HD + 2);
                dst[i] = O;
                if (i == 0) { dst[HD] = M; dst[HD + 1] = L; }
            }
        }
        if (!has_next) break;
        u = u_next;
        cur = nxt;
        have = cross;
    }
}

// merge the partial results of one (row, query head) written by attn_stream_kernel
template <int HD, bool ACT32>
__global__ __launch_bounds__(HD) void attn_stream_combine_kernel(AttnArgs a) {
    const int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
    const int G = a.n_q_heads / a.n_kv_heads, Hkv = a.n_kv_heads;
    const int kvh = h / G, j = h % G;
    const int rs = a.row_page_start[r], np = a.row_page_start[r + 1] - rs;
    const int first = (rs * Hkv + kvh * np) / a.units_per_wg;
    const int last = (rs * Hkv + kvh * np + np - 1) / a.units_per_wg;
    const int n_parts = last - first + 1;
    const float* base = a.part + (((size_t)r * Hkv + kvh) * a.n_chunks * G + j) * (HD + 2);
    const size_t cstride = (size_t)G * (HD + 2);
    // the first four parts (nearly always all of them) are requested at once instead of one after the other
    constexpr int PRE = 4;
    float pm[PRE], pl[PRE], po[PRE];
#pragma unroll
    for (int c = 0; c < PRE; ++c) {
        const float* src = base + (size_t)(c < n_parts ? c : n_parts - 1) * cstride;
        pm[c] = src[HD]; pl[c] = src[HD + 1]; po[c] = src[i];
    }
    float M = kNegBig;
#pragma unroll
    for (int c = 0; c < PRE; ++c)
        if (c < n_parts) M = fmaxf(M, pm[c]);
    for (int c = PRE; c < n_parts; ++c) M = fmaxf(M, base[c * cstride + HD]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int c = 0; c < PRE; ++c)
        if (c < n_parts) {
            const float sc = __builtin_amdgcn_exp2f(pm[c] - M);
            L += pl[c] * sc;
            O += po[c] * sc;
        }
    for (int c = PRE; c < n_parts; ++c) {
        const float sc = __builtin_amdgcn_exp2f(base[c * cstride + HD] - M);
        L += base[c * cstride + HD + 1] * sc;
        O += base[c * cstride + i] * sc;
    }
    ActStore<ACT32>::put(a.out, ((size_t)r * a.n_q_heads + h) * HD + i, O / L);
}

template <int HD, bool ACT32>
static hipError_t stream_impl(const AttnArgs& a, hipStream_t s) {
    const int G = a.n_q_heads / a.n_kv_heads;
    const size_t lds = (size_t)(4 * G * (HD + 4) + 128) * sizeof(float);
    const int wgs = (a.total_units + a.units_per_wg - 1) / a.units_per_wg;
    hipLaunchKernelGGL((attn_stream_kernel<HD, ACT32>), dim3(wgs), dim3(256), lds, s, a);
    return hipGetLastError();
}

template <int HD, bool ACT32>
static hipError_t stream_combine_impl(const AttnArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((attn_stream_combine_kernel<HD, ACT32>), dim3(a.n_rows, a.n_q_heads), dim3(HD), 0, s, a);
    return hipGetLastError();
}

static bool stream_args_ok(const AttnArgs& a) {
    // every (row, kv head) pair of max_pages pages must fit its partial slots: pages / U + 2 <= n_chunks
    return a.n_rows > 0 && a.row_page_start && a.units_per_wg > 0 && a.total_units > 0 && a.n_chunks > 0 &&
           a.n_q_heads / a.n_kv_heads <= kMaxGroup;
}

hipError_t launch_attn_stream(const AttnArgs& a, int hd, bool act32, hipStream_t s) {
    if (!stream_args_ok(a)) return hipErrorInvalidValue;
    switch (hd) {
        case 32:  return act32 ? stream_impl<32, true>(a, s) : stream_impl<32, false>(a, s);
        case 64:  return act32 ? stream_impl<64, true>(a, s) : stream_impl<64, false>(a, s);
        case 128: return act32 ? stream_impl<128, true>(a, s) : stream_impl<128, false>(a, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_attn_stream_combine(const AttnArgs& a, int hd, bool act32, hipStream_t s) {
    if (!stream_args_ok(a)) return hipErrorInvalidValue;
    switch (hd) {
        case 32:  return act32 ? stream_combine_impl<32, true>(a, s) : stream_combine_impl<32, false>(a, s);
        case 64:  return act32 ? stream_combine_impl<64, true>(a, s) : stream_combine_impl<64, false>(a, s);
        case 128: return act32 ? stream_combine_impl<128, true>(a, s) : stream_combine_impl<128, false>(a, s);
    }
    return hipErrorInvalidValue;
}

template <int HD, bool ACT32>
static hipError_t prefill_impl(const AttnArgs& a, int B, int max_new, hipStream_t s) {
    const int qblocks = (max_new + 15) / 16;
    hipLaunchKernelGGL((attn_prefill_kernel<HD, ACT32>), dim3(qblocks, (a.n_q_heads + 3) / 4, B), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_prefill(const AttnArgs& a, int hd, int B, int max_new, bool act32, hipStream_t s) {
    if (B <= 0 || max_new <= 0) return hipErrorInvalidValue;
    switch (hd) {
        case 32:  return act32 ? prefill_impl<32, true>(a, B, max_new, s) : prefill_impl<32, false>(a, B, max_new, s);
        case 64:  return act32 ? prefill_impl<64, true>(a, B, max_new, s) : prefill_impl<64, false>(a, B, max_new, s);
        case 128: return act32 ? prefill_impl<128, true>(a, B, max_new, s) : prefill_impl<128, false>(a, B, max_new, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace spiral
