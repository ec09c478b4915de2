// Weight-streaming projection kernel for the decode step (K a multiple of 128).
//
// out[m][n] = sum_k A[m][k] * W[n][k], M <= 128 rows per tile.  Every weight byte is used once, so
// the kernel is a stream over W; at M = 128 it also needs ~40 % of the matrix-core peak while
// streaming, which is why it is built on v_mfma_f32_32x32x16 (on gfx950 the 16x16x32 form issues
// at half the rate: 32 cycles for half the flops, measured).
//   * A workgroup (4 waves) owns 32*WN weight rows and all (<= 128) batch rows of its M tile.  The
//     waves form a WN x WM grid (WN*WM = 4): wave (wn, wm) multiplies weight rows [32 wn, 32 wn + 32)
//     with its 1/WM share of the batch rows, so no reduction between waves is needed.
//   * Weights go HBM -> registers directly in MFMA operand layout (lane = row l%32, 8 consecutive k at
//     (l/32)*8: one 16-byte load per k step of 16), PD chunks of 128 k ahead of use.
//   * The activations of a chunk (<= 128 rows x 128 k, re-read from L2) are loaded cooperatively by
//     the 256 threads in the same pipeline stage, parked in LDS (row stride 272 B) and read by the
//     waves as the other MFMA operand.  LDS is double buffered, one barrier per chunk.
//   * All prefetch loads are unconditional (past the end of the K range they re-read a valid
//     address): a branch around a load makes the compiler wait for every outstanding load.
// A grid-level split of K (blockIdx.y) supplies enough workgroups for the narrow projections; the
// consumer kernel adds the partial results in a fixed order (bit-reproducible, no float atomics).
#include <algorithm>

#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

// The weights are read once per step: non-temporal loads (no L2 allocation) leave L2 to the activation
// tile that every workgroup re-reads (LM head 188 -> 180 us, measured).
#ifndef STREAM_NT
#define STREAM_NT 1
#endif
#if STREAM_NT
#define WLOAD(p) __builtin_nontemporal_load(p)
#else
#define WLOAD(p) (*(p))
#endif

typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mma32(const u32x4& w, const u32x4& a, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, a), c, 0, 0, 0);
}

template <int M32>
struct Stage {
    u32x4 a[2 * M32];     // this thread's share of the activation chunk (32*M32 rows x 256 B)
    u32x4 w[8];           // this lane's weight fragments: 8 k steps of 16
};

// M32: batch tiles of 32 rows per workgroup; WN: waves along the weight rows (WM = 4 / WN along the
// batch); SWIGLU: waves wn < WN/2 hold gate rows, the others the matching up rows.
template <int M32, int WN, bool SWIGLU, int PD, bool FRAG = false, bool SAMPLE = false>
__global__ __launch_bounds__(256) void gemm_stream_kernel(GemmArgs g) {
    constexpr int WM = 4 / WN;
    constexpr int MW = M32 / WM;                    // batch tiles per wave
    static_assert(M32 % WM == 0, "every wave needs at least one batch tile");
    constexpr int ROWB = 272;                       // LDS bytes per activation row (256 + 16 pad)
    constexpr int BUF = 32 * M32 * ROWB;
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wn = wave / WM, wm = wave % WM;
    const int tile_m = blockIdx.x % g.m_tiles;
    const int tile_n = blockIdx.x / g.m_tiles;
    const int split = blockIdx.y;
    const int K = g.K;
    const int m0 = tile_m * (32 * M32);

    // ---- the 32 weight rows of this wave
    const uint16_t* wrow;
    int n_first;                                    // first output (or ffn) column of this wave
    if (SWIGLU) {
        constexpr int H = WN / 2;
        n_first = tile_n * (32 * H) + (wn % H) * 32;
        int f = n_first + l32; if (f >= g.N) f = g.N - 1;
        wrow = (const uint16_t*)(wn < H ? g.w[0] : g.w[1]) + (size_t)f * K + lh * 8;
    } else {
        n_first = tile_n * (32 * WN) + wn * 32;
        int n = n_first + l32; if (n >= g.N) n = g.N - 1;
        const uint16_t* base; int row;
        if (n < g.rows[0]) { base = (const uint16_t*)g.w[0]; row = n; }
        else if (n < g.rows[0] + g.rows[1]) { base = (const uint16_t*)g.w[1]; row = n - g.rows[0]; }
        else { base = (const uint16_t*)g.w[2]; row = n - g.rows[0] - g.rows[1]; }
        wrow = base + (size_t)row * K + lh * 8;
        if (FRAG) {
            const int t32 = min(tile_n * WN + wn, (g.N + 31) / 32 - 1);
            wrow = (const uint16_t*)g.wf + frag_block(t32, 0, K) + lane * 8;
        }
    }

    // ---- this thread's share of an activation chunk: 2*M32 segments of 16 B (row = s / 16, column = s % 16)
    const uint16_t* a_src[2 * M32];
    int a_dst[2 * M32];
#pragma unroll
    for (int i = 0; i < 2 * M32; ++i) {
        const int s = threadIdx.x + 256 * i;
        const int row = s >> 4, c16 = s & 15;
        int m = m0 + row; if (m >= g.M) m = g.M - 1;
        a_src[i] = (const uint16_t*)g.A + (size_t)m * K + c16 * 8;
        a_dst[i] = row * ROWB + c16 * 16;
    }
    // operand read: batch row (wm*MW + t)*32 + l32, k = ks*16 + lh*8
    const int frag_off = (wm * MW * 32 + l32) * ROWB + lh * 16;

    // ---- chunk range of this workgroup
    const int chunks = K >> 7;
    const int cb = (int)(((long long)chunks * split) / g.splits);
    const int ce = (int)(((long long)chunks * (split + 1)) / g.splits);
    const int NC = ce - cb;

    f32x16 acc[MW];
#pragma unroll
    for (int t = 0; t < MW; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    Stage<M32> st[PD];
    auto load = [&](Stage<M32>& S, int chunk) {
        const int cc = chunk < ce ? chunk : ce - 1;        // past the end: re-read the last chunk (cache hit)
        const size_t off = (size_t)cc * 128;
#pragma unroll
        for (int i = 0; i < 2 * M32; ++i) S.a[i] = *(const u32x4*)(a_src[i] + off);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            S.w[ks] = FRAG ? WLOAD((const u32x4*)(wrow + ((size_t)cc * 8 + ks) * 512)) : *(const u32x4*)(wrow + off + ks * 16);
    };
    auto iter = [&](Stage<M32>& S, int c) {
        char* buf = lds + (c & 1) * BUF;
#pragma unroll
        for (int i = 0; i < 2 * M32; ++i) *(u32x4*)(buf + a_dst[i]) = S.a[i];
        __syncthreads();
        // operand reads from LDS run one k step ahead of the MFMAs that consume them
        u32x4 af[2][MW];
#pragma unroll
        for (int t = 0; t < MW; ++t) af[0][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks + 1 < 8) {
#pragma unroll
                for (int t = 0; t < MW; ++t)
                    af[(ks + 1) & 1][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB + (ks + 1) * 32);
            }
            const u32x4 wp = FRAG ? S.w[ks] : prep_w(S.w[ks]);      // fragment-ordered copies are already widened
#pragma unroll
            for (int t = 0; t < MW; ++t) acc[t] = mma32(wp, af[ks & 1][t], acc[t]);
        }
        load(S, cb + c + PD);
    };

#pragma unroll
    for (int i = 0; i < PD; ++i) load(st[i], cb + i);
    int c = 0;
    for (; c + PD <= NC; c += PD) {
#pragma unroll
        for (int i = 0; i < PD; ++i) iter(st[i], c + i);
    }
#pragma unroll
    for (int i = 0; i < PD - 1; ++i)
        if (c + i < NC) iter(st[i], c + i);

    // ---- epilogue.  Accumulator layout of the 32x32 tile: lane holds batch row l32 and, in registers
    //      4b .. 4b+3, the weight rows 8b + 4*lh .. +3 (b = 0..3): four consecutive output columns each.
    if (!SWIGLU && SAMPLE) {
        // LM head without logits: score = logit / T + noise (the sampler's own expression), the best (score, index)
        // of the workgroup's columns per batch row goes to s_part[row][tile_n]; a second kernel picks among tiles.
        constexpr int R = 32 * M32;
        __syncthreads();                             // every wave is done with the activation buffers
        float* s_val = (float*)lds;                  // [WN][R]
        int* s_idx = (int*)(lds + WN * R * 4);
        const float T = g.s_temperature;
#pragma unroll
        for (int t = 0; t < MW; ++t) {
            const int row = (wm * MW + t) * 32 + l32;
            const int m = m0 + row;
            const uint64_t key = (T > 0.f && m < g.M) ? g.s_keys[m] : 0ull;
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int n = n_first + 8 * b + 4 * lh + i;
                    float sc = acc[t][4 * b + i];
                    if (T > 0.f) sc = sc / T + gumbel_noise(key, n);
                    if (n < g.N && better(sc, n, bv, bi)) { bv = sc; bi = n; }
                }
            const float ov = __shfl_xor(bv, 32, 64);
            const int oi = __shfl_xor(bi, 32, 64);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            if (lh == 0) { s_val[wn * R + row] = bv; s_idx[wn * R + row] = bi; }
        }
        __syncthreads();
        if ((int)threadIdx.x < R) {
            const int row = threadIdx.x, m = m0 + row;
            float bv = s_val[row];
            int bi = s_idx[row];
#pragma unroll
            for (int w = 1; w < WN; ++w)
                if (better(s_val[w * R + row], s_idx[w * R + row], bv, bi)) { bv = s_val[w * R + row]; bi = s_idx[w * R + row]; }
            if (m < g.M) g.s_part[(size_t)m * g.s_tiles + tile_n] = make_float2(bv, __int_as_float(bi));
        }
    } else if (!SWIGLU) {
        // Stores go through LDS so that every store instruction writes whole 128-byte lines (8 lanes x 16 B per
        // row, 8 rows): written straight from the accumulator layout a wave store touches 32 rows x 32 B, and the
        // partial-line traffic costs a quarter of the kernel (LM head 188 -> 143 us without its stores).
        float* out = (float*)g.out + (size_t)split * g.M * g.N;
        constexpr int TROW = 144;                    // bytes per staged row: 32 floats + 16 pad
        __syncthreads();                             // every wave is done with the activation buffers
        char* tb = lds + wave * (32 * TROW);         // this wave's own staging tile
        const int rr = lane >> 3, cg = lane & 7;     // read side: row rr + 8 * pass, floats 4 cg .. 4 cg + 3
#pragma unroll
        for (int t = 0; t < MW; ++t) {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                *(float4*)(tb + l32 * TROW + (8 * b + 4 * lh) * 4) =
                    make_float4(acc[t][4 * b], acc[t][4 * b + 1], acc[t][4 * b + 2], acc[t][4 * b + 3]);
            __builtin_amdgcn_wave_barrier();
            const int n = n_first + 4 * cg;
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                const int row = rr + 8 * ps;
                const float4 v = *(const float4*)(tb + row * TROW + cg * 16);
                const int m = m0 + (wm * MW + t) * 32 + row;
                if (m < g.M && n < g.N) *(float4*)(out + (size_t)m * g.N + n) = v;
            }
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        constexpr int H = WN / 2;
        // the up-projection waves hand their tiles to the gate waves through LDS
        __syncthreads();                            // everyone is done with the activation buffers
        float4* x = (float4*)lds;
        const int pair = (wn % H) * WM + wm;        // gate wave and up wave of the same tile share this slot
        if (wn >= H) {
#pragma unroll
            for (int t = 0; t < MW; ++t)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    x[((pair * MW + t) * 4 + b) * 64 + lane] =
                        make_float4(acc[t][4 * b], acc[t][4 * b + 1], acc[t][4 * b + 2], acc[t][4 * b + 3]);
        }
        __syncthreads();
        if (wn >= H) return;
        bool bad = false;
#pragma unroll
        for (int t = 0; t < MW; ++t) {
            const int m = m0 + (wm * MW + t) * 32 + l32;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int f = n_first + 8 * b + 4 * lh;
                const float4 u = x[((pair * MW + t) * 4 + b) * 64 + lane];
                if (m < g.M && f < g.N) {
                    ushort4 o;
                    o.x = f32_to_act16_noting(silu_f(acc[t][4 * b]) * u.x, bad);
                    o.y = f32_to_act16_noting(silu_f(acc[t][4 * b + 1]) * u.y, bad);
                    o.z = f32_to_act16_noting(silu_f(acc[t][4 * b + 2]) * u.z, bad);
                    o.w = f32_to_act16_noting(silu_f(acc[t][4 * b + 3]) * u.w, bad);
                    *(ushort4*)((uint16_t*)g.out + (size_t)m * g.N + f) = o;
                }
            }
        }
        report_saturation(g.sat_count, bad);
    }
}

// Gate/up projection with the SwiGLU epilogue kept in registers.  A wave's 32 weight rows are 16
// gate rows followed by the 16 up rows of the same ffn columns, so in the 32x32 accumulator tile a
// lane holds gate values in registers 0..7 and the matching up values in registers 8..15: no
// exchange between waves.  NW waves per workgroup, each with all M32 batch tiles; NW is chosen on
// the host so that the workgroups fill the 256 compute units in one round (9728 ffn columns are
// 608 wave tiles: 203 workgroups of 3 use every unit at most 3 tiles deep, 152 of 4 leave 104 idle).
template <int M32, int NW, int PD, bool FRAG = false>
__global__ __launch_bounds__(64 * NW) void swiglu_stream_kernel(GemmArgs g) {
    constexpr int NT = 64 * NW;
    constexpr int ROWB = 272;
    constexpr int BUF = 32 * M32 * ROWB;
    constexpr int NSEG = 32 * M32 * 16;             // 16-byte segments of an activation chunk
    constexpr int AI = (NSEG + NT - 1) / NT;
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tile_m = blockIdx.x % g.m_tiles;
    const int tile_n = blockIdx.x / g.m_tiles;
    const int K = g.K;
    const int m0 = tile_m * (32 * M32);

    const int f_first = (tile_n * NW + wave) * 16;  // first ffn column of this wave
    int f = f_first + (l32 & 15); if (f >= g.N) f = g.N - 1;
    const uint16_t* wrow = (const uint16_t*)(l32 < 16 ? g.w[0] : g.w[1]) + (size_t)f * K + lh * 8;
    if (FRAG)       // the interleaved gate/up matrix: tile t holds ffn columns 16 t .. 16 t + 15
        wrow = (const uint16_t*)g.wf + frag_block(min(tile_n * NW + wave, (g.N + 15) / 16 - 1), 0, K) + lane * 8;

    const uint16_t* a_src[AI];
    int a_dst[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) {
        int sgm = threadIdx.x + NT * i; if (sgm >= NSEG) sgm = NSEG - 1;   // the tail repeats the last segment
        const int row = sgm >> 4, c16 = sgm & 15;
        int m = m0 + row; if (m >= g.M) m = g.M - 1;
        a_src[i] = (const uint16_t*)g.A + (size_t)m * K + c16 * 8;
        a_dst[i] = row * ROWB + c16 * 16;
    }
    const int frag_off = l32 * ROWB + lh * 16;
    const int NC = K >> 7;

    f32x16 acc[M32];
#pragma unroll
    for (int t = 0; t < M32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    struct St { u32x4 a[AI]; u32x4 w[8]; };
    St st[PD];
    auto load = [&](St& S, int chunk) {
        const int cc = chunk < NC ? chunk : NC - 1;
        const size_t off = (size_t)cc * 128;
#pragma unroll
        for (int i = 0; i < AI; ++i) S.a[i] = *(const u32x4*)(a_src[i] + off);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            S.w[ks] = FRAG ? WLOAD((const u32x4*)(wrow + ((size_t)cc * 8 + ks) * 512)) : *(const u32x4*)(wrow + off + ks * 16);
    };
    auto iter = [&](St& S, int c) {
        char* buf = lds + (c & 1) * BUF;
#pragma unroll
        for (int i = 0; i < AI; ++i) *(u32x4*)(buf + a_dst[i]) = S.a[i];
        __syncthreads();
        u32x4 af[2][M32];
#pragma unroll
        for (int t = 0; t < M32; ++t) af[0][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks + 1 < 8) {
#pragma unroll
                for (int t = 0; t < M32; ++t)
                    af[(ks + 1) & 1][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB + (ks + 1) * 32);
            }
            const u32x4 wp = FRAG ? S.w[ks] : prep_w(S.w[ks]);      // fragment-ordered copies are already widened
#pragma unroll
            for (int t = 0; t < M32; ++t) acc[t] = mma32(wp, af[ks & 1][t], acc[t]);
        }
        load(S, c + PD);
    };

#pragma unroll
    for (int i = 0; i < PD; ++i) load(st[i], i);
    int c = 0;
    for (; c + PD <= NC; c += PD) {
#pragma unroll
        for (int i = 0; i < PD; ++i) iter(st[i], c + i);
    }
#pragma unroll
    for (int i = 0; i < PD - 1; ++i)
        if (c + i < NC) iter(st[i], c + i);

    // registers 4b..4b+3 hold tile rows 8b + 4*lh .. +3: b = 0, 1 are gate rows, b = 2, 3 the up rows 16 below
    bool bad = false;
#pragma unroll
    for (int t = 0; t < M32; ++t) {
        const int m = m0 + t * 32 + l32;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int fo = f_first + 8 * b + 4 * lh;
            if (m < g.M && fo < g.N) {
                ushort4 o;
                o.x = f32_to_act16_noting(silu_f(acc[t][4 * b]) * acc[t][4 * b + 8], bad);
                o.y = f32_to_act16_noting(silu_f(acc[t][4 * b + 1]) * acc[t][4 * b + 9], bad);
                o.z = f32_to_act16_noting(silu_f(acc[t][4 * b + 2]) * acc[t][4 * b + 10], bad);
                o.w = f32_to_act16_noting(silu_f(acc[t][4 * b + 3]) * acc[t][4 * b + 11], bad);
                *(ushort4*)((uint16_t*)g.out + (size_t)m * g.N + fo) = o;
            }
        }
    }
    report_saturation(g.sat_count, bad);
}

template <int M32, int NW, int PD>
static hipError_t launch_swiglu(const GemmArgs& a, hipStream_t s) {
    GemmArgs g = a;
    g.m_tiles = (a.M + 32 * M32 - 1) / (32 * M32);
    const int n_tiles = (a.N + 16 * NW - 1) / (16 * NW);
    const size_t lds_bytes = (size_t)2 * 32 * M32 * 272;
    if (a.wf) hipLaunchKernelGGL((swiglu_stream_kernel<M32, NW, PD, true>), dim3(n_tiles * g.m_tiles), dim3(64 * NW), lds_bytes, s, g);
    else hipLaunchKernelGGL((swiglu_stream_kernel<M32, NW, PD, false>), dim3(n_tiles * g.m_tiles), dim3(64 * NW), lds_bytes, s, g);
    return hipGetLastError();
}

// Waves per workgroup for the gate/up kernel: the count in {4, 5, 3} (ties in this order) that needs
// the fewest tile-deep rounds over the compute units.
static int swiglu_waves(int N, int m_tiles) {
    const int units = (N + 15) / 16;
    int best = 4; long best_cost = -1;
    for (int nw : {4, 5, 3}) {
        const long wgs = (long)((units + nw - 1) / nw) * m_tiles;
        const long cost = ((wgs + 255) / 256) * nw;
        if (best_cost < 0 || cost < best_cost) { best = nw; best_cost = cost; }
    }
    return best;
}

template <int M32, int WN, bool SWIGLU, int PD>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s, bool sample = false) {
    GemmArgs g = a;
    g.m_tiles = (a.M + 32 * M32 - 1) / (32 * M32);
    const int cols = SWIGLU ? 16 * WN : 32 * WN;
    const int n_tiles = (a.N + cols - 1) / cols;
    size_t lds_bytes = (size_t)2 * 32 * M32 * 272;
    if (SWIGLU) lds_bytes = std::max(lds_bytes, (size_t)2 * M32 * 4 * 64 * sizeof(float4));
    else lds_bytes = std::max(lds_bytes, (size_t)4 * 32 * 144);       // the four waves' output staging tiles
    if (sample) {
        if (SWIGLU || !a.wf || g.splits != 1 || !a.s_part || a.s_tiles != n_tiles) return hipErrorInvalidValue;
        hipLaunchKernelGGL((gemm_stream_kernel<M32, WN, false, PD, true, true>), dim3(n_tiles * g.m_tiles, 1), dim3(256),
                           lds_bytes, s, g);
    } else if (!SWIGLU && a.wf)
        hipLaunchKernelGGL((gemm_stream_kernel<M32, WN, false, PD, true>), dim3(n_tiles * g.m_tiles, g.splits), dim3(256),
                           lds_bytes, s, g);
    else
        hipLaunchKernelGGL((gemm_stream_kernel<M32, WN, SWIGLU, PD, false>), dim3(n_tiles * g.m_tiles, g.splits), dim3(256),
                           lds_bytes, s, g);
    return hipGetLastError();
}

template <bool SWIGLU>
static hipError_t launch_shape(const GemmArgs& a, int bn, hipStream_t s, bool sample = false) {
    // bn = weight rows per workgroup (128 or 64); narrower workgroups split the batch between waves
    if (a.M <= 32) return launch_one<1, 4, SWIGLU, 4>(a, s, sample);
    if (a.M <= 64) return bn >= 128 ? launch_one<2, 4, SWIGLU, 3>(a, s, sample) : launch_one<2, 2, SWIGLU, 3>(a, s, sample);
#ifndef STREAM_PD
#define STREAM_PD 2
#endif
#ifndef SWIGLU_PD
#define SWIGLU_PD 2
#endif
    return bn >= 128 ? launch_one<4, 4, SWIGLU, STREAM_PD>(a, s, sample) : launch_one<4, 2, SWIGLU, 3>(a, s, sample);
}

// columns of the LM head that one workgroup of the sampling epilogue covers (host code sizes s_part with it)
int gemm_sample_tile_cols(int M, int bn) { return (M > 32 && bn < 128) ? 64 : 128; }

hipError_t launch_gemm_stream(const GemmArgs& a, int epilogue, int bn, hipStream_t s) {
    if ((a.K & 127) || (a.N & 15) || a.splits < 1 || a.splits > (a.K >> 7)) return hipErrorInvalidValue;
    if (epilogue == EPI_SWIGLU) {
        if (a.splits != 1) return hipErrorInvalidValue;
        if (bn != 64) {
            // bn = 96 / 128 / 160 picks 3 / 4 / 5 waves, anything else the count that fills the chip best
            const int rows_wg = a.M <= 32 ? 32 : a.M <= 64 ? 64 : 128;
            const int nw = (bn == 96 || bn == 128 || bn == 160) ? bn / 32 : swiglu_waves(a.N, (a.M + rows_wg - 1) / rows_wg);
            if (a.M <= 32) return nw == 3 ? launch_swiglu<1, 3, 4>(a, s) : nw == 5 ? launch_swiglu<1, 5, 4>(a, s) : launch_swiglu<1, 4, 4>(a, s);
            if (a.M <= 64) return nw == 3 ? launch_swiglu<2, 3, 3>(a, s) : nw == 5 ? launch_swiglu<2, 5, 2>(a, s) : launch_swiglu<2, 4, 3>(a, s);
            return nw == 3 ? launch_swiglu<4, 3, SWIGLU_PD>(a, s) : nw == 5 ? launch_swiglu<4, 5, 2>(a, s) : launch_swiglu<4, 4, 2>(a, s);
        }
        return launch_shape<true>(a, bn, s);
    }
    return launch_shape<false>(a, bn, s, epilogue == EPI_SAMPLE);
}

}  // namespace spiral
