// Large-M projection kernel (prefill and the scoring pass): out[m][n] = sum_k A[m][k] * W[n][k] with
// thousands of rows, where the matrix cores, not HBM, are the bound.
//
// A workgroup (4 waves, one per SIMD) owns a 256 x 256 output tile and walks K in chunks of 64.  Both
// operand tiles of a chunk go global -> registers -> LDS (the bf16 weights are widened to half on the
// way; rows padded to 144 B so that operand reads are conflict free), double buffered: while the
// waves multiply chunk c out of one buffer the loads of chunk c + 1 are in flight, and they are parked
// in the other buffer in two halves ahead of the last two k steps' MFMAs; one barrier per chunk.
// Every wave owns a 128 x 128 quarter: per k step of 16 it reads 4 + 4 operand fragments from LDS (one
// step ahead of their use) for 16 v_mfma_f32_32x32x16 (256 accumulator registers), i.e. 128 flop per
// byte fetched from L2 against 64 for a 128 x 128 tile.  Measured at 8192 rows: 0.65-0.9 PFLOP/s
// (the vendor GEMM: 1.0-1.4 on the same shapes; the streaming kernel this replaces: 0.36-0.68).
// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the tile order is arranged so
// that each XCD (own L2) gets a contiguous run of tiles, ordered in bands of 4 row tiles.
#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mma32t(const u32x4& w, const u32x4& a, const f32x16& c) {
#if SPIRAL_ACT_F16
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, a), c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, a), c, 0, 0, 0);
#endif
}

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROW = 144;                          // LDS bytes per tile row: 64 k x 2 B + 16 pad
constexpr int TILE_BYTES = 256 * ROW;             // one operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // A tile then W tile
constexpr int GROUP_M = 4;

}  // namespace

// SWIGLU: W rows of a tile are, per 32-row MFMA tile, 16 gate rows followed by the 16 up rows of the
// same ffn columns (a workgroup covers 128 ffn columns); the epilogue applies SiLU(gate) * up in registers.
template <bool SWIGLU, int WMW, bool FRAG>
__global__ __launch_bounds__(256) void gemm_tile_kernel(GemmArgs g) {
    constexpr int BMT = 128 * WMW;                 // batch rows per workgroup
    constexpr int WNW = 4 / WMW;                    // waves along the weight rows
    constexpr int J = 256 / (32 * WNW);             // 32-row weight tiles per wave
    constexpr int A_BYTES = BMT * ROW;              // activation tile; the weight tile follows it
    constexpr int STAGE = A_BYTES + TILE_BYTES;
    constexpr int AI = BMT / 32;                    // activation 16-byte segments per thread
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wm = wave % WMW, wn = wave / WMW;     // this wave's 128 x (32 J) part of the tile
    const int K = g.K;

    // ---- tile of this workgroup
    const int n_cols = SWIGLU ? 128 : 256;          // output columns per workgroup
    const int m_tiles = (g.M + BMT - 1) / BMT, n_tiles = (g.N + n_cols - 1) / n_cols;
    const int total = m_tiles * n_tiles;
    const int per_xcd = (total + 7) / 8;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || t >= total) return;
    const int band = t / (GROUP_M * n_tiles);
    const int band_rows = min(GROUP_M, m_tiles - band * GROUP_M);
    const int tile_m = band * GROUP_M + (t % (GROUP_M * n_tiles)) % band_rows;
    const int tile_n = (t % (GROUP_M * n_tiles)) / band_rows;
    const int m0 = tile_m * BMT, n0 = tile_n * n_cols;

    // ---- global -> LDS assignment: 2048 16-byte segments per operand tile, 8 per thread (row = s / 8, column = s % 8)
    const uint16_t* a_src[AI];
    const uint16_t* w_src[8];
    int dst[8], wdst[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int sgm = threadIdx.x + 256 * i;
        const int row = sgm >> 3, c8 = sgm & 7;
        if (i < AI) {
            int m = m0 + row; if (m >= g.M) m = g.M - 1;
            a_src[i] = (const uint16_t*)g.A + (size_t)m * K + c8 * 8;
        }
        wdst[i] = row * ROW + c8 * 16;
        if (FRAG) {
            // fragment order (SwiGLU: the interleaved gate/up matrix): a wave reads whole 1 KB blocks.
            // Unit u = threadIdx.x + 256 i of a chunk: lane = u % 64, (row tile rt, k step ks) = u / 64.
            const int blk = (threadIdx.x >> 6) + 4 * i, rt = blk >> 2, ks = blk & 3;
            const int t_all = SWIGLU ? (g.N + 15) / 16 : (g.N + 31) / 32;
            const int t32 = min((SWIGLU ? n0 / 16 : n0 / 32) + rt, t_all - 1);
            w_src[i] = (const uint16_t*)g.wf + frag_block(t32, ks, K) + lane * 8;
            wdst[i] = (rt * 32 + l32) * ROW + ks * 32 + lh * 16;
        } else if (SWIGLU) {
            const int q = row >> 5, r = row & 31;
            int f = n0 + q * 16 + (r & 15); if (f >= g.N) f = g.N - 1;
            w_src[i] = (const uint16_t*)(r < 16 ? g.w[0] : g.w[1]) + (size_t)f * K + c8 * 8;
        } else {
            int n = n0 + row; if (n >= g.N) n = g.N - 1;
            const uint16_t* base; int rr;
            if (n < g.rows[0]) { base = (const uint16_t*)g.w[0]; rr = n; }
            else if (n < g.rows[0] + g.rows[1]) { base = (const uint16_t*)g.w[1]; rr = n - g.rows[0]; }
            else { base = (const uint16_t*)g.w[2]; rr = n - g.rows[0] - g.rows[1]; }
            w_src[i] = base + (size_t)rr * K + c8 * 8;
        }
        dst[i] = row * ROW + c8 * 16;
    }
    // operand fragments: row (w? * 128 + j * 32 + l32), k = ks * 16 + lh * 8
    const int a_frag = (wm * 128 + l32) * ROW + lh * 16;
    const int w_frag = A_BYTES + (wn * 32 * J + l32) * ROW + lh * 16;

    f32x16 acc[J][4];                               // [weight tile j][batch tile i]
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    const int NC = K / BK;
    u32x4 ra[AI], rw[8];
    auto load = [&](int c) {
        const int cc = c < NC ? c : NC - 1;
        const size_t off = (size_t)cc * BK;
#pragma unroll
        for (int i = 0; i < AI; ++i) ra[i] = *(const u32x4*)(a_src[i] + off);
#pragma unroll
        for (int i = 0; i < 8; ++i) rw[i] = *(const u32x4*)(w_src[i] + (FRAG ? (size_t)cc * (BK / 16) * 512 : off));
    };
    auto park = [&](int c) {
        char* buf = lds + (c & 1) * STAGE;
#pragma unroll
        for (int i = 0; i < AI; ++i) *(u32x4*)(buf + dst[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)(buf + A_BYTES + wdst[i]) = FRAG ? rw[i] : prep_w(rw[i]);
    };
    // One chunk: operand fragments of k step ks + 1 are read from LDS while the 16 MFMAs of step ks run.
    auto frags = [&](const char* buf, int ks, u32x4* af, u32x4* wf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *(const u32x4*)(buf + a_frag + i * 32 * ROW + ks * 32);
#pragma unroll
        for (int j = 0; j < J; ++j) wf[j] = *(const u32x4*)(buf + w_frag + j * 32 * ROW + ks * 32);
    };
    auto park_a = [&](int c) {
        char* buf = lds + (c & 1) * STAGE;
#pragma unroll
        for (int i = 0; i < AI; ++i) *(u32x4*)(buf + dst[i]) = ra[i];
    };
    auto park_w = [&](int c) {
        char* buf = lds + (c & 1) * STAGE;
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)(buf + A_BYTES + wdst[i]) = FRAG ? rw[i] : prep_w(rw[i]);
    };
    auto chunk = [&](int c) {
        const char* buf = lds + (c & 1) * STAGE;
        u32x4 af[2][4], wf[2][J];
        frags(buf, 0, af[0], wf[0]);
        load(c + 1);                                 // in flight during the arithmetic (past the end: a re-read)
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) frags(buf, ks + 1, af[(ks + 1) & 1], wf[(ks + 1) & 1]);
            // the next chunk's registers go to the other buffer (its readers finished before the last
            // barrier) in two halves ahead of the last two steps' MFMAs
            if (ks == 2) park_a(c + 1);
            if (ks == 3) park_w(c + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] = mma32t(wf[ks & 1][j], af[ks & 1][i], acc[j][i]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    load(0);
    park(0);
    __syncthreads();
    for (int c = 0; c < NC; ++c) {
        chunk(c);
        __syncthreads();
    }

    // ---- epilogue.  In a 32 x 32 tile a lane holds batch row l32 and, in registers 4b..4b+3, weight rows 8b + 4*lh .. +3.
    if (!SWIGLU) {
        float* out = (float*)g.out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + wm * 128 + i * 32 + l32;
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int n = n0 + (wn * J + j) * 32 + 8 * b + 4 * lh;
                    if (m < g.M && n < g.N)
                        *(float4*)(out + (size_t)m * g.N + n) =
                            make_float4(acc[j][i][4 * b], acc[j][i][4 * b + 1], acc[j][i][4 * b + 2], acc[j][i][4 * b + 3]);
                }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + wm * 128 + i * 32 + l32;
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int f = n0 + (wn * J + j) * 16 + 8 * b + 4 * lh;
                    if (m < g.M && f < g.N) {
                        ushort4 o;
                        o.x = f32_to_act16(silu_f(acc[j][i][4 * b]) * acc[j][i][4 * b + 8]);
                        o.y = f32_to_act16(silu_f(acc[j][i][4 * b + 1]) * acc[j][i][4 * b + 9]);
                        o.z = f32_to_act16(silu_f(acc[j][i][4 * b + 2]) * acc[j][i][4 * b + 10]);
                        o.w = f32_to_act16(silu_f(acc[j][i][4 * b + 3]) * acc[j][i][4 * b + 11]);
                        *(ushort4*)((uint16_t*)g.out + (size_t)m * g.N + f) = o;
                    }
                }
        }
    }
}

template <bool SWIGLU, int WMW, bool FRAG>
static hipError_t launch_tile(const GemmArgs& a, hipStream_t s) {
    const int cols = SWIGLU ? 128 : 256;
    const int m_tiles = (a.M + 128 * WMW - 1) / (128 * WMW);
    const int n_tiles = (a.N + cols - 1) / cols;
    const int per_xcd = (m_tiles * n_tiles + 7) / 8;
    const size_t lds_bytes = (size_t)2 * (128 * WMW * ROW + TILE_BYTES);
    hipError_t e = hipFuncSetAttribute((const void*)gemm_tile_kernel<SWIGLU, WMW, FRAG>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_tile_kernel<SWIGLU, WMW, FRAG>), dim3(per_xcd * 8), dim3(256), lds_bytes, s, a);
    return hipGetLastError();
}

// rows_per_tile: 256 (large M) or 128 (one tile of batch rows, weights streamed once through LDS)
hipError_t launch_gemm_tile(const GemmArgs& a, int epilogue, int rows_per_tile, hipStream_t s) {
    if ((a.K % BK) || (a.N & 3) || a.splits != 1) return hipErrorInvalidValue;
    const bool swiglu = epilogue == EPI_SWIGLU;
    if (rows_per_tile == 128) {
        if (a.wf) return swiglu ? launch_tile<true, 1, true>(a, s) : launch_tile<false, 1, true>(a, s);
        return swiglu ? launch_tile<true, 1, false>(a, s) : launch_tile<false, 1, false>(a, s);
    }
    if (a.wf) return swiglu ? launch_tile<true, 2, true>(a, s) : launch_tile<false, 2, true>(a, s);
    return swiglu ? launch_tile<true, 2, false>(a, s) : launch_tile<false, 2, false>(a, s);
}

}  // namespace spiral
