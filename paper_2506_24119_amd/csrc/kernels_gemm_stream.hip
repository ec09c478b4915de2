// Weight-streaming projection kernel for the decode step (K a multiple of 128).
//
// out[m][n] = sum_k A[m][k] * W[n][k], M <= 128 rows per tile.  Every weight byte is used once, so
// the kernel is organised around keeping many weight loads in flight:
//   * a workgroup owns 64 or 128 weight rows and all (<= 128) batch rows of its M tile; each of its
//     four waves owns 16 or 32 of those weight rows outright, so there is no reduction between waves;
//   * weights go HBM -> registers directly in MFMA operand layout (16 B per lane), PD chunks of 128 k
//     ahead of use; they are the only deep queue of vector-memory loads in the loop;
//   * the activations of a chunk (128 rows x 128 k, re-read from L2) are loaded cooperatively by the
//     256 threads in the same stage, parked in LDS (row stride 272 B: conflict-free ds_read_b128
//     for the MFMA operand pattern) and read by all four waves;
//   * LDS is double buffered, one barrier per chunk.
// A grid-level split of K (blockIdx.y) supplies enough workgroups for the narrow projections; the
// consumer kernel adds the partial results in a fixed order.
#include <algorithm>

#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

enum { SW_NONE = 0, SW_WIDE = 1, SW_NARROW = 2 };
// SW_WIDE:   SwiGLU, a wave owns 16 ffn columns: tile 0 = gate rows, tile 1 = up rows (NTW = 2)
// SW_NARROW: SwiGLU, workgroup owns 32 ffn columns: waves 0,1 gate rows, waves 2,3 the up rows (NTW = 1)

template <int MT, int NTW>
struct Stage {
    u32x4 a[MT];          // this thread's share of the activation chunk
    u32x4 w[NTW][4];      // this lane's weight fragments: 4 k steps of 32
};

template <int MT, int NTW, int MODE, int PD>
__global__ __launch_bounds__(256) void gemm_stream_kernel(GemmArgs g) {
    constexpr int ROWB = 272;                       // LDS bytes per activation row (256 + 16 pad)
    constexpr int BUF = 16 * MT * ROWB;
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int tile_m = blockIdx.x % g.m_tiles;
    const int tile_n = blockIdx.x / g.m_tiles;
    const int split = blockIdx.y;
    const int K = g.K;
    const int m0 = tile_m * (16 * MT);

    // ---- weight rows of this wave
    const uint16_t* wrow[NTW];
    int n_first;                                    // first output column (or ffn column) of this wave
    if (MODE == SW_WIDE) {
        n_first = tile_n * 64 + wave * 16;
        int f = n_first + li; if (f >= g.N) f = g.N - 1;
        wrow[0] = (const uint16_t*)g.w[0] + (size_t)f * K + lg * 8;
        wrow[NTW - 1] = (const uint16_t*)g.w[1] + (size_t)f * K + lg * 8;
    } else if (MODE == SW_NARROW) {
        n_first = tile_n * 32 + (wave & 1) * 16;
        int f = n_first + li; if (f >= g.N) f = g.N - 1;
        wrow[0] = (const uint16_t*)(wave < 2 ? g.w[0] : g.w[1]) + (size_t)f * K + lg * 8;
    } else {
        n_first = tile_n * (64 * NTW) + wave * (16 * NTW);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            int n = n_first + nt * 16 + li; if (n >= g.N) n = g.N - 1;
            const uint16_t* base; int row;
            if (n < g.rows[0]) { base = (const uint16_t*)g.w[0]; row = n; }
            else if (n < g.rows[0] + g.rows[1]) { base = (const uint16_t*)g.w[1]; row = n - g.rows[0]; }
            else { base = (const uint16_t*)g.w[2]; row = n - g.rows[0] - g.rows[1]; }
            wrow[nt] = base + (size_t)row * K + lg * 8;
        }
    }

    // ---- this thread's share of an activation chunk: MT segments of 16 B (row = s / 16, column = s % 16)
    const uint16_t* a_src[MT];
    int a_dst[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int s = threadIdx.x + 256 * i;
        const int row = s >> 4, c16 = s & 15;
        int m = m0 + row; if (m >= g.M) m = g.M - 1;
        a_src[i] = (const uint16_t*)g.A + (size_t)m * K + c16 * 8;
        a_dst[i] = row * ROWB + c16 * 16;
    }
    const int frag_off = li * ROWB + lg * 16;       // + mt*16*ROWB + ks*64

    // ---- chunk range of this workgroup
    const int chunks = K >> 7;
    const int cb = (int)(((long long)chunks * split) / g.splits);
    const int ce = (int)(((long long)chunks * (split + 1)) / g.splits);
    const int NC = ce - cb;

    f32x4 acc[NTW][MT];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    Stage<MT, NTW> st[PD];
    // Loads are unconditional (no branch around them) so that the compiler can count exactly how many
    // younger loads may stay in flight at each wait; past the end of the range every lane reads the same
    // valid 16 bytes instead, which costs one cache line.
    const uint16_t* dummy = (const uint16_t*)g.A;
    auto load = [&](Stage<MT, NTW>& S, int chunk) {
        const bool ok = chunk < ce;
        const size_t off = (size_t)chunk * 128;
#pragma unroll
        for (int i = 0; i < MT; ++i) S.a[i] = *(const u32x4*)(ok ? a_src[i] + off : dummy);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) S.w[nt][ks] = *(const u32x4*)(ok ? wrow[nt] + off + ks * 32 : dummy);
    };
    auto iter = [&](Stage<MT, NTW>& S, int c) {
        char* buf = lds + (c & 1) * BUF;
#pragma unroll
        for (int i = 0; i < MT; ++i) *(u32x4*)(buf + a_dst[i]) = S.a[i];
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 af[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) af[mt] = *(const u32x4*)(buf + frag_off + mt * 16 * ROWB + ks * 64);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const u32x4 wp = prep_w(S.w[nt][ks]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = mma_prepped(wp, af[mt], acc[nt][mt]);
            }
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

    // ---- epilogue: a lane holds 4 consecutive output columns (n_first + nt*16 + lg*4 ..) of batch row li
    if (MODE == SW_NONE) {
        float* out = (float*)g.out + (size_t)split * g.M * g.N;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = m0 + mt * 16 + li;
                const int n = n_first + nt * 16 + lg * 4;
                const f32x4 v = acc[nt][mt];
                if (m < g.M && n < g.N) *(float4*)(out + (size_t)m * g.N + n) = make_float4(v.x, v.y, v.z, v.w);
            }
    } else {
        if (MODE == SW_NARROW) {
            // waves 2,3 hand their up-projection tiles to waves 0,1 through LDS
            __syncthreads();                        // everyone is done with the activation buffers
            float4* x = (float4*)lds;
            if (wave >= 2) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const f32x4 v = acc[0][mt];
                    x[((wave - 2) * MT + mt) * 64 + lane] = make_float4(v.x, v.y, v.z, v.w);
                }
            }
            __syncthreads();
            if (wave >= 2) return;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = m0 + mt * 16 + li;
            const int f = n_first + lg * 4;
            const f32x4 gs = acc[0][mt];
            f32x4 us;
            if (MODE == SW_NARROW) {
                const float4 t = ((const float4*)lds)[(wave * MT + mt) * 64 + lane];
                us = f32x4{t.x, t.y, t.z, t.w};
            } else {
                us = acc[NTW - 1][mt];
            }
            if (m < g.M && f < g.N) {
                ushort4 o;
                o.x = f32_to_act16(silu_f(gs.x) * us.x);
                o.y = f32_to_act16(silu_f(gs.y) * us.y);
                o.z = f32_to_act16(silu_f(gs.z) * us.z);
                o.w = f32_to_act16(silu_f(gs.w) * us.w);
                *(ushort4*)((uint16_t*)g.out + (size_t)m * g.N + f) = o;
            }
        }
    }
}

template <int MT, int NTW, int MODE, int PD>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
    GemmArgs g = a;
    g.m_tiles = (a.M + 16 * MT - 1) / (16 * MT);
    const int cols = MODE == SW_WIDE ? 64 : (MODE == SW_NARROW ? 32 : 64 * NTW);
    const int n_tiles = (a.N + cols - 1) / cols;
    size_t lds_bytes = (size_t)2 * 16 * MT * 272;
    if (MODE == SW_NARROW) lds_bytes = std::max(lds_bytes, (size_t)2 * MT * 64 * sizeof(float4));
    hipLaunchKernelGGL((gemm_stream_kernel<MT, NTW, MODE, PD>), dim3(n_tiles * g.m_tiles, g.splits), dim3(256),
                       lds_bytes, s, g);
    return hipGetLastError();
}

template <int NTW, int MODE>
static hipError_t launch_m(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 16) return launch_one<1, NTW, MODE, 4>(a, s);
    if (a.M <= 32) return launch_one<2, NTW, MODE, 4>(a, s);
    if (a.M <= 64) return launch_one<4, NTW, MODE, 4>(a, s);
    return launch_one<8, NTW, MODE, 3>(a, s);
}

hipError_t launch_gemm_stream(const GemmArgs& a, int epilogue, int bn, hipStream_t s) {
    if ((a.K & 127) || (a.N & 15) || a.splits < 1 || a.splits > (a.K >> 7)) return hipErrorInvalidValue;
    if (epilogue == EPI_SWIGLU) {
        if (a.splits != 1) return hipErrorInvalidValue;
        return bn >= 128 ? launch_m<2, SW_WIDE>(a, s) : launch_m<1, SW_NARROW>(a, s);
    }
    return bn >= 128 ? launch_m<2, SW_NONE>(a, s) : launch_m<1, SW_NONE>(a, s);
}

}  // namespace spiral
