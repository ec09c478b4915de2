// Projections of the decode step: out[m][n] = sum_k A[m][k] * W[n][k] with 16-bit operands on the
// gfx950 matrix cores (v_mfma_f32_16x16x32, fp32 accumulation), and a plain FMA kernel for
// fp32-weight models.
//
// Shape of the problem: M is the batch (<= 128 rows at decode), every weight element is used once,
// so the kernel is a stream over W at HBM rate; the activations (M x K, a few hundred KB) are
// re-read from L2.  One workgroup owns a tile of BN weight rows x all M (<= 128) batch rows; its
// four waves split the workgroup's K range, so each wave reads a disjoint part of W straight into
// MFMA operand registers (16 B per lane, 64 contiguous bytes per row and instruction) without any
// barrier in the main loop; the four partial tiles are summed through LDS at the end.  A grid-level
// K split (blockIdx.y) multiplies the number of workgroups for the narrow projections; its partial
// sums are written separately and added, in a fixed order, by the consumer kernel, which keeps the
// result bit-reproducible.
//
// Weights are the MFMA "A" operand (rows i = output column n), activations the "B" operand
// (columns j = batch row m), so that a lane ends up with 4 consecutive n of one m.
#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

// MT: 16-row batch tiles per workgroup (M tile = 16*MT), NT: 16-row weight tiles (BN = 16*NT).
// For EPI_SWIGLU the first NT/2 weight tiles are gate rows and the last NT/2 the matching up rows.
template <int MT, int NT, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
    extern __shared__ float4 lds[];     // [4 waves (x2 for SwiGLU)][MT tiles][64 lanes] partial accumulators
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int tile_m = blockIdx.x % g.m_tiles;
    const int tile_n = blockIdx.x / g.m_tiles;
    const int split = blockIdx.y;
    const int K = g.K;
    const int m0 = tile_m * (16 * MT);

    // --- operand row pointers (16 B per lane at column lg*8 of each 32-wide k step)
    const uint16_t* wrow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const uint16_t* base;
        int row;
        if (EPI == EPI_SWIGLU) {
            constexpr int H = NT / 2;
            row = tile_n * (16 * H) + (nt % H) * 16 + li;
            if (row >= g.N) row = g.N - 1;
            base = (const uint16_t*)(nt < H ? g.w[0] : g.w[1]);
        } else {
            int n = tile_n * (16 * NT) + nt * 16 + li;
            if (n >= g.N) n = g.N - 1;
            if (n < g.rows[0]) { base = (const uint16_t*)g.w[0]; row = n; }
            else if (n < g.rows[0] + g.rows[1]) { base = (const uint16_t*)g.w[1]; row = n - g.rows[0]; }
            else { base = (const uint16_t*)g.w[2]; row = n - g.rows[0] - g.rows[1]; }
        }
        wrow[nt] = base + (size_t)row * K + lg * 8;
    }
    const uint16_t* arow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int m = m0 + mt * 16 + li;
        if (m >= g.M) m = g.M - 1;
        arow[mt] = (const uint16_t*)g.A + (size_t)m * K + lg * 8;
    }

    // --- this wave's k range, in steps of 32
    const int ksteps = K >> 5;
    const int units = g.splits * 4;
    const int u = split * 4 + wave;
    const int kb = (int)(((long long)ksteps * u) / units);
    const int ke = (int)(((long long)ksteps * (u + 1)) / units);

    f32x4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // --- main loop: stages of U k steps, ping-pong between two register stages so that the next
    //     stage's loads are in flight while the current one feeds the matrix cores
    constexpr int U = 2;
    u32x4 wf[2][U][NT], af[2][U][MT];
    auto load = [&](int k, u32x4 (&w)[U][NT], u32x4 (&a)[U][MT]) {
#pragma unroll
        for (int i = 0; i < U; ++i) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) w[i][nt] = *(const u32x4*)(wrow[nt] + (size_t)(k + i) * 32);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[i][mt] = *(const u32x4*)(arow[mt] + (size_t)(k + i) * 32);
        }
    };
    auto compute1 = [&](u32x4 (&w)[NT], u32x4 (&a)[MT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const u32x4 wp = prep_w(w[nt]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = mma_prepped(wp, a[mt], acc[nt][mt]);
        }
    };
    auto compute = [&](u32x4 (&w)[U][NT], u32x4 (&a)[U][MT]) {
#pragma unroll
        for (int i = 0; i < U; ++i) compute1(w[i], a[i]);
    };

    int k = kb;
    const int n_stage = (ke - kb) / U;          // full stages; the remainder is handled one step at a time
    if (n_stage > 0) {
        load(k, wf[0], af[0]);
        int st = 0;
        for (; st + 2 <= n_stage; st += 2) {
            load(k + U, wf[1], af[1]);
            compute(wf[0], af[0]);
            if (st + 2 < n_stage) load(k + 2 * U, wf[0], af[0]);
            compute(wf[1], af[1]);
            k += 2 * U;
        }
        if (st < n_stage) {                     // odd stage count: the last stage is already in wf[0]
            compute(wf[0], af[0]);
            k += U;
        }
    }
    for (; k < ke; ++k) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wf[0][0][nt] = *(const u32x4*)(wrow[nt] + (size_t)k * 32);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[0][0][mt] = *(const u32x4*)(arow[mt] + (size_t)k * 32);
        compute1(wf[0][0], af[0][0]);
    }

    // --- sum the four waves' partial tiles through LDS, one weight tile (SwiGLU: one gate/up pair)
    //     at a time so that at most 64 KB of LDS is needed; wave w finishes batch tiles mt = w, w+4
    if (EPI == EPI_STORE_F32) {
        float* out = (float*)g.out + (size_t)split * g.M * g.N;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const f32x4 v = acc[nt][mt];
                lds[(wave * MT + mt) * 64 + lane] = make_float4(v.x, v.y, v.z, v.w);
            }
            __syncthreads();
            for (int mt = wave; mt < MT; mt += 4) {
                float4 s = lds[mt * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const float4 o = lds[(w * MT + mt) * 64 + lane];
                    s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
                }
                // lane holds rows i = lg*4 .. +3 (output columns n) of column j = li (batch row m)
                const int m = m0 + mt * 16 + li;
                const int n = tile_n * (16 * NT) + nt * 16 + lg * 4;
                if (m < g.M && n < g.N) *(float4*)(out + (size_t)m * g.N + n) = s;
            }
            __syncthreads();
        }
    } else {
        constexpr int H = NT / 2;
        bool bad = false;
#pragma unroll
        for (int ft = 0; ft < H; ++ft) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const f32x4 v = acc[ft][mt];
                const f32x4 q = acc[ft + H][mt];
                lds[(wave * MT + mt) * 64 + lane] = make_float4(v.x, v.y, v.z, v.w);
                lds[((4 + wave) * MT + mt) * 64 + lane] = make_float4(q.x, q.y, q.z, q.w);
            }
            __syncthreads();
            for (int mt = wave; mt < MT; mt += 4) {
                float4 gs = lds[mt * 64 + lane];
                float4 us = lds[(4 * MT + mt) * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const float4 og = lds[(w * MT + mt) * 64 + lane];
                    const float4 ou = lds[((4 + w) * MT + mt) * 64 + lane];
                    gs.x += og.x; gs.y += og.y; gs.z += og.z; gs.w += og.w;
                    us.x += ou.x; us.y += ou.y; us.z += ou.z; us.w += ou.w;
                }
                const int m = m0 + mt * 16 + li;
                const int f = tile_n * (16 * H) + ft * 16 + lg * 4;
                if (m < g.M && f < g.N) {
                    ushort4 o;
                    o.x = f32_to_act16_noting(silu_f(gs.x) * us.x, bad);
                    o.y = f32_to_act16_noting(silu_f(gs.y) * us.y, bad);
                    o.z = f32_to_act16_noting(silu_f(gs.z) * us.z, bad);
                    o.w = f32_to_act16_noting(silu_f(gs.w) * us.w, bad);
                    *(ushort4*)((uint16_t*)g.out + (size_t)m * g.N + f) = o;
                }
            }
            __syncthreads();
        }
        report_saturation(g.sat_count, bad);
    }
}

// ---------------------------------------------------------------------------------------------
// fp32-weight models: one thread per output element, fp32 FMA.  Small correctness configuration only.
// ---------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(64) void gemm_f32_kernel(GemmArgs g) {
    const int n = blockIdx.x * 64 + threadIdx.x;
    if (n >= g.N) return;
    for (int m = blockIdx.y; m < g.M; m += gridDim.y) {
        const float* a = (const float*)g.A + (size_t)m * g.K;
        if (EPI == EPI_SWIGLU) {
            const float* wg = (const float*)g.w[0] + (size_t)n * g.K;
            const float* wu = (const float*)g.w[1] + (size_t)n * g.K;
            float sg = 0.f, su = 0.f;
            for (int k = 0; k < g.K; ++k) { sg = fmaf(a[k], wg[k], sg); su = fmaf(a[k], wu[k], su); }
            ((float*)g.out)[(size_t)m * g.N + n] = (sg / (1.0f + expf(-sg))) * su;
        } else {
            const float* w;
            if (n < g.rows[0]) w = (const float*)g.w[0] + (size_t)n * g.K;
            else if (n < g.rows[0] + g.rows[1]) w = (const float*)g.w[1] + (size_t)(n - g.rows[0]) * g.K;
            else w = (const float*)g.w[2] + (size_t)(n - g.rows[0] - g.rows[1]) * g.K;
            float s = 0.f;
            for (int k = 0; k < g.K; ++k) s = fmaf(a[k], w[k], s);
            ((float*)g.out)[(size_t)m * g.N + n] = s;
        }
    }
}

template <int MT, int NT, int EPI>
static hipError_t launch_mfma(const GemmArgs& a, hipStream_t s) {
    GemmArgs g = a;
    g.m_tiles = (a.M + 16 * MT - 1) / (16 * MT);
    const int bn = EPI == EPI_SWIGLU ? 8 * NT : 16 * NT;
    const int n_tiles = (a.N + bn - 1) / bn;
    const size_t lds_bytes = (size_t)(EPI == EPI_SWIGLU ? 8 : 4) * MT * 64 * sizeof(float4);
    hipLaunchKernelGGL((gemm_mfma_kernel<MT, NT, EPI>), dim3(n_tiles * g.m_tiles, g.splits), dim3(256), lds_bytes, s, g);
    return hipGetLastError();
}

template <int NT, int EPI>
static hipError_t launch_mfma_m(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 16) return launch_mfma<1, NT, EPI>(a, s);
    if (a.M <= 32) return launch_mfma<2, NT, EPI>(a, s);
    if (a.M <= 64) return launch_mfma<4, NT, EPI>(a, s);
    return launch_mfma<8, NT, EPI>(a, s);
}

// bn: weight rows per workgroup (32 or 64; SwiGLU counts gate + up rows)
hipError_t launch_gemm(const GemmArgs& a, int epilogue, bool w_bf16, int bn, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (!w_bf16) {
        if (a.splits != 1) return hipErrorInvalidValue;
        dim3 g((a.N + 63) / 64, a.M < 32768 ? a.M : 32768), b(64);
        if (epilogue == EPI_SWIGLU) hipLaunchKernelGGL((gemm_f32_kernel<EPI_SWIGLU>), g, b, 0, s, a);
        else hipLaunchKernelGGL((gemm_f32_kernel<EPI_STORE_F32>), g, b, 0, s, a);
        return hipGetLastError();
    }
    if ((a.K & 31) || (a.N & 3)) return hipErrorInvalidValue;
    // thousands of rows: the 256 x 256 LDS-tiled kernel, once its tiles fill most of the chip
    if (a.M >= 512 && bn != 1 && gemm_tile_usable(a) && (epilogue != EPI_SWIGLU || (a.N & 7) == 0)) {   // SwiGLU rows are stored 8 halves at a time
        const long tiles = (long)((a.M + 255) / 256) * ((a.N + (epilogue == EPI_SWIGLU ? 127 : 255)) / (epilogue == EPI_SWIGLU ? 128 : 256));
        if (tiles >= 200) return launch_gemm_tile(a, epilogue, s);
    }
    if ((a.K & 127) == 0 && (a.N & 15) == 0) return launch_gemm_stream(a, epilogue, bn, s);
    if (epilogue == EPI_SWIGLU) {
        if (a.splits != 1) return hipErrorInvalidValue;
        return bn >= 64 ? launch_mfma_m<4, EPI_SWIGLU>(a, s) : launch_mfma_m<2, EPI_SWIGLU>(a, s);
    }
    return bn >= 64 ? launch_mfma_m<4, EPI_STORE_F32>(a, s) : launch_mfma_m<2, EPI_STORE_F32>(a, s);
}

}  // namespace spiral
