// Learner-side scoring: log pi(target | context) for every row of a packed batch, without ever
// writing the [rows, vocab] logits.
//
// score_lmhead_kernel is the LM-head GEMM of the decode path (32x32x16 MFMA, weights HBM/L2 ->
// registers in operand layout, activations through LDS) with another epilogue: a workgroup owns 128
// rows and a range of 128-column vocabulary tiles; after each tile every lane folds its 16 logits of
// each row into a private running (max, sum of exp) pair and checks whether the row's target column
// is among them.  At the end of the range the pairs of a row (2 lanes x 4 waves) are merged through
// LDS and written as one partial per (row, range); score_merge_kernel combines the ranges:
//     logp = logit[target] - (M + ln sum_i s_i * exp(m_i - M)).
// score_objective_kernel evaluates the clipped importance-ratio surrogate and the REINFORCE sum in
// float64 with a fixed reduction order.
#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mma32s(const u32x4& w, const u32x4& a, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, a), c, 0, 0, 0);
}

constexpr int ROWB = 272;                 // LDS bytes per activation row (256 + 16 pad)
constexpr int BUF = 128 * ROWB;
constexpr int PD = 2;

}  // namespace

template <bool FRAG>
__global__ __launch_bounds__(256) void score_lmhead_kernel(ScoreArgs g) {
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tile_m = blockIdx.x % g.m_tiles;
    const int split = blockIdx.x / g.m_tiles;
    const int K = g.K;
    const int m0 = tile_m * 128;
    const int n_tiles = (g.V + 127) / 128;
    const int nt_begin = split * g.tiles_per_split;
    const int nt_end = min(nt_begin + g.tiles_per_split, n_tiles);

    const uint16_t* a_src[8];
    int a_dst[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int sgm = threadIdx.x + 256 * i;
        const int row = sgm >> 4, c16 = sgm & 15;
        int m = m0 + row; if (m >= g.M) m = g.M - 1;
        a_src[i] = (const uint16_t*)g.A + (size_t)m * K + c16 * 8;
        a_dst[i] = row * ROWB + c16 * 16;
    }
    const int frag_off = l32 * ROWB + lh * 16;
    const int NC = K >> 7;

    // this lane's rows (one per batch tile) and their targets
    int tgt[4];
    float m_run[4], s_run[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int m = m0 + t * 32 + l32;
        tgt[t] = m < g.M ? g.targets[m] : -1;
        m_run[t] = -INFINITY;
        s_run[t] = 0.f;
    }

    struct St { u32x4 a[8]; u32x4 w[8]; };
    for (int nt = nt_begin; nt < nt_end; ++nt) {
        const int n_first = nt * 128 + wave * 32;
        int n = n_first + l32; if (n >= g.V) n = g.V - 1;
        const uint16_t* wrow = FRAG ? (const uint16_t*)g.Wf + frag_block(min(nt * 4 + wave, (g.V + 31) / 32 - 1), 0, K) + lane * 8
                                    : (const uint16_t*)g.W + (size_t)n * K + lh * 8;

        f32x16 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

        St st[PD];
        auto load = [&](St& S, int chunk) {
            const int cc = chunk < NC ? chunk : NC - 1;
            const size_t off = (size_t)cc * 128;
#pragma unroll
            for (int i = 0; i < 8; ++i) S.a[i] = *(const u32x4*)(a_src[i] + off);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                S.w[ks] = FRAG ? *(const u32x4*)(wrow + ((size_t)cc * 8 + ks) * 512) : *(const u32x4*)(wrow + off + ks * 16);
        };
        auto iter = [&](St& S, int c) {
            char* buf = lds + (c & 1) * BUF;
#pragma unroll
            for (int i = 0; i < 8; ++i) *(u32x4*)(buf + a_dst[i]) = S.a[i];
            __syncthreads();
            u32x4 af[2][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) af[0][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                if (ks + 1 < 8) {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        af[(ks + 1) & 1][t] = *(const u32x4*)(buf + frag_off + t * 32 * ROWB + (ks + 1) * 32);
                }
                const u32x4 wp = FRAG ? S.w[ks] : prep_w(S.w[ks]);      // fragment-ordered copies are already widened
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[t] = mma32s(wp, af[ks & 1][t], acc[t]);
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
        __syncthreads();                       // the next tile's first LDS write must not overtake a slow wave's reads

        // registers 4b..4b+3 of a tile hold columns n_first + 8b + 4*lh .. +3 of row l32
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float mx = -INFINITY;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int col = n_first + 8 * b + 4 * lh + r;
                    if (col >= g.V) acc[t][4 * b + r] = -INFINITY;
                    mx = fmaxf(mx, acc[t][4 * b + r]);
                    if (col == tgt[t]) g.tgt_logit[m0 + t * 32 + l32] = acc[t][4 * b + r];
                }
            if (mx > -INFINITY) {
                const float m_new = fmaxf(m_run[t], mx);
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += __expf(acc[t][r] - m_new);
                s_run[t] = s_run[t] * __expf(m_run[t] - m_new) + sum;
                m_run[t] = m_new;
            }
        }
    }

    // ---- merge the 8 (max, sum) pairs of every row: the two lane halves, then the four waves
    float* s_m = (float*)lds;                  // [4 waves][128 rows]
    float* s_s = s_m + 512;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float om = __shfl_xor(m_run[t], 32, 64), os = __shfl_xor(s_run[t], 32, 64);
        const float M = fmaxf(m_run[t], om);
        const float S = (m_run[t] > -INFINITY ? s_run[t] * __expf(m_run[t] - M) : 0.f) + (om > -INFINITY ? os * __expf(om - M) : 0.f);
        if (lh == 0) { s_m[wave * 128 + t * 32 + l32] = M; s_s[wave * 128 + t * 32 + l32] = S; }
    }
    __syncthreads();
    if (threadIdx.x < 128) {
        const int row = threadIdx.x, m = m0 + row;
        if (m < g.M) {
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, s_m[w * 128 + row]);
            float S = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float mw = s_m[w * 128 + row];
                if (mw > -INFINITY) S += s_s[w * 128 + row] * __expf(mw - M);
            }
            float2* dst = (float2*)g.part + (size_t)m * g.n_splits + split;
            *dst = make_float2(M, S);
        }
    }
}

__global__ __launch_bounds__(256) void score_merge_kernel(ScoreArgs g, float* out) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= g.M) return;
    if (g.targets[m] < 0) { out[m] = 0.f; return; }
    const float2* p = (const float2*)g.part + (size_t)m * g.n_splits;
    float M = -INFINITY;
    for (int i = 0; i < g.n_splits; ++i) M = fmaxf(M, p[i].x);
    float S = 0.f;
    for (int i = 0; i < g.n_splits; ++i)
        if (p[i].x > -INFINITY) S += p[i].y * expf(p[i].x - M);
    out[m] = g.tgt_logit[m] - (M + logf(S));
}

// out[0] = sum mask * min(r * A, clip(r, 1 - eps, 1 + eps) * A), r = exp(new - old);  out[1] = sum mask * A * new
__global__ __launch_bounds__(1024) void score_objective_kernel(const float* logp_new, const float* logp_old, const float* adv,
                                                               const int32_t* mask, long long n, float eps, double* out) {
    __shared__ double s_a[1024], s_b[1024];
    double a = 0.0, b = 0.0;
    for (long long i = threadIdx.x; i < n; i += 1024) {
        if (mask && mask[i] == 0) continue;
        const double ln = logp_new[i], A = adv[i];
        const double r = exp(ln - (double)logp_old[i]);
        const double rc = fmin(fmax(r, 1.0 - (double)eps), 1.0 + (double)eps);
        a += fmin(r * A, rc * A);
        b += A * ln;
    }
    s_a[threadIdx.x] = a; s_b[threadIdx.x] = b;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) { s_a[threadIdx.x] += s_a[threadIdx.x + o]; s_b[threadIdx.x] += s_b[threadIdx.x + o]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) { out[0] = s_a[0]; out[1] = s_b[0]; }
}

hipError_t launch_score(const ScoreArgs& a, float* out, hipStream_t s) {
    if (a.M < 1 || a.V < 1 || (a.K & 127) || a.n_splits < 1 || a.tiles_per_split < 1) return hipErrorInvalidValue;
    ScoreArgs g = a;
    g.m_tiles = (a.M + 127) / 128;
    if (g.Wf) hipLaunchKernelGGL(score_lmhead_kernel<true>, dim3(g.m_tiles * g.n_splits), dim3(256), (size_t)2 * BUF, s, g);
    else hipLaunchKernelGGL(score_lmhead_kernel<false>, dim3(g.m_tiles * g.n_splits), dim3(256), (size_t)2 * BUF, s, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(score_merge_kernel, dim3((a.M + 255) / 256), dim3(256), 0, s, g, out);
    return hipGetLastError();
}

hipError_t launch_score_objective(const float* logp_new, const float* logp_old, const float* adv, const int32_t* mask,
                                  long long n, float eps, double* out, hipStream_t s) {
    hipLaunchKernelGGL(score_objective_kernel, dim3(1), dim3(1024), 0, s, logp_new, logp_old, adv, mask, n, eps, out);
    return hipGetLastError();
}

}  // namespace spiral
