// Large-M projection kernel (prefill and the scoring pass): out[m][n] = sum_k A[m][k] * W[n][k] with
// thousands of rows, where the matrix cores, not HBM, are the bound.
//
// A workgroup (4 waves, one per SIMD) owns a 256 x 256 output tile and walks K in chunks of 64.  Both
// operand tiles of a chunk go global -> registers -> LDS (rows padded to 144 B so that operand reads
// are conflict free; the weights come from the fragment-ordered copies, 1 KB contiguous per wave
// load, already in the operand type).  Three chunks are in flight: chunk c is multiplied out of one
// LDS buffer, chunk c + 1 moves from registers into the other buffer, and the global loads of chunk
// c + 2 are issued; the one barrier of a chunk sits before its last k step, so that the first operand reads of the
// next chunk are issued under MFMAs like all the others.  Every wave owns a 128 x 128 quarter: per k step of 16 it reads 4 + 4 operand
// fragments from LDS (one step ahead of their use) for 16 v_mfma_f32_32x32x16 (256 accumulator
// registers), i.e. 128 flop per byte fetched from L2 against 64 for a 128 x 128 tile; the issue order of
// a step is pinned (8 LDS reads, then 4 x (4 MFMAs, 1 LDS write, 1 global load)) so that LDS and memory
// traffic run under the MFMAs: issued as one burst at the start of a chunk the 16 loads of a thread cost a
// sixth of the kernel, spread over the k steps nothing measurable.  An isolated loop of this shape runs at 71 %
// of the nominal MFMA rate (a pure MFMA stream at 82 %: the clock under this load is ~2.0 GHz); the kernel delivers
// 1.0-1.15 PFLOP/s on 16,384 rows, the matrix cores busy 52-57 % of the cycles at 1.9-2.0 GHz (the vendor GEMM:
// 0.9-1.4 PFLOP/s on these shapes).  The clock follows the operand bits: with all-zero operands the gate/up
// projection takes 1.09 ms instead of 1.41 (1.50 PFLOP/s; the vendor GEMM 1.3-1.4 -> 1.9-2.0 PFLOP/s).
// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the tile order is arranged so
// that each XCD (own L2) gets a contiguous run of tiles, ordered in bands of 4 row tiles.
#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ f32x16 mma32t(const u32x4& w, const u32x4& a, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, a), c, 0, 0, 0);
}

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROW = 144;                          // LDS bytes per tile row: 64 k x 2 B + 16 pad
constexpr int TILE_BYTES = 256 * ROW;             // one operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // A tile then W tile
constexpr int GROUP_M = 4;

}  // namespace

// The weights are the fragment-ordered copies (frag_block(); SWIGLU: the interleaved gate/up matrix, a
// workgroup covers 128 ffn columns and the epilogue applies SiLU(gate) * up in registers).
// TEPI: 0 stores the fp32 product, 1 is the SwiGLU epilogue, 2 the q/k/v epilogue (the product never reaches memory:
// bias, per-head RMSNorm of q and k, RoPE, q stored as half, k and v appended to the sequence's page; head_dim 128,
// so a wave's 128 columns are exactly one head).
template <int TEPI>
__global__ __launch_bounds__(256) void gemm_tile_kernel(GemmArgs g, QkvPostArgs qa) {
    constexpr bool SWIGLU = TEPI == 1;
    constexpr int J = 4;                            // 32-row weight tiles per wave (and 4 batch tiles)
    constexpr int A_BYTES = TILE_BYTES;             // activation tile; the weight tile follows it
    constexpr int STAGE = STAGE_BYTES;
    extern __shared__ uint4 lds_raw[];
    char* lds = (char*)lds_raw;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;        // this wave's 128 x 128 quarter
    const int K = g.K;

    // ---- tile of this workgroup
    const int n_cols = SWIGLU ? 128 : 256;          // output columns per workgroup
    const int m_tiles = (g.M + BM - 1) / BM, n_tiles = (g.N + n_cols - 1) / n_cols;
    const int total = m_tiles * n_tiles;
    const int per_xcd = (total + 7) / 8;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || t >= total) return;
    const int band = t / (GROUP_M * n_tiles);
    const int band_rows = min(GROUP_M, m_tiles - band * GROUP_M);
    const int tile_m = band * GROUP_M + (t % (GROUP_M * n_tiles)) % band_rows;
    const int tile_n = (t % (GROUP_M * n_tiles)) / band_rows;
    const int m0 = tile_m * BM, n0 = tile_n * n_cols;

    // ---- global -> LDS assignment, 8 + 8 16-byte units per thread and chunk.
    //      Activations (row-major): unit i is row threadIdx.x / 8 + 32 i, 16-byte column threadIdx.x % 8
    //      (8 lanes read one 128-byte line).  Weights: a wave reads whole 1 KB fragment blocks, unit i is
    //      block (row tile i, k step threadIdx.x / 64) of the chunk, lane = threadIdx.x % 64.
    //      Offsets are 32-bit element offsets from the operand's base (the launcher checks that they fit).
    uint32_t a_off[8], w_off[8];
    const int dst0 = (threadIdx.x >> 3) * ROW + (threadIdx.x & 7) * 16;       // unit i lands 32 rows further down
    const int wdst0 = A_BYTES + l32 * ROW + (threadIdx.x >> 6) * 32 + lh * 16;
    {
        const int t_all = SWIGLU ? (g.N + 15) / 16 : (g.N + 31) / 32;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int m = m0 + (threadIdx.x >> 3) + 32 * i; if (m >= g.M) m = g.M - 1;
            a_off[i] = (uint32_t)m * (uint32_t)K + (threadIdx.x & 7) * 8;
            const int t32 = min((SWIGLU ? n0 / 16 : n0 / 32) + i, t_all - 1);
            w_off[i] = (uint32_t)frag_block(t32, threadIdx.x >> 6, K) + lane * 8;
        }
    }
    // operand fragments: row (w? * 128 + j * 32 + l32), k = ks * 16 + lh * 8
    const int a_frag = (wm * 128 + l32) * ROW + lh * 16;
    const int w_frag = A_BYTES + (wn * 128 + l32) * ROW + lh * 16;

    f32x16 acc[J][4];                               // [weight tile j][batch tile i]
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    const int NC = K / BK;
    // Two register stages: a chunk's global loads are issued two chunks before it is multiplied and
    // one chunk before it is parked in LDS, so the staging writes never wait for memory.
    u32x4 rg[2][16];                                // [stage][8 activation units, 8 weight units]
    auto load_unit = [&](const int st, const int cc, const int u) {
        if (u < 8) rg[st][u] = *(const u32x4*)((const uint16_t*)g.A + a_off[u] + (size_t)cc * BK);
        else rg[st][u] = *(const u32x4*)((const uint16_t*)g.wf + w_off[u - 8] + (size_t)cc * (BK / 16) * 512);
    };
    auto load = [&](const int st, int c) {
        const int cc = c < NC ? c : NC - 1;           // past the end: a re-read of the last chunk
#pragma unroll
        for (int u = 0; u < 16; ++u) load_unit(st, cc, u);
    };
    auto park_unit = [&](char* buf, const int st, const int u) {
        if (u < 8) *(u32x4*)(buf + dst0 + u * 32 * ROW) = rg[st][u];
        else *(u32x4*)(buf + wdst0 + (u - 8) * 32 * ROW) = rg[st][u];
    };
    auto frags = [&](const char* buf, int ks, u32x4* af, u32x4* wf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *(const u32x4*)(buf + a_frag + i * 32 * ROW + ks * 32);
#pragma unroll
        for (int j = 0; j < J; ++j) wf[j] = *(const u32x4*)(buf + w_frag + j * 32 * ROW + ks * 32);
    };
    // Chunk c sits in LDS buffer c & 1 and came through register stage c & 1.  The barrier of a chunk sits before
    // its last k step, not after it: by then every wave has issued (and waited for) its last operand reads of the
    // chunk and has parked all of chunk c + 1, so the last k step already reads the first fragments of chunk c + 1
    // and starts parking chunk c + 2 into the buffer that just became free - no operand read is ever exposed
    // behind a barrier.  Per k step: the 8 operand reads of the next step, four units parked, four units requested
    // (each unit is requested four k steps before it is parked), 16 MFMAs; issue order pinned to 8 reads, then
    // 4 x (4 MFMAs, 1 write, 1 global load) (other orders of the same instructions measured within noise).
    u32x4 af[2][4], wf[2][J];
    auto chunk = [&](int c, const int cu, const int nx) {
        char* buf = lds + cu * STAGE;                 // cu == c & 1
        char* other = lds + nx * STAGE;
        const int c2 = c + 2 < NC ? c + 2 : NC - 1;   // past the end: a re-read of the last chunk
        const int c3 = c + 3 < NC ? c + 3 : NC - 1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) {
                frags(buf, ks + 1, af[(ks + 1) & 1], wf[(ks + 1) & 1]);
#pragma unroll
                for (int u = 0; u < 4; ++u) park_unit(other, nx, (ks + 1) * 4 + u);
#pragma unroll
                for (int u = 0; u < 4; ++u) load_unit(cu, c2, (ks + 1) * 4 + u);
            } else {
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                frags(other, 0, af[0], wf[0]);
#pragma unroll
                for (int u = 0; u < 4; ++u) park_unit(buf, cu, u);
#pragma unroll
                for (int u = 0; u < 4; ++u) load_unit(nx, c3, u);
            }
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] = mma32t(wf[ks & 1][j], af[ks & 1][i], acc[j][i]);
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    load(0, 0);
    load(1, 1);
#pragma unroll
    for (int u = 0; u < 16; ++u) park_unit(lds, 0, u);
#pragma unroll
    for (int u = 0; u < 4; ++u) park_unit(lds + STAGE, 1, u);
#pragma unroll
    for (int u = 0; u < 4; ++u) load_unit(0, 2 < NC ? 2 : NC - 1, u);
    __syncthreads();
    frags(lds, 0, af[0], wf[0]);
    int c = 0;
    for (; c + 2 <= NC; c += 2) {
        chunk(c, 0, 1);
        chunk(c + 1, 1, 0);
    }
    if (c < NC) chunk(c, 0, 1);
    __syncthreads();                                  // the operand buffers are free for the epilogue

    // ---- epilogue.  In a 32 x 32 tile a lane holds batch row l32 and, in registers 4b..4b+3, weight rows 8b + 4*lh .. +3:
    //      written straight from there a store instruction touches 64 rows x 16 (or 8) bytes.  Each wave therefore
    //      turns its tile 32 rows at a time through a private LDS area (the operand buffers are free after the last
    //      barrier) and stores whole rows: 512 contiguous bytes per half wave (fp32), one 128-byte line per 8 lanes (SwiGLU).
    if (TEPI == 2) {
        const int head = (n0 + wn * 128) >> 7;
        const bool is_q = head < qa.n_q_heads, is_k = !is_q && head < qa.n_q_heads + qa.n_kv_heads;
        const int kvh = is_q ? 0 : (is_k ? head - qa.n_q_heads : head - qa.n_q_heads - qa.n_kv_heads);
        const uint16_t* bias = (const uint16_t*)(is_q ? qa.bq : (is_k ? qa.bk : qa.bv));      // bf16 like the weights, or null
        if (bias) bias += (is_q ? head : kvh) * 128;
        const float* gain = is_q ? qa.q_gain : (is_k ? qa.k_gain : nullptr);
        bool bad = false;
        if (head < qa.n_q_heads + 2 * qa.n_kv_heads) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m0 + wm * 128 + i * 32 + l32;
                const int mm = m < g.M ? m : g.M - 1;
                // this lane's 64 values of the head: dimension d = 32 j + 8 b + 4 lh + e sits in acc[j][i][4 b + e]
                if (bias) {
#pragma unroll
                    for (int j = 0; j < J; ++j)
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const ushort4 bb = *(const ushort4*)(bias + 32 * j + 8 * b + 4 * lh);
                            acc[j][i][4 * b] += bf16_bits_to_f32(bb.x);
                            acc[j][i][4 * b + 1] += bf16_bits_to_f32(bb.y);
                            acc[j][i][4 * b + 2] += bf16_bits_to_f32(bb.z);
                            acc[j][i][4 * b + 3] += bf16_bits_to_f32(bb.w);
                        }
                }
                if (gain) {
                    float ss = 0.f;
#pragma unroll
                    for (int j = 0; j < J; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) ss += acc[j][i][r] * acc[j][i][r];
                    ss += __shfl_xor(ss, 32, 64);
                    const float rs = rsqrtf(ss / 128.f + qa.eps);
#pragma unroll
                    for (int j = 0; j < J; ++j)
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const float4 gg = *(const float4*)(gain + 32 * j + 8 * b + 4 * lh);
                            acc[j][i][4 * b] = acc[j][i][4 * b] * rs * gg.x;
                            acc[j][i][4 * b + 1] = acc[j][i][4 * b + 1] * rs * gg.y;
                            acc[j][i][4 * b + 2] = acc[j][i][4 * b + 2] * rs * gg.z;
                            acc[j][i][4 * b + 3] = acc[j][i][4 * b + 3] * rs * gg.w;
                        }
                }
                if (is_q || is_k) {                      // rotate-half: d pairs with d + 64, i.e. tile j with tile j + 2
                    const float2* cs = qa.rope + (size_t)mm * 64;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const float4 c01 = *(const float4*)(cs + 32 * j + 8 * b + 4 * lh);
                            const float4 c23 = *(const float4*)(cs + 32 * j + 8 * b + 4 * lh + 2);
                            const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float lo = acc[j][i][4 * b + e], hi = acc[j + 2][i][4 * b + e];
                                acc[j][i][4 * b + e] = lo * co[e] - hi * si[e];
                                acc[j + 2][i][4 * b + e] = hi * co[e] + lo * si[e];
                            }
                        }
                }
                if (m < g.M) {
                    uint16_t* dst;
                    int slot = 0;
                    if (is_q) {
                        dst = qa.q + ((size_t)m * qa.n_q_heads + head) * 128;
                    } else {
                        const int2 pp = qa.row_page[m];
                        slot = pp.y & (kPageTokens - 1);
                        dst = qa.pages + ((size_t)pp.x * qa.n_kv_heads + kvh) * (size_t)(2 * kPageTokens * 128) +
                              (is_k ? 0 : kPageTokens * 128);
                    }
#pragma unroll
                    for (int j = 0; j < J; ++j)
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            ushort4 o;
                            o.x = f32_to_act16_noting(acc[j][i][4 * b], bad);
                            o.y = f32_to_act16_noting(acc[j][i][4 * b + 1], bad);
                            o.z = f32_to_act16_noting(acc[j][i][4 * b + 2], bad);
                            o.w = f32_to_act16_noting(acc[j][i][4 * b + 3], bad);
                            if (is_q) {
                                *(ushort4*)(dst + 32 * j + 8 * b + 4 * lh) = o;
                            } else if (is_k) {
                                // K element (token, d) sits at (d/32)*512 + (((d%32)/8)*16 + token)*8 + d%8; d%32 = 8 b + 4 lh + e
                                *(ushort4*)(dst + j * 512 + ((b * 16 + slot) << 3) + 4 * lh) = o;
                            } else {
                                // V element (d, token) sits at (d/32)*512 + ((token/4)*16 + d%16)*8 + ((d/16)%2)*4 + token%4
                                uint16_t* vb = dst + j * 512 + (((slot >> 2) * 16 + 8 * (b & 1) + 4 * lh) << 3) + ((b >> 1) << 2) + (slot & 3);
                                vb[0] = o.x; vb[8] = o.y; vb[16] = o.z; vb[24] = o.w;
                            }
                        }
                }
            }
        }
        report_saturation(qa.sat_count, bad);
    } else if (!SWIGLU) {
        float* out = (float*)g.out;
        constexpr int TROW = 128 * 4 + 16;              // staged row: 128 floats + pad
        char* tb = lds + wave * (32 * TROW);
        const int rr = lane >> 5, c4 = lane & 31;       // read side: row 2 p + rr, floats 4 c4 .. 4 c4 + 3
        const int n = n0 + wn * 128 + 4 * c4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    *(float4*)(tb + l32 * TROW + (j * 32 + 8 * b + 4 * lh) * 4) =
                        make_float4(acc[j][i][4 * b], acc[j][i][4 * b + 1], acc[j][i][4 * b + 2], acc[j][i][4 * b + 3]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 16; ++ps) {
                const int row = 2 * ps + rr;
                const float4 v = *(const float4*)(tb + row * TROW + c4 * 16);
                const int m = m0 + wm * 128 + i * 32 + row;
                if (m < g.M && n < g.N) *(float4*)(out + (size_t)m * g.N + n) = v;
            }
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        bool bad = false;
        constexpr int TROW = 64 * 2 + 16;               // staged row: 64 halves + pad
        char* tb = lds + wave * (32 * TROW);
        const int rr = lane >> 3, c8 = lane & 7;        // read side: row 8 p + rr, halves 8 c8 .. 8 c8 + 7
        const int f = n0 + wn * 64 + 8 * c8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    ushort4 o;
                    o.x = f32_to_act16_noting(silu_f(acc[j][i][4 * b]) * acc[j][i][4 * b + 8], bad);
                    o.y = f32_to_act16_noting(silu_f(acc[j][i][4 * b + 1]) * acc[j][i][4 * b + 9], bad);
                    o.z = f32_to_act16_noting(silu_f(acc[j][i][4 * b + 2]) * acc[j][i][4 * b + 10], bad);
                    o.w = f32_to_act16_noting(silu_f(acc[j][i][4 * b + 3]) * acc[j][i][4 * b + 11], bad);
                    *(ushort4*)(tb + l32 * TROW + (j * 16 + 8 * b + 4 * lh) * 2) = o;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                const int row = 8 * ps + rr;
                const u32x4 v = *(const u32x4*)(tb + row * TROW + c8 * 16);
                const int m = m0 + wm * 128 + i * 32 + row;
                if (m < g.M && f < g.N) *(u32x4*)((uint16_t*)g.out + (size_t)m * g.N + f) = v;
            }
            __builtin_amdgcn_wave_barrier();
        }
        report_saturation(g.sat_count, bad);
    }
}

template <int TEPI>
static hipError_t launch_tile(const GemmArgs& a, const QkvPostArgs& qa, hipStream_t s) {
    const int cols = TEPI == 1 ? 128 : 256;
    const int m_tiles = (a.M + BM - 1) / BM;
    const int n_tiles = (a.N + cols - 1) / cols;
    const int per_xcd = (m_tiles * n_tiles + 7) / 8;
    const size_t lds_bytes = (size_t)2 * STAGE_BYTES;
    hipError_t e = hipFuncSetAttribute((const void*)gemm_tile_kernel<TEPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_tile_kernel<TEPI>), dim3(per_xcd * 8), dim3(256), lds_bytes, s, a, qa);
    return hipGetLastError();
}

// needs the fragment-ordered weights (a.wf), K % 64 == 0 and operands small enough for 32-bit element offsets
bool gemm_tile_usable(const GemmArgs& a) {
    return a.wf != nullptr && a.splits == 1 && (a.K % BK) == 0 && (a.N & 3) == 0 &&
           (long long)a.M * a.K < (1ll << 31) && ((long long)a.N + 32) * 2 * a.K < (1ll << 31);
}

hipError_t launch_gemm_tile(const GemmArgs& a, int epilogue, hipStream_t s) {
    if (!gemm_tile_usable(a) || (epilogue == EPI_SWIGLU && (a.N & 7))) return hipErrorInvalidValue;
    const QkvPostArgs none = {};
    return epilogue == EPI_SWIGLU ? launch_tile<1>(a, none, s) : launch_tile<0>(a, none, s);
}

// The q/k/v projection with the work of qkv_post_kernel in its epilogue (qa.qkv and qa.n_part are not used).
bool gemm_tile_qkv_usable(const GemmArgs& a, const QkvPostArgs& qa, bool w_bf16) {
    const long tiles = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
    return w_bf16 && a.M >= 512 && tiles >= 200 && gemm_tile_usable(a) && qa.hd == 128 && (a.N & 255) == 0 &&
           a.N == (qa.n_q_heads + 2 * qa.n_kv_heads) * 128;
}

hipError_t launch_gemm_tile_qkv(const GemmArgs& a, const QkvPostArgs& qa, hipStream_t s) {
    if (!gemm_tile_qkv_usable(a, qa, true)) return hipErrorInvalidValue;
    return launch_tile<2>(a, qa, s);
}

}  // namespace spiral
