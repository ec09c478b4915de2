// Small memory-bound kernels of the decode path: embedding + RMSNorm, residual-add + RMSNorm,
// the fused q/k/v post-processing (bias | per-head RMSNorm, RoPE, KV append), the Gumbel-max
// sampler, and the by-value uploads that keep the library free of device allocations.
#include <algorithm>

#include "spiral_internal.h"
#include "mfma_ops.h"

namespace spiral {

// ---------------------------------------------------------------------------------------------
// plumbing
// ---------------------------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint4* p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (; i < n16; i += stride) p[i] = z;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    size_t n16 = bytes / 16;          // callers pass multiples of 16
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, n16);
    return hipGetLastError();
}

__global__ void upload_kernel(int32_t* dst, IntChunk c, int n) {
    int i = threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

hipError_t launch_upload(int32_t* dev_dst, const int32_t* host_src, int n, hipStream_t s) {
    for (int off = 0; off < n; off += kUploadInts) {
        IntChunk c;
        int m = n - off < kUploadInts ? n - off : kUploadInts;
        for (int i = 0; i < m; ++i) c.v[i] = host_src[off + i];
        hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(kUploadInts), 0, s, dev_dst + off, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// several short host arrays in one launch: segment j of the packed chunk goes to dst[j]
struct UploadPlan { int32_t* dst[4]; int32_t first[5]; };      // first[j] .. first[j + 1]: segment j inside the chunk
__global__ void upload_multi_kernel(UploadPlan p, IntChunk c, int n) {
    const int i = threadIdx.x;
    if (i >= n) return;
    int j = 0;
    while (j < 3 && i >= p.first[j + 1]) ++j;
    p.dst[j][i - p.first[j]] = c.v[i];
}

hipError_t launch_upload_multi(int32_t* const* dev_dst, const int32_t* const* host_src, const int* n, int n_seg, hipStream_t s) {
    if (n_seg < 1 || n_seg > 4) return hipErrorInvalidValue;
    int total = 0;
    for (int j = 0; j < n_seg; ++j) total += n[j];
    if (total > kUploadInts) {                       // too long for one chunk: one upload per array
        for (int j = 0; j < n_seg; ++j) {
            hipError_t e = launch_upload(dev_dst[j], host_src[j], n[j], s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    UploadPlan p;
    IntChunk c;
    int off = 0;
    for (int j = 0; j < 4; ++j) {
        p.first[j] = off;
        p.dst[j] = j < n_seg ? dev_dst[j] : nullptr;
        if (j < n_seg) { for (int i = 0; i < n[j]; ++i) c.v[off + i] = host_src[j][i]; off += n[j]; }
    }
    p.first[4] = off;
    hipLaunchKernelGGL(upload_multi_kernel, dim3(1), dim3(kUploadInts), 0, s, p, c, total);
    return hipGetLastError();
}

__global__ void scatter_kernel(int32_t* base, PairChunk c, int n) {
    int i = threadIdx.x;
    if (i < n) base[c.idx[i]] = c.val[i];
}

hipError_t launch_scatter(int32_t* dev_base, const int32_t* host_idx, const int32_t* host_val, int n, hipStream_t s) {
    const int per = kUploadInts / 2;
    for (int off = 0; off < n; off += per) {
        PairChunk c;
        int m = n - off < per ? n - off : per;
        for (int i = 0; i < m; ++i) { c.idx[i] = host_idx[off + i]; c.val[i] = host_val[off + i]; }
        hipLaunchKernelGGL(scatter_kernel, dim3(1), dim3(per), 0, s, dev_base, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// row -> (sequence, position) for a packed prefill batch
__global__ void prefill_meta_kernel(const int32_t* cu_rows, const int32_t* base_pos, const int32_t* seq_ids,
                                    int B, int n_rows, int32_t* row_seq, int32_t* row_pos) {
    int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    int lo = 0, hi = B - 1;              // largest b with cu_rows[b] <= r
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (cu_rows[mid] <= r) lo = mid; else hi = mid - 1;
    }
    row_seq[r] = seq_ids[lo];
    row_pos[r] = base_pos[lo] + (r - cu_rows[lo]);
}

hipError_t launch_prefill_meta(const int32_t* cu_rows, const int32_t* base_pos, const int32_t* seq_ids, int B,
                               int n_rows, int32_t* row_seq, int32_t* row_pos, hipStream_t s) {
    hipLaunchKernelGGL(prefill_meta_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, s,
                       cu_rows, base_pos, seq_ids, B, n_rows, row_seq, row_pos);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// block reduction (256 threads)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return t;
}

// ---------------------------------------------------------------------------------------------
// embedding gather + first RMSNorm (+ positions and the RoPE table of this step)
// One block per row.  h = x * rsqrt(mean(x^2) + eps) * gain.
// ---------------------------------------------------------------------------------------------
template <bool WBF16, bool ACT32>
__global__ __launch_bounds__(256) void embed_norm_kernel(EmbedArgs a, RopeFreq f) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    const int pos = a.row_pos[r];
    if ((int)threadIdx.x < a.half_hd) {
        double ang = (double)pos * f.inv_freq[threadIdx.x];
        a.rope[(size_t)r * a.half_hd + threadIdx.x] = make_float2((float)cos(ang), (float)sin(ang));
    }
    if (threadIdx.x == 255)
        a.row_page[r] = make_int2(a.block_table[(size_t)a.row_seq[r] * a.max_blocks + (pos >> 4)], pos);
    int tok = a.tokens[r];
    tok = tok < 0 ? 0 : (tok >= a.vocab ? a.vocab - 1 : tok);   // ids are validated by the caller; stay in bounds regardless
    float* x = a.x + (size_t)r * a.d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < a.d; i += 256) {
        float v;
        if (WBF16) v = bf16_bits_to_f32(((const uint16_t*)a.embed)[(size_t)tok * a.d + i]);
        else v = ((const float*)a.embed)[(size_t)tok * a.d + i];
        x[i] = v;
        ss += v * v;
    }
    ss = block_sum_256(ss, red);
    const float rs = rsqrtf(ss / (float)a.d + a.eps);
    for (int i = threadIdx.x; i < a.d; i += 256)
        ActStore<ACT32>::put(a.h, (size_t)r * a.d + i, x[i] * rs * a.gain[i]);
}

hipError_t launch_embed_norm(const EmbedArgs& a, const RopeFreq& f, bool w_bf16, bool act32, hipStream_t s) {
    dim3 g(a.n_rows), b(256);
    if (w_bf16 && !act32) hipLaunchKernelGGL((embed_norm_kernel<true, false>), g, b, 0, s, a, f);
    else if (!w_bf16 && act32) hipLaunchKernelGGL((embed_norm_kernel<false, true>), g, b, 0, s, a, f);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// residual add of the split-K projection partials + RMSNorm.  One block per output row.
// ---------------------------------------------------------------------------------------------
// Wide variant: d % 4 == 0 and d <= 8192.  One block of up to 1024 threads per row; a thread owns at
// most two groups of 4 columns, issues all of their partial-sum loads at once and keeps the sums in
// registers between the reduction and the normalised store.
template <bool ACT32>
__global__ __launch_bounds__(1024) void add_norm_wide_kernel(NormArgs a) {
    __shared__ float red[16];
    const int ro = blockIdx.x;
    const int ri = a.row_map ? a.row_map[ro] : ro;
    float* x = a.x + (size_t)ri * a.d;
    const size_t pstride = (size_t)a.rows_in * a.d;
    const float* prow = a.part + (size_t)ri * a.d;
    const int groups = a.d >> 2;
    float4 v[2], gn[2];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int gidx = threadIdx.x + j * blockDim.x;
        v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        gn[j] = *(const float4*)(a.gain + (gidx < groups ? gidx : groups - 1) * 4);     // with the other loads, not behind the barrier
        if (gidx < groups) {
            const int i = gidx * 4;
            float4 acc = *(const float4*)(x + i);
            float4 pv[16];
#pragma unroll
            for (int p = 0; p < 16; ++p)
                pv[p] = p < a.n_part ? *(const float4*)(prow + p * pstride + i) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int p = 0; p < 16; ++p) { acc.x += pv[p].x; acc.y += pv[p].y; acc.z += pv[p].z; acc.w += pv[p].w; }
            for (int p = 16; p < a.n_part; ++p) {
                const float4 q = *(const float4*)(prow + p * pstride + i);
                acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
            }
            if (a.n_part > 0) *(float4*)(x + i) = acc;
            v[j] = acc;
            ss += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
        }
    }
    ss = wave_sum(ss);
    const int wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < n_waves; ++w) tot += red[w];
    const float rs = rsqrtf(tot / (float)a.d + a.eps);
    bool bad = false;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int gidx = threadIdx.x + j * blockDim.x;
        if (gidx < groups) {
            const int i = gidx * 4;
            const size_t o = (size_t)ro * a.d + i;
            ActStore<ACT32>::put_noting(a.h, o, v[j].x * rs * gn[j].x, bad);
            ActStore<ACT32>::put_noting(a.h, o + 1, v[j].y * rs * gn[j].y, bad);
            ActStore<ACT32>::put_noting(a.h, o + 2, v[j].z * rs * gn[j].z, bad);
            ActStore<ACT32>::put_noting(a.h, o + 3, v[j].w * rs * gn[j].w, bad);
        }
    }
    report_saturation(a.sat_count, bad);
}

template <bool ACT32>
__global__ __launch_bounds__(256) void add_norm_kernel(NormArgs a) {
    __shared__ float red[4];
    const int ro = blockIdx.x;
    const int ri = a.row_map ? a.row_map[ro] : ro;
    float* x = a.x + (size_t)ri * a.d;
    const size_t pstride = (size_t)a.rows_in * a.d;
    const float* prow = a.part + (size_t)ri * a.d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < a.d; i += 256) {
        float v = x[i];
        for (int p = 0; p < a.n_part; ++p) v += prow[p * pstride + i];
        if (a.n_part > 0) x[i] = v;
        ss += v * v;
    }
    ss = block_sum_256(ss, red);
    const float rs = rsqrtf(ss / (float)a.d + a.eps);
    bool bad = false;
    for (int i = threadIdx.x; i < a.d; i += 256)
        ActStore<ACT32>::put_noting(a.h, (size_t)ro * a.d + i, x[i] * rs * a.gain[i], bad);
    report_saturation(a.sat_count, bad);
}

hipError_t launch_add_norm(const NormArgs& a, bool act32, hipStream_t s) {
    if ((a.d & 3) == 0 && a.d <= 8192) {
        int threads = ((a.d >> 2) + 63) & ~63;
        if (threads > 1024) threads = 1024;
        dim3 g(a.rows_out), b(threads);
        if (act32) hipLaunchKernelGGL((add_norm_wide_kernel<true>), g, b, 0, s, a);
        else hipLaunchKernelGGL((add_norm_wide_kernel<false>), g, b, 0, s, a);
        return hipGetLastError();
    }
    dim3 g(a.rows_out), b(256);
    if (act32) hipLaunchKernelGGL((add_norm_kernel<true>), g, b, 0, s, a);
    else hipLaunchKernelGGL((add_norm_kernel<false>), g, b, 0, s, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// q/k/v post-processing: sum the projection partials, add the bias, RMSNorm each q/k head over
// head_dim (before RoPE), rotate q/k (rotate-half pairing), store q as bf16 and append k, v to the
// sequence's page in MFMA operand order (layout in kernels_attn.hip).
// One wave per (row, head); lane p handles the pair (p, p + hd/2).
// ---------------------------------------------------------------------------------------------
// NP: the number of partials the kernel is built for (>= a.n_part).  Every load of a lane - partials, bias, gains,
// rotation, page look-up - is issued before the first use and none sits behind a branch: written as a loop over the
// partials the compiler waits for each pair before it requests the next, nine dependent round trips per wave.
template <bool WBF16, int NP>
__global__ __launch_bounds__(256) void qkv_post_kernel(QkvPostArgs a) {
    const int r = blockIdx.x;
    const int head = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n_heads = a.n_q_heads + 2 * a.n_kv_heads;
    if (head >= n_heads) return;
    const int hd = a.hd, half = hd >> 1;
    const int width = n_heads * hd;
    const bool is_q = head < a.n_q_heads;
    const bool is_k = !is_q && head < a.n_q_heads + a.n_kv_heads;
    const int kvh = is_q ? 0 : (is_k ? head - a.n_q_heads : head - a.n_q_heads - a.n_kv_heads);

    const void* bias = is_q ? a.bq : (is_k ? a.bk : a.bv);
    const int bias_off = (is_q ? head : kvh) * hd;
    const float* gain = is_q ? a.q_gain : (is_k ? a.k_gain : nullptr);

    const int2 pp = a.row_page[r];                       // (page, position): q heads read it too and ignore it
    const int slot = pp.y & (kPageTokens - 1);
    const size_t page_base = ((size_t)pp.x * a.n_kv_heads + kvh) * (size_t)(2 * kPageTokens * hd);

    bool bad = false;
    for (int p = lane; p < ((half + 63) & ~63); p += 64) {
        const bool act = p < half;
        const int pc = act ? p : half - 1;              // idle lanes re-read the last pair
        float pl[NP], ph[NP];
#pragma unroll
        for (int s = 0; s < NP; ++s) {
            const int sc = s < a.n_part ? s : a.n_part - 1;
            const float* src = a.qkv + ((size_t)sc * a.n_rows + r) * width + (size_t)head * hd;
            pl[s] = src[pc];
            ph[s] = src[pc + half];
        }
        float b_lo = 0.f, b_hi = 0.f, g_lo = 1.f, g_hi = 1.f;
        if (bias) {                                     // uniform over the wave
            if (WBF16) {
                b_lo = bf16_bits_to_f32(((const uint16_t*)bias)[bias_off + pc]);
                b_hi = bf16_bits_to_f32(((const uint16_t*)bias)[bias_off + pc + half]);
            } else {
                b_lo = ((const float*)bias)[bias_off + pc];
                b_hi = ((const float*)bias)[bias_off + pc + half];
            }
        }
        if (gain) { g_lo = gain[pc]; g_hi = gain[pc + half]; }
        const float2 cs = a.rope[(size_t)r * half + pc];
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int s = 0; s < NP; ++s)
            if (s < a.n_part) { lo += pl[s]; hi += ph[s]; }
        if (bias) { lo += b_lo; hi += b_hi; }
        if (!act) { lo = 0.f; hi = 0.f; }
        if (gain) {       // hd <= 128: the whole head sits in one pass of the wave
            const float ss = wave_sum(lo * lo + hi * hi);
            const float rs = rsqrtf(ss / (float)hd + a.eps);
            lo = lo * rs * g_lo; hi = hi * rs * g_hi;
        }
        if (!act) continue;
        if (is_q || is_k) {
            const float nlo = lo * cs.x - hi * cs.y;
            const float nhi = hi * cs.x + lo * cs.y;
            lo = nlo; hi = nhi;
        }
        if (is_q) {
            uint16_t* q = a.q + ((size_t)r * a.n_q_heads + head) * hd;
            q[p] = f32_to_act16_noting(lo, bad);
            q[p + half] = f32_to_act16_noting(hi, bad);
        } else if (is_k) {
            // K element (token, d) sits at (d/32)*512 + (((d%32)/8)*16 + token)*8 + d%8
            uint16_t* K = a.pages + page_base;
            const int d0 = p, d1 = p + half;
            K[(d0 >> 5) * 512 + ((((d0 & 31) >> 3) * 16 + slot) << 3) + (d0 & 7)] = f32_to_act16_noting(lo, bad);
            K[(d1 >> 5) * 512 + ((((d1 & 31) >> 3) * 16 + slot) << 3) + (d1 & 7)] = f32_to_act16_noting(hi, bad);
        } else {
            // V element (d, token) sits at (d/32)*512 + ((token/4)*16 + d%16)*8 + ((d/16)%2)*4 + token%4
            uint16_t* V = a.pages + page_base + (size_t)kPageTokens * hd;
            const int d0 = p, d1 = p + half;
            V[(d0 >> 5) * 512 + ((((slot >> 2) * 16) + (d0 & 15)) << 3) + (((d0 >> 4) & 1) << 2) + (slot & 3)] = f32_to_act16_noting(lo, bad);
            V[(d1 >> 5) * 512 + ((((slot >> 2) * 16) + (d1 & 15)) << 3) + (((d1 >> 4) & 1) << 2) + (slot & 3)] = f32_to_act16_noting(hi, bad);
        }
    }
    report_saturation(a.sat_count, bad);
}

template <int NP>
static void launch_qkv_post_np(const QkvPostArgs& a, bool w_bf16, dim3 g, hipStream_t s) {
    if (w_bf16) hipLaunchKernelGGL((qkv_post_kernel<true, NP>), g, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((qkv_post_kernel<false, NP>), g, dim3(256), 0, s, a);
}

hipError_t launch_qkv_post(const QkvPostArgs& a, bool w_bf16, hipStream_t s) {
    const int n_heads = a.n_q_heads + 2 * a.n_kv_heads;
    if (a.n_part < 1 || a.n_part > 16 || a.hd < 2) return hipErrorInvalidValue;
    dim3 g(a.n_rows, (n_heads + 3) / 4);
    if (a.n_part == 1) launch_qkv_post_np<1>(a, w_bf16, g, s);
    else if (a.n_part <= 5) launch_qkv_post_np<5>(a, w_bf16, g, s);
    else if (a.n_part <= 8) launch_qkv_post_np<8>(a, w_bf16, g, s);
    else launch_qkv_post_np<16>(a, w_bf16, g, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Weight repack: row-major [N][K] bf16 rows -> fragment order (frag_block()), in the matrix cores' operand type.  Rows come from up to
// three stacked blocks (q | k | v), or, interleaved, tile t takes rows 16 t .. 16 t + 15 of src0 (gate)
// followed by the same rows of src1 (up).  Rows past the end are zero.  One thread per 16 bytes.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void repack_kernel(const uint16_t* s0, const uint16_t* s1, const uint16_t* s2, int r0, int r1,
                                                     int r2, int K, int interleave16, uint4* dst, long long n_units) {
    const int ksteps = K >> 4;
    for (long long u = (long long)blockIdx.x * 256 + threadIdx.x; u < n_units; u += (long long)gridDim.x * 256) {
        const int lane = (int)(u & 63);
        const long long blk = u >> 6;
        const int ks = (int)(blk % ksteps), t = (int)(blk / ksteps);
        const int l32 = lane & 31, lh = lane >> 5;
        const uint16_t* src = nullptr;
        if (interleave16) {
            const int row = t * 16 + (l32 & 15);
            if (row < r0) src = (l32 < 16 ? s0 : s1) + (size_t)row * K;
        } else {
            int row = t * 32 + l32;
            if (row < r0) src = s0 + (size_t)row * K;
            else if (row < r0 + r1) src = s1 + (size_t)(row - r0) * K;
            else if (row < r0 + r1 + r2) src = s2 + (size_t)(row - r0 - r1) * K;
        }
        uint4 v = src ? *(const uint4*)(src + ks * 16 + lh * 8) : make_uint4(0u, 0u, 0u, 0u);
        // the copy holds the operand type of the matrix cores (bf16 widened to half exactly as the kernels
        // do it in registers when they read row-major weights), so the GEMM kernels skip the conversion
        const u32x4 c = prep_w(u32x4{v.x, v.y, v.z, v.w});
        dst[u] = make_uint4(c.x, c.y, c.z, c.w);
    }
}

hipError_t launch_repack(const void* src0, const void* src1, const void* src2, int rows0, int rows1, int rows2, int K,
                         bool interleave16, void* dst, hipStream_t s) {
    if (K & 15) return hipErrorInvalidValue;
    const long long tiles = interleave16 ? (rows0 + 15) / 16 : (rows0 + rows1 + rows2 + 31) / 32;
    const long long n_units = tiles * (K >> 4) * 64;
    const int blocks = (int)std::min<long long>((n_units + 255) / 256, 65536);
    hipLaunchKernelGGL(repack_kernel, dim3(blocks), dim3(256), 0, s, (const uint16_t*)src0, (const uint16_t*)src1,
                       (const uint16_t*)src2, rows0, rows1, rows2, K, interleave16 ? 1 : 0, (uint4*)dst, n_units);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Gumbel-max sampler: token = argmax_v(logit_v / T + g_v), lowest index on ties; T == 0 => greedy.
// One block of 1024 threads per row; every thread scans a strided slice, then a wave shuffle
// reduction and a 16-entry LDS reduction pick the winner.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sample_kernel(const float* logits, int V, float temperature, int mode,
                                                      KeyChunk keys, const float* noise, int32_t* out) {
    // mode 0: greedy; 1: generated noise; 2: noise buffer
    __shared__ float s_v[16];
    __shared__ int s_i[16];
    const int row = blockIdx.x;
    const float* lr = logits + (size_t)row * V;
    const float* nr = noise ? noise + (size_t)row * V : nullptr;
    const uint64_t key = keys.key[row];
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    // eight loads in flight per thread (past the end they re-read the last entry: a branch around a load makes
    // every load wait)
    for (int base = threadIdx.x; base < V; base += 1024 * 8) {
        float l[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) l[u] = lr[min(base + u * 1024, V - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int v = base + u * 1024;
            if (v >= V) continue;
            float sc = l[u];
            if (mode != 0) {
                const float g = mode == 2 ? nr[v] : gumbel_noise(key, v);
                sc = sc / temperature + g;      // IEEE division, as the definition states it
            }
            if (better(sc, v, bv, bi)) { bv = sc; bi = v; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_v[wave] = bv; s_i[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
        out[row] = bi == 0x7FFFFFFF ? 0 : bi;
    }
}

hipError_t launch_sample(const float* logits, int B, int V, float temperature, const uint64_t* host_keys,
                         const float* noise, int32_t* out, hipStream_t s) {
    const int mode = temperature == 0.0f ? 0 : (noise ? 2 : 1);
    for (int off = 0; off < B; off += 128) {
        KeyChunk k;
        const int m = B - off < 128 ? B - off : 128;
        for (int i = 0; i < m; ++i) k.key[i] = host_keys ? host_keys[off + i] : 0;
        hipLaunchKernelGGL(sample_kernel, dim3(m), dim3(1024), 0, s, logits + (size_t)off * V, V, temperature, mode,
                           k, noise ? noise + (size_t)off * V : nullptr, out + off);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// Measurement: a pure streaming read with the access pattern of the decode step's once-read streams (every
// wave keeps eight 16-byte loads per lane in flight, non-temporal), as the yardstick for "what this GPU streams".
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* p, size_t n16) {
    size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * 8;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 256 * 7 < n16; i += stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + 256 * u);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    asm volatile("" ::"v"(acc.x ^ acc.y ^ acc.z ^ acc.w));      // keeps the loads alive; nothing is written
}

hipError_t launch_stream_read(const void* p, size_t bytes, int workgroups, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, s, (const u32x4*)p, bytes / 16);
    return hipGetLastError();
}

// Second half of the fused LM head + sampler: the winner among the per-tile (score, index) pairs of a row.
__global__ __launch_bounds__(256) void sample_pick_kernel(const float2* part, int n_tiles, int32_t* out) {
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const int row = blockIdx.x;
    const float2* pr = part + (size_t)row * n_tiles;
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int t = threadIdx.x; t < n_tiles; t += 256) {
        const float2 e = pr[t];
        const int i = __float_as_int(e.y);
        if (better(e.x, i, bv, bi)) { bv = e.x; bi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_v[wave] = bv; s_i[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w)
            if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
        out[row] = bi == 0x7FFFFFFF ? 0 : bi;
    }
}

hipError_t launch_sample_pick(const float2* part, int B, int n_tiles, int32_t* out, hipStream_t s) {
    hipLaunchKernelGGL(sample_pick_kernel, dim3(B), dim3(256), 0, s, part, n_tiles, out);
    return hipGetLastError();
}

}  // namespace spiral
