// Truncated (top-k / top-p) Gumbel-max sampler.
//
// Per row: z_v = logit_v / T; the keep set is { z_v >= tau } with tau the larger of the k-th largest z
// (top-k) and the z at which the descending running sum of softmax(z) over the top-k survivors first
// reaches p (top-p); the token is the argmax of z + g over the keep set.  Both thresholds are found by
// a most-significant-digit-first radix descent over an order-preserving 32-bit key of z, 8 bits per
// pass: top-k walks a histogram of counts, top-p a histogram of probability mass.  Mass is held in
// 64-bit fixed point (float64 exp(z - max) * 2^45: integer adds in any order give the same sum, so the
// result is bit-reproducible, and the running sums agree with exact arithmetic to ~2e-9 of the largest
// term summed over a 152k vocabulary); a token lighter than 2^-46 of the heaviest one counts as zero.
// One block of 1024 threads per row; each wave fills its own histogram copy in LDS.
#include "spiral_internal.h"

namespace spiral {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

// larger float <=> larger key; -0 and +0 share a key
__device__ __forceinline__ uint32_t order_key(float z) {
    const uint32_t b = __float_as_uint(z + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__device__ __forceinline__ uint64_t shfl_down_u64(uint64_t v, int d) {
    const uint32_t lo = __shfl_down((uint32_t)v, d, 64), hi = __shfl_down((uint32_t)(v >> 32), d, 64);
    return ((uint64_t)hi << 32) | lo;
}

struct Select {
    uint32_t prefix;       // digits fixed so far (high bits)
    uint64_t remaining;    // how much (count or mass) must still be covered from the top of the current bucket
};

// Among the 256 bins (sum over the waves' copies), walking from bin 255 down, the bin in which the
// running total first reaches `remaining`.  Executed by wave 0; result broadcast through LDS.
__device__ __forceinline__ void pick_bin(const uint64_t* hist, int shift, Select* sel, uint64_t* total_out, int lane) {
    uint64_t b[4];
    uint64_t mine = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint64_t s = 0;
        for (int w = 0; w < kWaves; ++w) s += hist[w * 256 + lane * 4 + i];
        b[i] = s;
        mine += s;
    }
    // suffix sums over lanes: above = total of the bins of all higher lanes
    uint64_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = shfl_down_u64(incl, d);
        if (lane + d < 64) incl += o;
    }
    const uint64_t above = incl - mine;
    if (lane == 0 && total_out) *total_out = incl;
    const uint64_t need = sel->remaining;
    if (above < need && need <= incl) {             // exactly one lane when need <= total
        uint64_t acc = above;
#pragma unroll
        for (int i = 3; i >= 0; --i) {
            if (acc + b[i] >= need) {
                sel->prefix |= (uint32_t)(lane * 4 + i) << shift;
                sel->remaining = need - acc;
                break;
            }
            acc += b[i];
        }
    }
}

}  // namespace

__global__ __launch_bounds__(kThreads) void sample_truncated_kernel(const float* logits, int V, float temperature, int top_k,
                                                                    float top_p, int use_noise_buffer, KeyChunk keys,
                                                                    const float* noise, int32_t* out, float* tau_out) {
    __shared__ uint64_t hist[kWaves * 256];
    __shared__ Select sel;
    __shared__ uint64_t s_total;
    __shared__ float s_red[kWaves];
    __shared__ int s_idx[kWaves];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* lr = logits + (size_t)row * V;
    uint64_t* my_hist = hist + wave * 256;

    auto clear_hist = [&] {
        for (int i = tid; i < kWaves * 256; i += kThreads) hist[i] = 0;
        __syncthreads();
    };

    // ---- max of z (the softmax reference point)
    float zmax = -INFINITY;
    for (int v = tid; v < V; v += kThreads) zmax = fmaxf(zmax, lr[v] / temperature);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 64));
    if (lane == 0) s_red[wave] = zmax;
    __syncthreads();
    zmax = s_red[0];
    for (int w = 1; w < kWaves; ++w) zmax = fmaxf(zmax, s_red[w]);
    __syncthreads();

    uint32_t floor_key = 0;                      // keys below it are cut

    // ---- top-k: the key of the k-th largest z
    if (top_k > 0 && top_k < V) {
        if (tid == 0) { sel.prefix = 0; sel.remaining = (uint64_t)top_k; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            clear_hist();
            const uint32_t prefix = sel.prefix;
            for (int v = tid; v < V; v += kThreads) {
                const uint32_t key = order_key(lr[v] / temperature);
                if (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
                    atomicAdd((unsigned long long*)&my_hist[(key >> shift) & 255u], 1ull);
            }
            __syncthreads();
            if (wave == 0) pick_bin(hist, shift, &sel, nullptr, lane);
            __syncthreads();
        }
        floor_key = sel.prefix;
        __syncthreads();
    }

    // ---- top-p over the survivors: the key at which the descending running mass first reaches p * Z
    if (top_p < 1.0f) {
        if (tid == 0) { sel.prefix = 0; sel.remaining = 0; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            clear_hist();
            const uint32_t prefix = sel.prefix;
            for (int v = tid; v < V; v += kThreads) {
                const float z = lr[v] / temperature;
                const uint32_t key = order_key(z);
                if (key >= floor_key && (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))) {
                    const uint64_t mass = (uint64_t)(exp((double)z - (double)zmax) * 35184372088832.0);      // 2^45
                    atomicAdd((unsigned long long*)&my_hist[(key >> shift) & 255u], (unsigned long long)mass);
                }
            }
            __syncthreads();
            if (pass == 0) {
                // the first histogram holds the whole surviving mass Z: fix the target, then pick
                if (wave == 0) {
                    uint64_t mine = 0;
                    for (int i = 0; i < 4; ++i)
                        for (int w = 0; w < kWaves; ++w) mine += hist[w * 256 + lane * 4 + i];
#pragma unroll
                    for (int d = 1; d < 64; d <<= 1) {
                        const uint64_t o = shfl_down_u64(mine, d);
                        if (lane + d < 64) mine += o;
                    }
                    if (lane == 0) {
                        const uint64_t Z = mine;
                        uint64_t target = (uint64_t)ceil((double)top_p * (double)Z);
                        if (target < 1) target = 1;
                        if (target > Z) target = Z;
                        sel.remaining = target;
                        s_total = Z;
                    }
                }
                __syncthreads();
            }
            if (wave == 0) pick_bin(hist, shift, &sel, nullptr, lane);
            __syncthreads();
        }
        if (sel.prefix > floor_key) floor_key = sel.prefix;
        __syncthreads();
    }

    // ---- Gumbel-max over the keep set
    const float* nr = use_noise_buffer ? noise + (size_t)row * V : nullptr;
    const uint64_t key64 = keys.key[row];
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int v = tid; v < V; v += kThreads) {
        const float z = lr[v] / temperature;
        if (order_key(z) < floor_key) continue;
        float g;
        if (nr) {
            g = nr[v];
        } else {
            const uint32_t r = (uint32_t)(mix64(key64 + (uint64_t)v * 0x9E3779B97F4A7C15ull) >> 32);
            const float u = ((float)(r >> 9) + 0.5f) * 1.1920928955078125e-07f;   // 2^-23
            g = -logf(-logf(u));
        }
        const float sc = z + g;
        if (sc > bv || (sc == bv && v < bi)) { bv = sc; bi = v; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { s_red[wave] = bv; s_idx[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w)
            if (s_red[w] > bv || (s_red[w] == bv && s_idx[w] < bi)) { bv = s_red[w]; bi = s_idx[w]; }
        out[row] = bi == 0x7FFFFFFF ? 0 : bi;
        if (tau_out) tau_out[row] = floor_key == 0 ? -INFINITY : key_value(floor_key);
    }
}

hipError_t launch_sample_truncated(const float* logits, int B, int V, float temperature, int top_k, float top_p,
                                   const uint64_t* host_keys, const float* noise, int32_t* out, float* tau_out,
                                   hipStream_t s) {
    for (int off = 0; off < B; off += 128) {
        KeyChunk k;
        const int m = B - off < 128 ? B - off : 128;
        for (int i = 0; i < m; ++i) k.key[i] = host_keys ? host_keys[off + i] : 0;
        hipLaunchKernelGGL(sample_truncated_kernel, dim3(m), dim3(kThreads), 0, s, logits + (size_t)off * V, V, temperature,
                           top_k, top_p, noise ? 1 : 0, k, noise ? noise + (size_t)off * V : nullptr, out + off,
                           tau_out ? tau_out + off : nullptr);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace spiral
