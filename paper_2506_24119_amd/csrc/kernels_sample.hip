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
//
// With a workspace the same thresholds are found in three sweeps of the row instead of up to nine, and by several
// workgroups per row: (1) row maximum; (2) one histogram of count and mass over 4096 bins that are linear in
// zmax - z (width 1/128; the last bin takes everything 32 or more below the maximum, whose mass is zero in the
// 2^45 fixed point); an integer prefix sum over the bins names the bin that holds the cut; (3) one sweep that
// scores the tokens in the bins above the cut for the Gumbel-max and copies the tokens of the cut bin (a few
// hundred to a few thousand) to a candidate list, on which the radix descent then runs in LDS.  Bin order follows
// key order and the masses are the same integers, so the threshold is the one the single-kernel path finds, bit for
// bit; a row whose cut bin holds more candidates than the list (many equal scores) is left to that path.
#include <algorithm>

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

// f(logit, v) for v = lo + tid, lo + tid + kThreads, ... < hi, with U loads in flight per thread (issued before the
// first use; past the end they re-read the last entry, a branch around a load would make every load wait)
template <int U, class F>
__device__ __forceinline__ void sweep(const float* lr, int lo, int hi, int tid, F&& f) {
    for (int base = lo + tid; base < hi; base += kThreads * U) {
        float l[U];
#pragma unroll
        for (int u = 0; u < U; ++u) l[u] = lr[min(base + u * kThreads, hi - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = base + u * kThreads;
            if (v < hi) f(l[u], v);
        }
    }
}

__device__ __forceinline__ uint64_t shfl_down_u64(uint64_t v, int d) {
    const uint32_t lo = __shfl_down((uint32_t)v, d, 64), hi = __shfl_down((uint32_t)(v >> 32), d, 64);
    return ((uint64_t)hi << 32) | lo;
}

// 2^(j/32), j = 0..31
__device__ const double kExp2Tab[32] = {
    1.0, 1.0218971486541166, 1.0442737824274138, 1.0671404006768237,
    1.0905077326652577, 1.1143867425958924, 1.1387886347566916, 1.1637248587775775,
    1.189207115002721, 1.215247359980469, 1.241857812073484, 1.2690509571917332,
    1.2968395546510096, 1.3252366431597413, 1.3542555469368927, 1.383909881963832,
    1.4142135623730951, 1.4451808069770467, 1.4768261459394993, 1.5091644275934228,
    1.5422108254079407, 1.5759808451078865, 1.6104903319492543, 1.645755478153965,
    1.681792830507429, 1.718619298122478, 1.7562521603732995, 1.7947090750031072,
    1.8340080864093424, 1.8741676341103, 1.9152065613971474, 1.9571441241754002};

// floor(exp(z - zmax) * 2^45) for z <= zmax; zero from 32 below the maximum on (exp(-32) * 2^45 < 1) and for
// z = -inf.  exp(x) = 2^(k/32) * exp(r) with k = round(32 x / ln 2): the table gives 2^((k mod 32)/32), the Taylor
// series to the 6th power exp(r) for |r| <= ln 2 / 64 (remainder 4e-18), ldexp the rest; 4e-16 of exp() at worst.
__device__ __forceinline__ uint64_t mass45(float z, float zmax) {
    const double x = (double)z - (double)zmax;
    if (!(x > -32.0)) return 0;
    const double k = rint(x * 46.16624130844683);
    double r = fma(-k, 0.021660849392489467, x);       // ln 2 / 32, high part (12 trailing zero bits: k * hi is exact)
    r = fma(-k, 8.823528300947368e-15, r);             // low part
    double p = 1.0 / 720.0;
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    const int ki = (int)k;                              // <= 0
    return (uint64_t)ldexp(kExp2Tab[ki & 31] * p, (ki >> 5) + 45);
}

constexpr int kBins = 4096;           // linear in zmax - z, 1/128 wide; the last one is everything >= 32 below the maximum
constexpr int kCap = 8192;            // candidates of a row that the in-LDS resolution takes
constexpr int kMaxSlices = 8;         // workgroups per row

// What the prefix sum over a row's histogram decides (one per row, in the workspace).
struct TruncRow {
    float zmax;
    int cand_lo, cand_hi;             // tokens in bins [cand_lo, cand_hi] go to the candidate list; bins below cand_lo are kept
    int fallback;                     // more candidates than the list holds: the single-kernel path does this row
    uint64_t need_mass;               // top-p alone: fixed-point mass still to be covered inside the candidate bin
    uint32_t need_count;              // top-k: how many of the candidates, from the largest, are kept
    int n_cand;
};

__device__ __forceinline__ int bin_of(float z, float zmax) {
    const float d = zmax - z;
    return d < 32.f ? max((int)(d * 128.f), 0) : kBins - 1;      // NaN and -inf land in the last bin
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
                                                                    const float* noise, int32_t* out, float* tau_out,
                                                                    const TruncRow* only_flagged) {
    __shared__ uint64_t hist[kWaves * 256];
    __shared__ Select sel;
    __shared__ uint64_t s_total;
    __shared__ float s_red[kWaves];
    __shared__ int s_idx[kWaves];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (only_flagged && !only_flagged[row].fallback) return;       // the multi-kernel path has done this row
    const float* lr = logits + (size_t)row * V;
    uint64_t* my_hist = hist + wave * 256;

    auto clear_hist = [&] {
        for (int i = tid; i < kWaves * 256; i += kThreads) hist[i] = 0;
        __syncthreads();
    };

    // ---- max of z (the softmax reference point)
    float zmax = -INFINITY;
    sweep<8>(lr, 0, V, tid, [&](float l, int) { zmax = fmaxf(zmax, l / temperature); });
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
            sweep<8>(lr, 0, V, tid, [&](float l, int) {
                const uint32_t key = order_key(l / temperature);
                if (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
                    atomicAdd((unsigned long long*)&my_hist[(key >> shift) & 255u], 1ull);
            });
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
            sweep<8>(lr, 0, V, tid, [&](float l, int) {
                const float z = l / temperature;
                const uint32_t key = order_key(z);
                if (key >= floor_key && (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))) {
                    const uint64_t mass = mass45(z, zmax);
                    atomicAdd((unsigned long long*)&my_hist[(key >> shift) & 255u], (unsigned long long)mass);
                }
            });
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
    sweep<8>(lr, 0, V, tid, [&](float l, int v) {
        const float z = l / temperature;
        if (order_key(z) < floor_key) return;
        const float sc = z + (nr ? nr[v] : gumbel_noise(key64, v));
        if (better(sc, v, bv, bi)) { bv = sc; bi = v; }
    });
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

// ---- the multi-workgroup path (needs a workspace) ---------------------------------------------------------------

// vocabulary range of slice blockIdx.x of gridDim.x
__device__ __forceinline__ void slice_range(int V, int& lo, int& hi) {
    const int per = (V + (int)gridDim.x - 1) / (int)gridDim.x;
    lo = (int)blockIdx.x * per;
    hi = min(V, lo + per);
}

__global__ __launch_bounds__(kThreads) void trunc_max_kernel(const float* logits, int V, float* lmax_part) {
    __shared__ float s_red[kWaves];
    const int row = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* lr = logits + (size_t)row * V;
    int lo, hi;
    slice_range(V, lo, hi);
    float m = -INFINITY;
    sweep<8>(lr, lo, hi, tid, [&](float l, int) { m = fmaxf(m, l); });
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w) m = fmaxf(m, s_red[w]);
        lmax_part[row * kMaxSlices + blockIdx.x] = m;
    }
}

// the row maximum of z: division by T > 0 is monotone, so max(l / T) = max(l) / T
__device__ __forceinline__ float row_zmax(const float* lmax_part, int row, int slices, float temperature) {
    float m = lmax_part[row * kMaxSlices];
    for (int i = 1; i < slices; ++i) m = fmaxf(m, lmax_part[row * kMaxSlices + i]);
    return m / temperature;
}

__global__ __launch_bounds__(kThreads) void trunc_hist_kernel(const float* logits, int V, float temperature, const float* lmax_part,
                                                              int want_mass, uint64_t* hist_mass, uint32_t* hist_cnt) {
    __shared__ uint64_t hm[kBins];
    __shared__ uint32_t hc[kBins];
    const int row = blockIdx.y, tid = threadIdx.x;
    const float* lr = logits + (size_t)row * V;
    for (int i = tid; i < kBins; i += kThreads) { hm[i] = 0; hc[i] = 0; }
    const float zmax = row_zmax(lmax_part, row, gridDim.x, temperature);
    __syncthreads();
    int lo, hi;
    slice_range(V, lo, hi);
    sweep<8>(lr, lo, hi, tid, [&](float l, int) {
        const float z = l / temperature;
        const int b = bin_of(z, zmax);
        atomicAdd(&hc[b], 1u);
        if (want_mass) {
            const uint64_t m = mass45(z, zmax);
            if (m) atomicAdd((unsigned long long*)&hm[b], (unsigned long long)m);
        }
    });
    __syncthreads();
    const size_t base = ((size_t)row * gridDim.x + blockIdx.x) * kBins;
    for (int i = tid; i < kBins; i += kThreads) { hist_mass[base + i] = hm[i]; hist_cnt[base + i] = hc[i]; }
}

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int d) {
    const uint32_t lo = __shfl_up((uint32_t)v, d, 64), hi = __shfl_up((uint32_t)(v >> 32), d, 64);
    return ((uint64_t)hi << 32) | lo;
}

// Prefix sums over the bins of a row (bin 0 = the largest z) and the bin in which the cut falls.
__global__ __launch_bounds__(kThreads) void trunc_plan_kernel(int V, float temperature, int top_k, float top_p, int slices,
                                                              const float* lmax_part, const uint64_t* hist_mass,
                                                              const uint32_t* hist_cnt, TruncRow* rows) {
    __shared__ uint64_t w_mass[kWaves];
    __shared__ uint32_t w_cnt[kWaves];
    __shared__ int s_found;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t bm[4];
    uint32_t bc[4];
    uint64_t tm = 0;
    uint32_t tc = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint64_t m = 0;
        uint32_t c = 0;
        for (int s = 0; s < slices; ++s) {
            const size_t at = ((size_t)row * slices + s) * kBins + tid * 4 + i;
            m += hist_mass[at];
            c += hist_cnt[at];
        }
        bm[i] = m; bc[i] = c;
        tm += m; tc += c;
    }
    // inclusive scan over the lanes of a wave, then over the waves
    uint64_t im = tm;
    uint32_t ic = tc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t om = shfl_up_u64(im, d);
        const uint32_t oc = __shfl_up(ic, d, 64);
        if (lane >= d) { im += om; ic += oc; }
    }
    if (lane == 63) { w_mass[wave] = im; w_cnt[wave] = ic; }
    if (tid == 0) s_found = 0;
    __syncthreads();
    uint64_t before_m = im - tm, total_m = 0;
    uint32_t before_c = ic - tc;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) { before_m += w_mass[w]; before_c += w_cnt[w]; }
        total_m += w_mass[w];
    }
    const bool by_count = top_k > 0 && top_k < V;
    const bool by_mass = top_p < 1.0f;
    uint64_t target = 0;
    if (!by_count) {
        target = (uint64_t)ceil((double)top_p * (double)total_m);
        if (target < 1) target = 1;
        if (target > total_m) target = total_m;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = tid * 4 + i;
        const bool here = by_count ? (before_c < (uint32_t)top_k && (uint32_t)top_k <= before_c + bc[i])
                                   : (before_m < target && target <= before_m + bm[i]);
        if (here) {                                          // exactly one bin of the row
            TruncRow r;
            r.zmax = row_zmax(lmax_part, row, slices, temperature);
            r.cand_hi = b;
            r.need_mass = 0;
            if (by_count && by_mass) {                       // top-p needs the mass of the top-k survivors: resolve both on the list
                r.cand_lo = 0;
                r.need_count = (uint32_t)top_k;
                r.n_cand = (int)(before_c + bc[i]);
            } else {
                r.cand_lo = b;
                r.need_count = by_count ? (uint32_t)top_k - before_c : 0u;
                r.need_mass = by_count ? 0ull : target - before_m;
                r.n_cand = (int)bc[i];
            }
            r.fallback = r.n_cand > kCap ? 1 : 0;
            rows[row] = r;
            s_found = 1;
        }
        before_m += bm[i];
        before_c += bc[i];
    }
    __syncthreads();
    if (tid == 0 && !s_found) {                              // no bin qualifies (a row of NaN): the single kernel's business
        TruncRow r = {};
        r.fallback = 1;
        rows[row] = r;
    }
}

// One sweep: tokens above the candidate bins compete for the Gumbel-max right away, tokens in them are listed.
__global__ __launch_bounds__(kThreads) void trunc_select_kernel(const float* logits, int V, float temperature, const TruncRow* rows,
                                                                int use_noise_buffer, KeyChunk keys, const float* noise,
                                                                uint2* cand, int* cand_n, float2* part) {
    __shared__ int s_n;
    __shared__ float s_red[kWaves];
    __shared__ int s_idx[kWaves];
    const int row = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TruncRow r = rows[row];
    if (r.fallback) return;
    const float* lr = logits + (size_t)row * V;
    const float* nr = use_noise_buffer ? noise + (size_t)row * V : nullptr;
    const uint64_t key64 = keys.key[row];
    const size_t seg = (size_t)row * gridDim.x + blockIdx.x;
    uint2* my_cand = cand + seg * kCap;
    if (tid == 0) s_n = 0;
    __syncthreads();
    int lo, hi;
    slice_range(V, lo, hi);
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    sweep<8>(lr, lo, hi, tid, [&](float l, int v) {
        const float z = l / temperature;
        const int b = bin_of(z, r.zmax);
        if (b < r.cand_lo) {
            const float sc = z + (nr ? nr[v] : gumbel_noise(key64, v));
            if (better(sc, v, bv, bi)) { bv = sc; bi = v; }
        } else if (b <= r.cand_hi) {
            const int slot = atomicAdd(&s_n, 1);
            if (slot < kCap) my_cand[slot] = make_uint2(order_key(z), (uint32_t)v);
        }
    });
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { s_red[wave] = bv; s_idx[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w)
            if (better(s_red[w], s_idx[w], bv, bi)) { bv = s_red[w]; bi = s_idx[w]; }
        part[seg] = make_float2(bv, __int_as_float(bi));
        cand_n[seg] = min(s_n, kCap);
    }
}

// The radix descent of the single-kernel path on the candidate list (in LDS), then the Gumbel-max over the kept
// candidates and the slices' winners among the tokens above the cut bin.
__global__ __launch_bounds__(kThreads) void trunc_resolve_kernel(int V, int top_k, float top_p, int slices, const TruncRow* rows,
                                                                 int use_noise_buffer, KeyChunk keys, const float* noise,
                                                                 const uint2* cand, const int* cand_n, const float2* part,
                                                                 int32_t* out, float* tau_out) {
    extern __shared__ uint4 lds_raw[];
    uint2* list = (uint2*)lds_raw;                            // [kCap]
    uint64_t* hist = (uint64_t*)(list + kCap);                // [kWaves][256]
    __shared__ Select sel;
    __shared__ float s_red[kWaves];
    __shared__ int s_idx[kWaves];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TruncRow r = rows[row];
    if (r.fallback) return;
    uint64_t* my_hist = hist + wave * 256;

    int n = 0;
    for (int s = 0; s < slices; ++s) {
        const size_t seg = (size_t)row * slices + s;
        const int m = min(cand_n[seg], kCap - n);
        for (int i = tid; i < m; i += kThreads) list[n + i] = cand[seg * kCap + i];
        n += m;
    }
    __syncthreads();

    auto clear_hist = [&] {
        for (int i = tid; i < kWaves * 256; i += kThreads) hist[i] = 0;
        __syncthreads();
    };
    const bool by_count = top_k > 0 && top_k < V;
    const bool by_mass = top_p < 1.0f;
    uint32_t floor_key = 0;

    if (by_count) {
        if (tid == 0) { sel.prefix = 0; sel.remaining = (uint64_t)r.need_count; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            clear_hist();
            const uint32_t prefix = sel.prefix;
            for (int i = tid; i < n; i += kThreads) {
                const uint32_t key = list[i].x;
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
    if (by_mass) {
        if (tid == 0) { sel.prefix = 0; sel.remaining = r.need_mass; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            clear_hist();
            const uint32_t prefix = sel.prefix;
            for (int i = tid; i < n; i += kThreads) {
                const uint32_t key = list[i].x;
                if (key >= floor_key && (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))) {
                    const uint64_t mass = mass45(key_value(key), r.zmax);
                    atomicAdd((unsigned long long*)&my_hist[(key >> shift) & 255u], (unsigned long long)mass);
                }
            }
            __syncthreads();
            if (pass == 0) {
                // with top-k in front the target is a share of the survivors' mass, known only now; alone it came with
                // the row (and cannot exceed the list's mass: the same integers were summed for the histogram)
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
                        uint64_t target = by_count ? (uint64_t)ceil((double)top_p * (double)Z) : sel.remaining;
                        if (target < 1) target = 1;
                        if (target > Z) target = Z;
                        sel.remaining = target;
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

    const float* nr = use_noise_buffer ? noise + (size_t)row * V : nullptr;
    const uint64_t key64 = keys.key[row];
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int i = tid; i < n; i += kThreads) {
        const uint2 e = list[i];
        if (e.x < floor_key) continue;
        const int v = (int)e.y;
        const float sc = key_value(e.x) + (nr ? nr[v] : gumbel_noise(key64, v));
        if (better(sc, v, bv, bi)) { bv = sc; bi = v; }
    }
    if (tid < slices) {
        const float2 e = part[(size_t)row * slices + tid];
        const int i = __float_as_int(e.y);
        if (better(e.x, i, bv, bi)) { bv = e.x; bi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { s_red[wave] = bv; s_idx[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w)
            if (better(s_red[w], s_idx[w], bv, bi)) { bv = s_red[w]; bi = s_idx[w]; }
        out[row] = bi == 0x7FFFFFFF ? 0 : bi;
        if (tau_out) tau_out[row] = floor_key == 0 ? -INFINITY : key_value(floor_key);
    }
}

namespace {
// workgroups per row: enough to put a workgroup on every compute unit, slices of at least 8192 tokens
int trunc_slices(int rows, int V) {
    int s = (256 + rows - 1) / rows;
    s = std::min(s, kMaxSlices);
    s = std::min(s, std::max(1, V / 8192));
    return std::max(s, 1);
}
struct TruncLayout { size_t lmax, hist_mass, hist_cnt, rows, cand, cand_n, part, total; };
TruncLayout trunc_layout(int rows, int slices) {
    TruncLayout L;
    size_t at = 0;
    auto take = [&](size_t bytes) { const size_t o = at; at += (bytes + 255) & ~(size_t)255; return o; };
    L.lmax = take((size_t)rows * kMaxSlices * sizeof(float));
    L.hist_mass = take((size_t)rows * slices * kBins * sizeof(uint64_t));
    L.hist_cnt = take((size_t)rows * slices * kBins * sizeof(uint32_t));
    L.rows = take((size_t)rows * sizeof(TruncRow));
    L.cand = take((size_t)rows * slices * kCap * sizeof(uint2));
    L.cand_n = take((size_t)rows * slices * sizeof(int));
    L.part = take((size_t)rows * slices * sizeof(float2));
    L.total = at;
    return L;
}
}  // namespace

// rows of a batch are processed 128 at a time (the row keys travel by value), one chunk after the other on the stream
size_t sample_truncated_workspace_bytes(int B, int V) {
    const int rows = std::min(B, 128);
    return trunc_layout(rows, trunc_slices(rows, V)).total;
}

hipError_t launch_sample_truncated_ws(const float* logits, int B, int V, float temperature, int top_k, float top_p,
                                      const uint64_t* host_keys, const float* noise, int32_t* out, float* tau_out,
                                      void* workspace, hipStream_t s) {
    const int rows_max = std::min(B, 128);
    const int slices = trunc_slices(rows_max, V);
    const TruncLayout L = trunc_layout(rows_max, slices);
    char* ws = (char*)workspace;
    float* lmax = (float*)(ws + L.lmax);
    uint64_t* hist_mass = (uint64_t*)(ws + L.hist_mass);
    uint32_t* hist_cnt = (uint32_t*)(ws + L.hist_cnt);
    TruncRow* rows = (TruncRow*)(ws + L.rows);
    uint2* cand = (uint2*)(ws + L.cand);
    int* cand_n = (int*)(ws + L.cand_n);
    float2* part = (float2*)(ws + L.part);
    const size_t resolve_lds = (size_t)kCap * sizeof(uint2) + (size_t)kWaves * 256 * sizeof(uint64_t);
    hipError_t e0 = hipFuncSetAttribute((const void*)trunc_resolve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)resolve_lds);
    if (e0 != hipSuccess) return e0;
    for (int off = 0; off < B; off += 128) {
        KeyChunk k;
        const int m = B - off < 128 ? B - off : 128;
        for (int i = 0; i < m; ++i) k.key[i] = host_keys ? host_keys[off + i] : 0;
        const float* lg = logits + (size_t)off * V;
        const float* nz = noise ? noise + (size_t)off * V : nullptr;
        hipLaunchKernelGGL(trunc_max_kernel, dim3(slices, m), dim3(kThreads), 0, s, lg, V, lmax);
        hipLaunchKernelGGL(trunc_hist_kernel, dim3(slices, m), dim3(kThreads), 0, s, lg, V, temperature, lmax,
                           top_p < 1.0f ? 1 : 0, hist_mass, hist_cnt);
        hipLaunchKernelGGL(trunc_plan_kernel, dim3(m), dim3(kThreads), 0, s, V, temperature, top_k, top_p, slices, lmax,
                           hist_mass, hist_cnt, rows);
        hipLaunchKernelGGL(trunc_select_kernel, dim3(slices, m), dim3(kThreads), 0, s, lg, V, temperature, rows, noise ? 1 : 0, k,
                           nz, cand, cand_n, part);
        hipLaunchKernelGGL(trunc_resolve_kernel, dim3(m), dim3(kThreads), resolve_lds, s, V, top_k, top_p, slices, rows,
                           noise ? 1 : 0, k, nz, cand, cand_n, part, out + off, tau_out ? tau_out + off : nullptr);
        // rows with too many candidates for the list (flagged by the plan kernel): the single-kernel path, others return at once
        hipLaunchKernelGGL(sample_truncated_kernel, dim3(m), dim3(kThreads), 0, s, lg, V, temperature, top_k, top_p, noise ? 1 : 0,
                           k, nz, out + off, tau_out ? tau_out + off : nullptr, (const TruncRow*)rows);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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
                           tau_out ? tau_out + off : nullptr, (const TruncRow*)nullptr);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace spiral
