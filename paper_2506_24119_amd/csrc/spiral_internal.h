// Internal declarations shared by the host API and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "spiral.h"

// host-side hooks shared by the library's translation units (defined with the C ABI's host code)
int spiral_set_error(int code, const char* text);
int spiral_decode_workspace_need(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B, const char* who,
                                 size_t* need);
int spiral_decode_on_workspace(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B, const int32_t* dev_in_tokens,
                               void* dev_ws, size_t ws_bytes, float* dev_logits, void* stream, const char* who);

namespace spiral {

// ---------------------------------------------------------------------------------------------
// Activation storage between kernels.
//   fp32-weight models: fp32 activations, plain FMA GEMMs.
//   bf16-weight models: IEEE-half activations feeding the f16 MFMAs; the bf16 weights are widened to half
//   (exact for every bf16 value whose magnitude is in half's normal range).  bf16 activations (8 significant
//   bits) fail the logit tolerance at 36 layers, so there is no such variant.
// ---------------------------------------------------------------------------------------------
constexpr int kPageTokens = 16;
constexpr int kMaxGroup = 16;          // q heads per kv head handled by one attention tile
constexpr int kUploadInts = 768;       // ints carried by value in one upload launch (3 KB of kernel arguments)

struct IntChunk { int32_t v[kUploadInts]; };
struct PairChunk { int32_t idx[kUploadInts / 2]; int32_t val[kUploadInts / 2]; };
struct KeyChunk { uint64_t key[128]; };
struct RopeFreq { double inv_freq[64]; };   // theta^(-2j/hd), j < hd/2 <= 64

// GEMM: out[m][n] = sum_k A[m][k] * W[n][k]; W is up to three row blocks stacked along n
// (q|k|v) or, for the SwiGLU epilogue, the gate and up matrices addressed by the same row.
// EPI_SAMPLE (LM head only): no logits are written; every workgroup reduces its 128 vocabulary columns to the
// best (score, index) per batch row, score = logit / T + Gumbel noise (or the logit itself when greedy).
enum GemmEpilogue { EPI_STORE_F32 = 0, EPI_SWIGLU = 1, EPI_SAMPLE = 2 };

struct GemmArgs {
    const void* A;        // activations [M][K] (act type)
    const void* w[3];     // weight row blocks, [rows][K]
    const void* wf;       // or null: the same rows (SwiGLU: gate/up interleaved 16 + 16) in fragment order, see frag_block()
    int32_t rows[3];      // rows in each block
    int32_t M, N, K;      // N = total output columns (SwiGLU: ffn width)
    void* out;            // STORE_F32: fp32 [splits][M][N]; SWIGLU: act [M][N]
    int32_t splits;       // grid split of K (STORE_F32 only)
    int32_t m_tiles;      // ceil(M / rows per tile)
    // EPI_SAMPLE: per-row generator keys (device), temperature (0: greedy), partial winners [M][s_tiles] (score, index bits)
    const uint64_t* s_keys;
    float2* s_part;
    float s_temperature;
    int32_t s_tiles;
    int32_t* sat_count;   // or null: incremented when an activation left the half-precision range (SwiGLU output)
};

struct AttnArgs {
    const uint16_t* q;        // bf16 [rows][Hq][hd]
    const uint16_t* pages;    // this layer's pages: [page][Hkv]{K[16][hd], V[hd][16]}
    const int32_t* block_table;   // [max_seqs][max_blocks]
    const int32_t* row_seq;   // [rows]
    const int32_t* row_pos;   // [rows] position of the row's token
    const int32_t* cu_rows;   // prefill: [B+1] first row of each sequence; decode: unused
    const int32_t* row_page_start;   // decode stream: [rows + 1] prefix sum of the rows' page counts
    float* part;              // decode: [rows][Hkv][chunks][G][hd + 2]
    void* out;                // act [rows][Hq*hd]
    int32_t n_rows, n_q_heads, n_kv_heads, max_blocks, chunk_pages, n_chunks;
    int32_t units_per_wg, total_units;   // decode stream: (row, kv head, page) units per workgroup, and in all
    float scale_log2e;        // log2(e) / sqrt(hd)
};

// Launchers (defined in the kernel translation units).  All enqueue on `s` and return the launch status.
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_upload(int32_t* dev_dst, const int32_t* host_src, int n, hipStream_t s);
hipError_t launch_upload_multi(int32_t* const* dev_dst, const int32_t* const* host_src, const int* n, int n_seg, hipStream_t s);
hipError_t launch_scatter(int32_t* dev_base, const int32_t* host_idx, const int32_t* host_val, int n, hipStream_t s);
hipError_t launch_prefill_meta(const int32_t* cu_rows, const int32_t* base_pos, const int32_t* seq_ids, int B,
                               int n_rows, int32_t* row_seq, int32_t* row_pos, hipStream_t s);

struct EmbedArgs {
    const int32_t* tokens;    // [rows]
    const void* embed;        // [vocab][d]
    const float* gain;        // [d]
    float* x;                 // [rows][d]
    void* h;                  // act [rows][d]
    const int32_t* row_pos;   // [rows] position of each row's token
    float2* rope;             // [rows][hd/2] (cos, sin), written
    int32_t n_rows, d, half_hd, vocab;
    float eps;
    // the page that takes each row's k and v, looked up here once for all layers: row_page[r] = (page, position)
    const int32_t* row_seq; const int32_t* block_table; int32_t max_blocks;
    int2* row_page;           // [rows], written
};
hipError_t launch_embed_norm(const EmbedArgs& a, const RopeFreq& f, bool w_bf16, bool act32, hipStream_t s);

struct NormArgs {
    float* x;                 // [rows_in][d] residual, updated in place when n_part > 0
    const float* part;        // [n_part][rows_in][d] projections to add, or null
    const float* gain;        // [d]
    void* h;                  // act [rows_out][d]
    const int32_t* row_map;   // null, or [rows_out] source row of each output row
    int32_t rows_in, rows_out, d, n_part;
    float eps;
    int32_t* sat_count;       // or null
};
hipError_t launch_add_norm(const NormArgs& a, bool act32, hipStream_t s);

struct QkvPostArgs {
    const float* qkv;         // [n_part][rows][(Hq+2Hkv)*hd]
    const void* bq; const void* bk; const void* bv;   // weight dtype, or null
    const float* q_gain; const float* k_gain;         // [hd] or null
    const float2* rope;       // [rows][hd/2]
    const int2* row_page;     // [rows] (physical page, position) of the row's token, from embed_norm_kernel
    uint16_t* q;              // half [rows][Hq][hd]
    uint16_t* pages;          // this layer's pages
    int32_t n_rows, n_part, n_q_heads, n_kv_heads, hd;
    float eps;
    int32_t* sat_count;       // or null
};
hipError_t launch_qkv_post(const QkvPostArgs& a, bool w_bf16, hipStream_t s);

hipError_t launch_gemm(const GemmArgs& a, int epilogue, bool w_bf16, int bn, hipStream_t s);
bool gemm_tile_usable(const GemmArgs& a);                                                  // fragment-ordered weights, K % 64 == 0, ...
hipError_t launch_gemm_tile(const GemmArgs& a, int epilogue, hipStream_t s);
bool gemm_tile_qkv_usable(const GemmArgs& a, const QkvPostArgs& qa, bool w_bf16);          // ... and head_dim 128, whole heads per tile
hipError_t launch_gemm_tile_qkv(const GemmArgs& a, const QkvPostArgs& qa, hipStream_t s);  // q/k/v projection + qkv_post in one kernel
hipError_t launch_gemm_stream(const GemmArgs& a, int epilogue, int bn, hipStream_t s);   // K % 128 == 0, N % 16 == 0
hipError_t launch_attn_stream(const AttnArgs& a, int hd, bool act32, hipStream_t s);
hipError_t launch_attn_stream_combine(const AttnArgs& a, int hd, bool act32, hipStream_t s);
hipError_t launch_attn_prefill(const AttnArgs& a, int hd, int B, int max_new, bool act32, hipStream_t s);

hipError_t launch_stream_read(const void* p, size_t bytes, int workgroups, hipStream_t s);
hipError_t launch_sample_pick(const float2* part, int B, int n_tiles, int32_t* out, hipStream_t s);
int gemm_sample_tile_cols(int M, int bn);     // LM-head columns per workgroup of the sampling epilogue
hipError_t launch_sample(const float* logits, int B, int V, float temperature, const uint64_t* host_keys,
                         const float* noise, int32_t* out, hipStream_t s);
// Fragment order of a 16-bit weight matrix [N][K] (N padded to a multiple of 32, K % 16 == 0): 1 KB blocks
// (32 rows x 16 k), block (t, ks) at element offset (t * (K / 16) + ks) * 512; inside a block lane
// l = (k % 16 / 8) * 32 + row % 32 holds 8 consecutive k: exactly the operand registers of one
// v_mfma_f32_32x32x16 step, so a wave's load instruction reads one contiguous block (8 cache lines
// instead of 32 half-used ones).
__host__ __device__ inline size_t frag_block(int t, int ks, int K) { return ((size_t)t * (K >> 4) + ks) * 512; }
hipError_t launch_repack(const void* src0, const void* src1, const void* src2, int rows0, int rows1, int rows2, int K,
                         bool interleave16, void* dst, hipStream_t s);

// scoring: per-row log-probability of a target token under the LM head's softmax
struct ScoreArgs {
    const void* A;            // act [M][K]: final-normed hidden states
    const void* W;            // bf16 [V][K] LM head
    const void* Wf;           // or null: the LM head in fragment order
    const int32_t* targets;   // [M] target token of each row, < 0: none
    float* part;              // [M][n_splits] (max, sum exp) pairs
    float* tgt_logit;         // [M]
    int32_t M, V, K, n_splits, tiles_per_split, m_tiles;
};
hipError_t launch_score(const ScoreArgs& a, float* out, hipStream_t s);
hipError_t launch_score_objective(const float* logp_new, const float* logp_old, const float* adv, const int32_t* mask,
                                  long long n, float eps, double* out, hipStream_t s);
hipError_t launch_sample_truncated(const float* logits, int B, int V, float temperature, int top_k, float top_p,
                                   const uint64_t* host_keys, const float* noise, int32_t* out, float* tau_out,
                                   hipStream_t s);
// the same thresholds and draw by several workgroups per row and three sweeps; `workspace` holds
// sample_truncated_workspace_bytes(B, V) bytes
size_t sample_truncated_workspace_bytes(int B, int V);
hipError_t launch_sample_truncated_ws(const float* logits, int B, int V, float temperature, int top_k, float top_p,
                                      const uint64_t* host_keys, const float* noise, int32_t* out, float* tau_out,
                                      void* workspace, hipStream_t s);

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {       // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// round to nearest even; finite values beyond the half range saturate at +-65504, NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
    const float c = fminf(fmaxf(f, -65504.0f), 65504.0f);      // fmin/fmax drop a NaN operand: put it back
    _Float16 h = (_Float16)(f != f ? f : c);
    return __builtin_bit_cast(uint16_t, h);
}
// true when f32_to_f16_bits(f) is not a rounding of f: saturated, infinite or NaN
__device__ __forceinline__ bool f16_out_of_range(float f) { return !(fabsf(f) <= 65504.0f); }

__device__ __forceinline__ uint16_t f32_to_act16(float f) {
    return f32_to_f16_bits(f);
}

// conversion that also notes a value the 16-bit format cannot hold (callers report it through the pool's counter)
__device__ __forceinline__ uint16_t f32_to_act16_noting(float f, bool& bad) {
    bad = bad || f16_out_of_range(f);
    return f32_to_act16(f);
}
// one increment per lane that saw an unrepresentable value (rare: the branch is normally not taken)
__device__ __forceinline__ void report_saturation(int32_t* counter, bool bad) {
    if (counter && bad) atomicAdd(counter, 1);
}

template <bool ACT32> struct ActStore;
template <> struct ActStore<true> {
    typedef float type;
    static __device__ __forceinline__ void put(void* base, size_t i, float v) { ((float*)base)[i] = v; }
    static __device__ __forceinline__ void put_noting(void* base, size_t i, float v, bool&) { ((float*)base)[i] = v; }
};
template <> struct ActStore<false> {
    typedef uint16_t type;
    static __device__ __forceinline__ void put(void* base, size_t i, float v) { ((uint16_t*)base)[i] = f32_to_act16(v); }
    static __device__ __forceinline__ void put_noting(void* base, size_t i, float v, bool& bad) {
        ((uint16_t*)base)[i] = f32_to_act16_noting(v, bad);
    }
};

// ---- the sampler's counter generator (same stream in every kernel that draws noise)
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// standard Gumbel noise of vocabulary entry v under a row key: u = ((r >> 9) + 0.5) * 2^-23, g = -ln(-ln u)
__device__ __forceinline__ float gumbel_noise(uint64_t key, int v) {
    const uint32_t r = (uint32_t)(mix64(key + (uint64_t)v * 0x9E3779B97F4A7C15ull) >> 32);
    const float u = ((float)(r >> 9) + 0.5f) * 1.1920928955078125e-07f;   // 2^-23
    return -logf(-logf(u));
}
// argmax order: larger score wins, equal scores go to the lower index
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace spiral
