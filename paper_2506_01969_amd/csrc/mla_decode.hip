// MLA decode attention for gfx950 (MI355X): split-KV main kernel + LSE combine kernel + C ABI.
//
// Problem (paper Section 3.1, decoding setup of Section 4.1): for every sequence b and each of
// 16 heads, one query row of 576 bf16 attends over N_b latent KV rows of 576 bf16 shared by all
// heads; V is the first 512 columns of the same row.  out = softmax(scale * q K^T) V, plus the
// log-sum-exp of the scaled scores (the L of Algorithm 1's last step).
//
// Orientation.  Both contractions run in the transposed form of equations (1)-(4):
//     S^T = K Q^T   (tokens on the MFMA M axis, heads on N, contraction over the 576 dims)
//     O^T = V^T P^T (value columns on M, heads on N, contraction over tokens)
// On gfx950 the reason is not padding (a 16-row MFMA shape exists) but register layout: the
// 16x16 result of S^T leaves every lane holding ONE head (column) and four consecutive tokens
// (rows), which is exactly the B-operand layout the second product wants for P^T, and the
// per-head softmax statistics and the per-head rescale factor of Algorithm 1 become per-lane
// scalars.  The transpose of equation (4) is folded into the addressing of the final store.
//
// Work decomposition.  One workgroup (4 wavefronts) per (sequence, KV chunk).  Each wavefront is
// an independent online-softmax worker (the m / l / rescale recurrence of Algorithm 1) over
// every 4th 32-token tile of the chunk, with a private LDS tile, so the main loop has no
// barrier.  A tile is fetched with 16-byte coalesced global loads into registers (in flight
// while the previous tile is being computed), written once to LDS, and read twice from LDS: as
// the K operand (ds_read_b128) and, through the transposing LDS read ds_read_b64_tr_b16, as the
// V^T operand.  The four wavefronts merge their (m, l, O) through LDS at the end of the chunk;
// chunks are merged by the combine kernel.
//
// P is fed to the second MFMA as a two-term bf16 split (hi + lo): a single bf16 rounding of P
// costs ~2^-9 relative error per term, which is outside the 1e-4 RMSE bound at short KV.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

#include "mla_decode.h"

namespace {

constexpr int kHeads = MLA_NUM_HEADS;        // 16
constexpr int kDqk = MLA_D_QK;               // 576
constexpr int kDv = MLA_D_V;                 // 512
constexpr int kRowBytes = kDqk * 2;          // 1152 bytes per KV row
constexpr int kLdsRow = kRowBytes + 16;      // LDS row stride: +16 B so 16 rows hit 64 distinct banks
constexpr int kTile = 32;                    // tokens per wavefront step (MFMA K of the PV product)
constexpr int kWaves = 4;                    // wavefronts per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kWaveLds = kTile * kLdsRow;    // 37,376 B private tile per wavefront
constexpr int kKSteps = kDqk / 32;           // 18 MFMA k-steps over the 576 dims
constexpr int kDvTiles = kDv / 16;           // 32 output tiles of 16 value columns
constexpr int kStatsOff = kWaves * kWaveLds; // m and l of the 4 wavefronts live after the tiles
constexpr int kRescaleOff = kStatsOff + 2 * kWaves * kHeads * 4;  // 2 KB per wavefront, cold rescale path
constexpr int kLdsBytes = kRescaleOff + kWaves * 2048;
constexpr int kChunkGranule = kWaves * kTile;  // 128: chunk lengths are multiples of this
static_assert(kChunkGranule == MLA_CHUNK_GRANULE, "header and kernel disagree on the chunk granule");
constexpr int kCombineThreads = 128;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

struct Params {
    const char *q;            // bf16 [batch][16][576]
    const char *kv;           // bf16 rows of 576
    long long kv_batch_bytes; // bytes between sequences
    const int *seqlens;       // [batch]
    float *out;               // [batch][16][512]
    float *lse;               // [batch][16]
    float *part_out;          // [batch][splits_max][16][512]
    float *part_lse;          // [batch][splits_max][16], base-2 log-sum-exp of scale*log2(e)*q.k
    int max_seqlen;
    int chunk_len;
    int splits_max;
    float scale_log2e;        // scale * log2(e): scores are kept in the base-2 domain
};

__device__ __forceinline__ u32x4 load_stream16(const char *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ float wave_xor_max(float v, int mask) {
    return fmaxf(v, __shfl_xor(v, mask, 64));
}

constexpr float kLazyLog2 = 8.0f;   // the softmax reference moves only when exceeded by 2^8

// O <- O * alpha with O resident in accumulation registers (AGPRs), which the vector ALU cannot
// address.  Each 16x16 tile takes a round trip through a small private LDS slot (AGPR -> LDS ->
// VGPR, multiply, and the result is copied back), so the accumulators' own live range has no
// VALU use and the register allocator leaves them in place on the hot path.  This path is cold
// (see kLazyLog2).
__device__ __forceinline__ void rescale_accumulators(f32x4 (&o)[kDvTiles], float alpha, char *slot) {
#pragma unroll
    for (int c = 0; c < kDvTiles; c += 2) {
        *reinterpret_cast<volatile f32x4 *>(slot) = o[c];
        *reinterpret_cast<volatile f32x4 *>(slot + 1024) = o[c + 1];
        f32x4 t0 = *reinterpret_cast<volatile f32x4 *>(slot);
        f32x4 t1 = *reinterpret_cast<volatile f32x4 *>(slot + 1024);
        o[c] = t0 * alpha;
        o[c + 1] = t1 * alpha;
    }
}

// Main kernel: one workgroup per (sequence, chunk); steps a1-a7 of the hot path.
__global__ void __launch_bounds__(kThreads, 1) mla_decode_split_kernel(const Params p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront in workgroup (scalar)
    const int l = tid & 63;       // lane
    const int r16 = l & 15;       // MFMA row/column index owned by this lane
    const int g = l >> 4;         // MFMA k-group (0..3)

    const int b = blockIdx.x / p.splits_max;
    const int s = blockIdx.x - b * p.splits_max;
    int n = p.seqlens[b];
    n = n < 0 ? 0 : (n > p.max_seqlen ? p.max_seqlen : n);
    const int t_begin = s * p.chunk_len;
    if (t_begin >= n) return;     // chunk past the end of this sequence (uniform over the workgroup)
    const int t_end = min(n, t_begin + p.chunk_len);
    const int num_splits = (n + p.chunk_len - 1) / p.chunk_len;
    const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;
    const char *kv_b = p.kv + (long long)b * p.kv_batch_bytes;

    // Q^T as the MFMA B operand: lane (head r16, k-group g) holds dims 32*kk + 8*g .. +8.
    bf16x8 qf[kKSteps];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + ((long long)b * kHeads + r16) * kRowBytes) + g;
#pragma unroll
        for (int kk = 0; kk < kKSteps; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, qp[4 * kk]);
    }

    char *my = smem + w * kWaveLds;                       // private tile of this wavefront
    // LDS addresses (bytes) of the three access patterns
    char *wr_main = my + l * 16;                          // row i, 16-byte chunk l            (+ i*kLdsRow)
    char *wr_rest = my + (l >> 3) * kLdsRow + 1024 + (l & 7) * 16;  // rows 8j + l/8, chunk 64 + l%8 (+ j*8*kLdsRow)
    const char *rd_k = my + r16 * kLdsRow + g * 16;       // K operand: token r16 (+16), chunk 4*kk + g
    // V^T operand through the transposing read: within each 16-lane group, lane j points at
    // row j/4, columns 4*(j%4)..+3 of a 4x16 block and receives column j, rows 0..3.
    const char *rd_v = my + (4 * g + (r16 >> 2)) * kLdsRow + (r16 & 3) * 8;

    f32x4 o[kDvTiles];
#pragma unroll
    for (int ct = 0; ct < kDvTiles; ++ct) o[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;      // running maximum of this lane's head (base-2 domain)
    float l_run = 0.f;            // this lane's share of the running sum

    u32x4 st[kTile + 4];          // one tile in flight: 36 x 16 B per lane

    // Rows past the end of the sequence are never fetched: their addresses are clamped to the
    // last valid row (their scores are masked below, so the duplicate has weight zero).
    auto issue_loads = [&](int tile) {
        const int tb = t_begin + tile * kTile;
#pragma unroll
        for (int i = 0; i < kTile; ++i) {
            const int row = min(tb + i, n - 1);
            st[i] = load_stream16(kv_b + (long long)row * kRowBytes + l * 16);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = min(tb + 8 * j + (l >> 3), n - 1);
            st[kTile + j] = load_stream16(kv_b + (long long)row * kRowBytes + 1024 + (l & 7) * 16);
        }
    };

    if (w < n_tiles) issue_loads(w);

    for (int tile = w; tile < n_tiles; tile += kWaves) {
        const int tb = t_begin + tile * kTile;

        // ---- a2: registers -> private LDS tile --------------------------------------------
#pragma unroll
        for (int i = 0; i < kTile; ++i) *reinterpret_cast<u32x4 *>(wr_main + i * kLdsRow) = st[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(wr_rest + j * 8 * kLdsRow) = st[kTile + j];

        // next tile of this wavefront goes in flight now and lands while this one is computed
        if (tile + kWaves < n_tiles) issue_loads(tile + kWaves);

        // ---- a3: S^T = K Q^T for tokens 0..15 and 16..31 of the tile (equation (1)) ------
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < kKSteps; ++kk) {
            const bf16x8 k0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(rd_k + kk * 64));
            const bf16x8 k1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(rd_k + 16 * kLdsRow + kk * 64));
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[kk], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[kk], s1, 0, 0, 0);
        }
        // this lane now holds, for head r16, tokens tb + 4g + i (s0[i]) and tb + 16 + 4g + i (s1[i])

        // ---- a4: scale (base-2 domain) and mask the tail ----------------------------------
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = (tb + 4 * g + i < t_end) ? s0[i] * p.scale_log2e : -INFINITY;
            x[4 + i] = (tb + 16 + 4 * g + i < t_end) ? s1[i] * p.scale_log2e : -INFINITY;
        }

        // ---- a5: online softmax (Algorithm 1: m, l update) ---------------------------------
        // The reference maximum m_run moves lazily: exponentials are taken against the current
        // reference and O, l are rescaled by exp(m_old - m_new) (the R of Algorithm 1) only when
        // some head's tile maximum exceeds its reference by more than kLazyLog2 (so p <= 2^8).
        // Any reference gives the same O / l and m + log l; moving it rarely keeps the 128
        // accumulator registers out of the vector ALU on almost every tile.
        float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        mx = wave_xor_max(mx, 16);
        mx = wave_xor_max(mx, 32);                       // finite: every tile has >= 1 valid token
        if (tile == w) {
            m_run = mx;                                  // first tile: O = 0 and l = 0, nothing to rescale
        } else if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazyLog2) != 0) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            rescale_accumulators(o, alpha, smem + kRescaleOff + w * 2048 + l * 16);
            l_run *= alpha;
            m_run = m_new;
        }
        float pr[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pr[i] = __builtin_amdgcn_exp2f(x[i] - m_run);
            l_run += pr[i];
        }

        // P^T as B operand, two-term bf16 split
        bf16x8 p_hi, p_lo;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p_hi[i] = (__bf16)pr[i];
            p_lo[i] = (__bf16)(pr[i] - (float)p_hi[i]);
        }

        // ---- a6: O^T += V^T P^T (equation (3)), V^T from the same LDS tile ------------------
#pragma unroll
        for (int ct = 0; ct < kDvTiles; ++ct) {
            const i16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) i16x4 *)(lds_char *)(rd_v + ct * 32));
            const i16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) i16x4 *)(lds_char *)(rd_v + 16 * kLdsRow + ct * 32));
            const i16x4 vv[2] = {v0, v1};
            bf16x8 vt;
            __builtin_memcpy(&vt, vv, 16);
            o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, p_hi, o[ct], 0, 0, 0);
            o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, p_lo, o[ct], 0, 0, 0);
        }
    }

    // ---- a7: merge the four wavefronts, normalise, write (the epilogue of Algorithm 1) --------
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    float *stat_m = reinterpret_cast<float *>(smem + kStatsOff);
    float *stat_l = stat_m + kWaves * kHeads;
    if (g == 0) {
        stat_m[w * kHeads + r16] = m_run;
        stat_l[w * kHeads + r16] = l_run;
    }
    // own accumulators into the own (now idle) tile: [ct][lane] x 16 B
#pragma unroll
    for (int ct = 0; ct < kDvTiles; ++ct) *reinterpret_cast<f32x4 *>(my + ct * 1024 + l * 16) = o[ct];
    __syncthreads();

    float m_tot = stat_m[r16];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) m_tot = fmaxf(m_tot, stat_m[ww * kHeads + r16]);
    float f[kWaves];
    float l_tot = 0.f;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) {
        f[ww] = __builtin_amdgcn_exp2f(stat_m[ww * kHeads + r16] - m_tot);   // 0 for an idle wavefront
        l_tot += f[ww] * stat_l[ww * kHeads + r16];
    }
    const float inv_l = 1.0f / l_tot;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) f[ww] *= inv_l;

    const bool direct = (num_splits == 1);
    float *dst = direct ? p.out + ((long long)b * kHeads + r16) * kDv
                        : p.part_out + (((long long)b * p.splits_max + s) * kHeads + r16) * kDv;
    // wavefront w finishes value tiles 8w .. 8w+7; lane holds head r16, columns 16ct + 4g .. +3
#pragma unroll
    for (int c = 0; c < kDvTiles / kWaves; ++c) {
        const int ct = w * (kDvTiles / kWaves) + c;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            const f32x4 part = *reinterpret_cast<const f32x4 *>(smem + ww * kWaveLds + ct * 1024 + l * 16);
            acc += part * f[ww];
        }
        *reinterpret_cast<f32x4 *>(dst + ct * 16 + g * 4) = acc;   // equation (4): transpose by addressing
    }
    if (w == 0 && g == 0) {
        const float lse2 = m_tot + __builtin_amdgcn_logf(l_tot);   // v_log_f32 is log2
        if (direct) p.lse[b * kHeads + r16] = lse2 * 0.6931471805599453f;
        else p.part_lse[((long long)b * p.splits_max + s) * kHeads + r16] = lse2;
    }
}

// Combine kernel (step a8): per (sequence, head), merge the chunk partials by log-sum-exp.
// The same m / l recurrence as Algorithm 1, applied across chunks instead of KV blocks.
__global__ void __launch_bounds__(kCombineThreads) mla_decode_combine_kernel(const Params p) {
    const int b = blockIdx.x / kHeads;
    const int h = blockIdx.x - b * kHeads;
    const int t = threadIdx.x;                // 128 threads x 4 columns
    int n = p.seqlens[b];
    n = n < 0 ? 0 : (n > p.max_seqlen ? p.max_seqlen : n);
    const int ns = (n + p.chunk_len - 1) / p.chunk_len;
    if (ns == 1) return;                      // the main kernel wrote out / lse directly
    float *out = p.out + ((long long)b * kHeads + h) * kDv + t * 4;
    if (ns == 0) {                            // empty sequence
        *reinterpret_cast<f32x4 *>(out) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t == 0) p.lse[b * kHeads + h] = -INFINITY;
        return;
    }
    const float *pl = p.part_lse + (long long)b * p.splits_max * kHeads + h;
    float m = -INFINITY;
    for (int s = 0; s < ns; ++s) m = fmaxf(m, pl[s * kHeads]);
    float sum = 0.f;
    for (int s = 0; s < ns; ++s) sum += __builtin_amdgcn_exp2f(pl[s * kHeads] - m);
    const float tot = m + __builtin_amdgcn_logf(sum);
    const float *po = p.part_out + ((long long)b * p.splits_max * kHeads + h) * kDv + t * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < ns; ++s) {
        const float wgt = __builtin_amdgcn_exp2f(pl[s * kHeads] - tot);
        acc += *reinterpret_cast<const f32x4 *>(po + (long long)s * kHeads * kDv) * wgt;
    }
    *reinterpret_cast<f32x4 *>(out) = acc;
    if (t == 0) p.lse[b * kHeads + h] = tot * 0.6931471805599453f;
}

// ---- host side ---------------------------------------------------------------------------------

inline size_t workspace_bytes_for(int batch, int splits_max) {
    // partial outputs + partial LSEs, each part 16-byte aligned
    const size_t po = (size_t)batch * splits_max * kHeads * kDv * sizeof(float);
    const size_t pl = (size_t)batch * splits_max * kHeads * sizeof(float);
    return po + ((pl + 15) & ~(size_t)15);
}

// Split plan (step a0): tokens per workgroup so that batch * splits covers every compute unit
// about `kUnitsPerCu` times; one workgroup is resident per compute unit.
constexpr int kUnitsPerCu = 2;
constexpr int kMinChunk = 256;

int plan_chunk_len(int batch, int max_seqlen_kv, int num_cus) {
    const long long total = (long long)batch * max_seqlen_kv;
    const long long units = (long long)num_cus * kUnitsPerCu;
    long long chunk = (total + units - 1) / units;
    if (chunk < kMinChunk) chunk = kMinChunk;
    chunk = (chunk + kChunkGranule - 1) / kChunkGranule * kChunkGranule;
    // even out the chunks of one sequence: same number of splits, smallest chunk that covers it
    const long long splits = (max_seqlen_kv + chunk - 1) / chunk;
    chunk = (max_seqlen_kv + splits - 1) / splits;
    chunk = (chunk + kChunkGranule - 1) / kChunkGranule * kChunkGranule;
    return (int)chunk;
}

bool misaligned(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; }

mla_status_t check_shape(int batch, int num_heads, int max_seqlen_kv) {
    if (batch <= 0 || max_seqlen_kv <= 0 || num_heads <= 0) return MLA_ERR_INVALID_ARG;
    if (num_heads != kHeads) return MLA_ERR_UNSUPPORTED_SHAPE;
    if ((long long)batch * max_seqlen_kv > (1ll << 40)) return MLA_ERR_INVALID_ARG;
    return MLA_OK;
}

mla_status_t validate(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                      const int32_t *cache_seqlens, int batch, int num_heads, int max_seqlen_kv,
                      float scale, const float *out, const float *lse, const void *workspace) {
    mla_status_t st = check_shape(batch, num_heads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (!q || !kv_cache || !cache_seqlens || !out || !lse || !workspace) return MLA_ERR_INVALID_ARG;
    if (misaligned(q) || misaligned(kv_cache) || misaligned(out) || misaligned(workspace) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u) || (reinterpret_cast<uintptr_t>(cache_seqlens) & 3u))
        return MLA_ERR_INVALID_ARG;
    if (kv_batch_stride < (int64_t)max_seqlen_kv * kDqk || (kv_batch_stride & 7) != 0) return MLA_ERR_INVALID_ARG;
    if (!(scale == scale) || std::isinf(scale)) return MLA_ERR_INVALID_ARG;
    return MLA_OK;
}

// Everything below runs only after validate() passed.
mla_status_t launch(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                    const int32_t *cache_seqlens, int batch, int max_seqlen_kv, float scale,
                    float *out, float *lse, void *workspace, size_t workspace_bytes, int chunk_len,
                    int phases, void *stream) {
    if (chunk_len <= 0 || chunk_len % kChunkGranule != 0) return MLA_ERR_INVALID_ARG;
    const int splits_max = (max_seqlen_kv + chunk_len - 1) / chunk_len;
    if ((long long)batch * splits_max > 0x7fffffffll) return MLA_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_bytes_for(batch, splits_max)) return MLA_ERR_WORKSPACE_TOO_SMALL;

    // the main kernel needs more dynamic LDS than the default limit: raise it once per device
    static std::mutex mu;
    static bool attr_done[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MLA_ERR_HIP;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!attr_done[dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(mla_decode_split_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
                return MLA_ERR_HIP;
            attr_done[dev] = true;
        }
    }

    Params p;
    p.q = static_cast<const char *>(q);
    p.kv = static_cast<const char *>(kv_cache);
    p.kv_batch_bytes = (long long)kv_batch_stride * 2;
    p.seqlens = cache_seqlens;
    p.out = out;
    p.lse = lse;
    p.part_out = static_cast<float *>(workspace);
    p.part_lse = p.part_out + (size_t)batch * splits_max * kHeads * kDv;
    p.max_seqlen = max_seqlen_kv;
    p.chunk_len = chunk_len;
    p.splits_max = splits_max;
    p.scale_log2e = scale * 1.4426950408889634f;

    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (phases & MLA_PHASE_SPLIT) {
        hipLaunchKernelGGL(mla_decode_split_kernel, dim3(batch * splits_max), dim3(kThreads), kLdsBytes, hs, p);
        if (hipGetLastError() != hipSuccess) return MLA_ERR_HIP;
    }
    if (phases & MLA_PHASE_COMBINE) {
        hipLaunchKernelGGL(mla_decode_combine_kernel, dim3(batch * kHeads), dim3(kCombineThreads), 0, hs, p);
        if (hipGetLastError() != hipSuccess) return MLA_ERR_HIP;
    }
    return MLA_OK;
}

}  // namespace

extern "C" {

mla_status_t mla_decode_workspace_size_for_chunk(int batch, int max_seqlen_kv, int chunk_len,
                                                 size_t *bytes, int *num_splits_max) {
    if (!bytes) return MLA_ERR_INVALID_ARG;
    mla_status_t st = check_shape(batch, kHeads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (chunk_len <= 0 || chunk_len % kChunkGranule != 0) return MLA_ERR_INVALID_ARG;
    const int splits_max = (max_seqlen_kv + chunk_len - 1) / chunk_len;
    *bytes = workspace_bytes_for(batch, splits_max);
    if (num_splits_max) *num_splits_max = splits_max;
    return MLA_OK;
}

mla_status_t mla_decode_workspace_size(int batch, int num_heads, int max_seqlen_kv, int num_cus,
                                       size_t *bytes, int *chunk_len, int *num_splits_max) {
    if (!bytes) return MLA_ERR_INVALID_ARG;
    mla_status_t st = check_shape(batch, num_heads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (num_cus < 0) return MLA_ERR_INVALID_ARG;
    if (num_cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return MLA_ERR_HIP;
        if (hipDeviceGetAttribute(&num_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || num_cus <= 0)
            return MLA_ERR_HIP;
    }
    const int chunk = plan_chunk_len(batch, max_seqlen_kv, num_cus);
    if (chunk_len) *chunk_len = chunk;
    return mla_decode_workspace_size_for_chunk(batch, max_seqlen_kv, chunk, bytes, num_splits_max);
}

static mla_status_t planned_chunk(int batch, int max_seqlen_kv, int *chunk) {
    int dev = 0, num_cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MLA_ERR_HIP;
    if (hipDeviceGetAttribute(&num_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || num_cus <= 0)
        return MLA_ERR_HIP;
    *chunk = plan_chunk_len(batch, max_seqlen_kv, num_cus);
    return MLA_OK;
}

mla_status_t mla_decode_ex(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                           const int32_t *cache_seqlens, int batch, int num_heads, int max_seqlen_kv,
                           float scale, float *out, float *lse, void *workspace, size_t workspace_bytes,
                           int chunk_len, int phases, void *stream) {
    mla_status_t st = validate(q, kv_cache, kv_batch_stride, cache_seqlens, batch, num_heads, max_seqlen_kv,
                               scale, out, lse, workspace);
    if (st != MLA_OK) return st;
    if (chunk_len < 0 || chunk_len % kChunkGranule != 0) return MLA_ERR_INVALID_ARG;
    if (phases <= 0 || (phases & ~(MLA_PHASE_SPLIT | MLA_PHASE_COMBINE)) != 0) return MLA_ERR_INVALID_ARG;
    if (chunk_len == 0) {
        st = planned_chunk(batch, max_seqlen_kv, &chunk_len);
        if (st != MLA_OK) return st;
    }
    return launch(q, kv_cache, kv_batch_stride, cache_seqlens, batch, max_seqlen_kv, scale, out, lse,
                  workspace, workspace_bytes, chunk_len, phases, stream);
}

mla_status_t mla_decode(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                        const int32_t *cache_seqlens, int batch, int num_heads, int max_seqlen_kv,
                        float scale, float *out, float *lse, void *workspace, size_t workspace_bytes,
                        void *stream) {
    return mla_decode_ex(q, kv_cache, kv_batch_stride, cache_seqlens, batch, num_heads, max_seqlen_kv, scale,
                         out, lse, workspace, workspace_bytes, 0, MLA_PHASE_SPLIT | MLA_PHASE_COMBINE, stream);
}

const char *mla_status_string(mla_status_t status) {
    switch (status) {
        case MLA_OK: return "ok";
        case MLA_ERR_INVALID_ARG: return "invalid argument";
        case MLA_ERR_UNSUPPORTED_SHAPE: return "unsupported shape (need 16 heads, d_qk 576, d_v 512, q_len 1)";
        case MLA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MLA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
