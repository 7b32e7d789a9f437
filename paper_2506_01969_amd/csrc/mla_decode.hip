// MLA decode attention for gfx950 (MI355X): split-KV main kernel + LSE combine kernel + C ABI.
//
// Problem (paper Section 3.1, decoding setup of Section 4.1): for every sequence b and each of
// 16 heads, one query row of 576 bf16 attends over N_b latent KV rows of 576 bf16 shared by all
// heads; V is the first 512 columns of the same row.  out = softmax(scale * q K^T) V, plus the
// log-sum-exp of the scaled scores (the L of Algorithm 1's last step).  Variants of the same
// kernel take fp16 inputs and several query tokens per sequence (template parameters below).
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
// Work decomposition.  The KV rows of all sequences form one stream of 128-token units
// (a sequence of N tokens holds ceil(N/128) units).  The grid is persistent: workgroup k of G
// takes the contiguous unit range [k*U/G, (k+1)*U/G) of that stream, whatever the lengths are,
// so ragged batches are balanced to one unit and every workgroup streams the same amount.
// A range may cross sequence boundaries; each (workgroup, sequence) part of it is a "piece" and
// ends with its own epilogue (the next piece's first loads are issued before that epilogue).
// Every workgroup derives the partition from cache_seqlens on the device (one vector load and a
// wave scan), so the host never needs the lengths.  The assignment is static: results are
// bit-identical from run to run.
//
// Each wavefront is an independent online-softmax worker (the m / l / rescale recurrence of
// Algorithm 1) over every 4th 32-token tile of the piece, with a private LDS tile, so the main
// loop has no barrier.  A tile is fetched with 16-byte coalesced global loads into registers (in
// flight while the previous tile is being computed; the 36 loads of a tile are issued one by one
// between the MFMAs of the tile before it, never in a burst: a wavefront waits at a load
// instruction until the compute unit's memory path has room for it), written once to LDS, and
// read twice from LDS: as the K operand (ds_read_b128) and, through the transposing LDS read
// ds_read_b64_tr_b16, as the V^T operand.  The four wavefronts of a
// workgroup merge their (m, l, O) through LDS at the end of the piece; a sequence shared by
// several workgroups is finished by the combine kernel.
//
// Several query tokens per sequence (speculative / multi-token decoding, kShare = 2).  A workgroup
// takes two tokens: wavefronts 0 and 2 work for the first, 1 and 3 for the second.  Every
// wavefront still stages its own tiles, and then takes its own tile and its neighbour's (0 <-> 1,
// 2 <-> 3), read from the neighbour's LDS region, for its own token.  A KV row is thus fetched
// once for both tokens, every wavefront keeps a tile of its own in flight as with one token, and
// only the LDS reads and the MFMA work double.  Two workgroup barriers per round (neighbour's
// tile written / everyone done reading) replace the barrier-free loop.  More than two tokens are
// spread over teams of ceil(q_len / 2) such workgroups that stream the same KV rows at the same
// time behind one L2 cache.
//
// P is fed to the second MFMA as a two-term bf16 split (hi + lo): a single bf16 rounding of P
// costs ~2^-9 relative error per term, which is outside the 1e-4 RMSE bound at short KV.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>
#include <type_traits>

#include "mla_decode.h"
#include "mla_plan.h"

namespace {

constexpr int kHeads = MLA_NUM_HEADS;        // 16
constexpr int kDqk = MLA_D_QK;               // 576
constexpr int kDv = MLA_D_V;                 // 512
constexpr int kRowBytes = kDqk * 2;          // 1152 bytes per KV row
constexpr int kLdsPad = 32;                  // bytes between the rows of a tile in LDS
constexpr int kLdsRow = kRowBytes + kLdsPad; // LDS row stride 1184 B = 32 mod 64: see the access patterns in the main kernel
constexpr int kTile = 32;                    // tokens per wavefront step (MFMA K of the PV product)
constexpr int kWaves = 4;                    // wavefronts per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kWaveLds = kTile * kLdsRow;    // 37,888 B private tile per wavefront
constexpr int kTileLoads = kTile * kRowBytes / 1024;   // 36 loads of 64 lanes x 16 B per tile
static_assert(kTileLoads * 1024 == kTile * kRowBytes, "a tile must be a whole number of 1 KB pieces");
static_assert(kRowBytes == mla_plan::kRowBytes && kTile == mla_plan::kTileRows && kTileLoads == mla_plan::kTileLoads,
              "the plan header and the kernel disagree on the tile");
constexpr int kKSteps = kDqk / 32;           // 18 MFMA k-steps over the 576 dims
constexpr int kDvTiles = kDv / 16;           // 32 output tiles of 16 value columns
constexpr int kStatsOff = kWaves * kWaveLds; // m and l of the 4 wavefronts live after the tiles
constexpr int kRescaleOff = kStatsOff + 2 * kWaves * kHeads * 4;  // a slot per wavefront: cold rescale path (2 KB), P of the direct orientation
constexpr int kPStride = 36;                 // floats between the heads of P in that slot (direct orientation): 4 mod 16, see there
constexpr int kSlotBytes = kHeads * kPStride * 4;   // 2304
constexpr int kLdsBytes = kRescaleOff + kWaves * kSlotBytes;
static_assert(kLdsBytes <= 160 * 1024, "LDS of one compute unit");
static_assert(kWaves * kTile == MLA_UNIT_TOKENS && mla_plan::kUnitCoarse == MLA_UNIT_TOKENS && mla_plan::kUnitFine == MLA_UNIT_TOKENS_FINE,
              "header and kernel disagree on the scheduling units");
constexpr int kCombineCols = 128;               // threads that cover the 512 value columns, 4 each
constexpr int kCombineWide = 4;                 // groups of such threads per block when a sequence has many pieces,
constexpr int kCombineWidest = 16;              // and when it has more than 64 (one or two sequences over all compute units)
constexpr int kSchedMfma = 0x008;              // instruction classes of sched_group_barrier
constexpr int kSchedDsRead = 0x100;
constexpr int kSchedVmemRead = 0x020;
constexpr int kKAhead = 4;                     // k-steps of K operand reads in flight ahead of the QK MFMAs
constexpr int kVAhead = 6;                     // value tiles of V^T reads in flight ahead of the PV MFMAs

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

struct Params {
    const char *q;            // 16-bit floats [batch][16][576]
    const char *kv;           // 16-bit float rows of 576
    long long kv_batch_bytes; // bytes between sequences
    const int *seqlens;       // [batch]
    float *out;               // [batch][16][512]
    float *lse;               // [batch][16]
    float *part_out;          // [(num_wg + batch) * q_len][16][512]: slot of (team k, sequence b, token j) is (k + b) q_len + j
    float *part_lse;          // [(num_wg + batch) * q_len][16], base-2 log-sum-exp of scale*log2(e)*q.k
    int batch;                // sequences
    int q_len;                // query tokens per sequence
    int max_seqlen;
    int num_wg;               // G: teams (one workgroup per two query tokens) the unit stream is divided over
    int unit;                 // KV rows per unit of the stream: 128, or 32 for a short stream
    int stream_out;           // nonzero: the epilogue's stores are marked non-temporal (short streams, see launch())
    float scale_log2e;        // scale * log2(e): scores are kept in the base-2 domain
    long long *timeline;      // measurement build only (MLA_TIMELINE), else null: where the kernels leave their time stamps
};

// Measurement build (-DMLA_TIMELINE, a library of its own that the benchmark's --timeline mode loads):
// every wavefront of the main kernel and the first thread of every merge block record the 100 MHz
// real-time counter at the phase boundaries marked MLA_STAMP below (the first time each is passed) and
// write them to Params::timeline when they finish.  In the product build the marks compile to nothing.
#ifdef MLA_TIMELINE
#define MLA_STAMPS(n) long long stamps[n] = {}
#define MLA_STAMP(i) do { if (stamps[i] == 0) stamps[i] = (long long)__builtin_amdgcn_s_memrealtime(); } while (0)
constexpr int kSplitStamps = 8, kCombineStamps = 4;
constexpr long long kCombineStampBase = 1 << 20;      // in stamps, after the main kernel's
#else
#define MLA_STAMPS(n) ((void)0)
#define MLA_STAMP(i) ((void)0)
#endif

// The integer rules of the partition (units, ranges, slots, tile offsets) live in mla_plan.h, shared
// with the host code and the CPU tests; below are only their wave-parallel evaluations.
__device__ __forceinline__ int clamped_len(const Params &p, int b) { return mla_plan::clamp_len(p.seqlens[b], p.max_seqlen); }

__device__ __forceinline__ int units_at(const Params &p, int b) { return mla_plan::units_of(clamped_len(p, b), p.unit); }

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel primitives: row shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 (2) added to all of row 1 (3),
// then lane 31 added to rows 2 and 3.  A lane without a source keeps 0 as its addend.  Ten vector
// instructions and no trip through the LDS crossbar, which the shuffle builtins would take six times.
__device__ __forceinline__ int wave_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Sequences base .. base + 63, one per lane: the clamped length and the number of units of the
// sequences up to and including the lane's (carry = units of the sequences before base).  The
// lengths are fetched with one vector load instead of a chain of dependent scalar loads.
struct LaneScan {
    int len, incl;
};
__device__ __forceinline__ LaneScan scan_lengths(const Params &p, int lane, int base, int carry) {
    const int i = base + lane;
    LaneScan s;
    s.len = i < p.batch ? clamped_len(p, i) : 0;
    s.incl = wave_scan(mla_plan::units_of(s.len, p.unit)) + carry;
    return s;
}

// Units of all sequences (total) and of the sequences before b.  Every wavefront computes this for
// itself; the results are wave-uniform.
__device__ __forceinline__ void unit_sums(const Params &p, int lane, int b, int &total, int &before_b) {
    int carry = 0, bef = 0;
    for (int base = 0; base < p.batch; base += 64) {
        const LaneScan s = scan_lengths(p, lane, base, carry);
        if (b == base) bef = carry;
        else if (b > base && b < base + 64) bef = __builtin_amdgcn_readlane(s.incl, b - base - 1);
        carry = __builtin_amdgcn_readlane(s.incl, 63);
    }
    total = carry;
    before_b = bef;
}

// The sequence that holds unit `target` of the stream (0 <= target < total units), the stream index
// of that sequence's first unit and its length, from the scan of one chunk of 64 sequences; returns
// false if the unit lies beyond the chunk.  b = number of sequences whose inclusive prefix is <= target.
__device__ __forceinline__ bool locate_in_chunk(const Params &p, const LaneScan &s, int lane, int base, int carry, int target,
                                                int &b, int &first, int &n) {
    if (__builtin_amdgcn_readlane(s.incl, 63) <= target) return false;
    const unsigned long long below = __builtin_amdgcn_ballot_w64(base + lane < p.batch && s.incl <= target);
    const int in_chunk = __builtin_popcountll(below);          // the lanes below form a prefix: the scan never decreases
    b = base + in_chunk;
    first = in_chunk ? __builtin_amdgcn_readlane(s.incl, in_chunk - 1) : carry;
    n = __builtin_amdgcn_readlane(s.len, in_chunk);
    return true;
}

__device__ __forceinline__ void locate_unit(const Params &p, int lane, int target, int &b, int &first, int &n) {
    int carry = 0;
    b = first = n = 0;
    for (int base = 0; base < p.batch; base += 64) {
        const LaneScan s = scan_lengths(p, lane, base, carry);
        if (locate_in_chunk(p, s, lane, base, carry, target, b, first, n)) return;
        carry = __builtin_amdgcn_readlane(s.incl, 63);
    }
}

// 16-byte streaming load at (wave-uniform base) + (32-bit lane offset): the uniform part stays in
// scalar registers and the lane part is one VGPR, so a tile's 36 loads cost no address arithmetic.
// kReuse = false marks the load as streaming (no other reader of the row); with several query
// tokens the rows ARE read again, by the other workgroups of the team, so the hint is left off.
template <bool kReuse>
__device__ __forceinline__ u32x4 load_stream16(const char *uniform_base, unsigned lane_off) {
    if constexpr (kReuse) return *reinterpret_cast<const u32x4 *>(uniform_base + lane_off);
    else return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(uniform_base + lane_off));
}

// Transposing LDS read of a 4 (rows) x 16 (columns) block of 16-bit elements per 16-lane group.
__device__ __forceinline__ i16x4 read_tr16(const char *lds_addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) i16x4 *)(lds_char *)lds_addr);
}

__device__ __forceinline__ float wave_xor_max(float v, int mask) {
    return fmaxf(v, __shfl_xor(v, mask, 64));
}

// One 16x16x32 matrix-core step on 16-bit operands held as raw bits; kDtype selects bf16 or fp16.
template <int kDtype>
__device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (kDtype == MLA_DTYPE_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

constexpr float kLazyLog2 = 8.0f;   // the softmax reference moves only when exceeded by 2^8

// O <- O * alpha with O resident in accumulation registers (AGPRs), which the vector ALU cannot
// address.  Each 16x16 tile takes a round trip through a small private LDS slot (AGPR -> LDS ->
// VGPR, multiply, and the result is copied back), so the accumulators' own live range has no
// VALU use and the register allocator leaves them in place on the hot path.  This path is cold
// (see kLazyLog2).
__device__ __forceinline__ void rescale_accumulators(f32x4 (&o)[kDvTiles], f32x4 alpha, char *slot) {
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

// Main kernel (steps a0-a7 of the hot path): persistent grid, workgroup k streams its share of
// the unit stream piece by piece.
// kShare: query tokens per workgroup (1, or 2 with the wavefront pairs described at the top).
// kTeam: several workgroups read every KV row (more query tokens than one workgroup takes), so the
// loads are not marked as streaming.
//
// kDirect = false is the transposed orientation of equations (1)-(4) described at the top of this
// file.  kDirect = true is the original orientation of Section 3.1, kept for comparison:
//     S = Q K^T   (heads on the MFMA M axis, tokens on N)
//     O = P V     (heads on M, value columns on N, contraction over tokens)
// The same registers feed the first product with the operands swapped, but its result now leaves a
// lane with ONE token and four heads: the softmax maximum of a head needs a reduction across 16
// lanes, every lane carries the running statistics of four heads, and P has to be transposed
// across lanes (through 2 KB of LDS) before it can enter the second product.
template <int kDtype, bool kTeam, bool kDirect, int kShare>
__global__ void __launch_bounds__(kThreads, 1) mla_decode_split_kernel(const Params p) {
    static_assert(kShare == 1 || (kShare == 2 && !kDirect), "tokens per workgroup");
    constexpr int kGroups = kWaves / kShare;      // wavefronts that work for the same query token
    extern __shared__ __attribute__((aligned(16))) char smem[];

    MLA_STAMPS(8);
    MLA_STAMP(0);                 // wavefront started
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront in workgroup (scalar)
    const int l = tid & 63;       // lane
    const int r16 = l & 15;       // MFMA row/column index owned by this lane
    const int g = l >> 4;         // MFMA k-group (0..3)

    // ---- a0 on the device: this workgroup's range of the unit stream -------------------------
    // With more than kShare query tokens per sequence, ceil(q_len / kShare) workgroups form a team:
    // all of them take the same share of the unit stream, each for its own query tokens, so they
    // stream the same KV rows at the same time and only the first to ask brings a row in from HBM;
    // the others find it in the L2 cache (they run a little faster for it and so never fall far
    // behind).  The members of a team are a multiple of 8 workgroup ids apart: workgroups are
    // dealt to the 8 XCDs in turn and each XCD has its own L2, so this puts a team behind one L2.
    const int members = (p.q_len + kShare - 1) / kShare; // workgroups per team
    const int team_stride = gridDim.x / members;         // number of teams, rounded up to a multiple of 8
    const int jt = blockIdx.x / team_stride;             // member of the team
    const int k = blockIdx.x - jt * team_stride;         // team
    const int tk = w & (kShare - 1);                     // this wavefront's query token within the workgroup
    const int j = jt * kShare + tk;                      // query token of this wavefront (scalar)
    const bool has_token = j < p.q_len;                  // odd q_len: the last wavefront pair has one token only
    // Up to 64 sequences (one per lane): one vector load of the lengths and one scan give the total,
    // this team's range, its first sequence and that sequence's length.  Larger batches take a
    // second pass over the lengths once the total is known.
    int total_units, unused;
    const LaneScan first_chunk = scan_lengths(p, l, 0, 0);
    if (p.batch <= 64) total_units = __builtin_amdgcn_readlane(first_chunk.incl, 63);
    else unit_sums(p, l, 0, total_units, unused);
    MLA_STAMP(1);                 // lengths read and summed
    // never more workgroups than units: every active workgroup then holds at least one unit
    const int active = mla_plan::active_teams(total_units, p.num_wg);
    if (k >= active) return;                        // uniform over the workgroup
    int u_lo, u_hi;                                 // u_hi > u_lo
    mla_plan::unit_range(k, total_units, active, u_lo, u_hi);
    int b, seq_first, n_first;                      // first sequence of the range, stream index of its first unit, its length
    if (p.batch <= 64) locate_in_chunk(p, first_chunk, l, 0, 0, u_lo, b, seq_first, n_first);
    else locate_unit(p, l, u_lo, b, seq_first, n_first);

    char *my = smem + w * kWaveLds;                       // private tile of this wavefront
    // LDS addresses (bytes) of the three access patterns
    // write side: piece i, lane l holds chunk 64 i + l; lanes at or past the row boundary inside
    // the piece (lane 72 (q+1) - 64 i, a function of i mod 9) skip the row padding
    char *wr_flat[9];
#pragma unroll
    for (int r = 0; r < 9; ++r) {
        const int boundary = 72 * ((r * 64) / 72 + 1) - r * 64;     // 72, 8, 16, ..., 56, 64
        wr_flat[r] = my + l * 16 + (l >= boundary ? kLdsPad : 0);
    }
    // Bank behaviour of the three LDS access patterns, measured one pattern at a time with a probe kernel
    // and the SQ_LDS_BANK_CONFLICT counter (64 banks of 4 bytes, 256 bytes per cycle):
    //   K operand, ds_read_b128: lane (r16, g) reads 16 bytes of row r16 at chunk 4 kk + g.  A cycle serves
    //     lanes 0..7 of one 16-lane group together with lanes 8..15 of another, so rows 0..7 must fall on
    //     eight distinct 16-byte bank groups that, shifted by the other group's 16 g, miss those of rows
    //     8..15.  A row stride of 32 mod 64 bytes does that (rows r and r + 8 share a bank group, the four
    //     groups alternate between the even and the odd ones): every stride of 16 or 48 mod 64, such as
    //     1152 + 16, costs each of these reads a second pass, whatever the order of the rows.
    //   V^T operand, ds_read_b64_tr_b16: a cycle serves 32 lanes = eight rows x 32 bytes; with this stride
    //     rows 4g + q (q = the lane's quad) of k-groups g = 0, 1 and of g = 2, 3 tile the 64 banks exactly.
    //   tile write, ds_write_b128: conflict-free for every position of the row boundary inside a load.
    // So token t of a 16-token score block simply sits on MFMA position t, in both orientations; the
    // contraction index 8g + i of the second product stands for token 4g + i (i < 4) or 16 + 4g + i - 4.
    const int k_row = r16;
    const int k_off = k_row * kLdsRow + g * 16;           // K operand: token k_row (+16), chunk 4*kk + g
    // V^T operand (direct orientation: V) through the transposing read: within each 16-lane group,
    // lane j points at row j/4, columns 4*(j%4)..+3 of a 4x16 block and receives column j, rows 0..3.
    // Tokens of the two reads, in the order of the other operand's 8 k-values: 4g .. 4g+3 and 16 more.
    const int v_row = 4 * g + (r16 >> 2);
    const int v_off = v_row * kLdsRow + (r16 & 3) * 8;
    constexpr int kVSecond = 16 * kLdsRow;
    // direct orientation: P crosses lanes as fp32 [16 heads][32 tokens], in the rescale path's slot
    float *p_tr = reinterpret_cast<float *>(smem + kRescaleOff + w * kSlotBytes);
    float *stat_m = reinterpret_cast<float *>(smem + kStatsOff);
    float *stat_l = stat_m + kWaves * kHeads;
    const unsigned lane16 = (unsigned)l * 16;               // global-load lane offsets (bytes)

    // ---- the piece being worked on (this team's units of one sequence) -----------------------
    int n, ub, t_begin, t_end, n_tiles;   // t_end: end of what this wavefront's token sees; n_tiles: tiles staged
    bool direct;
    const char *kv_b;
    long long row;                    // row of q, out and lse
    auto set_piece = [&](int first_unit, int n_b) {   // uses b and seq_first; n_b: length of sequence b
        n = n_b;
        ub = mla_plan::units_of(n, p.unit);                    // > 0
        // the tiles staged cover what the last token of this workgroup sees
        const mla_plan::Piece pc = mla_plan::piece_of(n, ub, seq_first, first_unit, u_hi, p.unit, p.q_len, has_token ? j : p.q_len - 1,
                                                      min(jt * kShare + kShare - 1, p.q_len - 1), has_token);
        t_begin = pc.t_begin;
        t_end = pc.t_end;                                      // may be <= t_begin: nothing visible here
        n_tiles = pc.n_tiles;
        direct = pc.whole;                                     // this team covers the whole sequence
        kv_b = p.kv + (long long)b * p.kv_batch_bytes;
        row = (long long)b * p.q_len + (has_token ? j : p.q_len - 1);   // a wavefront without a token reads a valid q and writes nothing
    };

    u32x4 st[kTileLoads];             // one tile in flight: 36 x 16 B per lane
    // A tile is 32 consecutive rows = 36,864 contiguous bytes, fetched as 36 pieces of 1 KB
    // (lane l of piece i reads 16-byte chunk 64 i + l).  Fully sequential 1 KB requests
    // stream measurably faster from HBM than row-shaped ones.  Rows past the end of the
    // sequence are never fetched: chunk indices are clamped to the last valid chunk (the
    // scores of those rows are masked below, so whatever lands there has weight zero and
    // is finite data of a valid row).
    auto issue_loads = [&](int tile) {              // tile of the current piece
        const int tb = t_begin + tile * kTile;
        const int valid_rows = min(n - tb, kTile);                 // >= 1
        const int last_chunk16 = mla_plan::last_chunk_offset(valid_rows);    // byte offset of the last valid chunk
        const char *tile_base = kv_b + (long long)tb * kRowBytes;
#pragma unroll
        for (int i = 0; i < kTileLoads; ++i) {
            const int piece = mla_plan::piece_offset(i, last_chunk16);       // scalar
            st[i] = load_stream16<kTeam>(tile_base + piece, mla_plan::lane_offset(lane16, last_chunk16, piece));
        }
    };
    // ---- a1: Q^T as the MFMA B operand: lane (head r16, k-group g) holds dims 32*kk + 8*g .. +8
    u32x4 qf[kKSteps];
    auto load_q = [&]() {                           // q of the current piece's row
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(p.q + (row * kHeads + r16) * kRowBytes) + g;
#pragma unroll
        for (int kk = 0; kk < kKSteps; ++kk) qf[kk] = qp[4 * kk];
    };

    // The first tile is requested before q: loads come back in order, the tile is needed first (for
    // the LDS write) and q only after it (for the first product), so q's trip overlaps that write.
    set_piece(u_lo, n_first);
    MLA_STAMP(2);                 // range located, first piece known
    if (w < n_tiles) issue_loads(w);
    load_q();
    MLA_STAMP(3);                 // first tile and q requested (the wavefront waits here while the memory path is full)
    while (true) {
        // this wavefront's tiles of the piece: w, w + 4, w + 8, ...; the first tile and q are on their way
        int cur = w, nxt = w + kWaves;
        // Q must be resident before the first product.  It is waited for once, after the first tile
        // has been written to LDS and before any load of the next tile is issued; left to the
        // compiler, the wait would sit in the tile loop with a count that also drains the loads of
        // the next tile.
        auto wait_for_q = [&]() {
#pragma unroll
            for (int kk = 0; kk < kKSteps; ++kk) asm volatile("" : "+v"(qf[kk]));
        };

        f32x4 o[kDvTiles];
#pragma unroll
        for (int ct = 0; ct < kDvTiles; ++ct) o[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m_run = -INFINITY;      // softmax reference of this lane's head (base-2 domain)
        float l_run = 0.f;            // this lane's share of the running sum
        f32x4 m4 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};   // direct orientation: heads 4g .. 4g+3
        f32x4 l4 = {0.f, 0.f, 0.f, 0.f};

        bool first_tile = true;

        // ---- a2: registers -> private LDS tile --------------------------------------------
        // chunk c = 64 i + l goes to row c / 72, column chunk c % 72: byte 16 (c + c / 72).
        // The registers are not refilled here: the loads of the next tile are issued one by one
        // between the MFMAs of the tile(s) worked on next (below).  A compute unit takes in about
        // 58 GB/s at most, whatever is in flight, and a wavefront waits at a load instruction until
        // the memory path has room for it: a burst of 36 loads per wavefront costs up to 2.5 us during
        // which it issues nothing else, while one load per 30-100 ns of matrix-core work costs nothing.
        auto write_tile = [&]() {
#pragma unroll
            for (int i = 0; i < kTileLoads; ++i)
                *reinterpret_cast<u32x4 *>(wr_flat[i % 9] + i * 1024 + ((i * 64) / 72) * kLdsPad) = st[i];
        };
        const char *rf_base = nullptr;    // next tile to fetch while tiles are worked on
        int rf_last = 0;                  // byte offset of its last valid 16-byte chunk
        auto refill_piece = [&](int i) {
            const int piece = mla_plan::piece_offset(i, rf_last);           // scalar
            st[i] = load_stream16<kTeam>(rf_base + piece, mla_plan::lane_offset(lane16, rf_last, piece));
        };
        // The tile to fetch next: this wavefront's next tile of the piece; after its last tile, 36 reads
        // of the sequence's first KB, which cost next to nothing and keep the loop free of a second variant.
        auto set_refill = [&]() {
            const bool fetch = nxt < n_tiles;
            const int ntb = fetch ? t_begin + nxt * kTile : 0;
            rf_last = fetch ? mla_plan::last_chunk_offset(min(n - ntb, kTile)) : 1008;
            rf_base = kv_b + (long long)ntb * kRowBytes;
        };
        constexpr int kHalfLoads = kTileLoads / 2;     // 18 = 9 with the k-steps + 9 with the value tiles

        // ---- a3 to a6 on the 32 rows from row tb of the sequence that sit in an LDS tile (rd_k, rd_v:
        // this lane's read addresses in that tile), for this wavefront's query token.  refill says
        // which loads of the next tile go between the MFMAs: 0 none; 3 all 36, one per k-step and one
        // per value tile for the first 18 (one query token: one tile per round); 1 or 2 the first or
        // second 18, one per other k-step and other value tile (two tokens: two tiles per round)
        auto process_tile = [&](auto refill, const char *rd_k, const char *rd_v, const int tb) {
            constexpr int kRefill = decltype(refill)::value;
            constexpr int kRefillBase = kRefill == 2 ? kHalfLoads : 0;
            // ---- a3: S^T = K Q^T for tokens 0..15 and 16..31 of the tile (equation (1)) --
            // LDS reads run kKAhead k-steps ahead of the MFMAs that consume them.
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
            {
                u32x4 kb[kKAhead][2];
#pragma unroll
                for (int kk = 0; kk < kKAhead; ++kk) {
                    kb[kk][0] = *reinterpret_cast<const u32x4 *>(rd_k + kk * 64);
                    kb[kk][1] = *reinterpret_cast<const u32x4 *>(rd_k + 16 * kLdsRow + kk * 64);
                }
#pragma unroll
                for (int kk = 0; kk < kKSteps; ++kk) {
                    const u32x4 k0 = kb[kk % kKAhead][0];
                    const u32x4 k1 = kb[kk % kKAhead][1];
                    if (kk + kKAhead < kKSteps) {
                        kb[kk % kKAhead][0] = *reinterpret_cast<const u32x4 *>(rd_k + (kk + kKAhead) * 64);
                        kb[kk % kKAhead][1] = *reinterpret_cast<const u32x4 *>(rd_k + 16 * kLdsRow + (kk + kKAhead) * 64);
                    }
                    if constexpr (kDirect) {
                        s0 = mfma_16x16x32<kDtype>(qf[kk], k0, s0);
                        s1 = mfma_16x16x32<kDtype>(qf[kk], k1, s1);
                    } else {
                        s0 = mfma_16x16x32<kDtype>(k0, qf[kk], s0);
                        s1 = mfma_16x16x32<kDtype>(k1, qf[kk], s1);
                    }
                    if constexpr (kRefill == 3) {
                        refill_piece(kk);
                    } else if constexpr (kRefill != 0) {
                        if (kk % 2 == 0) refill_piece(kRefillBase + kk / 2);
                    }
                }
                // pin that interleaving for the instruction scheduler: reads first, then
                // (2 MFMA, 2 LDS reads) per k-step, so LDS latency hides behind the MFMAs
                __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2 * kKAhead, 0);
#pragma unroll
                for (int kk = 0; kk < kKSteps; ++kk) {
                    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 2, 0);
                    if (kk + kKAhead < kKSteps) __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 0);
                    if constexpr (kRefill == 3) {
                        __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 0);
                    } else if constexpr (kRefill != 0) {
                        if (kk % 2 == 0) __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 0);
                    }
                }
            }
            float pr[8];
            if constexpr (kDirect) {
                // this lane holds, for token tb + k_row (s0) and tb + 16 + k_row (s1), heads 4g + i
                const bool v0 = tb + k_row < t_end, v1 = tb + 16 + k_row < t_end;
                f32x4 x0, x1, mx4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x0[i] = v0 ? s0[i] * p.scale_log2e : -INFINITY;
                    x1[i] = v1 ? s1[i] * p.scale_log2e : -INFINITY;
                    float mm = fmaxf(x0[i], x1[i]);
                    mm = wave_xor_max(mm, 1);
                    mm = wave_xor_max(mm, 2);
                    mm = wave_xor_max(mm, 4);
                    mm = wave_xor_max(mm, 8);           // over the 16 lanes (tokens) of this k-group
                    mx4[i] = mm;
                }
                if (first_tile) {
                    m4 = mx4;
                    first_tile = false;
                } else {
                    bool move = false;
#pragma unroll
                    for (int i = 0; i < 4; ++i) move |= mx4[i] > m4[i] + kLazyLog2;
                    if (__builtin_amdgcn_ballot_w64(move) != 0) {
                        f32x4 alpha;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float m_new = fmaxf(m4[i], mx4[i]);
                            alpha[i] = __builtin_amdgcn_exp2f(m4[i] - m_new);
                            m4[i] = m_new;
                        }
                        rescale_accumulators(o, alpha, smem + kRescaleOff + w * kSlotBytes + l * 16);
                        l4 *= alpha;
                    }
                }
                // P[head 4g+i][token] -> LDS, then this lane takes head r16, tokens 4g .. 4g+3 and 16 more
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(x0[i] - m4[i]);
                    const float p1 = __builtin_amdgcn_exp2f(x1[i] - m4[i]);
                    l4[i] += p0 + p1;
                    p_tr[(4 * g + i) * kPStride + r16] = p0;
                    p_tr[(4 * g + i) * kPStride + 16 + r16] = p1;
                }
                // (heads 36 floats apart: the four k-groups' stores then fall on 64 distinct banks)
                const f32x4 lo4 = *reinterpret_cast<const f32x4 *>(p_tr + r16 * kPStride + 4 * g);      // same wavefront:
                const f32x4 hi4 = *reinterpret_cast<const f32x4 *>(p_tr + r16 * kPStride + 16 + 4 * g); // LDS keeps its order
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pr[i] = lo4[i];
                    pr[4 + i] = hi4[i];
                }
            } else {
            // this lane now holds, for head r16, tokens tb + 4g + i (s0[i]) and 16 more (s1[i])

            // ---- a4: scale (base-2 domain) and mask the tail ------------------------------
            float x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = (tb + 4 * g + i < t_end) ? s0[i] * p.scale_log2e : -INFINITY;
                x[4 + i] = (tb + 16 + 4 * g + i < t_end) ? s1[i] * p.scale_log2e : -INFINITY;
            }

            // ---- a5: online softmax (Algorithm 1: m, l update) -----------------------------
            // The reference maximum m_run moves lazily: exponentials are taken against the
            // current reference and O, l are rescaled by exp(m_old - m_new) (the R of Algorithm
            // 1) only when some head's tile maximum exceeds its reference by more than
            // kLazyLog2 (so p <= 2^8).  Any reference gives the same O / l and m + log l; moving
            // it rarely keeps the 128 accumulator registers out of the vector ALU on almost
            // every tile.
            float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            mx = wave_xor_max(mx, 16);
            mx = wave_xor_max(mx, 32);                       // finite: every tile has >= 1 valid token
            if (first_tile) {
                m_run = mx;                                  // first tile: O = 0 and l = 0, nothing to rescale
                first_tile = false;
            } else if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazyLog2) != 0) {
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                rescale_accumulators(o, f32x4{alpha, alpha, alpha, alpha}, smem + kRescaleOff + w * kSlotBytes + l * 16);
                l_run *= alpha;
                m_run = m_new;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                pr[i] = __builtin_amdgcn_exp2f(x[i] - m_run);
                l_run += pr[i];
            }
            }   // orientation

            // P^T as B operand.  bf16: two-term split hi + lo (16 significant bits); fp16: one term
            // (11 significant bits; p <= 2^8 is far inside the fp16 range).
            u32x4 p_hi, p_lo;
            if constexpr (kDtype == MLA_DTYPE_BF16) {
                bf16x8 hi, lo;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    hi[i] = (__bf16)pr[i];
                    lo[i] = (__bf16)(pr[i] - (float)hi[i]);
                }
                p_hi = __builtin_bit_cast(u32x4, hi);
                p_lo = __builtin_bit_cast(u32x4, lo);
            } else {
                f16x8 hi;
#pragma unroll
                for (int i = 0; i < 8; ++i) hi[i] = (_Float16)pr[i];
                p_hi = __builtin_bit_cast(u32x4, hi);
                p_lo = p_hi;    // unused
            }
            constexpr int kPTerms = (kDtype == MLA_DTYPE_BF16) ? 2 : 1;

            // ---- a6: O^T += V^T P^T (equation (3)), V^T from the same LDS tile --------------
            // The transposing reads run kVAhead value tiles ahead of their MFMAs.
            {
                i16x4 vb[kVAhead][2];
                const char *rd_v2 = rd_v + kVSecond;      // the tile's other 16 rows
#pragma unroll
                for (int ct = 0; ct < kVAhead; ++ct) {
                    vb[ct][0] = read_tr16(rd_v + ct * 32);
                    vb[ct][1] = read_tr16(rd_v2 + ct * 32);
                }
#pragma unroll
                for (int ct = 0; ct < kDvTiles; ++ct) {
                    const i16x4 vv[2] = {vb[ct % kVAhead][0], vb[ct % kVAhead][1]};
                    u32x4 vt;
                    __builtin_memcpy(&vt, vv, 16);
                    if (ct + kVAhead < kDvTiles) {
                        vb[ct % kVAhead][0] = read_tr16(rd_v + (ct + kVAhead) * 32);
                        vb[ct % kVAhead][1] = read_tr16(rd_v2 + (ct + kVAhead) * 32);
                    }
                    if constexpr (kDirect) {
                        o[ct] = mfma_16x16x32<kDtype>(p_hi, vt, o[ct]);
                        if constexpr (kPTerms == 2) o[ct] = mfma_16x16x32<kDtype>(p_lo, vt, o[ct]);
                    } else {
                        o[ct] = mfma_16x16x32<kDtype>(vt, p_hi, o[ct]);
                        if constexpr (kPTerms == 2) o[ct] = mfma_16x16x32<kDtype>(vt, p_lo, o[ct]);
                    }
                    if constexpr (kRefill == 3) {
                        if (ct < kTileLoads - kKSteps) refill_piece(kKSteps + ct);
                    } else if constexpr (kRefill != 0) {
                        if (ct % 2 == 0 && ct / 2 < kHalfLoads - kKSteps / 2) refill_piece(kRefillBase + kKSteps / 2 + ct / 2);
                    }
                }
                __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2 * kVAhead, 1);
#pragma unroll
                for (int ct = 0; ct < kDvTiles; ++ct) {
                    __builtin_amdgcn_sched_group_barrier(kSchedMfma, kPTerms, 1);
                    if (ct + kVAhead < kDvTiles) __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 1);
                    if constexpr (kRefill == 3) {
                        if (ct < kTileLoads - kKSteps) __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
                    } else if constexpr (kRefill != 0) {
                        if (ct % 2 == 0 && ct / 2 < kHalfLoads - kKSteps / 2) __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
                    }
                }
            }
        };

        if constexpr (kShare == 1) {
            while (cur < n_tiles) {
                set_refill();
                write_tile();
                if (cur == w) wait_for_q();
                MLA_STAMP(4);     // first tile arrived and written to LDS, q arrived
                process_tile(std::integral_constant<int, 3>{}, my + k_off, my + v_off, t_begin + cur * kTile);
                cur = nxt;
                nxt += kWaves;
            }
        } else {
            // Two wavefronts, one per query token, share the tiles that each of them stages: every
            // wavefront takes its own tile first and then its neighbour's tile, for its own token.  Each
            // KV row is fetched once for both tokens and every wavefront still keeps a tile of its own
            // in flight.  The barriers are reached by all wavefronts the same number of times
            // (n_tiles is the same for all of them).
            for (int base = 0; base < n_tiles; base += kWaves) {
                // While the two tiles are worked on, the registers are refilled with this wavefront's next tile.
                set_refill();
                if (cur < n_tiles) write_tile();
                if (base == 0) wait_for_q();
                {
                    const int tb = t_begin + cur * kTile;
                    if (cur < n_tiles && tb < t_end) {               // own tile: staged, and visible to this token
                        process_tile(std::integral_constant<int, 1>{}, my + k_off, my + v_off, tb);
                    } else {
#pragma unroll
                        for (int i = 0; i < kHalfLoads; ++i) refill_piece(i);
                    }
                }
                __syncthreads();                                     // the neighbour's tile is in LDS
                {
                    const int ws = w ^ 1;
                    const int tb = t_begin + (base + ws) * kTile;
                    if (base + ws < n_tiles && tb < t_end) {         // staged, and visible to this token
                        const char *tile = smem + ws * kWaveLds;
                        process_tile(std::integral_constant<int, 2>{}, tile + k_off, tile + v_off, tb);
                    } else {
#pragma unroll
                        for (int i = kHalfLoads; i < kTileLoads; ++i) refill_piece(i);
                    }
                }
                __syncthreads();                                     // before the tiles are overwritten
                cur = nxt;
                nxt += kWaves;
            }
        }

        MLA_STAMP(5);             // last tile of the (first) piece done
        // ---- the next piece's q and first tile go in flight before this piece's epilogue, so a
        // workgroup whose share crosses a sequence boundary does not restart from an empty pipeline
        const bool ep_direct = direct;
        const long long ep_row = row;
        const long long slot = mla_plan::slot_of(k, b, p.q_len, j);
        const bool more = seq_first + ub < u_hi;
        if (more) {
            const int first_unit = seq_first + ub;
            seq_first = first_unit;
            b = mla_plan::next_nonempty(p.seqlens, b + 1, p.max_seqlen, p.unit);   // empty sequences hold no units
            set_piece(first_unit, clamped_len(p, b));
            if (w < n_tiles) issue_loads(w);
            load_q();
        }

        // ---- a7: merge the four wavefronts, normalise, write (the epilogue of Algorithm 1) ----
        if constexpr (kDirect) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = l4[i];
                s += __shfl_xor(s, 1, 64);
                s += __shfl_xor(s, 2, 64);
                s += __shfl_xor(s, 4, 64);
                s += __shfl_xor(s, 8, 64);
                if (r16 == 0) {
                    stat_m[w * kHeads + 4 * g + i] = m4[i];
                    stat_l[w * kHeads + 4 * g + i] = s;
                }
            }
        } else {
            l_run += __shfl_xor(l_run, 16, 64);
            l_run += __shfl_xor(l_run, 32, 64);
            if (g == 0) {
                stat_m[w * kHeads + r16] = m_run;
                stat_l[w * kHeads + r16] = l_run;
            }
        }
        // own accumulators into the own (now idle) tile: [ct][lane] x 16 B
#pragma unroll
        for (int ct = 0; ct < kDvTiles; ++ct) *reinterpret_cast<f32x4 *>(my + ct * 1024 + l * 16) = o[ct];
        __syncthreads();
        MLA_STAMP(6);             // all four wavefronts have put their accumulators in LDS

        // Statistics of the head(s) whose accumulator elements this lane holds: head r16 in all four
        // elements (transposed orientation), or heads 4g .. 4g+3, one per element (direct orientation).
        // The wavefronts merged are those of this wavefront's token: tk, tk + kShare, ...
        f32x4 f[kGroups];
        float lse2_of[4];
        constexpr int kStatHeads = kDirect ? 4 : 1;
#pragma unroll
        for (int i = 0; i < kStatHeads; ++i) {
            const int hd = kDirect ? 4 * g + i : r16;
            float m_tot = stat_m[tk * kHeads + hd];
#pragma unroll
            for (int ww = 1; ww < kGroups; ++ww) m_tot = fmaxf(m_tot, stat_m[(tk + ww * kShare) * kHeads + hd]);
            const bool none = (m_tot == -INFINITY);      // the whole workgroup drew no tile of this sequence
            float fw[kGroups];
            float l_tot = 0.f;
#pragma unroll
            for (int ww = 0; ww < kGroups; ++ww) {
                fw[ww] = none ? 0.f : __builtin_amdgcn_exp2f(stat_m[(tk + ww * kShare) * kHeads + hd] - m_tot);   // 0 for an idle wavefront
                l_tot += fw[ww] * stat_l[(tk + ww * kShare) * kHeads + hd];
            }
            const float inv_l = none ? 0.f : 1.0f / l_tot;
#pragma unroll
            for (int ww = 0; ww < kGroups; ++ww) {
                if constexpr (kDirect) f[ww][i] = fw[ww] * inv_l;
                else f[ww] = f32x4{fw[ww] * inv_l, fw[ww] * inv_l, fw[ww] * inv_l, fw[ww] * inv_l};
            }
            lse2_of[i] = none ? -INFINITY : m_tot + __builtin_amdgcn_logf(l_tot);   // v_log_f32 is log2
        }

        float *dst = ep_direct ? p.out + ep_row * kHeads * kDv : p.part_out + slot * kHeads * kDv;
        // of its token's 32 value tiles, this wavefront finishes an equal share (8 with one token)
        constexpr int kFinish = kDvTiles / kGroups;
#pragma unroll
        for (int c = 0; c < kFinish; ++c) {
            const int ct = (w / kShare) * kFinish + c;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < kGroups; ++ww) {
                const f32x4 part = *reinterpret_cast<const f32x4 *>(smem + (tk + ww * kShare) * kWaveLds + ct * 1024 + l * 16);
                acc += part * f[ww];
            }
            if constexpr (kDirect) {      // element i: head 4g + i, column 16 ct + r16
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[(4 * g + i) * kDv + ct * 16 + r16] = acc[i];
            } else {                      // head r16, columns 16 ct + 4g .. +3; equation (4): transpose by addressing
                f32x4 *to = reinterpret_cast<f32x4 *>(dst + r16 * kDv + ct * 16 + g * 4);
                if (has_token) {
                    if (p.stream_out) __builtin_nontemporal_store(acc, to);
                    else *to = acc;
                }
            }
        }
        if (w < kShare && has_token && (kDirect ? r16 == 0 : g == 0)) {
#pragma unroll
            for (int i = 0; i < kStatHeads; ++i) {
                const int hd = kDirect ? 4 * g + i : r16;
                if (ep_direct) p.lse[ep_row * kHeads + hd] = lse2_of[i] * 0.6931471805599453f;
                else p.part_lse[slot * kHeads + hd] = lse2_of[i];
            }
        }

#ifdef MLA_TIMELINE
        if (!more && p.timeline) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the results have left
            MLA_STAMP(7);
            if (l == 0)
                for (int i = 0; i < kSplitStamps; ++i) p.timeline[((long long)blockIdx.x * kWaves + w) * kSplitStamps + i] = stamps[i];
        }
#endif
        if (!more) break;
        __syncthreads();              // the tiles are overwritten next; everyone must be done reading them
    }
}

// Combine kernel (step a8): per (sequence, head), merge the partial results of the workgroups
// that shared the sequence by log-sum-exp: the m / l recurrence of Algorithm 1 applied across
// workgroups instead of KV blocks.  The set of workgroups follows from the same partition.
// kCombineGroups thread groups take the pieces in turn; the 512 value columns are divided over
// kCombineSlices blocks (a block is one compute unit's worth of memory intake: with hundreds of pieces
// per sequence and few sequences, one block per (sequence, head) would read 2 KB per piece alone).
template <int kCombineGroups, int kCombineSlices>
__global__ void __launch_bounds__(kCombineCols * kCombineGroups / kCombineSlices) mla_decode_combine_kernel(const Params p) {
    constexpr int kGroupThreads = kCombineCols / kCombineSlices;   // threads of a group, 4 columns each
    MLA_STAMPS(4);
    MLA_STAMP(0);                 // block started
    const int rh = blockIdx.x / kCombineSlices;
    const int slice = blockIdx.x - rh * kCombineSlices;
    const int row = rh / kHeads;              // (sequence, query token)
    const int h = rh - row * kHeads;
    const int b = row / p.q_len;
    const int j = row - b * p.q_len;
    const int t = threadIdx.x % kGroupThreads;        // thread within its group
    const int pg = threadIdx.x / kGroupThreads;       // group of pieces
    const int col = (slice * kGroupThreads + t) * 4;  // this thread's four columns
    const bool writes_lse = (slice == 0 && threadIdx.x == 0);
    int total_units, seq_first;
    unit_sums(p, threadIdx.x & 63, b, total_units, seq_first);
    MLA_STAMP(1);                 // lengths read and summed
    const int ub = units_at(p, b);
    float *out = p.out + ((long long)row * kHeads + h) * kDv + col;
    if (ub == 0) {                            // empty sequence
        if (pg == 0) *reinterpret_cast<f32x4 *>(out) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (writes_lse) p.lse[row * kHeads + h] = -INFINITY;
        return;
    }
    const int active = mla_plan::active_teams(total_units, p.num_wg);       // as in the main kernel
    int k_first, k_last;
    mla_plan::bound_teams(seq_first, ub, total_units, active, k_first, k_last);
    const int ns = k_last - k_first + 1;
    if (ns == 1) return;                      // the main kernel wrote out / lse directly
    // the pieces of this row sit q_len slots apart
    const long long first_slot = mla_plan::slot_of(k_first, b, p.q_len, j);
    const int lstep = p.q_len * kHeads;
    const long long ostep = (long long)p.q_len * kHeads * kDv;
    const float *pl = p.part_lse + first_slot * kHeads + h;
    const float *po = p.part_out + (first_slot * kHeads + h) * kDv + col;
    // The kernel is a chain of memory round trips, so the pieces are dealt to the block's thread
    // groups in turn (one group, or four when the host expects more than kBatch pieces per sequence:
    // few sequences over many workgroups), and each group issues every load of up to kBatch of its pieces (their
    // log-sum-exps and the thread's four columns) before anything is waited for; more pieces than
    // that are folded in batch by batch with the same running-maximum recurrence.  The groups'
    // results are merged through LDS at the end.
    constexpr int kBatch = 16;
    float m = -INFINITY, sum = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = pg; s0 < ns; s0 += kBatch * kCombineGroups) {
        float ls[kBatch];
        f32x4 v[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int si = s0 + i * kCombineGroups;
            const bool on = si < ns;
            ls[i] = on ? pl[si * lstep] : -INFINITY;
            v[i] = on ? *reinterpret_cast<const f32x4 *>(po + si * ostep) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
        float mb = m;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) mb = fmaxf(mb, ls[i]);
        if (mb == -INFINITY) continue;        // nothing but empty pieces so far
        const float keep = __builtin_amdgcn_exp2f(m - mb);     // 0 when m is still -inf
        sum *= keep;
        acc *= keep;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const float wgt = __builtin_amdgcn_exp2f(ls[i] - mb);   // 0 for an empty or absent piece
            sum += wgt;
            if (ls[i] != -INFINITY) acc += v[i] * wgt;              // (an empty piece holds zeros anyway)
        }
        m = mb;
    }
    // merge the groups: group 0 folds in the (m, sum, acc) of the others
    if constexpr (kCombineGroups > 1) {
        __shared__ f32x4 g_acc[kCombineGroups - 1][kGroupThreads];
        __shared__ float g_m[kCombineGroups - 1], g_sum[kCombineGroups - 1];
        if (pg > 0) {
            g_acc[pg - 1][t] = acc;
            if (t == 0) {
                g_m[pg - 1] = m;
                g_sum[pg - 1] = sum;
            }
        }
        __syncthreads();
        if (pg > 0) return;
        float mb = m;
#pragma unroll
        for (int i = 0; i < kCombineGroups - 1; ++i) mb = fmaxf(mb, g_m[i]);
        if (mb != -INFINITY) {
            const float keep = __builtin_amdgcn_exp2f(m - mb);
            sum *= keep;
            acc *= keep;
#pragma unroll
            for (int i = 0; i < kCombineGroups - 1; ++i) {
                const float wgt = __builtin_amdgcn_exp2f(g_m[i] - mb);      // 0 for a group without pieces
                sum += wgt * g_sum[i];
                if (g_m[i] != -INFINITY) acc += g_acc[i][t] * wgt;
            }
            m = mb;
        }
    }
    if (m == -INFINITY) {                     // a query token that sees no row at all (length < q_len)
        *reinterpret_cast<f32x4 *>(out) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (writes_lse) p.lse[row * kHeads + h] = -INFINITY;
        return;
    }
    const float tot = m + __builtin_amdgcn_logf(sum);
    acc *= 1.0f / sum;
    MLA_STAMP(2);                 // partial results arrived and merged
    *reinterpret_cast<f32x4 *>(out) = acc;
#ifdef MLA_TIMELINE
    if (p.timeline) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        MLA_STAMP(3);             // result stored
        if (threadIdx.x == 0)
            for (int i = 0; i < kCombineStamps; ++i) p.timeline[kCombineStampBase + (long long)blockIdx.x * kCombineStamps + i] = stamps[i];
    }
#endif
    if (writes_lse) p.lse[row * kHeads + h] = tot * 0.6931471805599453f;
}

// Diagnostic kernel: the partition exactly as the two kernels above derive it (the same device
// functions on the same arguments), written out as a table of 8 ints per record.  Block x < G writes
// team x's record {total units, active teams, first unit, end unit, first sequence, that sequence's
// first unit, its clamped length, 0} (first unit .. first unit of the sequence are -1 for an idle team); block G + b writes sequence b's record
// {total units, first unit, units, first team, last team, 0, 0, 0} (teams -1 for an empty sequence).
__global__ void __launch_bounds__(64) mla_decode_plan_kernel(const Params p, int *table) {
    const int l = threadIdx.x;
    int rec[8] = {0, 0, -1, -1, -1, -1, 0, 0};
    if ((int)blockIdx.x < p.num_wg) {
        const int k = blockIdx.x;
        int total_units, unused;
        unit_sums(p, l, 0, total_units, unused);
        const int active = mla_plan::active_teams(total_units, p.num_wg);
        rec[0] = total_units;
        rec[1] = active;
        if (k < active) {
            mla_plan::unit_range(k, total_units, active, rec[2], rec[3]);
            if (p.batch <= 64) {                       // the same two routes as the split kernel
                const LaneScan s = scan_lengths(p, l, 0, 0);
                locate_in_chunk(p, s, l, 0, 0, rec[2], rec[4], rec[5], rec[6]);
            } else {
                locate_unit(p, l, rec[2], rec[4], rec[5], rec[6]);
            }
        }
    } else {
        const int b = blockIdx.x - p.num_wg;
        unit_sums(p, l, b, rec[0], rec[1]);
        rec[2] = units_at(p, b);
        rec[3] = rec[4] = -1;
        rec[5] = 0;
        if (rec[2] > 0)
            mla_plan::bound_teams(rec[1], rec[2], rec[0], mla_plan::active_teams(rec[0], p.num_wg), rec[3], rec[4]);
    }
    if (l < 8) {
        int v = rec[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) v = l == i ? rec[i] : v;
        table[(long long)blockIdx.x * 8 + l] = v;
    }
}

// ---- host side ---------------------------------------------------------------------------------

static_assert(mla_plan::kMaxQLen == MLA_MAX_Q_LEN && mla_plan::kSlotFloats == kHeads * kDv, "plan header and ABI header disagree");

constexpr int kMaxWorkgroups = 1 << 16;

// Workspace of mla_decode_static(): for callers that cannot allocate.  Sized for the automatic plan
// on up to MLA_STATIC_MAX_WORKGROUPS compute units and MLA_STATIC_MAX_ROWS (sequence, query token)
// rows: 19.2 MB that every GPU the library runs on holds until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress(); kernels get the device address it returns.
constexpr size_t kStaticBytes = (2 * MLA_STATIC_MAX_WORKGROUPS + MLA_STATIC_MAX_ROWS + MLA_MAX_Q_LEN) * (size_t)(kHeads * kDv + kHeads) * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

bool misaligned(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; }

constexpr int kMaxQLen = MLA_MAX_Q_LEN;

int unit_tokens_for(int flags, int batch, int max_seqlen_kv, int teams) {
    return (flags & MLA_UNIT_FINE) ? mla_plan::kUnitFine : (flags & MLA_UNIT_COARSE) ? mla_plan::kUnitCoarse
                                                          : mla_plan::unit_for(batch, max_seqlen_kv, teams);
}

mla_status_t check_shape(int batch, int num_heads, int max_seqlen_kv) {
    if (batch <= 0 || max_seqlen_kv <= 0 || num_heads <= 0) return MLA_ERR_INVALID_ARG;
    if (num_heads != kHeads) return MLA_ERR_UNSUPPORTED_SHAPE;
    // unit counts are summed in 32-bit integers on the device (a 288 GB cache holds < 2^28 tokens)
    if ((long long)batch * max_seqlen_kv > (1ll << 30)) return MLA_ERR_INVALID_ARG;
    if (batch > (1 << 20)) return MLA_ERR_INVALID_ARG;
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
    // scores are kept in fp32: with |scale| <= MLA_MAX_ABS_SCALE they stay finite for any inputs of magnitude
    // below 1e14, so every tile has a finite maximum and the softmax never forms inf - inf
    if (!(std::fabs(scale) <= MLA_MAX_ABS_SCALE)) return MLA_ERR_INVALID_ARG;      // also rejects NaN
    return MLA_OK;
}

// The launch call's own return value says whether THIS launch was accepted; hipGetLastError() would
// also report (and clear) an error left behind by an earlier, unrelated runtime call of the thread.
hipError_t launch_kernel(const void *fn, int blocks, int threads, size_t lds_bytes, hipStream_t stream, const Params &p) {
    Params copy = p;
    void *args[] = {&copy};
    return hipLaunchKernel(fn, dim3(blocks), dim3(threads), args, lds_bytes, stream);
}

long long *timeline_buffer = nullptr;      // set only through mla_timeline_buffer() of the measurement build

// Everything below runs only after validate() passed.
mla_status_t launch(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                    const int32_t *cache_seqlens, int batch, int q_len, int max_seqlen_kv, float scale,
                    float *out, float *lse, void *workspace, size_t workspace_bytes, int num_wg,
                    int flags, int dtype, void *stream) {
    if (num_wg <= 0 || num_wg > kMaxWorkgroups) return MLA_ERR_INVALID_ARG;
    const bool direct_orientation = (flags & MLA_ORIENT_DIRECT) != 0;
    if (direct_orientation && (q_len > 1 || dtype != MLA_DTYPE_BF16)) return MLA_ERR_UNSUPPORTED_SHAPE;
    // the workspace holds one slot per (team, sequence, query token)
    const mla_plan::Spread plan = mla_plan::spread_for(q_len, num_wg, direct_orientation);
    const int teams = plan.teams;
    if (workspace_bytes < mla_plan::workspace_bytes(batch * q_len, num_wg)) return MLA_ERR_WORKSPACE_TOO_SMALL;

    // the main kernel needs more dynamic LDS than the default limit: raise it once per device
    static std::mutex mu;
    static bool attr_done[64][7] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MLA_ERR_HIP;
    typedef void (*kernel_fn)(const Params);
    static const kernel_fn kernels[7] = {
        mla_decode_split_kernel<MLA_DTYPE_BF16, false, false, 1>, mla_decode_split_kernel<MLA_DTYPE_F16, false, false, 1>,
        mla_decode_split_kernel<MLA_DTYPE_BF16, true, false, 2>,  mla_decode_split_kernel<MLA_DTYPE_F16, true, false, 2>,
        mla_decode_split_kernel<MLA_DTYPE_BF16, false, true, 1>,
        mla_decode_split_kernel<MLA_DTYPE_BF16, false, false, 2>, mla_decode_split_kernel<MLA_DTYPE_F16, false, false, 2>};
    // 0, 1: one query token; 2, 3: teams of workgroups with two tokens each; 4: one token, direct
    // orientation; 5, 6: two tokens, one workgroup per team
    const int variant = direct_orientation ? 4 : (plan.share == 1 ? 0 : plan.members > 1 ? 2 : 5) + (dtype == MLA_DTYPE_F16 ? 1 : 0);
    const kernel_fn split_fn = kernels[variant];
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!attr_done[dev][variant]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(split_fn),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
                return MLA_ERR_HIP;
            attr_done[dev][variant] = true;
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
    p.part_lse = p.part_out + ((size_t)teams + batch) * q_len * kHeads * kDv;
    p.batch = batch;
    p.q_len = q_len;
    p.max_seqlen = max_seqlen_kv;
    p.num_wg = teams;
    p.unit = unit_tokens_for(flags, batch, max_seqlen_kv, teams);
    // With a short stream all workgroups finish within a few microseconds of each other and their
    // partial results (32 KB each) are still dirty in the L2 caches when the kernel ends; the merge
    // kernel then starts only after they have been written back (4 us for 256 of them, against 2 us
    // when the workgroups finish apart).  Marked non-temporal, the stores leave for memory as they
    // are issued: batch 16, KV 512 ... 4096: 1.0 us less per call; batch 32, KV 4096: 1.5 us less.
    // With a long stream the same marking costs 1 us (batch 16, KV 16K and 64K), so it is not used there.
    p.stream_out = (long long)batch * ((max_seqlen_kv + mla_plan::kUnitCoarse - 1) / mla_plan::kUnitCoarse) <= 4ll * teams;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.timeline = timeline_buffer;

    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (flags & MLA_PHASE_SPLIT) {
        const int team_stride = plan.members > 1 ? (teams + 7) / 8 * 8 : teams;   // see the kernel: a team behind one L2
        if (launch_kernel(reinterpret_cast<const void *>(split_fn), team_stride * plan.members, kThreads, kLdsBytes, hs, p) != hipSuccess)
            return MLA_ERR_HIP;
    }
    if (flags & MLA_PHASE_COMBINE) {
        // pieces per sequence: about teams / batch, plus the two at its ends
        const int pieces = teams / batch + 2;
        // batch 1 or 2 on 256 workgroups (258 / 130 pieces): 16 groups x 16 slices, 4.5 us less per call at batch 1
        // than 4 x 4; batch 4 (66 pieces) is 0.5 us faster with 4 x 4
        const int width = pieces > 100 ? kCombineWidest : pieces > 16 ? kCombineWide : 1;
        const kernel_fn combine_fn = width == kCombineWidest ? mla_decode_combine_kernel<kCombineWidest, kCombineWidest>
                                     : width == kCombineWide ? mla_decode_combine_kernel<kCombineWide, kCombineWide>
                                                             : mla_decode_combine_kernel<1, 1>;
        if (launch_kernel(reinterpret_cast<const void *>(combine_fn), batch * q_len * kHeads * width, kCombineCols, 0, hs, p) != hipSuccess)
            return MLA_ERR_HIP;
    }
    return MLA_OK;
}

}  // namespace

extern "C" {

// Automatic plan.  One workgroup fills a compute unit (LDS), and a compute unit takes in about
// 58 GB/s at most, so HBM is saturated by well under all of them.  With one query token and a long
// KV stream (more than 8 units of 128 rows per compute unit) the plan is a persistent workgroup on
// 13 of every 16 compute units: measured over the batch 16 / 32, KV 16K ... 64K grid and the
// ragged batch, 176 ... 224 workgroups are within 1 % of each other and 208 is the best or second
// best everywhere, while 256 is 1-2 % slower at the long end (the slowest workgroup gets later).
// With a short stream every compute unit is used, so that each workgroup holds as few units as
// possible (batch 32, KV 2K: 27.9 us on 256 workgroups, 33.1 us on 208).  With several query
// tokens every KV row is worked on q_len times, the kernel is bound by what a compute unit can
// do, and every compute unit is used (batch 16, KV 64K, two tokens: 190.7 us on 256, 199.3 us on 208).
static mla_status_t planned_workgroups(int batch, int q_len, int max_seqlen_kv, int *num_wg, int *num_wg_max) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MLA_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return MLA_ERR_HIP;
    *num_wg = mla_plan::workgroups_for(batch, q_len, max_seqlen_kv, cus);
    if (num_wg_max) *num_wg_max = cus;
    return MLA_OK;
}

mla_status_t mla_decode_workspace_size(int batch, int num_heads, int max_seqlen_kv, int num_workgroups,
                                       size_t *bytes, int *num_workgroups_used) {
    if (!bytes) return MLA_ERR_INVALID_ARG;
    mla_status_t st = check_shape(batch, num_heads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return MLA_ERR_INVALID_ARG;
    int size_for = num_workgroups;
    if (num_workgroups == 0) {        // the size covers the plan for any number of query tokens
        st = planned_workgroups(batch, 1, max_seqlen_kv, &num_workgroups, &size_for);
        if (st != MLA_OK) return st;
    }
    *bytes = mla_plan::workspace_bytes(batch, size_for);
    if (num_workgroups_used) *num_workgroups_used = num_workgroups;
    return MLA_OK;
}

mla_status_t mla_decode_workspace_size_for(int batch, int num_heads, int max_seqlen_kv, int num_compute_units,
                                           size_t *bytes, int *num_workgroups_used) {
    if (!bytes) return MLA_ERR_INVALID_ARG;
    mla_status_t st = check_shape(batch, num_heads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (num_compute_units < 1 || num_compute_units > kMaxWorkgroups) return MLA_ERR_INVALID_ARG;
    *bytes = mla_plan::workspace_bytes(batch, num_compute_units);      // covers the plan for any number of query tokens
    if (num_workgroups_used) *num_workgroups_used = mla_plan::workgroups_for(batch, 1, max_seqlen_kv, num_compute_units);
    return MLA_OK;
}

mla_status_t mla_decode_typed(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                              const int32_t *cache_seqlens, int batch, int q_len, int num_heads,
                              int max_seqlen_kv, int dtype, float scale, float *out, float *lse,
                              void *workspace, size_t workspace_bytes, int num_workgroups, int flags,
                              void *stream) {
    if (dtype != MLA_DTYPE_BF16 && dtype != MLA_DTYPE_F16) return MLA_ERR_INVALID_ARG;
    if (batch <= 0) return MLA_ERR_INVALID_ARG;
    if (q_len < 1 || q_len > kMaxQLen) return MLA_ERR_UNSUPPORTED_SHAPE;
    if (batch > (1 << 20)) return MLA_ERR_INVALID_ARG;
    mla_status_t st = validate(q, kv_cache, kv_batch_stride, cache_seqlens, batch * q_len, num_heads,
                               max_seqlen_kv, scale, out, lse, workspace);
    if (st != MLA_OK) return st;
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return MLA_ERR_INVALID_ARG;
    if ((flags & ~(MLA_PHASE_SPLIT | MLA_PHASE_COMBINE | MLA_ORIENT_DIRECT | MLA_UNIT_FINE | MLA_UNIT_COARSE)) != 0) return MLA_ERR_INVALID_ARG;
    if ((flags & MLA_UNIT_FINE) && (flags & MLA_UNIT_COARSE)) return MLA_ERR_INVALID_ARG;
    if ((flags & (MLA_PHASE_SPLIT | MLA_PHASE_COMBINE)) == 0) return MLA_ERR_INVALID_ARG;
    if (num_workgroups == 0) {
        st = planned_workgroups(batch, q_len, max_seqlen_kv, &num_workgroups, nullptr);
        if (st != MLA_OK) return st;
    }
    return launch(q, kv_cache, kv_batch_stride, cache_seqlens, batch, q_len, max_seqlen_kv, scale, out, lse,
                  workspace, workspace_bytes, num_workgroups, flags, dtype, stream);
}

mla_status_t mla_decode_ex(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                           const int32_t *cache_seqlens, int batch, int num_heads, int max_seqlen_kv,
                           float scale, float *out, float *lse, void *workspace, size_t workspace_bytes,
                           int num_workgroups, int flags, void *stream) {
    return mla_decode_typed(q, kv_cache, kv_batch_stride, cache_seqlens, batch, 1, num_heads, max_seqlen_kv,
                            MLA_DTYPE_BF16, scale, out, lse, workspace, workspace_bytes, num_workgroups, flags,
                            stream);
}

mla_status_t mla_decode(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                        const int32_t *cache_seqlens, int batch, int num_heads, int max_seqlen_kv,
                        float scale, float *out, float *lse, void *workspace, size_t workspace_bytes,
                        void *stream) {
    return mla_decode_ex(q, kv_cache, kv_batch_stride, cache_seqlens, batch, num_heads, max_seqlen_kv, scale,
                         out, lse, workspace, workspace_bytes, 0, MLA_PHASE_SPLIT | MLA_PHASE_COMBINE, stream);
}

mla_status_t mla_decode_static(const void *q, const void *kv_cache, int64_t kv_batch_stride,
                               const int32_t *cache_seqlens, int batch, int q_len, int num_heads,
                               int max_seqlen_kv, int dtype, float scale, float *out, float *lse,
                               void *stream) {
    if (dtype != MLA_DTYPE_BF16 && dtype != MLA_DTYPE_F16) return MLA_ERR_INVALID_ARG;
    if (batch <= 0 || batch > (1 << 20)) return MLA_ERR_INVALID_ARG;
    if (q_len < 1 || q_len > kMaxQLen) return MLA_ERR_UNSUPPORTED_SHAPE;
    // the device address of this GPU's copy of the array, looked up once per device
    static std::mutex mu;
    static void *scratch_ptr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MLA_ERR_HIP;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!scratch_ptr[dev]) {
            void *ptr = nullptr;
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MLA_ERR_HIP;
            scratch_ptr[dev] = ptr;
        }
        ws = scratch_ptr[dev];
    }
    mla_status_t st = validate(q, kv_cache, kv_batch_stride, cache_seqlens, batch * q_len, num_heads,
                               max_seqlen_kv, scale, out, lse, ws);
    if (st != MLA_OK) return st;
    int num_wg = 0;
    st = planned_workgroups(batch, q_len, max_seqlen_kv, &num_wg, nullptr);
    if (st != MLA_OK) return st;
    if (batch * q_len > MLA_STATIC_MAX_ROWS || num_wg > MLA_STATIC_MAX_WORKGROUPS) return MLA_ERR_STATIC_LIMIT;
    return launch(q, kv_cache, kv_batch_stride, cache_seqlens, batch, q_len, max_seqlen_kv, scale, out, lse,
                  ws, kStaticBytes, num_wg, MLA_PHASE_SPLIT | MLA_PHASE_COMBINE, dtype, stream);
}

mla_status_t mla_decode_plan_table(const int32_t *cache_seqlens, int batch, int q_len, int max_seqlen_kv,
                                   int num_workgroups, int flags, int32_t *table, int *teams, int *unit_tokens,
                                   void *stream) {
    if (!cache_seqlens || !table || !teams || !unit_tokens) return MLA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(cache_seqlens) & 3u) || (reinterpret_cast<uintptr_t>(table) & 3u)) return MLA_ERR_INVALID_ARG;
    if (q_len < 1 || q_len > kMaxQLen) return MLA_ERR_UNSUPPORTED_SHAPE;
    mla_status_t st = check_shape(batch, kHeads, max_seqlen_kv);
    if (st != MLA_OK) return st;
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return MLA_ERR_INVALID_ARG;
    if ((flags & ~(MLA_ORIENT_DIRECT | MLA_UNIT_FINE | MLA_UNIT_COARSE)) != 0) return MLA_ERR_INVALID_ARG;
    if ((flags & MLA_UNIT_FINE) && (flags & MLA_UNIT_COARSE)) return MLA_ERR_INVALID_ARG;
    if (num_workgroups == 0) {
        st = planned_workgroups(batch, q_len, max_seqlen_kv, &num_workgroups, nullptr);
        if (st != MLA_OK) return st;
    }
    const mla_plan::Spread plan = mla_plan::spread_for(q_len, num_workgroups, (flags & MLA_ORIENT_DIRECT) != 0);
    Params p = {};
    p.seqlens = cache_seqlens;
    p.batch = batch;
    p.q_len = q_len;
    p.max_seqlen = max_seqlen_kv;
    p.num_wg = plan.teams;
    p.unit = unit_tokens_for(flags, batch, max_seqlen_kv, plan.teams);
    *teams = plan.teams;
    *unit_tokens = p.unit;
    void *args[] = {&p, &table};
    if (hipLaunchKernel(reinterpret_cast<const void *>(mla_decode_plan_kernel), dim3(plan.teams + batch), dim3(64), args, 0,
                        static_cast<hipStream_t>(stream)) != hipSuccess)
        return MLA_ERR_HIP;
    return MLA_OK;
}

mla_status_t mla_decode_planned_workgroups(int batch, int q_len, int max_seqlen_kv, int *num_workgroups) {
    if (!num_workgroups || batch <= 0 || max_seqlen_kv <= 0) return MLA_ERR_INVALID_ARG;
    if (q_len < 1 || q_len > kMaxQLen) return MLA_ERR_UNSUPPORTED_SHAPE;
    return planned_workgroups(batch, q_len, max_seqlen_kv, num_workgroups, nullptr);
}

#ifdef MLA_TIMELINE
// Measurement build only: where the kernels of later calls leave their time stamps (device memory of
// at least 8 MB + 32 bytes per merge block, zeroed by the caller), or NULL to switch them off.
void mla_timeline_buffer(void *device_buffer) { timeline_buffer = static_cast<long long *>(device_buffer); }
#endif

const char *mla_status_string(mla_status_t status) {
    switch (status) {
        case MLA_OK: return "ok";
        case MLA_ERR_INVALID_ARG: return "invalid argument";
        case MLA_ERR_UNSUPPORTED_SHAPE: return "unsupported shape (need 16 heads, d_qk 576, d_v 512, q_len 1 to 8; direct orientation: bf16, q_len 1)";
        case MLA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MLA_ERR_HIP: return "HIP runtime error";
        case MLA_ERR_STATIC_LIMIT: return "too large for the library's static workspace (mla_decode_static: batch * q_len <= 64, <= 256 compute units)";
    }
    return "unknown status";
}

}  // extern "C"
