// The integer plan of the MLA decode library: how the KV rows of a batch are divided over a
// persistent grid of workgroups, which partial-result slot each (workgroup, sequence, query token)
// owns, and which byte offsets a tile's loads touch.  Everything here is pure integer arithmetic on
// plain arguments, usable from host code and from the kernels alike, so that the two kernels, the
// host-side sizing and the CPU tests all evaluate the SAME functions.
//
// The paper has no split over the KV length (Algorithm 1 walks all KV blocks of a sequence in one
// thread block); the split is this library's way of filling 256 compute units from 16 sequences, and
// the merge of its pieces is the m / l recurrence of Algorithm 1 applied across pieces.
//
// Terms.  A *unit* is `unit` consecutive KV rows of one sequence (128, or 32 for short streams); a
// sequence of n rows holds ceil(n / unit) units, the last one possibly partial.  The units of all
// sequences, in batch order, form the *stream* of U units.  A *team* is the set of workgroups that
// stream the same rows (one workgroup, or ceil(q_len / 2) of them with several query tokens); team k
// of A active teams takes stream units [floor(k U / A), floor((k + 1) U / A)).  The part of a team's
// range inside one sequence is a *piece*.
#ifndef MLA_PLAN_H
#define MLA_PLAN_H

#include <stddef.h>

#if defined(__HIPCC__)
#define MLA_PLAN_FN __host__ __device__ inline
#else
#define MLA_PLAN_FN inline
#endif

namespace mla_plan {

constexpr int kRowBytes = 1152;                 // one KV row: 576 16-bit values
constexpr int kTileRows = 32;                   // rows a wavefront stages at a time
constexpr int kTileBytes = kTileRows * kRowBytes;
constexpr int kLoadBytes = 1024;                // one load instruction of a wavefront: 64 lanes x 16 B
constexpr int kTileLoads = kTileBytes / kLoadBytes;   // 36
constexpr int kUnitCoarse = 128;                // one tile for each of a workgroup's four wavefronts
constexpr int kUnitFine = 32;                   // one tile
constexpr int kMaxShare = 2;                    // query tokens one workgroup can take
constexpr int kMaxQLen = 8;
constexpr int kSlotFloats = 16 * 512;           // one partial result: 16 heads x 512 value columns

MLA_PLAN_FN int clamp_len(int n, int max_seqlen) { return n < 0 ? 0 : (n > max_seqlen ? max_seqlen : n); }

MLA_PLAN_FN int units_of(int n, int unit) { return (n + unit - 1) / unit; }

// KV rows that query token j of q_len sees in a sequence of n rows: the new tokens are the last
// q_len rows and attention is causal among them.
MLA_PLAN_FN int visible_len(int n, int q_len, int j) {
    const int v = n - (q_len - 1 - j);
    return v < 0 ? 0 : v;
}

// Never more teams than units: every active team then holds at least one unit.
MLA_PLAN_FN int active_teams(int total_units, int teams) { return total_units < teams ? total_units : teams; }

// Range [floor(k U / A), floor((k + 1) U / A)) of team k < A, A <= 65536, in 32-bit arithmetic: with
// U = q A + r, floor(k U / A) = k q + floor(k r / A), and k r < A^2 fits an unsigned int.  (A 64-bit
// division costs the kernel's start several hundred nanoseconds.)
MLA_PLAN_FN void unit_range(int k, int total_units, int active, int &lo, int &hi) {
    const unsigned A = (unsigned)active, q = (unsigned)total_units / A, r = (unsigned)total_units % A;
    lo = (int)((unsigned)k * q + (unsigned)k * r / A);
    hi = (int)((unsigned)(k + 1) * q + (unsigned)(k + 1) * r / A);
}

// Teams bound to the sequence that owns stream units [seq_first, seq_first + ub), ub > 0: team k is
// bound iff its range [floor(k U / A), floor((k+1) U / A)) meets that interval, which gives
//   first = ceil((seq_first + 1) A / U) - 1,   last = ceil((seq_first + ub) A / U) - 1.
MLA_PLAN_FN void bound_teams(int seq_first, int ub, int total_units, int active, int &first, int &last) {
    const long long U = total_units, A = active;
    first = (int)((((long long)seq_first + 1) * A + U - 1) / U) - 1;
    last = (int)((((long long)seq_first + ub) * A + U - 1) / U) - 1;
}

// The sequence that holds stream unit `target` (0 <= target < total units) and the stream index of
// that sequence's first unit: the definition, evaluated serially.  (The kernels evaluate the same rule
// with a wavefront-wide scan; the two are compared on the device through mla_decode_plan_table().)
MLA_PLAN_FN void locate_unit_serial(const int *lens, int batch, int max_seqlen, int unit, int target, int &b, int &first) {
    int start = 0;
    b = 0;
    for (int i = 0; i < batch; ++i) {
        const int u = units_of(clamp_len(lens[i], max_seqlen), unit);
        if (start + u > target) break;
        start += u;
        b = i + 1;
    }
    first = start;
}

// The next sequence at or after b that holds at least one unit.  Only called while units of the
// team's range remain, so such a sequence exists before the end of the batch.
MLA_PLAN_FN int next_nonempty(const int *lens, int b, int max_seqlen, int unit) {
    while (units_of(clamp_len(lens[b], max_seqlen), unit) == 0) ++b;
    return b;
}

// Partial-result slot of (team k, sequence b, query token j).  A team's sequences are consecutive
// and so are a sequence's teams, so k + b is different for every (team, sequence) pair that occurs.
MLA_PLAN_FN long long slot_of(int k, int b, int q_len, int j) { return ((long long)k + b) * q_len + j; }

// One piece, as one wavefront sees it.
struct Piece {
    int t_begin;     // first row of the piece
    int t_end;       // end of the rows this wavefront's query token sees inside the piece (may be <= t_begin)
    int n_tiles;     // tiles of 32 rows the workgroup stages for the piece (what its last token sees)
    bool whole;      // the piece is the whole sequence: the result goes straight to out / lse
};

// The piece of the sequence of n rows (ub = units_of(n) > 0, first stream unit seq_first) that starts
// at stream unit first_unit inside a team's range ending at u_hi.  j: the wavefront's query token,
// j_last: the last query token of the wavefront's workgroup (both < q_len), has_token: j is real.
MLA_PLAN_FN Piece piece_of(int n, int ub, int seq_first, int first_unit, int u_hi, int unit, int q_len, int j,
                           int j_last, bool has_token) {
    Piece pc;
    const int u_begin = first_unit - seq_first;
    const int u_end = (u_hi - seq_first < ub) ? u_hi - seq_first : ub;      // > u_begin
    const int row_end = u_end * unit;
    pc.t_begin = u_begin * unit;
    const int vis = visible_len(n, q_len, j);
    pc.t_end = has_token ? (vis < row_end ? vis : row_end) : 0;
    const int vis_last = visible_len(n, q_len, j_last);
    const int stage_end = vis_last < row_end ? vis_last : row_end;
    pc.n_tiles = stage_end > pc.t_begin ? (stage_end - pc.t_begin + kTileRows - 1) / kTileRows : 0;
    pc.whole = (u_begin == 0 && u_end == ub);
    return pc;
}

// Loads of the tile that starts at row tb of a sequence of n rows (tb < n): load i of lane l reads
// 16 bytes at row-tb-relative offset piece_offset(i, last) + lane_offset(16 l, last, piece), where
// last = last_chunk_offset(min(n - tb, 32)).  Offsets are clamped to the tile's last valid 16-byte
// chunk, so no byte at or past row n is ever addressed.
MLA_PLAN_FN int last_chunk_offset(int valid_rows) { return (valid_rows * (kRowBytes / 16) - 1) * 16; }
MLA_PLAN_FN int piece_offset(int i, int last) { return i * kLoadBytes < last ? i * kLoadBytes : last; }
MLA_PLAN_FN unsigned lane_offset(unsigned lane16, int last, int piece) {
    const unsigned room = (unsigned)(last - piece);
    return lane16 < room ? lane16 : room;
}

// ---- host-side plan -------------------------------------------------------------------------

// How q_len query tokens are spread: `share` tokens per workgroup, `members` workgroups per team,
// `teams` ranges of the unit stream.
struct Spread {
    int share, members, teams;
};

MLA_PLAN_FN Spread spread_for(int q_len, int num_wg, bool direct_orientation) {
    Spread s;
    s.share = (q_len >= 2 && !direct_orientation) ? 2 : 1;
    s.members = (q_len + s.share - 1) / s.share;
    s.teams = num_wg / s.members > 0 ? num_wg / s.members : 1;
    return s;
}

// One partial slot per (team, sequence, query token) that can occur: (teams + sequences) x q_len.
// `rows` counts sequences x tokens.  A workgroup takes at most kMaxShare tokens, so
// teams x q_len <= kMaxShare x num_wg, or q_len (one team) if that is larger.
MLA_PLAN_FN size_t workspace_slots(int rows, int num_wg) {
    return (size_t)kMaxShare * (size_t)num_wg + (size_t)rows + kMaxQLen;
}

MLA_PLAN_FN size_t workspace_bytes(int rows, int num_wg) {
    const size_t slots = workspace_slots(rows, num_wg);
    const size_t po = slots * kSlotFloats * sizeof(float);
    const size_t pl = slots * 16 * sizeof(float);
    return po + ((pl + 15) & ~(size_t)15);
}

// The unit: 128 rows (one tile for each wavefront of a workgroup), or 32 rows (one tile) for a tiny
// batch: one whose tiles number at most a quarter of the workgroups.  Such a batch then spreads over
// four times as many compute units, each of which takes in a quarter as much before its first product
// (batch 1, KV 512 and 1024: 1.7 us less per call).  Beyond that size the finer unit only multiplies
// the partial results to merge (batch 1, KV 8192: 4.7 us more per call with 256 tiles than with 64 units).
MLA_PLAN_FN int unit_for(int batch, int max_seqlen, int num_wg) {
    const long long tiles = (long long)batch * ((max_seqlen + kUnitFine - 1) / kUnitFine);
    return 4 * tiles <= num_wg ? kUnitFine : kUnitCoarse;
}

// Workgroups of the automatic plan on a device of `cus` compute units: 13 of every 16 for one query
// token and a long stream (more than 8 coarse units per compute unit), every one otherwise.
MLA_PLAN_FN int workgroups_for(int batch, int q_len, int max_seqlen, int cus) {
    const long long coarse = (long long)batch * ((max_seqlen + kUnitCoarse - 1) / kUnitCoarse);
    const int n = (q_len > 1 || coarse <= 8ll * cus) ? cus : cus * 13 / 16;
    return n < 1 ? 1 : n;
}

}  // namespace mla_plan

#endif  // MLA_PLAN_H
