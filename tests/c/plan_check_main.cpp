/*
 * Exhaustive host check of the integer plan in paper_2506_01969_amd/csrc/mla_plan.h, the same functions
 * the two kernels and the host-side sizing evaluate (tests/test_plan_host.py builds this file under
 * -fsanitize=address,undefined and runs it).  For thousands of seeded cases -- lengths with zeros,
 * exact multiples of the unit and values beyond max_seqlen, more than 64 sequences, 1 to 8 query
 * tokens, 1 to 1000 workgroups, both units, both orientations -- it walks every team's range piece by
 * piece the way the split kernel does and checks:
 *   - every unit of the stream is taken by exactly one team, and every row below a token's causal
 *     limit is handed to that token by exactly one piece, inside the tiles the piece stages;
 *   - the teams the combine kernel derives for a sequence (bound_teams) are exactly the teams whose
 *     range meets the sequence, and a piece is marked whole iff it is the sequence's only piece;
 *   - every (team, sequence, token) slot is unique and lies inside the workspace the size query
 *     returns, partial log-sum-exps included;
 *   - every byte a tile load, a refill or the idle refill addresses lies inside rows [0, n) of its
 *     sequence, every q / out row index inside the batch, and the scan for the next non-empty
 *     sequence stops inside the batch.
 * The lengths live in an array of exactly `batch` ints, so a read past it trips AddressSanitizer.
 */
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <vector>

#include "mla_plan.h"

using namespace mla_plan;

static unsigned long long rng_state = 88172645463325252ull;
static unsigned rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (unsigned)(rng_state >> 16);
}
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (unsigned)(hi - lo + 1)); }

#define CHECK(cond)                                                                            \
    do {                                                                                       \
        if (!(cond)) {                                                                         \
            std::printf("FAILED %s (line %d) case %d: batch %d q_len %d G %d unit %d\n", #cond, __LINE__, \
                        case_id, batch, q_len, num_wg, unit);                                  \
            std::exit(1);                                                                      \
        }                                                                                      \
    } while (0)

static long long checked_loads = 0;

// every byte the 36 loads of the tile at row tb touch lies in [0, n * 1152)
static bool tile_loads_in_bounds(int n, int tb) {
    if (tb < 0 || tb >= n) return false;
    const int valid = n - tb < kTileRows ? n - tb : kTileRows;
    const int last = last_chunk_offset(valid);
    for (int i = 0; i < kTileLoads; ++i) {
        const int piece = piece_offset(i, last);
        for (unsigned lane = 0; lane < 64; ++lane) {
            const long long off = (long long)tb * kRowBytes + piece + lane_offset(lane * 16, last, piece);
            if (off < 0 || off + 16 > (long long)n * kRowBytes) return false;
            ++checked_loads;
        }
    }
    return true;
}

static void run_case(int case_id, int batch, int max_seqlen, const std::vector<int> &raw_lens, int q_len, int num_wg,
                     int unit, bool direct_orientation) {
    int *lens = (int *)std::malloc(sizeof(int) * batch);       // exactly batch entries
    for (int i = 0; i < batch; ++i) lens[i] = raw_lens[i];
    std::vector<int> n_of(batch), ub_of(batch), first_of(batch);
    int U = 0;
    for (int i = 0; i < batch; ++i) {
        n_of[i] = clamp_len(lens[i], max_seqlen);
        CHECK(n_of[i] >= 0 && n_of[i] <= max_seqlen);
        ub_of[i] = units_of(n_of[i], unit);
        CHECK((long long)ub_of[i] * unit >= n_of[i] && (long long)(ub_of[i] - 1) * unit < n_of[i] + (n_of[i] == 0));
        first_of[i] = U;
        U += ub_of[i];
    }
    const Spread sp = spread_for(q_len, num_wg, direct_orientation);
    CHECK(sp.share >= 1 && sp.share <= kMaxShare && sp.members * sp.share >= q_len && sp.teams >= 1);
    CHECK((long long)sp.teams * sp.members <= num_wg || sp.teams == 1);
    const int teams = sp.teams;
    const int A = active_teams(U, teams);
    const size_t ws_bytes = workspace_bytes(batch * q_len, num_wg);
    // the library places the partial log-sum-exps after (teams + batch) * q_len partial results
    const long long slots_laid_out = ((long long)teams + batch) * q_len;
    CHECK((size_t)slots_laid_out * (kSlotFloats + 16) * sizeof(float) <= ws_bytes);

    std::vector<int> unit_taken(U, 0);
    std::map<int, std::set<int>> teams_of_seq;
    std::set<long long> slots;
    std::vector<long long> rows_seen(batch * kMaxQLen, 0);    // per (sequence, token): rows its pieces hand to it
    std::map<int, int> whole_pieces;

    int prev_hi = 0;
    for (int k = 0; k < A; ++k) {
        int u_lo, u_hi;
        unit_range(k, U, A, u_lo, u_hi);
        CHECK(u_lo == prev_hi && u_hi > u_lo && u_hi <= U);
        CHECK(u_lo == (int)((long long)k * U / A) && u_hi == (int)((long long)(k + 1) * U / A));   // the 32-bit form is exact
        prev_hi = u_hi;
        int b, seq_first;
        locate_unit_serial(lens, batch, max_seqlen, unit, u_lo, b, seq_first);
        CHECK(b >= 0 && b < batch && seq_first == first_of[b] && ub_of[b] > 0 && u_lo < first_of[b] + ub_of[b]);
        int first_unit = u_lo;
        while (true) {
            const int n = n_of[b], ub = ub_of[b];
            CHECK(ub > 0 && first_unit >= seq_first && first_unit < seq_first + ub);
            teams_of_seq[b].insert(k);
            const int u_end_stream = u_hi < seq_first + ub ? u_hi : seq_first + ub;
            for (int u = first_unit; u < u_end_stream; ++u) ++unit_taken[u];
            // every member workgroup of the team and every wavefront role in it
            for (int jt = 0; jt < sp.members; ++jt) {
                const int j_last = (jt * sp.share + sp.share - 1 < q_len - 1) ? jt * sp.share + sp.share - 1 : q_len - 1;
                for (int tk = 0; tk < sp.share; ++tk) {
                    const int j = jt * sp.share + tk;
                    const bool has_token = j < q_len;
                    const Piece pc = piece_of(n, ub, seq_first, first_unit, u_hi, unit, q_len, has_token ? j : q_len - 1, j_last, has_token);
                    CHECK(pc.t_begin == (first_unit - seq_first) * unit && pc.t_begin < n);
                    CHECK(pc.whole == (first_unit == seq_first && u_hi >= seq_first + ub));
                    CHECK(pc.t_end <= n && (!has_token ? pc.t_end == 0 : true));
                    // rows of q, out and lse: inside the batch
                    const long long row = (long long)b * q_len + (has_token ? j : q_len - 1);
                    CHECK(row >= 0 && row < (long long)batch * q_len);
                    if (has_token) {
                        const long long slot = slot_of(k, b, q_len, j);
                        CHECK(slot >= 0 && slot < slots_laid_out);
                        CHECK(slots.insert(slot).second);                       // unique
                        if (pc.whole) ++whole_pieces[b * kMaxQLen + j];
                    }
                    // staged tiles: all inside [0, n), the first and last of them and a few between are
                    // checked load by load; the token's visible rows of this piece are all covered
                    CHECK(pc.n_tiles >= 0);
                    if (pc.n_tiles > 0) {
                        CHECK(pc.t_begin + (pc.n_tiles - 1) * kTileRows < n);
                        const int probes[5] = {0, pc.n_tiles - 1, pc.n_tiles / 2, 1 % pc.n_tiles, rnd_in(0, pc.n_tiles - 1)};
                        for (int t : probes) CHECK(tile_loads_in_bounds(n, pc.t_begin + t * kTileRows));
                    }
                    CHECK(pc.t_end <= pc.t_begin + pc.n_tiles * kTileRows || pc.t_end <= pc.t_begin);
                    if (has_token && pc.t_end > pc.t_begin) rows_seen[b * kMaxQLen + j] += pc.t_end - pc.t_begin;
                }
            }
            // the refill after the last tile of a wavefront reads the sequence's first 1024 bytes
            CHECK(n >= 1 && 1008 + 16 <= (long long)n * kRowBytes);
            const bool more = seq_first + ub < u_hi;
            if (!more) break;
            first_unit = seq_first + ub;
            seq_first = first_unit;
            b = next_nonempty(lens, b + 1, max_seqlen, unit);                  // ASan: must stay inside lens[]
            CHECK(b < batch && first_of[b] == seq_first);
        }
    }
    CHECK(A == 0 ? U == 0 : prev_hi == U);
    for (int u = 0; u < U; ++u) CHECK(unit_taken[u] == 1);
    // the pieces of a sequence are disjoint (each unit is taken once), so a token sees every row below
    // its causal limit exactly once iff the rows its pieces hand to it add up to that limit
    for (int i = 0; i < batch; ++i)
        for (int j = 0; j < q_len; ++j) CHECK(rows_seen[i * kMaxQLen + j] == visible_len(n_of[i], q_len, j));
    for (int i = 0; i < batch; ++i) {
        if (ub_of[i] == 0) {
            CHECK(teams_of_seq.count(i) == 0);
            continue;
        }
        int k_first, k_last;
        bound_teams(first_of[i], ub_of[i], U, A, k_first, k_last);
        const std::set<int> &got = teams_of_seq[i];
        CHECK(k_first >= 0 && k_last < A && k_first <= k_last);
        CHECK((int)got.size() == k_last - k_first + 1 && *got.begin() == k_first && *got.rbegin() == k_last);
        // the combine kernel returns at once iff one team holds the sequence; then that piece was whole
        for (int j = 0; j < q_len; ++j) CHECK((whole_pieces.count(i * kMaxQLen + j) ? whole_pieces[i * kMaxQLen + j] : 0) == (k_first == k_last ? 1 : 0));
        // slots the combine kernel reads for this row: first_slot + s * q_len, s < pieces
        for (int j = 0; j < q_len; ++j)
            for (int s = 0; s <= k_last - k_first; ++s) CHECK(slots.count(slot_of(k_first, i, q_len, j) + (long long)s * q_len) == 1);
    }
    std::free(lens);
}

int main() {
    int cases = 0;
    for (int case_id = 0; case_id < 6000; ++case_id) {
        const int batch = case_id % 7 == 0 ? rnd_in(65, 200) : rnd_in(1, 40);
        const int max_choices[6] = {1, 33, 130, 700, 4096, 20000};
        const int max_seqlen = max_choices[rnd() % 6];
        const int unit = case_id % 2 ? kUnitFine : kUnitCoarse;
        std::vector<int> lens(batch);
        for (int i = 0; i < batch; ++i) {
            const unsigned kind = rnd() % 10;
            if (kind == 0) lens[i] = 0;
            else if (kind == 1) lens[i] = max_seqlen;
            else if (kind == 2) lens[i] = (rnd_in(0, max_seqlen) / unit) * unit;       // exact multiples of the unit
            else if (kind == 3) lens[i] = max_seqlen + rnd_in(1, 1000);                 // clamped on the device
            else if (kind == 4) lens[i] = -rnd_in(1, 5);                                // clamped to 0
            else lens[i] = rnd_in(0, max_seqlen);
        }
        if (case_id % 11 == 0)
            for (int i = 0; i < batch; ++i) lens[i] = 0;                                // nothing at all
        const int q_len = case_id % 3 == 0 ? rnd_in(2, kMaxQLen) : 1;
        const int wg_choices[8] = {1, 2, 3, rnd_in(4, 16), rnd_in(17, 100), 208, 256, rnd_in(257, 1000)};
        const int num_wg = wg_choices[rnd() % 8];
        run_case(case_id, batch, max_seqlen, lens, q_len, num_wg, unit, q_len == 1 && case_id % 5 == 0);
        ++cases;
    }
    // the automatic plan and the unit rule
    int bad = 0;
    bad += workgroups_for(16, 1, 65536, 256) != 208;
    bad += workgroups_for(16, 1, 4096, 256) != 256;
    bad += workgroups_for(16, 2, 65536, 256) != 256;
    bad += workgroups_for(1, 1, 1, 1) != 1;
    bad += unit_for(1, 512, 256) != kUnitFine;          // 16 tiles for 256 workgroups
    bad += unit_for(1, 2048, 256) != kUnitFine;         // 64 tiles
    bad += unit_for(1, 2049, 256) != kUnitCoarse;
    bad += unit_for(16, 512, 256) != kUnitCoarse;       // 256 tiles
    bad += unit_for(16, 65536, 208) != kUnitCoarse;
    if (bad) {
        std::printf("FAILED automatic plan / unit rule (%d)\n", bad);
        return 1;
    }
    std::printf("ok %d cases %lld loads\n", cases, checked_loads);
    return 0;
}
