// Batched dynamic program for the constrained layer-wise compression problem on gfx950.
//
// Sec. 3.2 (Eq. 2-3) and App. A (Alg. 1) define the computation; include/spdy_dp.h states the
// arithmetic contract (fp32, one add per update, smallest level / smallest t win ties).
//
// Mapping.  Alg. 1's triple loop (layer, level, time) is a min-plus recurrence with no reuse of a
// D_{l-1} element across levels (every level shifts the row by a different tau), so there is no
// contraction to put on the matrix cores: the work per (l, s, t) is one LDS read, one fp32 add
// and a min (plus a compare and a select when the level itself is tracked).  The remark after
// Alg. 1 (vectorise over t by shifting the row) is what the lanes do here:
//   * a prepare kernel subtracts each layer's smallest time from the layer and from the budget
//     (rows shrink to B - M + 1 buckets), bounds the reachable part of each row and fixes the
//     order in which the levels of a layer are visited;
//   * the row of D of a candidate stays in LDS for the whole solve, with a +inf apron of one
//     group width on its left, so a level whose shift falls inside a group of buckets needs no
//     per-lane bounds test; levels whose shift lies beyond the group are never visited;
//   * the time axis is cut into chunks of 64 buckets; a wave keeps a group of R chunks in
//     registers (running minimum, and the level when tracked) and sweeps the layer once; lane i
//     holds the i-th entry of the layer (a level, or with the D record all levels of one shift,
//     which one update serves), ballots find the applicable entries and v_readlane moves shift
//     and error to scalar registers, so the sweep issues no memory instruction besides the LDS
//     reads;
//   * when D itself is recorded and a layer has at most 64 levels, a lane takes four consecutive
//     buckets and reads them with one aligned ds_read_b128 (twice the LDS bytes per clock of
//     narrower reads on this chip); the words a shift that is not a multiple of four needs from
//     the quad below come from the lane to the left through a DPP operand of the add.  Otherwise
//     lane i works on bucket 64*c + i of a chunk: every ds_read_b32 of the shifted row touches
//     64 consecutive dwords (conflict-free for any shift);
//   * the waves of a workgroup are split at run time into teams, one candidate per team, so
//     that each wave owns as many chunks as its registers hold whatever the reduced row length
//     is; when every wave holds all its chunks of the row in registers the row is updated in
//     place (one row per candidate), otherwise two rows alternate;
//   * two workgroups of eight waves share a compute unit, and in a launch of one or two rounds
//     of workgroups they take turns at the instruction priority, so that neither runs on the
//     other's leftovers and then alone;
//   * a compute unit wants about sixteen waves of this loop, each with a long group.  Where the
//     usual shape does not give that, a D-record workgroup has sixteen waves: with no more
//     candidates than compute units the second eight divide each layer's ENTRIES with the first
//     eight on the same chunks; a row too long for eight waves' registers is updated in place by
//     sixteen waves with up to the whole LDS of the unit.
// A row that is longer still lives in global memory (two alternating rows per candidate) and is
// computed tile by tile, the part of the previous row a tile reads being staged in LDS first.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include <mutex>

#include "spdy_dp.h"

// Workspace of spdy_dp_solve_batched_static: device memory that belongs to the loaded code
// object, so the entry point never allocates.  In host code this name is only a handle for
// hipGetSymbolAddress; the address the kernels get is looked up once per device.
static __device__ __align__(256) unsigned char scratch[SPDY_DP_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kWave = 64;            // lanes per wavefront = buckets per chunk
// The fill kernel's shape per record variant.  D record: 8 waves of up to 128 registers, each
// keeping up to 26 chunks of a row (two workgroups, 16 waves, per compute unit): long sweeps
// between the barriers of a layer.  Level record: 16 waves of up to 64 registers with up to 10
// chunks each (value and level per chunk).
constexpr int kMaxGroup = 26;        // most chunks a wave keeps in registers at once (D record)
constexpr int kMaxGroupLevel = 10;   // same when the level is tracked too
// In the instantiation for small batches (kTurns) a wave keeps up to 28: a row of 105 - 112
// chunks (the paper's own sizes, T = 10^4) then still splits into two teams of four waves.  The
// other instantiation stays at 26: with 28 its inner loops are the same instruction for
// instruction, but stress_k256 ran 5 % slower (code placement), and long launches gain nothing.
constexpr int kMaxGroupTurns = 28;
template <bool kLevel, bool kTurns> constexpr int group_limit()
{
    return kLevel ? kMaxGroupLevel : (kTurns ? kMaxGroupTurns : kMaxGroup);
}
constexpr int kFillWaves = 8;        // waves of a fill workgroup (D record)
constexpr int kFillWavesLevel = 16;  // (level record)
constexpr int kMaxFillWaves = 16;
template <bool kLevel> constexpr int fill_waves() { return kLevel ? kFillWavesLevel : kFillWaves; }
constexpr int kPriorityTurn = 13;    // log2 of the 100 MHz ticks a workgroup keeps the priority
constexpr int kWalkThreads = 256;    // D-record walk back: 4 waves = 4 candidates per workgroup
constexpr int kLdsStatic = 8192 + 256;    // the fill kernel's static LDS (entry tables, argmin)
constexpr int kLdsBytes = 160 * 1024 - kLdsStatic;       // dynamic LDS a workgroup can get
constexpr int kLdsHalf = 80 * 1024 - kLdsStatic;         // lets two workgroups share a compute unit
// +inf apron left of every row: a group's width, plus one chunk because the 128-bit reads of the
// sweep start one lane (four buckets) below the group
constexpr int kHalo = kMaxGroupTurns * kWave + kWave;
// The longest row the waves of a workgroup can hold in registers (and so update in place), with
// its apron, fits the smaller LDS allocation for either record, and two rows that are any longer
// do not: the in-place case and the launch with the smaller allocation coincide.
constexpr bool kInPlaceFits =
    (kFillWaves * kMaxGroupTurns * kWave + kHalo) * 4 <= kLdsHalf &&
    (kFillWavesLevel * kMaxGroupLevel * kWave + kHalo) * 4 <= kLdsHalf &&
    2 * (kFillWaves * kMaxGroup * kWave + kWave + kHalo) * 4 > kLdsHalf &&
    2 * (kFillWavesLevel * kMaxGroupLevel * kWave + kWave + kHalo) * 4 > kLdsHalf;
static_assert(kInPlaceFits, "path 1 must be exactly the in-place case");
constexpr int kBatch = 8;                 // level tables are padded to a multiple of this
constexpr unsigned kNoLevel = 0xFF;
constexpr size_t kAlign = 256;
constexpr int kMetaHeader = 20;      // int32 words before the per-layer arrays
// meta: header | m_l [L] | chunks of row l [L] | chunk boundaries of the team waves [L][stride]
//       | largest usable shift of layer l [L]
constexpr int kRangeStride = kMaxFillWaves + 1;

// kMetaPath: 0 = rows in global memory, 1 / 2 = rows in LDS, fill kernel launched with the
// smaller / larger LDS allocation, 3 = one row in LDS updated in place by a workgroup of twice
// the waves that has a compute unit's LDS to itself (D record; rows too long for path 1),
// 4 = rows in global memory, a workgroup of twice the waves (D record).
// kMetaTeamWaves x kMetaTeams <= waves of a fill workgroup.
// kMetaInPlace: every wave of a team holds all its chunks of a row in registers, so one row per
// candidate suffices (written back between two barriers); otherwise two rows alternate.
enum MetaWord {
    kMetaBudget = 0, kMetaMinTime = 1, kMetaRow = 2, kMetaPath = 3, kMetaTeamWaves = 4,
    kMetaTeams = 5, kMetaInPlace = 6,
    kMetaStage = 7,     // bytes of LDS the global-row launch has for the windows of its tiles
    // what the choice of the path was made from (read back by tests, not by the kernels)
    kMetaWaves = 8,     // waves of a fill workgroup
    kMetaMaxGroup = 9,  // most chunks a wave keeps in registers
    kMetaLdsSmall = 10, // dynamic LDS bytes of the in-place launch
    kMetaLdsLarge = 11, // dynamic LDS bytes of the two-row launch (0: not enqueued)
    kMetaHalo = 12,     // floats of the +inf apron left of a row
    kMetaSplit = 13,    // 1: the in-place launch has twice kMetaWaves waves (see dp_fill, kSplit)
    kMetaWideWaves = 14, // waves of the wide in-place launch (0: not enqueued)
    kMetaWideGroup = 15, // most chunks one of its waves keeps in registers
    kMetaLdsWide = 16,   // its dynamic LDS bytes
    kMetaGlobalWaves = 17 // waves of the global-row launch
};

enum Variant { kValueRecord = 0, kLevelRecord = 1 };

// ---------------------------------------------------------------------------------------------
// Workspace layout (host side, shared by every entry point)
struct Layout {
    int status;
    int variant;
    size_t row;          // buckets per padded row for the full budget (multiple of 64)
    bool may_spill;      // rows of the full budget may exceed LDS: the global-row launch is needed
    size_t s8;           // levels per layer padded to a multiple of kBatch
    size_t meta_off;     // int32 meta[kMetaHeader + (3 + kRangeStride) L]
    size_t shifts_off;   // int32 shifts[L][s8]: tau - m_l of the r-th visited entry
    size_t order_off;    // int32 order[L][s8]: level index at position r of the visiting order
    size_t start_off;    // int32 start[L][s8 + kBatch]: first position of entry r (D record)
    size_t entry_off;    // int32 entry[L][s8]: the entry that level s belongs to (D record)
    size_t tstar_off;    // int32 tstar[K]
    size_t record_off;   // float D[K][L][row]  or  uint8 P[K][L][row]
    size_t rows_value;   // float rows[K][2][kHalo + row] after the record, when may_spill
    size_t rows_level;
    size_t total_value;  // bytes needed by the D-record variant
    size_t total_level;  // bytes needed by the level-record variant
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// `workspace_bytes` selects the variant; pass SIZE_MAX to get the sizes only.  `rec_rows`: rows
// of the record per candidate (L, or fewer for the solve with checkpoints).
Layout make_layout(int K, int L, int S, int B, size_t workspace_bytes, long long rec_rows = -1)
{
    Layout lay{};
    if (K <= 0 || L <= 0 || S <= 0 || B < 0) {
        lay.status = SPDY_DP_ERR_DIM;
        return lay;
    }
    if (S > 255) {
        lay.status = SPDY_DP_ERR_LEVELS;
        return lay;
    }
    if (B > INT32_MAX - 2 * kWave * kMaxGroupTurns) {   // bucket indices are int32 on the device
        lay.status = SPDY_DP_ERR_OVERFLOW;
        return lay;
    }
    lay.row = align_up((size_t)B + 1, kWave);
    const unsigned __int128 cells = (unsigned __int128)K * ((unsigned __int128)L + 2) *
                                    (lay.row + kHalo);
    if (cells * sizeof(float) + (unsigned __int128)K * 16 + (unsigned __int128)L * 4096 >
        (unsigned __int128)1 << 62) {
        lay.status = SPDY_DP_ERR_OVERFLOW;
        return lay;
    }
    const size_t row_bytes = (lay.row + kHalo) * sizeof(float);
    lay.may_spill = 2 * row_bytes > (size_t)kLdsBytes;
    lay.s8 = align_up((size_t)S, kBatch);
    lay.meta_off = 0;
    lay.shifts_off =
        align_up((kMetaHeader + (3 + (size_t)kRangeStride) * L) * sizeof(int32_t), kAlign);
    lay.order_off = align_up(lay.shifts_off + (size_t)L * lay.s8 * sizeof(int32_t), kAlign);
    lay.start_off = align_up(lay.order_off + (size_t)L * lay.s8 * sizeof(int32_t), kAlign);
    lay.entry_off =
        align_up(lay.start_off + (size_t)L * (lay.s8 + kBatch) * sizeof(int32_t), kAlign);
    lay.tstar_off = align_up(lay.entry_off + (size_t)L * lay.s8 * sizeof(int32_t), kAlign);
    lay.record_off = align_up(lay.tstar_off + (size_t)K * sizeof(int32_t), kAlign);
    const size_t rows = lay.may_spill ? 2 * (size_t)K * row_bytes : 0;
    const size_t nrec = rec_rows < 0 ? (size_t)L : (size_t)rec_rows;
    lay.rows_value = align_up(lay.record_off + (size_t)K * nrec * lay.row * sizeof(float), kAlign);
    lay.rows_level = align_up(lay.record_off + (size_t)K * nrec * lay.row, kAlign);
    lay.total_value = lay.rows_value + rows;
    lay.total_level = lay.rows_level + rows;
    if (workspace_bytes >= lay.total_value)
        lay.variant = kValueRecord;
    else if (workspace_bytes >= lay.total_level)
        lay.variant = kLevelRecord;
    else {
        lay.status = SPDY_DP_ERR_WORKSPACE;
        return lay;
    }
    lay.status = SPDY_DP_OK;
    return lay;
}

// ---------------------------------------------------------------------------------------------
// Sum of `v` over a workgroup of 256 threads (returned to every thread); if `exclusive` is given
// it receives the sum over the threads before this one.  part: 8 words of LDS.
__device__ __forceinline__ long long block_scan_256(long long v, long long *part,
                                                    long long *exclusive)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    long long incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const long long o = __shfl_up(incl, off, kWave);
        if (lane >= off)
            incl += o;
    }
    __syncthreads();                              // part may still be read from a previous call
    if (lane == kWave - 1)
        part[wave] = incl;
    __syncthreads();
    long long before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const long long p = part[w];
        before += w < wave ? p : 0;
        total += p;
    }
    if (exclusive)
        *exclusive = before + incl - v;
    return total;
}

// Prepare, workgroup 0: per-layer smallest time m_l, M = sum m_l, reduced budget B - M, and how
// many 64-bucket chunks of each reduced row can hold a finite value (the largest reachable
// reduced time after layer l is sum_{j<=l} max_s (tau[j][s] - m_j) over the levels that fit the
// reduced budget).  It also picks the path: which launch of the fill kernel (LDS allocation
// lds_small or lds_large bytes, `waves` waves per workgroup) fits, into how many teams its waves
// split, and whether one row per candidate is enough; and it records each layer's largest usable
// shift (the tiles of the global-row path size their window in LDS by it).  Thread i owns a slice
// of layers.
__device__ void prepare_budget(const int32_t *__restrict__ tau, int K, int slots, int L, int S,
                               int B, int waves, int max_group, int lds_small, int lds_large,
                               int lds_stage, int split, int wide_waves, int wide_group,
                               int lds_wide, int global_waves, int32_t *__restrict__ meta)
{
    __shared__ long long s_sum[8];
    __shared__ int s_budget, s_team_waves;
    const int tid = threadIdx.x;
    int32_t *mn = meta + kMetaHeader;
    int32_t *nact = meta + kMetaHeader + L;
    const int per = (L + 255) / 256;
    const int l0 = min(L, tid * per), l1 = min(L, l0 + per);

    long long local = 0;
    for (int l = l0; l < l1; ++l) {
        const int32_t *tau_l = tau + (size_t)l * S;
        int m = INT32_MAX;
        for (int s0 = 0; s0 < S; s0 += 8) {       // eight loads in flight per round trip
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = tau_l[min(s0 + i, S - 1)];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                m = min(m, v[i]);
        }
        mn[l] = m;
        local += m;
    }
    const long long M = block_scan_256(local, s_sum, nullptr);
    if (tid == 0) {
        const int bp = (M > B) ? -1 : (int)(B - M);
        const int rowp = bp < 0 ? 0 : (bp + kWave) / kWave * kWave;
        meta[kMetaBudget] = bp;
        meta[kMetaMinTime] = M > INT32_MAX ? INT32_MAX : (int)M;
        meta[kMetaRow] = rowp;
        int path = 1, teams = 1, inplace = 0;     // an infeasible table is reported by path 1
        int plan_waves = waves;                   // waves of the launch that does the work
        if (bp >= 0) {
            const long long one_row = ((long long)rowp + kHalo) * (long long)sizeof(float);
            const int want = (rowp / kWave + max_group - 1) / max_group;   // waves per candidate
            inplace = want <= waves ? 1 : 0;
            // a row updated in place always fits lds_small (kInPlaceFits), so path 1 is exactly
            // the in-place case of a workgroup of `waves` waves
            const long long team_lds = inplace ? one_row : 2 * one_row;
            const int lds = lds_small;
            path = inplace ? 1 : (team_lds <= lds_large ? 2 : 0);
            // a longer row that the waves of the wide launch can still hold in registers, and
            // that fits its LDS, is updated in place there
            if (!inplace && wide_waves > 0 &&
                (rowp / kWave + wide_group - 1) / wide_group <= wide_waves && one_row <= lds_wide) {
                path = 3;
                inplace = 1;
                plan_waves = wide_waves;
            } else if (path == 0 && global_waves > waves) {
                path = 4;                         // the global-row launch of twice the waves
                plan_waves = global_waves;
            } else if (inplace) {
                // as many candidates per workgroup as keeps every wave at <= max_group chunks
                teams = waves / want;
                const long long fit = lds / team_lds;
                if (teams > fit)
                    teams = (int)fit;
                // with fewer candidates than the chip has room for, fewer candidates share a
                // workgroup, so that each gets more waves and finishes sooner
                const int spread = (K + slots - 1) / slots;
                if (teams > spread)
                    teams = spread;
            }
        }
        meta[kMetaPath] = path;
        meta[kMetaTeams] = teams;
        meta[kMetaTeamWaves] = plan_waves / teams;
        meta[kMetaInPlace] = inplace;
        meta[kMetaStage] = lds_stage;
        meta[kMetaWaves] = waves;
        meta[kMetaMaxGroup] = max_group;
        meta[kMetaLdsSmall] = lds_small;
        meta[kMetaLdsLarge] = lds_large;
        meta[kMetaHalo] = kHalo;
        meta[kMetaSplit] = split;
        meta[kMetaWideWaves] = wide_waves;
        meta[kMetaWideGroup] = wide_group;
        meta[kMetaLdsWide] = lds_wide;
        meta[kMetaGlobalWaves] = global_waves;
        s_budget = bp;
        s_team_waves = plan_waves / teams;
    }
    __syncthreads();
    const int bp = s_budget;
    const int tw = s_team_waves;
    local = 0;
    for (int l = l0; l < l1; ++l) {
        int span = 0;
        if (bp >= 0) {
            const int32_t *tau_l = tau + (size_t)l * S;
            const int m = mn[l];
            for (int s0 = 0; s0 < S; s0 += 8) {
                int v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    v[i] = tau_l[min(s0 + i, S - 1)];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const long long d = (long long)v[i] - m;
                    if (d <= bp)
                        span = max(span, (int)d);
                }
            }
        }
        nact[l] = span;
        meta[kMetaHeader + (2 + (size_t)kRangeStride) * L + l] = span;
        local += span;
    }
    long long h = 0;                              // sum of the slices before this thread's
    block_scan_256(local, s_sum, &h);
    for (int l = l0; l < l1; ++l) {
        h += nact[l];
        const long long top = h < bp ? h : bp;
        const int n = bp < 0 ? 0 : (int)((top + kWave) / kWave);
        nact[l] = n;
        // wave w of a team sweeps chunks [w n / tw, (w + 1) n / tw) of this row
        int32_t *range = meta + kMetaHeader + 2 * L + (size_t)l * kRangeStride;
        for (int w = 0; w <= tw; ++w)
            range[w] = (int)((long long)w * n / tw);
    }
}

// Prepare, workgroup 1 + l: what the fill visits in layer l, in which order, with the shifts
// tau - m_l; padding up to s8 gets shift INT32_MAX, which no group of buckets can use.
//   level tracked (sorted = 0): one entry per level, ascending in s, so that ties go to the
//     smallest s through the strict "<"; entry r is level r.
//   D record (sorted = 1): the levels are ordered by ascending shift, ties by index, and levels
//     with the SAME shift form one entry: they read the same cell of D_{l-1}, and a rounded add
//     is monotone in the addend, so min_s fl(p + e_s) = fl(p + min_s e_s) bit for bit (up to
//     the sign of a zero): one update with the smallest error of the entry's levels serves them
//     all.  Entry r covers positions start[r] .. start[r + 1] - 1 of `order`, level s belongs
//     to entry entry[s]; the entries a group of buckets can use form a prefix.
//   D record, at most 64 levels (sorted = 2): as above, but the entries are ordered by
//     (shift mod 4, shift): the sweep reads four consecutive buckets per lane with one aligned
//     128-bit LDS read and treats the four residues of the shift separately; the usable entries
//     of a residue then form a prefix of that residue's run.
// One thread per level (S <= 255).
__device__ void prepare_order(const int32_t *__restrict__ tau, int l, int S, int s8, int sorted,
                              int32_t *__restrict__ shifts, int32_t *__restrict__ order,
                              int32_t *__restrict__ start, int32_t *__restrict__ entry_of)
{
    __shared__ int32_t s_shift[256];
    __shared__ int32_t s_level[256];
    __shared__ int s_entries;
    const int s = threadIdx.x;
    int32_t *shifts_l = shifts + (size_t)l * s8;
    int32_t *order_l = order + (size_t)l * s8;
    bool twin = false;                            // a later level of the layer takes the same time
    if (s < S) {
        const int32_t *tau_l = tau + (size_t)l * S;
        const int mine = tau_l[s];
        int rank = 0, m = INT32_MAX;
        for (int o = 0; o < S; ++o)
            m = min(m, tau_l[o]);
        const int residues = sorted == 2 ? 3 : 0;
        const int mine_class = (mine - m) & residues;
        for (int o = 0; o < S; ++o) {
            const int other = tau_l[o];
            const int other_class = (other - m) & residues;
            const bool before = other_class != mine_class ? other_class < mine_class
                                                          : (other < mine || (other == mine && o < s));
            rank += before ? 1 : 0;
            twin |= o > s && other == mine;
        }
        if (!sorted)
            rank = s;
        order_l[rank] = s;
        if (sorted) {
            s_shift[rank] = mine - m;
            s_level[rank] = s;
        } else {
            shifts_l[rank] = mine - m;
        }
    } else if (s < s8) {
        order_l[s] = 0;
        if (!sorted)
            shifts_l[s] = INT32_MAX;
    }
    int32_t *start_l = start + (size_t)l * (s8 + kBatch);
    if (!sorted) {
        // level order: start[0..1] holds, for the first 64 levels, the set of those that have
        // such a twin (the only ones that can make a later level not worth visiting)
        const unsigned long long twins = __ballot(twin);
        if (s == 0) {
            start_l[0] = (int32_t)(twins & 0xFFFFFFFFull);
            start_l[1] = (int32_t)(twins >> 32);
        }
        return;
    }
    __syncthreads();
    const int r = threadIdx.x;                    // a position of the sorted order
    if (r < S) {
        int entry = 0;                            // distinct shifts before position r
        for (int o = 1; o <= r; ++o)
            entry += s_shift[o] != s_shift[o - 1] ? 1 : 0;
        if (r == 0 || s_shift[r] != s_shift[r - 1]) {
            shifts_l[entry] = s_shift[r];
            start_l[entry] = r;
        }
        entry_of[(size_t)l * s8 + s_level[r]] = entry;
        if (r == S - 1)
            s_entries = entry + 1;
    }
    __syncthreads();
    for (int e = s_entries + r; e < s8 + kBatch; e += 256) {
        start_l[e] = S;                           // the last entry ends here; padding is empty
        if (e < s8)
            shifts_l[e] = INT32_MAX;
    }
}

__global__ __launch_bounds__(256) void dp_prepare(const int32_t *__restrict__ tau, int K,
                                                  int slots, int L, int S,
                                                  int s8, int B, int waves, int max_group,
                                                  int lds_small, int lds_large, int lds_stage,
                                                  int sorted, int split, int wide_waves,
                                                  int wide_group, int lds_wide, int global_waves,
                                                  int32_t *__restrict__ meta,
                                                  int32_t *__restrict__ shifts,
                                                  int32_t *__restrict__ order,
                                                  int32_t *__restrict__ start,
                                                  int32_t *__restrict__ entry_of)
{
    if (blockIdx.x == 0)
        prepare_budget(tau, K, slots, L, S, B, waves, max_group, lds_small, lds_large, lds_stage,
                       split, wide_waves, wide_group, lds_wide, global_waves, meta);
    else
        prepare_order(tau, blockIdx.x - 1, S, s8, sorted, shifts, order, start, entry_of);
}

// ---------------------------------------------------------------------------------------------
// v_min_f32 / v_min3_f32 without the canonicalising v_max the compiler puts in front of fminf
// (no NaN can occur: err is finite or +inf and D starts at -0 / +inf).
__device__ __forceinline__ void vmin(float &b, float x)
{
    asm("v_min_f32 %0, %0, %1" : "+v"(b) : "v"(x));
}
__device__ __forceinline__ void vmin3(float &b, float x, float y)
{
    asm("v_min3_f32 %0, %0, %1, %2" : "+v"(b) : "v"(x), "v"(y));
}

// Where err[k][l][s] comes from: an explicit table, or the product of a per-layer sensitivity
// c[k][l] and a per-level weight w[s] (Eq. 4), formed with one fp32 multiply when it is needed.
struct ErrRow {          // the S errors of one (candidate, layer)
    const float *err_kl; // explicit row, or nullptr
    const float *w;
    float c_kl;
    __device__ __forceinline__ float at(int s) const
    {
        return err_kl ? err_kl[s] : __fmul_rn(c_kl, w[s]);
    }
};
struct ErrSource {
    const float *err;    // [K][L][S], or nullptr
    const float *c;      // [K][L]
    const float *w;      // [S]
    __device__ __forceinline__ ErrRow row(size_t k, int l, int L, int S) const
    {
        ErrRow r;
        r.err_kl = err ? err + (k * L + l) * S : nullptr;
        r.w = w;
        r.c_kl = err ? 0.0f : c[k * L + l];
        return r;
    }
    // The same source seen from candidate k (its [L][S] table or its [L] sensitivities), so that
    // a loop over the layers of one candidate does not redo the 64-bit index arithmetic.
    __device__ __forceinline__ ErrSource of_candidate(size_t k, int L, int S) const
    {
        return ErrSource{err ? err + k * L * S : nullptr, c ? c + k * L : nullptr, w};
    }
    __device__ __forceinline__ ErrRow layer(int l, int S) const   // of a per-candidate view
    {
        ErrRow r;
        r.err_kl = err ? err + (size_t)l * S : nullptr;
        r.w = w;
        r.c_kl = err ? 0.0f : c[l];
        return r;
    }
};

// Re-solving candidates that share their first layers with an already solved incumbent
// (Alg. 4 resamples a few sensitivities of the incumbent): candidate k's tables equal the
// incumbent's for layers < first_layer[k], so its rows of D do too, and the fill starts at
// layer first_layer[k] from the incumbent's recorded row first_layer[k] - 1.
struct Resume {
    const int32_t *first_layer;   // [K] in [0, L], or nullptr: every candidate starts at layer 0
    const float *inc_rec;         // the incumbent's D record, float [L][pitch]
    __device__ __forceinline__ int start(int k, int L) const
    {
        if (!first_layer)
            return 0;
        const int f = first_layer[k];
        return f < 0 ? 0 : (f > L ? L : f);
    }
};

// Solving with a fraction of the record (Sec. 3.2 counts O(L T) memory for the matrices): a
// first pass over all layers keeps only every `stride`-th row of D (checkpoints) and finds the
// final time; then, from the last block of `stride` layers to the first, the block's rows are
// filled again from the checkpoint below it into a small block record and walked back.
//   pass 0 (checkpoints): layers [0, L); row l is kept at slot (l + 1) / stride - 1 when
//                         (l + 1) is a multiple of stride and l + 1 < L
//   pass 1 (one block)  : layers [begin, end), starting from checkpoint slot begin / stride - 1
//                         (from scratch when begin = 0); row l is kept at slot l - begin of the
//                         block record; no final argmin
struct Blocks {
    int pass;
    int begin, end;
    int stride;
    int slots;                    // checkpoint rows per candidate
    float *ckpt;                  // [K][slots][pitch]
    float *block;                 // [K][stride][pitch]
};

struct LevelEntry {   // one visited level of one layer of one candidate
    int32_t shift;    // tau - m_l (INT32_MAX in padding entries)
    float err;
    unsigned long long keep = ~0ull;   // wave-uniform: which of the first 64 entries to visit
};

// The prepare kernel's tables of one layer (see prepare_order).
struct LayerTable {
    const int32_t *shift;   // [s8]
    const int32_t *order;   // [s8]
    const int32_t *start;   // [s8 + kBatch], D record only
    const int32_t *entry;   // [s8], D record only
    int limit;              // a larger shift than this (the reduced budget) is never usable
    // An entry beyond the budget could still "apply" to the padding buckets at the end of a row;
    // it is taken out here, so that every shift the sweep uses is at most the layer's largest
    // usable one (the staged tiles of the global-row path size their window by that).
    __device__ __forceinline__ int32_t usable(int32_t shift) const
    {
        return shift > limit ? INT32_MAX : shift;
    }
};
struct LevelTables {
    const int32_t *shifts, *order, *start, *entry;
    int s8;
    int limit = INT32_MAX;  // set by the fill once it knows the reduced budget
    __device__ __forceinline__ LayerTable layer(int l) const
    {
        return LayerTable{shifts + (size_t)l * s8, order + (size_t)l * s8,
                          start + (size_t)l * (s8 + kBatch), entry + (size_t)l * s8, limit};
    }
};

// This lane's entry of the 64 visited entries of a layer starting at entry `blk`.  With the D
// record an entry stands for all levels of one shift and carries the smallest of their errors.
template <bool kLevel>
__device__ __forceinline__ LevelEntry load_level(LayerTable tl, ErrRow er, int s8, int blk,
                                                 int lane)
{
    LevelEntry p;
    p.shift = INT32_MAX;
    p.err = __builtin_inff();
    const int r = blk + lane;
    if (r < s8) {
        p.shift = tl.usable(tl.shift[r]);
        if constexpr (kLevel) {
            p.err = er.at(tl.order[r]);
        } else {
            const int end = tl.start[r + 1];
            for (int j = tl.start[r]; j < end; ++j) {
                const float e = er.at(tl.order[j]);
                p.err = e < p.err ? e : p.err;
            }
        }
    }
    return p;
}

// Layers of at most 64 levels (one lane per level): what a wave loads for the NEXT layer while
// it sweeps a layer.  No load depends on another, so all are in flight during the sweep.
//   shift : shift of entry `lane` (every wave)
//   raw   : error of level `lane`; with the level record entry r is level r and this is the
//           entry's error; with the D record only the first wave of a team loads it, with
//   entry : the entry level `lane` belongs to, and folds the errors of a team's candidate into
//           the team's table in LDS with one atomic min per lane (publish_entries).
struct LevelFetch {
    int32_t shift;
    float raw;
    int32_t entry;
};

template <bool kLevel>
__device__ __forceinline__ LevelFetch fetch_levels(LayerTable tl, ErrRow er, int S, int s8,
                                                   int lane, bool producer)
{
    LevelFetch f;
    f.shift = lane < s8 ? tl.usable(tl.shift[lane]) : INT32_MAX;
    f.raw = __builtin_inff();
    f.entry = 0;
    if (lane < S && (kLevel || producer)) {
        f.raw = er.at(lane);
        if constexpr (!kLevel)
            f.entry = tl.entry[lane];
    }
    return f;
}

// Level record: a level need not be visited when an earlier level of the layer takes the same
// time with an error no larger: it reads the same cell of D_{l-1}, a rounded add is monotone in
// the addend, so its value cannot be strictly smaller than the earlier one's and the strict "<"
// never selects it.  Bit r of the result is set when level r has to be visited; one wave.
// `twins`: the levels that have a later level of the same time (from the prepare kernel).
__device__ __forceinline__ unsigned long long levels_to_visit(const LevelFetch &f,
                                                              unsigned long long twins, int lane)
{
    bool skip = false;
    while (twins) {
        const int r = __builtin_ctzll(twins);
        twins &= twins - 1;
        const int shift = __builtin_amdgcn_readlane(f.shift, r);
        const float err = __builtin_bit_cast(
            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, f.raw), r));
        skip |= lane > r && f.shift == shift && err <= f.raw;
    }
    return __ballot(!skip);
}

__device__ __forceinline__ unsigned long long load_twins(LayerTable tl)
{
    return (unsigned long long)(uint32_t)tl.start[0] |
           ((unsigned long long)(uint32_t)tl.start[1] << 32);
}

// table[r] = smallest error among the levels of entry r (+inf for unused entries); one wave.
__device__ __forceinline__ void publish_entries(float *table, const LevelFetch &f, int S, int lane)
{
    table[lane] = __builtin_inff();
    if (lane < S)
        __hip_atomic_fetch_min(&table[f.entry], f.raw, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
}

// The table words of the next layer that are still being loaded while a layer is swept.  Loads
// and stores retire through one in-order counter, so a wait for these loads placed after the
// record stores of a layer would also wait for those stores; `settle` makes the compiler wait
// for the loads where it is called (right after the sweep, when they have long arrived).
struct Pending {
    const LevelFetch *fetch;
    const LevelEntry *entry;
    __device__ __forceinline__ void settle() const
    {
        asm volatile("" ::"v"(fetch->raw), "v"(fetch->shift), "v"(fetch->entry),
                     "v"(entry->shift), "v"(entry->err));
    }
};

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// The levels of one layer swept over one group of R chunks (R*64 consecutive reduced buckets
// from t0); best[j] / arg[j] belong to bucket t0 + 64*j + lane.
//   prev  : row of the previous layer, prev[-kHalo .. -1] reads +inf
//   first : lane i holds visited entry i of the layer (entries 0..63)
//   tl / er : the layer's tables, for entries >= 64
// A level applies to the group if its shift does not exceed the group's last bucket; lanes
// left of the shift then read the +inf apron.  The applicable levels of a 64-block are found
// with one ballot and walked in ascending position.
template <int R, bool kLevel>
__device__ __forceinline__ void sweep_group(const float *__restrict__ prev, LevelEntry first,
                                            LayerTable tl, ErrRow er, int s8, int t0, int lane,
                                            float (&best)[R], unsigned (&arg)[R])
{
#pragma unroll
    for (int j = 0; j < R; ++j) {
        best[j] = __builtin_inff();
        arg[j] = kNoLevel;
    }
    const int last = t0 + R * kWave - 1;      // last bucket of the group
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): see fill_group_quads
    const char *pl = reinterpret_cast<const char *>(prev + t0 + lane);
    auto row_at = [&](int shift) {
        return reinterpret_cast<const float *>(pl - (size_t)((unsigned)shift * 4u));
    };

    // (with S <= 64 this loop runs once; telling the compiler so made the code slower)
    for (int blk = 0; blk < s8; blk += kWave) {
        const LevelEntry mine =
            blk == 0 ? first : load_level<kLevel>(tl, er, s8, blk, lane);
        unsigned long long use = __ballot(mine.shift <= last);
        if (blk == 0)
            use &= first.keep;
        if constexpr (kLevel) {
            while (use) {
                const int i = __builtin_ctzll(use);
                use &= use - 1;
                const float *p = row_at(__builtin_amdgcn_readlane(mine.shift, i));
                const float e = lane_value(mine.err, i);
                const unsigned s = (unsigned)(blk + i);   // visiting order = level index here
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    // strict "<" decides the level; the value is the min either way (the sign
                    // of a zero may differ from a select's, the walk back re-sums the cost)
                    const float v = p[j * kWave] + e;
                    arg[j] = v < best[j] ? s : arg[j];
                    vmin(best[j], v);
                }
            }
        } else {
            // sorted by shift: the applicable levels are the first n_use of the block
            const int n_use = __builtin_popcountll(use);
            int i = 0;
            for (; i + 2 <= n_use; i += 2) {
                const float *p0 = row_at(__builtin_amdgcn_readlane(mine.shift, i));
                const float *p1 = row_at(__builtin_amdgcn_readlane(mine.shift, i + 1));
                const float e0 = lane_value(mine.err, i);
                const float e1 = lane_value(mine.err, i + 1);
#pragma unroll
                for (int j = 0; j < R; ++j)
                    vmin3(best[j], p0[j * kWave] + e0, p1[j * kWave] + e1);
            }
            if (i < n_use) {
                const float *p0 = row_at(__builtin_amdgcn_readlane(mine.shift, i));
                const float e0 = lane_value(mine.err, i);
#pragma unroll
                for (int j = 0; j < R; ++j)
                    vmin(best[j], p0[j * kWave] + e0);
            }
            if (n_use < kWave)
                break;                        // later blocks only hold larger shifts
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The D-record sweep with 128-bit LDS reads (layers of at most 64 levels).  Aligned 128-bit reads
// move twice the bytes per clock of narrower ones, so a lane takes four consecutive buckets:
//   * the first 252 Q buckets of a wave's group are Q "quad chunks": lane i >= 1 owns buckets
//     252 j + 4 (i - 1) .. + 3 of quad chunk j, and one read gives it the four values
//     row[4 q .. 4 q + 3] of the aligned quad q = (its own quad) - (shift / 4);
//   * a shift that is not a multiple of four needs the last (shift mod 4) values of the quad
//     below, which is exactly what the lane to the left has read: they come over with the add
//     itself (DPP wave_shr:1).  Lane 0 has no bucket of its own: it reads the quad below lane
//     1's and only serves as that left neighbour (63 of 64 lanes work);
//   * the residue decides which operands cross lanes, so the entries of a layer are visited by
//     residue (the prepare kernel orders them that way) and each residue has its own code;
//   * the remaining buckets of the group, fewer than 252, are covered by T ordinary chunks of 64
//     (32-bit reads, lane = bucket) placed at the END of the group; they may overlap the quad
//     chunks by up to 63 buckets, which are then computed twice with the same result.
// R chunks of 64 thus become Q quad chunks and T tail chunks, 4 Q + T <= R + 1 registers.
typedef float float4v __attribute__((ext_vector_type(4)));
constexpr int kQuadLanes = kWave - 1;             // lanes of a quad chunk that own buckets
constexpr int kQuadChunk = 4 * kQuadLanes;        // 252 buckets
constexpr int quad_chunks(int R) { return R * kWave / kQuadChunk; }
constexpr int tail_chunks(int R)
{
    return (R * kWave - quad_chunks(R) * kQuadChunk + kWave - 1) / kWave;
}

// x of the lane to the left (lane 0 gets 0.0f, which nothing uses)
__device__ __forceinline__ float from_left(float x)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138 /* wave_shr:1 */, 0xf, 0xf, true));
}

// The four values D_{l-1}[t - shift] for the four buckets t of a lane, from the aligned quad `own`
// it has read and the quad the lane to its left has read; kRes = shift mod 4.
template <int kRes>
__device__ __forceinline__ void shifted_quad(float4v own, float e, float (&v)[4])
{
    const float o[4] = {own.x, own.y, own.z, own.w};
#pragma unroll
    for (int c = 0; c < 4; ++c)
        v[c] = (c >= kRes ? o[c - kRes] : from_left(o[4 + c - kRes])) + e;
}

// kSplit: the waves of a workgroup come in two halves that sweep the same chunks, each visiting
// every other pair of the run's entries (a run's odd last entry counts as a pair); `skip`: the
// run's first pair is the other half's.
template <int Q, int T, int kRes, bool kSplit>
__device__ __forceinline__ void sweep_residue(const float4v *quads, const float *tail,
                                              LevelEntry mine, unsigned long long use, bool skip,
                                              float (&bq)[Q > 0 ? Q : 1][4], float (&bt)[T > 0 ? T : 1])
{
    auto visit_two = [&](int i) {
        const int s0 = __builtin_amdgcn_readlane(mine.shift, i);
        const int s1 = __builtin_amdgcn_readlane(mine.shift, i + 1);
        float e0 = lane_value(mine.err, i);
        float e1 = lane_value(mine.err, i + 1);
        asm volatile("" : "+v"(e0), "+v"(e1));    // addends of the cross-lane adds live in VGPRs
        if constexpr (Q > 0) {
            const float4v *q0 = quads - (s0 >> 2);
            const float4v *q1 = quads - (s1 >> 2);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                float a[4], b[4];
                shifted_quad<kRes>(q0[j * kQuadLanes], e0, a);
                shifted_quad<kRes>(q1[j * kQuadLanes], e1, b);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    vmin3(bq[j][c], a[c], b[c]);
            }
        }
        if constexpr (T > 0) {
            const float *p0 = tail - s0;
            const float *p1 = tail - s1;
#pragma unroll
            for (int j = 0; j < T; ++j)
                vmin3(bt[j], p0[j * kWave] + e0, p1[j * kWave] + e1);
        }
    };
    auto visit_one = [&](int i) {
        const int s0 = __builtin_amdgcn_readlane(mine.shift, i);
        float e0 = lane_value(mine.err, i);
        asm volatile("" : "+v"(e0));
        if constexpr (Q > 0) {
            const float4v *q0 = quads - (s0 >> 2);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                float a[4];
                shifted_quad<kRes>(q0[j * kQuadLanes], e0, a);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    vmin(bq[j][c], a[c]);
            }
        }
        if constexpr (T > 0) {
            const float *p0 = tail - s0;
#pragma unroll
            for (int j = 0; j < T; ++j)
                vmin(bt[j], p0[j * kWave] + e0);
        }
    };
    // the usable entries of a residue are consecutive positions of the visiting order
    int i = use ? __builtin_ctzll(use) : 0;
    int n = __builtin_popcountll(use);
    if constexpr (kSplit) {
        if (skip) {
            i += 2;
            n -= 2;
        }
        for (; n >= 2; n -= 4, i += 4)
            visit_two(i);
        if (n == 1)
            visit_one(i);
    } else {
        for (; n >= 2; n -= 2, i += 2)
            visit_two(i);
        if (n)
            visit_one(i);
    }
}

// One group of R chunks of one layer (D record, at most 64 levels): sweep with 128-bit reads,
// store the record, write the new row values; the barrier protocol is fill_group's.
// prev + t0 is 16-byte aligned (rows, aprons and chunk starts are multiples of four floats).
// kSplit (in place only): this wave has a twin in the other half of the workgroup with the same
// group; the two visit alternate pairs of the layer's entries, the second half (`half` = 1)
// leaves its minima in `part` (indexed like the row) before the barrier, and the first half
// folds them into its own behind it.  min is exact and order-blind here, so the row is the one
// a single wave would have computed.
template <int R, bool inplace, bool kSplit>
__device__ __forceinline__ void fill_group_quads(const float *prev, float *cur, float *rec,
                                                 LevelEntry first, int t0, int lane,
                                                 Pending pending, int half, float *part)
{
    static_assert(!kSplit || inplace, "the halves meet at the in-place barrier");
    if constexpr (R == 0) {
        pending.settle();
        if (inplace)
            __syncthreads();
    } else {
        constexpr int Q = quad_chunks(R), T = tail_chunks(R);
        constexpr int tail0 = (R - T) * kWave;    // first bucket of the tail chunks in the group
        float bq[Q > 0 ? Q : 1][4], bt[T > 0 ? T : 1];
#pragma unroll
        for (int j = 0; j < Q; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                bq[j][c] = __builtin_inff();
#pragma unroll
        for (int j = 0; j < T; ++j)
            bt[j] = __builtin_inff();
        const int last = t0 + R * kWave - 1;      // last bucket of the group
        const float4v *quads = reinterpret_cast<const float4v *>(prev + t0) + (lane - 1);
        const float *tail = prev + t0 + tail0 + lane;
        const unsigned long long use = __ballot(first.shift <= last);
        const int residue = first.shift & 3;
        // Scalar loads and LDS reads share one counter, and scalar loads return out of order: while
        // one is in flight (the wall clock of the priority turns, the next layer's chunk range)
        // every wait for an LDS read in the sweep has to be a wait for ALL of them, and a wave
        // cannot start on the first quads while the later ones arrive.  Let them land first.
        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0), nothing else
        const unsigned long long use0 = use & __ballot(residue == 0);
        const unsigned long long use1 = use & __ballot(residue == 1);
        const unsigned long long use2 = use & __ballot(residue == 2);
        const unsigned long long use3 = use & __ballot(residue == 3);
        // kSplit: the pairs of entries are numbered through the four runs; half h visits the
        // pairs whose number is h mod 2, so both halves get every residue's kind of work
        int turn = half;
        sweep_residue<Q, T, 0, kSplit>(quads, tail, first, use0, turn & 1, bq, bt);
        if constexpr (kSplit)
            turn += (__builtin_popcountll(use0) + 1) >> 1;
        sweep_residue<Q, T, 1, kSplit>(quads, tail, first, use1, turn & 1, bq, bt);
        if constexpr (kSplit)
            turn += (__builtin_popcountll(use1) + 1) >> 1;
        sweep_residue<Q, T, 2, kSplit>(quads, tail, first, use2, turn & 1, bq, bt);
        if constexpr (kSplit)
            turn += (__builtin_popcountll(use2) + 1) >> 1;
        sweep_residue<Q, T, 3, kSplit>(quads, tail, first, use3, turn & 1, bq, bt);
        pending.settle();
        const int tq = t0 + 4 * (lane - 1);       // this lane's first bucket of quad chunk 0
        const int tt = t0 + tail0 + lane;
        if constexpr (kSplit) {
            if (half) {
                if (lane > 0) {
#pragma unroll
                    for (int j = 0; j < Q; ++j) {
                        const float4v v = {bq[j][0], bq[j][1], bq[j][2], bq[j][3]};
                        *reinterpret_cast<float4v *>(part + tq + j * kQuadChunk) = v;
                    }
                }
#pragma unroll
                for (int j = 0; j < T; ++j)
                    part[tt + j * kWave] = bt[j];
            }
            __syncthreads();                      // every read of the row is done, `part` is written
            if (half)
                return;
            if (lane > 0) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const float4v v = *reinterpret_cast<const float4v *>(part + tq + j * kQuadChunk);
                    vmin(bq[j][0], v.x);
                    vmin(bq[j][1], v.y);
                    vmin(bq[j][2], v.z);
                    vmin(bq[j][3], v.w);
                }
            }
#pragma unroll
            for (int j = 0; j < T; ++j)
                vmin(bt[j], part[tt + j * kWave]);
        }
        if (rec) {       // streamed: the record is not read again before the walk back
            if (lane > 0) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const float4v v = {bq[j][0], bq[j][1], bq[j][2], bq[j][3]};
                    __builtin_nontemporal_store(
                        v, reinterpret_cast<float4v *>(rec + tq + j * kQuadChunk));
                }
            }
#pragma unroll
            for (int j = 0; j < T; ++j)
                __builtin_nontemporal_store(bt[j], &rec[tt + j * kWave]);
        }
        if (inplace && !kSplit)
            __syncthreads();
        if (lane > 0) {
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const float4v v = {bq[j][0], bq[j][1], bq[j][2], bq[j][3]};
                *reinterpret_cast<float4v *>(cur + tq + j * kQuadChunk) = v;
            }
        }
#pragma unroll
        for (int j = 0; j < T; ++j)
            cur[tt + j * kWave] = bt[j];
    }
}

// One group of one layer: sweep, store the record, and write the new row values to `cur`.
// With `inplace` cur aliases prev, so a workgroup barrier separates the last read of the row
// from the first write (every wave of the workgroup calls this exactly once per layer then,
// with R = 0 if it has no chunks).
template <int R, bool kLevel, bool inplace>
__device__ __forceinline__ void fill_group(const float *prev, float *cur, uint8_t *choice,
                                           float *rec, LevelEntry first, LayerTable tl, ErrRow er,
                                           int s8, int t0, int lane, Pending pending)
{
    if constexpr (R == 0) {
        pending.settle();
        if (inplace)
            __syncthreads();
    } else {
        float best[R];
        unsigned arg[R];
        sweep_group<R, kLevel>(prev, first, tl, er, s8, t0, lane, best, arg);
        pending.settle();
        const int tl = t0 + lane;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if constexpr (kLevel)
                choice[tl + j * kWave] = (uint8_t)arg[j];
            else if (rec)   // streamed: the record is not read again before the walk back
                __builtin_nontemporal_store(best[j], &rec[tl + j * kWave]);
        }
        if (inplace)
            __syncthreads();
#pragma unroll
        for (int j = 0; j < R; ++j)
            cur[tl + j * kWave] = best[j];
    }
}

template <bool kLevel, bool inplace, int kMax, bool kQuads, bool kSplit = false>
__device__ __forceinline__ void fill_group_n(int r, const float *prev, float *cur, uint8_t *choice,
                                             float *rec, LevelEntry first, LayerTable tl,
                                             ErrRow er, int s8, int t0, int lane, Pending pending,
                                             int half = 0, float *part = nullptr)
{
    static_assert(!kSplit || kQuads, "only the 128-bit sweep splits a layer's entries");
    switch (r) {
#define SPDY_CASE(RR)                                                                          \
    case RR:                                                                                   \
        if constexpr (RR <= kMax) {                                                            \
            if constexpr (kQuads)                                                              \
                fill_group_quads<RR, inplace, kSplit>(prev, cur, rec, first, t0, lane,         \
                                                      pending, half, part);                    \
            else                                                                               \
                fill_group<RR, kLevel, inplace>(prev, cur, choice, rec, first, tl, er, s8, t0, \
                                                lane, pending);                                \
        }                                                                                      \
        break;
        SPDY_CASE(0)
        SPDY_CASE(1)
        SPDY_CASE(2)
        SPDY_CASE(3)
        SPDY_CASE(4)
        SPDY_CASE(5)
        SPDY_CASE(6)
        SPDY_CASE(7)
        SPDY_CASE(8)
        SPDY_CASE(9)
        SPDY_CASE(10)
        SPDY_CASE(11)
        SPDY_CASE(12)
        SPDY_CASE(13)
        SPDY_CASE(14)
        SPDY_CASE(15)
        SPDY_CASE(16)
        SPDY_CASE(17)
        SPDY_CASE(18)
        SPDY_CASE(19)
        SPDY_CASE(20)
        SPDY_CASE(21)
        SPDY_CASE(22)
        SPDY_CASE(23)
        SPDY_CASE(24)
        SPDY_CASE(25)
        SPDY_CASE(26)
        SPDY_CASE(27)
        SPDY_CASE(28)
#undef SPDY_CASE
    }
}

// (value, t) pairs ordered by value, then by smaller t.
__device__ __forceinline__ void argmin_merge(float &bv, int &bt, float v, int t)
{
    if (v < bv || (v == bv && t < bt)) {
        bv = v;
        bt = t;
    }
}

__device__ __forceinline__ void write_result(float bv, int bt, int k, int32_t *tstar, float *cost)
{
    cost[k] = bv;
    tstar[k] = (bv < __builtin_inff()) ? bt : -1;   // -1: no profile meets the budget
}

// ---------------------------------------------------------------------------------------------
// The fill (Eq. 2-3 for all L layers) and the final argmin over t.  The waves of a workgroup
// form `teams` teams of `tw` waves; team i of workgroup b solves candidate b * teams + i.
// Barriers are workgroup-wide, so every team steps through the layers together.
//   kPath    : which of the launches this is (it returns at once unless the prepare kernel chose
//              it).  1: rows in LDS, updated in place: a layer is swept, barrier, written back to
//              the same row, barrier.  2: two rows in LDS alternate, one barrier per layer.
//              0: two rows of kHalo + pitch floats in `rows` in global memory, one candidate per
//              workgroup.  (A row that can be updated in place always fits the smaller LDS
//              allocation and two longer ones never do, so path 1 is exactly the in-place case
//              of a workgroup of the usual size; each instantiation holds only its own way of
//              stepping through a layer.)
//              3 (D record): path 1's code in a workgroup of twice the waves with up to a whole
//              compute unit's LDS: rows of up to twice path 1's length are still updated in
//              place (one candidate per workgroup, one workgroup per compute unit at a time).
//              4 (D record): path 0's code in a workgroup of twice the waves with a whole compute
//              unit's LDS for the window (its tiles are twice as long).
//   kNarrow  : S <= 64, one lane per level: the next layer's table is loaded without dependent
//              loads while a layer is swept (a separate instantiation, so that the waits of the
//              two ways of loading do not meet in one control-flow join)
//   kBlocks  : the checkpoint / block passes of the small-record solve (D record only); the
//              plain instantiation ignores `blocks`
//   kTurns   : the workgroups that share a compute unit take turns at the instruction priority
//              (see the layer loop); `units` is the number of compute units
//   kSplit   : launched with twice the waves the plan was made for (D record, in place, S <= 64,
//              no more candidates than compute units, so a workgroup has its unit to itself and
//              one wave per SIMD and candidate issues too little).  Wave w of the second half is
//              the twin of wave w of the first: same team, same chunks, the other pairs of each
//              layer's entries (see fill_group_quads).  The second half only sweeps; tables,
//              record, row and the final argmin are the first half's.  The partial rows of the
//              second half lie in LDS behind the smaller allocation (the launch gets twice that).
// `pitch` is the record's row pitch (elements per (k, l) row).
template <bool kLevel, int kPath, bool kNarrow, bool kBlocks, bool kTurns = false,
          bool kSplit = false>
__global__ __launch_bounds__(fill_waves<kLevel>() * (kSplit || kPath >= 3 ? 2 : 1) * kWave,
                             kLevel ? 8 : 4)
void dp_fill(
    ErrSource src, const int32_t *__restrict__ meta, LevelTables tables, int units, int K, int L,
    int S, int pitch, uint8_t *__restrict__ choice, float *__restrict__ drec,
    float *__restrict__ rows, int32_t *__restrict__ tstar, float *__restrict__ cost, Resume resume,
    Blocks blocks)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ float s_best[kMaxFillWaves];
    __shared__ int s_time[kMaxFillWaves];
    // per team and for two layers: merged errors (D record), or in the same storage one 64-bit
    // set of levels to visit (level record)
    __shared__ __attribute__((aligned(8))) float s_entries[2][kMaxFillWaves][kWave];
    constexpr bool kGlobal = kPath == 0 || kPath == 4;     // rows in global memory
    constexpr bool kLds = !kGlobal, inplace = kPath == 1 || kPath == 3;
    static_assert(kPath < 3 || (!kLevel && !kBlocks && !kTurns && !kSplit),
                  "the launches of twice the waves are plain D-record fills");
    constexpr bool kQuads = !kLevel && kNarrow;  // the D-record sweep with 128-bit LDS reads
    static_assert(!kSplit || (kQuads && kPath == 1 && !kBlocks && !kTurns),
                  "the split launch is the plain in-place D-record fill");
    if (meta[kMetaPath] != kPath)
        return;                                  // another launch does the work
    const int bp = meta[kMetaBudget];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    if (bp < 0) {                                // even the fastest levels exceed the budget
        if (tid == 0 && !(kBlocks && blocks.pass == 1))
            write_result(__builtin_inff(), 0, blockIdx.x, tstar, cost);
        return;
    }
    tables.limit = kGlobal ? bp : INT32_MAX;     // only the tiles of global rows depend on it
    const int teams = meta[kMetaTeams];
    const int tw = meta[kMetaTeamWaves];
    if ((long long)blockIdx.x * teams >= K)
        return;                                  // the first ceil(K / teams) workgroups suffice
    const int row = meta[kMetaRow];
    const int lane = tid & (kWave - 1);
    int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    int half = 0;                                // kSplit: 1 for the twins of the planned waves
    if constexpr (kSplit) {
        const int planned = nthreads / (2 * kWave);
        half = wave >= planned ? 1 : 0;
        wave -= half * planned;
    }
    const bool lead = half == 0;
    const int team = wave / tw;
    const int wv = wave - team * tw;             // this wave's index in its team
    // Which share of the row this wave sweeps.  The low chunks of a row cost less than the high
    // ones (fewer levels reach them), and wave w of a workgroup runs on SIMD w mod 4: with the
    // shares in wave order one SIMD would hold the cheap shares of every team and another the
    // expensive ones.  Every second group of four waves therefore takes its shares in reverse.
    const bool mirrored = (tw & (tw - 1)) == 0 && ((wave >> 2) & 1);
    const int share = mirrored ? wv ^ (min(tw, 4) - 1) : wv;
    const int k = blockIdx.x * teams + team;
    const bool active = team < teams && k < K;

    // rows: [apron | row] once (in place) or twice per team
    const int stride = kHalo + (kLds ? row : pitch);
    const int team_floats = inplace ? stride : 2 * stride;
    float *base = kLds ? lds + (size_t)(team < teams ? team : 0) * team_floats
                       : rows + (size_t)blockIdx.x * team_floats;
    float *buf0 = base + kHalo;
    float *buf1 = inplace ? buf0 : buf0 + stride;

    // D before the first layer: time 0 costs nothing, nothing else is reachable (Eq. 3 then is
    // the general update).  -0.0f + e returns e bit for bit for every e, +0.0f would not for
    // e = -0.0f.  Aprons and chunks a layer does not compute keep this +inf.
    if constexpr (kLds) {
        for (int i = tid; i < teams * team_floats; i += nthreads)
            lds[i] = (i % team_floats == kHalo) ? -0.0f : __builtin_inff();
    } else {
        for (int i = tid; i < team_floats; i += nthreads)
            if (i % stride < kHalo + row)
                base[i] = (i == kHalo) ? -0.0f : __builtin_inff();
    }
    __syncthreads();

    const int32_t *nact = meta + kMetaHeader + L;
    const size_t ke = active ? k : 0;            // candidate whose errors this wave reads

    // a candidate that shares its first l0 layers with the incumbent starts from the incumbent's
    // row l0 - 1, placed where layer l0 reads its previous row
    const int l0 = active ? resume.start(k, L) : 0;
    if (l0 > 0 && lead) {
        float *dst = (l0 & 1) ? buf1 : buf0;
        const float *from = resume.inc_rec + (size_t)(l0 - 1) * pitch;
        const int n = nact[l0 - 1] * kWave;
        for (int t = wv * kWave + lane; t < n; t += tw * kWave)
            dst[t] = from[t];
        if (wv == 0 && lane == 0 && dst != buf0)
            buf0[0] = __builtin_inff();          // undo the layer-0 start value
    }
    if (resume.first_layer)
        __syncthreads();
    // a block pass starts from the checkpoint below the block
    const int lb = kBlocks ? blocks.begin : 0;   // layers [lb, le) are filled
    const int le = kBlocks ? blocks.end : L;
    if constexpr (kBlocks) {
        if (lb > 0) {
            float *dst = (lb & 1) ? buf1 : buf0;
            const float *from =
                blocks.ckpt + (ke * blocks.slots + (size_t)(lb / blocks.stride - 1)) * pitch;
            const int n = nact[lb - 1] * kWave;
            if (active)
                for (int t = wv * kWave + lane; t < n; t += tw * kWave)
                    dst[t] = from[t];
            if (active && wv == 0 && lane == 0 && dst != buf0)
                buf0[0] = __builtin_inff();      // undo the layer-0 start value
            __syncthreads();
        }
    }

    // this candidate's part of the inputs and of the record
    const ErrSource mine = src.of_candidate(ke, L, S);
    uint8_t *choice_k = kLevel ? choice + ke * L * pitch : nullptr;
    float *drec_k = kLevel ? nullptr : drec + ke * L * pitch;
    if constexpr (kBlocks)
        drec_k = blocks.pass == 0 ? blocks.ckpt + ke * blocks.slots * pitch
                                  : blocks.block + ke * blocks.stride * pitch;

    // lane i keeps visited entry i of the layer being swept; the next layer's is fetched early
    const int s8 = tables.s8;
    // S <= 64: the first wave of a team prepares, for the next layer, the team's table of merged
    // errors (D record) or the set of levels worth visiting (level record)
    const bool producer = kNarrow && share == 0 && team < teams && lead;
    // kSplit: where the twins of this wave's team leave their minima
    float *part = kSplit ? lds + kLdsHalf / (int)sizeof(float) + (size_t)(team < teams ? team : 0) * row
                         : nullptr;
    unsigned long long *keep =
        reinterpret_cast<unsigned long long *>(&s_entries[0][0][0]) + (team < teams ? team : 0);
    float *table = &s_entries[0][team < teams ? team : 0][0];
    LevelEntry next_first{INT32_MAX, 0.0f};
    LevelFetch next_fetch{INT32_MAX, 0.0f, 0};
    if constexpr (kNarrow) {
        next_fetch = fetch_levels<kLevel>(tables.layer(lb), mine.layer(lb, S), S, s8, lane,
                                          producer);
        if (producer) {
            if constexpr (kLevel) {
                const unsigned long long visit =
                    levels_to_visit(next_fetch, load_twins(tables.layer(lb)), lane);
                if (lane == 0)
                    keep[(lb & 1) * kMaxFillWaves] = visit;
            } else {
                publish_entries(table + (lb & 1) * kMaxFillWaves * kWave, next_fetch, S, lane);
            }
        }
        __syncthreads();
    } else {
        next_first = load_level<kLevel>(tables.layer(lb), mine.layer(lb, S), s8, 0, lane);
    }
    Pending{&next_fetch, &next_first}.settle();   // no load is in flight at the loop's head
    // chunk boundaries of this wave
    const int32_t *range = meta + kMetaHeader + 2 * L + (size_t)lb * kRangeStride + share;
    int c_next = range[0], c_end_next = range[1];
    // Two workgroups share a compute unit, and the hardware serves the older one first: left
    // alone, the first `units` workgroups of a launch run at full speed, the second `units` on what
    // is left and then by themselves, at barely more than half the unit's LDS rate.  The
    // instruction priority therefore alternates between the two halves of the last 2 * units
    // workgroups with the wall clock (100 MHz; 2^13 ticks = 82 us per turn), so both advance
    // alike and finish together.  Earlier workgroups of a longer launch are left alone: a
    // compute unit then always holds an older and a younger one, and a new one takes over when
    // the older is done.  A launch with no more workgroups than compute units has no pairs.
    // (kTurns: a separate instantiation, launched for batches of one or two rounds of
    // workgroups; the other one is exactly the code without any of this.)
    const unsigned turn = ((unsigned)blockIdx.x / (unsigned)units) & 1u;
    const int nwg = (K + teams - 1) / teams;
    const bool take_turns = kTurns && nwg > units && (long long)blockIdx.x + 2 * units >= nwg;
    unsigned long long now = take_turns ? wall_clock64() : 0;
    for (int l = lb; l < le; ++l) {
        if constexpr (kTurns) {
            if (take_turns) {
                if ((turn ^ (unsigned)(now >> kPriorityTurn)) & 1u)
                    __builtin_amdgcn_s_setprio(1);
                else
                    __builtin_amdgcn_s_setprio(0);
                now = wall_clock64();            // read now, looked at a layer later: no wait
            }
        }
        LevelEntry first = next_first;
        if constexpr (kNarrow) {
            first.shift = next_fetch.shift;
            first.err = kLevel ? next_fetch.raw : table[(l & 1) * kMaxFillWaves * kWave + lane];
            if constexpr (kLevel)
                first.keep = keep[(l & 1) * kMaxFillWaves];
        }
        if (l + 1 < le) {
            const LayerTable tn = tables.layer(l + 1);
            const ErrRow en = mine.layer(l + 1, S);
            if constexpr (kNarrow)
                next_fetch = fetch_levels<kLevel>(tn, en, S, s8, lane, producer);
            else
                next_first = load_level<kLevel>(tn, en, s8, 0, lane);
        }
        const float *prev = (l & 1) ? buf1 : buf0;
        float *cur = (l & 1) ? buf0 : buf1;
        int c = 0, c_end = 0;                    // this wave's chunks of the row
        if (active && l >= l0) {
            c = c_next;
            c_end = c_end_next;
        }
        if (l + 1 < le) {                        // the next layer's, read a layer ahead
            range += kRangeStride;
            c_next = range[0];
            c_end_next = range[1];
        }
        uint8_t *choice_l = kLevel ? choice_k + (size_t)l * pitch : nullptr;
        float *drec_l = kLevel ? nullptr : drec_k + (size_t)l * pitch;
        if constexpr (kBlocks) {
            if (blocks.pass == 1)
                drec_l = drec_k + (size_t)(l - lb) * pitch;
            else if ((l + 1) % blocks.stride == 0 && l + 1 < L)
                drec_l = drec_k + (size_t)((l + 1) / blocks.stride - 1) * pitch;
            else
                drec_l = nullptr;                // this row is not kept
        } else if constexpr (!kLevel) {
            __builtin_assume(drec_l != nullptr);
        }
        const LayerTable tl = tables.layer(l);
        const ErrRow er = mine.layer(l, S);
        constexpr int kMax = group_limit<kLevel, kTurns>();
        const Pending pending{&next_fetch, &next_first};
        if constexpr (inplace) {                 // c_end - c <= kMax by construction
            fill_group_n<kLevel, true, kMax, kQuads, kSplit>(min(c_end - c, kMax), prev, cur,
                                                             choice_l, drec_l, first, tl, er, s8,
                                                             c * kWave, lane, pending, half, part);
        } else {
            // Rows in global memory: the row is computed in tiles of at most kMax chunks per
            // wave, and the part of the previous row a tile reads (the tile itself and the
            // layer's largest usable shift to its left) is first copied to LDS, so the sweep
            // reads LDS as in the resident case.  One candidate per workgroup here, so every
            // wave takes the same number of trips.  A layer whose largest shift leaves no room
            // for a tile is swept from global memory.
            int tile = 0, span = 0;
            if constexpr (kGlobal) {
                span = meta[kMetaHeader + (2 + (size_t)kRangeStride) * L + l];
                tile = (meta[kMetaStage] / (int)sizeof(float) - span - 8) / kWave / tw * tw;
                tile = min(tile, tw * kMax);
            }
            if (kGlobal && tile >= tw) {
                const int n_l = (active && l >= l0) ? nact[l] : 0;
                if (n_l == 0)
                    pending.settle();
                for (int c0 = 0; c0 < n_l; c0 += tile) {
                    const int nt = min(tile, n_l - c0);
                    // (lo a multiple of four floats: rows and aprons are, so the copy moves 16
                    // bytes per lane, eight loads in flight per lane; four floats more than the
                    // largest shift, for the lane left of a group's first quad)
                    const int lo = max(((c0 * kWave - span) & ~3) - 4, -kHalo);
                    const int len4 = ((c0 + nt) * kWave - lo) / 4;
                    const float4 *from = reinterpret_cast<const float4 *>(prev + lo);
                    float4 *to = reinterpret_cast<float4 *>(lds);
                    for (int i0 = 0; i0 < len4; i0 += 8 * nthreads) {
                        float4 v[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j)   // (past the end: the last element again)
                            v[j] = from[min(i0 + j * nthreads + tid, len4 - 1)];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int i = i0 + j * nthreads + tid;
                            if (i < len4)
                                to[i] = v[j];
                        }
                    }
                    __syncthreads();
                    const int cb = c0 + (int)((long long)share * nt / tw);
                    const int ce = c0 + (int)((long long)(share + 1) * nt / tw);
                    fill_group_n<kLevel, false, kMax, kQuads>(ce - cb, lds - lo, cur, choice_l, drec_l,
                                                      first, tl, er, s8, cb * kWave, lane,
                                                      pending);
                    __syncthreads();             // the next tile overwrites the staged part
                }
            } else {
                while (c < c_end) {
                    const int n = c_end - c;
                    const int groups = (n + kMax - 1) / kMax;
                    const int r = (n + groups - 1) / groups;
                    fill_group_n<kLevel, false, kMax, kQuads>(r, prev, cur, choice_l, drec_l, first, tl,
                                                      er, s8, c * kWave, lane, pending);
                    c += r;
                }
            }
        }
        // the table of the next layer; the barrier that ends this layer publishes it
        if (producer && l + 1 < le) {
            if constexpr (kLevel) {
                const unsigned long long visit =
                    levels_to_visit(next_fetch, load_twins(tables.layer(l + 1)), lane);
                if (lane == 0)
                    keep[((l + 1) & 1) * kMaxFillWaves] = visit;
            } else {
                publish_entries(table + ((l + 1) & 1) * kMaxFillWaves * kWave, next_fetch, S,
                                lane);
            }
        }
        __syncthreads();
    }

    if constexpr (kBlocks) {
        if (blocks.pass == 1)
            return;                              // the final time is known from pass 0
    }
    // final argmin over t' <= bp within each team
    const float *last = (L & 1) ? buf1 : buf0;
    float bv = __builtin_inff();
    int bt = INT32_MAX;
    if (active && lead)
        for (int t = wv * kWave + lane; t <= bp; t += tw * kWave)
            argmin_merge(bv, bt, last[t], t);
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float ov = __shfl_down(bv, off, kWave);
        const int ot = __shfl_down(bt, off, kWave);
        argmin_merge(bv, bt, ov, ot);
    }
    if (lane == 0 && lead) {
        s_best[wave] = bv;
        s_time[wave] = bt;
    }
    __syncthreads();
    if (active && lead && wv == 0 && lane == 0) {
        for (int w = 1; w < tw; ++w)
            argmin_merge(bv, bt, s_best[wave + w], s_time[wave + w]);
        write_result(bv, bt, k, tstar, cost);
    }
}

// Final argmin for another budget on an already filled D record: the rows hold exact-time costs
// and do not depend on the budget, so a smaller budget only shortens the range of the argmin
// (Sec. 3.2: the answer is min over t <= T of the last row).  One workgroup per candidate.
__global__ __launch_bounds__(256) void dp_budget_argmin(const int32_t *__restrict__ meta,
                                                        const float *__restrict__ drec, int L,
                                                        int pitch, int budget,
                                                        int32_t *__restrict__ tstar,
                                                        float *__restrict__ cost)
{
    __shared__ float s_best[4];
    __shared__ int s_time[4];
    const int k = blockIdx.x, tid = threadIdx.x;
    const int bp = meta[kMetaBudget];
    // reduced budget: t' <= budget - M, and never beyond what the fill computed
    const long long reduced = (long long)budget - meta[kMetaMinTime];
    long long top = reduced < bp ? reduced : bp;
    if (bp >= 0) {
        const long long computed = (long long)meta[kMetaHeader + 2 * L - 1] * kWave - 1;
        top = top < computed ? top : computed;
    }
    float bv = __builtin_inff();
    int bt = INT32_MAX;
    if (bp >= 0) {
        const float *last = drec + ((size_t)k * L + (L - 1)) * pitch;
        for (int t = tid; t <= top; t += blockDim.x)
            argmin_merge(bv, bt, last[t], t);
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float ov = __shfl_down(bv, off, kWave);
        const int ot = __shfl_down(bt, off, kWave);
        argmin_merge(bv, bt, ov, ot);
    }
    if ((tid & (kWave - 1)) == 0) {
        s_best[tid / kWave] = bv;
        s_time[tid / kWave] = bt;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            argmin_merge(bv, bt, s_best[w], s_time[w]);
        write_result(bv, bt, k, tstar, cost);
    }
}

// ---------------------------------------------------------------------------------------------
// Walk back (last loop of Alg. 1).

// Level record: one lane per candidate, L dependent one-byte reads; the cost is re-summed over
// the profile in layer order (exactly the sum Alg. 1's strict "<" sweep carries to the cell).
__global__ void dp_backtrace_levels(const int32_t *__restrict__ tau, ErrSource src,
                                    const int32_t *__restrict__ meta,
                                    const uint8_t *__restrict__ choice,
                                    const int32_t *__restrict__ tstar, int K, int L, int S,
                                    int pitch, int16_t *__restrict__ profile,
                                    float *__restrict__ cost)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K)
        return;
    int16_t *prof = profile + (size_t)k * L;
    int t = tstar[k];
    if (t < 0) {
        for (int l = 0; l < L; ++l)
            prof[l] = -1;
        return;
    }
    const int32_t *mn = meta + kMetaHeader;
    const uint8_t *choice_k = choice + (size_t)k * L * pitch;
    bool ok = true;
    for (int l = L - 1; l >= 0; --l) {
        const int s = choice_k[(size_t)l * pitch + t];
        prof[l] = (int16_t)s;
        if (s >= S) {        // cannot happen on a filled table; never index tau out of range
            ok = false;
            break;
        }
        t -= tau[(size_t)l * S + s] - mn[l];
        if (t < 0) {
            ok = false;
            break;
        }
    }
    if (!ok) {
        cost[k] = __builtin_nanf("");
        return;
    }
    __threadfence();
    float acc = -0.0f;
    for (int l = 0; l < L; ++l)
        acc += src.row(k, l, L, S).at(prof[l]);
    cost[k] = acc;
}

// D record: one wave per candidate.  At (l, t) the lanes try the levels in parallel: lane s
// forms D_{l-1}[t - shift_s] + err[l][s] with the same single fp32 add as the fill and compares
// it with D_l[t]; the lowest matching level is the one a strict "<" sweep would have kept.
// Only the gather of D_{l-1} depends on t, so it is issued first and the shifts and errors of the
// next layer down are fetched behind it: one memory round trip per layer on the critical path.
// The cost is then re-summed over the profile in layer order, which reproduces the sign of a
// zero exactly as the level-tracking sweep would (min(+0, -0) is order-blind).
// kLevelBlocks: 64-level blocks a lane holds (1 for S <= 64, 4 for S <= 255).
template <int kLevelBlocks>
struct LayerLevels {
    int shift[kLevelBlocks];      // tau[l][s] - m_l for s = 64 b + lane (INT32_MAX past S)
    float err[kLevelBlocks];
    int reach;                    // computed buckets of row l - 1 (1 for l = 0: only t = 0)
};

template <int kLevelBlocks>
__device__ __forceinline__ LayerLevels<kLevelBlocks> load_layer(
    const int32_t *__restrict__ tau, ErrRow er, const int32_t *__restrict__ meta, int l, int L,
    int S, int lane)
{
    LayerLevels<kLevelBlocks> v;
    const int m = meta[kMetaHeader + l];
    v.reach = l > 0 ? meta[kMetaHeader + L + l - 1] * kWave : 1;
#pragma unroll
    for (int b = 0; b < kLevelBlocks; ++b) {
        const int s = b * kWave + lane;
        v.shift[b] = INT32_MAX;
        v.err[b] = __builtin_inff();
        if (s < S) {
            v.shift[b] = tau[(size_t)l * S + s] - m;
            v.err[b] = er.at(s);
        }
    }
    return v;
}

// kBlocks: the walk through one block of layers [blocks.begin, blocks.end) of the small-record
// solve: rows come from the block record, the row below the block from its checkpoint; tstar
// holds the time to start from and receives the time below the block; the cost is re-summed
// after the first block (the last one walked).
template <int kLevelBlocks, bool kBlocks>
__global__ __launch_bounds__(kWalkThreads) void dp_backtrace_values(
    const int32_t *__restrict__ tau, ErrSource src, const int32_t *__restrict__ meta,
    const float *__restrict__ drec,
    int32_t *__restrict__ tstar, int K, int L, int S, int pitch,
    int16_t *__restrict__ profile, float *__restrict__ cost, Resume resume, Blocks blocks)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int k = blockIdx.x * (kWalkThreads / kWave) + threadIdx.x / kWave;
    if (k >= K)
        return;
    int16_t *prof = profile + (size_t)k * L;
    const int lb = kBlocks ? blocks.begin : 0;   // layers [lb, le) are walked
    const int le = kBlocks ? blocks.end : L;
    int t = tstar[k];
    if (t < 0) {
        for (int l = lb + lane; l < le; l += kWave)
            prof[l] = t == -1 ? -1 : -2;         // -1: no profile meets the budget
        return;
    }
    const float *drec_k = drec + (size_t)k * L * pitch;
    const int l0 = resume.start(k, L);           // rows below l0 are the incumbent's
    auto row_of = [&](int l) {
        if constexpr (kBlocks) {
            if (l >= lb)
                return blocks.block + ((size_t)k * blocks.stride + (l - lb)) * pitch;
            return blocks.ckpt + ((size_t)k * blocks.slots + (lb / blocks.stride - 1)) * pitch;
        } else {
            return (l < l0 ? resume.inc_rec : drec_k) + (size_t)l * pitch;
        }
    };
    float target = row_of(le - 1)[t];
    LayerLevels<kLevelBlocks> next =
        load_layer<kLevelBlocks>(tau, src.row(k, le - 1, L, S), meta, le - 1, L, S, lane);
    bool ok = true;
    for (int l = le - 1; l >= lb; --l) {
        const LayerLevels<kLevelBlocks> cur = next;
        const float *prow = row_of(l > 0 ? l - 1 : 0);       // row of layer l - 1
        // issue the gather of D_{l-1} first, then the next layer's table behind it
        int u[kLevelBlocks];
        float pv[kLevelBlocks];
        bool valid[kLevelBlocks];
#pragma unroll
        for (int b = 0; b < kLevelBlocks; ++b) {
            const long long uu = (long long)t - cur.shift[b];
            valid[b] = b * kWave < S && uu >= 0 && uu < cur.reach;
            u[b] = valid[b] ? (int)uu : 0;
            pv[b] = __builtin_inff();
            if (valid[b])
                pv[b] = l > 0 ? __builtin_nontemporal_load(&prow[u[b]]) : -0.0f;
        }
        if (l > lb)
            next = load_layer<kLevelBlocks>(tau, src.row(k, l - 1, L, S), meta, l - 1, L, S, lane);
        int found = -1, next_t = 0;
        float next_target = 0.0f;
#pragma unroll
        for (int b = 0; b < kLevelBlocks; ++b) {
            if (b * kWave < S && found < 0) {
                const bool match = valid[b] && pv[b] + cur.err[b] == target;
                const unsigned long long mask = __ballot(match);
                if (mask) {
                    const int first = __builtin_ctzll(mask);
                    found = b * kWave + first;
                    next_t = __shfl(u[b], first, kWave);
                    next_target = __shfl(pv[b], first, kWave);
                }
            }
        }
        if (found < 0) {     // cannot happen on a filled record
            ok = false;
            break;
        }
        if (lane == 0)
            prof[l] = (int16_t)found;
        t = next_t;
        target = next_target;
    }
    if (!ok) {
        for (int l = lane; l < L; l += kWave)
            prof[l] = -2;
        if (lane == 0) {
            cost[k] = __builtin_nanf("");
            if constexpr (kBlocks)
                tstar[k] = -2;                   // the blocks below are marked the same way
        }
        return;
    }
    if constexpr (kBlocks) {
        if (lb > 0) {                            // more blocks follow: hand the time down
            if (lane == 0)
                tstar[k] = t;
            return;
        }
    }
    // Lane 0 wrote the profile; make it visible to the wave, then re-sum the cost in layer order.
    // Lane i fetches the error of layer 64 b + i (all layers of a block of 64 in one round trip
    // instead of one after the other); the sum itself runs over the lanes in order.
    __threadfence();
    float acc = -0.0f;
    for (int base = 0; base < L; base += kWave) {
        const int l = base + lane;
        float e = 0.0f;
        if (l < L)
            e = src.row(k, l, L, S).at(prof[l]);
        const int n = min(kWave, L - base);
        for (int i = 0; i < n; ++i)
            acc += lane_value(e, i);
    }
    if (lane == 0)
        cost[k] = acc;
}

int launch_status()
{
    return hipGetLastError() == hipSuccess ? SPDY_DP_OK : SPDY_DP_ERR_LAUNCH;
}

// What the host keeps per device between calls: the number of compute units (asked once, not per
// solve) and where this device's copy of `scratch` lives.
constexpr int kMaxDevices = 64;
struct DeviceState {
    int units = 0;
    void *scratch = nullptr;
};
std::mutex g_device_lock;
DeviceState g_device[kMaxDevices];

// The current device's state; `with_scratch` also resolves the device address of `scratch`.
// Returns SPDY_DP_OK or SPDY_DP_ERR_LAUNCH (the runtime refused a query).
int device_state(bool with_scratch, DeviceState *out)
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return SPDY_DP_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(g_device_lock);
    DeviceState &st = g_device[device];
    if (st.units <= 0) {
        int units = 0;
        if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, device) !=
                hipSuccess || units <= 0)
            return SPDY_DP_ERR_LAUNCH;
        st.units = units;
    }
    if (with_scratch && !st.scratch) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return SPDY_DP_ERR_LAUNCH;
        st.scratch = ptr;
    }
    *out = st;
    return SPDY_DP_OK;
}

template <bool kLevel, bool kNarrow, bool kBlocks = false>
int launch_fill(const Layout &lay, const int32_t *tau, ErrSource src, Resume resume, int K, int L,
                int S, int B, char *ws, float *cost, hipStream_t q, Blocks blocks = Blocks{})
{
    int32_t *meta = reinterpret_cast<int32_t *>(ws + lay.meta_off);
    int32_t *shifts = reinterpret_cast<int32_t *>(ws + lay.shifts_off);
    int32_t *order = reinterpret_cast<int32_t *>(ws + lay.order_off);
    int32_t *start = reinterpret_cast<int32_t *>(ws + lay.start_off);
    int32_t *entry = reinterpret_cast<int32_t *>(ws + lay.entry_off);
    int32_t *tstar = reinterpret_cast<int32_t *>(ws + lay.tstar_off);
    uint8_t *choice = kLevel ? reinterpret_cast<uint8_t *>(ws + lay.record_off) : nullptr;
    float *drec = kLevel ? nullptr : reinterpret_cast<float *>(ws + lay.record_off);
    float *rows = reinterpret_cast<float *>(ws + (kLevel ? lay.rows_level : lay.rows_value));
    const int pitch = (int)lay.row;
    const int nchunks = pitch / kWave;
    const int s8 = (int)lay.s8;

    // The reduced row length is only known on the device, so the fill kernel is enqueued with an
    // LDS allocation that lets two workgroups share a compute unit and, if a row of the full
    // budget could need more, once more with a larger one (and once with the rows in global
    // memory if even that may not do); the prepare kernel picks the launch that fits and the
    // others return at once.  A row that the waves of a workgroup can hold in registers is
    // updated in place whatever the reduced length turns out to be, so one row bounds the need;
    // otherwise two rows alternate.
    // workgroups the chip holds at once: two per compute unit for either variant
    DeviceState dev;
    if (device_state(false, &dev) != SPDY_DP_OK)
        return SPDY_DP_ERR_LAUNCH;
    const int units = dev.units;
    // Workgroups that take turns at the priority pay off when a launch is one or two rounds of
    // workgroups (measured: K = 4 x units 4 % faster, 16 x units no gain and a slightly slower
    // kernel), and need pairs of workgroups to begin with.
    const bool turns = K > units && (long long)K <= 4LL * units;
    const int waves = nchunks < fill_waves<kLevel>() ? nchunks : fill_waves<kLevel>();
    const int max_group = turns ? group_limit<kLevel, true>() : group_limit<kLevel, false>();
    const size_t row_bytes = (lay.row + kHalo) * sizeof(float);
    const bool beyond_place = (long long)nchunks > (long long)waves * max_group;
    const size_t need = beyond_place ? 2 * row_bytes : row_bytes;
    const int lds_small = kLdsHalf;
    // D record: a row too long for the in-place launch may still be updated in place by a
    // workgroup of twice the waves that takes up to a whole compute unit's LDS (every length the
    // two-row launch could take is covered by it, so that launch is not enqueued then).
    constexpr bool can_widen = !kLevel && !kBlocks;
    const bool wide = can_widen && beyond_place;
    const int wide_waves = wide ? 2 * fill_waves<kLevel>() : 0;
    const int wide_group = group_limit<kLevel, false>();
    const int lds_wide = wide ? (int)(row_bytes < (size_t)kLdsBytes ? row_bytes : kLdsBytes) : 0;
    const int lds_large = (need <= (size_t)kLdsHalf || wide) ? 0
                          : (need <= (size_t)kLdsBytes ? (int)need : kLdsBytes);
    // whether the full budget's row may have to live in global memory (implies lay.may_spill)
    const bool in_memory =
        wide ? ((long long)nchunks > (long long)wide_waves * wide_group ||
                row_bytes > (size_t)kLdsBytes)
             : need > (size_t)kLdsBytes;
    auto in_place = turns ? dp_fill<kLevel, 1, kNarrow, kBlocks, true>
                          : dp_fill<kLevel, 1, kNarrow, kBlocks, false>;
    // A candidate that has a compute unit to itself gets twice the waves (the second half takes
    // every other pair of each layer's entries and needs a second row in LDS for its minima).
    constexpr bool can_split = !kLevel && kNarrow && !kBlocks;
    const bool split = can_split && K <= units;
    int place_threads = waves * kWave, place_lds = lds_small;
    if constexpr (can_split) {
        if (split) {
            in_place = dp_fill<kLevel, 1, kNarrow, kBlocks, false, true>;
            place_threads *= 2;
            place_lds *= 2;
            static_assert(2 * kLdsHalf <= kLdsBytes, "two half allocations fit one workgroup");
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(in_place),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kLdsBytes) != hipSuccess)
                return SPDY_DP_ERR_LAUNCH;
        }
    }
    auto two_rows = dp_fill<kLevel, 2, kNarrow, kBlocks>;
    auto in_global = dp_fill<kLevel, 0, kNarrow, kBlocks>;
    auto wide_place = dp_fill<kLevel, can_widen ? 3 : 1, kNarrow, kBlocks>;   // (3 when it exists)
    // The D record's global-row launch also has twice the waves (one workgroup per compute unit
    // with all of its LDS for the window; measured against two workgroups of the usual size with
    // half the LDS each: 11 % faster on a batch of four candidates per unit).
    const bool wide_global = can_widen && waves == fill_waves<kLevel>();
    const int global_waves = wide_global ? 2 * waves : waves;
    if constexpr (can_widen) {
        if (wide_global)
            in_global = dp_fill<kLevel, 4, kNarrow, kBlocks>;
    }
    if (wide &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(wide_place),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return SPDY_DP_ERR_LAUNCH;
    // always the same limit, so that calls from several host threads cannot undo each other's
    if (lds_large &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(two_rows),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return SPDY_DP_ERR_LAUNCH;
    // The global-row launch stages its tiles' windows in LDS: all of it with one workgroup per
    // compute unit; workgroups of the usual size take half of it when there are candidates for
    // two per unit (one sweeps while the other copies).
    const int lds_stage = (K > units && !wide_global) ? kLdsHalf : kLdsBytes;
    if (in_memory &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(in_global),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return SPDY_DP_ERR_LAUNCH;

    if (!(kBlocks && blocks.pass == 1))          // the block passes reuse pass 0's tables
        hipLaunchKernelGGL(dp_prepare, dim3(L + 1), dim3(256), 0, q, tau, K, 2 * units, L, S, s8,
                           B, waves, max_group, lds_small, lds_large, lds_stage,
                           kLevel ? 0 : (kNarrow ? 2 : 1), split ? 1 : 0, wide_waves, wide_group,
                           lds_wide, global_waves, meta, shifts, order, start, entry);
    const LevelTables tables{shifts, order, start, entry, s8};
    hipLaunchKernelGGL(in_place, dim3(K), dim3(place_threads), place_lds, q, src, meta, tables,
                       units, K, L, S, pitch, choice, drec, rows, tstar, cost, resume, blocks);
    if (wide)
        hipLaunchKernelGGL(wide_place, dim3(K), dim3(wide_waves * kWave), lds_wide, q, src, meta,
                           tables, units, K, L, S, pitch, choice, drec, rows, tstar, cost, resume,
                           blocks);
    if (lds_large)
        hipLaunchKernelGGL(two_rows, dim3(K), dim3(waves * kWave), lds_large, q, src, meta, tables,
                           units, K, L, S, pitch, choice, drec, rows, tstar, cost, resume, blocks);
    if (in_memory)
        hipLaunchKernelGGL(in_global, dim3(K), dim3(global_waves * kWave), lds_stage, q, src, meta, tables,
                           units, K, L, S, pitch, choice, drec, rows, tstar, cost, resume, blocks);
    return launch_status();
}

int validate(const Layout &lay, const void *workspace)
{
    if (lay.status != SPDY_DP_OK)
        return lay.status;
    if (!workspace)
        return SPDY_DP_ERR_NULL;
    return SPDY_DP_OK;
}

int fill_impl(const int32_t *tau, ErrSource src, int K, int L, int S, int B, float *cost,
              void *workspace, size_t workspace_bytes, void *stream, Resume resume = Resume{})
{
    if (!tau || !cost)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B, workspace_bytes);
    const int st = validate(lay, workspace);
    if (st != SPDY_DP_OK)
        return st;
    hipStream_t q = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    (void)hipGetLastError();
    if (S <= kWave)
        return lay.variant == kLevelRecord
                   ? launch_fill<true, true>(lay, tau, src, resume, K, L, S, B, ws, cost, q)
                   : launch_fill<false, true>(lay, tau, src, resume, K, L, S, B, ws, cost, q);
    return lay.variant == kLevelRecord
               ? launch_fill<true, false>(lay, tau, src, resume, K, L, S, B, ws, cost, q)
               : launch_fill<false, false>(lay, tau, src, resume, K, L, S, B, ws, cost, q);
}

int backtrace_impl(const int32_t *tau, ErrSource src, int K, int L, int S, int B,
                   int16_t *profile, float *cost, const void *workspace, size_t workspace_bytes,
                   void *stream, Resume resume = Resume{})
{
    if (!tau || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B, workspace_bytes);
    const int st = validate(lay, workspace);
    if (st != SPDY_DP_OK)
        return st;
    hipStream_t q = static_cast<hipStream_t>(stream);
    const char *ws = static_cast<const char *>(workspace);
    const int32_t *meta = reinterpret_cast<const int32_t *>(ws + lay.meta_off);
    const int32_t *tstar = reinterpret_cast<const int32_t *>(ws + lay.tstar_off);
    (void)hipGetLastError();
    if (lay.variant == kLevelRecord) {
        hipLaunchKernelGGL(dp_backtrace_levels, dim3((K + kWave - 1) / kWave), dim3(kWave), 0, q,
                           tau, src, meta, reinterpret_cast<const uint8_t *>(ws + lay.record_off),
                           tstar, K, L, S, (int)lay.row, profile, cost);
    } else {
        const int per_block = kWalkThreads / kWave;
        auto narrow = dp_backtrace_values<1, false>;
        auto wide = dp_backtrace_values<4, false>;
        hipLaunchKernelGGL(S <= kWave ? narrow : wide, dim3((K + per_block - 1) / per_block), dim3(kWalkThreads), 0, q, tau,
                           src, meta, reinterpret_cast<const float *>(ws + lay.record_off),
                           const_cast<int32_t *>(tstar), K, L, S, (int)lay.row, profile, cost,
                           resume, Blocks{});
    }
    return launch_status();
}

int solve_impl(const int32_t *tau, ErrSource src, int K, int L, int S, int B, int16_t *profile,
               float *cost, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!tau || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    const int st = fill_impl(tau, src, K, L, S, B, cost, workspace, workspace_bytes, stream);
    if (st != SPDY_DP_OK)
        return st;
    return backtrace_impl(tau, src, K, L, S, B, profile, cost, workspace, workspace_bytes, stream);
}

// The stride of the solve with checkpoints: the caller's, or about sqrt(L), which makes the
// checkpoints and the block record the same size.
int checkpoint_stride(int L, int stride)
{
    if (stride > 0)
        return stride < L ? stride : L;
    int j = 1;
    while ((long long)j * j < L)
        ++j;
    return j;
}

// Pass 0 over all layers (checkpoints, final time), then per block of `stride` layers, last
// first: fill the block's rows from the checkpoint below it and walk through them.
int checkpointed_impl(const int32_t *tau, ErrSource src, int K, int L, int S, int B, int stride,
                      int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    if (!tau || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    if (L <= 0)
        return SPDY_DP_ERR_DIM;
    const int j = checkpoint_stride(L, stride);
    const int nblocks = (L + j - 1) / j;
    const int slots = nblocks - 1;
    const Layout lay = make_layout(K, L, S, B, workspace_bytes, (long long)slots + j);
    int st = validate(lay, workspace);
    if (st != SPDY_DP_OK)
        return st;
    if (lay.variant != kValueRecord)
        return SPDY_DP_ERR_WORKSPACE;
    hipStream_t q = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    (void)hipGetLastError();
    Blocks blocks{};
    blocks.stride = j;
    blocks.slots = slots;
    blocks.ckpt = reinterpret_cast<float *>(ws + lay.record_off);
    blocks.block = blocks.ckpt + (size_t)K * slots * lay.row;
    auto fill = [&]() {
        return S <= kWave
                   ? launch_fill<false, true, true>(lay, tau, src, Resume{}, K, L, S, B, ws, cost,
                                                    q, blocks)
                   : launch_fill<false, false, true>(lay, tau, src, Resume{}, K, L, S, B, ws, cost,
                                                     q, blocks);
    };
    blocks.pass = 0;
    blocks.begin = 0;
    blocks.end = L;
    st = fill();
    if (st != SPDY_DP_OK)
        return st;
    const int32_t *meta = reinterpret_cast<const int32_t *>(ws + lay.meta_off);
    int32_t *tstar = reinterpret_cast<int32_t *>(ws + lay.tstar_off);
    const int per_block = kWalkThreads / kWave;
    blocks.pass = 1;
    for (int b = nblocks - 1; b >= 0; --b) {
        blocks.begin = b * j;
        blocks.end = (b + 1) * j < L ? (b + 1) * j : L;
        st = fill();
        if (st != SPDY_DP_OK)
            return st;
        auto narrow = dp_backtrace_values<1, true>;
        auto wide = dp_backtrace_values<4, true>;
        hipLaunchKernelGGL(S <= kWave ? narrow : wide, dim3((K + per_block - 1) / per_block), dim3(kWalkThreads), 0, q, tau,
                           src, meta, nullptr, tstar, K, L, S, (int)lay.row, profile, cost,
                           Resume{}, blocks);
        st = launch_status();
        if (st != SPDY_DP_OK)
            return st;
    }
    return SPDY_DP_OK;
}

int budgets_impl(const int32_t *tau, ErrSource src, int K, int L, int S, const int32_t *budgets,
                 int J, int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                 void *stream)
{
    if (!tau || !budgets || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    if (J <= 0)
        return SPDY_DP_ERR_DIM;
    int bmax = budgets[0];
    for (int j = 0; j < J; ++j) {
        if (budgets[j] < 0)
            return SPDY_DP_ERR_DIM;
        bmax = budgets[j] > bmax ? budgets[j] : bmax;
    }
    const Layout lay = make_layout(K, L, S, bmax, workspace_bytes);
    int st = validate(lay, workspace);
    if (st != SPDY_DP_OK)
        return st;
    if (lay.variant != kValueRecord)
        return SPDY_DP_ERR_WORKSPACE;            // the last row of D is only kept in the D record
    // one fill for the largest budget (cost[0..K) is scratch until its own walk back)
    st = fill_impl(tau, src, K, L, S, bmax, cost, workspace, workspace_bytes, stream);
    if (st != SPDY_DP_OK)
        return st;
    hipStream_t q = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    const int32_t *meta = reinterpret_cast<const int32_t *>(ws + lay.meta_off);
    int32_t *tstar = reinterpret_cast<int32_t *>(ws + lay.tstar_off);
    const float *drec = reinterpret_cast<const float *>(ws + lay.record_off);
    for (int j = 0; j < J; ++j) {
        float *cost_j = cost + (size_t)j * K;
        hipLaunchKernelGGL(dp_budget_argmin, dim3(K), dim3(256), 0, q, meta, drec, L, (int)lay.row,
                           budgets[j], tstar, cost_j);
        st = backtrace_impl(tau, src, K, L, S, bmax, profile + (size_t)j * K * L, cost_j,
                            workspace, workspace_bytes, stream);
        if (st != SPDY_DP_OK)
            return st;
    }
    return SPDY_DP_OK;
}

int resume_impl(const int32_t *tau, ErrSource src, const int32_t *first_layer, int K, int L, int S,
                int B, const void *incumbent, size_t incumbent_bytes, int16_t *profile,
                float *cost, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!tau || !first_layer || !incumbent || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B, workspace_bytes);
    int st = validate(lay, workspace);
    if (st != SPDY_DP_OK)
        return st;
    const Layout inc = make_layout(1, L, S, B, incumbent_bytes);
    if (inc.status != SPDY_DP_OK)
        return inc.status;
    if (lay.variant != kValueRecord || inc.variant != kValueRecord)
        return SPDY_DP_ERR_WORKSPACE;            // rows of D are only kept in the D record
    const char *a = static_cast<const char *>(incumbent);
    const char *b = static_cast<const char *>(workspace);
    if (a < b + workspace_bytes && b < a + incumbent_bytes)
        return SPDY_DP_ERR_WORKSPACE;            // the fill would overwrite the rows it resumes from
    Resume resume;
    resume.first_layer = first_layer;
    resume.inc_rec =
        reinterpret_cast<const float *>(static_cast<const char *>(incumbent) + inc.record_off);
    st = fill_impl(tau, src, K, L, S, B, cost, workspace, workspace_bytes, stream, resume);
    if (st != SPDY_DP_OK)
        return st;
    return backtrace_impl(tau, src, K, L, S, B, profile, cost, workspace, workspace_bytes, stream,
                          resume);
}

}  // namespace

extern "C" {

size_t spdy_dp_workspace_bytes(int K, int L, int S, int B)
{
    const Layout lay = make_layout(K, L, S, B, SIZE_MAX);
    return lay.status == SPDY_DP_OK ? lay.total_value : 0;
}

size_t spdy_dp_workspace_bytes_min(int K, int L, int S, int B)
{
    const Layout lay = make_layout(K, L, S, B, SIZE_MAX);
    return lay.status == SPDY_DP_OK ? lay.total_level : 0;
}

int spdy_dp_workspace_layout(int K, int L, int S, int B, size_t workspace_bytes, size_t out[8])
{
    if (!out)
        return SPDY_DP_ERR_NULL;
    const Layout lay = make_layout(K, L, S, B, workspace_bytes);
    if (lay.status != SPDY_DP_OK)
        return lay.status;
    out[0] = (size_t)lay.variant;
    out[1] = lay.meta_off;
    out[2] = lay.tstar_off;
    out[3] = lay.record_off;
    out[4] = lay.row;
    out[5] = (size_t)L;
    out[6] = (size_t)kMetaHeader;
    out[7] = (size_t)kRangeStride;
    return SPDY_DP_OK;
}

int spdy_dp_fill(const int32_t *tau, const float *err, int K, int L, int S, int B, float *cost,
                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return fill_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, B, cost, workspace,
                     workspace_bytes, stream);
}

int spdy_dp_backtrace(const int32_t *tau, const float *err, int K, int L, int S, int B,
                      int16_t *profile, float *cost, const void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return backtrace_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, B, profile, cost,
                          workspace, workspace_bytes, stream);
}

int spdy_dp_solve_batched(const int32_t *tau, const float *err, int K, int L, int S, int B,
                          int16_t *profile, float *cost, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return solve_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, B, profile, cost, workspace,
                      workspace_bytes, stream);
}

int spdy_dp_solve_batched_static(const int32_t *tau, const float *err, int K, int L, int S, int B,
                                 int16_t *profile, float *cost, void *stream)
{
    if (!tau || !err || !profile || !cost)
        return SPDY_DP_ERR_NULL;
    // sizes first: nothing is looked up or enqueued for a problem that does not fit
    const Layout lay = make_layout(K, L, S, B, SPDY_DP_STATIC_WORKSPACE_BYTES);
    if (lay.status == SPDY_DP_ERR_WORKSPACE)
        return SPDY_DP_ERR_STATIC_LIMIT;
    if (lay.status != SPDY_DP_OK)
        return lay.status;
    DeviceState dev;
    const int st = device_state(true, &dev);
    if (st != SPDY_DP_OK)
        return st;
    return solve_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, B, profile, cost,
                      dev.scratch, SPDY_DP_STATIC_WORKSPACE_BYTES, stream);
}

int spdy_dp_solve_sensitivities(const int32_t *tau, const float *c, const float *w, int K, int L,
                                int S, int B, int16_t *profile, float *cost, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    if (!c || !w)
        return SPDY_DP_ERR_NULL;
    return solve_impl(tau, ErrSource{nullptr, c, w}, K, L, S, B, profile, cost, workspace,
                      workspace_bytes, stream);
}

int spdy_dp_solve_budgets(const int32_t *tau, const float *err, int K, int L, int S,
                          const int32_t *budgets, int J, int16_t *profile, float *cost,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return budgets_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, budgets, J, profile, cost,
                        workspace, workspace_bytes, stream);
}

int spdy_dp_solve_from_incumbent(const int32_t *tau, const float *err, const int32_t *first_layer,
                                 int K, int L, int S, int B, const void *incumbent_workspace,
                                 size_t incumbent_bytes, int16_t *profile, float *cost,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return resume_impl(tau, ErrSource{err, nullptr, nullptr}, first_layer, K, L, S, B,
                       incumbent_workspace, incumbent_bytes, profile, cost, workspace,
                       workspace_bytes, stream);
}

size_t spdy_dp_workspace_bytes_checkpointed(int K, int L, int S, int B, int stride)
{
    if (L <= 0)
        return 0;
    const int j = checkpoint_stride(L, stride);
    const Layout lay = make_layout(K, L, S, B, SIZE_MAX, (long long)((L + j - 1) / j - 1) + j);
    return lay.status == SPDY_DP_OK ? lay.total_value : 0;
}

int spdy_dp_solve_checkpointed(const int32_t *tau, const float *err, int K, int L, int S, int B,
                               int stride, int16_t *profile, float *cost, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (!err)
        return SPDY_DP_ERR_NULL;
    return checkpointed_impl(tau, ErrSource{err, nullptr, nullptr}, K, L, S, B, stride, profile,
                             cost, workspace, workspace_bytes, stream);
}

const char *spdy_dp_strerror(int status)
{
    switch (status) {
    case SPDY_DP_OK: return "ok";
    case SPDY_DP_ERR_NULL: return "a required pointer is NULL";
    case SPDY_DP_ERR_DIM: return "K, L and S must be positive and B non-negative";
    case SPDY_DP_ERR_LEVELS: return "S exceeds 255 levels (a recorded level is one byte)";
    case SPDY_DP_ERR_WORKSPACE: return "workspace smaller than spdy_dp_workspace_bytes_min()";
    case SPDY_DP_ERR_OVERFLOW: return "problem size overflows the index arithmetic";
    case SPDY_DP_ERR_LAUNCH: return "HIP runtime refused a kernel launch";
    case SPDY_DP_ERR_STATIC_LIMIT:
        return "problem needs more than the built-in workspace of spdy_dp_solve_batched_static";
    default: return "unknown status";
    }
}

}  // extern "C"
