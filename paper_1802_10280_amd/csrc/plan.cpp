// Host-side plan builder for the LDS-tiled sconv kernel.
//
// Input: the stretched CSR of escoin_sconv_pack (offsets into the padded CHW input, Section
// 3.1).  Output: an opaque blob holding
//   - geometry tables, so the kernel needs no index arithmetic of its own:
//       items:   for every thread of a workgroup, the input words it stages per channel chunk:
//                offset in the (unpadded) input and the LDS byte that holds it; words of the
//                zero frame have no item and stay +0.0f -- pad_in folded into the staging;
//       lanes:   which 16-byte group of the window each lane of a wave reads and which four
//                output positions it owns;
//       dst_lut: for every computed position of a tile, where it goes in the E*F output plane
//                (-1 = a position on the padded pitch that is not an output);
//   - the nonzeros re-sorted per (output-channel group, channel chunk, wave, row, alignment
//     class), each with its LDS byte offset, so that the records a workgroup needs for one
//     chunk are one contiguous block it can copy into LDS (Section 3.3 stages colidx/value on
//     chip).
//
// LDS window.  The padded input of a tile is split into stride*stride phase planes (phase =
// coordinate mod stride), so that Algorithm 2's f(0,h,w) is h*pitch + w for every stride; each
// plane is `front` unused floats followed by rows of `pitch` floats.  A tap (r, s) of phase
// (r % stride, s % stride) reads, for position p, the window word
//     o + p,   o = front + (r / stride) * pitch + s / stride.
// A lane owns four consecutive positions 4g .. 4g+3 and fetches the aligned 16 bytes at
// 4g + (o - o % 4); the class o % 4 says how the four words it needs straddle that block and
// the next one, which the neighbouring lane has fetched (the kernel moves it across with a
// lane shift).  Class 3 is served from the following block and the previous lane instead.
#include <limits.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

#include "common.h"
#include "plan.h"

namespace escoin {

bool tiled_variant_exists(int K, int Q, int B);       // sconv_tiled.hip
bool tiled_wide_staging_exists(int K, int Q, int B);  // sconv_tiled.hip
bool tiled_dma_staging_exists(int K, int Q, int B);   // sconv_tiled.hip

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }
inline uint64_t align_up64(uint64_t a, uint64_t b) { return (a + b - 1) / b * b; }

constexpr int kLdsBudgetBytes = 160 * 1024;
constexpr int kRunLanes = 62;  // lanes of a 64-lane run that own outputs (both ends only lend data)

struct Geometry {
    int n_phases = 0;
    int phase_a[kMaxPhases], phase_b[kMaxPhases];
    std::vector<int> tap_phase;  // [R*S] index into phase_*
    std::vector<int> tap_class;  // [R*S] o % 4
    std::vector<int> tap_aoff;   // [R*S] aligned word offset the lane adds to its group base
    int max_aoff = 0;
};

// Cost of a class in lane-shift moves per record: 0, 1, 2 words from the next lane, or (class
// 3) one word from the previous lane.
inline int class_cost(int c) { return c == 0 ? 0 : (c == 2 ? 2 : 1); }

// Front padding of a phase plane: at least one whole group (the lane left of the first group
// reads it), and the residue that makes the taps' alignment classes cheapest.
int choose_front(const Dims& d, int pitch) {
    int best_front = 4, best_cost = INT_MAX;
    for (int front = 4; front < 8; ++front) {
        int cost = 0;
        for (int r = 0; r < d.R; ++r)
            for (int s = 0; s < d.S; ++s)
                cost += class_cost((front + (r / d.stride) * pitch + s / d.stride) % 4);
        if (cost < best_cost) {
            best_cost = cost;
            best_front = front;
        }
    }
    return best_front;
}

// Row pitch of one image inside a phase plane.
//   - stride 1: W + pad suffices instead of W + 2*pad.  The `pad` zero columns that follow a
//     row's W inputs serve as its right padding and, because rows follow each other without
//     gaps, as the left padding of what comes next; a tap never reaches further than that
//     (its column is at most Wp - 1, i.e. `pad - 1` past those zeros' first word).  A row of
//     outputs must fit as well: with more padding than the filter needs F exceeds W + pad.
//   - other strides: the width of a phase plane, ceil(Wp / stride).
//   - rounded up to a multiple of 4 when that costs at most 15 % more positions (then every
//     filter row has the same alignment classes: three instead of four for a 3-wide filter, so
//     longer record segments and fewer lane shifts), and always when several images share a
//     tile, so that a lane's four positions never straddle two images.
inline int image_pitch(const Dims& d, int NB) {
    const int p = d.stride == 1 ? std::max(d.W + d.pad, d.F) : ceil_div(d.Wp, d.stride), p4 = round_up(p, 4);
    return (NB > 1 || p4 * 100 <= p * 115) ? p4 : p;
}
// A tile that holds NB images lays them side by side: one wide image whose rows are the NB
// images' rows one after the other (row pitch NB * image pitch).  Consecutive lanes then read
// consecutive 16-byte groups whatever image they belong to (conflict-free: the group numbers of
// the 64 lanes advance by one per lane, which is what the 64 LDS banks want), and only the two
// ends of a run lend data instead of two lanes per image.
inline int wide_pitch(const Dims& d, int NB) { return NB * image_pitch(d, NB); }
// Floats of one channel's plane set (all NB images of one phase): the rows, the unused front,
// and zeros behind the last row for its taps' right padding; a multiple of 4 * NB so that
// the per-image share is a whole number of 16-byte groups.
inline int wide_plane_floats(const Dims& d, int NB, int front, int rows_in) {
    return round_up(front + rows_in * wide_pitch(d, NB) + 4 + (d.stride == 1 ? d.pad : 0), 4 * NB);
}
// Lane-table entries of a tile: its 16-byte groups and one lending group on either side.
inline int lane_entries(const Dims& d, int NB, int TH) { return ceil_div(TH * wide_pitch(d, NB), 4) + 2; }

int build_geometry(const Dims& d, int pitch, int front, Geometry* g) {
    g->n_phases = 0;
    g->tap_phase.assign((size_t)d.R * d.S, -1);
    g->tap_class.assign((size_t)d.R * d.S, 0);
    g->tap_aoff.assign((size_t)d.R * d.S, 0);
    g->max_aoff = 0;
    for (int r = 0; r < d.R; ++r) {
        for (int s = 0; s < d.S; ++s) {
            const int a = r % d.stride, b = s % d.stride;
            int ph = -1;
            for (int i = 0; i < g->n_phases; ++i)
                if (g->phase_a[i] == a && g->phase_b[i] == b) ph = i;
            if (ph < 0) {
                if (g->n_phases == kMaxPhases) return ESCOIN_ERANGE;
                ph = g->n_phases++;
                g->phase_a[ph] = a;
                g->phase_b[ph] = b;
            }
            const int o = front + (r / d.stride) * pitch + s / d.stride;
            const int cls = o % 4;
            const int aoff = o - cls + (cls == 3 ? 4 : 0);
            const size_t tap = (size_t)r * d.S + s;
            g->tap_phase[tap] = ph;
            g->tap_class[tap] = cls;
            g->tap_aoff[tap] = aoff;
            g->max_aoff = std::max(g->max_aoff, aoff);
        }
    }
    return ESCOIN_OK;
}

// Channel chunks: the first one holds CC0 channels, the others CC (the last one what is left).
inline int chunk_of(const PlanHeader& h, int c) { return c < h.CC0 ? 0 : 1 + (c - h.CC0) / h.CC; }
inline int chunk_start(const PlanHeader& h, int ch) { return ch == 0 ? 0 : h.CC0 + (ch - 1) * h.CC; }

// Fills every derived field of `h` from the knobs K, Q, B, WM, WS, CC, CC0, NB, TH (already set).
// n_mgroups is the count before long rows are split (build_plan_once may add groups).
int derive(const Dims& d, PlanHeader* h, Geometry* g) {
    h->pitch = wide_pitch(d, h->NB);
    h->pitch1 = image_pitch(d, h->NB);
    h->front = choose_front(d, h->pitch);
    int rc = build_geometry(d, h->pitch, h->front, g);
    if (rc != ESCOIN_OK) return rc;
    h->n_phases = g->n_phases;
    h->TH = std::min(h->TH, d.E);
    h->n_tiles = ceil_div(d.E, h->TH);
    h->rows_in = h->TH + (d.R - 1) / d.stride;
    h->plane_stride = wide_plane_floats(d, h->NB, h->front, h->rows_in) / h->NB;
    h->P4 = round_up(h->TH * h->pitch, 4);
    // lanes: the groups -1 .. P4/4 of the (wide) tile; a run of 64 lanes owns the outputs of
    // its 62 inner lanes, so consecutive runs overlap by two entries
    const int entries = lane_entries(d, h->NB, h->TH);
    const int runs = std::max(1, ceil_div(entries - 2, kRunLanes));
    h->WQ = ceil_div(runs, h->Q);
    h->CC = std::min(h->CC, d.C);
    // the staging key holds the channel inside the chunk in 14 bits
    if (h->CC > kMaxChunkChannels) return ESCOIN_ERANGE;
    h->CC0 = h->CC0 > 0 ? std::min(h->CC0, h->CC) : h->CC;
    h->n_chunks = d.C <= h->CC0 ? 1 : 1 + ceil_div(d.C - h->CC0, h->CC);
    h->CS = std::max(1, std::min(h->CS, h->n_chunks));
    h->WS = std::max(1, std::min(h->WS, h->WM));
    h->n_mgroups = (int)std::min<long long>(INT32_MAX, ((long long)d.M * h->WS + (long long)h->K * h->WM - 1) / ((long long)h->K * h->WM));
    // Behind the channel planes every window buffer keeps a stretch nothing writes: a record
    // that only fills up a batch points there and multiplies zeros, whatever the input holds.
    h->zero_floats = round_up(h->P4 + 16, 4);
    // two window buffers (the next chunk is fetched while the current one is consumed) plus a
    // zeroed tail
    const long long buf = (long long)h->n_phases * h->CC * h->NB * h->plane_stride + h->zero_floats;
    if (buf * 8 > kLdsBudgetBytes) return ESCOIN_ERANGE;
    h->buf_floats = (int)buf;
    // Lanes past the tile's last group still read: at most one group past it in a wave's first
    // run and 62 groups further for each following run of that wave.
    h->tail_floats = round_up(g->max_aoff + 16 + 4 * kRunLanes * (h->Q - 1), 4);
    if ((long long)h->NB * d.C * d.H * d.W >= (long long)INT32_MAX) return ESCOIN_ERANGE;
    if (h->WQ * h->WM > 16) return ESCOIN_ERANGE;  // at most 1024 threads per workgroup
    return ESCOIN_OK;
}

// Default knobs.  Every (K, Q, WM) choice and tile shape gets a relative cost, in units of the
// time one wave needs for one filter row: rounds of workgroups over the compute units, times
// a fixed part (set-up, first fetch, store) plus the K rows of one wave.  Two position runs
// per lane cost about 1.75x one; a wave runs faster when fewer waves share its SIMD; short
// channel chunks mean many barriers and much padding of the record batches; workgroups of few
// waves stage a larger share of the window per wave.  The constants were fitted to measured
// sweeps over the layer shapes of the bundled workloads.  The cheapest wins; ties go to more
// rows per wave.  The channel chunk then takes the LDS that is left.
void choose_defaults(const Dims& d, const escoin_sconv_tuning* t, PlanHeader* h) {
    // the last two are searched only when the caller asks for that K or Q
    static const int kPairs[7][2] = {{4, 2}, {2, 2}, {4, 1}, {2, 1}, {1, 1}, {1, 2}, {8, 1}};
    const int pitch = image_pitch(d, 1);
    const int img_groups = ceil_div(d.E * pitch, 4);
    int bestK = 2, bestQ = 1, bestTH = d.E, bestNB = 1, bestWM = 1, bestWS = 1;
    double best_score = -1.0;
    static const int kWaves[5] = {16, 12, 8, 6, 4};
    static const double kStageShare[5] = {1.0, 1.02, 1.08, 1.2, 1.4};
    // Splitting every channel over WS waves multiplies the workgroups by WS at the same K and
    // Q: what a launch with too few workgroups for the compute units needs (small batches).
    for (int WS = 1; WS <= 16; WS *= 2)
    for (int i = 0; i < 7 * 5; ++i) {
        if (t && t->WS > 0 && WS != 1) continue;  // the caller fixed it: one pass
        const int ws = (t && t->WS > 0) ? t->WS : WS;
        const int K = kPairs[i / 5][0], Q = kPairs[i / 5][1];
        if (t && t->K > 0 && t->K != K) continue;
        if (t && t->Q > 0 && t->Q != Q) continue;
        if (i / 5 == 5 && !(t && t->K == 1 && t->Q == 2)) continue;
        if (i / 5 == 6 && !(t && t->K == 8)) continue;
        if (!(t && t->Q > 0) && Q == 2 && d.stride > 1) continue;  // several phase planes: LDS goes to CC
        // fewer waves per workgroup give more workgroups (small batches need that) but every
        // wave then stages a larger share of the window
        int WM = kWaves[i % 5];
        double stage_share = kStageShare[i % 5];
        if (t && t->WM > 0) {
            if (i % 5) continue;
            WM = t->WM;
            stage_share = 1.0;
        } else if (WM > ceil_div(d.M * ws, K)) {
            if (i % 5 + 1 < 5 && kWaves[i % 5 + 1] >= ceil_div(d.M * ws, K)) continue;
            WM = ceil_div(d.M * ws, K);
        }
        if (ws > WM) continue;
        const int wave_groups = kRunLanes * Q;  // groups one wave can own
        const int mgroups = ceil_div(d.M * ws, K * WM);
        // a wave's share of its K rows, with a little lost to shorter record segments, and the
        // pass that adds the partial sums
        const double split = ws == 1 ? 1.0 : (1.0 + 0.15 * std::log2((double)ws)) / ws;
        const double merge = ws == 1 ? 0.0 : 0.25;
        auto consider = [&](int TH, int NB) {
            const long long wgs = (long long)ceil_div(d.E, TH) * ceil_div(d.N, NB) * mgroups;
            // the launch deals the workgroups out evenly over the 8 XCDs of 32 compute units
            const double rounds =
                (double)ceil_div(ceil_div((int)std::min<long long>(wgs, 1 << 20), 8), 32);
            // channels per chunk the staging registers allow
            const int rows = std::min(d.H, (TH - 1) * d.stride + d.R);
            const int runs = std::max(1, ceil_div(lane_entries(d, NB, TH) - 2, kRunLanes));
            const int WQ = ceil_div(runs, Q);
            if (WQ * WM > 16) return;
            const double cc_est = (double)kMaxItemsPerThread * 64 * WM * WQ / ((double)rows * d.W * NB);
            const double chunk = std::sqrt(std::min(1.0, std::min((double)d.C, cc_est) / 16.0));
            const int per_simd = ceil_div(WM * WQ, 4);
            const double crowd = per_simd >= 4 ? 1.0 : (per_simd == 3 ? 0.9 : 0.8);
            const double row_cost = Q == 2 ? (NB == 1 ? 1.75 : 1.9) : 1.0;
            const double cost = rounds * (0.6 + merge + K * split * row_cost * crowd / chunk) * stage_share;
            const double score = 1.0 / cost * (1.0 + 1e-3 * K);
            if (score > best_score) {
                best_score = score; bestK = K; bestQ = Q; bestTH = TH; bestNB = NB; bestWM = WM; bestWS = ws;
            }
        };
        if (t && (t->NB > 0 || t->TH > 0)) {  // the caller fixed the tile
            consider(t->TH > 0 ? std::min(t->TH, d.E) : d.E, t->NB > 0 ? t->NB : 1);
        } else if (img_groups <= wave_groups) {  // whole images: NB of them per workgroup
            int nb_max = 1;
            while (nb_max < d.N && lane_entries(d, nb_max + 1, d.E) - 2 <= wave_groups) ++nb_max;
            for (int NB = nb_max; NB >= 1; --NB) {
                if (ceil_div(lane_entries(d, NB, d.E) - 2, kRunLanes) < Q) break;  // idle position run
                consider(d.E, NB);
            }
        } else {  // a band of rows of one image
            int TH = std::max(1, wave_groups * 4 / pitch);
            TH = ceil_div(d.E, ceil_div(d.E, TH));  // even out the bands
            consider(TH, 1);
        }
    }
    if (best_score < 0) {  // the caller fixed a (K, Q) outside the table
        bestK = (t && t->K > 0) ? t->K : 2;
        bestQ = (t && t->Q > 0) ? t->Q : 1;
        bestWM = std::min(16, ceil_div(d.M, bestK));
    }
    h->K = bestK;
    h->Q = bestQ;
    h->B = (t && t->B > 0) ? t->B : 2;
    h->TH = (t && t->TH > 0) ? t->TH : bestTH;
    h->NB = (t && t->NB > 0) ? t->NB : ((t && t->TH > 0 && t->TH < d.E) ? 1 : bestNB);
    h->WM = (t && t->WM > 0) ? t->WM : bestWM;
    h->WS = (t && t->WS > 0) ? t->WS : bestWS;
    h->CC0 = (t && t->CC0 > 0) ? t->CC0 : 0;
    if (t && t->CC > 0) {
        h->CC = t->CC;
    } else {
        Geometry g;
        PlanHeader probe = *h;
        probe.CC = 1;
        const int lds_target = 128 * 1024;  // the rest holds the two record buffers
        if (derive(d, &probe, &g) == ESCOIN_OK) {
            const int per_c = 2 * probe.n_phases * probe.NB * probe.plane_stride * 4;
            // the most the LDS target allows; build_plan evens the chunks out
            h->CC = std::max(1, std::min(d.C, (lds_target - 8 * probe.zero_floats) / per_c));
        } else {
            h->CC = 1;
        }
    }
}

struct RowNz {
    uint32_t off_bytes;
    float val;
};

// One attempt with the knobs in `h`.
int build_plan_once(const Dims& d, const int32_t* rowptr, const int32_t* stretched, const float* value,
                    PlanHeader h, void* out, size_t out_bytes, size_t* bytes) {
    const int nnz = rowptr[d.M];
    Geometry g;
    int rc = derive(d, &h, &g);
    if (rc != ESCOIN_OK) return rc;
    h.nnz = nnz;
    const int threads = 64 * h.WQ * h.WM;

    // ---- decode every nonzero: stretched offset -> (c, r, s) -> (chunk, class, LDS byte offset)
    const int plane_in = d.Hp * d.Wp;
    const int chan_stride = h.NB * h.plane_stride;  // floats between channels of one phase
    std::vector<int> nz_chunk((size_t)nnz), nz_class((size_t)nnz);
    std::vector<uint32_t> nz_off((size_t)nnz);
    for (int j = 0; j < nnz; ++j) {
        const int off = stretched[j];
        if (off < 0 || off >= d.C * plane_in) return ESCOIN_EINVAL;
        const int c = off / plane_in;
        const int rem = off - c * plane_in;
        const int r = rem / d.Wp, s = rem - r * d.Wp;
        if (r >= d.R || s >= d.S) return ESCOIN_EINVAL;  // not an offset weight stretching makes
        const int chunk = chunk_of(h, c), cl = c - chunk_start(h, chunk);
        const int tap = r * d.S + s;
        const long long fl = ((long long)g.tap_phase[tap] * h.CC + cl) * chan_stride + g.tap_aoff[tap];
        // An explicit zero contributes nothing to any sum (the definition skips it as well), so
        // it gets no record: chunk -1.  Without values (size query) every entry counts.
        nz_chunk[j] = (value && value[j] == 0.0f) ? -1 : chunk;
        nz_class[j] = g.tap_class[tap];
        nz_off[j] = (uint32_t)(fl * 4);
    }
    // Per row, chunk and class: how many nonzeros.
    const int B = h.B;
    std::vector<int> rcc((size_t)d.M * h.n_chunks * kClasses, 0);
    std::vector<long long> nnz_row(d.M, 0);
    long long nnz_total = 0;
    for (int m = 0; m < d.M; ++m)
        for (int j = rowptr[m]; j < rowptr[m + 1]; ++j)
            if (nz_chunk[j] >= 0) {
                rcc[((size_t)m * h.n_chunks + nz_chunk[j]) * kClasses + nz_class[j]]++;
                nnz_row[m]++;
                nnz_total++;
            }

    // ---- output channels -> accumulator rows.  A wave has K accumulator rows; a channel takes
    // `parts` of them, in different waves of one workgroup, each with a share of its nonzeros
    // (the partial sums meet in LDS after the last chunk).  Every channel gets at least WS
    // parts; a channel whose nonzeros exceed a wave's fair share by more than a quarter gets
    // more, as long as accumulator rows are free (or, beyond twice the fair share, by adding a
    // channel group), so that one long CSR row cannot hold up its workgroup.
    const int slots_per_group = h.WM * h.K;
    std::vector<int> parts(d.M, h.WS);
    long long n_vrows = (long long)d.M * h.WS;
    long long n_groups = std::max<long long>(1, (n_vrows + slots_per_group - 1) / slots_per_group);
    for (;;) {
        const double fair = std::max(1.0, (double)nnz_total / ((double)n_groups * h.WM));
        int worst = -1;
        double worst_part = 0.0;
        for (int m = 0; m < d.M; ++m) {
            if (parts[m] >= h.WM) continue;
            const double sz = (double)nnz_row[m] / parts[m];
            if (sz > worst_part) { worst_part = sz; worst = m; }
        }
        if (worst < 0 || worst_part <= 1.25 * fair) break;
        if (n_groups * slots_per_group - n_vrows <= 0) {
            if (worst_part <= 2.0 * fair) break;
            ++n_groups;
            continue;
        }
        ++parts[worst];
        ++n_vrows;
    }
    if (n_groups > (1 << 24)) return ESCOIN_ERANGE;
    h.n_mgroups = (int)n_groups;
    const int bins = h.n_mgroups * h.WM;

    // Channels to groups, longest first, each to the group with the least work so far that
    // still has room for all its parts.
    std::vector<int> order(d.M);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return nnz_row[a] > nnz_row[b]; });
    std::vector<std::vector<int>> group_rows(h.n_mgroups);
    {
        std::vector<long long> load(h.n_mgroups, 0);
        std::vector<int> room(h.n_mgroups, slots_per_group);
        for (int i = 0; i < d.M; ++i) {
            const int m = order[i];
            int best = -1, roomiest = 0;
            for (int gi = 0; gi < h.n_mgroups; ++gi) {
                if (room[gi] > room[roomiest]) roomiest = gi;
                if (room[gi] >= parts[m] && (best < 0 || load[gi] < load[best])) best = gi;
            }
            if (best < 0) {  // fragmented free rows: fewer parts for this channel
                best = roomiest;
                parts[m] = room[best];
                if (parts[m] < 1) return ESCOIN_ERANGE;  // cannot happen: rows were counted above
            }
            group_rows[best].push_back(m);
            load[best] += nnz_row[m] + 1;
            room[best] -= parts[m];
        }
    }

    // Nonzeros of a (row, chunk, class) segment are dealt to the row's parts in turn, starting
    // at a part that rotates with the segment so that no part collects all the remainders.
    auto part_count = [&](int m, int ch, int cls, int part) {
        const int n = rcc[((size_t)m * h.n_chunks + ch) * kClasses + cls], P = parts[m];
        const int rot = (ch * kClasses + cls) % P;
        const int first = ((part - rot) % P + P) % P;  // index of the part's first nonzero
        return n / P + (first < n % P ? 1 : 0);
    };

    // Parts to waves.  The waves of a workgroup meet at a barrier after every chunk, so a
    // workgroup's time is the sum over chunks of its slowest wave: the parts, longest first,
    // each go to the wave (with a free accumulator row, and if possible without another part of
    // the same channel) where they raise that sum the least.
    std::vector<RowSlot> slot((size_t)bins * h.K);
    for (auto& sl : slot) { sl.m = -1; sl.my_region = -1; sl.first_region = 0; sl.n_partials = 0; }
    std::vector<int32_t> slot_part((size_t)bins * h.K, 0);
    std::vector<int32_t> group_regions(h.n_mgroups, 0);
    std::vector<int32_t> row_slot0(d.M, -1);        // index into row_slots of the row's part 0
    std::vector<int32_t> row_slots;                 // slot index of every part, rows one after the other
    row_slots.reserve((size_t)n_vrows);
    int max_regions = 0;
    {
        struct Item { int m, part; long long total; };
        std::vector<Item> items_v;
        std::vector<int> batches, wave_load((size_t)h.WM * h.n_chunks), peak(h.n_chunks), wave_rows(h.WM);
        std::vector<char> has_row;
        for (int mg = 0; mg < h.n_mgroups; ++mg) {
            items_v.clear();
            for (int m : group_rows[mg])
                for (int pt = 0; pt < parts[m]; ++pt) items_v.push_back({m, pt, 0});
            batches.assign(items_v.size() * (size_t)h.n_chunks, 0);
            for (size_t i = 0; i < items_v.size(); ++i)
                for (int ch = 0; ch < h.n_chunks; ++ch) {
                    int nb = 0;
                    for (int cls = 0; cls < kClasses; ++cls)
                        nb += ceil_div(part_count(items_v[i].m, ch, cls, items_v[i].part), B);
                    batches[i * h.n_chunks + ch] = nb;
                    items_v[i].total += nb;
                }
            std::vector<int> idx(items_v.size());
            std::iota(idx.begin(), idx.end(), 0);
            std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return items_v[a].total > items_v[b].total; });
            std::fill(wave_load.begin(), wave_load.end(), 0);
            std::fill(peak.begin(), peak.end(), 0);
            std::fill(wave_rows.begin(), wave_rows.end(), 0);
            has_row.assign((size_t)h.WM * group_rows[mg].size(), 0);
            // local index of a row inside this group
            std::vector<std::pair<int, int>> loc;  // (m, local)
            for (size_t i = 0; i < group_rows[mg].size(); ++i) loc.push_back({group_rows[mg][i], (int)i});
            std::sort(loc.begin(), loc.end());
            auto local_of = [&](int m) {
                return std::lower_bound(loc.begin(), loc.end(), std::make_pair(m, 0))->second;
            };
            std::vector<int> placed_wave(items_v.size(), -1), placed_k(items_v.size(), -1);
            for (int i : idx) {
                const int lm = local_of(items_v[i].m);
                int best = -1;
                long long best_rise = 0, best_total = 0;
                bool best_sibling = true;
                for (int w = 0; w < h.WM; ++w) {
                    if (wave_rows[w] >= h.K) continue;
                    const bool sibling = has_row[(size_t)w * group_rows[mg].size() + lm] != 0;
                    long long rise = 0, tot = 0;
                    for (int ch = 0; ch < h.n_chunks; ++ch) {
                        const int v = wave_load[(size_t)w * h.n_chunks + ch] + batches[(size_t)i * h.n_chunks + ch];
                        rise += std::max(0, v - peak[ch]);
                        tot += wave_load[(size_t)w * h.n_chunks + ch];
                    }
                    const bool better = best < 0 || (sibling != best_sibling ? !sibling
                                                     : (rise != best_rise ? rise < best_rise : tot < best_total));
                    if (better) { best = w; best_rise = rise; best_total = tot; best_sibling = sibling; }
                }
                if (best < 0) return ESCOIN_ERANGE;  // cannot happen: the group has room for its parts
                for (int ch = 0; ch < h.n_chunks; ++ch) {
                    int& v = wave_load[(size_t)best * h.n_chunks + ch];
                    v += batches[(size_t)i * h.n_chunks + ch];
                    peak[ch] = std::max(peak[ch], v);
                }
                has_row[(size_t)best * group_rows[mg].size() + lm] = 1;
                placed_wave[i] = best;
                placed_k[i] = wave_rows[best]++;
            }
            // slots and LDS regions: part 0 owns the channel, the other parts lend partial sums
            int regions = 0;
            size_t i = 0;
            for (int m : group_rows[mg]) {
                row_slot0[m] = (int32_t)row_slots.size();
                for (int pt = 0; pt < parts[m]; ++pt, ++i) {
                    const size_t si = ((size_t)mg * h.WM + placed_wave[i]) * h.K + placed_k[i];
                    slot[si].m = m;
                    slot_part[si] = pt;
                    if (pt == 0) {
                        slot[si].first_region = regions;
                        slot[si].n_partials = parts[m] - 1;
                    } else {
                        slot[si].my_region = regions++;
                    }
                    row_slots.push_back((int32_t)si);
                }
            }
            group_regions[mg] = regions;
            max_regions = std::max(max_regions, regions);
        }
    }
    h.max_regions = max_regions;

    // ---- staging items per tile: every input word the window needs and where it lives in LDS
    struct WindowWord {
        int32_t src, dst;  // offset inside an H*W input plane; word index inside a window buffer
    };
    std::vector<std::vector<WindowWord>> items(h.n_tiles);
    const long long phase_stride = (long long)h.CC * h.NB * h.plane_stride;
    for (int t = 0; t < h.n_tiles; ++t) {
        const int h0 = t * h.TH;
        for (int ph = 0; ph < g.n_phases; ++ph) {
            for (int i = 0; i < h.rows_in; ++i) {
                const int y = (h0 + i) * d.stride + g.phase_a[ph] - d.pad;
                if (y < 0 || y >= d.H) continue;
                for (int jx = 0; jx < h.pitch1; ++jx) {  // image 0; image nl sits nl * pitch1 further
                    const int x = jx * d.stride + g.phase_b[ph] - d.pad;
                    if (x < 0 || x >= d.W) continue;
                    WindowWord it;
                    it.src = y * d.W + x;
                    it.dst = (int32_t)(ph * phase_stride + h.front + i * h.pitch + jx);
                    items[t].push_back(it);
                }
            }
        }
    }
    // Input order (row, column): with full-width tiles every row is complete, so the words of
    // a tile are one stretch of each input plane.  When planes are whole 16-byte groups and the
    // stretch starts on one, it splits into runs of 4 consecutive, 16-byte aligned input words
    // (a run may span two rows) that one wide load can fetch, if the kernel variant has such
    // loads.  The loop below checks the alignment tile by tile.
    h.VW = ((d.H * d.W) % 4 == 0 && tiled_wide_staging_exists(h.K, h.Q, h.B)) ? 4 : 1;
    for (auto& v : items) {
        std::stable_sort(v.begin(), v.end(), [](const WindowWord& a, const WindowWord& b) { return a.src < b.src; });
        for (size_t i = 0; i < v.size() && h.VW > 1; ++i)
            if (v[i].src % h.VW != (int)(i % h.VW) || (i % h.VW && v[i].src != v[i - 1].src + 1)) h.VW = 1;
    }
    size_t n_items = 0;
    for (auto& v : items) n_items = std::max(n_items, v.size());
    if (n_items % h.VW) h.VW = 1;
    // Planes that are not whole 16-byte groups (7x7, 13x13): when a tile takes whole planes, the
    // words of one image and chunk are still one stretch of memory, (channel, row, column).  With
    // C and CC multiples of 4 that stretch starts 16-byte aligned and ends on a run boundary in
    // every chunk (also the shorter last one), so it splits into runs of 4 the same way; a run
    // may then span two channels.
    bool flat_runs = false;
    if (h.VW == 1 && tiled_wide_staging_exists(h.K, h.Q, h.B) && h.n_tiles == 1 && d.C % 4 == 0 &&
        h.CC % 4 == 0 && h.CC0 % 4 == 0 && (int)items[0].size() == d.H * d.W) {
        flat_runs = true;
        for (size_t i = 0; i < items[0].size(); ++i) flat_runs = flat_runs && items[0][i].src == (int)i;
        if (flat_runs) h.VW = 4;
    }
    n_items = std::max<size_t>(n_items, 1);
    if ((long long)n_items * h.CC * h.NB > (long long)kMaxItemsPerThread * threads) return ESCOIN_ERANGE;
    h.n_items = (int32_t)n_items;

    // ---- lanes of every position run
    const int gpi = h.P4 / 4;
    std::vector<LaneSlot> entries;
    for (int gi = -1; gi <= gpi; ++gi) {
        LaneSlot e;
        e.base_word = 4 * gi;
        e.pos0 = (gi >= 0 && gi < gpi) ? 4 * gi : -1;
        e.nloc = gi >= 0 ? ((4 * gi) % h.pitch) / h.pitch1 : 0;  // which of the images side by side
        entries.push_back(e);
    }
    const int runs = h.WQ * h.Q;
    std::vector<LaneSlot> lanes((size_t)runs * 64);
    for (int r = 0; r < runs; ++r)
        for (int l = 0; l < 64; ++l) {
            const size_t e = (size_t)r * kRunLanes + l;
            LaneSlot s;
            if (e < entries.size()) {
                s = entries[e];
                if (l == 0 || l == 63) s.pos0 = -1;  // run ends only lend their group
            } else {  // idle lane: shadow an entry in the same banks (16 groups back), own nothing
                long long idx = (long long)e;
                while (idx >= (long long)entries.size()) idx -= 16;
                s = entries[idx >= 0 ? (size_t)idx : e % entries.size()];
                s.pos0 = -1;
            }
            lanes[(size_t)r * 64 + l] = s;
        }

    // ---- count batches per (group, chunk, wave, row, class); a group's chunk block is contiguous
    const size_t seg_stride = 1 + (size_t)h.K * kClasses;
    std::vector<uint32_t> seg((size_t)bins * h.n_chunks * seg_stride, 0);
    std::vector<uint32_t> blk((size_t)h.n_mgroups * h.n_chunks * 2, 0);
    uint64_t total_batches = 0, max_block = 0;
    for (int mg = 0; mg < h.n_mgroups; ++mg) {
        for (int ch = 0; ch < h.n_chunks; ++ch) {
            if (total_batches > 0xFFFFFFF0ull) return ESCOIN_ERANGE;
            const uint64_t block_start = total_batches;
            for (int wm = 0; wm < h.WM; ++wm) {
                const int bin = mg * h.WM + wm;
                uint32_t* sg = &seg[((size_t)bin * h.n_chunks + ch) * seg_stride];
                sg[0] = (uint32_t)(total_batches - block_start);
                for (int k = 0; k < h.K; ++k) {
                    const size_t si = (size_t)bin * h.K + k;
                    const int m = slot[si].m;
                    for (int cls = 0; cls < kClasses; ++cls) {
                        const int nb = m < 0 ? 0 : ceil_div(part_count(m, ch, cls, slot_part[si]), B);
                        sg[1 + k * kClasses + cls] = (uint32_t)nb;
                        total_batches += nb;
                    }
                }
            }
            blk[((size_t)mg * h.n_chunks + ch) * 2] = (uint32_t)block_start;
            blk[((size_t)mg * h.n_chunks + ch) * 2 + 1] = (uint32_t)(total_batches - block_start);
            max_block = std::max(max_block, total_batches - block_start);
        }
    }
    const uint64_t n_records = (total_batches + 2) * B + 16;  // spare: copies round up, reads run ahead
    if (n_records > 0x7FFFFFFFull) return ESCOIN_ERANGE;
    h.n_records = (int32_t)n_records;
    // one record buffer: the largest block plus the batch the record prefetch reads past a
    // wave's last one
    const uint64_t rec_buf = align_up64(max_block * B * 8 + (uint64_t)B * 8 + 16, 64);
    h.rec_buf_bytes = (int32_t)rec_buf;
    // after the last chunk the same LDS holds the partial sums of split channels: one region
    // per lending accumulator row, 16 bytes per lane and position run of every position wave
    const uint64_t region_bytes = (uint64_t)h.WQ * h.Q * 64 * 16;
    const uint64_t lds_bytes = std::max(((uint64_t)2 * h.buf_floats + h.tail_floats) * 4 + 2 * rec_buf,
                                        (uint64_t)h.max_regions * region_bytes);
    if (lds_bytes > (uint64_t)kLdsBudgetBytes) return ESCOIN_ERANGE;
    h.lds_bytes = (int32_t)lds_bytes;

    // ---- launch order.  The workgroup ids are dealt to the 8 XCDs in contiguous ranges of the
    // job order.  Tile-major order lets the workgroups of one input tile share it in one L2, but
    // every XCD then reads the whole record stream; cutting the channel groups into MB blocks
    // (order: block, tile, group) makes an XCD read 1/MB of the records and MB/8 of the input
    // tiles instead of 1/8.  MB minimises input * MB + records * 8 / MB.
    {
        const double in_bytes = 4.0 * d.N * d.C * d.H * d.W, rec_bytes = 8.0 * (double)n_records;
        int best_mb = 1;
        double best = in_bytes + 8.0 * rec_bytes;
        for (int mb = 2; mb <= 8 && mb <= h.n_mgroups; mb *= 2) {
            const double t = in_bytes * mb + rec_bytes * 8.0 / mb;
            if (t < 0.9 * best) { best = t; best_mb = mb; }
        }
        h.MB = best_mb;
    }

    // ---- section layout
    uint64_t off = align_up64(sizeof(PlanHeader), 256);
    h.off_items = off;
    off = align_up64(off + (uint64_t)h.n_tiles * kMaxItemsPerThread * threads * sizeof(StageSlot), 256);
    h.off_lanes = off;
    off = align_up64(off + (uint64_t)lanes.size() * sizeof(LaneSlot), 256);
    h.off_dst_lut = off;
    off = align_up64(off + (uint64_t)h.n_tiles * h.P4 * 4, 256);
    h.off_perm = off;
    off = align_up64(off + (uint64_t)slot.size() * sizeof(RowSlot) + (uint64_t)h.n_mgroups * 4, 256);
    h.off_blk = off;
    off = align_up64(off + (uint64_t)blk.size() * 4, 256);
    h.off_seg = off;
    off = align_up64(off + (uint64_t)seg.size() * 4, 256);
    h.off_rec = off;
    off = align_up64(off + n_records * 8, 256);
    // Staging by global -> LDS copies: one DmaSlot per 16-byte slot of a window buffer's channel
    // planes, 64 slots per copy.  The room is set aside whenever the plan's runs of four input
    // words might qualify (decided below, once the staging table is written) and a wave would
    // issue no more than kMaxDmaPerWave copies per chunk.
    const int dma_copies = ceil_div((h.buf_floats - h.zero_floats) / 4, 64);
    const bool dma_room = h.VW == 4 && !flat_runs && tiled_dma_staging_exists(h.K, h.Q, h.B) &&
                          dma_copies <= kMaxDmaPerWave * h.WQ * h.WM;
    h.n_dma = 0;
    h.off_dma = off;
    if (dma_room) off = align_up64(off + (uint64_t)h.n_tiles * dma_copies * 64 * sizeof(DmaSlot), 256);
    h.off_zero = off;
    off = align_up64(off + 64, 256);
    h.total_bytes = off;
    *bytes = (size_t)off;
    if (!out) return ESCOIN_OK;
    if (out_bytes < off) return ESCOIN_ESIZE;

    char* base = (char*)out;
    std::memset(base, 0, (size_t)off);
    std::memcpy(base, &h, sizeof(h));

    // ---- items / lanes / dst_lut
    // The (channel, image, word) triples of a chunk are dealt to the threads round-robin, so a
    // wave's loads of one slot touch consecutive input words.
    StageSlot* slots = (StageSlot*)(base + h.off_items);
    bool wide_commit = h.VW == 4;
    int32_t* dst = (int32_t*)(base + h.off_dst_lut);
    for (int t = 0; t < h.n_tiles; ++t) {
        const int h0 = t * h.TH;
        // Runs of VW words are dealt to the threads round-robin (a wave's loads of one slot
        // touch consecutive runs); a thread's slots j*VW .. j*VW+VW-1 hold one run.
        const int n_runs = h.n_items / h.VW;
        const int flat_per_image = h.CC * h.n_items / 4;  // runs of one image's stretch
        const long long total_runs = flat_runs ? (long long)flat_per_image * h.NB : (long long)n_runs * h.CC * h.NB;
        for (int j = 0; j < kMaxItemsPerThread; ++j)
            for (int tid = 0; tid < threads; ++tid) {
                StageSlot sl;
                sl.src = -1;
                sl.key = 0;
                const long long run = tid + (long long)(j / h.VW) * threads;
                if (run < total_runs) {
                    int cl, nl, i;
                    if (flat_runs) {
                        nl = (int)(run / flat_per_image);
                        const int f = (int)(run - (long long)nl * flat_per_image) * 4 + j % 4;
                        cl = f / h.n_items;
                        i = f - cl * h.n_items;
                    } else {
                        const int cn = (int)(run / n_runs);
                        i = (int)(run - (long long)cn * n_runs) * h.VW + j % h.VW;
                        cl = cn / h.NB;
                        nl = cn - cl * h.NB;
                    }
                    if ((size_t)i < items[t].size()) {
                        sl.src = (nl * d.C + cl) * (d.H * d.W) + items[t][i].src;
                        // channel cl's plane set, then image nl's columns inside the wide rows
                        const long long word =
                            items[t][i].dst + (long long)cl * h.NB * h.plane_stride + nl * h.pitch1;
                        sl.key = (uint32_t)(word * 4) | ((uint32_t)cl << kKeyOffsetBits);
                    }
                }
                slots[((size_t)t * kMaxItemsPerThread + j) * threads + tid] = sl;
            }
        // can a run be committed with one 16-byte LDS write?
        if (h.VW == 4)
            for (int j = 0; j < kMaxItemsPerThread; j += 4)
                for (int tid = 0; tid < threads; ++tid) {
                    const StageSlot* q = &slots[((size_t)t * kMaxItemsPerThread + j) * threads + tid];
                    if (q[0].src < 0) continue;
                    for (int i = 0; i < 4; ++i) {
                        const StageSlot& w = q[(size_t)i * threads];
                        if (w.src < 0 || w.key != q[0].key + 4u * i || (q[0].key & 15u)) wide_commit = false;
                    }
                }
        for (int p = 0; p < h.P4; ++p) {
            const int hh = p / h.pitch, w = (p - hh * h.pitch) % h.pitch1;  // column inside its image
            dst[(size_t)t * h.P4 + p] =
                (hh < h.TH && h0 + hh < d.E && w < d.F) ? (h0 + hh) * d.F + w : -1;
        }
    }
    h.WW = wide_commit ? 4 : 1;
    // Every staged run lands on one aligned 16-byte slot: the same staging can be done by
    // global -> LDS copies, slot by slot (slots without a run read zeros).
    if (wide_commit && dma_room) {
        h.n_dma = dma_copies;
        DmaSlot* dma = (DmaSlot*)(base + h.off_dma);
        const size_t per_tile = (size_t)dma_copies * 64;
        for (size_t i = 0; i < (size_t)h.n_tiles * per_tile; ++i) { dma[i].src = -1; dma[i].chan = 0; }
        for (int t = 0; t < h.n_tiles; ++t)
            for (int j = 0; j < kMaxItemsPerThread; j += 4)
                for (int tid = 0; tid < threads; ++tid) {
                    const StageSlot& q = slots[((size_t)t * kMaxItemsPerThread + j) * threads + tid];
                    if (q.src < 0) continue;
                    const uint32_t byte = q.key & ((1u << kKeyOffsetBits) - 1);
                    DmaSlot& ds = dma[(size_t)t * per_tile + byte / 16];
                    ds.src = q.src;
                    ds.chan = (int32_t)(q.key >> kKeyOffsetBits);
                }
    }
    std::memcpy(base, &h, sizeof(h));  // the header once more, now with WW and n_dma
    std::memcpy(base + h.off_lanes, lanes.data(), lanes.size() * sizeof(LaneSlot));
    std::memcpy(base + h.off_perm, slot.data(), slot.size() * sizeof(RowSlot));
    std::memcpy(base + h.off_perm + slot.size() * sizeof(RowSlot), group_regions.data(), (size_t)h.n_mgroups * 4);
    std::memcpy(base + h.off_blk, blk.data(), blk.size() * 4);
    std::memcpy(base + h.off_seg, seg.data(), seg.size() * 4);

    // ---- records: per (group, chunk, wave, accumulator row, class) in CSR order, padded to whole
    // batches with (the stretch of zeros behind the channel planes, value 0.0f)
    RowNz* rec = (RowNz*)(base + h.off_rec);
    const uint32_t pad_off = (uint32_t)(((uint64_t)h.buf_floats - h.zero_floats) * 4 + 16);
    for (uint64_t i = 0; i < n_records; ++i) {
        rec[i].off_bytes = pad_off;
        rec[i].val = 0.0f;
    }
    std::vector<uint64_t> cursor;
    std::vector<int> seen((size_t)h.n_chunks * kClasses);
    for (int m = 0; m < d.M; ++m) {
        const int P = parts[m];
        // where each part's records of every (chunk, class) segment start
        cursor.assign((size_t)P * h.n_chunks * kClasses, 0);
        for (int pt = 0; pt < P; ++pt) {
            const size_t si = (size_t)row_slots[(size_t)row_slot0[m] + pt];
            const int bin = (int)(si / h.K), k = (int)(si % h.K), mg = bin / h.WM;
            for (int ch = 0; ch < h.n_chunks; ++ch) {
                const uint32_t* sg = &seg[((size_t)bin * h.n_chunks + ch) * seg_stride];
                uint64_t at = (uint64_t)blk[((size_t)mg * h.n_chunks + ch) * 2] + sg[0];
                for (int kk = 0; kk < k * kClasses; ++kk) at += sg[1 + kk];
                for (int cls = 0; cls < kClasses; ++cls) {
                    cursor[((size_t)pt * h.n_chunks + ch) * kClasses + cls] = at * B;
                    at += sg[1 + k * kClasses + cls];
                }
            }
        }
        std::fill(seen.begin(), seen.end(), 0);
        for (int j = rowptr[m]; j < rowptr[m + 1]; ++j) {
            if (nz_chunk[j] < 0) continue;
            const size_t sc = (size_t)nz_chunk[j] * kClasses + nz_class[j];
            const int pt = (seen[sc]++ + (int)(sc % P)) % P;
            uint64_t& at = cursor[(size_t)pt * h.n_chunks * kClasses + sc];
            rec[at].off_bytes = nz_off[j];
            rec[at].val = value[j];
            ++at;
        }
    }
    return ESCOIN_OK;
}

}  // namespace

// Builds the plan into `out` (or only sizes it when out == nullptr).  Returns a code; the
// byte count goes to *bytes.
int build_plan(const escoin_conv_desc* desc, const int32_t* rowptr, const int32_t* stretched,
               const float* value, const escoin_sconv_tuning* tuning, void* out, size_t out_bytes,
               size_t* bytes) {
    Dims d;
    int rc = make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (!rowptr || !bytes) return ESCOIN_EINVAL;
    if (rowptr[0] != 0) return ESCOIN_EINVAL;
    for (int m = 0; m < d.M; ++m)
        if (rowptr[m + 1] < rowptr[m]) return ESCOIN_EINVAL;
    const int nnz = rowptr[d.M];
    if (nnz > 0 && (!stretched || (out && !value))) return ESCOIN_EINVAL;
    if (tuning) {
        const int32_t* f = &tuning->K;
        for (int i = 0; i < 10; ++i)
            if (f[i] < 0) return ESCOIN_EINVAL;
    }

    PlanHeader h;
    std::memset(&h, 0, sizeof(h));
    h.magic = kPlanMagic;
    h.version = kPlanVersion;
    h.C = d.C; h.H = d.H; h.W = d.W; h.M = d.M; h.R = d.R; h.S = d.S;
    h.stride = d.stride; h.pad = d.pad; h.E = d.E; h.F = d.F;
    choose_defaults(d, tuning, &h);
    if (!tiled_variant_exists(h.K, h.Q, h.B)) return ESCOIN_EINVAL;
    // Knobs the caller did not fix shrink until the window, the staging registers and the
    // record block all fit: first the channel chunk, then the band height / images per group.
    const bool auto_cc = !(tuning && tuning->CC > 0);
    const bool auto_tile = !(tuning && (tuning->TH > 0 || tuning->NB > 0));
    const bool auto_cs = !(tuning && tuning->CS > 0);
    h.CS = auto_cs ? 1 : tuning->CS;
    for (;;) {
        // h.CC is the longest chunk that fits; the chunks of this attempt are evened out below it.
        // (A short first chunk, CC0 < CC, is the caller's choice: measured on the bundled layers
        // it gains 3-4 % when a layer runs alone with its input in the caches and loses 1-3 %
        // in a pass over several layers, where the first fetch comes from HBM.)
        PlanHeader trial = h;
        if (auto_cc) {
            // planes that are not whole 16-byte groups can still be staged with 16-byte loads
            // when every chunk is a multiple of 4 channels
            const bool quads = (d.H * d.W) % 4 != 0 && d.C % 4 == 0 && h.CC >= 8;
            const int cap = quads ? h.CC - h.CC % 4 : h.CC;
            trial.CC = ceil_div(d.C, ceil_div(d.C, cap));
            if (quads) trial.CC = std::min(cap, round_up(trial.CC, 4));
        }
        rc = build_plan_once(d, rowptr, stretched, value, trial, out, out_bytes, bytes);
        if (rc != ESCOIN_ERANGE) return rc;
        if (auto_cc && h.CC > 1) {
            h.CC = std::max(1, h.CC - std::max(1, h.CC / 8));
        } else if (auto_tile && h.NB > 1) {
            h.NB = h.NB / 2;
        } else if (auto_tile && h.TH > 1) {
            h.TH = (h.TH + 1) / 2;
        } else if (!(tuning && tuning->WM > 0) && h.WM > 1) {  // too many waves for this tile
            h.WM = h.WM / 2;
            if (!(tuning && tuning->WS > 0)) h.WS = std::min(h.WS, h.WM);
        } else {
            return rc;
        }
    }
}

}  // namespace escoin

extern "C" {

int escoin_sconv_plan_size(const escoin_conv_desc* desc, const int32_t* rowptr,
                           const int32_t* colidx_stretched, const escoin_sconv_tuning* tuning,
                           size_t* plan_bytes) {
    return escoin::build_plan(desc, rowptr, colidx_stretched, nullptr, tuning, nullptr, 0, plan_bytes);
}

int escoin_sconv_plan_build(const escoin_conv_desc* desc, const int32_t* rowptr,
                            const int32_t* colidx_stretched, const float* value,
                            const escoin_sconv_tuning* tuning, void* plan, size_t plan_bytes) {
    if (!plan) return ESCOIN_EINVAL;
    size_t need = 0;
    return escoin::build_plan(desc, rowptr, colidx_stretched, value, tuning, plan, plan_bytes, &need);
}

}  // extern "C"
