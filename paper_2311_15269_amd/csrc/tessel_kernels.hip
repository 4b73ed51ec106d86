// HIP kernels (gfx950) that score repetend candidates: one candidate per lane.
//
// Per candidate (Tessel, arXiv 2311.15269; Alg. 1, body of the loop over repetends):
//   decode   index -> lead vector (n_i of Eq. 3) + per-device block orders
//   build    walk the orders in an executable (topological) sequence, detect orders that
//            can never run, repair them in the REPAIR space, track the per-device memory
//            prefix (Eq. 1 [2]) and leave a compact "program" of the window
//   period   the repetend time t_R of Eq. 4 (with compaction of neighbouring repetends):
//            the least period of the rigidly repeated window.  The window is a max-plus
//            linear map on (device free times, end times of the micro-batches that are in
//            flight at the window boundary); its growth rate is the maximum cycle ratio
//   argmin   (period, index) lexicographic, lane -> wave -> block record -> grid merge
//
// Two kernels compute the same thing:
//   eval_kernel       general: multi-device blocks, cyclic device scan, 16-bit program in LDS,
//                     Karp's formula over V+1 sweeps; also decodes the best candidate
//   eval_fast_kernel  single-device blocks: bit-mask build, program words in VGPRs, eigenvector
//                     test after every sweep; what it cannot finish goes to the general kernel
//
// State that is indexed per lane at run time (device records, micro-batch tokens) lives in
// LDS laid out [slot][lane], which is bank-conflict free for any per-lane slot.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <stdlib.h>
#include <algorithm>

#include "tessel_device.h"

namespace tessel {


struct BlockRec {
    int32_t  period;
    uint32_t n_retried;          // candidates whose first sweeps found no eigenvector (they got more in the same launch)
    uint64_t index;
    uint32_t n_status[kNumStatus];
    uint32_t n_evaluated;
    uint32_t n_sweeps;           // window sweeps spent on period computations
    uint32_t n_blocks;           // blocks placed by the build (fast kernel)
    uint32_t pad;
};

constexpr uint32_t kDrawLeadBase = 0u;
constexpr uint32_t kDrawOrdBase = 128u;

// ------------------------------------------------------------------ 4-bit counters per type
// next micro-batch index of every block type: lead + occurrences placed, 4 bits each
struct Mu {
    uint64_t lo, hi;
    static constexpr int kTypeBits = 5;          // of a program entry of the path for graphs
    __device__ __forceinline__ void clear() { lo = 0; hi = 0; }
    __device__ __forceinline__ uint32_t get(uint32_t g) const
    {
        uint64_t w = g < 16 ? lo : hi;
        return (uint32_t)(w >> ((g & 15u) * 4u)) & 15u;
    }
    __device__ __forceinline__ void set(uint32_t g, uint32_t v)
    {
        uint64_t m = 15ull << ((g & 15u) * 4u), x = (uint64_t)v << ((g & 15u) * 4u);
        if (g < 16) lo = (lo & ~m) | x; else hi = (hi & ~m) | x;
    }
    __device__ __forceinline__ void inc(uint32_t g)
    {
        uint64_t x = 1ull << ((g & 15u) * 4u);
        if (g < 16) lo += x; else hi += x;
    }
};

// the same for up to 64 block types and windows of up to 16 micro-batches, 8 bits each (problems that only the general
// kernel's path for graphs takes)
struct MuWide {
    uint64_t w[8];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int k = 0; k < 8; k++) w[k] = 0;
    }
    __device__ __forceinline__ uint64_t word(uint32_t g) const
    {
        const uint64_t a = g & 8u ? w[1] : w[0], b = g & 8u ? w[3] : w[2], c = g & 8u ? w[5] : w[4], d = g & 8u ? w[7] : w[6];
        const uint64_t lo = g & 16u ? b : a, hi = g & 16u ? d : c;
        return g & 32u ? hi : lo;
    }
    __device__ __forceinline__ uint32_t get(uint32_t g) const { return (uint32_t)(word(g) >> ((g & 7u) * 8u)) & 255u; }
    __device__ __forceinline__ void add(uint32_t g, uint64_t x)
    {
#pragma unroll
        for (int k = 0; k < 8; k++) w[k] += (g >> 3) == (uint32_t)k ? x : 0ull;
    }
    __device__ __forceinline__ void set(uint32_t g, uint32_t v)
    {
        const uint32_t sh = (g & 7u) * 8u;
        add(g, ((uint64_t)v << sh) - (word(g) & (255ull << sh)));
    }
    __device__ __forceinline__ void inc(uint32_t g) { add(g, 1ull << ((g & 7u) * 8u)); }
    static constexpr int kTypeBits = 6;          // of a program entry
};

__device__ __forceinline__ uint32_t byte_of(uint32_t packed, uint32_t y) { return (packed >> (8u * y)) & 0xFFu; }

// entry y of eight: a select tree, so that the table comes through scalar loads
template <class T>
__device__ __forceinline__ T sel8(const T (&v)[kMaxLTW], uint32_t y)
{
    const T a = y & 1u ? v[1] : v[0], b = y & 1u ? v[3] : v[2], c = y & 1u ? v[5] : v[4], d = y & 1u ? v[7] : v[6];
    const T lo = y & 2u ? b : a, hi = y & 2u ? d : c;
    return y & 4u ? hi : lo;
}
__device__ __forceinline__ uint32_t sel4u(const uint32_t (&v)[kMaxLT], uint32_t y)
{
    uint32_t a = y & 1u ? v[1] : v[0];
    uint32_t b = y & 1u ? v[3] : v[2];
    return y & 2u ? b : a;
}

__device__ __forceinline__ int sel4(const int32_t (&v)[kMaxLTW], uint32_t y)
{
    int a = y & 1u ? v[1] : v[0];
    int b = y & 1u ? v[3] : v[2];
    return y & 2u ? b : a;
}

// remove the 2-bit entry at position pos (entries above move down)
__device__ __forceinline__ uint64_t remove_at(uint64_t x, uint32_t pos)
{
    uint64_t low = x & ((1ull << (2u * pos)) - 1ull);
    uint64_t high = ((x >> (2u * pos)) >> 2) << (2u * pos);
    return low | high;
}

// position of the first entry equal to y among the first len entries, or 64 if none
__device__ __forceinline__ uint32_t find_first(uint64_t x, uint32_t len, uint32_t y)
{
    uint64_t z = x ^ (0x5555555555555555ull * y);
    uint64_t hit = ~(z | (z >> 1)) & 0x5555555555555555ull;
    if (len < 32) hit &= (1ull << (2u * len)) - 1ull;
    return hit ? (uint32_t)__builtin_ctzll(hit) >> 1 : 64u;
}

// ------------------------------------------------------------------ one window sweep (general kernel)
// Program entry: bits 0-4 home code of the block type (device*4 + symbol), bits 5-10 token
// slot.  s = max(free time of its device(s), end of the micro-batch's previous block);
// both become s + t.  A chain's first block reads a token slot nobody has written: 0.
template <bool TP>
__device__ __forceinline__ void sweep_window(const KParams &P, const uint16_t *prog, uint32_t *state,
                                             const int32_t *t_tab, const uint32_t *mask_tab)
{
    const int total = P.total;
    for (int k = 0; k < total; k++) {
        uint32_t e = prog[k * kWave];
        uint32_t loc = e & 31u, ts = e >> 5;
        uint32_t tok = state[ts * kWave];
        uint32_t t = (uint32_t)t_tab[loc];
        if (!TP) {
            uint32_t ds = loc >> 2;
            uint32_t en = max(state[ds * kWave], tok) + t;
            state[ds * kWave] = en;
            state[ts * kWave] = en;
        } else {
            uint32_t mask = mask_tab[loc], s = tok;
            for (int d = 0; d < P.D; d++)
                if (mask >> d & 1u) s = max(s, state[d * kWave]);
            uint32_t en = s + t;
            for (int d = 0; d < P.D; d++)
                if (mask >> d & 1u) state[d * kWave] = en;
            state[ts * kWave] = en;
        }
    }
    // window boundary: micro-batches mu >= N_R are mu - N_R of the next window
    for (int p = 0; p < P.npaths; p++)
        for (int mu = 0; mu < P.NR; mu++) {
            int base = P.D + p * 2 * P.NR + mu;
            state[base * kWave] = state[(base + P.NR) * kWave];
            state[(base + P.NR) * kWave] = 0;
        }
}

__device__ __forceinline__ int reduced_slot(const KParams &P, int v)
{
    if (v < P.D) return v;
    int p = (v - P.D) / P.NR, mu = (v - P.D) % P.NR;
    return P.D + p * 2 * P.NR + mu;
}

// Least period of the repeated window = ceil(maximum cycle ratio) of the max-plus map x -> F(x)
// that one sweep applies to the V = D + npaths*N_R boundary values (plus the constant 0 that
// keeps start times non-negative).  Karp: with x(j) the vector after j+1 sweeps from 0 and
// n = V+1 sweeps in total, lambda = max_v min_{j<n-1} (x_v(n-1) - x_v(j)) / (n-1-j).
// Two passes over the same sweeps so that no history has to be stored.  (General kernel.)
// Before that, the shortcut the fast kernel lives on: iterate x <- F(x) from 0; as soon as every boundary value that
// means anything (`live`: devices with blocks, micro-batches that are in flight at the boundary) has grown by the
// same delta over one sweep, x is an eigenvector and delta the maximum cycle ratio, exactly.
constexpr int kGeneralTries = 6;
template <int VM, bool TP>
__device__ __forceinline__ int least_period(const KParams &P, const uint16_t *prog, uint32_t *state, const int32_t *t_tab,
                            const uint32_t *mask_tab, uint32_t live)
{
    const int V = P.nsweeps - 1, n = P.nsweeps;
    uint32_t xn[VM], bn[VM], bd[VM];
    for (int s = 0; s < P.nslots; s++) state[s * kWave] = 0;
    {
        uint32_t *prev = xn;
#pragma unroll
        for (int v = 0; v < VM; v++) prev[v] = 0;
        bool done = false;
        uint32_t T = 0;
        for (int j = 0; j < kGeneralTries; j++) {
            if (__ballot(!done) == 0) break;
            sweep_window<TP>(P, prog, state, t_tab, mask_tab);
            bool same = true, have = false;
            uint32_t delta = 0;
#pragma unroll
            for (int v = 0; v < VM; v++) {
                if (v < V) {
                    const uint32_t x = state[reduced_slot(P, v) * kWave];
                    const uint32_t dv = x - prev[v];
                    prev[v] = x;
                    if (live >> v & 1u) {
                        if (!have) { delta = dv; have = true; }
                        else if (dv != delta) same = false;
                    }
                }
            }
            if (!done && same && have) { T = delta; done = true; }
        }
        // every lane of the wave is here for a candidate that needs a period (the caller's lanes diverged before)
        if (done) return (int)T;
    }
    for (int s = 0; s < P.nslots; s++) state[s * kWave] = 0;
    for (int j = 0; j < n; j++) sweep_window<TP>(P, prog, state, t_tab, mask_tab);
#pragma unroll
    for (int v = 0; v < VM; v++) {
        xn[v] = v < V ? state[reduced_slot(P, v) * kWave] : 0u;
        bn[v] = 0xFFFFFFFFu; bd[v] = 1u;
    }
    for (int s = 0; s < P.nslots; s++) state[s * kWave] = 0;
    for (int j = 0; j < n - 1; j++) {
        sweep_window<TP>(P, prog, state, t_tab, mask_tab);
        uint32_t den = (uint32_t)(n - 1 - j);
#pragma unroll
        for (int v = 0; v < VM; v++) {
            if (v < V) {
                uint32_t a = xn[v] - state[reduced_slot(P, v) * kWave];
                // a/den < bn/bd  <=>  a*bd < bn*den   (all below 2^31, checked at problem creation)
                bool better = bn[v] == 0xFFFFFFFFu || (uint64_t)a * bd[v] < (uint64_t)bn[v] * den;
                if (better) { bn[v] = a; bd[v] = den; }
            }
        }
    }
    uint32_t T = 0;
#pragma unroll
    for (int v = 0; v < VM; v++) {
        if (v < V) {
            uint32_t c = (bn[v] + bd[v] - 1u) / bd[v];
            T = max(T, c);
        }
    }
    return (int)T;
}

// ------------------------------------------------------------------ candidate decoding
// index -> leads (4-bit counters by block type id) and, per device, the order of its blocks as
// 2-bit local symbols (first block in the lowest bits).  Returns kOk or the structural reject
// reason of the FACTORIAL space.
// (Problems with more than four block types on a device, sampled spaces only: the third bit of the symbol at position p
// is bit p of rem2[d].)
template <int DM, class CNT = Mu>
__device__ __forceinline__ int decode_candidate(const KParams &P, uint64_t idx, uint64_t (&rem)[DM], int (&remlen)[DM], CNT &mu,
                                                uint32_t (&rem2)[DM])
{
    const uint32_t NR = (uint32_t)P.NR;
    mu.clear();
#pragma unroll
    for (int d = 0; d < DM; d++) rem2[d] = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) { rem[d] = 0; remlen[d] = 0; }
    if (P.space == kFactorial) {
        uint64_t rest = idx;
        bool dup = false, tpm = false;
        uint64_t seen_types = 0;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= P.D) continue;
            const uint32_t n = (uint32_t)P.ntd[d] * NR;
            uint32_t r = (uint32_t)(rest % P.cdev[d]);
            rest /= P.cdev[d];
            uint64_t list = P.init_list[d], o = 0;
            uint32_t firstlab = 0xFFFFFFFFu, seencnt = 0;
            for (uint32_t pos = 0; pos < n; pos++) {
                uint32_t f = P.fact[n - 1 - pos];
                uint32_t digit = r / f;
                r -= digit * f;
                uint32_t code = (uint32_t)(list >> (5u * digit)) & 31u;
                uint64_t low = list & ((1ull << (5u * digit)) - 1ull);
                list = low | (((list >> (5u * digit)) >> 5) << (5u * digit));
                uint32_t y = code >> 3, lab = code & 7u;
                o |= (uint64_t)y << (2u * pos);
                uint32_t fl = byte_of(firstlab, y), sc = byte_of(seencnt, y);
                if (fl == 0xFFu) firstlab = (firstlab & ~(0xFFu << (8u * y))) | (lab << (8u * y));
                else {
                    uint32_t want = fl + sc;                 // labels continue cyclically (Property 1)
                    if (want >= NR) want -= NR;
                    if (lab != want) dup = true;
                }
                seencnt += 1u << (8u * y);
            }
            rem[d] = o; remlen[d] = (int)n;
            for (int y = 0; y < P.ntd[d]; y++) {
                uint32_t g = byte_of(P.type_of[d], (uint32_t)y), fl = byte_of(firstlab, (uint32_t)y);
                if (seen_types >> g & 1u) { if (mu.get(g) != fl) tpm = true; }
                else { mu.set(g, fl); seen_types |= 1ull << g; }
            }
        }
        if (dup) return kDup;
        if (tpm) return kTpMismatch;
        if (P.dag) {
            for (int e = 0; e < P.ndeps; e++)
                if (mu.get(P.dsrc[e]) < mu.get(P.ddst[e])) return kProp2;
        } else
        for (int g = 0; g < P.K; g++) {
            int p = P.pred[g];
            if (p >= 0 && mu.get((uint32_t)p) < mu.get((uint32_t)g)) return kProp2;
        }
    } else if (P.space == kCanonical) {
        uint64_t rest = idx;
        const uint32_t B = NR + 1;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= P.D) continue;
            const uint32_t n = (uint32_t)P.ntd[d] * NR;
            uint64_t r = rest % P.cdev[d];
            rest /= P.cdev[d];
            uint32_t c[kMaxLT];
#pragma unroll
            for (int y = 0; y < kMaxLT; y++) c[y] = y < P.ntd[d] ? NR : 0u;
            uint64_t o = 0;
            for (uint32_t pos = 0; pos < n; pos++) {
                bool chosen = false;
#pragma unroll
                for (int y = 0; y < kMaxLT; y++) {
                    if (!chosen && c[y] > 0) {
                        c[y]--;
                        uint64_t w = P.wtab[((c[0] * B + c[1]) * B + c[2]) * B + c[3]];
                        if (r < w) { o |= (uint64_t)y << (2u * pos); chosen = true; }
                        else { r -= w; c[y]++; }
                    }
                }
            }
            rem[d] = o; remlen[d] = (int)n;
        }
        const int8_t *row = P.leadtab + rest * (uint64_t)P.K;
        for (int g = 0; g < P.K; g++) mu.set((uint32_t)g, (uint32_t)row[g]);
    } else {
        uint64_t z = mix64(P.seed + 0x9E3779B97F4A7C15ULL * (idx + 1));
        const uint32_t a = (uint32_t)z, b = (uint32_t)(z >> 32);
        if (P.has_fixed) {
            for (int g = 0; g < P.K; g++) mu.set((uint32_t)g, P.fixed[g]);
        } else if (P.dag) {
            // consumers before producers: a type's lead is the largest (consumer's lead + step) over its dependencies
            for (int k = 0; k < P.K; k++) {
                const uint32_t i = P.rtopo[k];
                uint32_t lead = 0;
                for (int e = 0; e < P.ndeps; e++) {
                    if (P.dsrc[e] != i) continue;
                    const uint32_t u = (stream_word(a, b, (kDrawLeadBase + (uint32_t)e) >> 1) >> (16u * ((uint32_t)e & 1u))) & 0xFFFFu;
                    const uint32_t step = (P.dcross[e] && u < P.step_q16) ? 1u : 0u;
                    lead = max(lead, mu.get(P.ddst[e]) + step);
                }
                mu.set(i, min(NR - 1u, lead));
            }
        } else {
            for (int k = 0; k < P.K; k++) {
                uint32_t i = P.rtopo[k];
                int j = P.succ[i];
                uint32_t lead = 0;
                if (j >= 0) {
                    uint32_t e = kDrawLeadBase + P.edge_out[i];
                    uint32_t u = (stream_word(a, b, e >> 1) >> (16u * (e & 1u))) & 0xFFFFu;
                    uint32_t step = (P.cross_out[i] && u < P.step_q16) ? 1u : 0u;
                    lead = min(NR - 1u, mu.get((uint32_t)j) + step);
                }
                mu.set(i, lead);
            }
        }
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= P.D) continue;
            const uint32_t n = (uint32_t)P.ntd[d] * NR;
            uint32_t c0 = P.ntd[d] > 0 ? NR : 0u, c1 = P.ntd[d] > 1 ? NR : 0u, c2 = P.ntd[d] > 2 ? NR : 0u;
            uint32_t cw = 0;                              // up to eight types: the blocks left of every type, four bits each
            for (int y = 0; y < P.ntd[d]; y++) cw |= NR << (4 * y);
            uint64_t o = 0;
            uint32_t o2 = 0;
            uint32_t word = 0;
            for (uint32_t pos = 0; pos < n; pos++) {
                uint32_t j = kDrawOrdBase + 32u * (uint32_t)d + pos;
                if ((pos & 1u) == 0) word = stream_word(a, b, j >> 1);
                uint32_t u = (word >> (16u * (pos & 1u))) & 0xFFFFu;
                uint32_t digit = (u * (n - pos)) >> 16;
                uint32_t y;
                if (P.many) {
                    // symbol = number of cumulative counts at or below the digit
                    uint32_t acc = 0;
                    y = 0;
#pragma unroll
                    for (int k = 0; k < kMaxLTW - 1; k++) { acc += (cw >> (4 * k)) & 15u; y += digit >= acc ? 1u : 0u; }
                    cw -= 1u << (4u * y);
                    o2 |= (y >> 2) << pos;
                } else {
                    y = (digit >= c0) + (digit >= c0 + c1) + (digit >= c0 + c1 + c2);
                    c0 -= y == 0; c1 -= y == 1; c2 -= y == 2;
                }
                o |= (uint64_t)(y & 3u) << (2u * pos);
            }
            rem[d] = o; remlen[d] = (int)n; rem2[d] = o2;
        }
    }

    return kOk;
}

template <int DM, class CNT = Mu>
__device__ __forceinline__ int decode_candidate(const KParams &P, uint64_t idx, uint64_t (&rem)[DM], int (&remlen)[DM], CNT &mu)
{
    uint32_t rem2[DM];
    return decode_candidate<DM, CNT>(P, idx, rem, remlen, mu, rem2);
}

// ------------------------------------------------------------------ one candidate (general path)
template <int DM, int VM>
__device__ __forceinline__ int evaluate(const KParams &P, uint64_t idx, uint16_t *prog, uint32_t *state, const int32_t *t_tab,
                        const uint32_t *mask_tab, int &period, int (&peak)[DM], DevDetail *detail)
{
    uint64_t rem[DM];
    int remlen[DM];
    Mu mu;
    period = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) peak[d] = 0;
    {
        int st = decode_candidate<DM>(P, idx, rem, remlen, mu);
        if (st != kOk) return st;
    }

    if (detail) {
        for (int g = 0; g < P.K; g++) detail->leads[g] = (int)mu.get((uint32_t)g);
        for (int d = 0; d < kMaxDW; d++) detail->order_len[d] = 0;
    }

    // ---------------- memory at the window entry: blocks that ran before it (type i has
    // handled micro-batches 0 .. lead_i - 1)
    int memcur[DM];
#pragma unroll
    for (int d = 0; d < DM; d++) {
        memcur[d] = 0;
        if (d < P.D)
            for (int y = 0; y < P.ntd[d]; y++)
                memcur[d] += P.m_of[d][y] * (int)mu.get(byte_of(P.type_of[d], (uint32_t)y));
        peak[d] = INT_MIN;
    }

    // ---------------- build: place blocks in an executable sequence
    const bool repair = P.space == kSampledRepair;
    int placed = 0;
    const int total = P.total;
    bool deadlock = false;

    // places block type g (its next occurrence) taking entry pos[dd] of every device dd it occupies
    auto place = [&](uint32_t g, uint32_t mask, uint32_t home, uint32_t tokbase, int m, uint32_t pos_d, int d_static) {
        uint32_t mug = mu.get(g);
        prog[placed * kWave] = (uint16_t)(home | ((tokbase + mug) << 5));
        mu.inc(g);
        placed++;
#pragma unroll
        for (int dd = 0; dd < DM; dd++) {
            if (dd >= P.D) continue;
            bool here = (mask >> dd) & 1u;
            if (!here) continue;
            uint32_t pos = 0;
            if (dd == d_static) pos = pos_d;
            else if (pos_d != 0xFFFFFFFFu && repair) {
                // multi-device block placed out of line: its earliest entry on the other devices
                uint32_t ysym = 0;
                for (int y = 0; y < P.ntd[dd]; y++) if (byte_of(P.type_of[dd], (uint32_t)y) == g) ysym = (uint32_t)y;
                pos = find_first(rem[dd], (uint32_t)remlen[dd], ysym);
            }
            rem[dd] = remove_at(rem[dd], pos);
            remlen[dd]--;
            memcur[dd] += m;
            peak[dd] = max(peak[dd], memcur[dd]);
            if (detail) detail->orders[dd][detail->order_len[dd]++] = (int)g;
        }
    };

    while (placed < total && !deadlock) {
        bool progress = false;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= P.D || remlen[d] == 0) continue;
            uint32_t y = (uint32_t)rem[d] & 3u;
            uint32_t g = byte_of(P.type_of[d], y), pr = byte_of(P.pred_of[d], y);
            uint32_t mask = byte_of(P.mask_of[d], y);
            bool ok = pr == 0xFFu || mu.get(pr) > mu.get(g);
            if (P.tp && mask != (1u << d)) {
                // a multi-device block runs when it heads the list of all its devices; it is
                // placed from its lowest device
                if ((mask & ((1u << d) - 1u)) != 0) ok = false;
#pragma unroll
                for (int dd = 0; dd < DM; dd++) {
                    if (dd >= P.D || dd == d || !((mask >> dd) & 1u)) continue;
                    bool head = remlen[dd] > 0 && byte_of(P.type_of[dd], (uint32_t)rem[dd] & 3u) == g;
                    if (!head) ok = false;
                }
            }
            if (ok) {
                place(g, mask, byte_of(P.home_of[d], y), byte_of(P.tok_of[d], y), sel4(P.m_of[d], y), 0u, d);
                progress = true;
            }
        }
        if (progress) continue;
        if (!repair) { deadlock = true; break; }
        // Nothing at the head of any list can run.  Ascending over devices, then over the
        // device's remaining entries in list order: the first block whose producers are
        // placed goes next (only the first entry of each type can be that block).
        bool done = false;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (done || d >= P.D || remlen[d] == 0) continue;
            uint32_t best_pos = 64u, best_y = 0;
#pragma unroll
            for (int y = 0; y < kMaxLT; y++) {
                if (y >= P.ntd[d]) continue;
                uint32_t g = byte_of(P.type_of[d], (uint32_t)y), pr = byte_of(P.pred_of[d], (uint32_t)y);
                bool ready = pr == 0xFFu || mu.get(pr) > mu.get(g);
                uint32_t pos = ready ? find_first(rem[d], (uint32_t)remlen[d], (uint32_t)y) : 64u;
                if (pos < best_pos) { best_pos = pos; best_y = (uint32_t)y; }
            }
            if (best_pos < 64u) {
                uint32_t y = best_y;
                place(byte_of(P.type_of[d], y), byte_of(P.mask_of[d], y), byte_of(P.home_of[d], y),
                      byte_of(P.tok_of[d], y), sel4(P.m_of[d], y), best_pos, d);
                done = true;
            }
        }
        if (!done) { deadlock = true; }     // cannot happen: unplaced blocks form a DAG
    }
    if (deadlock) {
#pragma unroll
        for (int d = 0; d < DM; d++) peak[d] = 0;
        return kDeadlock;
    }
    int peak_max = INT_MIN;
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D || peak[d] == INT_MIN) peak[d] = 0;      // a device without blocks
        if (d < P.D) peak_max = max(peak_max, peak[d]);
    }
    if (peak_max > P.M) return kMem;

    // ---------------- period
    // boundary values that mean anything: devices with blocks; micro-batch j of a chain is in flight at the
    // boundary when the chain's first block is j or more ahead (its counter now reads lead + N_R)
    uint32_t live = 0;
    for (int d = 0; d < P.D; d++) live |= (P.ntd[d] > 0 ? 1u : 0u) << d;
    for (int g = 0, path = 0; g < P.K; g++)
        if (P.pred[g] < 0) {
            const int lead = (int)mu.get((uint32_t)g) - P.NR;
            for (int j = 0; j < P.NR; j++)
                if (lead > j && P.D + path * P.NR + j < 32) live |= 1u << (P.D + path * P.NR + j);
            path++;
        }
    period = P.tp ? least_period<VM, true>(P, prog, state, t_tab, mask_tab, live)
                  : least_period<VM, false>(P, prog, state, t_tab, mask_tab, live);
    return kOk;
}

// ------------------------------------------------------------------ dependency graphs that are not chains
// A block type may have several producers and several consumers (Sec. III-A, Eq. 1 [3]).  State of a sweep, in LDS
// [slot][lane]: the D device times, then for every unbranched stretch of the graph with a type somebody consumes a
// ring of 2 N_R end times by micro-batch (micro-batches N_R and up belong to the next window and move down at the
// window boundary) and N_R more slots for the boundary's comparison.  Program entry: type id
// in bits 0-4 (0-5 for problems with more than 32 types), micro-batch above.  Tables by type id in LDS: t, device mask,
// producer mask (two words where there are more than 32 types), first ring slot.
struct DagTables {
    const int32_t *t; const uint32_t *mask, *pred, *pred_hi, *tok;
    __device__ __forceinline__ uint64_t producers(uint32_t g) const { return pred[g] | (pred_hi ? (uint64_t)pred_hi[g] << 32 : 0ull); }
};

template <int TB>
__device__ __forceinline__ void sweep_window_dag(const KParams &P, const DagTables &Tb, const uint16_t *prog, uint32_t *state)
{
    const int total = P.total;
    for (int k = 0; k < total; k++) {
        const uint32_t e = prog[k * kWave];
        const uint32_t g = e & ((1u << TB) - 1u), m = e >> TB;
        uint32_t s = 0;
        for (uint32_t rest = Tb.mask[g]; rest; rest &= rest - 1u) s = max(s, state[__builtin_ctz(rest) * kWave]);
        for (uint64_t rest = Tb.producers(g); rest; rest &= rest - 1ull) s = max(s, state[(Tb.tok[__builtin_ctzll(rest)] + m) * kWave]);
        const uint32_t en = s + (uint32_t)Tb.t[g];
        for (uint32_t rest = Tb.mask[g]; rest; rest &= rest - 1u) state[__builtin_ctz(rest) * kWave] = en;
        if (Tb.tok[g] != kNoRing) state[(Tb.tok[g] + m) * kWave] = en;
    }
}

// The window boundary: every ring moves down by N_R micro-batches and the device times stay, all less `shift` (0, or
// the period under test: times are then taken from the start of the next window, not below 0).  Returns whether every
// value that crosses the boundary and means anything grew by `want` over the window (`first`: by any one amount,
// which is handed back in `want`): ring entries below the lead of the ring's first type (micro-batches it handled
// before the window), compared with the copy the last boundary kept of them behind the ring (later types of the
// ring's stretch overwrite the entries themselves); device times against `prevfree`.
template <int DM, class CNT>
__device__ __forceinline__ bool boundary_dag(const KParams &P, const DagTables &Tb, uint32_t *state, const CNT &lead, uint32_t (&prevfree)[DM],
                                             uint32_t shift, bool first, uint32_t &want, uint32_t &top)
{
    bool same = true, have = !first;
    top = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D) continue;
        const uint32_t x = state[d * kWave], y = x > shift ? x - shift : 0u;
        if (P.ntd[d] > 0) {
            const uint32_t dv = y - prevfree[d];
            if (!have) { want = dv; have = true; } else if (dv != want) same = false;
        }
        prevfree[d] = y; state[d * kWave] = y;
        top = max(top, y);
    }
    for (int r = 0; r < P.ntok; r++) {
        const uint32_t base = P.ring_base[r], kept = P.ring_kept[r];
        const uint32_t lg = lead.get((uint32_t)P.ring_head[r]);
        for (int m = 0; m < P.NR; m++) {
            const uint32_t old = state[(kept + m) * kWave], x = state[(base + m + P.NR) * kWave];
            const uint32_t y = x > shift ? x - shift : 0u;
            if ((uint32_t)m < lg) {
                const uint32_t dv = y - old;
                if (!have) { want = dv; have = true; } else if (dv != want) same = false;
                top = max(top, y);
            }
            const uint32_t keep = (uint32_t)m < lg ? y : 0u;
            state[(base + m) * kWave] = keep;
            state[(kept + m) * kWave] = keep;
            state[(base + m + P.NR) * kWave] = 0;
        }
    }
    return same && have;
}

// Least period of the repeated window.  First the eigenvector search of the other kernels (sweeps from 0 until every
// boundary value grows by the same amount, which is then the period); if that does not settle, the definition: the
// least T in [LB, UB] for which start times exist, by bisection; start times exist for T iff the sweeps from 0, with
// every boundary value taken T later each time, come to rest (Kleene iteration of the longest-path equations; it
// rests after at most as many windows as values cross the boundary, or passes UB).
template <int DM, class CNT>
__device__ __forceinline__ int least_period_dag(const KParams &P, const DagTables &Tb, const uint16_t *prog, uint32_t *state, const CNT &lead)
{
    uint32_t prevfree[DM];
    auto reset = [&]() {
        for (int s = 0; s < P.nslots; s++) state[s * kWave] = 0;
#pragma unroll
        for (int d = 0; d < DM; d++) prevfree[d] = 0;
    };
    reset();
    bool done = false;
    uint32_t T = 0;
    for (int j = 0; j < P.dag_tries; j++) {
        if (__ballot(!done) == 0) break;
        sweep_window_dag<CNT::kTypeBits>(P, Tb, prog, state);
        uint32_t delta = 0, top;
        const bool eig = boundary_dag<DM>(P, Tb, state, lead, prevfree, 0u, true, delta, top);
        if (!done && eig) { T = delta; done = true; }
    }
    if (__ballot(!done) == 0) return (int)T;
    // bisection, the same number of steps in every lane; lanes that have their period keep a fixed interval
    int crossing = P.D;
    for (int r = 0; r < P.ntok; r++) crossing += (int)lead.get((uint32_t)P.ring_head[r]);
    uint32_t lo = done ? T : (uint32_t)P.LB, hi = done ? T : (uint32_t)P.UB;
    int steps = 0;
    for (uint32_t span = (uint32_t)(P.UB - P.LB); span; span >>= 1) steps++;
    for (int it = 0; it < steps; it++) {
        const uint32_t mid = lo + (hi - lo) / 2u;
        const bool open = lo < hi;
        reset();
        bool decided = !open, feasible = false;
        // (crossing + 2 windows bound the iteration; the loop runs until every lane of the wave has decided)
        for (int w = 0; w < kMaxKW * kMaxNRW + kMaxDW + 2; w++) {
            if (__ballot(!decided) == 0) break;
            sweep_window_dag<CNT::kTypeBits>(P, Tb, prog, state);
            uint32_t zero = 0, top;
            const bool rest = boundary_dag<DM>(P, Tb, state, lead, prevfree, mid, false, zero, top);
            if (!decided) {
                if (rest) { decided = true; feasible = true; }
                else if (top > (uint32_t)P.UB || w > crossing + 1) { decided = true; feasible = false; }
            }
        }
        if (open) { if (feasible) hi = mid; else lo = mid + 1u; }
    }
    return (int)hi;
}

// One candidate of a problem whose dependency graph is not a set of chains, or that is too wide for the other paths
// (general kernel only).  A device's order is kept as three bit planes of its symbols (bit p of plane k = bit k of the
// symbol at position p; up to eight block types per device) and the mask of the entries not yet placed.
__device__ __forceinline__ uint32_t even_bits(uint64_t x);
template <int DM, class CNT>
__device__ __forceinline__ int evaluate_dag(const KParams &P, const DagTables &Tb, uint64_t idx, uint16_t *prog, uint32_t *state,
                                            int &period, int (&peak)[DM], DevDetail *detail)
{
    uint32_t p0[DM], p1[DM], p2[DM], alive[DM];
    CNT mu;
    period = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) peak[d] = 0;
    {
        uint64_t rem[DM];
        int remlen[DM];
        int st = decode_candidate<DM, CNT>(P, idx, rem, remlen, mu, p2);
        if (st != kOk) return st;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            p0[d] = even_bits(rem[d]); p1[d] = even_bits(rem[d] >> 1);
            alive[d] = remlen[d] >= 32 ? 0xFFFFFFFFu : (1u << remlen[d]) - 1u;
        }
    }
    const CNT lead = mu;
    if (detail) {
        for (int g = 0; g < P.K; g++) detail->leads[g] = (int)mu.get((uint32_t)g);
        for (int d = 0; d < kMaxDW; d++) detail->order_len[d] = 0;
    }
    auto type_at = [&](int d, uint32_t y) -> uint32_t { return y < 4u ? byte_of(P.type_of[d], y) : byte_of(P.type_of_hi[d], y - 4u); };
    int memcur[DM];
#pragma unroll
    for (int d = 0; d < DM; d++) {
        memcur[d] = 0;
        if (d < P.D)
            for (int y = 0; y < P.ntd[d]; y++)
                memcur[d] += P.m_of[d][y] * (int)mu.get(type_at(d, (uint32_t)y));
        peak[d] = INT_MIN;
    }
    const bool repair = P.space == kSampledRepair;
    int placed = 0;
    const int total = P.total;
    // a block may run when every producer has handled its micro-batch: in this window (counter ahead) or in the last
    // one (micro-batch below the producer's lead, which the counter is ahead of too)
    auto ready = [&](uint32_t g, uint64_t preds) -> bool {
        const uint32_t mg = mu.get(g);
        bool ok = true;
        for (uint64_t rest = preds; rest; rest &= rest - 1ull) ok = ok && mu.get((uint32_t)__builtin_ctzll(rest)) > mg;
        return ok;
    };
    // symbol at position pos of device d; entries of symbol y still to be placed
    auto symbol = [&](uint32_t a0, uint32_t a1, uint32_t a2, uint32_t pos) -> uint32_t {
        return ((a0 >> pos) & 1u) | (((a1 >> pos) & 1u) << 1) | (((a2 >> pos) & 1u) << 2);
    };
    auto left_of = [&](uint32_t a0, uint32_t a1, uint32_t a2, uint32_t al, uint32_t y) -> uint32_t {
        return al & (y & 1u ? a0 : ~a0) & (y & 2u ? a1 : ~a1) & (y & 4u ? a2 : ~a2);
    };
    // places the block of type g whose entry on device d_static sits at pos_d; on its other devices its earliest entry
    // (the head there when the block was placed as the head of all its lists)
    auto place = [&](uint32_t g, uint32_t mask, int m, uint32_t pos_d, int d_static) {
        prog[placed * kWave] = (uint16_t)(g | (mu.get(g) << CNT::kTypeBits));
        mu.inc(g);
        placed++;
#pragma unroll
        for (int dd = 0; dd < DM; dd++) {
            if (dd >= P.D || !((mask >> dd) & 1u)) continue;
            uint32_t pos = pos_d;
            if (dd != d_static) {
                uint32_t ysym = 0;
                for (int y = 0; y < P.ntd[dd]; y++) if (type_at(dd, (uint32_t)y) == g) ysym = (uint32_t)y;
                const uint32_t mine = left_of(p0[dd], p1[dd], p2[dd], alive[dd], ysym);
                pos = mine ? (uint32_t)__builtin_ctz(mine) : 0u;
            }
            alive[dd] &= ~(1u << pos);
            memcur[dd] += m;
            peak[dd] = max(peak[dd], memcur[dd]);
            if (detail) detail->orders[dd][detail->order_len[dd]++] = (int)g;
        }
    };
    bool deadlock = false;
    while (placed < total && !deadlock) {
        bool progress = false;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= P.D || alive[d] == 0) continue;
            const uint32_t pos = (uint32_t)__builtin_ctz(alive[d]);
            const uint32_t y = symbol(p0[d], p1[d], p2[d], pos);
            const uint32_t g = type_at(d, y), mask = Tb.mask[g];
            bool ok = ready(g, sel8(P.predmask_of[d], y));
            if (mask != (1u << d)) {
                // a multi-device block runs when it heads the list of all its devices; it is placed from its lowest device
                if ((mask & ((1u << d) - 1u)) != 0) ok = false;
#pragma unroll
                for (int dd = 0; dd < DM; dd++) {
                    if (dd >= P.D || dd == d || !((mask >> dd) & 1u)) continue;
                    const uint32_t hp = (uint32_t)__builtin_ctz(alive[dd] | 0x80000000u);
                    if (!(alive[dd] != 0 && type_at(dd, symbol(p0[dd], p1[dd], p2[dd], hp)) == g)) ok = false;
                }
            }
            if (ok) { place(g, mask, sel8(P.m_of[d], y), pos, d); progress = true; }
        }
        if (progress) continue;
        if (!repair) { deadlock = true; break; }
        bool done = false;
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (done || d >= P.D || alive[d] == 0) continue;
            uint32_t best_pos = 64u, best_y = 0;
#pragma unroll
            for (int y = 0; y < kMaxLTW; y++) {
                if (y >= P.ntd[d]) continue;
                const bool ok = ready(type_at(d, (uint32_t)y), P.predmask_of[d][y]);
                const uint32_t mine = left_of(p0[d], p1[d], p2[d], alive[d], (uint32_t)y);
                const uint32_t pos = ok && mine ? (uint32_t)__builtin_ctz(mine) : 64u;
                if (pos < best_pos) { best_pos = pos; best_y = (uint32_t)y; }
            }
            if (best_pos < 64u) {
                const uint32_t g = type_at(d, best_y);
                place(g, Tb.mask[g], sel8(P.m_of[d], best_y), best_pos, d);
                done = true;
            }
        }
        if (!done) deadlock = true;         // cannot happen: unplaced blocks form a DAG
    }
    if (deadlock) {
#pragma unroll
        for (int d = 0; d < DM; d++) peak[d] = 0;
        return kDeadlock;
    }
    int peak_max = INT_MIN;
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D || peak[d] == INT_MIN) peak[d] = 0;
        if (d < P.D) peak_max = max(peak_max, peak[d]);
    }
    if (peak_max > P.M) return kMem;
    period = least_period_dag<DM, CNT>(P, Tb, prog, state, lead);
    return kOk;
}

__device__ __forceinline__ bool key_less(int pa, uint64_t ia, int pb, uint64_t ib)
{
    return pa < pb || (pa == pb && ia < ib);
}

// ==================================================================== fast path
// Single-device blocks only.  Block types are addressed by their code c = device*4 + symbol, so
// that bit c of a 32-bit mask means "type c": R = types whose next occurrence may be placed now
// (producer ahead and occurrences left), HM = the type at the head of every device's list.
// One block is placed per step and lane:
//   heads first   : lowest set bit of R & HM            (any order of runnable heads gives the
//                                                         same per-device orders)
//   else repair   : lowest device with a runnable type = lowest set bit of R; inside the device
//                   the earliest remaining entry whose type is runnable
// A device's order is kept as two bit planes (bit p of lo/hi = low/high bit of the symbol at
// position p) and a mask of the entries not yet placed.  The per-device record is picked by a
// run-time device number and therefore lives in LDS [device][lane]; masks and the 4-bit
// micro-batch counters stay in VGPRs.

// the window's program: six 5-bit type codes a word, in executable order.  It is written and read with a
// wave-uniform word index, so it can live in VGPRs (indirect register addressing) and costs no LDS.
typedef uint32_t u32x32 __attribute__((ext_vector_type(32)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
struct FastProgram {
    u32x32 a;
    u32x16 b;
    __device__ __forceinline__ uint32_t get(int i) const { return i < 32 ? a[i] : b[i - 32]; }
    __device__ __forceinline__ void set(int i, uint32_t v) { if (i < 32) a[i] = v; else b[i - 32] = v; }
};

constexpr int kFastTableWords = 16 * kMaxK;      // uniform tables at the start of the fast kernel's LDS
constexpr int kSweepTabWord = 12 * kMaxK;        // ... of which the sweeps' three tables by code; a multiple of 64 words, so
                                                 // that one two-address LDS read fetches a code's first and third word
constexpr int kTpTableWords = 5 * kMaxK;         // the TP variants' own tables behind them
// Everything a lane reads by a run-time index lies word by word: word w of entry i at w * 64 + i words, so that
// lanes with different entries hit different banks, a lane's words of one entry come with two-address reads
// (stride 64 words), and an LDS atomic on one word of the records meets no bank twice.

struct FastLds {
    uint32_t *sw_tab;     // [32]  by code, for the sweeps of problems without blocks on several devices:
                          //       t << 16 | LDS address of the time of the code's device (lane 0)
    uint32_t *ch_tab;     // [32]  by code, right behind sw_tab: LDS address of the first token of the code's chain (lane 0)
    uint32_t *in_tab;     // [32]  by code, behind ch_tab: 1 << s | s, s = 16 + 4 * symbol: counter increment and field position
    uint4 *tt_tab;        // [32]  by code, for the sweeps of the TP variants: x: t, y: byte offset of the first token slot of the code's
                          //       chain, z: byte offset of its device's words, w: bit offset of its micro-batch counter
    uint32_t *type_tab;   // [4][64], code in the low half of every 64: what placing one block of the type does:
                          //   word 0: added to the last word of its device record: memory delta << 16, one waiting
                          //      micro-batch of the type less, one more for its consumer if that sits on the same device
                          //   word 1: one-hot mask of the consumer's code (0: none)
                          //   word 2: consumer on another device: LDS address of the last word of that device's record
                          //      (lane 0); otherwise, TP variants: 0xFFFFFFFF, else that of the type's own device
                          //      (word 3 is 0 then).  Not TP: 4 * symbol of the type in bits 16-19
                          //   word 3: the increment of that word (one waiting micro-batch of the consumer)
                          // the upper halves hold chain_tab, vtab, cum_tab, predbit_tab
    uint32_t *chain_tab;  // [32]  KParams::chain_tab
    uint32_t *vtab;       // [32]  KParams::vtab
    uint32_t *cum_tab, *predbit_tab;   // [32] each: KParams::cum_code, pred_bit
    uint32_t *grp_tab;    // [32]  TP variants: KParams::grp_code
    uint32_t rec;         // build: LDS address of the records [DM][4][64]: word 0: low plane, 1: high plane,
                          //        2: not-yet-placed mask, 3: micro-batches waiting at the input of the 4 types
                          //        (4 bits each) | memory now (signed) << 16
    // sweeps: three arrays [slot][64] in a row at distances known at compile time
    uint32_t *dfree;      // [DM] time at which the device is free
    uint32_t *dcnt;       // [DM] next micro-batch of the device's 4 types (4 bits each, in the upper half of the word)
    uint32_t *tok;        // [token slots] end time of the micro-batch's latest block
};

// problem scalars, read once per workgroup
template <int DM>
struct FastConst {
    int D, K, NR, M, total, nslots, npaths, nsweeps, space, has_fixed, nwords, ndeps;
    uint32_t step_q16;
    uint64_t seed;
    int ntd[DM];
    uint32_t mpack[DM];
    // blocks on several devices (TP variants of the kernel only)
    int ntp;
    uint32_t slow;
    uint32_t tpg[kMaxD];
};

__device__ __forceinline__ uint32_t bfi(uint32_t sel, uint32_t a, uint32_t b) { return (sel & a) | (~sel & b); }

// position of the lowest set bit; all ones for 0, which "& 28", shift counts and bit-field offsets (all of them use the
// low five bits) read as 31: no guard bit has to be set first
__device__ __forceinline__ uint32_t low_bit(uint32_t x)
{
    uint32_t r;
    asm("v_ffbl_b32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}

// a * b + c for a, b below 2^24, low 32 bits: the full-rate 24-bit multiply-add (b uniform)
__device__ __forceinline__ uint32_t mad24(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(b), "v"(c));
    return r;
}

// keeps a value in a VGPR at this point, so that the loads above it are issued together instead of
// being sunk into later branches
#define TESSEL_PIN(x) asm volatile("" : "+v"(x))

// One block of the window: s = max(device free, previous block of the micro-batch); both become s + t.  The
// micro-batch it handles is the device's counter of its type in `cnt`, the counter word as it was before the
// caller's atomic incremented it (the caller may have the next node's atomic in flight already).
__device__ __forceinline__ void sweep_node(const FastLds &L, const uint4 tt, uint32_t cnt, uint32_t lane4)
{
    // device times, counters and tokens lie at fixed distances in one array, so the three addresses of a block
    // share their registers: tt.z = the device's offset, tt.y = the chain's first token slot
    const uint32_t mu = __builtin_amdgcn_ubfe(cnt, tt.w, 4);
    uint32_t *fr = (uint32_t *)((char *)L.dfree + (tt.z + lane4));
    uint32_t *tk = (uint32_t *)((char *)L.dfree + (tt.y + lane4 + (mu << 8)));
    const uint32_t en = max(*fr, *tk) + tt.x;
    *fr = en;
    *tk = en;
}

// The same for problems with blocks on several devices: the block waits for all devices of its code group `G` (one
// nibble per device) and frees them together.  Counter and token are those of the type's code on its lowest device,
// which is the code the program holds.
template <int DM>
__device__ __forceinline__ void sweep_node_group(const FastLds &L, const uint4 tt, uint32_t cnt, uint32_t lane, uint32_t G, int D)
{
    const uint32_t mu = __builtin_amdgcn_ubfe(cnt, tt.w, 4);
    uint32_t *tk = (uint32_t *)((char *)L.dfree + (tt.y + lane * 4u + (mu << 8)));
    uint32_t s = *tk;
#pragma unroll
    for (int dd = 0; dd < DM; dd++)
        if (dd < D && ((G >> (4 * dd)) & 15u)) s = max(s, L.dfree[dd * kWave + lane]);
    const uint32_t en = s + tt.x;
#pragma unroll
    for (int dd = 0; dd < DM; dd++)
        if (dd < D && ((G >> (4 * dd)) & 15u)) L.dfree[dd * kWave + lane] = en;
    *tk = en;
}

// LDS accesses by byte address: address arithmetic stays integer arithmetic, and a constant added to an
// address goes into the instruction's offset field.
typedef __attribute__((address_space(3))) uint32_t lds_word;
__device__ __forceinline__ uint32_t lds_address(const void *p) { return (uint32_t)(uintptr_t)(const lds_word *)p; }
__device__ __forceinline__ uint32_t lds_load(uint32_t a) { return *(const lds_word *)(uintptr_t)a; }
__device__ __forceinline__ void lds_store(uint32_t a, uint32_t v) { *(lds_word *)(uintptr_t)a = v; }
__device__ __forceinline__ uint32_t lds_fetch_add(uint32_t a, uint32_t v)
{
    return __hip_atomic_fetch_add((lds_word *)(uintptr_t)a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// a lane's device record: four words at a stride of 64 words (two two-address accesses)
constexpr uint32_t kRecWordStep = kWave * 4u, kRecDevStep = 4u * kRecWordStep;
__device__ __forceinline__ uint4 rec_load(uint32_t a)
{
    return make_uint4(lds_load(a), lds_load(a + kRecWordStep), lds_load(a + 2u * kRecWordStep), lds_load(a + 3u * kRecWordStep));
}
__device__ __forceinline__ void rec_store(uint32_t a, const uint4 v)
{
    lds_store(a, v.x); lds_store(a + kRecWordStep, v.y); lds_store(a + 2u * kRecWordStep, v.z); lds_store(a + 3u * kRecWordStep, v.w);
}

// The blocks of one sweep for problems whose blocks sit on one device each, as a software pipeline four blocks deep.
// Per block: its table word is read (T); one returning LDS atomic reads and increments the counter word of its
// device (A), which names the micro-batch and with it the token; device time and token are read (R); s = max of the
// two, both become s + t (W).  As a dependent chain T -> A -> R -> W the wave would wait for the LDS three times a
// block, so block k + 3 does T, block k + 2 A and block k + 1 R before block k does W.  R(k + 1) then misses what
// W(k) writes: when block k + 1 runs on the same device or handles the same micro-batch as block k, the value read is
// replaced by block k's end time (two compares, two selects).  LDS keeps a wave's accesses in order, so W(k - 1) and
// everything older is seen.
// Table word of a code: t << 16 | LDS address of its device's time (lane 0); with several chains (MC) a second
// table holds the LDS address of the chain's first token (lane 0).  A device's counter word holds the next micro-batch
// of its four types in its upper half, four bits each; the third table word of a code, 1 << s | s with s = 16 +
// 4 * symbol, is both the increment of the atomic (the low half of the counter word only collects the s, below 2^16
// over a window) and, by its low five bits, the position of the field.
// Past the last block the stages T, A and R run on code 0 (a counter that the window boundary resets anyway, reads
// inside the arrays); stage W does not.
template <int DM, bool MC>
__device__ __forceinline__ void sweep_blocks(const FastConst<DM> &C, const FastLds &L, const FastProgram &prog, uint32_t lane4)
{
    const int total = C.total, nfull = total / 6, tail = total - 6 * nfull;
    constexpr uint32_t tab = kSweepTabWord * 4u;                // the kernel's LDS starts at address 0 (checked at its start)
    const uint32_t lane_tok = lds_address(L.dfree) + 2u * DM * kWave * 4u + lane4;
    struct Tst { uint32_t tt, w2, ch; };                        // T done
    struct Ast { uint32_t tt, fa, w2, cnt, ch; };               // A done
    struct Rst { uint32_t tt, fa, ta, fr, tk; };                // R done
    auto stage_t = [&](uint32_t w, int pos) -> Tst {
        Tst o;
        const uint32_t c4 = (pos == 0 ? w << 2 : w >> (5 * pos - 2)) & 0x7Cu;
        o.tt = lds_load(c4 + tab);
        o.w2 = lds_load(c4 + tab + 2u * kMaxK * 4u);
        o.ch = MC ? lds_load(c4 + tab + kMaxK * 4u) : 0u;
        return o;
    };
    auto stage_a = [&](const Tst &x) -> Ast {
        Ast o;
        o.tt = x.tt; o.ch = x.ch; o.w2 = x.w2;
        o.fa = (x.tt & 0xFFFFu) + lane4;
        o.cnt = lds_fetch_add(o.fa + DM * kWave * 4u, x.w2);
        return o;
    };
    auto stage_r = [&](const Ast &x) -> Rst {
        Rst o;
        o.tt = x.tt; o.fa = x.fa;
        const uint32_t mu = __builtin_amdgcn_ubfe(x.cnt, x.w2, 4);      // (the offset is the low five bits of w2)
        o.ta = MC ? (mu << 8) + lane4 + x.ch : (mu << 8) + lane_tok;
        o.fr = lds_load(x.fa);
        o.tk = lds_load(o.ta);
        return o;
    };
    auto stage_w = [&](const Rst &x) {
        const uint32_t en = max(x.fr, x.tk) + (x.tt >> 16);
        lds_store(x.fa, en);
        lds_store(x.ta, en);
    };
    // per program word: the six table words first (they depend on the word only), then the blocks, the counter
    // atomic one block ahead of the times
    auto word = [&](uint32_t w, int nblocks) {
        Tst t[6];
#pragma unroll
        for (int j = 0; j < 6; j++) if (j < nblocks) t[j] = stage_t(w, j);
        Ast a = stage_a(t[0]);
#pragma unroll
        for (int j = 0; j < 6; j++)
            if (j < nblocks) {
                Ast an = a;
                if (j + 1 < nblocks) an = stage_a(t[j + 1]);
                stage_w(stage_r(a));
                a = an;
            }
    };
    for (int i = 0; i < nfull; i++) word(prog.get(i), 6);
    if (tail > 0) {
        const uint32_t w = prog.get(nfull);
        if (tail == 1) word(w, 1); else if (tail == 2) word(w, 2); else if (tail == 3) word(w, 3); else if (tail == 4) word(w, 4); else word(w, 5);
    }
}

// One sweep of the window over the program, then the window boundary.
template <int DM, bool TP>
__device__ __forceinline__ void sweep_fast(const FastConst<DM> &C, const FastLds &L, const FastProgram &prog, int lane,
                                           const Mu &lead_code, bool active)
{
    // a lane without a complete program (rejected candidate, lane past the end of the range) must not run one:
    // its counters would leave the token ring
    if (!active) return;
    const uint32_t lane4 = (uint32_t)lane * 4u;
    if (TP) {
        for (int k = 0; k < C.total; k++) {
            const uint32_t code = (prog.get(k / 6) >> (5 * (k % 6))) & 31u;
            const uint4 tt = L.tt_tab[code];
            uint32_t *cp = (uint32_t *)((char *)L.dfree + (tt.z + lane4)) + DM * kWave;
            const uint32_t cnt = *cp;
            *cp = cnt + (1u << tt.w);
            sweep_node_group<DM>(L, tt, cnt, (uint32_t)lane, L.grp_tab[code], C.D);
        }
    } else {
        if (C.npaths > 1) sweep_blocks<DM, true>(C, L, prog, lane4);
        else sweep_blocks<DM, false>(C, L, prog, lane4);
    }
    // window boundary: micro-batches mu >= N_R are mu - N_R of the next window; counters restart at the leads
    for (int p = 0; p < C.npaths; p++)
        for (int mu = 0; mu < C.NR; mu++) {
            int base = p * 2 * C.NR + mu;
            L.tok[base * kWave + lane] = L.tok[(base + C.NR) * kWave + lane];
            L.tok[(base + C.NR) * kWave + lane] = 0;
        }
#pragma unroll
    for (int d = 0; d < DM; d++)
        if (d < C.D) L.dcnt[d * kWave + lane] = (uint32_t)((d < 4 ? lead_code.lo : lead_code.hi) >> (16 * (d & 3))) << 16;
}

template <int DM>
__device__ __forceinline__ void reset_sweep_state(const FastConst<DM> &C, const FastLds &L, int lane, const Mu &lead_code)
{
    for (int d = 0; d < C.D; d++) L.dfree[d * kWave + lane] = 0;
    for (int s = 0; s < C.nslots - C.D; s++) L.tok[s * kWave + lane] = 0;
#pragma unroll
    for (int d = 0; d < DM; d++)
        if (d < C.D) L.dcnt[d * kWave + lane] = (uint32_t)((d < 4 ? lead_code.lo : lead_code.hi) >> (16 * (d & 3))) << 16;
}

// Period of the repeated window.  The sweep is a max-plus linear map F on the boundary vector x
// (device free times, in-flight micro-batch end times).  If after some sweep every live component
// has grown by the same delta, x is an eigenvector of F and delta is its eigenvalue = the maximum
// cycle ratio, exactly.  Almost every candidate gets there within two or three sweeps; one that has
// not after the sweeps allowed (`tries`) is handed on by the caller: to a queue of candidates that get more
// sweeps, from there to the general kernel (Karp's formula).
template <int DM, int VM, bool TP>
__device__ __forceinline__ int period_fast(const FastConst<DM> &C, const FastLds &L, const FastProgram &prog, int lane,
                                           const Mu &lead_code, bool want, int tries,
                                           uint32_t &nsweeps_used)
{
    const int V = C.nsweeps - 1;
    const uint32_t lane4 = (uint32_t)lane * 4u;
    // byte offset (from the device times) of boundary value v: a device's free time or a carried token
    auto value_offset = [&](uint32_t e) -> uint32_t {
        const uint32_t slot = e & 63u;
        return ((e >> 6 & 1u) ? slot : 2u * DM + slot - (uint32_t)C.D) * (kWave * 4u) + lane4;
    };
    uint32_t live = 0;                                    // per lane: which boundary values mean anything
#pragma unroll
    for (int v = 0; v < VM; v++) {
        if (v < V) {
            const uint32_t e = L.vtab[v];
            const bool on = (e >> 6 & 1u) ? (e >> 17 & 1u) != 0 : lead_code.get((e >> 7) & 31u) > ((e >> 13) & 15u);
            live |= (on ? 1u : 0u) << v;
        }
    }
    reset_sweep_state<DM>(C, L, lane, lead_code);
    uint32_t prev[VM];
#pragma unroll
    for (int v = 0; v < VM; v++) prev[v] = 0;
    int T = 0;
    bool done = !want;
    for (int j = 0; j < tries; j++) {
        if (__ballot(!done) == 0) break;
        sweep_fast<DM, TP>(C, L, prog, lane, lead_code, !done);
        nsweeps_used += done ? 0u : 1u;
        bool same = true, have = false;
        uint32_t delta = 0;
#pragma unroll
        for (int v = 0; v < VM; v++) {
            if (v < V) {
                const uint32_t x = *(const uint32_t *)((const char *)L.dfree + value_offset(L.vtab[v]));
                const uint32_t dv = x - prev[v];
                prev[v] = x;
                if (live >> v & 1u) {
                    if (!have) { delta = dv; have = true; }
                    else if (dv != delta) same = false;
                }
            }
        }
        if (!done && same && have) { T = (int)delta; done = true; }
    }
    return done ? T : -1;        // -1: no eigenvector within the sweeps allowed (the caller hands the candidate on)
}

// even bits of a 64-bit word, compacted (bit 2p -> bit p)
__device__ __forceinline__ uint32_t even_bits(uint64_t x)
{
    x &= 0x5555555555555555ull;
    x = (x | (x >> 1)) & 0x3333333333333333ull;
    x = (x | (x >> 2)) & 0x0F0F0F0F0F0F0F0Full;
    x = (x | (x >> 4)) & 0x00FF00FF00FF00FFull;
    x = (x | (x >> 8)) & 0x0000FFFF0000FFFFull;
    x = (x | (x >> 16)) & 0x00000000FFFFFFFFull;
    return (uint32_t)x;
}

// even bits of a 32-bit word, compacted (bit 2p -> bit p)
__device__ __forceinline__ uint32_t even_bits32(uint32_t x)
{
    x &= 0x55555555u;
    x = (x | (x >> 1)) & 0x33333333u;
    x = (x | (x >> 2)) & 0x0F0F0F0Fu;
    x = (x | (x >> 4)) & 0x00FF00FFu;
    x = (x | (x >> 8)) & 0x0000FFFFu;
    return x;
}

// MODE: 0 exhaustive spaces, 1 sampled without repair, 2 sampled with repair.
// TP: some block type occupies several devices.  Such a type has one code on every device it occupies, and R, X
// hold all of them.  It is a runnable head only when it heads all its devices; placing it takes its earliest entry
// out of every one of them.
// Builds the candidate's window: validity, memory, the program of the window in executable order and the leads by
// code.  Returns kOk or the reason of the rejection; the period is the sweeps' business (period_fast).
// what the build carries from block to block besides the per-device records in LDS
struct BuildState {
    uint32_t R, HM, X;               // by code: runnable types, heads of the devices, exhausted types
    int worst;                       // largest memory prefix over all devices so far (Eq. 1 [2])
    int status;
};

template <int DM, int MODE, bool TP>
__device__ __forceinline__ void build_begin(const KParams &P, const FastConst<DM> &C, uint64_t idx, const FastLds &L, int lane,
                                            Mu &lead_code, BuildState &S)
{
    uint32_t plo[DM], phi[DM];       // order planes per device
    int nlen[DM];
    const uint32_t NR = (uint32_t)C.NR;
    int status = kOk;
    constexpr bool sampled = MODE != 0;    // kSampledStrict / kSampledRepair; else the exhaustive spaces
    Mu leads_type;                   // by type id (exhaustive spaces, fixed leads)
    leads_type.lo = 0; leads_type.hi = 0;
    uint32_t ka = 0, kb = 0;
    if (sampled) {
        const uint64_t z = mix64(C.seed + 0x9E3779B97F4A7C15ULL * (idx + 1));
        ka = (uint32_t)z; kb = (uint32_t)(z >> 32);
#pragma unroll
        for (int d = 0; d < DM; d++) {
            plo[d] = phi[d] = 0; nlen[d] = 0;
            if (d >= C.D) continue;
            const uint32_t n = (uint32_t)C.ntd[d] * NR;
            // cumulative counts of the remaining blocks by type, t1 <= t2 <= t3 <= 32: a digit below t1 picks
            // symbol 0, below t2 symbol 1, ...  The three are kept as bytes of one word, as 0x80 - t, so that
            // one add of the replicated digit leaves "digit >= t" in bit 7 of every byte (no carry between
            // bytes: 0x60 <= 0x80 - t + digit < 0xA0).
            const uint32_t c1 = C.ntd[d] > 0 ? NR : 0u, c2 = c1 + (C.ntd[d] > 1 ? NR : 0u), c3 = c2 + (C.ntd[d] > 2 ? NR : 0u);
            uint32_t tq = 0x808080u - (c1 | (c2 << 8) | (c3 << 16));
            // the 2-bit symbols are collected 16 to a word and split into the two planes at the end
            uint32_t acc[2] = {0u, 0u};
            auto pick = [&](uint32_t draw, uint32_t left, uint32_t &into, uint32_t at) {
                const uint32_t digit = (uint32_t)(((uint64_t)draw * (uint64_t)((left << 16) & 0xFFFFFFu)) >> 32);    // (draw * left) >> 16 as a
                                                                                                       // 24-bit high multiply (left <= 32)
                const uint32_t ge = mad24(digit, 0x010101u, tq) & 0x808080u;
                tq += (ge >> 7) ^ 0x010101u;                     // a threshold above the digit loses one block
                into |= (uint32_t)__builtin_popcount(ge) << (2u * at);   // symbol = number of thresholds at or below the digit
            };
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t from = 16u * (uint32_t)h, to = min(n, from + 16u);
                for (uint32_t pos = from; pos < to; pos += 2) {
                    const uint32_t word = stream_word(ka, kb, (kDrawOrdBase + 32u * (uint32_t)d + pos) >> 1);
                    pick(word & 0xFFFFu, n - pos, acc[h], pos - from);
                    if (pos + 1 < n) pick(word >> 16, n - pos - 1u, acc[h], pos + 1u - from);
                }
            }
            const uint32_t lo = even_bits32(acc[0]) | (even_bits32(acc[1]) << 16);
            const uint32_t hi = even_bits32(acc[0] >> 1) | (even_bits32(acc[1] >> 1) << 16);
            plo[d] = lo; phi[d] = hi; nlen[d] = (int)n;
        }
        if (C.has_fixed)
            for (int g = 0; g < C.K; g++) leads_type.set((uint32_t)g, P.fixed[g]);
    } else {
        uint64_t ord[DM];
        status = decode_candidate<DM>(P, idx, ord, nlen, leads_type);
#pragma unroll
        for (int d = 0; d < DM; d++) { plo[d] = even_bits(ord[d]); phi[d] = even_bits(ord[d] >> 1); }
    }

    // leads by code, walking every chain from its last block to its first; R gets a type as soon
    // as its producer's lead is ahead (the previous window already handled that micro-batch)
    Mu mu, Q;                        // leads by code; micro-batches waiting at the input of every type
    mu.lo = 0; mu.hi = 0;
    Q.lo = Q.hi = 0xFFFFFFFFFFFFFFFFull;          // 15: a chain's first block never waits
    uint32_t R = 0, HM = 0, X = 0;
    const bool draw_leads = sampled && !C.has_fixed;
    if (draw_leads) {
        // every dependency between different device sets steps the lead with probability step_q16 / 65536;
        // a lead is the number of steps from its type to the end of the chain, capped at N_R - 1
        uint32_t S = 0;
        for (int e = 0; e < C.ndeps; e += 2) {
            const uint32_t wv = stream_word(ka, kb, (kDrawLeadBase + (uint32_t)e) >> 1);
            // (the dependency's bit through scalar loads: the index is the same in every lane)
            const uint32_t b0 = P.dep_bit[e], b1 = e + 1 < C.ndeps ? P.dep_bit[e + 1] : 0u;
            S |= (wv & 0xFFFFu) < C.step_q16 ? b0 : 0u;
            S |= (wv >> 16) < C.step_q16 ? b1 : 0u;
        }
#pragma unroll
        for (int d = 0; d < DM; d++) {
            if (d >= C.D) continue;
            uint32_t mud = 0, qd = 0;
#pragma unroll
            for (int y = 0; y < kMaxLT; y++) {
                if (y >= C.ntd[d]) continue;
                const int c = 4 * d + y;
                const uint32_t pb = L.predbit_tab[c];
                const uint32_t cnt = (uint32_t)__builtin_popcount(S & L.cum_tab[c]);
                const uint32_t lead = min(NR - 1u, cnt);
                // micro-batches its producer handled in the previous window already; 15: no producer, never waits
                const uint32_t wait = pb ? min(NR - 1u, cnt + ((S & pb) ? 1u : 0u)) - lead : 15u;
                mud |= lead << (4 * y);
                qd |= wait << (4 * y);
                R |= (wait ? 1u : 0u) << c;
            }
            if (d < 4) { mu.lo |= (uint64_t)mud << (16 * d); Q.lo = (Q.lo & ~(0xFFFFull << (16 * d))) | ((uint64_t)qd << (16 * d)); }
            else { mu.hi |= (uint64_t)mud << (16 * (d - 4)); Q.hi = (Q.hi & ~(0xFFFFull << (16 * (d - 4)))) | ((uint64_t)qd << (16 * (d - 4))); }
        }
    } else {
        for (int k = 0; k < C.K; k++) {
            const uint32_t ct = L.chain_tab[k];
            const uint32_t c = ct & 63u, sc = (ct >> 6) & 63u;
            const bool has_succ = sc != 63u;
            const uint32_t lead_succ = mu.get(sc & 31u);
            const uint32_t lead = leads_type.get(ct >> 21);
            mu.set(c, lead);
            if (has_succ) Q.set(sc & 31u, lead - lead_succ);          // handled by the previous window already
            if (has_succ && lead > lead_succ) R |= 1u << (sc & 31u);
            if ((ct >> 20) & 1u) R |= 1u << c;
        }
        if (TP)
            for (int c = 0; c < 4 * C.D; c++) {           // the other codes of a type copy its lowest device's
                const uint32_t h = P.home_code[c];
                if (h == 63u || h == (uint32_t)c) continue;
                mu.set((uint32_t)c, mu.get(h));
                Q.set((uint32_t)c, Q.get(h));
                R |= ((R >> h) & 1u) << c;
            }
    }

    // per-device records
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= C.D) continue;
        const uint32_t mud = (uint32_t)((d < 4 ? mu.lo : mu.hi) >> (16 * (d & 3))) & 0xFFFFu;
        const uint32_t qd = (uint32_t)((d < 4 ? Q.lo : Q.hi) >> (16 * (d & 3))) & 0xFFFFu;
        int mem0 = 0;
#pragma unroll
        for (int y = 0; y < kMaxLT; y++) {
            if (y >= C.ntd[d]) continue;
            const uint32_t lead = (mud >> (4 * y)) & 15u;
            mem0 += ((int)(C.mpack[d] << (24 - 8 * y)) >> 24) * (int)lead;     // blocks that ran before the window
        }
        const uint32_t alive = nlen[d] >= 32 ? 0xFFFFFFFFu : (1u << nlen[d]) - 1u;
        rec_store(L.rec + (uint32_t)d * kRecDevStep + (uint32_t)lane * 4u, make_uint4(plo[d], phi[d], alive, qd | ((uint32_t)mem0 << 16)));
        if (nlen[d] > 0) HM |= 1u << (4 * d + ((plo[d] & 1u) | ((phi[d] & 1u) << 1)));
    }

    lead_code = mu;
    S.R = R; S.HM = HM; S.X = X; S.worst = INT_MIN; S.status = status;
}

// Places the blocks of program words [w_from, w_to) (six blocks a word).  `live`: the lane holds a candidate.
template <int DM, int MODE, bool TP>
__device__ __forceinline__ void build_words(const KParams &P, const FastConst<DM> &C, const FastLds &L, int lane, bool live,
                                            int w_from, int w_to, FastProgram &prog, BuildState &S)
{
    // With repair every candidate has an executable order (the blocks not yet placed form a DAG, so some type
    // is always runnable): no lane ever stops building, not even one without a candidate of the range (it scores
    // a real candidate whose result is dropped), and the per-lane predicate disappears from the loop.
    constexpr bool repair = MODE == 2;
    const int total = C.total;
    uint32_t R = S.R, HM = S.HM, X = S.X;
    int worst = S.worst, status = S.status;
    bool building = repair || (live && status == kOk);
    const uint32_t lane4 = (uint32_t)lane * 4u;
    const uint32_t rec_lane = L.rec + lane4;
    // one program word = six blocks
    auto word = [&](int wi) -> uint32_t {
        uint32_t acc = 0;
        const int nj = __builtin_amdgcn_readfirstlane(min(6, total - wi * 6));
#pragma unroll 1
        for (int j = 0; j < nj; j++) {
            uint32_t hm = R & HM;
            if (TP)
                for (int k = 0; k < C.ntp; k++) hm = (hm & C.tpg[k]) == C.tpg[k] ? hm : hm & ~C.tpg[k];
            const uint32_t sel = hm ? hm : (repair ? R : 0u);
            if (!repair && building && sel == 0) { status = kDeadlock; building = false; }
            const uint32_t b = low_bit(sel);
            uint32_t d4 = repair ? min(b & 28u, 4u * (DM - 1)) : building ? b & 28u : 0u;    // 4 * device
            TESSEL_PIN(d4);
            const uint32_t ra = (d4 << 8) + rec_lane;          // (kRecDevStep = 4 << 8)
            const uint4 a = rec_load(ra);
            // earliest remaining entry of the device whose type is runnable: a 4-way multiplexer keyed by the two
            // planes.  (When the device was picked for its runnable head this is the head: nothing precedes it.)
            const int r4 = (int)(R >> d4);
            const uint32_t r0 = (uint32_t)__builtin_amdgcn_sbfe(r4, 0, 1), r1 = (uint32_t)__builtin_amdgcn_sbfe(r4, 1, 1),
                           r2 = (uint32_t)__builtin_amdgcn_sbfe(r4, 2, 1), r3 = (uint32_t)__builtin_amdgcn_sbfe(r4, 3, 1);
            const uint32_t gate = bfi(a.y, bfi(a.x, r3, r2), bfi(a.x, r1, r0));
            const uint32_t p = low_bit(a.z & gate);
            // its symbol, as two all-or-nothing masks
            const uint32_t ly = (uint32_t)__builtin_amdgcn_sbfe((int)a.x, p, 1), hy = (uint32_t)__builtin_amdgcn_sbfe((int)a.y, p, 1);
            // c = d4 + y with y = (ly & 1) | (hy & 2): ly, hy are 0 or -1, so c = d4 - ly - 2 hy
            uint32_t c;
            asm("v_mad_i32_i24 %0, %1, -2, %2" : "=v"(c) : "v"(hy), "v"(d4 - ly));
            const uint32_t c4 = c << 2;
            const uint4 e = rec_load(c4);                      // (the table of the types starts the kernel's LDS, at address 0)
            // take the entry out; new head of the device.  (When the device is empty now the bit set below is
            // meaningless, and harmless: all its types are exhausted, and R never holds an exhausted type.)
            const uint32_t alive = a.z & ~(1u << p);
            const uint32_t p2 = low_bit(alive);
            const uint32_t y2 = __builtin_amdgcn_ubfe(a.x, p2, 1) | (__builtin_amdgcn_ubfe(a.y, p2, 1) << 1);
            const uint32_t hm_new = (HM & ~(15u << d4)) | (1u << (d4 + y2));
            // one waiting micro-batch is consumed; the type stays runnable while another one waits and
            // entries of it remain; its consumer gets one more and becomes runnable
            // remaining entries of the same type: alive & ~(lo ^ ly) & ~(hi ^ hy)
            const uint32_t rest = __builtin_amdgcn_bitop3_b32(__builtin_amdgcn_bitop3_b32(alive, a.x, ly, 0x90), a.y, hy, 0x90);
            // two or more were waiting (the shift, 4 * symbol, comes with the table entry where no type sits on several devices)
            const uint32_t more = (a.w >> (TP ? 4u * (c & 3u) : e.z >> 16)) & 14u;
            const uint32_t onec = 1u << c;
            // exhausted: no entry of the type is left; it stays runnable only if entries are left and another
            // micro-batch waits
            const bool exhausted = rest == 0, stalled = exhausted | (more == 0);
            uint32_t x_new = X | (exhausted ? onec : 0u);
            TESSEL_PIN(x_new);          // (the old X dies here: no second copy of the mask across the step)
            const uint32_t r_new = __builtin_amdgcn_bitop3_b32(R, stalled ? onec : 0u, e.y & ~x_new, 0xBA);      // (R & ~t) | z
            // the record's last word: waiting counts (16 bits) and the device's memory prefix (upper 16 bits,
            // signed); one sum updates both
            const uint32_t w_new = a.w + e.x;
            const bool active = repair || building;
            uint32_t r_fin = r_new, x_fin = x_new, hm_fin = hm_new;
            if (active) {
                lds_store(ra + 2u * kRecWordStep, alive);
                lds_store(ra + 3u * kRecWordStep, w_new);
                // (without blocks on several devices every table entry names a word: a type without a consumer on
                // another device adds 0 to its own record)
                if (!TP) lds_fetch_add((e.z & 0xFFFFu) + lane4, e.w);
                else if (e.z != 0xFFFFFFFFu) lds_fetch_add(e.z + lane4, e.w);
                worst = max(worst, (int)w_new >> 16);
                // the program names a type by its code on its lowest device
                acc |= (TP ? (uint32_t)__builtin_ctz(L.grp_tab[c]) : c) << (5 * j);
            }
            if (TP) {
                const bool slow = active && ((C.slow >> c) & 1u);
                if (__ballot(slow) != 0 && slow) {
                    // the type sits on several devices, or its consumer does: all codes of the type in R and X, its
                    // earliest entry out of every other device it occupies, one more waiting micro-batch on every
                    // device of the consumer (the table entry of such a type leaves all that to this path)
                    const uint32_t G = L.grp_tab[c], Gs = e.y;
                    const int mtype = (int)e.w;
                    x_fin = X | (rest == 0 ? G : 0u);
                    r_fin = (R & ~G) | (min(rest, more) != 0 ? G : 0u) | (Gs & ~x_fin);
#pragma unroll
                    for (int dd = 0; dd < DM; dd++) {
                        const uint32_t nib = (G >> (4 * dd)) & 15u;
                        if (dd >= C.D || nib == 0 || 4u * dd == d4) continue;
                        const uint32_t sym = (uint32_t)__builtin_ctz(nib);
                        const uint32_t rq = (uint32_t)dd * kRecDevStep + rec_lane;
                        const uint4 q = rec_load(rq);
                        const uint32_t ls = 0u - (sym & 1u), hs = 0u - (sym >> 1);
                        const uint32_t same = q.z & ~(q.x ^ ls) & ~(q.y ^ hs);
                        const uint32_t pos = (uint32_t)__builtin_ctz(same | 0x80000000u);
                        const uint32_t left = q.z & ~(1u << pos);
                        const uint32_t wq = q.w + ((uint32_t)mtype << 16) - (1u << (4u * sym));
                        lds_store(rq + 2u * kRecWordStep, left);
                        lds_store(rq + 3u * kRecWordStep, wq);
                        worst = max(worst, (int)wq >> 16);
                        const uint32_t ph = (uint32_t)__builtin_ctz(left | 0x80000000u);
                        const uint32_t yh = __builtin_amdgcn_ubfe(q.x, ph, 1) | (__builtin_amdgcn_ubfe(q.y, ph, 1) << 1);
                        hm_fin = (hm_fin & ~(15u << (4 * dd))) | (1u << (4 * dd + yh));
                    }
#pragma unroll
                    for (int dd = 0; dd < DM; dd++) {
                        const uint32_t nib = (Gs >> (4 * dd)) & 15u;
                        if (dd >= C.D || nib == 0) continue;
                        lds_fetch_add((uint32_t)dd * kRecDevStep + 3u * kRecWordStep + rec_lane, 1u << (4u * (uint32_t)__builtin_ctz(nib)));
                    }
                }
            }
            if (active) { R = r_fin; X = x_fin; HM = hm_fin; }
        }
        return acc;
    };
    // the program is two register vectors: one loop for each, so that a store never has to choose between them
    for (int wi = w_from; wi < min(w_to, 32); wi++) {
        if (!repair && __ballot(building) == 0) break;
        prog.a[wi] = word(wi);
    }
    for (int wi = max(w_from, 32); wi < w_to; wi++) {
        if (!repair && __ballot(building) == 0) break;
        prog.b[wi - 32] = word(wi);
    }
    S.R = R; S.HM = HM; S.X = X; S.worst = worst; S.status = status;
}

// the build's verdict once all blocks are placed
template <int DM>
__device__ __forceinline__ int build_end(const FastConst<DM> &C, const BuildState &S, int &peak_max)
{
    peak_max = 0;
    if (S.status != kOk) return S.status;
    int worst = S.worst;
#pragma unroll
    for (int d = 0; d < DM; d++)
        if (d < C.D && C.ntd[d] == 0) worst = max(worst, 0);      // a device without blocks holds nothing
    peak_max = worst;
    return worst > C.M ? kMem : kOk;
}

template <int DM, int VM, int MODE, bool TP = false>
__global__ __launch_bounds__(kWave, MODE ? 4 : 3) void eval_fast_kernel(const KParams *__restrict__ Pp, uint64_t first, uint64_t count,
                                                          BlockRec *__restrict__ recs, int32_t *__restrict__ code_out,
                                                          int32_t *__restrict__ peak_out, int tries, int retry_tries,
                                                          uint64_t *__restrict__ out_list, uint32_t *__restrict__ out_count,
                                                          uint32_t out_cap, uint32_t *__restrict__ overflow, uint32_t *ring_base,
                                                          uint32_t ring_words, int stage_words)
{
    extern __shared__ uint32_t lds[];
    // the sweeps address their tables by LDS byte address from 0: the kernel has no other LDS in front of this array
    if (lds_address(lds) != 0u) { if (threadIdx.x == 0) *overflow = 0x100u; return; }
    const KParams &P = *Pp;
    const int lane = threadIdx.x;
    FastLds L;
    L.type_tab = lds;                                         // 4 x 64 words, the upper half of every 64:
    L.chain_tab = lds + kMaxK;
    L.vtab = lds + 3 * kMaxK;
    L.cum_tab = lds + 5 * kMaxK;
    L.predbit_tab = lds + 7 * kMaxK;
    L.tt_tab = (uint4 *)(lds + kFastTableWords);              // 128 words, TP variants only
    L.grp_tab = lds + kFastTableWords + 4 * kMaxK;            // TP variants only
    L.sw_tab = lds + kSweepTabWord;
    L.ch_tab = lds + kSweepTabWord + kMaxK;
    L.in_tab = lds + kSweepTabWord + 2 * kMaxK;
    uint32_t *base = lds + kFastTableWords + (TP ? kTpTableWords : 0);
    L.rec = lds_address(base);
    // the sweep state is only used once the build is over: it shares the records' space when it fits
    const int ntok = P.nslots - P.D;
    const bool share = DM * 2 + ntok <= DM * 4;
    uint32_t *sweep_base = share ? base : base + DM * kWave * 4;
    L.dfree = sweep_base;                       // [DM] device times, [DM] counters, then the tokens
    L.dcnt = sweep_base + DM * kWave;
    L.tok = sweep_base + 2 * DM * kWave;
    if (lane < kMaxK) {
        const uint32_t inf = P.info_loc[lane];
        if (TP) L.tt_tab[lane] = make_uint4((uint32_t)P.t_loc[lane], ((((inf >> 12) & 63u) - (uint32_t)P.D + 2u * DM) << 8),
                                    ((uint32_t)lane >> 2) * (kWave * 4u), 16u + 4u * ((uint32_t)lane & 3u));
        {
            const uint32_t su = inf & 63u, dev = (uint32_t)lane >> 2, y = (uint32_t)lane & 3u;
            const int32_t m = (int32_t)(inf << 6) >> 24;
            const bool has_su = su != 63u, same = has_su && (su >> 2) == dev;
            const uint32_t inc = has_su ? 1u << (4u * (su & 3u)) : 0u;
            const uint32_t last = L.rec + 3u * kRecWordStep;          // last word of device 0's record, lane 0
            uint4 e;
            if (TP && ((P.slow_mask >> lane) & 1u))
                // a type on several devices, or with such a consumer: the step's slow path does the consumer's part
                e = make_uint4(((uint32_t)m << 16) - (1u << (4u * y)), has_su ? P.grp_code[su & 31u] : 0u, 0xFFFFFFFFu, (uint32_t)m);
            else
                e = make_uint4(((uint32_t)m << 16) - (1u << (4u * y)) + (same ? inc : 0u),
                               has_su ? 1u << (su & 31u) : 0u,
                               has_su && !same ? last + (su >> 2) * kRecDevStep + (TP ? 0u : y << 18)
                                               : TP ? 0xFFFFFFFFu : last + (dev < (uint32_t)DM ? dev : 0u) * kRecDevStep + (y << 18),
                               has_su && !same ? inc : 0u);
            L.type_tab[lane] = e.x; L.type_tab[2 * kMaxK + lane] = e.y; L.type_tab[4 * kMaxK + lane] = e.z; L.type_tab[6 * kMaxK + lane] = e.w;
        }
        {
            // codes no block type has: device 0, chain 0, t = 0 (the pipeline of the sweeps reads code 0 past the end)
            const bool used = P.t_loc[lane] != 0;
            const uint32_t dev = used ? (uint32_t)lane >> 2 : 0u, rel = used ? ((inf >> 12) & 63u) - (uint32_t)P.D : 0u;
            L.sw_tab[lane] = ((uint32_t)P.t_loc[lane] << 16) | (lds_address(L.dfree) + dev * (kWave * 4u));
            L.ch_tab[lane] = lds_address(L.dfree) + (2u * DM + rel) * (kWave * 4u);
            L.in_tab[lane] = (1u << (16u + 4u * ((uint32_t)lane & 3u))) | (16u + 4u * ((uint32_t)lane & 3u));
        }
        L.chain_tab[lane] = P.chain_tab[lane];
        L.vtab[lane] = lane < 24 ? P.vtab[lane] : 0u;
        if (TP) L.grp_tab[lane] = P.grp_code[lane] ? P.grp_code[lane] : 1u << lane;
        L.cum_tab[lane] = P.cum_code[lane]; L.predbit_tab[lane] = P.pred_bit[lane];
    }
    __syncthreads();
    FastConst<DM> C;
    C.D = P.D; C.K = P.K; C.NR = P.NR; C.M = P.M; C.total = P.total; C.nslots = P.nslots; C.npaths = P.npaths;
    C.nsweeps = P.nsweeps; C.space = P.space; C.has_fixed = P.has_fixed; C.nwords = (P.total + 5) / 6; C.ndeps = P.K - P.npaths;
    C.step_q16 = P.step_q16; C.seed = P.seed;
#pragma unroll
    for (int d = 0; d < DM; d++) { C.ntd[d] = P.ntd[d]; C.mpack[d] = P.mpack[d]; }
    C.ntp = TP ? P.ntp : 0; C.slow = TP ? P.slow_mask : 0u;
#pragma unroll
    for (int k = 0; k < kMaxD; k++) C.tpg[k] = TP ? P.tp_group[k] : 0u;

    int best = INT_MAX;
    uint64_t best_idx = 0;
    // counters of the whole wave (uniform values: they live in scalar registers)
    uint32_t cnt[kNumStatus];
#pragma unroll
    for (int s = 0; s < kNumStatus; s++) cnt[s] = 0;
    uint32_t nev = 0;
    uint32_t nsw = 0;                // per lane: window sweeps
    // The kernel works in three phases with a queue between each two, so that every phase runs on full waves
    // although candidates drop out on the way:
    //   A  decode + the first `stage_words` words of the build, one new candidate per lane;
    //   B  the rest of the build for the candidates that are still alive after A (with repair, and no per-candidate
    //      peak wanted: whose memory is within the cap so far; most candidates that exceed it do so early);
    //   C  the window sweeps for the candidates that survive the build.
    // A survivor of A appends its state (masks, records, program so far) to ring 1 of this wave in global memory,
    // a survivor of B program and leads to ring 2; B and C run whenever 64 candidates wait in their ring, one per
    // lane.  Ring layout: [word][slot]; slot = ring tail + rank of the lane among the survivors.
    // A candidate whose boundary vector is no eigenvector yet after the `tries` sweeps of C goes, with its program, to
    // ring 3 and gets up to `retry_tries` sweeps from the start when 64 of them wait there (a wave sweeps until its
    // slowest lane is done: a straggler among 63 finished lanes would cost a whole sweep of the wave).  What is still
    // open then is appended to the list of the general kernel.
    uint32_t *ring1 = ring_base + (size_t)blockIdx.x * 3u * ring_words, *ring2 = ring1 + ring_words, *ring3 = ring2 + ring_words;
    uint32_t head1 = 0, count1 = 0, head2 = 0, count2 = 0, head3 = 0, count3 = 0, nretry = 0, nblocks = 0;           // wave-uniform
    const int nwords = C.nwords;
    const bool split = stage_words < nwords;                         // tiny windows: A builds all of it
    const int wordsA = split ? stage_words : nwords;
    const int chunksA = (wordsA + 3) / 4, chunksAll = (nwords + 3) / 4;
    const bool drop_mem = MODE == 2 && peak_out == nullptr;          // a rejected candidate's peak is that of the whole window
    // every phase has a program of its own (words it does not write stay undefined and are never read), so that no
    // program lives on from one phase to the next
    Mu lead_code;
    BuildState S;

    auto rank_in = [&](uint64_t m) -> uint32_t {
        return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    };
    // a candidate the build rejects is final
    auto reject = [&](bool rejected, uint64_t idx, int status, int pk) {
        nev += (uint32_t)__builtin_popcountll(__ballot(rejected));
#pragma unroll
        for (int s = 1; s < kNumStatus; s++) cnt[s] += (uint32_t)__builtin_popcountll(__ballot(rejected && status == s));
        if (rejected) {
            if (code_out) code_out[idx - first] = -status;
            if (peak_out) peak_out[idx - first] = status == kMem ? pk : 0;
        }
    };
    auto push_program = [&](bool ok, uint64_t idx, int pk, const FastProgram &prog, uint32_t *ring, uint32_t tail) -> uint32_t {
        const uint64_t okm = __ballot(ok);
        if (okm == 0) return 0u;
        if (ok) {
            uint32_t *dst = ring + ((tail + rank_in(okm)) & (kRingSlots - 1u));
            dst[0 * kRingSlots] = (uint32_t)lead_code.lo; dst[1 * kRingSlots] = (uint32_t)(lead_code.lo >> 32);
            dst[2 * kRingSlots] = (uint32_t)lead_code.hi; dst[3 * kRingSlots] = (uint32_t)(lead_code.hi >> 32);
            dst[4 * kRingSlots] = (uint32_t)idx; dst[5 * kRingSlots] = (uint32_t)(idx >> 32);
            dst[6 * kRingSlots] = (uint32_t)pk;
#pragma unroll
            for (int c4 = 0; c4 < 12; c4++)
                if (c4 < chunksAll) {
#pragma unroll
                    for (int w = 4 * c4; w < 4 * c4 + 4; w++) dst[(kRingMetaWords + w) * kRingSlots] = prog.get(w);
                }
        }
        return (uint32_t)__builtin_popcountll(okm);
    };
    // phase C on the first n candidates of ring 2, or (`again`) of ring 3
    // (Wave priority by phase, set where a phase starts: the sweeps wait for the LDS after every few instructions and
    // issue first (3), then the second build phase (2), then the first (1: a build step waits for two rounds of LDS
    // reads); the decode, which always has an instruction ready, fills what is left (0).  Measured on windows of 256
    // blocks: 32.5 ms per 2^26 candidates against 37.3 with all waves equal; decode and first build phase both at 0
    // with the second at 1 or 2: 33.6 to 33.8; both build phases at 3: 34.3; the sweeps alone at 3: 35.9.)
    auto sweep_from_ring = [&](uint32_t n, bool again) {
        __builtin_amdgcn_s_setprio(3);
        __threadfence_block();         // the stores of this wave's other lanes must be visible to the loads below
        const bool have = (uint32_t)lane < n;
        const uint32_t *src = (again ? ring3 : ring2) + (((again ? head3 : head2) + (uint32_t)lane) & (kRingSlots - 1u));
        // every lane loads (a lane without a candidate reads a slot behind the last one: stale words, results dropped)
        FastProgram prog;
        lead_code.lo = (uint64_t)src[0 * kRingSlots] | ((uint64_t)src[1 * kRingSlots] << 32);
        lead_code.hi = (uint64_t)src[2 * kRingSlots] | ((uint64_t)src[3 * kRingSlots] << 32);
        const uint64_t idx = have ? (uint64_t)src[4 * kRingSlots] | ((uint64_t)src[5 * kRingSlots] << 32) : first;
        const int pk = (int)src[6 * kRingSlots];
#pragma unroll
        for (int c4 = 0; c4 < 12; c4++)
            if (c4 < chunksAll) {
#pragma unroll
                for (int w = 4 * c4; w < 4 * c4 + 4; w++) prog.set(w, src[(kRingMetaWords + w) * kRingSlots]);
            }
        if (again) { head3 = (head3 + n) & (kRingSlots - 1u); count3 -= n; }
        else { head2 = (head2 + n) & (kRingSlots - 1u); count2 -= n; }
        const int T = period_fast<DM, VM, TP>(C, L, prog, lane, lead_code, have, again ? retry_tries : tries, nsw);
        const bool open = have && T < 0;                  // no eigenvector within the sweeps allowed
        if (!again) {
            const uint32_t k = push_program(open, idx, pk, prog, ring3, head3 + count3);
            count3 += k; nretry += k;
        } else if (open) {
            const uint32_t at = atomicAdd(out_count, 1u);
            if (at < out_cap) out_list[at] = idx; else *overflow = 1u;
        }
        const bool scored = have && T >= 0;
        const uint32_t ns = (uint32_t)__builtin_popcountll(__ballot(scored));
        nev += ns;
        cnt[kOk] += ns;
        if (scored) {
            if (key_less(T, idx, best, best_idx)) { best = T; best_idx = idx; }
            if (code_out) code_out[idx - first] = T;
            if (peak_out) peak_out[idx - first] = pk;
        }
    };
    // the end of the build for the candidates the lanes hold: verdict, then ring 2 or out
    auto finish_build = [&](bool have, uint64_t idx, const FastProgram &prog) {
        int pk;
        const int status = build_end<DM>(C, S, pk);
        reject(have && status != kOk, idx, status, pk);
        count2 += push_program(have && status == kOk, idx, pk, prog, ring2, head2 + count2);
    };
    // phase B on the first n candidates of ring 1
    auto build_from_ring = [&](uint32_t n) {
        __builtin_amdgcn_s_setprio(2);
        __threadfence_block();
        const bool have = (uint32_t)lane < n;
        const uint32_t *src = ring1 + ((head1 + (uint32_t)lane) & (kRingSlots - 1u));
        FastProgram prog;
        S.status = kOk;
        S.R = src[0 * kRingSlots]; S.HM = src[1 * kRingSlots]; S.X = src[2 * kRingSlots]; S.worst = (int)src[3 * kRingSlots];
        lead_code.lo = (uint64_t)src[4 * kRingSlots] | ((uint64_t)src[5 * kRingSlots] << 32);
        lead_code.hi = (uint64_t)src[6 * kRingSlots] | ((uint64_t)src[7 * kRingSlots] << 32);
        const uint64_t idx = have ? (uint64_t)src[8 * kRingSlots] | ((uint64_t)src[9 * kRingSlots] << 32) : first;
#pragma unroll
        for (int d = 0; d < DM; d++)
            if (d < C.D)
                rec_store(L.rec + (uint32_t)d * kRecDevStep + (uint32_t)lane * 4u,
                          make_uint4(src[(kStageMetaWords + 4 * d) * kRingSlots], src[(kStageMetaWords + 4 * d + 1) * kRingSlots],
                                     src[(kStageMetaWords + 4 * d + 2) * kRingSlots], src[(kStageMetaWords + 4 * d + 3) * kRingSlots]));
#pragma unroll
        for (int c4 = 0; c4 < 12; c4++)
            if (c4 < chunksA) {
#pragma unroll
                for (int w = 4 * c4; w < 4 * c4 + 4; w++) prog.set(w, src[(kStageMetaWords + 4 * DM + w) * kRingSlots]);
            }
        head1 = (head1 + n) & (kRingSlots - 1u);
        count1 -= n;
        build_words<DM, MODE, TP>(P, C, L, lane, have, wordsA, nwords, prog, S);
        nblocks += n * (uint32_t)(C.total - min(C.total, 6 * wordsA));
        finish_build(have, idx, prog);
    };

    const uint64_t stride = (uint64_t)gridDim.x * kWave;
    const uint64_t rounds = (count + stride - 1) / stride;          // the same trip count for every lane of the grid
    // phase A on the next 64 candidates of the wave's share
    auto build_new = [&](uint64_t r) {
        const uint64_t kk = r * stride + (uint64_t)blockIdx.x * kWave + lane;
        const bool valid = kk < count;
        const uint64_t idx = valid ? first + kk : first;
        __builtin_amdgcn_s_setprio(0);
        build_begin<DM, MODE, TP>(P, C, idx, L, lane, lead_code, S);
        FastProgram prog;
        __builtin_amdgcn_s_setprio(1);
        build_words<DM, MODE, TP>(P, C, L, lane, valid, 0, wordsA, prog, S);
        nblocks += (uint32_t)__builtin_popcountll(__ballot(valid)) * (uint32_t)min(C.total, 6 * wordsA);
        if (!split) { finish_build(valid, idx, prog); return; }
        const bool over = drop_mem && S.status == kOk && S.worst > C.M;
        reject(valid && (S.status != kOk || over), idx, over ? (int)kMem : S.status, 0);
        const bool ok = valid && S.status == kOk && !over;
        const uint64_t okm = __ballot(ok);
        if (okm == 0) return;
        if (ok) {
            uint32_t *dst = ring1 + ((head1 + count1 + rank_in(okm)) & (kRingSlots - 1u));
            dst[0 * kRingSlots] = S.R; dst[1 * kRingSlots] = S.HM; dst[2 * kRingSlots] = S.X; dst[3 * kRingSlots] = (uint32_t)S.worst;
            dst[4 * kRingSlots] = (uint32_t)lead_code.lo; dst[5 * kRingSlots] = (uint32_t)(lead_code.lo >> 32);
            dst[6 * kRingSlots] = (uint32_t)lead_code.hi; dst[7 * kRingSlots] = (uint32_t)(lead_code.hi >> 32);
            dst[8 * kRingSlots] = (uint32_t)idx; dst[9 * kRingSlots] = (uint32_t)(idx >> 32);
#pragma unroll
            for (int d = 0; d < DM; d++)
                if (d < C.D) {
                    const uint4 q = rec_load(L.rec + (uint32_t)d * kRecDevStep + (uint32_t)lane * 4u);
                    dst[(kStageMetaWords + 4 * d) * kRingSlots] = q.x; dst[(kStageMetaWords + 4 * d + 1) * kRingSlots] = q.y;
                    dst[(kStageMetaWords + 4 * d + 2) * kRingSlots] = q.z; dst[(kStageMetaWords + 4 * d + 3) * kRingSlots] = q.w;
                }
#pragma unroll
            for (int c4 = 0; c4 < 12; c4++)
                if (c4 < chunksA) {
#pragma unroll
                    for (int w = 4 * c4; w < 4 * c4 + 4; w++) dst[(kStageMetaWords + 4 * DM + w) * kRingSlots] = prog.get(w);
                }
        }
        count1 += (uint32_t)__builtin_popcountll(okm);
    };

    // Later phases first: a ring is served as soon as it holds 64 candidates, so that it never holds more than 127;
    // when the wave's share is used up the rings are drained on partial waves.  Every condition is wave-uniform.
    for (uint64_t r = 0;;) {
        const bool fresh = r < rounds;
        // (one call for both rings of programs, so that the sweeps exist once in the code)
        const bool again = count3 >= (uint32_t)kWave || (!fresh && count1 == 0 && count2 == 0 && count3 > 0);
        const bool sweep = again || count2 >= (uint32_t)kWave || (!fresh && count1 == 0 && count2 > 0);
        if (sweep) sweep_from_ring(min(again ? count3 : count2, (uint32_t)kWave), again);
        else if (count1 >= (uint32_t)kWave || (!fresh && count1 > 0)) build_from_ring(min(count1, (uint32_t)kWave));
        else if (fresh) build_new(r++);
        else break;
    }
    if (!recs) return;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int op = __shfl_xor(best, off);
        uint32_t ilo = __shfl_xor((uint32_t)best_idx, off), ihi = __shfl_xor((uint32_t)(best_idx >> 32), off);
        uint64_t oi = ((uint64_t)ihi << 32) | ilo;
        if (key_less(op, oi, best, best_idx)) { best = op; best_idx = oi; }
        nsw += __shfl_xor(nsw, off);
    }
    if (lane == 0) {
        BlockRec rr;
        rr.period = best; rr.n_retried = nretry; rr.index = best_idx; rr.n_evaluated = nev; rr.n_sweeps = nsw; rr.n_blocks = nblocks; rr.pad = 0;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) rr.n_status[s] = cnt[s];
        recs[blockIdx.x] = rr;
    }
}

// ------------------------------------------------------------------ kernels
// Problems with more than kMaxD devices, kMaxK block types, kMaxLT types on a device or kMaxNR micro-batches per window (DM above kMaxD)
// are scored as dependency graphs, with the per-lane state and program in global memory (`far`: one region of
// far_words(P) words per workgroup) where the LDS of a workgroup does not hold them: 24 devices with 40 rings of 24
// slots and 384 program entries need 300 KB.
// (`where`: 1 = only the program lives there, the state stays in LDS; 2 = both)
__host__ __device__ inline size_t far_words(const KParams &P, int where)
{
    const size_t state = where == 2 ? (size_t)P.nslots * kWave * 4 : 0, prog = where ? (size_t)P.total * kWave * 2 : 0;
    return ((state + prog + 255) & ~(size_t)255) / 4;
}

template <int DM, int VM>
__global__ __launch_bounds__(kWave) void eval_kernel(const KParams *__restrict__ Pp, uint64_t first, uint64_t count,
                                                     BlockRec *__restrict__ recs, int32_t *__restrict__ code_out,
                                                     int32_t *__restrict__ peak_out, DevDetail *__restrict__ detail,
                                                     const uint64_t *__restrict__ list, const uint32_t *__restrict__ list_count,
                                                     uint32_t *far, int where)
{
    const KParams &P = *Pp;
    extern __shared__ uint32_t lds[];
    constexpr bool wide = DM > kMaxD;
    // with a list: score the listed candidates (all inside [first, first + count)) instead of the range
    if (list) count = min(*list_count, kWsListCap);
    constexpr int KT = wide ? kMaxKW : kMaxK;             // entries of a table by type
    int32_t *t_tab = (int32_t *)lds;
    uint32_t *mask_tab = lds + KT;
    // (wide problems: behind their five tables in LDS, or in this workgroup's region of the workspace: `where` = 1 the
    // program, 2 state and program)
    uint32_t *region = wide && where ? far + (size_t)blockIdx.x * far_words(P, where) : nullptr;
    uint32_t *state_all = !wide ? lds + 4 * kMaxK : where == 2 ? region : lds + 5 * kMaxKW;
    uint16_t *prog_all = where == 1 ? (uint16_t *)region : (uint16_t *)(state_all + P.nslots * kWave);
    const int lane = threadIdx.x;
    // by home code for chain problems, by type id (with the producers and the token rings) for the others
    DagTables Tb;
    Tb.t = t_tab; Tb.mask = mask_tab; Tb.pred = lds + 2 * KT; Tb.tok = lds + 3 * KT; Tb.pred_hi = wide ? lds + 4 * KT : nullptr;
    if (lane < KT) {
        t_tab[lane] = P.dag ? P.t_type[lane] : P.t_loc[lane];
        mask_tab[lane] = P.dag ? P.mask_type[lane] : P.mask_loc[lane];
        lds[2 * KT + lane] = (uint32_t)P.predmask[lane];
        lds[3 * KT + lane] = P.tokbase[lane];
        if (wide) lds[4 * KT + lane] = (uint32_t)(P.predmask[lane] >> 32);
    }
    __syncthreads();
    uint32_t *state = state_all + lane;
    uint16_t *prog = prog_all + lane;

    int best = INT_MAX;
    uint64_t best_idx = 0;
    uint32_t cnt[kNumStatus];
#pragma unroll
    for (int s = 0; s < kNumStatus; s++) cnt[s] = 0;
    uint32_t nev = 0;

    const uint64_t stride = (uint64_t)gridDim.x * kWave;
    for (uint64_t kk = (uint64_t)blockIdx.x * kWave + lane; kk < count; kk += stride) {
        const uint64_t idx = list ? list[kk] : first + kk;
        const uint64_t k = idx - first;
        int period, peak[DM];
        int status;
        if constexpr (wide) status = evaluate_dag<DM, MuWide>(P, Tb, idx, prog, state, period, peak, detail);
        else status = P.dag ? evaluate_dag<DM, Mu>(P, Tb, idx, prog, state, period, peak, detail)
                            : evaluate<DM, VM>(P, idx, prog, state, t_tab, mask_tab, period, peak, detail);
        nev++;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) cnt[s] += status == s;
        if (status == kOk && key_less(period, idx, best, best_idx)) { best = period; best_idx = idx; }
        int pk = 0;
        if (status == kOk || status == kMem) {
            pk = INT_MIN;
#pragma unroll
            for (int d = 0; d < DM; d++) if (d < P.D) pk = max(pk, peak[d]);
        }
        if (code_out) code_out[k] = status == kOk ? period : -status;
        if (peak_out) peak_out[k] = pk;
        if (detail) {
            detail->status = status; detail->period = period;
            for (int d = 0; d < kMaxDW; d++) detail->peak[d] = 0;
#pragma unroll
            for (int d = 0; d < DM; d++) if (d < P.D) detail->peak[d] = peak[d];
        }
    }
    if (!recs) return;
    // wave argmin over the total order (period, index); sums of the counters
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int op = __shfl_xor(best, off);
        uint32_t ilo = __shfl_xor((uint32_t)best_idx, off), ihi = __shfl_xor((uint32_t)(best_idx >> 32), off);
        uint64_t oi = ((uint64_t)ihi << 32) | ilo;
        if (key_less(op, oi, best, best_idx)) { best = op; best_idx = oi; }
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) cnt[s] += __shfl_xor(cnt[s], off);
        nev += __shfl_xor(nev, off);
    }
    if (lane == 0) {
        BlockRec r;
        r.period = best; r.n_retried = 0; r.index = best_idx; r.n_evaluated = nev; r.n_sweeps = 0; r.n_blocks = 0; r.pad = 0;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) r.n_status[s] = cnt[s];
        recs[blockIdx.x] = r;
    }
}

// The two instantiations for problems beyond the fast kernel's limits (16 and 32 devices) take as long to compile as
// everything else in this file: tessel_wide.hip includes this file up to here and holds them, so that the two halves
// build side by side.
#define TESSEL_EVAL_KERNEL_ARGS const KParams *, uint64_t, uint64_t, BlockRec *, int32_t *, int32_t *, DevDetail *, const uint64_t *, const uint32_t *, uint32_t *, int
#ifdef TESSEL_WIDE_INSTANTIATIONS
template __global__ void eval_kernel<16, 1>(TESSEL_EVAL_KERNEL_ARGS);
template __global__ void eval_kernel<32, 1>(TESSEL_EVAL_KERNEL_ARGS);
#else
extern template __global__ void eval_kernel<16, 1>(TESSEL_EVAL_KERNEL_ARGS);
extern template __global__ void eval_kernel<32, 1>(TESSEL_EVAL_KERNEL_ARGS);

// merges the block records of one launch into the running best (one wave)
__global__ __launch_bounds__(kWave) void merge_kernel(const BlockRec *recs, int nrecs, DevResult *res)
{
    const int lane = threadIdx.x;
    int best = INT_MAX;
    uint64_t best_idx = 0, nev = 0, nsw = 0, nbl = 0, cnt[kNumStatus];
    uint32_t nre = 0;
#pragma unroll
    for (int s = 0; s < kNumStatus; s++) cnt[s] = 0;
    for (int k = lane; k < nrecs; k += kWave) {
        BlockRec r = recs[k];
        nre += r.n_retried;
        if (key_less(r.period, r.index, best, best_idx)) { best = r.period; best_idx = r.index; }
        nev += r.n_evaluated;
        nsw += r.n_sweeps;
        nbl += r.n_blocks;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) cnt[s] += r.n_status[s];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int op = __shfl_xor(best, off);
        uint32_t ilo = __shfl_xor((uint32_t)best_idx, off), ihi = __shfl_xor((uint32_t)(best_idx >> 32), off);
        uint64_t oi = ((uint64_t)ihi << 32) | ilo;
        if (key_less(op, oi, best, best_idx)) { best = op; best_idx = oi; }
        uint32_t lo = __shfl_xor((uint32_t)nev, off), hi = __shfl_xor((uint32_t)(nev >> 32), off);
        nev += ((uint64_t)hi << 32) | lo;
        uint32_t slo = __shfl_xor((uint32_t)nsw, off), shi = __shfl_xor((uint32_t)(nsw >> 32), off);
        nsw += ((uint64_t)shi << 32) | slo;
        uint32_t blo = __shfl_xor((uint32_t)nbl, off), bhi = __shfl_xor((uint32_t)(nbl >> 32), off);
        nbl += ((uint64_t)bhi << 32) | blo;
        nre += __shfl_xor(nre, off);
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) {
            uint32_t l2 = __shfl_xor((uint32_t)cnt[s], off), h2 = __shfl_xor((uint32_t)(cnt[s] >> 32), off);
            cnt[s] += ((uint64_t)h2 << 32) | l2;
        }
    }
    if (lane == 0) {
        if (key_less(best, best_idx, res->period, res->index)) { res->period = best; res->index = best_idx; }
        // the pass over the list of deferred candidates has run (stream order)
        res->n_retried += nre;
        res->n_deferred += min(res->defer_count, kWsListCap);
        res->defer_count = 0;
        res->n_evaluated += nev;
        res->n_sweeps += nsw;
        res->n_blocks += nbl;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) res->n_status[s] += cnt[s];
    }
}

// only the counter of the deferred list (after a per-candidate scoring call)
__global__ void clear_defer_kernel(DevResult *res)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) res->defer_count = 0;
}

__global__ void reset_kernel(DevResult *res)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        res->period = INT_MAX; res->pad = 0; res->index = ~0ull; res->n_evaluated = 0; res->n_sweeps = 0; res->n_blocks = 0;
        res->n_retried = 0; res->n_deferred = 0; res->overflow = 0; res->defer_count = 0;
        for (int s = 0; s < kNumStatus; s++) res->n_status[s] = 0;
    }
}

// ------------------------------------------------------------------ launchers
typedef void (*eval_fn)(const KParams *, uint64_t, uint64_t, BlockRec *, int32_t *, int32_t *, DevDetail *, const uint64_t *,
                        const uint32_t *, uint32_t *, int);
typedef void (*fast_fn)(const KParams *, uint64_t, uint64_t, BlockRec *, int32_t *, int32_t *, int, int, uint64_t *, uint32_t *,
                        uint32_t, uint32_t *, uint32_t *, uint32_t, int);

// problems too wide for the fast kernel and the chain path (their state stays in LDS where 64 KB hold it)
static bool wide_problem(const KParams &kp) { return kp.D > kMaxD || kp.K > kMaxK || kp.many || kp.NR > kMaxNR; }

static eval_fn pick_kernel(const KParams &kp)
{
    const int V = kp.nsweeps - 1;
    if (kp.D > 16) return eval_kernel<32, 1>;
    if (wide_problem(kp)) return eval_kernel<16, 1>;
    if (kp.D <= 2 && V <= 4) return eval_kernel<2, 4>;
    if (kp.D <= 4 && V <= 8) return eval_kernel<4, 8>;
    if (kp.D <= 8 && V <= 16) return eval_kernel<8, 16>;
    return eval_kernel<8, 24>;
}

static int fast_dm(const KParams &kp) { return kp.D <= 2 ? 2 : kp.D <= 4 ? 4 : 8; }

static fast_fn pick_fast(const KParams &kp)
{
    const int V = kp.nsweeps - 1;
    if (!kp.fast_ok) return nullptr;
    if (kp.fast_tp) {
        // blocks on several devices
        if (kp.space == kSampledRepair)
            return kp.D <= 2 ? eval_fast_kernel<2, 24, 2, true> : kp.D <= 4 ? eval_fast_kernel<4, 24, 2, true> : eval_fast_kernel<8, 24, 2, true>;
        if (kp.space == kSampledStrict)
            return kp.D <= 2 ? eval_fast_kernel<2, 24, 1, true> : kp.D <= 4 ? eval_fast_kernel<4, 24, 1, true> : eval_fast_kernel<8, 24, 1, true>;
        return kp.D <= 2 ? eval_fast_kernel<2, 24, 0, true> : kp.D <= 4 ? eval_fast_kernel<4, 24, 0, true> : eval_fast_kernel<8, 24, 0, true>;
    }
    if (kp.space == kSampledRepair) {
        if (kp.D <= 2) return V <= 4 ? eval_fast_kernel<2, 4, 2> : eval_fast_kernel<2, 24, 2>;
        if (kp.D <= 4) return V <= 8 ? eval_fast_kernel<4, 8, 2> : eval_fast_kernel<4, 24, 2>;
        return V <= 16 ? eval_fast_kernel<8, 16, 2> : eval_fast_kernel<8, 24, 2>;
    }
    if (kp.space == kSampledStrict) {
        if (kp.D <= 2) return V <= 4 ? eval_fast_kernel<2, 4, 1> : eval_fast_kernel<2, 24, 1>;
        if (kp.D <= 4) return V <= 8 ? eval_fast_kernel<4, 8, 1> : eval_fast_kernel<4, 24, 1>;
        return V <= 16 ? eval_fast_kernel<8, 16, 1> : eval_fast_kernel<8, 24, 1>;
    }
    if (kp.D <= 2) return V <= 4 ? eval_fast_kernel<2, 4, 0> : eval_fast_kernel<2, 24, 0>;
    if (kp.D <= 4) return V <= 8 ? eval_fast_kernel<4, 8, 0> : eval_fast_kernel<4, 24, 0>;
    return V <= 16 ? eval_fast_kernel<8, 16, 0> : eval_fast_kernel<8, 24, 0>;
}

// state and program of the general kernel's lanes: in LDS, except for wide problems that 64 KB do not hold
// (the LDS one workgroup may ask for: what the device reports, 64 KB where there is none to ask)
static size_t lds_per_workgroup()
{
    static size_t cap = 0;
    if (!cap) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess &&
            v >= 64 * 1024)
            cap = (size_t)v < (size_t)160 * 1024 ? (size_t)v : (size_t)160 * 1024;
        else {
            (void)hipGetLastError();
            cap = 64 * 1024;
        }
    }
    return cap;
}
constexpr size_t kLdsAllBytes = 20 * 1024;       // state and program in LDS up to this much per workgroup (8 workgroups per CU)
constexpr size_t kLdsStateBytes = 40 * 1024;     // the state alone up to this much (4 per CU)
// Where the lanes' state and program of a wide problem live: 0 = in LDS, 1 = the program in the workspace, 2 = both.
// (TESSEL_FAR_MODE: tuning knob, honoured where the LDS allows it.)
static int far_mode(const KParams &kp)
{
    if (!wide_problem(kp)) return 0;
    const size_t tables = (size_t)5 * kMaxKW * 4, state = (size_t)kp.nslots * kWave * 4, prog = (size_t)kp.total * kWave * 2;
    int mode = tables + state + prog <= kLdsAllBytes ? 0 : tables + state <= kLdsStateBytes ? 1 : 2;
    if (const char *env = getenv("TESSEL_FAR_MODE")) {
        const int want = atoi(env);
        if (want == 2 || (want == 1 && tables + state <= lds_per_workgroup()) || (want == 0 && tables + state + prog <= lds_per_workgroup()))
            mode = want;
    }
    if (mode == 0 && tables + state + prog > lds_per_workgroup()) mode = 1;
    if (mode == 1 && tables + state > lds_per_workgroup()) mode = 2;
    return mode;
}
static size_t far_bytes(const KParams &kp) { return far_words(kp, far_mode(kp)) * 4; }

static size_t general_lds_bytes(const KParams &kp)
{
    if (wide_problem(kp)) {
        const int where = far_mode(kp);
        return (size_t)5 * kMaxKW * 4 + (where == 2 ? 0 : (size_t)kp.nslots * kWave * 4) + (where ? 0 : (((size_t)kp.total * kWave * 2 + 255) & ~(size_t)255));
    }
    return (size_t)4 * kMaxK * 4 + (size_t)kp.nslots * kWave * 4 + (size_t)kp.total * kWave * 2;
}

static size_t fast_lds_bytes(const KParams &kp)
{
    const int ntok = kp.nslots - kp.D;
    const bool share = fast_dm(kp) * 2 + ntok <= fast_dm(kp) * 4;
    return (size_t)(kFastTableWords + (kp.fast_tp ? kTpTableWords : 0)) * 4 + (size_t)fast_dm(kp) * kWave * 16 +
           (share ? 0 : (size_t)(fast_dm(kp) * 2 + ntok) * kWave * 4);
}

LaunchShape eval_launch_shape(const KParams &kp, int num_cus, int max_blocks)
{
    LaunchShape s;
    s.threads = kWave;
    fast_fn ff = pick_fast(kp);
    s.lds_bytes = ff ? fast_lds_bytes(kp) : general_lds_bytes(kp);
    // resident workgroups per CU as the runtime computes them from LDS and registers
    int per_cu = 0;
    const void *fn = ff ? (const void *)ff : (const void *)pick_kernel(kp);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWave, s.lds_bytes) != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        per_cu = (int)((160 * 1024) / ((s.lds_bytes + 511) / 512 * 512));
    }
    if (per_cu > 16) per_cu = 16;
    if (far_mode(kp) == 2 && per_cu > 4) per_cu = 4;                 // (keeps the state regions of a launch small)
    if (const char *env = getenv("TESSEL_BLOCKS_PER_CU")) {        // tuning knob: fewer resident workgroups per CU
        int want = atoi(env);
        if (want >= 1 && want < per_cu) per_cu = want;
    }
    if (per_cu < 1) per_cu = 1;
    s.blocks = num_cus * per_cu;
    if (max_blocks > 0 && s.blocks > max_blocks) s.blocks = max_blocks;      // a workspace with room for fewer queues
    return s;
}

// program words the fast kernel builds before the candidates that are still alive queue for the rest (most
// candidates that exceed the memory cap do so within the first blocks of the window): about two sevenths of the
// window, a multiple of four words; windows of fewer than ten words are built in one go
static int stage_words(const KParams &kp)
{
    const int nwords = (kp.total + 5) / 6;
    if (const char *env = getenv("TESSEL_STAGE_WORDS")) {           // tuning knob
        const int want = atoi(env);
        if (want >= 0 && want <= nwords) return want;
    }
    // (measured on windows of 256 blocks: 12 of 43 words; the queues move program words four at a time)
    return nwords >= 10 ? (nwords * 2 / 7 + 3) / 4 * 4 : nwords;
}

// the rings of the fast kernel's waves lie behind the block records, two per wave; words of one ring
static uint32_t ring_words(const KParams &kp)
{
    const int nwords = (kp.total + 5) / 6;
    const int program = (nwords + 3) / 4 * 4 + kRingMetaWords;
    const int stage = (nwords + 3) / 4 * 4 + kStageMetaWords + 4 * fast_dm(kp);     // any stage_words
    return (uint32_t)(program > stage ? program : stage) * kRingSlots;
}

// behind the records of one launch: one per workgroup of the scoring kernels, or one (smaller) per workgroup of the
// completion search, whose grid is 16 workgroups per compute unit at most
static size_t ring_offset(int blocks, int num_cus)
{
    const size_t eval = (size_t)(blocks + kDeferBlocks) * sizeof(BlockRec), comp = (size_t)num_cus * 16 * sizeof(CompRec);
    return (kWsBlockRecOff + (eval > comp ? eval : comp) + 256 + 255) & ~(size_t)255;
}

size_t eval_workspace_bytes(const KParams &kp, int num_cus, int max_blocks)
{
    const LaunchShape s = eval_launch_shape(kp, num_cus, max_blocks);
    return ring_offset(s.blocks, num_cus) + (pick_fast(kp) ? (size_t)s.blocks * 3 * ring_words(kp) * 4 : (size_t)s.blocks * far_bytes(kp));
}

// where the state regions of the general kernel's workgroups start (wide problems whose state does not fit the LDS)
static uint32_t *far_base(const KParams &kp, void *ws, int num_cus, int max_blocks)
{
    if (!far_mode(kp)) return nullptr;
    return (uint32_t *)((char *)ws + ring_offset(eval_launch_shape(kp, num_cus, max_blocks).blocks, num_cus));
}

static int launch_general(const KParams &kp, const KParams *kp_dev, uint64_t first, uint64_t count, int blocks, BlockRec *recs,
                          int32_t *code, int32_t *peak, DevDetail *detail, const uint64_t *list, const uint32_t *list_count,
                          uint32_t *far, hipStream_t st)
{
    const int where = far_mode(kp);
    if (where && !far) return (int)hipErrorInvalidValue;
    eval_fn fn = pick_kernel(kp);
    const size_t lds = general_lds_bytes(kp);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(kWave), lds, st, kp_dev, first, count, recs, code, peak, detail, list, list_count, far, where);
    return (int)hipGetLastError();
}

// Scores [first, first+count).  Where the problem allows it: the fast kernel (a short eigenvector search, a longer one
// for the candidates that did not converge), then the general kernel over what it could not finish (next to nothing).  Otherwise the general kernel alone.  Returns the number of block records written (recs may be
// null: per-candidate outputs only) or a negative HIP error.
static int launch_pass(const KParams &kp, uint64_t first, uint64_t count, void *ws, int num_cus, int max_blocks, BlockRec *recs,
                       int32_t *code, int32_t *peak, bool general, hipStream_t st)
{
    const KParams *kp_dev = (const KParams *)((char *)ws + kWsParamsOff);
    DevResult *res = (DevResult *)((char *)ws + kWsResultOff);
    uint64_t *list = (uint64_t *)((char *)ws + kWsListOff);
    LaunchShape s = eval_launch_shape(kp, num_cus, max_blocks);
    uint64_t need = (count + kWave - 1) / kWave;
    const int blocks = need < (uint64_t)s.blocks ? (int)need : s.blocks;
    if (blocks < 1) return 0;
    fast_fn ff = general ? nullptr : pick_fast(kp);
    if (!ff) {
        int rc = launch_general(kp, kp_dev, first, count, blocks, recs, code, peak, nullptr, nullptr, nullptr,
                                far_base(kp, ws, num_cus, max_blocks), st);
        return rc ? -rc : blocks;
    }
    const size_t lds = fast_lds_bytes(kp);
    uint32_t *ring = (uint32_t *)((char *)ws + ring_offset(s.blocks, num_cus));
    hipLaunchKernelGGL(ff, dim3(blocks), dim3(kWave), lds, st, kp_dev, first, count, recs, code, peak, kp.eigen_tries, kp.retry_tries,
                       list, &res->defer_count, kWsListCap, &res->overflow, ring, ring_words(kp), stage_words(kp));
    int rc = (int)hipGetLastError();
    if (rc) return -rc;
    rc = launch_general(kp, kp_dev, first, count, kDeferBlocks, recs ? recs + blocks : nullptr, code, peak, nullptr, list,
                        &res->defer_count, nullptr, st);
    return rc ? -rc : blocks + kDeferBlocks;
}

int launch_eval(const KParams &kp, uint64_t first, uint64_t count, void *ws, int num_cus, int max_blocks, void *stream, uint64_t max_piece)
{
    hipStream_t st = (hipStream_t)stream;
    BlockRec *recs = (BlockRec *)((char *)ws + kWsBlockRecOff);
    DevResult *res = (DevResult *)((char *)ws + kWsResultOff);
    // pieces of at most max_piece candidates, so that the lists of unfinished candidates stay small
    for (uint64_t done = 0; done < count;) {
        const uint64_t piece = count - done < max_piece ? count - done : max_piece;
        int n = launch_pass(kp, first + done, piece, ws, num_cus, max_blocks, recs, nullptr, nullptr, false, st);
        if (n < 0) return -n;
        if (n > 0) {
            hipLaunchKernelGGL(merge_kernel, dim3(1), dim3(kWave), 0, st, recs, n, res);
            int rc = (int)hipGetLastError();
            if (rc) return rc;
        }
        done += piece;
    }
    return 0;
}

int launch_score(const KParams &kp, uint64_t first, uint64_t count, int32_t *code, int32_t *peak, void *ws, int num_cus,
                 int max_blocks, bool general, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    DevResult *res = (DevResult *)((char *)ws + kWsResultOff);
    // pieces in which no list can overflow: the per-candidate outputs of a dropped candidate would stay unwritten
    const uint64_t max_piece = kSafePerLaunch;
    for (uint64_t done = 0; done < count;) {
        const uint64_t piece = count - done < max_piece ? count - done : max_piece;
        int n = launch_pass(kp, first + done, piece, ws, num_cus, max_blocks, nullptr, code + done, peak ? peak + done : nullptr, general, st);
        if (n < 0) return -n;
        hipLaunchKernelGGL(clear_defer_kernel, dim3(1), dim3(1), 0, st, res);
        int rc = (int)hipGetLastError();
        if (rc) return rc;
        done += piece;
    }
    return 0;
}

int launch_detail(const KParams &kp, uint64_t index, void *ws, int num_cus, int max_blocks, void *stream)
{
    int rc = launch_general(kp, (const KParams *)((char *)ws + kWsParamsOff), index, 1, 1, nullptr, nullptr, nullptr,
                            (DevDetail *)((char *)ws + kWsDetailOff), nullptr, nullptr, far_base(kp, ws, num_cus, max_blocks),
                            (hipStream_t)stream);
    return rc;
}

int launch_reset(void *ws, void *stream)
{
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, (DevResult *)((char *)ws + kWsResultOff));
    return (int)hipGetLastError();
}

size_t block_rec_bytes(int blocks) { return (size_t)blocks * sizeof(BlockRec); }

// ------------------------------------------------------------------ a workspace the library holds itself
// For callers that cannot allocate device memory: one buffer per GPU, part of the code object, shared by every call
// on that GPU (it keeps the last call's contents; the kernels clear what has to start at zero).  In host code the
// array's name stands for the symbol, not for device memory: its address on the current device comes from
// hipGetSymbolAddress, once per device.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

int scratch_workspace(void **ptr, size_t *bytes)
{
    constexpr int kMaxGpus = 64;
    static void *address[kMaxGpus] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxGpus) return (int)hipErrorInvalidDevice;
    if (!address[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        address[dev] = p;
    }
    *ptr = address[dev];
    *bytes = kScratchBytes;
    return 0;
}

// the largest grid of the scoring kernels whose records and queues fit `bytes`; 0: not even one workgroup
int eval_blocks_that_fit(const KParams &kp, int num_cus, size_t bytes)
{
    const size_t per_block = sizeof(BlockRec) + (pick_fast(kp) ? (size_t)3 * ring_words(kp) * 4 : far_bytes(kp));
    const size_t fixed = ring_offset(0, num_cus) + 512;
    if (bytes < fixed + per_block) return 0;
    int blocks = (int)std::min<size_t>((bytes - fixed) / per_block, (size_t)num_cus * 16);
    while (blocks > 0 && eval_workspace_bytes(kp, num_cus, blocks) > bytes) blocks--;
    return blocks;
}


// ==================================================================== searched completion
// Warm-up and cool-down around R copies of the best window (Sec. IV-C).  The paper orders the two outer
// phases with a time-optimal solver; here many perturbed greedy list schedules are tried, one per lane,
// and the shortest complete schedule wins.  Completion candidate `ordinal`: per phase every block type
// offers its lowest unscheduled micro-batch (Property 1); an offered block is eligible when its producer's
// block of the same micro-batch is scheduled and its memory delta fits on all its devices; the eligible
// block with the smallest (earliest start + jitter, micro-batch, type id) is appended at its earliest
// start.  jitter(type, mu) = (draw * (J + 1)) >> 16 with draw number type*N + mu of the stream keyed by the
// ordinal; ordinal 0 has no jitter (the plain greedy schedule).
// Per-lane state in LDS [slot][lane], 16-bit words: end time of the latest block of every micro-batch in flight
// (a ring per chain), free time and memory of every device, next micro-batch and its jitter of every type; behind
// it, for problems with every type on one device, one 32-bit sort key per type.
constexpr int kCompParamWords = 352;       // start of the LDS: the parameter block's copy, then three tables of kMaxK words at the end
static_assert(sizeof(CompParams) <= (kCompParamWords - 3 * kMaxK) * 4, "parameter block and per-type tables share the start of the LDS");

__global__ __launch_bounds__(kWave) void complete_kernel(const CompParams *__restrict__ cpg, const CompMatrix *__restrict__ cmg,
                                                         uint64_t first, uint64_t count,
                                                         CompRec *__restrict__ recs, int32_t *__restrict__ makespan_out)
{
    extern __shared__ uint32_t lds[];
    for (int w = threadIdx.x; w < (int)(sizeof(CompParams) / 4); w += kWave) lds[w] = ((const uint32_t *)cpg)[w];
    __syncthreads();
    const CompParams &cp = *(const CompParams *)lds;
    const int lane = threadIdx.x;
    uint16_t *state = (uint16_t *)(lds + kCompParamWords) + lane;      // 16-bit words: all times stay below 65536 (checked by the host)
    const int D = cp.D, K = cp.K, N = cp.N, NR = cp.NR, M = cp.M, J = cp.J, R = cp.R;
    // a type's next micro-batch (low 10 bits) and the jitter of that block (high 6 bits) share a word: N < 1024 and
    // J < 64 (checked by the host)
    const int TR = cp.tok_ring, tmask = TR - 1;          // end times of the micro-batches in flight: [chain][mu mod TR]
    const int trs = __builtin_ctz((uint32_t)TR);         // (a power of two)
    // (one more slot behind the state and one more row behind the keys take the stores of lanes that have nothing to
    // store, so that no store needs a branch)
    const int oTok = 0, oFree = cp.npaths * TR, oMem = oFree + D, oNext = oMem + D, oTrash = oNext + K, nstate = oTrash + 1;
    // Problems with every type on one device (and at most 8 chains) take a path that keeps, per type, the sort key of
    // its offered block in LDS and touches only the types a scheduled block can change: its own type and its consumers
    // are recomputed (`redo`); of the other types on its device (`aff`) a key that exists only moves to the device's new
    // free time and is checked against its new memory.  Tables, per type: `ptab` lead (8 bits), memory delta (8,
    // signed), producer + 1 (6), device (3), chain (3), 1 (a type of the problem) in one word.
    bool single_dev = cp.npaths <= 8 && !cp.dag;
    for (int i = 0; i < K; i++) single_dev = single_dev && (cp.mask[i] & (cp.mask[i] - 1)) == 0 && cp.mask[i] != 0;
    uint32_t *ptab = lds + kCompParamWords - 3 * kMaxK, *aff = lds + kCompParamWords - 2 * kMaxK, *redo = lds + kCompParamWords - kMaxK;
    if (lane < kMaxK) {
        uint32_t pw = 0, af = 0, rd = 0;
        if (lane < K) {
            pw = (uint32_t)cp.lead[lane] | ((uint32_t)(uint8_t)cp.m[lane] << 8) | ((uint32_t)(cp.pred[lane] + 1) << 16) |
                 ((uint32_t)__builtin_ctz((uint32_t)cp.mask[lane] | 0x100u) << 22) | ((uint32_t)cp.path[lane] << 25) | 1u << 28;
            rd = 1u << lane;
            for (int j = 0; j < K; j++) {
                if (cp.pred[j] == lane) rd |= 1u << j;
                if ((cp.mask[j] & cp.mask[lane]) != 0) af |= 1u << j;
            }
            af &= ~rd;
        }
        ptab[lane] = pw; aff[lane] = af; redo[lane] = rd;
    }
    // some type has several consumers, or more than three other types on its device (wave-uniform)
    const bool crowded = __ballot(lane < K && (__builtin_popcount(redo[lane]) > 2 || __builtin_popcount(aff[lane]) > 3)) != 0;
    __syncthreads();
    uint32_t *ckey = lds + kCompParamWords + (nstate + 1) / 2 * kWave + lane;      // [type][lane], behind the 16-bit state
    // ... and behind the keys what the replay of the R windows needs.  Either their (max, +) matrix: kMatIn slot
    // numbers of the inputs, kMatOut of the outputs, then one row of kMatIn path lengths per output; or (no matrix: too
    // many values cross the windows) one word per block of the window: device (3 bits), chain (3), micro-batch within
    // the first window = lead + occurrence (8), has a producer (1), t (16)
    uint32_t *rtab = lds + kCompParamWords + (nstate + 1) / 2 * kWave + (K + 1) * kWave;
    const int nin = single_dev ? cmg->nin : 0, nout = cmg->nout;
    if (nin > 0) {
        for (int s = lane; s < kMatIn; s += kWave) rtab[s] = cmg->in_slot[s];
        for (int s = lane; s < kMatOut; s += kWave) rtab[kMatIn + s] = cmg->out_slot[s];
        for (int s = lane; s < nout * kMatIn; s += kWave) rtab[kMatIn + kMatOut + s] = (uint32_t)cmg->a[s / kMatIn][s % kMatIn];
        __syncthreads();
    } else if (single_dev) {
        for (int s = lane; s < cp.nseq; s += kWave) {
            const uint32_t pw = ptab[cp.seq[s]];
            rtab[s] = (pw >> 22 & 7u) | (pw >> 25 & 7u) << 3 | ((pw & 255u) + (uint32_t)cp.occ[s]) << 6 |
                      ((pw >> 16 & 63u) != 0 ? 1u << 14 : 0u) | (uint32_t)cp.t[cp.seq[s]] << 16;
        }
        __syncthreads();
    }
#define TESSEL_ST(slot) state[(slot) * kWave]
    int best = INT_MAX;
    uint64_t best_ord = 0;
    const uint64_t stride = (uint64_t)gridDim.x * kWave;
    const uint64_t rounds = (count + stride - 1) / stride;          // the same trip count for every lane of the grid
    for (uint64_t r = 0; r < rounds; r++) {
        const uint64_t kk = r * stride + (uint64_t)blockIdx.x * kWave + lane;
        const bool live = kk < count;
        const uint64_t c = first + (live ? kk : 0);
        uint32_t kb;
        const uint32_t ka = stream_keys(((uint64_t)cp.seed_hi << 32) | cp.seed_lo, c, kb);
        const bool noisy = c != 0 && J > 0;
        auto jitter = [&](int i, int mu) -> uint32_t {
            return noisy ? (stream_draw16(ka, kb, (uint32_t)(i * N + mu)) * (uint32_t)(J + 1)) >> 16 : 0u;
        };
        for (int s = 0; s < nstate; s++) TESSEL_ST(s) = 0;
        bool fail = false;
        for (int phase = 0; phase < 2; phase++) {
            // ---- greedy phase: 0 warm-up (micro-batches below the leads), 1 cool-down (the rest up to N)
            int left = 0;                                       // blocks of this phase not yet scheduled
            for (int i = 0; i < K; i++) {
                const int mu = (int)TESSEL_ST(oNext + i) & 1023, hi = phase ? N : (int)cp.lead[i];
                TESSEL_ST(oNext + i) = (uint16_t)((uint32_t)mu | (mu < hi ? jitter(i, mu) : 0u) << 10);
                left += max(hi - mu, 0);
            }
            // sort key of the block type i offers, (start + jitter, micro-batch, type) in one word, smallest first:
            // start + jitter < 2^16 (checked by the host) in bits 15-30, micro-batch < 2^10, type < 2^5.  All ones:
            // nothing offered, or its producer has not handled the micro-batch yet; bit 31 on a key: offered, but its
            // memory does not fit now (the key below stays valid)
            auto offer_key = [&](int i) -> uint32_t {
                const uint32_t pw = ptab[i];
                const bool has_a = (pw >> 16 & 63u) != 0;
                const int hi = phase ? N : (int)(pw & 255u), a = (int)(pw >> 16 & 63u) - 1, d = (int)(pw >> 22 & 7u);
                const int mi = (int)(int8_t)(pw >> 8);
                const int nj = (int)TESSEL_ST(oNext + i), mu = nj & 1023;
                const int na = (int)TESSEL_ST(oNext + (has_a ? a : i)) & 1023;
                const int fr = (int)TESSEL_ST(oFree + d), me = (int)(int16_t)TESSEL_ST(oMem + d);
                const int tk = (int)TESSEL_ST(oTok + ((int)(pw >> 25 & 7u) << trs) + (mu & tmask));
                const bool offered = (mu < hi) & (!has_a | (na > mu)), fits = (mi <= 0) | (me + mi <= M);
                const uint32_t key = (uint32_t)(max(has_a ? tk : 0, fr) + (nj >> 10));
                return offered ? (key << 15) | ((uint32_t)mu << 5) | (uint32_t)i | (fits ? 0u : 0x80000000u) : 0xFFFFFFFFu;
            };
            if (single_dev) {
                // ---- every type on one device: one straight-line step per scheduled block
                for (int i = 0; i < K; i++) ckey[i * kWave] = offer_key(i);
                for (;;) {
                    const bool busy = live && !fail && left > 0;
                    if (__ballot(busy) == 0) break;
                    uint32_t bestp = 0xFFFFFFFFu;
#pragma unroll 8
                    for (int i = 0; i < K; i++) bestp = min(bestp, ckey[i * kWave]);
                    const bool placed = busy && bestp < 0x80000000u;
                    fail = fail | (busy && !placed);              // blocks left, none eligible: no schedule
                    // A lane that places nothing goes through the step with type 0 and writes nothing.  The step is
                    // three rounds of LDS reads, each issued as a whole before anything waits for it (the values are
                    // pinned so that no read sinks into a branch): (1) the table words of the block's type; (2) what
                    // they name: the memory of its device, the table word and counter of its consumer, key, table word
                    // and counter of the other types on its device, its producer's counter and the end time its own
                    // next micro-batch waits for; (3) after the writes of the block, the consumer's device and token.
                    const int b = placed ? (int)(bestp & 31u) : 0, bmu = (int)(bestp >> 5 & 1023u), mu1 = bmu + 1;
                    uint32_t pw = ptab[b], rdw = redo[b], af = aff[b], tb = (uint32_t)cp.t[b], njb = TESSEL_ST(oNext + b);
                    TESSEL_PIN(pw); TESSEL_PIN(rdw); TESSEL_PIN(af); TESSEL_PIN(tb); TESSEL_PIN(njb);
                    const uint32_t rd = rdw & ~(1u << b), af1 = af & (af - 1u), af2 = af1 & (af1 - 1u);
                    const bool has_c = placed && rd != 0, h0 = placed && af != 0, h1 = placed && af1 != 0, h2 = placed && af2 != 0;
                    const int c = has_c ? __builtin_ctz(rd) : b;
                    const int a0 = h0 ? __builtin_ctz(af) : b, a1 = h1 ? __builtin_ctz(af1) : b, a2 = h2 ? __builtin_ctz(af2) : b;
                    const int d = (int)(pw >> 22 & 7u), mi_b = (int)(int8_t)(pw >> 8), hi_b = phase ? N : (int)(pw & 255u);
                    const bool has_ab = (pw >> 16 & 63u) != 0;
                    uint32_t me_old = TESSEL_ST(oMem + d), pwc = ptab[c], njc = TESSEL_ST(oNext + c);
                    uint32_t k0 = ckey[a0 * kWave], p0 = ptab[a0], n0 = TESSEL_ST(oNext + a0);
                    uint32_t k1 = ckey[a1 * kWave], p1 = ptab[a1], n1 = TESSEL_ST(oNext + a1);
                    uint32_t k2 = ckey[a2 * kWave], p2 = ptab[a2], n2 = TESSEL_ST(oNext + a2);
                    uint32_t napb = TESSEL_ST(oNext + (has_ab ? (int)(pw >> 16 & 63u) - 1 : b));
                    uint32_t tkb = TESSEL_ST(oTok + ((int)(pw >> 25 & 7u) << trs) + (mu1 & tmask));
                    TESSEL_PIN(me_old); TESSEL_PIN(pwc); TESSEL_PIN(njc); TESSEL_PIN(k0); TESSEL_PIN(p0); TESSEL_PIN(n0);
                    TESSEL_PIN(k1); TESSEL_PIN(p1); TESSEL_PIN(n1); TESSEL_PIN(k2); TESSEL_PIN(p2); TESSEL_PIN(n2);
                    TESSEL_PIN(napb); TESSEL_PIN(tkb);
                    const int en = (int)(bestp >> 15) - (int)(njb >> 10) + (int)tb;
                    const int me_new = (int)(int16_t)me_old + mi_b;
                    uint32_t jn = (stream_draw16(ka, kb, (uint32_t)(b * N + mu1)) * (uint32_t)(J + 1)) >> 16;
                    TESSEL_PIN(jn);
                    jn = noisy ? jn : 0u;
                    const uint32_t njb_new = (uint32_t)mu1 | (mu1 < hi_b ? jn : 0u) << 10;
                    TESSEL_ST(placed ? oFree + d : oTrash) = (uint16_t)en;
                    TESSEL_ST(placed ? oMem + d : oTrash) = (uint16_t)me_new;
                    TESSEL_ST(placed ? oTok + ((int)(pw >> 25 & 7u) << trs) + (bmu & tmask) : oTrash) = (uint16_t)en;
                    TESSEL_ST(placed ? oNext + b : oTrash) = (uint16_t)njb_new;
                    left -= placed ? 1 : 0;
                    // round 3: the consumer's device and the end time of the micro-batch it waits for, as they are now
                    const int dc = (int)(pwc >> 22 & 7u), muc = (int)(njc & 1023u);
                    uint32_t frc = TESSEL_ST(oFree + dc), mec = TESSEL_ST(oMem + dc);
                    uint32_t tkc = TESSEL_ST(oTok + ((int)(pwc >> 25 & 7u) << trs) + (muc & tmask));
                    TESSEL_PIN(frc); TESSEL_PIN(mec); TESSEL_PIN(tkc);
                    // The scheduled block changes what its own type and its consumer offer (recomputed; the block's
                    // own values are at hand), and for the other types on its device (three at most) the free time and
                    // the memory: start = max(end of the producer's block, device free), and the device was free no
                    // later than now before, so the new key is max(old key, new free time + jitter); the same
                    // micro-batch stays offered.
                    const uint32_t blocked = 0x80000000u;
                    uint32_t key_b, key_c;
                    {
                        const bool offered = (mu1 < hi_b) & (!has_ab | ((int)(napb & 1023u) > mu1));
                        const bool fits = (mi_b <= 0) | (me_new + mi_b <= M);
                        const uint32_t key = (uint32_t)max(has_ab ? (int)tkb : 0, en) + (njb_new >> 10);
                        uint32_t word = (key << 15) | ((uint32_t)mu1 << 5) | (uint32_t)b | (fits ? 0u : blocked);
                        TESSEL_PIN(word);                  // (computed in every lane: cheaper than a branch around it)
                        key_b = offered ? word : 0xFFFFFFFFu;
                    }
                    {
                        const int hic = phase ? N : (int)(pwc & 255u), mic = (int)(int8_t)(pwc >> 8);
                        const bool offered = (muc < hic) & (mu1 > muc);            // (its producer is the block's type)
                        const bool fits = (mic <= 0) | ((int)(int16_t)mec + mic <= M);
                        const uint32_t key = max(tkc, frc) + (njc >> 10);
                        uint32_t word = (key << 15) | ((uint32_t)muc << 5) | (uint32_t)c | (fits ? 0u : blocked);
                        TESSEL_PIN(word);
                        key_c = offered ? word : 0xFFFFFFFFu;
                    }
                    auto moved = [&](uint32_t k, uint32_t pwi, uint32_t nji) -> uint32_t {
                        const int mi = (int)(int8_t)(pwi >> 8);
                        const uint32_t start = max(k << 1 >> 16, (uint32_t)en + (nji >> 10));
                        const bool fits = (mi <= 0) | (me_new + mi <= M);
                        uint32_t word = (start << 15) | (k & 0x7FFFu) | (fits ? 0u : blocked);
                        TESSEL_PIN(word);
                        return k == 0xFFFFFFFFu ? k : word;
                    };
                    k0 = moved(k0, p0, n0); k1 = moved(k1, p1, n1); k2 = moved(k2, p2, n2);
                    ckey[(placed ? b : K) * kWave] = key_b;
                    ckey[(has_c ? c : K) * kWave] = key_c;
                    ckey[(h0 ? a0 : K) * kWave] = k0;
                    ckey[(h1 ? a1 : K) * kWave] = k1;
                    ckey[(h2 ? a2 : K) * kWave] = k2;
                    if (crowded) {
                        // a type with several consumers, or more than four types on a device: the rest one by one
                        uint32_t todo = placed ? rd & (rd - 1u) : 0u;
                        while (__ballot(todo != 0u) != 0) {
                            if (todo != 0u) {
                                const int i = __builtin_ctz(todo);
                                todo &= todo - 1u;
                                ckey[i * kWave] = offer_key(i);
                            }
                        }
                        todo = placed ? af2 & (af2 - 1u) : 0u;
                        while (__ballot(todo != 0u) != 0) {
                            if (todo != 0u) {
                                const int i = __builtin_ctz(todo);
                                todo &= todo - 1u;
                                ckey[i * kWave] = moved(ckey[i * kWave], ptab[i], TESSEL_ST(oNext + i));
                            }
                        }
                    }
                }
            } else
            for (;;) {
                int bi = -1, bmu = 0, best_est = 0, bkey = 0;
                const bool any = left > 0;
                for (int i = 0; i < K; i++) {
                    const int hi = phase ? N : (int)cp.lead[i];
                    if (hi == 0) continue;                       // nothing of this type in the phase (uniform)
                    const int nj = (int)TESSEL_ST(oNext + i), mu = nj & 1023;
                    const bool offered = mu < hi;
                    if (__ballot(offered) == 0) continue;        // every lane is through with the type
                    const int a = cp.pred[i], mi = cp.m[i];
                    const uint32_t mask = cp.mask[i];
                    bool ok = offered;
                    int est = 0;
                    if (cp.dag) {
                        // every producer has handled the micro-batch; the latest of their end times
                        for (uint32_t rest = cp.predmask[i]; rest; rest &= rest - 1u) {
                            const int pa = __builtin_ctz(rest);
                            ok = ok && ((int)TESSEL_ST(oNext + pa) & 1023) > mu;
                            est = max(est, (int)TESSEL_ST(oTok + (int)cp.path[pa] * TR + (mu & tmask)));
                        }
                    } else if (a >= 0) {
                        ok = ok && ((int)TESSEL_ST(oNext + a) & 1023) > mu;
                        est = (int)TESSEL_ST(oTok + (int)cp.path[i] * TR + (mu & tmask));
                    }
                    for (uint32_t rest = mask; rest; rest &= rest - 1u) {          // the block's devices (uniform)
                        const int d = __builtin_ctz(rest);
                        if (mi > 0 && (int)(int16_t)TESSEL_ST(oMem + d) + mi > M) ok = false;
                        est = max(est, (int)TESSEL_ST(oFree + d));
                    }
                    const int key = est + (nj >> 10);
                    // types ascend, so on equal (key, micro-batch) the earlier type stays
                    if (ok && (bi < 0 || key < bkey || (key == bkey && mu < bmu))) { bi = i; bmu = mu; best_est = est; bkey = key; }
                }
                const bool busy = live && !fail && any;
                if (__ballot(busy) == 0) break;
                if (busy && bi < 0) fail = true;                  // blocks left, none eligible: no schedule
                if (busy && bi >= 0) {
                    const int en = best_est + cp.t[bi];
                    const int mi = cp.m[bi], hi = phase ? N : (int)cp.lead[bi];
                    const uint32_t mask = cp.mask[bi];
                    for (int d = 0; d < D; d++)
                        if (mask >> d & 1u) { TESSEL_ST(oFree + d) = (uint16_t)en; TESSEL_ST(oMem + d) = (uint16_t)((int)(int16_t)TESSEL_ST(oMem + d) + mi); }
                    TESSEL_ST(cp.path[bi] != 0xFF ? oTok + (int)cp.path[bi] * TR + (bmu & tmask) : oTrash) = (uint16_t)en;
                    TESSEL_ST(oNext + bi) = (uint16_t)((uint32_t)(bmu + 1) | (bmu + 1 < hi ? jitter(bi, bmu + 1) : 0u) << 10);
                    left--;
                }
            }
            if (phase == 1) break;
            // ---- the R windows: the same blocks at the same micro-batches in every lane.  (Every type on one device:
            // from the per-type table, and without the memory, which a whole window leaves as it was: the deltas on a
            // device sum to zero, and the window itself was scored against the cap.)
            if (nin > 0) {
                // all R windows at once: every slot they write = max over the slots they read first of (value + longest path)
                int x[kMatIn];
#pragma unroll
                for (int j = 0; j < kMatIn; j++) x[j] = j < nin ? (int)TESSEL_ST(__builtin_amdgcn_readfirstlane((int)rtab[j])) : 0;
                for (int o = 0; o < nout; o++) {
                    const int4 *row = (const int4 *)(rtab + kMatIn + kMatOut + o * kMatIn);
                    int acc = 0;                         // (every output has a path from some input, and times are >= 0)
#pragma unroll
                    for (int q = 0; q < kMatIn / 4; q++) {
                        const int4 a = row[q];
                        acc = max(acc, max(x[4 * q] + a.x, x[4 * q + 1] + a.y));
                        acc = max(acc, max(x[4 * q + 2] + a.z, x[4 * q + 3] + a.w));
                    }
                    TESSEL_ST(__builtin_amdgcn_readfirstlane((int)rtab[kMatIn + o])) = (uint16_t)acc;
                }
            } else if (single_dev) {
                for (int k = 0; k < R; k++)
                    for (int s = 0; s < cp.nseq; s++) {
                        const uint32_t rw = (uint32_t)__builtin_amdgcn_readfirstlane((int)rtab[s]);
                        const int mu = (int)(rw >> 6 & 255u) + NR * k, d = (int)(rw & 7u);
                        const int tok = oTok + ((int)(rw >> 3 & 7u) << trs) + (mu & tmask);
                        int est = (int)TESSEL_ST(oFree + d);
                        if (rw >> 14 & 1u) est = max(est, (int)TESSEL_ST(tok));
                        const int en = est + (int)(rw >> 16);
                        TESSEL_ST(oFree + d) = (uint16_t)en;
                        TESSEL_ST(tok) = (uint16_t)en;
                    }
            } else
            for (int k = 0; k < R; k++)
                for (int s = 0; s < cp.nseq; s++) {
                    const int i = cp.seq[s], mu = (int)cp.lead[i] + (int)cp.occ[s] + NR * k;
                    const uint32_t mask = cp.mask[i];
                    const int tok = cp.path[i] != 0xFF ? oTok + (int)cp.path[i] * TR + (mu & tmask) : oTrash;
                    int est = 0;
                    if (cp.dag)
                        for (uint32_t rest = cp.predmask[i]; rest; rest &= rest - 1u)
                            est = max(est, (int)TESSEL_ST(oTok + (int)cp.path[__builtin_ctz(rest)] * TR + (mu & tmask)));
                    else if (cp.pred[i] >= 0) est = (int)TESSEL_ST(tok);
                    for (uint32_t rest = mask; rest; rest &= rest - 1u) est = max(est, (int)TESSEL_ST(oFree + __builtin_ctz(rest)));
                    const int en = est + cp.t[i];
                    for (uint32_t rest = mask; rest; rest &= rest - 1u) {
                        const int d = __builtin_ctz(rest);
                        TESSEL_ST(oFree + d) = (uint16_t)en; TESSEL_ST(oMem + d) = (uint16_t)((int)(int16_t)TESSEL_ST(oMem + d) + cp.m[i]);
                    }
                    TESSEL_ST(tok) = (uint16_t)en;
                }
            for (int i = 0; i < K; i++) TESSEL_ST(oNext + i) = (uint16_t)((int)cp.lead[i] + NR * R);
        }
        int makespan = 0;
        for (int d = 0; d < D; d++) makespan = max(makespan, (int)TESSEL_ST(oFree + d));
        if (fail) makespan = INT_MAX;
        if (!live) continue;
        if (makespan_out) makespan_out[kk] = makespan;
        if (makespan < best || (makespan == best && c < best_ord)) { best = makespan; best_ord = c; }
    }
#undef TESSEL_ST
    if (!recs) return;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int om = __shfl_xor(best, off);
        uint32_t ilo = __shfl_xor((uint32_t)best_ord, off), ihi = __shfl_xor((uint32_t)(best_ord >> 32), off);
        uint64_t oo = ((uint64_t)ihi << 32) | ilo;
        if (key_less(om, oo, best, best_ord)) { best = om; best_ord = oo; }
    }
    if (lane == 0) { CompRec rr; rr.makespan = best; rr.pad = 0; rr.ordinal = best_ord; recs[blockIdx.x] = rr; }
}

__global__ void complete_merge_kernel(const CompRec *__restrict__ recs, int nrecs, DevCompletion *__restrict__ res)
{
    const int lane = threadIdx.x;
    int best = INT_MAX;
    uint64_t best_ord = ~0ull;
    for (int k = lane; k < nrecs; k += kWave)
        if (key_less(recs[k].makespan, recs[k].ordinal, best, best_ord)) { best = recs[k].makespan; best_ord = recs[k].ordinal; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int om = __shfl_xor(best, off);
        uint32_t ilo = __shfl_xor((uint32_t)best_ord, off), ihi = __shfl_xor((uint32_t)(best_ord >> 32), off);
        uint64_t oo = ((uint64_t)ihi << 32) | ilo;
        if (key_less(om, oo, best, best_ord)) { best = om; best_ord = oo; }
    }
    if (lane == 0 && best != INT_MAX && key_less(best, best_ord, res->makespan, res->ordinal)) { res->makespan = best; res->ordinal = best_ord; }
}

__global__ void completion_reset_kernel(DevCompletion *res)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { res->makespan = INT_MAX; res->pad = 0; res->ordinal = ~0ull; }
}

size_t completion_lds_bytes(const CompParams &cp, const CompMatrix &cm)
{
    // 16-bit state, then one 32-bit sort key per type, then the windows' matrix or one word per block of the window
    const size_t replay = cm.nin > 0 ? (size_t)(kMatIn + kMatOut + cm.nout * kMatIn) * 4 : (size_t)cp.nseq * 4;
    return (size_t)kCompParamWords * 4 + (size_t)((cp.npaths * cp.tok_ring + 2 * cp.D + cp.K + 1 + 1) / 2 * 2) * kWave * 2 +
           (size_t)(cp.K + 1) * kWave * 4 +
           ((replay + 15) & ~(size_t)15);
}

int launch_completions(const CompParams &cp, const CompMatrix &cm, uint64_t first, uint64_t count, int32_t *makespan_out, void *ws,
                       int num_cus, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = completion_lds_bytes(cp, cm);
    if (lds > 64 * 1024) return -1;
    static bool attr_set = false;
    if (!attr_set && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)complete_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    int per_cu = (int)((160 * 1024) / ((lds + 511) / 512 * 512));
    if (per_cu > 16) per_cu = 16;
    if (per_cu < 1) per_cu = 1;
    uint64_t need = (count + kWave - 1) / kWave;
    const int blocks = need < (uint64_t)(num_cus * per_cu) ? (int)need : num_cus * per_cu;
    if (blocks < 1) return 0;
    CompRec *recs = makespan_out ? nullptr : (CompRec *)((char *)ws + kWsBlockRecOff);
    hipLaunchKernelGGL(complete_kernel, dim3(blocks), dim3(kWave), lds, st, (const CompParams *)((char *)ws + kWsCompParamsOff),
                       (const CompMatrix *)((char *)ws + kWsCompMatrixOff), first,
                       count, recs, makespan_out);
    int rc = (int)hipGetLastError();
    if (rc || !recs) return rc;
    hipLaunchKernelGGL(complete_merge_kernel, dim3(1), dim3(kWave), 0, st, (const CompRec *)recs, blocks,
                       (DevCompletion *)((char *)ws + kWsCompletionOff));
    return (int)hipGetLastError();
}

int launch_completion_reset(void *ws, void *stream)
{
    hipLaunchKernelGGL(completion_reset_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, (DevCompletion *)((char *)ws + kWsCompletionOff));
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------ achievable VALU rate
// Sixteen independent accumulators per lane, one add and one unsigned max each per round: 32
// full-rate integer VALU instructions per round with no dependency closer than 16 instructions.
// What this kernel sustains is the practical ceiling the scoring kernels are compared with.
constexpr int kProbeAcc = 16;

__global__ __launch_bounds__(256) void alu_probe_kernel(uint32_t *out, int rounds, uint32_t inc, uint32_t floor_)
{
    uint32_t a[kProbeAcc];
#pragma unroll
    for (int j = 0; j < kProbeAcc; j++) a[j] = threadIdx.x * 2654435761u + j;
    for (int r = 0; r < rounds; r++) {
#pragma unroll
        for (int j = 0; j < kProbeAcc; j++) a[j] = max(a[j] + inc, floor_);
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < kProbeAcc; j++) x ^= a[j];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = x;
}

int launch_alu_probe(uint32_t *out, int blocks, int rounds, void *stream)
{
    hipLaunchKernelGGL(alu_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, rounds, 0x9E3779B9u, 12345u);
    return (int)hipGetLastError();
}

#endif  // TESSEL_WIDE_INSTANTIATIONS

}  // namespace tessel
