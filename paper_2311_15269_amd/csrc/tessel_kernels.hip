// HIP kernels (gfx950) that score repetend candidates: one candidate per lane.
//
// Per candidate (Tessel, arXiv 2311.15269; Alg. 1, body of the loop over repetends):
//   decode   index -> lead vector (n_i of Eq. 3) + per-device block orders
//   build    walk the orders in an executable (topological) sequence, detect orders that
//            can never run, repair them in the REPAIR space, track the per-device memory
//            prefix (Eq. 1 [2]) and leave a compact "program" of the window in LDS
//   period   the repetend time t_R of Eq. 4 (with compaction of neighbouring repetends):
//            the least period of the rigidly repeated window.  The window is a max-plus
//            linear map on (device free times, end times of the micro-batches that are in
//            flight at the window boundary); its growth rate is the maximum cycle ratio,
//            obtained exactly from Karp's formula after V+1 sweeps of the window
//   argmin   (period, index) lexicographic, lane -> wave -> block record -> grid merge
//
// State that is indexed per lane at run time (device free times, micro-batch tokens, the
// program) lives in LDS laid out [slot][lane], which is bank-conflict free for any
// per-lane slot; everything else is in VGPRs.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>

#include "tessel_device.h"

namespace tessel {

struct BlockRec {
    int32_t  period;
    int32_t  pad;
    uint64_t index;
    uint32_t n_status[kNumStatus];
    uint32_t n_evaluated;
    uint32_t pad2;
};

// ------------------------------------------------------------------ counter-based sampler
// SplitMix64 finaliser keys the candidate; MurmurHash3's 32-bit finaliser, with the second
// key folded in between its multiplications, gives the w-th word; two 16-bit draws a word.
__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}
__device__ __forceinline__ uint32_t stream_word(uint32_t a, uint32_t b, uint32_t w)
{
    uint32_t x = a + w * 0x9E3779B9u;
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= b;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
constexpr uint32_t kDrawLeadBase = 0u;
constexpr uint32_t kDrawOrdBase = 128u;

// ------------------------------------------------------------------ 4-bit counters per type
// next micro-batch index of every block type: lead + occurrences placed, 4 bits each
struct Mu {
    uint64_t lo, hi;
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

__device__ __forceinline__ uint32_t byte_of(uint32_t packed, uint32_t y) { return (packed >> (8u * y)) & 0xFFu; }

__device__ __forceinline__ int sel4(const int32_t (&v)[kMaxLT], uint32_t y)
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

// ------------------------------------------------------------------ one window sweep
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
// Two passes over the same sweeps so that no history has to be stored.
template <int VM, bool TP>
__device__ __forceinline__ int least_period(const KParams &P, const uint16_t *prog, uint32_t *state, const int32_t *t_tab,
                            const uint32_t *mask_tab)
{
    const int V = P.nsweeps - 1, n = P.nsweeps;
    uint32_t xn[VM], bn[VM], bd[VM];
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
template <int DM>
__device__ __forceinline__ int decode_candidate(const KParams &P, uint64_t idx, uint64_t (&rem)[DM], int (&remlen)[DM], Mu &mu)
{
    const uint32_t NR = (uint32_t)P.NR;
    mu.lo = 0; mu.hi = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) { rem[d] = 0; remlen[d] = 0; }
    if (P.space == kFactorial) {
        uint64_t rest = idx;
        bool dup = false, tpm = false;
        uint32_t seen_types = 0;
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
                else { mu.set(g, fl); seen_types |= 1u << g; }
            }
        }
        if (dup) return kDup;
        if (tpm) return kTpMismatch;
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
            uint64_t o = 0;
            uint32_t word = 0;
            for (uint32_t pos = 0; pos < n; pos++) {
                uint32_t j = kDrawOrdBase + 32u * (uint32_t)d + pos;
                if ((pos & 1u) == 0) word = stream_word(a, b, j >> 1);
                uint32_t u = (word >> (16u * (pos & 1u))) & 0xFFFFu;
                uint32_t digit = (u * (n - pos)) >> 16;
                uint32_t y = (digit >= c0) + (digit >= c0 + c1) + (digit >= c0 + c1 + c2);
                c0 -= y == 0; c1 -= y == 1; c2 -= y == 2;
                o |= (uint64_t)y << (2u * pos);
            }
            rem[d] = o; remlen[d] = (int)n;
        }
    }

    return kOk;
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
        for (int d = 0; d < kMaxD; d++) detail->order_len[d] = 0;
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
    period = P.tp ? least_period<VM, true>(P, prog, state, t_tab, mask_tab)
                  : least_period<VM, false>(P, prog, state, t_tab, mask_tab);
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
// The per-device data that is picked by a run-time device number lives in LDS [device][lane];
// masks and the 4-bit micro-batch counters stay in VGPRs.

struct FastLds {
    uint32_t *t_tab;      // [32]  t by code
    uint32_t *info_tab;   // [32]  packed consumer/producer/token base/memory delta by code
    uint4 *recA;          // [DM][64] order (64 bit) | not-yet-placed mask (bit 2*pos)
    uint2 *recB;          // [DM][64] x: lead+N_R of the 4 types (4 bits each); y: memory now (lo16) | peak (hi16)
    uint32_t *prog;       // [ceil(total/3)][64] three 10-bit entries a word: code | slot<<5
    uint32_t *state;      // [nslots][64]
};

__device__ __forceinline__ uint32_t ctz64_parts(uint32_t lo, uint32_t hi)
{
    return lo ? (uint32_t)__builtin_ctz(lo) : 32u + (uint32_t)__builtin_ctz(hi | 0x80000000u);
}
__device__ __forceinline__ uint32_t bfi(uint32_t sel, uint32_t a, uint32_t b) { return (sel & a) | (~sel & b); }

// one sweep of the window over the 10-bit program
__device__ __forceinline__ void sweep_fast(const KParams &P, const FastLds &L, int lane)
{
    const int total = P.total;
    const int nwords = (total + 2) / 3;
    for (int i = 0; i < nwords; i++) {
        uint32_t w = L.prog[i * kWave + lane];
#pragma unroll
        for (int j = 0; j < 3; j++) {
            if (3 * i + j < total) {
                uint32_t e = (w >> (10 * j)) & 1023u;
                uint32_t code = e & 31u, ts = e >> 5, ds = code >> 2;
                uint32_t en = max(L.state[ds * kWave + lane], L.state[ts * kWave + lane]) + L.t_tab[code];
                L.state[ds * kWave + lane] = en;
                L.state[ts * kWave + lane] = en;
            }
        }
    }
    for (int p = 0; p < P.npaths; p++)
        for (int mu = 0; mu < P.NR; mu++) {
            int base = P.D + p * 2 * P.NR + mu;
            L.state[base * kWave + lane] = L.state[(base + P.NR) * kWave + lane];
            L.state[(base + P.NR) * kWave + lane] = 0;
        }
}

// Period of the repeated window.  The sweep is a max-plus linear map F on the boundary vector x
// (device free times, in-flight micro-batch end times).  If after some sweep every live component
// has grown by the same delta, x is an eigenvector of F and delta is its eigenvalue = the maximum
// cycle ratio, exactly.  Almost every candidate gets there within two or three sweeps; the rest
// take Karp's formula over V+1 sweeps (two passes, no history).
template <int VM>
__device__ __forceinline__ int period_fast(const KParams &P, const FastLds &L, int lane, const Mu &leads, bool want)
{
    const int V = P.nsweeps - 1, n = P.nsweeps;
    uint32_t live = 0;                                    // per lane: which boundary values mean anything
#pragma unroll
    for (int v = 0; v < VM; v++) {
        if (v < P.D) live |= (P.ntd[v] > 0 ? 1u : 0u) << v;
        else if (v < V) live |= (leads.get(P.v_src[v]) > (uint32_t)P.v_j[v] ? 1u : 0u) << v;
    }
    for (int s = 0; s < P.nslots; s++) L.state[s * kWave + lane] = 0;
    uint32_t prev[VM];
#pragma unroll
    for (int v = 0; v < VM; v++) prev[v] = 0;
    int T = 0;
    bool done = !want;
    constexpr int kTry = 6;
    for (int j = 0; j < kTry; j++) {
        if (__ballot(!done) == 0) break;
        sweep_fast(P, L, lane);
        bool same = true, have = false;
        uint32_t delta = 0;
#pragma unroll
        for (int v = 0; v < VM; v++) {
            if (v < V) {
                uint32_t x = L.state[reduced_slot(P, v) * kWave + lane];
                uint32_t dv = x - prev[v];
                prev[v] = x;
                if (live >> v & 1u) {
                    if (!have) { delta = dv; have = true; }
                    else if (dv != delta) same = false;
                }
            }
        }
        if (!done && same && have) { T = (int)delta; done = true; }
    }
    if (__ballot(!done) == 0) return T;
    // rare: no eigenvector yet.  Karp over n = V+1 sweeps, twice.
    uint32_t xn[VM], bn[VM], bd[VM];
    for (int s = 0; s < P.nslots; s++) L.state[s * kWave + lane] = 0;
    for (int j = 0; j < n; j++) sweep_fast(P, L, lane);
#pragma unroll
    for (int v = 0; v < VM; v++) {
        xn[v] = v < V ? L.state[reduced_slot(P, v) * kWave + lane] : 0u;
        bn[v] = 0xFFFFFFFFu; bd[v] = 1u;
    }
    for (int s = 0; s < P.nslots; s++) L.state[s * kWave + lane] = 0;
    for (int j = 0; j < n - 1; j++) {
        sweep_fast(P, L, lane);
        uint32_t den = (uint32_t)(n - 1 - j);
#pragma unroll
        for (int v = 0; v < VM; v++) {
            if (v < V) {
                uint32_t a = xn[v] - L.state[reduced_slot(P, v) * kWave + lane];
                bool better = bn[v] == 0xFFFFFFFFu || (uint64_t)a * bd[v] < (uint64_t)bn[v] * den;
                if (better) { bn[v] = a; bd[v] = den; }
            }
        }
    }
    uint32_t Tk = 0;
#pragma unroll
    for (int v = 0; v < VM; v++)
        if (v < V) Tk = max(Tk, (bn[v] + bd[v] - 1u) / bd[v]);
    return done ? T : (int)Tk;
}

template <int DM, int VM>
__device__ __forceinline__ int evaluate_fast(const KParams &P, uint64_t idx, const FastLds &L, int lane, int &period, int &peak_max,
                                             bool valid)
{
    uint64_t ord[DM];
    int nlen[DM];
    Mu leads;
    period = 0; peak_max = 0;
    int status = decode_candidate<DM>(P, idx, ord, nlen, leads);
    const uint32_t NR = (uint32_t)P.NR;

    // counters by code, ready / exhausted / head masks, per-device records
    Mu mu;
    mu.lo = 0; mu.hi = 0;
    uint32_t R = 0, HM = 0, X = 0;
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D) continue;
        uint32_t lim = 0;
        int mem0 = 0;
#pragma unroll
        for (int y = 0; y < kMaxLT; y++) {
            if (y >= P.ntd[d]) continue;
            uint32_t g = byte_of(P.type_of[d], (uint32_t)y), lead = leads.get(g);
            mu.set((uint32_t)(4 * d + y), lead);
            lim |= (lead + NR) << (4 * y);
            mem0 += P.m_of[d][y] * (int)lead;                 // blocks that ran before the window
        }
        uint64_t alive = nlen[d] >= 32 ? 0x5555555555555555ull : ((1ull << (2 * nlen[d])) - 1ull) & 0x5555555555555555ull;
        L.recA[d * kWave + lane] = make_uint4((uint32_t)ord[d], (uint32_t)(ord[d] >> 32), (uint32_t)alive, (uint32_t)(alive >> 32));
        L.recB[d * kWave + lane] = make_uint2(lim, ((uint32_t)mem0 & 0xFFFFu) | (0x8000u << 16));
        if (nlen[d] > 0) HM |= 1u << (4 * d + ((uint32_t)ord[d] & 3u));
    }
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D) continue;
#pragma unroll
        for (int y = 0; y < kMaxLT; y++) {
            if (y >= P.ntd[d]) continue;
            uint32_t c = (uint32_t)(4 * d + y), pr = (P.info_loc[c] >> 6) & 63u;
            bool ready = pr == 63u || mu.get(pr) > mu.get(c);
            R |= (ready ? 1u : 0u) << c;
        }
    }

    const bool repair = P.space == kSampledRepair;
    const int total = P.total;
    bool building = valid && status == kOk;
    uint32_t acc = 0;
    for (int k = 0; k < total; k++) {
        if (__ballot(building) == 0) break;
        uint32_t hm = R & HM;
        uint32_t sel = hm ? hm : (repair ? R : 0u);
        if (building && sel == 0) { status = kDeadlock; building = false; }
        const uint32_t b = (uint32_t)__builtin_ctz(sel | 0x80000000u) & 31u;
        const uint32_t d = building ? b >> 2 : 0u;
        const uint4 a = L.recA[d * kWave + lane];
        uint2 bb = L.recB[d * kWave + lane];
        const uint4 inf4 = *(const uint4 *)(L.info_tab + 4 * d);
        // earliest remaining entry of device d whose type is allowed (all types when its head runs)
        const uint32_t r4 = hm ? 15u : (R >> (4 * d)) & 15u;
        const uint32_t r0 = 0u - (r4 & 1u), r1 = 0u - ((r4 >> 1) & 1u), r2 = 0u - ((r4 >> 2) & 1u), r3 = 0u - (r4 >> 3);
        const uint32_t h_lo = (a.x >> 1) | (a.y << 31), h_hi = a.y >> 1;
        const uint32_t g_lo = bfi(h_lo, bfi(a.x, r3, r2), bfi(a.x, r1, r0));
        const uint32_t g_hi = bfi(h_hi, bfi(a.y, r3, r2), bfi(a.y, r1, r0));
        const uint32_t u_lo = a.z & g_lo, u_hi = a.w & g_hi;
        const uint32_t p = ctz64_parts(u_lo, u_hi) & 63u;
        const uint64_t ordw = ((uint64_t)a.y << 32) | a.x;
        const uint32_t y = (uint32_t)(ordw >> p) & 3u;
        const uint32_t c = 4u * d + y;
        const uint32_t info = y & 2u ? (y & 1u ? inf4.w : inf4.z) : (y & 1u ? inf4.y : inf4.x);
        // take the entry out, new head of the device
        uint64_t alive = (((uint64_t)a.w << 32) | a.z) & ~(1ull << p);
        const uint32_t al_lo = (uint32_t)alive, al_hi = (uint32_t)(alive >> 32);
        const uint32_t p2 = ctz64_parts(al_lo, al_hi) & 63u;
        const uint32_t y2 = (uint32_t)(ordw >> p2) & 3u;
        uint32_t hm_new = HM & ~(15u << (4 * d));
        if (alive) hm_new |= 1u << (4 * d + y2);
        // counters and readiness of this type and of its consumer
        const uint32_t mg = mu.get(c);
        const uint32_t lim = (bb.x >> (4 * y)) & 15u;
        const uint32_t pr = (info >> 6) & 63u, su = info & 63u;
        const bool exhausted = mg + 1u == lim;
        const bool ready_c = !exhausted && (pr == 63u || mu.get(pr) > mg + 1u);
        uint32_t r_new = (R & ~(1u << c)) | ((ready_c ? 1u : 0u) << c);
        const uint32_t x_new = X | ((exhausted ? 1u : 0u) << c);
        if (su != 63u) r_new |= (1u << su) & ~x_new;
        // memory prefix of the device (Eq. 1 [2])
        const int m = (int)(info << 6) >> 24;
        const int memcur = (int)(int16_t)(bb.y & 0xFFFFu) + m;
        const int pk = max((int)(int16_t)(bb.y >> 16), memcur);
        const uint32_t entry = c | ((((info >> 12) & 63u) + mg) << 5);
        const int sh = 10 * (k % 3);
        if (building) {
            R = r_new; X = x_new; HM = hm_new;
            mu.inc(c);
            L.recA[d * kWave + lane].z = al_lo;
            L.recA[d * kWave + lane].w = al_hi;
            L.recB[d * kWave + lane].y = ((uint32_t)memcur & 0xFFFFu) | ((uint32_t)pk << 16);
            acc |= entry << sh;
        }
        if (k % 3 == 2 || k == total - 1) {
            L.prog[(k / 3) * kWave + lane] = acc;
            acc = 0;
        }
    }
    if (status != kOk) return status;
    int worst = INT_MIN;
#pragma unroll
    for (int d = 0; d < DM; d++) {
        if (d >= P.D) continue;
        int pk = (int)(int16_t)(L.recB[d * kWave + lane].y >> 16);
        if (P.ntd[d] == 0) pk = 0;
        worst = max(worst, pk);
    }
    peak_max = worst;
    if (valid && worst > P.M) status = kMem;
    int T = period_fast<VM>(P, L, lane, leads, valid && status == kOk);
    if (status == kOk) period = T;
    return status;
}

template <int DM, int VM>
__global__ __launch_bounds__(kWave) void eval_fast_kernel(const KParams *__restrict__ Pp, uint64_t first, uint64_t count,
                                                          BlockRec *__restrict__ recs, int32_t *__restrict__ code_out,
                                                          int32_t *__restrict__ peak_out)
{
    extern __shared__ uint32_t lds[];
    const KParams &P = *Pp;
    const int lane = threadIdx.x;
    FastLds L;
    L.t_tab = lds;
    L.info_tab = lds + kMaxK;
    L.recA = (uint4 *)(lds + 2 * kMaxK);
    L.recB = (uint2 *)(lds + 2 * kMaxK + DM * kWave * 4);
    // the sweep state is only used once the build is over: it shares the build records' space when it fits
    const bool share = P.nslots <= DM * 6;
    L.state = share ? lds + 2 * kMaxK : lds + 2 * kMaxK + DM * kWave * 6;
    L.prog = share ? lds + 2 * kMaxK + DM * kWave * 6 : L.state + P.nslots * kWave;
    if (lane < kMaxK) { L.t_tab[lane] = (uint32_t)P.t_loc[lane]; L.info_tab[lane] = P.info_loc[lane]; }
    __syncthreads();

    int best = INT_MAX;
    uint64_t best_idx = 0;
    uint32_t cnt[kNumStatus];
#pragma unroll
    for (int s = 0; s < kNumStatus; s++) cnt[s] = 0;
    uint32_t nev = 0;
    const uint64_t stride = (uint64_t)gridDim.x * kWave;
    const uint64_t rounds = (count + stride - 1) / stride;          // the same trip count for every lane of the grid
    for (uint64_t r = 0; r < rounds; r++) {
        const uint64_t k = r * stride + (uint64_t)blockIdx.x * kWave + lane;
        const bool valid = k < count;
        int period, pk;
        int status = evaluate_fast<DM, VM>(P, first + (valid ? k : 0), L, lane, period, pk, valid);
        if (!valid) continue;
        nev++;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) cnt[s] += status == s;
        if (status == kOk && period < best) { best = period; best_idx = first + k; }
        if (code_out) code_out[k] = status == kOk ? period : -status;
        if (peak_out) peak_out[k] = (status == kOk || status == kMem) ? pk : 0;
    }
    if (!recs) return;
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
        BlockRec rr;
        rr.period = best; rr.pad = 0; rr.index = best_idx; rr.n_evaluated = nev; rr.pad2 = 0;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) rr.n_status[s] = cnt[s];
        recs[blockIdx.x] = rr;
    }
}

// ------------------------------------------------------------------ kernels
template <int DM, int VM>
__global__ __launch_bounds__(kWave) void eval_kernel(const KParams *__restrict__ Pp, uint64_t first, uint64_t count,
                                                     BlockRec *__restrict__ recs, int32_t *__restrict__ code_out,
                                                     int32_t *__restrict__ peak_out, DevDetail *__restrict__ detail)
{
    const KParams &P = *Pp;
    extern __shared__ uint32_t lds[];
    int32_t *t_tab = (int32_t *)lds;
    uint32_t *mask_tab = lds + kMaxK;
    uint32_t *state_all = lds + 2 * kMaxK;
    uint16_t *prog_all = (uint16_t *)(state_all + P.nslots * kWave);
    const int lane = threadIdx.x;
    if (lane < kMaxK) { t_tab[lane] = P.t_loc[lane]; mask_tab[lane] = P.mask_loc[lane]; }
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
    for (uint64_t k = (uint64_t)blockIdx.x * kWave + lane; k < count; k += stride) {
        int period, peak[DM];
        int status = evaluate<DM, VM>(P, first + k, prog, state, t_tab, mask_tab, period, peak, detail);
        nev++;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) cnt[s] += status == s;
        if (status == kOk && period < best) { best = period; best_idx = first + k; }   // ascending k: first wins
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
            for (int d = 0; d < kMaxD; d++) detail->peak[d] = 0;
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
        r.period = best; r.pad = 0; r.index = best_idx; r.n_evaluated = nev; r.pad2 = 0;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) r.n_status[s] = cnt[s];
        recs[blockIdx.x] = r;
    }
}

// merges the block records of one launch into the running best (one wave)
__global__ __launch_bounds__(kWave) void merge_kernel(const BlockRec *recs, int nrecs, DevResult *res)
{
    const int lane = threadIdx.x;
    int best = INT_MAX;
    uint64_t best_idx = 0, nev = 0, cnt[kNumStatus];
#pragma unroll
    for (int s = 0; s < kNumStatus; s++) cnt[s] = 0;
    for (int k = lane; k < nrecs; k += kWave) {
        BlockRec r = recs[k];
        if (key_less(r.period, r.index, best, best_idx)) { best = r.period; best_idx = r.index; }
        nev += r.n_evaluated;
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
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) {
            uint32_t l2 = __shfl_xor((uint32_t)cnt[s], off), h2 = __shfl_xor((uint32_t)(cnt[s] >> 32), off);
            cnt[s] += ((uint64_t)h2 << 32) | l2;
        }
    }
    if (lane == 0) {
        if (key_less(best, best_idx, res->period, res->index)) { res->period = best; res->index = best_idx; }
        res->n_evaluated += nev;
#pragma unroll
        for (int s = 0; s < kNumStatus; s++) res->n_status[s] += cnt[s];
    }
}

__global__ void reset_kernel(DevResult *res)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        res->period = INT_MAX; res->pad = 0; res->index = ~0ull; res->n_evaluated = 0;
        for (int s = 0; s < kNumStatus; s++) res->n_status[s] = 0;
    }
}

// ------------------------------------------------------------------ launchers
typedef void (*eval_fn)(const KParams *, uint64_t, uint64_t, BlockRec *, int32_t *, int32_t *, DevDetail *);
typedef void (*fast_fn)(const KParams *, uint64_t, uint64_t, BlockRec *, int32_t *, int32_t *);

static eval_fn pick_kernel(const KParams &kp)
{
    const int V = kp.nsweeps - 1;
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
    if (kp.D <= 2) return V <= 4 ? eval_fast_kernel<2, 4> : eval_fast_kernel<2, 24>;
    if (kp.D <= 4) return V <= 8 ? eval_fast_kernel<4, 8> : eval_fast_kernel<4, 24>;
    return V <= 16 ? eval_fast_kernel<8, 16> : eval_fast_kernel<8, 24>;
}

static size_t general_lds_bytes(const KParams &kp)
{
    return (size_t)2 * kMaxK * 4 + (size_t)kp.nslots * kWave * 4 + (size_t)kp.total * kWave * 2;
}

static size_t fast_lds_bytes(const KParams &kp)
{
    const bool share = kp.nslots <= fast_dm(kp) * 6;
    return (size_t)2 * kMaxK * 4 + (size_t)fast_dm(kp) * kWave * 24 + (share ? 0 : (size_t)kp.nslots * kWave * 4) +
           (size_t)((kp.total + 2) / 3) * kWave * 4;
}

LaunchShape eval_launch_shape(const KParams &kp, int num_cus)
{
    LaunchShape s;
    s.threads = kWave;
    s.lds_bytes = pick_fast(kp) ? fast_lds_bytes(kp) : general_lds_bytes(kp);
    int per_cu = (int)((160 * 1024) / (s.lds_bytes + 512));
    if (per_cu > 8) per_cu = 8;
    if (per_cu < 1) per_cu = 1;
    s.blocks = num_cus * per_cu;
    return s;
}

// general == true forces the general kernel (the only one that writes the decoded candidate)
static int launch_common(const KParams &kp, const KParams *kp_dev, uint64_t first, uint64_t count, int blocks, BlockRec *recs,
                         int32_t *code, int32_t *peak, DevDetail *detail, bool general, hipStream_t st)
{
    fast_fn ff = general ? nullptr : pick_fast(kp);
    const size_t lds = ff ? fast_lds_bytes(kp) : general_lds_bytes(kp);
    const void *fn = ff ? (const void *)ff : (const void *)pick_kernel(kp);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    if (ff) hipLaunchKernelGGL(ff, dim3(blocks), dim3(kWave), lds, st, kp_dev, first, count, recs, code, peak);
    else hipLaunchKernelGGL(pick_kernel(kp), dim3(blocks), dim3(kWave), lds, st, kp_dev, first, count, recs, code, peak, detail);
    return (int)hipGetLastError();
}

static int grid_for(const KParams &kp, uint64_t count, int num_cus)
{
    LaunchShape s = eval_launch_shape(kp, num_cus);
    uint64_t need = (count + kWave - 1) / kWave;
    return need < (uint64_t)s.blocks ? (int)need : s.blocks;
}

int launch_eval(const KParams &kp, uint64_t first, uint64_t count, void *ws, int num_cus, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    int blocks = grid_for(kp, count, num_cus);
    if (blocks < 1) return 0;
    BlockRec *recs = (BlockRec *)((char *)ws + kWsBlockRecOff);
    int rc = launch_common(kp, (const KParams *)((char *)ws + kWsParamsOff), first, count, blocks, recs, nullptr, nullptr,
                           nullptr, false, st);
    if (rc) return rc;
    hipLaunchKernelGGL(merge_kernel, dim3(1), dim3(kWave), 0, st, recs, blocks, (DevResult *)((char *)ws + kWsResultOff));
    return (int)hipGetLastError();
}

int launch_score(const KParams &kp, uint64_t first, uint64_t count, int32_t *code, int32_t *peak, void *ws, int num_cus,
                 bool general, void *stream)
{
    int blocks = grid_for(kp, count, num_cus);
    if (blocks < 1) return 0;
    return launch_common(kp, (const KParams *)((char *)ws + kWsParamsOff), first, count, blocks, nullptr, code, peak, nullptr,
                         general, (hipStream_t)stream);
}

int launch_detail(const KParams &kp, uint64_t index, void *ws, void *stream)
{
    return launch_common(kp, (const KParams *)((char *)ws + kWsParamsOff), index, 1, 1, nullptr, nullptr, nullptr,
                         (DevDetail *)((char *)ws + kWsDetailOff), true, (hipStream_t)stream);
}

int launch_reset(void *ws, void *stream)
{
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, (DevResult *)((char *)ws + kWsResultOff));
    return (int)hipGetLastError();
}

size_t block_rec_bytes(int blocks) { return (size_t)blocks * sizeof(BlockRec); }

}  // namespace tessel
