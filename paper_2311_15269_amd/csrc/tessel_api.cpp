// Host side of the C ABI declared in include/tessel.h: validation of the problem statement
// (Sec. III-A of the Tessel paper), static tables for the kernels, launches, result read-back,
// and schedule completion (Sec. IV-C) for the best repetend.  All candidate scoring is done
// by the kernels in tessel_kernels.hip; nothing here falls back to the CPU for it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstdlib>
#include <cstdint>
#include <cstring>
#include <atomic>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/tessel.h"
#include "tessel_device.h"

using namespace tessel;

namespace tessel { size_t block_rec_bytes(int blocks); }

struct tessel_problem {
    uint64_t id = 0;                    // never reused: names the handle as the owner of a workspace
    KParams kp;
    std::vector<int32_t> t, m;
    std::vector<uint32_t> mask;
    std::vector<int32_t> dep_src, dep_dst;
    std::vector<int8_t> leadtab;        // CANONICAL
    std::vector<uint64_t> wtab;         // CANONICAL
    uint64_t nlead = 0;
    uint64_t count = 0;
    int num_cus = 0;
    void *ws = nullptr;                 // workspace the running best lives in
    int max_blocks = 0;                 // 0, or the largest grid that workspace has queues for (the library's own buffer)
    bool ws_ready = false;
    hipStream_t stream = nullptr;
    int last_hip = 0;
    bool have_detail = false;
    bool force_general = false;         // TESSEL_FORCE_GENERAL=1: score with the general kernel only
    uint64_t detail_index = 0;
    DevDetail detail;
    DevResult result;
    // index ranges scored since the last reset (adjacent ones merged), and whether launches are cut into the
    // small pieces in which no list of unfinished candidates can overflow
    std::vector<std::pair<uint64_t, uint64_t>> ranges;
    bool safe_pieces = false;
    bool best_dirty = true;             // candidates were scored (or the search was reset) since the best was fetched
    // searched completion
    bool comp_ready = false;            // CompParams of (comp_index, N, J) are in the workspace
    uint64_t comp_index = 0;            // best candidate they were built for
    CompParams comp;
    CompMatrix comp_matrix;
};

static_assert(kScratchBytes == TESSEL_NOALLOC_SCRATCH_BYTES, "header and library disagree on the size of the library's own workspace");

static int hip_fail(tessel_problem *p, int e) { p->last_hip = e; return TESSEL_E_HIP; }

// Which handle a device workspace belongs to.  The kernels read the problem's parameter block, the running best and
// the queues from the workspace itself, so a buffer serves one handle at a time: binding it to another handle ends
// the first one's search, and that handle's next scoring call binds it anew (a new search), while its calls that
// read results are refused.  (Host memory only; the one piece of state shared between handles.)
namespace {
std::mutex g_owner_mutex;
std::unordered_map<const void *, uint64_t> g_owner;
std::atomic<uint64_t> g_next_id{1};

bool owns_workspace(const tessel_problem *p)
{
    if (!p->ws || !p->ws_ready) return false;
    std::lock_guard<std::mutex> lock(g_owner_mutex);
    auto it = g_owner.find(p->ws);
    return it != g_owner.end() && it->second == p->id;
}
void take_workspace(const tessel_problem *p, const void *ws)
{
    std::lock_guard<std::mutex> lock(g_owner_mutex);
    g_owner[ws] = p->id;
}
void release_workspaces(const tessel_problem *p)
{
    std::lock_guard<std::mutex> lock(g_owner_mutex);
    for (auto it = g_owner.begin(); it != g_owner.end();)
        if (it->second == p->id) it = g_owner.erase(it); else ++it;
}
}  // namespace

extern "C" const char *tessel_strerror(int code)
{
    switch (code) {
    case TESSEL_OK: return "ok";
    case TESSEL_E_INVALID_ARG: return "invalid argument";
    case TESSEL_E_BAD_DEP: return "dependency graph of a micro-batch has a cycle";
    case TESSEL_E_UNBALANCED_MEMORY: return "memory deltas on a device do not sum to zero";
    case TESSEL_E_TOOBIG: return "count or time bound too large";
    case TESSEL_E_WORKSPACE: return "workspace missing, misaligned or too small, or a launch overflowed its retry list (submit smaller ranges)";
    case TESSEL_E_HIP: return "HIP runtime error";
    case TESSEL_E_NO_FEASIBLE: return "no feasible candidate scored";
    case TESSEL_E_RANGE: return "range outside the candidate space or too few micro-batches";
    case TESSEL_E_UNSUPPORTED: return "problem outside the limits of this implementation";
    case TESSEL_E_NO_SCHEDULE: return "no warm-up/cool-down order fits the memory cap";
    default: return "unknown error";
    }
}

// number of distinct sequences of a multiset; 0 on 64-bit overflow
static uint64_t multiset_sequences(const int *cnt, int ntypes)
{
    unsigned __int128 r = 1;
    unsigned placed = 0;
    for (int y = 0; y < ntypes; y++)
        for (int k = 1; k <= cnt[y]; k++) {
            placed++;
            r = r * placed / (unsigned)k;
            if (r >> 64) return 0;
        }
    return (uint64_t)r;
}

// lead vectors of the CANONICAL space: Property 2 on every dependency, minimum 0,
// lexicographic with type 0 most significant
static bool gen_leads(const tessel_problem &p, int K, int NR, std::vector<int8_t> &tab, size_t limit)
{
    std::vector<int> cur(K, 0);
    int i = 0;
    cur[0] = -1;
    while (i >= 0) {
        cur[i]++;
        if (cur[i] >= NR) { i--; continue; }
        bool ok = true;
        for (size_t e = 0; e < p.dep_src.size() && ok; e++) {
            int a = p.dep_src[e], b = p.dep_dst[e];
            if (std::max(a, b) == i && cur[a] < cur[b]) ok = false;
        }
        if (!ok) continue;
        if (i == K - 1) {
            if (*std::min_element(cur.begin(), cur.end()) == 0) {
                if (tab.size() / K >= limit) return false;
                for (int k = 0; k < K; k++) tab.push_back((int8_t)cur[k]);
            }
        } else {
            i++;
            cur[i] = -1;
        }
    }
    return true;
}

extern "C" int tessel_problem_create(const tessel_problem_desc *desc, tessel_problem **out)
{
    if (!desc || !out) return TESSEL_E_INVALID_ARG;
    *out = nullptr;
    const int D = desc->num_devices, K = desc->num_block_types, NR = desc->nr;
    if (D < 1 || K < 1 || NR < 1 || desc->num_deps < 0 || !desc->time || !desc->mem || !desc->dev_mask ||
        (desc->num_deps > 0 && (!desc->dep_src || !desc->dep_dst)) || desc->space < 0 || desc->space > 3 ||
        desc->lead_step_q16 > 65536u)
        return TESSEL_E_INVALID_ARG;
    if (D > kMaxDW) return TESSEL_E_UNSUPPORTED;
    for (int i = 0; i < K; i++)
        if (desc->time[i] < 1 || desc->dev_mask[i] == 0 || (D < 32 && (desc->dev_mask[i] >> D))) return TESSEL_E_INVALID_ARG;
    for (int e = 0; e < desc->num_deps; e++)
        if (desc->dep_src[e] < 0 || desc->dep_src[e] >= K || desc->dep_dst[e] < 0 || desc->dep_dst[e] >= K ||
            desc->dep_src[e] == desc->dep_dst[e])
            return TESSEL_E_INVALID_ARG;
    if (desc->fixed_leads) {
        if (desc->space == TESSEL_SPACE_FACTORIAL) return TESSEL_E_INVALID_ARG;
        for (int i = 0; i < K; i++) if (desc->fixed_leads[i] < 0 || desc->fixed_leads[i] >= NR) return TESSEL_E_INVALID_ARG;
        for (int e = 0; e < desc->num_deps; e++)
            if (desc->fixed_leads[desc->dep_src[e]] < desc->fixed_leads[desc->dep_dst[e]]) return TESSEL_E_INVALID_ARG;
    }
    // acyclic?
    {
        std::vector<int> indeg(K, 0), done(K, 0);
        for (int e = 0; e < desc->num_deps; e++) indeg[desc->dep_dst[e]]++;
        int n = 0;
        for (bool again = true; again;) {
            again = false;
            for (int i = 0; i < K; i++) if (!done[i] && indeg[i] == 0) {
                done[i] = 1; n++; again = true;
                for (int e = 0; e < desc->num_deps; e++) if (desc->dep_src[e] == i) indeg[desc->dep_dst[e]]--;
            }
        }
        if (n != K) return TESSEL_E_BAD_DEP;
    }
    for (int d = 0; d < D; d++) {
        int net = 0;
        for (int i = 0; i < K; i++) if (desc->dev_mask[i] >> d & 1u) net += desc->mem[i];
        if (net != 0) return TESSEL_E_UNBALANCED_MEMORY;
    }
    // limits of the kernels
    if (K > kMaxKW || NR > kMaxNRW) return TESSEL_E_UNSUPPORTED;
    std::vector<int> indeg(K, 0), outdeg(K, 0);
    for (int e = 0; e < desc->num_deps; e++) { outdeg[desc->dep_src[e]]++; indeg[desc->dep_dst[e]]++; }
    // disjoint chains take the fast kernel and the chain path of the general one; any other graph (Sec. III-A allows
    // any acyclic one) the general kernel's path for graphs, which TESSEL_FORCE_DAG=1 also forces on chains (tests)
    bool chains = true;
    for (int i = 0; i < K; i++) if (indeg[i] > 1 || outdeg[i] > 1) chains = false;
    { const char *fd = getenv("TESSEL_FORCE_DAG"); if (fd && fd[0] == '1') chains = false; }
    // more than kMaxD devices or kMaxK block types: the tables by (device, symbol) code of the chain path and of the fast
    // kernel have no room for them; such a problem is scored as a graph, chains or not
    // ... and so is one with more than kMaxLT block types on a device (3-bit symbols; sampled spaces only, at most 32
    // blocks per device and window)
    bool many = false;
    for (int d = 0; d < D; d++) {
        int n = 0;
        for (int i = 0; i < K; i++) n += desc->dev_mask[i] >> d & 1u;
        if (n > kMaxLTW || n * NR > kMaxPos) return TESSEL_E_UNSUPPORTED;
        if (n > kMaxLT) many = true;
    }
    // ... and one with a window of more than kMaxNR micro-batches (8-bit instead of 4-bit counters; sampled spaces only)
    const bool longwin = NR > kMaxNR;
    if ((many || longwin) && desc->space != TESSEL_SPACE_SAMPLED_STRICT && desc->space != TESSEL_SPACE_SAMPLED_REPAIR) return TESSEL_E_UNSUPPORTED;
    const bool wide = D > kMaxD || K > kMaxK || many || longwin;
    if (wide) chains = false;
    if (!chains && desc->num_deps > kMaxDeps) return TESSEL_E_UNSUPPORTED;

    tessel_problem *p = new (std::nothrow) tessel_problem();
    if (!p) return TESSEL_E_INVALID_ARG;
    p->id = g_next_id.fetch_add(1);
    p->t.assign(desc->time, desc->time + K);
    p->m.assign(desc->mem, desc->mem + K);
    p->mask.assign(desc->dev_mask, desc->dev_mask + K);
    p->dep_src.assign(desc->dep_src, desc->dep_src + desc->num_deps);
    p->dep_dst.assign(desc->dep_dst, desc->dep_dst + desc->num_deps);
    KParams &kp = p->kp;
    memset(&kp, 0, sizeof kp);
    kp.D = D; kp.K = K; kp.NR = NR; kp.M = desc->mem_cap; kp.total = K * NR; kp.space = desc->space;
    kp.seed = desc->seed; kp.step_q16 = desc->lead_step_q16;
    kp.has_fixed = desc->fixed_leads != nullptr;
    for (int i = 0; i < K; i++) kp.fixed[i] = desc->fixed_leads ? (uint8_t)desc->fixed_leads[i] : 0;
    for (int i = 0; i < K && i < kMaxK; i++) { kp.pred[i] = -1; kp.succ[i] = -1; }
    for (int e = 0; e < desc->num_deps && chains; e++) {
        int a = desc->dep_src[e], b = desc->dep_dst[e];
        kp.succ[a] = (int8_t)b; kp.pred[b] = (int8_t)a;
        kp.edge_out[a] = (uint8_t)e;
        kp.cross_out[a] = desc->dev_mask[a] != desc->dev_mask[b];
    }
    if (!chains) {
        kp.dag = 1; kp.ndeps = desc->num_deps;
        kp.dag_tries = 8;
        if (const char *env = getenv("TESSEL_DAG_TRIES")) {        // test knob: 0 leaves every period to the bisection
            int v = atoi(env);
            if (v >= 0 && v <= 64) kp.dag_tries = v;
        }
        for (int i = 0; i < K; i++) { kp.t_type[i] = desc->time[i]; kp.mask_type[i] = desc->dev_mask[i]; kp.tokbase[i] = (uint16_t)kNoRing; }
        for (int e = 0; e < desc->num_deps; e++) {
            const int a = desc->dep_src[e], b = desc->dep_dst[e];
            kp.dsrc[e] = (uint8_t)a; kp.ddst[e] = (uint8_t)b; kp.dcross[e] = desc->dev_mask[a] != desc->dev_mask[b];
            kp.predmask[b] |= 1ull << a;
        }
        // End times by micro-batch, 2 N_R slots per ring behind the devices (and for a shared ring N_R more: what the last
        // window boundary left in the ring's lower half, for the comparison at the next one).  A stretch of the graph without branches
        // (a -> b with a's only consumer b and b's only producer a) shares one ring: b reads a's end time of a
        // micro-batch and puts its own in its place, which only b's consumers read.  A chain is one ring.
        {
            std::vector<int> head(K), next_in(K, -1);
            for (int i = 0; i < K; i++) head[i] = i;
            for (int e = 0; e < desc->num_deps; e++) {
                const int a = desc->dep_src[e], b = desc->dep_dst[e];
                bool twice = false;                          // (a dependency listed twice counts once)
                for (int f = 0; f < e; f++) if (desc->dep_src[f] == a && desc->dep_dst[f] == b) twice = true;
                int outs = 0, ins = 0;
                for (int f = 0; f < desc->num_deps; f++) {
                    bool seen = false;
                    for (int h = 0; h < f; h++) if (desc->dep_src[h] == desc->dep_src[f] && desc->dep_dst[h] == desc->dep_dst[f]) seen = true;
                    if (seen) continue;
                    outs += desc->dep_src[f] == a; ins += desc->dep_dst[f] == b;
                }
                if (!twice && outs == 1 && ins == 1) next_in[a] = b;
            }
            std::vector<char> inner(K, 0);
            int slots = 0;
            for (int i = 0; i < K; i++) if (next_in[i] >= 0) inner[next_in[i]] = 1;
            for (int i = 0; i < K; i++) {
                if (inner[i]) continue;                       // i starts a stretch
                bool consumed = false;
                for (int g = i; g >= 0; g = next_in[g]) consumed = consumed || outdeg[g] > 0;
                if (!consumed) continue;
                const int base = D + slots;
                const bool shared = next_in[i] >= 0;
                kp.ring_head[kp.ntok] = (uint8_t)i;
                kp.ring_base[kp.ntok] = (uint16_t)base;
                kp.ring_kept[kp.ntok] = (uint16_t)(shared ? base + 2 * NR : base);
                for (int g = i; g >= 0; g = next_in[g]) if (outdeg[g] > 0) kp.tokbase[g] = (uint16_t)base;
                kp.ntok++;
                slots += (shared ? 3 : 2) * NR;
            }
            kp.nslots = D + slots;
        }
        // consumers before producers
        std::vector<int> left(outdeg), done(K, 0);
        int n = 0;
        for (bool again = true; again;) {
            again = false;
            for (int i = 0; i < K; i++) if (!done[i] && left[i] == 0) {
                done[i] = 1; kp.rtopo[n++] = (uint8_t)i; again = true;
                for (int e = 0; e < desc->num_deps; e++) if (desc->dep_dst[e] == i) left[desc->dep_src[e]]--;
            }
        }
    }
    // chains and their token slots; reverse topological order = walk every chain from its end
    std::vector<int> path_of(K, 0);
    int npaths = 0, nrt = 0;
    if (chains) {
        for (int i = 0; i < K; i++) if (kp.pred[i] < 0) {
            for (int g = i; g >= 0; g = kp.succ[g]) path_of[g] = npaths;
            npaths++;
        }
        for (int i = 0; i < K; i++) if (kp.succ[i] < 0)
            for (int g = i; g >= 0; g = kp.pred[g]) kp.rtopo[nrt++] = (uint8_t)g;
        kp.npaths = npaths;
        kp.nslots = D + npaths * 2 * NR;
        kp.nsweeps = D + npaths * NR + 1;
        if (kp.nslots > 63 || kp.nsweeps - 1 > 24) { delete p; return TESSEL_E_UNSUPPORTED; }
    } else {
        kp.npaths = 0;
        kp.nsweeps = D + 1;                       // (only sizes the register arrays of the chain path, unused here)
        // state and program of a workgroup must fit the LDS a kernel may ask for
        // (problems too wide for the other paths keep both in global memory when they have to)
        if (!wide && (size_t)4 * kMaxK * 4 + (size_t)kp.nslots * kWave * 4 + (size_t)K * NR * kWave * 2 > 64 * 1024) { delete p; return TESSEL_E_UNSUPPORTED; }
    }
    int sumt = 0;
    for (int i = 0; i < K; i++) {
        if (desc->time[i] > (1 << 20)) { delete p; return TESSEL_E_TOOBIG; }
        sumt += desc->time[i];
    }
    kp.UB = NR * sumt;
    // the period kernel multiplies (sweeps * UB) by a sweep count
    if ((int64_t)kp.UB * kp.nsweeps * kp.nsweeps >= (int64_t)1 << 31) { delete p; return TESSEL_E_TOOBIG; }
    kp.LB = 0;
    for (int d = 0; d < kMaxDW; d++) kp.type_of[d] = kp.type_of_hi[d] = 0xFFFFFFFFu;
    kp.many = many;
    for (int d = 0; d < kMaxD; d++) { kp.pred_of[d] = 0xFFFFFFFFu; kp.mask_of[d] = kp.tok_of[d] = kp.home_of[d] = 0; }
    std::vector<int> home(K, -1);
    for (int d = 0; d < D; d++) {
        int n = 0, busy = 0;
        for (int i = 0; i < K; i++) if (desc->dev_mask[i] >> d & 1u) {
            if (n >= kMaxLTW) { delete p; return TESSEL_E_UNSUPPORTED; }
            if (home[i] < 0) home[i] = d * 4 + n;
            if (n < 4) kp.type_of[d] = (kp.type_of[d] & ~(0xFFu << (8 * n))) | ((uint32_t)i << (8 * n));
            else kp.type_of_hi[d] = (kp.type_of_hi[d] & ~(0xFFu << (8 * (n - 4)))) | ((uint32_t)i << (8 * (n - 4)));
            if (!wide) {
                uint32_t pr = kp.pred[i] < 0 ? 0xFFu : (uint32_t)kp.pred[i];
                kp.pred_of[d] = (kp.pred_of[d] & ~(0xFFu << (8 * n))) | (pr << (8 * n));
                kp.mask_of[d] |= (desc->dev_mask[i] & 0xFFu) << (8 * n);
                kp.tok_of[d] |= (uint32_t)(D + path_of[i] * 2 * NR) << (8 * n);
                kp.home_of[d] |= (uint32_t)home[i] << (8 * n);
                kp.t_of[d][n] = desc->time[i];
            }
            kp.predmask_of[d][n] = kp.predmask[i];
            kp.m_of[d][n] = desc->mem[i];
            busy += desc->time[i];
            n++;
        }
        kp.ntd[d] = n;
        kp.LB = std::max(kp.LB, NR * busy);
    }
    for (int i = 0; i < K; i++) {
        if (!wide) { kp.t_loc[home[i]] = desc->time[i]; kp.mask_loc[home[i]] = desc->dev_mask[i]; }
        if (desc->dev_mask[i] & (desc->dev_mask[i] - 1)) kp.tp = 1;
    }
    // tables of the fast kernel: single-device blocks, small memory deltas, few slots
    if (!wide) {
        bool ok = chains && kp.nslots <= 32 && kp.nsweeps - 1 <= 24;
        // every (device, local symbol) is a code; a type on several devices has one code per device
        std::vector<std::vector<int>> code_on(K, std::vector<int>(D, -1));
        for (int d = 0; d < D; d++)
            for (int y = 0; y < kp.ntd[d]; y++) code_on[(kp.type_of[d] >> (8 * y)) & 0xFFu][d] = d * 4 + y;
        for (int c = 0; c < kMaxK; c++) kp.home_code[c] = 63;
        for (int i = 0; i < K; i++) {
            uint32_t grp = 0;
            for (int d = 0; d < D; d++) if (code_on[i][d] >= 0) grp |= 1u << code_on[i][d];
            for (int d = 0; d < D; d++) if (code_on[i][d] >= 0) { kp.grp_code[code_on[i][d]] = grp; kp.home_code[code_on[i][d]] = (uint8_t)home[i]; }
            const bool multi = (desc->dev_mask[i] & (desc->dev_mask[i] - 1)) != 0;
            const bool multi_next = kp.succ[i] >= 0 && (desc->dev_mask[kp.succ[i]] & (desc->dev_mask[kp.succ[i]] - 1)) != 0;
            if (multi) { if (kp.ntp < kMaxD) kp.tp_group[kp.ntp++] = grp; else ok = false; }
            if (multi || multi_next) kp.slow_mask |= grp;
        }
        kp.fast_tp = kp.tp;
        // the memory prefix of a device is kept in 8 bits: entry (lead <= N_R-1 each) plus N_R occurrences
        for (int d = 0; d < D; d++) {
            long span = 0;
            for (int i = 0; i < K; i++) if (desc->dev_mask[i] >> d & 1u) span += (long)std::abs(desc->mem[i]) * (2 * NR - 1);
            if (span > 120) ok = false;
        }
        for (int i = 0; i < K; i++) if (desc->mem[i] < -127 || desc->mem[i] > 127) ok = false;
        for (int i = 0; i < K; i++) if (desc->time[i] > 65535) ok = false;      // the sweep table keeps t in 16 bits
        for (int i = 0; i < kMaxK; i++) kp.info_loc[i] = 63u | (63u << 6);
        for (int i = 0; i < K && ok; i++) {
            uint32_t su = kp.succ[i] < 0 ? 63u : (uint32_t)home[kp.succ[i]];
            uint32_t pr = kp.pred[i] < 0 ? 63u : (uint32_t)home[kp.pred[i]];
            uint32_t tokbase = (uint32_t)(D + path_of[i] * 2 * NR);
            for (int d = 0; d < D; d++) if (code_on[i][d] >= 0)
                kp.info_loc[code_on[i][d]] = su | (pr << 6) | (tokbase << 12) | (((uint32_t)desc->mem[i] & 0xFFu) << 18);
        }
        for (int k = 0; k < K && ok; k++) {
            int i = kp.rtopo[k];
            uint32_t su = kp.succ[i] < 0 ? 63u : (uint32_t)home[kp.succ[i]];
            kp.chain_tab[k] = (uint32_t)home[i] | (su << 6) | ((uint32_t)(kp.succ[i] < 0 ? 0 : kp.edge_out[i]) << 12) |
                              ((uint32_t)(kp.succ[i] >= 0 && kp.cross_out[i]) << 19) | ((uint32_t)(kp.pred[i] < 0) << 20) |
                              ((uint32_t)i << 21);
        }
        {
            // chain_tab lists every chain from its last block to its first, one chain after the other
            std::vector<int> pos(K, 0);
            for (int k = 0; k < K; k++) pos[kp.rtopo[k]] = k;
            for (int i = 0; i < K && ok; i++) {
                uint32_t cum = 0;
                for (int g = i; kp.succ[g] >= 0; g = kp.succ[g]) cum |= 1u << pos[g];
                for (int d = 0; d < D; d++) if (code_on[i][d] >= 0) {
                    kp.cum_code[code_on[i][d]] = cum;
                    kp.pred_bit[code_on[i][d]] = kp.pred[i] < 0 ? 0u : 1u << pos[kp.pred[i]];
                }
                if (kp.succ[i] >= 0 && kp.edge_out[i] < kMaxK) kp.dep_bit[kp.edge_out[i]] = kp.cross_out[i] ? 1u << pos[i] : 0u;
            }
            if (desc->num_deps > kMaxK) ok = false;
        }
        for (int d = 0; d < D; d++) {
            kp.vtab[d] = (uint32_t)d | (1u << 6) | ((uint32_t)(kp.ntd[d] > 0) << 17);
            for (int y = 0; y < kp.ntd[d]; y++) kp.mpack[d] |= ((uint32_t)kp.m_of[d][y] & 0xFFu) << (8 * y);
        }
        int v = D, path = 0;
        for (int i = 0; i < K && ok; i++) if (kp.pred[i] < 0) {
            for (int j = 0; j < NR; j++, v++)
                if (v < 24) kp.vtab[v] = (uint32_t)(D + path * 2 * NR + j) | ((uint32_t)home[i] << 7) | ((uint32_t)j << 13);
            path++;
        }
        kp.fast_ok = ok;
        kp.eigen_tries = kFirstPassTries;
        kp.retry_tries = kRetryTries;
        if (const char *env = getenv("TESSEL_EIGEN_TRIES")) {      // test knobs: force candidates onto the longer search
            int v = atoi(env);
            if (v >= 0 && v <= 64) kp.eigen_tries = v;
        }
        if (const char *env = getenv("TESSEL_RETRY_TRIES")) {      // ... and from there to the general kernel
            int v = atoi(env);
            if (v >= 0 && v <= 64) kp.retry_tries = v;
        }
    }
    // candidate count and the tables of the exhaustive spaces
    if (desc->space == TESSEL_SPACE_FACTORIAL) {
        kp.fact[0] = 1;
        for (int n = 1; n <= 12; n++) kp.fact[n] = kp.fact[n - 1] * (uint32_t)n;
        unsigned __int128 c = 1;
        for (int d = 0; d < D; d++) {
            int n = kp.ntd[d] * NR;
            if (n > 12) { delete p; return n > 20 ? TESSEL_E_TOOBIG : TESSEL_E_UNSUPPORTED; }
            kp.cdev[d] = kp.fact[n];
            uint64_t list = 0;
            int k = 0;
            for (int y = 0; y < kp.ntd[d]; y++)
                for (int l = 0; l < NR; l++, k++) list |= (uint64_t)((y << 3) | l) << (5 * k);
            kp.init_list[d] = list;
            c *= kp.cdev[d];
            if (c >> 64) { delete p; return TESSEL_E_TOOBIG; }
        }
        p->count = (uint64_t)c;
    } else if (desc->space == TESSEL_SPACE_CANONICAL) {
        if (kp.has_fixed) {
            for (int i = 0; i < K; i++) p->leadtab.push_back((int8_t)desc->fixed_leads[i]);
        } else if (!gen_leads(*p, K, NR, p->leadtab, (kWsTablesMax / 2) / K)) {
            delete p; return TESSEL_E_TOOBIG;
        }
        p->nlead = p->leadtab.size() / K;
        unsigned __int128 c = p->nlead;
        for (int d = 0; d < D; d++) {
            int cnt[kMaxLT];
            for (int y = 0; y < kMaxLT; y++) cnt[y] = y < kp.ntd[d] ? NR : 0;
            kp.cdev[d] = multiset_sequences(cnt, kMaxLT);
            if (!kp.cdev[d]) { delete p; return TESSEL_E_TOOBIG; }
            c *= kp.cdev[d];
            if (c >> 64) { delete p; return TESSEL_E_TOOBIG; }
        }
        p->count = (uint64_t)c;
        const int B = NR + 1;
        p->wtab.resize((size_t)B * B * B * B);
        for (int c0 = 0; c0 < B; c0++) for (int c1 = 0; c1 < B; c1++) for (int c2 = 0; c2 < B; c2++) for (int c3 = 0; c3 < B; c3++) {
            int cnt[4] = {c0, c1, c2, c3};
            p->wtab[(((size_t)c0 * B + c1) * B + c2) * B + c3] = multiset_sequences(cnt, 4);   // 0 only where never needed
        }
    } else {
        if (desc->num_deps > 128) { delete p; return TESSEL_E_UNSUPPORTED; }
        p->count = UINT64_MAX;
    }
    p->result.period = INT_MAX;
    { const char *fg = getenv("TESSEL_FORCE_GENERAL"); p->force_general = fg && fg[0] == '1'; }
    if (p->force_general) kp.fast_ok = 0;
    *out = p;
    return TESSEL_OK;
}

extern "C" void tessel_problem_destroy(tessel_problem *p)
{
    if (!p) return;
    release_workspaces(p);
    delete p;
}

extern "C" int tessel_candidate_count(const tessel_problem *p, uint64_t *count)
{
    if (!p || !count) return TESSEL_E_INVALID_ARG;
    *count = p->count;
    return TESSEL_OK;
}

static int ensure_device(tessel_problem *p)
{
    if (p->num_cus) return TESSEL_OK;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    p->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    return TESSEL_OK;
}

static size_t workspace_need(const tessel_problem *p, int num_cus)
{
    return eval_workspace_bytes(p->kp, num_cus, 0);
}

extern "C" int tessel_workspace_bytes(const tessel_problem *p, size_t *bytes)
{
    if (!p || !bytes) return TESSEL_E_INVALID_ARG;
    // sized for the grid the launcher uses on the current device (16 workgroups per compute unit at most); for 512
    // compute units where no device can be asked
    int cus = p->num_cus;
    if (!cus) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        else
            (void)hipGetLastError();
    }
    *bytes = workspace_need(p, cus ? cus : 512);
    return TESSEL_OK;
}

static int range_ok(const tessel_problem *p, uint64_t first, uint64_t count)
{
    if (p->count == UINT64_MAX) return first + count >= first ? TESSEL_OK : TESSEL_E_RANGE;
    if (first > p->count || count > p->count - first) return TESSEL_E_RANGE;
    return TESSEL_OK;
}

// binds the workspace: uploads the tables of the exhaustive spaces and clears the running best
static int bind_workspace(tessel_problem *p, void *ws, size_t bytes, hipStream_t st, int max_blocks = 0)
{
    if (!ws || ((uintptr_t)ws & 255u)) return TESSEL_E_WORKSPACE;
    int rc = ensure_device(p);
    if (rc) return rc;
    if (bytes < eval_workspace_bytes(p->kp, p->num_cus, max_blocks)) return TESSEL_E_WORKSPACE;
    if (p->ws == ws && owns_workspace(p)) return TESSEL_OK;
    char *base = (char *)ws + kWsTablesOff;
    size_t lead_bytes = (p->leadtab.size() + 255) & ~(size_t)255, w_bytes = p->wtab.size() * sizeof(uint64_t);
    if (lead_bytes + w_bytes > kWsTablesMax) return TESSEL_E_TOOBIG;
    if (!p->leadtab.empty()) {
        hipError_t e = hipMemcpyAsync(base, p->leadtab.data(), p->leadtab.size(), hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return hip_fail(p, (int)e);
        e = hipMemcpyAsync(base + lead_bytes, p->wtab.data(), w_bytes, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return hip_fail(p, (int)e);
        p->kp.leadtab = (const int8_t *)base;
        p->kp.wtab = (const uint64_t *)(base + lead_bytes);
    }
    hipError_t pe = hipMemcpyAsync((char *)ws + kWsParamsOff, &p->kp, sizeof(KParams), hipMemcpyHostToDevice, st);
    if (pe != hipSuccess) return hip_fail(p, (int)pe);
    int e = launch_reset(ws, st);
    if (e) return hip_fail(p, e);
    p->ws = ws; p->ws_ready = true; p->have_detail = false; p->max_blocks = max_blocks;
    p->comp_ready = false;              // the completion parameters lived in the workspace bound before
    p->ranges.clear();
    p->best_dirty = true;
    p->result.period = INT_MAX;
    take_workspace(p, ws);
    return TESSEL_OK;
}

extern "C" int tessel_eval_candidates(tessel_problem *p, uint64_t first, uint64_t count, void *workspace_dev,
                                      size_t workspace_bytes, void *hip_stream)
{
    if (!p) return TESSEL_E_INVALID_ARG;
    int rc = range_ok(p, first, count);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    rc = bind_workspace(p, workspace_dev, workspace_bytes, st);
    if (rc) return rc;
    p->stream = st;
    p->have_detail = false;
    if (count == 0) return TESSEL_OK;
    p->best_dirty = true;
    if (!p->ranges.empty() && p->ranges.back().first + p->ranges.back().second == first) p->ranges.back().second += count;
    else p->ranges.push_back({first, count});
    int e = launch_eval(p->kp, first, count, workspace_dev, p->num_cus, p->max_blocks, st, p->safe_pieces ? kSafePerLaunch : kMaxPerLaunch);
    return e ? hip_fail(p, e) : TESSEL_OK;
}

// tessel_eval_candidates in the library's own device buffer: no allocation anywhere on the way
extern "C" int tessel_eval_candidates_noalloc(tessel_problem *p, uint64_t first, uint64_t count, void *hip_stream)
{
    if (!p) return TESSEL_E_INVALID_ARG;
    int rc = range_ok(p, first, count);
    if (rc) return rc;
    if (count > TESSEL_NOALLOC_MAX_CANDIDATES) return TESSEL_E_TOOBIG;
    rc = ensure_device(p);
    if (rc) return rc;
    void *ws = nullptr;
    size_t bytes = 0;
    int e = scratch_workspace(&ws, &bytes);
    if (e) return hip_fail(p, e);
    const int blocks = eval_blocks_that_fit(p->kp, p->num_cus, bytes);
    if (blocks < 1) return TESSEL_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    // (a buffer bound with another grid limit, i.e. by the other entry point, cannot be this one: no rebinding check needed)
    rc = bind_workspace(p, ws, bytes, st, blocks);
    if (rc) return rc;
    p->stream = st;
    p->have_detail = false;
    if (count == 0) return TESSEL_OK;
    p->best_dirty = true;
    if (!p->ranges.empty() && p->ranges.back().first + p->ranges.back().second == first) p->ranges.back().second += count;
    else p->ranges.push_back({first, count});
    e = launch_eval(p->kp, first, count, ws, p->num_cus, p->max_blocks, st, p->safe_pieces ? kSafePerLaunch : kMaxPerLaunch);
    return e ? hip_fail(p, e) : TESSEL_OK;
}

extern "C" int tessel_score_candidates(tessel_problem *p, uint64_t first, uint64_t count, int32_t *code_dev,
                                       int32_t *peak_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    if (!p || !code_dev) return TESSEL_E_INVALID_ARG;
    int rc = range_ok(p, first, count);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    // the workspace carries the tables of the exhaustive spaces; binding a new one clears the running best
    rc = bind_workspace(p, workspace_dev, workspace_bytes, st);
    if (rc) return rc;
    p->stream = st;
    if (count == 0) return TESSEL_OK;
    int e = launch_score(p->kp, first, count, code_dev, peak_dev, workspace_dev, p->num_cus, p->max_blocks, p->force_general, st);
    return e ? hip_fail(p, e) : TESSEL_OK;
}

extern "C" int tessel_alu_probe(int blocks, int rounds, uint32_t *out_dev, size_t out_bytes, void *hip_stream,
                                uint64_t *lane_ops)
{
    if (blocks < 1 || blocks > (1 << 20) || rounds < 1 || rounds > (1 << 24) || !out_dev) return TESSEL_E_INVALID_ARG;
    if (out_bytes < (size_t)blocks * kProbeThreads * sizeof(uint32_t)) return TESSEL_E_WORKSPACE;
    if (lane_ops) *lane_ops = (uint64_t)blocks * kProbeThreads * (uint64_t)rounds * kProbeLaneOpsPerRound;
    return launch_alu_probe(out_dev, blocks, rounds, hip_stream) ? TESSEL_E_HIP : TESSEL_OK;
}

extern "C" int tessel_reset(tessel_problem *p)
{
    if (!p) return TESSEL_E_INVALID_ARG;
    p->have_detail = false;
    p->result.period = INT_MAX;
    p->ranges.clear();
    p->best_dirty = true;
    if (!owns_workspace(p)) { p->ws_ready = false; return TESSEL_OK; }     // (another handle's by now: nothing of ours is left in it)
    int e = launch_reset(p->ws, p->stream);
    return e ? hip_fail(p, e) : TESSEL_OK;
}

static int fetch_best(tessel_problem *p)
{
    if (!p->ws || !p->ws_ready) { memset(&p->result, 0, sizeof p->result); p->result.period = INT_MAX; return TESSEL_OK; }
    if (!owns_workspace(p)) return TESSEL_E_WORKSPACE;       // another handle has bound the buffer since: the running best is gone
    hipError_t e = hipStreamSynchronize(p->stream);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    e = hipMemcpy(&p->result, (char *)p->ws + kWsResultOff, sizeof(DevResult), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    if (p->result.overflow && !p->safe_pieces) {
        // some launch left more candidates unfinished than its list holds, so the running best is incomplete:
        // score every range again, from now on in pieces small enough for the lists
        p->safe_pieces = true;
        int le = launch_reset(p->ws, p->stream);
        if (le) return hip_fail(p, le);
        for (const auto &r : p->ranges) {
            le = launch_eval(p->kp, r.first, r.second, p->ws, p->num_cus, p->max_blocks, p->stream, kSafePerLaunch);
            if (le) return hip_fail(p, le);
        }
        e = hipStreamSynchronize(p->stream);
        if (e != hipSuccess) return hip_fail(p, (int)e);
        e = hipMemcpy(&p->result, (char *)p->ws + kWsResultOff, sizeof(DevResult), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return hip_fail(p, (int)e);
    }
    if (p->result.period == INT_MAX) { p->have_detail = false; return TESSEL_OK; }
    if (p->have_detail && p->detail_index == p->result.index) { p->best_dirty = false; return TESSEL_OK; }
    // decode and re-score the best candidate on the GPU for its peaks and orders
    int le = launch_detail(p->kp, p->result.index, p->ws, p->num_cus, p->max_blocks, p->stream);
    if (le) return hip_fail(p, le);
    e = hipStreamSynchronize(p->stream);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    e = hipMemcpy(&p->detail, (char *)p->ws + kWsDetailOff, sizeof(DevDetail), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    p->have_detail = true; p->detail_index = p->result.index;
    p->best_dirty = false;
    return TESSEL_OK;
}

extern "C" int tessel_best(tessel_problem *p, tessel_result *out)
{
    if (!p || !out) return TESSEL_E_INVALID_ARG;
    int rc = fetch_best(p);
    if (rc) return rc;
    memset(out, 0, sizeof *out);
    out->lower_bound = p->kp.LB;
    out->n_evaluated = p->result.n_evaluated;
    out->n_feasible = p->result.n_status[kOk];
    for (int s = 1; s < kNumStatus; s++) out->n_reject[s] = p->result.n_status[s];
    out->n_window_sweeps = p->result.n_sweeps;
    out->n_blocks_placed = p->result.n_blocks;
    if (p->result.overflow) return TESSEL_E_WORKSPACE;       // more candidates deferred than the list holds
    if (p->result.period == INT_MAX) { out->period = -1; return TESSEL_E_NO_FEASIBLE; }
    out->period = p->result.period;
    out->index = p->result.index;
    out->peak_max = INT_MIN;
    for (int d = 0; d < p->kp.D; d++) { out->peak_mem[d] = p->detail.peak[d]; out->peak_max = std::max(out->peak_max, p->detail.peak[d]); }
    if (p->detail.status != kOk || p->detail.period != p->result.period) return TESSEL_E_HIP;   // kernels disagree: never expected
    return TESSEL_OK;
}

// ---- host post-processing of the single best candidate ---------------------------------
namespace {

struct Edge { int u, v, w, lag; };

// Difference constraints of the repeated window for the decoded candidate (Eq. 1 [1] and [3]
// with the window-to-window lags), then the least non-negative start times at period T.
std::vector<int> least_starts(const tessel_problem *p, const DevDetail &c, int T)
{
    const int NR = p->kp.NR, K = p->kp.K, D = p->kp.D;
    std::vector<Edge> edges;
    for (size_t e = 0; e < p->dep_src.size(); e++) {
        int i = p->dep_src[e], j = p->dep_dst[e], delta = c.leads[i] - c.leads[j];
        for (int q = 0; q < NR; q++) {
            int qp = q - delta;
            edges.push_back(qp >= 0 ? Edge{i * NR + qp, j * NR + q, p->t[i], 0} : Edge{i * NR + qp + NR, j * NR + q, p->t[i], 1});
        }
    }
    for (int d = 0; d < D; d++) {
        std::vector<int> occ(K, 0), nodes;
        for (int k = 0; k < c.order_len[d]; k++) { int g = c.orders[d][k]; nodes.push_back(g * NR + occ[g]++); }
        for (size_t k = 0; k + 1 < nodes.size(); k++) edges.push_back(Edge{nodes[k], nodes[k + 1], p->t[nodes[k] / NR], 0});
        if (!nodes.empty()) edges.push_back(Edge{nodes.back(), nodes.front(), p->t[nodes.back() / NR], 1});
    }
    std::vector<int> s(K * NR, 0);
    for (int pass = 0; pass <= K * NR; pass++) {
        bool changed = false;
        for (const Edge &e : edges) {
            int v = s[e.u] + e.w - e.lag * T;
            if (v > s[e.v]) { s[e.v] = v; changed = true; }
        }
        if (!changed) break;
    }
    return s;
}

}  // namespace

extern "C" int tessel_best_candidate(tessel_problem *p, int32_t *leads, int32_t *order_len, int32_t *orders, int32_t *starts)
{
    if (!p) return TESSEL_E_INVALID_ARG;
    int rc = fetch_best(p);
    if (rc) return rc;
    if (p->result.period == INT_MAX) return TESSEL_E_NO_FEASIBLE;
    const DevDetail &c = p->detail;
    if (leads) for (int i = 0; i < p->kp.K; i++) leads[i] = c.leads[i];
    if (order_len) for (int d = 0; d < p->kp.D; d++) order_len[d] = c.order_len[d];
    if (orders) for (int d = 0; d < p->kp.D; d++) for (int k = 0; k < kMaxPos; k++) orders[d * kMaxPos + k] = k < c.order_len[d] ? c.orders[d][k] : -1;
    if (starts) {
        std::vector<int> s = least_starts(p, c, c.period);
        for (size_t k = 0; k < s.size(); k++) starts[k] = s[k];
    }
    return TESSEL_OK;
}

// Sec. IV-C.  Warm-up = blocks (i, mu) with mu < lead_i, steady = R windows, cool-down = the rest
// (Eq. 5-6 for every micro-batch the windows do not cover).  Warm-up and cool-down are ordered by a
// serial greedy list schedule: of the blocks of the phase that are ready (producers scheduled) and
// fit the cap on each device they occupy, append the one with the smallest (earliest start,
// micro-batch, type).  A block starts at the maximum of its devices' free times and its producers'
// ends, which is also the earliest start for the final per-device orders.
// Completion candidate `ordinal` with jitter amplitude J around R copies of the best window; ordinal 0 or
// J = 0: the plain greedy schedule.  Per phase every type offers its lowest unscheduled micro-batch.
static int complete_with(tessel_problem *p, tessel_schedule *out, uint64_t ordinal, int J)
{
    const DevDetail &c = p->detail;
    const int N = out->num_microbatches, K = p->kp.K, D = p->kp.D, NR = p->kp.NR, M = p->kp.M;
    int maxlead = 0;
    for (int i = 0; i < K; i++) maxlead = std::max(maxlead, c.leads[i]);
    const int R = N >= 1 ? (N - maxlead) / NR : 0;
    if (R < 1 || out->capacity < K * N) return TESSEL_E_RANGE;
    std::vector<int> finish(K * N, -1), next(K, 0);
    std::vector<int> dev_free(D, 0), dev_mem(D, 0);
    for (int d = 0; d < D; d++) out->dev_len[d] = 0;
    std::vector<std::vector<int>> producers(K);
    for (size_t e = 0; e < p->dep_src.size(); e++) producers[p->dep_dst[e]].push_back(p->dep_src[e]);
    uint32_t kb = 0;
    const uint32_t ka = stream_keys(p->kp.seed + kCompletionKey, ordinal, kb);
    const bool noisy = ordinal != 0 && J > 0;

    auto earliest = [&](int i, int mu, int &est) -> bool {      // false if a producer is not scheduled yet
        est = 0;
        for (int a : producers[i]) {
            if (next[a] <= mu) return false;
            est = std::max(est, finish[a * N + mu]);
        }
        for (int d = 0; d < D; d++) if (p->mask[i] >> d & 1u) est = std::max(est, dev_free[d]);
        return true;
    };
    auto commit = [&](int i, int mu, int est) {
        out->start[i * N + mu] = est;
        finish[i * N + mu] = est + p->t[i];
        next[i] = mu + 1;
        for (int d = 0; d < D; d++) if (p->mask[i] >> d & 1u) {
            dev_free[d] = est + p->t[i];
            dev_mem[d] += p->m[i];
            out->dev_order[(size_t)d * out->capacity + out->dev_len[d]++] = i * N + mu;
        }
    };
    auto greedy_phase = [&](bool warmup) -> int {
        for (;;) {
            int pick = -1, pick_mu = 0, pick_est = 0, pick_key = 0;
            bool left = false;
            for (int i = 0; i < K; i++) {
                const int hi = warmup ? c.leads[i] : N, mu = next[i];
                if (mu >= hi) continue;
                left = true;
                int est;
                if (!earliest(i, mu, est)) continue;
                bool fits = true;
                if (p->m[i] > 0)
                    for (int d = 0; d < D; d++) if ((p->mask[i] >> d & 1u) && dev_mem[d] + p->m[i] > M) fits = false;
                if (!fits) continue;
                const int key = est + (noisy ? (int)((stream_draw16(ka, kb, (uint32_t)(i * N + mu)) * (uint32_t)(J + 1)) >> 16) : 0);
                if (pick < 0 || key < pick_key || (key == pick_key && mu < pick_mu)) { pick = i; pick_mu = mu; pick_est = est; pick_key = key; }
            }
            if (!left) return TESSEL_OK;
            if (pick < 0) return TESSEL_E_NO_SCHEDULE;
            commit(pick, pick_mu, pick_est);
        }
    };

    int rc = greedy_phase(true);
    if (rc) return rc;
    for (int k = 0; k < R; k++) {
        // replay the window in any executable sequence of the decoded per-device orders
        std::vector<int> pos(D, 0);
        int left = K * NR;
        while (left > 0) {
            bool moved = false;
            for (int d = 0; d < D; d++) {
                if (pos[d] >= c.order_len[d]) continue;
                int i = c.orders[d][pos[d]], mu = next[i], est;
                bool heads = true;
                for (int dd = 0; dd < D; dd++)
                    if ((p->mask[i] >> dd & 1u) && (pos[dd] >= c.order_len[dd] || c.orders[dd][pos[dd]] != i)) heads = false;
                if (!heads || !earliest(i, mu, est)) continue;
                commit(i, mu, est);
                for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) pos[dd]++;
                left--; moved = true;
            }
            if (!moved) return TESSEL_E_NO_SCHEDULE;
        }
    }
    rc = greedy_phase(false);
    if (rc) return rc;
    out->makespan = *std::max_element(finish.begin(), finish.end());
    out->period = c.period;
    out->num_windows = R;
    return TESSEL_OK;
}

extern "C" int tessel_complete_schedule(tessel_problem *p, tessel_schedule *out)
{
    if (!p || !out || !out->start || !out->dev_order || !out->dev_len) return TESSEL_E_INVALID_ARG;
    int rc = fetch_best(p);
    if (rc) return rc;
    if (p->result.period == INT_MAX) return TESSEL_E_NO_FEASIBLE;
    return complete_with(p, out, 0, 0);
}

// ---- searched completion: many perturbed greedy completions scored on the GPU -----------------------
// uploads what the kernel needs of the problem and of the best candidate (once per best candidate, N, J)
// The R replayed windows as a (max, +) matrix (CompMatrix), for problems whose types sit on one device each and that
// the kernel's per-type path takes.  A dry run of the replay finds the state slots read before they are written (the
// inputs) and the slots written (the outputs); one run per input with that input at 0 and the others at "no path"
// gives the longest paths.
static void window_matrix(const CompParams &cp, CompMatrix &cm)
{
    memset(&cm, 0, sizeof cm);
    bool single = cp.npaths <= 8 && !cp.dag;
    for (int i = 0; i < cp.K; i++) single = single && cp.mask[i] != 0 && (cp.mask[i] & (cp.mask[i] - 1)) == 0;
    if (!single) return;
    const int TR = cp.tok_ring, tmask = TR - 1, oFree = cp.npaths * TR, nslot = oFree + cp.D;      // rings first, then the devices
    struct Blk { int fr, tk, t; bool has_a; };
    std::vector<Blk> blocks;
    for (int k = 0; k < cp.R; k++)
        for (int s = 0; s < cp.nseq; s++) {
            const int i = cp.seq[s], mu = (int)cp.lead[i] + (int)cp.occ[s] + cp.NR * k;
            blocks.push_back({oFree + __builtin_ctz((unsigned)cp.mask[i]), (int)cp.path[i] * TR + (mu & tmask), cp.t[i], cp.pred[i] >= 0});
        }
    std::vector<int> state(nslot, 0);                       // 0 untouched, 1 read first, 2 written first; then: written at all
    std::vector<char> written(nslot, 0);
    for (const Blk &b : blocks) {
        if (!state[b.fr]) state[b.fr] = 1;
        if (b.has_a && !state[b.tk]) state[b.tk] = 1;
        if (!state[b.fr]) state[b.fr] = 2;
        if (!state[b.tk]) state[b.tk] = 2;
        written[b.fr] = written[b.tk] = 1;
    }
    std::vector<int> in, out;
    for (int v = 0; v < nslot; v++) { if (state[v] == 1) in.push_back(v); if (written[v]) out.push_back(v); }
    if (in.empty() || (int)in.size() > kMatIn || (int)out.size() > kMatOut) return;
    const long long none = -(1ll << 60);
    for (int o = 0; o < kMatOut; o++) for (int j = 0; j < kMatIn; j++) cm.a[o][j] = kNoPath;
    for (size_t j = 0; j < in.size(); j++) {
        std::vector<long long> x(nslot, none);
        x[in[j]] = 0;
        for (const Blk &b : blocks) {
            long long est = x[b.fr];
            if (b.has_a) est = std::max(est, x[b.tk]);
            x[b.fr] = x[b.tk] = est + b.t;
        }
        for (size_t o = 0; o < out.size(); o++) if (x[out[o]] >= 0) cm.a[o][j] = (int32_t)x[out[o]];
    }
    for (size_t o = 0; o < out.size(); o++) {               // every output must depend on some input
        bool any = false;
        for (size_t j = 0; j < in.size(); j++) any = any || cm.a[o][j] != kNoPath;
        if (!any) return;
    }
    for (size_t j = 0; j < in.size(); j++) cm.in_slot[j] = (uint16_t)in[j];
    for (size_t o = 0; o < out.size(); o++) cm.out_slot[o] = (uint16_t)out[o];
    cm.nin = (int32_t)in.size(); cm.nout = (int32_t)out.size();
}

static int bind_completion(tessel_problem *p, int N, int J)
{
    if (p->ws && p->ws_ready && !owns_workspace(p)) return TESSEL_E_WORKSPACE;      // the buffer is another handle's by now
    // (problems beyond the limits of the fast kernel keep their types, devices and micro-batches in more bits than the
    // completion kernel's tables hold; their greedy completion needs no kernel)
    if (p->kp.D > kMaxD || p->kp.K > kMaxK || p->kp.many || p->kp.NR > kMaxNR) return TESSEL_E_UNSUPPORTED;
    if (p->comp_ready && !p->best_dirty && p->comp_index == p->result.index && p->result.period != INT_MAX && p->comp.N == N &&
        p->comp.J == J)
        return TESSEL_OK;                                   // nothing new since the best was fetched: no wait
    int rc = fetch_best(p);
    if (rc) return rc;
    if (p->result.period == INT_MAX) return TESSEL_E_NO_FEASIBLE;
    if (p->comp_ready && p->comp_index == p->result.index && p->comp.N == N && p->comp.J == J) return TESSEL_OK;
    const DevDetail &c = p->detail;
    const int K = p->kp.K, D = p->kp.D, NR = p->kp.NR;
    if (N < 1 || J < 0 || J > 65535) return TESSEL_E_INVALID_ARG;
    int maxlead = 0;
    for (int i = 0; i < K; i++) maxlead = std::max(maxlead, c.leads[i]);
    const int R = (N - maxlead) / NR;
    if (R < 1) return TESSEL_E_RANGE;
    CompParams &cp = p->comp;
    memset(&cp, 0, sizeof cp);
    cp.D = D; cp.K = K; cp.NR = NR; cp.M = p->kp.M; cp.N = N; cp.J = J; cp.R = R; cp.nseq = K * NR;
    { const uint64_t seed = p->kp.seed + kCompletionKey; cp.seed_lo = (uint32_t)seed; cp.seed_hi = (uint32_t)(seed >> 32); }
    int npaths = 0;
    std::vector<std::vector<int>> producers(K);
    for (size_t e = 0; e < p->dep_src.size(); e++) producers[p->dep_dst[e]].push_back(p->dep_src[e]);
    for (int i = 0; i < K; i++) {
        if (p->m[i] < -128 || p->m[i] > 127) return TESSEL_E_UNSUPPORTED;
        cp.t[i] = p->t[i]; cp.m[i] = (int8_t)p->m[i]; cp.mask[i] = (uint8_t)p->mask[i];
        cp.pred[i] = p->kp.dag ? (int8_t)-1 : p->kp.pred[i];
        cp.lead[i] = (uint8_t)c.leads[i];
    }
    if (p->kp.dag) {
        // any acyclic graph: every type somebody consumes keeps the end times of its own blocks
        cp.dag = 1;
        std::vector<char> consumed(K, 0);
        for (size_t e = 0; e < p->dep_src.size(); e++) { consumed[p->dep_src[e]] = 1; cp.predmask[p->dep_dst[e]] |= 1u << p->dep_src[e]; }
        for (int i = 0; i < K; i++) cp.path[i] = consumed[i] ? (uint8_t)npaths++ : (uint8_t)0xFF;
    } else
    for (int i = 0; i < K; i++) if (p->kp.pred[i] < 0) {                 // chains numbered by their first type
        for (int g = i; g >= 0; g = p->kp.succ[g]) cp.path[g] = (uint8_t)npaths;
        npaths++;
    }
    cp.npaths = npaths;
    {
        // Phases and windows follow one another for all types together, so two types are never further apart than
        // (largest - smallest lead) + NR micro-batches; a ring of the next power of two above that holds every
        // micro-batch still on its way through a chain
        int lo = c.leads[0], hi = c.leads[0];
        for (int i = 1; i < K; i++) { lo = std::min(lo, c.leads[i]); hi = std::max(hi, c.leads[i]); }
        int ring = 1;
        while (ring < hi - lo + NR + 1) ring *= 2;
        cp.tok_ring = ring;
    }
    // one executable sequence of the window (the device orders of the best candidate)
    {
        std::vector<int> pos(D, 0), occ(K, 0);
        int n = 0;
        while (n < K * NR) {
            bool moved = false;
            for (int d = 0; d < D; d++) {
                if (pos[d] >= c.order_len[d]) continue;
                const int i = c.orders[d][pos[d]];
                bool heads = true;
                for (int dd = 0; dd < D; dd++)
                    if ((p->mask[i] >> dd & 1u) && (pos[dd] >= c.order_len[dd] || c.orders[dd][pos[dd]] != i)) heads = false;
                // its producers' blocks of the same micro-batch must come first: in this window, or they ran in an earlier one
                bool fed = true;
                for (int a : producers[i]) if (c.leads[a] + occ[a] <= c.leads[i] + occ[i]) fed = false;
                if (!heads || !fed) continue;
                cp.seq[n] = (uint8_t)i; cp.occ[n] = (uint8_t)occ[i]; n++;
                occ[i]++;
                for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) pos[dd]++;
                moved = true;
            }
            if (!moved) return TESSEL_E_NO_SCHEDULE;
        }
    }
    {
        // the kernel keeps times, memory and jitter in 16 bits
        long long total = 0;
        for (int i = 0; i < K; i++) total += (long long)p->t[i] * N;
        if (total + J > 65535 || std::abs(p->kp.M) > 30000 || N > 1023 || J > 63) return TESSEL_E_TOOBIG;
    }

    window_matrix(cp, p->comp_matrix);
    if (const char *env = getenv("TESSEL_REPLAY_BLOCKS")) {        // test knob: replay the windows block by block
        if (env[0] == '1') p->comp_matrix.nin = 0;
    }
    if (completion_lds_bytes(cp, p->comp_matrix) > 64 * 1024) return TESSEL_E_TOOBIG;
    hipError_t e = hipMemcpyAsync((char *)p->ws + kWsCompParamsOff, &cp, sizeof cp, hipMemcpyHostToDevice, p->stream);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    e = hipMemcpyAsync((char *)p->ws + kWsCompMatrixOff, &p->comp_matrix, sizeof(CompMatrix), hipMemcpyHostToDevice, p->stream);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    int le = launch_completion_reset(p->ws, p->stream);
    if (le) return hip_fail(p, le);
    p->comp_ready = true; p->comp_index = p->result.index;
    return TESSEL_OK;
}

extern "C" int tessel_search_completions(tessel_problem *p, int32_t num_microbatches, int32_t jitter, uint64_t first,
                                         uint64_t count)
{
    if (!p) return TESSEL_E_INVALID_ARG;
    if (first + count < first) return TESSEL_E_RANGE;
    int rc = bind_completion(p, num_microbatches, jitter);
    if (rc) return rc;
    int e = launch_completions(p->comp, p->comp_matrix, first, count, nullptr, p->ws, p->num_cus, p->stream);
    return e < 0 ? TESSEL_E_TOOBIG : e ? hip_fail(p, e) : TESSEL_OK;
}

extern "C" int tessel_score_completions(tessel_problem *p, int32_t num_microbatches, int32_t jitter, uint64_t first,
                                        uint64_t count, int32_t *makespan_dev)
{
    if (!p || !makespan_dev) return TESSEL_E_INVALID_ARG;
    if (first + count < first) return TESSEL_E_RANGE;
    int rc = bind_completion(p, num_microbatches, jitter);
    if (rc) return rc;
    int e = launch_completions(p->comp, p->comp_matrix, first, count, makespan_dev, p->ws, p->num_cus, p->stream);
    return e < 0 ? TESSEL_E_TOOBIG : e ? hip_fail(p, e) : TESSEL_OK;
}

extern "C" int tessel_best_completion(tessel_problem *p, tessel_schedule *out, uint64_t *ordinal)
{
    if (!p || !out || !out->start || !out->dev_order || !out->dev_len) return TESSEL_E_INVALID_ARG;
    if (!p->comp_ready || !p->ws) return TESSEL_E_NO_FEASIBLE;
    if (!owns_workspace(p)) return TESSEL_E_WORKSPACE;
    if (out->num_microbatches != p->comp.N) return TESSEL_E_INVALID_ARG;
    hipError_t e = hipStreamSynchronize(p->stream);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    DevCompletion best;
    e = hipMemcpy(&best, (char *)p->ws + kWsCompletionOff, sizeof best, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(p, (int)e);
    if (best.makespan == INT_MAX) return TESSEL_E_NO_SCHEDULE;
    int rc = complete_with(p, out, best.ordinal, p->comp.J);
    if (rc) return rc;
    if (out->makespan != best.makespan) return TESSEL_E_HIP;        // host and kernel disagree: never expected
    if (ordinal) *ordinal = best.ordinal;
    return TESSEL_OK;
}

// ---- Sec. IV-D: global sequence of blocks and send/receive pairs -----------------------------------
extern "C" int tessel_instantiate(const tessel_problem *p, const tessel_schedule *sched, tessel_op *ops, int32_t capacity,
                                  int32_t *num_ops)
{
    if (!p || !sched || !sched->start || !num_ops || (capacity > 0 && !ops) || sched->num_microbatches < 1)
        return TESSEL_E_INVALID_ARG;
    const int K = p->kp.K, D = p->kp.D, N = sched->num_microbatches;
    const int ndeps = (int)p->dep_src.size();
    for (int x = 0; x < K * N; x++) if (sched->start[x] < 0) return TESSEL_E_INVALID_ARG;
    auto lowest = [](uint32_t mask) { int d = 0; while (!(mask >> d & 1u)) d++; return d; };
    // blocks by (start time, lowest device); two blocks of one device never start together (t >= 1)
    std::vector<int> seq(K * N);
    for (int x = 0; x < K * N; x++) seq[x] = x;
    std::stable_sort(seq.begin(), seq.end(), [&](int a, int b) {
        if (sched->start[a] != sched->start[b]) return sched->start[a] < sched->start[b];
        return lowest(p->mask[a / N]) < lowest(p->mask[b / N]);
    });
    std::vector<tessel_op> out;
    out.reserve((size_t)K * N * 2);
    for (size_t at = 0; at < seq.size();) {
        size_t end = at;
        while (end < seq.size() && sched->start[seq[end]] == sched->start[seq[at]]) end++;
        for (size_t k = at; k < end; k++)
            out.push_back({TESSEL_OP_BLOCK, seq[k], (int32_t)p->mask[seq[k] / N], sched->start[seq[k]], 0});
        for (size_t k = at; k < end; k++) {
            const int i = seq[k] / N, mu = seq[k] % N;
            for (int e = 0; e < ndeps; e++) {
                if (p->dep_src[e] != i) continue;
                const int j = p->dep_dst[e];
                const uint32_t need = p->mask[j] & ~p->mask[i];        // consumer devices without the tensor
                for (int v = 0; v < D; v++)
                    if (need >> v & 1u) out.push_back({TESSEL_OP_SENDRECV, seq[k], lowest(p->mask[i]), v, j * N + mu});
            }
        }
        at = end;
    }
    *num_ops = (int32_t)out.size();
    if ((size_t)capacity < out.size()) return TESSEL_E_RANGE;
    std::copy(out.begin(), out.end(), ops);
    return TESSEL_OK;
}

// ---- Alg. 1: the loop over window sizes around the scoring kernels -------------------------

// CalMaxInflight of Alg. 1 (the paper gives no formula): one micro-batch alone, blocks in topological
// order with the smallest type id first, holds at most hold_d on device d; floor(M / hold_d) of them fit.
static int max_inflight(const tessel_problem_desc *desc, int unbounded)
{
    const int K = desc->num_block_types;
    std::vector<int> indeg(K, 0), done(K, 0), topo;
    for (int e = 0; e < desc->num_deps; e++) indeg[desc->dep_dst[e]]++;
    for (;;) {
        int pick = -1;
        for (int i = 0; i < K; i++) if (!done[i] && indeg[i] == 0) { pick = i; break; }
        if (pick < 0) break;
        done[pick] = 1; topo.push_back(pick);
        for (int e = 0; e < desc->num_deps; e++) if (desc->dep_src[e] == pick) indeg[desc->dep_dst[e]]--;
    }
    int best = unbounded;
    for (int d = 0; d < desc->num_devices; d++) {
        int run = 0, hold = 0;
        for (int i : topo) if (desc->dev_mask[i] >> d & 1u) { run += desc->mem[i]; hold = std::max(hold, run); }
        if (hold > 0) best = std::min(best, desc->mem_cap / hold);
    }
    return best;
}

extern "C" int tessel_search_workspace_bytes(const tessel_problem_desc *desc, const tessel_search *in, size_t *bytes)
{
    if (!desc || !in || !bytes || in->max_nr < 1 || in->max_nr > TESSEL_MAX_NR) return TESSEL_E_INVALID_ARG;
    size_t need = 0;
    int limit = in->max_nr;
    for (int nr = 1; nr <= limit; nr++) {
        tessel_problem_desc d = *desc;
        d.nr = nr; d.fixed_leads = nullptr;
        tessel_problem *p = nullptr;
        int rc = tessel_problem_create(&d, &p);
        if (rc) return rc;
        if (nr == 1 && in->use_inflight_bound) limit = std::max(1, std::min(limit, max_inflight(desc, in->max_nr)));
        size_t b = 0;
        rc = tessel_workspace_bytes(p, &b);
        tessel_problem_destroy(p);
        if (rc) return rc;
        need = std::max(need, b);
    }
    *bytes = need;
    return TESSEL_OK;
}

extern "C" int tessel_search_run(const tessel_problem_desc *desc, tessel_search *io, void *workspace_dev,
                                 size_t workspace_bytes, void *hip_stream, tessel_problem **best_out)
{
    if (best_out) *best_out = nullptr;
    if (!desc || !io || io->max_nr < 1 || io->max_nr > TESSEL_MAX_NR) return TESSEL_E_INVALID_ARG;
    const uint64_t per_launch = io->launch_candidates ? io->launch_candidates : (uint64_t)1 << 24;
    io->inflights = 0; io->lower_bound = 0; io->nr_tried = 0; io->best_nr = 0; io->best_period = -1;
    io->early_exit = 0; io->best_index = 0;
    for (int n = 0; n <= TESSEL_MAX_NR; n++) { io->period_nr[n] = -1; io->index_nr[n] = 0; io->evaluated_nr[n] = 0; }

    int limit = io->max_nr;
    for (int nr = 1; nr <= limit && !io->early_exit; nr++) {
        tessel_problem_desc d = *desc;
        d.nr = nr; d.fixed_leads = nullptr;
        tessel_problem *p = nullptr;
        int rc = tessel_problem_create(&d, &p);
        if (rc) return rc;
        if (nr == 1) {
            io->lower_bound = p->kp.LB;
            io->inflights = max_inflight(desc, io->max_nr);
            if (io->use_inflight_bound) limit = std::min(limit, io->inflights);
            if (limit < 1) { tessel_problem_destroy(p); break; }
        }
        io->nr_tried = nr;
        const uint64_t n = std::min(p->count, io->max_candidates);
        tessel_result r;
        for (uint64_t first = 0; first < n && !io->early_exit; first += per_launch) {
            const uint64_t cnt = std::min(per_launch, n - first);
            rc = tessel_eval_candidates(p, first, cnt, workspace_dev, workspace_bytes, hip_stream);
            if (rc) { tessel_problem_destroy(p); return rc; }
            rc = tessel_best(p, &r);                                  // waits for the launch
            if (rc && rc != TESSEL_E_NO_FEASIBLE) { tessel_problem_destroy(p); return rc; }
            io->evaluated_nr[nr] = r.n_evaluated;
            if (rc == TESSEL_OK) {
                io->period_nr[nr] = r.period; io->index_nr[nr] = r.index;
                // launches ascend in index, so the running best is what a candidate-by-candidate scan
                // would hold after the first candidate that reaches the bound
                if (r.period == nr * io->lower_bound) io->early_exit = 1;
            }
        }
        if (io->period_nr[nr] >= 0 &&
            (io->best_period < 0 || (int64_t)io->period_nr[nr] * io->best_nr < (int64_t)io->best_period * nr)) {
            io->best_period = io->period_nr[nr]; io->best_nr = nr; io->best_index = io->index_nr[nr];
        }
        tessel_problem_destroy(p);
    }
    if (io->best_nr == 0) return TESSEL_E_NO_FEASIBLE;
    if (best_out) {
        tessel_problem_desc d = *desc;
        d.nr = io->best_nr; d.fixed_leads = nullptr;
        tessel_problem *p = nullptr;
        int rc = tessel_problem_create(&d, &p);
        if (rc) return rc;
        rc = tessel_eval_candidates(p, io->best_index, 1, workspace_dev, workspace_bytes, hip_stream);
        tessel_result r;
        if (!rc) rc = tessel_best(p, &r);
        if (!rc && (r.period != io->best_period || r.index != io->best_index)) rc = TESSEL_E_HIP;   // never expected
        if (rc) { tessel_problem_destroy(p); return rc; }
        *best_out = p;
    }
    return TESSEL_OK;
}

extern "C" int tessel_last_hip_error(const tessel_problem *p) { return p ? p->last_hip : 0; }
