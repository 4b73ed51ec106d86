// Shared between the host side of the library and its HIP kernels: the kernel-argument
// block that carries one problem's static tables, and the records the kernels write.
// (Not part of the public ABI; the oracle does not see this file.)
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define TESSEL_HD __host__ __device__ inline
#else
#define TESSEL_HD inline
#endif

namespace tessel {

// ------------------------------------------------------------------ counter-based sampler
// SplitMix64 finaliser keys a candidate ordinal; MurmurHash3's 32-bit finaliser, with the second
// key folded in between its multiplications, gives the w-th word; two 16-bit draws a word.
TESSEL_HD uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}
TESSEL_HD uint32_t stream_word(uint32_t a, uint32_t b, uint32_t w)
{
    uint32_t x = a + w * 0x9E3779B9u;
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= b;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
// 16-bit draw number j of the stream keyed by (seed, ordinal)
TESSEL_HD uint32_t stream_keys(uint64_t seed, uint64_t ordinal, uint32_t &kb)
{
    const uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * (ordinal + 1));
    kb = (uint32_t)(z >> 32);
    return (uint32_t)z;
}
TESSEL_HD uint32_t stream_draw16(uint32_t ka, uint32_t kb, uint32_t j)
{
    return (stream_word(ka, kb, j >> 1) >> (16u * (j & 1u))) & 0xFFFFu;
}
constexpr uint64_t kCompletionKey = 0x632BE59BD9B4E019ULL;      // separates the completion stream from the candidates'

constexpr int kMaxD = 8;         // simulated devices of the problems the fast kernel and the chain path of the general one take
constexpr int kMaxDW = 32;       // ... of any problem: more than kMaxD go the general kernel's path for graphs
constexpr int kMaxLT = 4;        // block types per device of the problems the fast kernel and the chain path take
constexpr int kMaxLTW = 8;       // ... of any problem (sampled spaces): more than kMaxLT go the general kernel's path for graphs
constexpr int kMaxNR = 8;        // micro-batches per window of the problems the fast kernel, the chain path and the exhaustive spaces take
constexpr int kMaxNRW = 16;      // ... of any problem (sampled spaces): more than kMaxNR go the general kernel's path for graphs
constexpr int kMaxK = 32;        // block types of the problems the fast kernel and the chain path of the general one take
constexpr int kMaxKW = 64;       // ... of any problem: more than kMaxK go the general kernel's path for graphs
constexpr int kMaxPos = kMaxLT * kMaxNR;   // blocks per device and window (32)
constexpr int kMaxDeps = 128;     // dependencies of a micro-batch whose graph is not a set of chains
constexpr uint32_t kNoRing = 0xFFFFu;   // no ring of end times (KParams::tokbase)
constexpr int kNumStatus = 6;
constexpr int kWave = 64;

enum Space { kFactorial = 0, kCanonical = 1, kSampledStrict = 2, kSampledRepair = 3 };
enum Status { kOk = 0, kDup = 1, kTpMismatch = 2, kProp2 = 3, kDeadlock = 4, kMem = 5 };

// Everything a kernel needs to know about the problem (Table I of the paper: D, K, M,
// t_B, m_B, d_B, dependencies) plus derived tables.  "local symbol" y = position of a block
// type among the types of one device (ascending type id); a device order is a sequence of
// local symbols (2 bits each; 3 where a device holds more than four types).
struct KParams {
    int32_t D, K, NR, M;
    int32_t total;               // K * NR blocks per window
    int32_t space;               // Space
    int32_t tp;                  // some block occupies more than one device
    int32_t npaths;              // dependency chains
    int32_t nslots;              // D device slots + npaths * 2*NR token slots
    int32_t nsweeps;             // D + npaths*NR + 1 window sweeps determine the period
    int32_t LB, UB;
    int32_t has_fixed;
    uint32_t step_q16;
    uint64_t seed;
    int32_t  ntd[kMaxDW];        // block types on device d
    uint32_t type_of[kMaxDW];    // 4 x 8 bit: type id of local symbol y (0xFF = none)
    uint32_t type_of_hi[kMaxDW]; // ... of local symbols 4-7
    uint32_t pred_of[kMaxD];     // 4 x 8 bit: type id of its producer (0xFF = none)
    uint32_t mask_of[kMaxD];     // 4 x 8 bit: device mask of that type
    uint32_t tok_of[kMaxD];      // 4 x 8 bit: first token slot of the type's chain
    uint32_t home_of[kMaxD];     // 4 x 8 bit: (lowest device)*4 + local symbol there
    int32_t  t_of[kMaxD][kMaxLT];
    int32_t  m_of[kMaxDW][kMaxLTW];
    int8_t   succ[kMaxK];        // consumer type of type g or -1
    uint8_t  edge_out[kMaxK];    // position of the dependency g -> succ[g] in the caller's list
    uint8_t  cross_out[kMaxK];   // that dependency joins different device sets
    uint8_t  rtopo[kMaxKW];      // types, consumers before producers
    uint8_t  fixed[kMaxKW];      // fixed leads
    int8_t   pred[kMaxK];        // producer type of type g or -1
    int32_t  t_loc[kMaxK];       // t by home code (device*4 + symbol)
    uint32_t mask_loc[kMaxK];    // device mask by home code
    uint32_t fact[13];           // FACTORIAL: n! for n <= 12
    uint64_t init_list[kMaxDW];  // FACTORIAL: labelled blocks of a device, 5 bits each (y<<3 | label)
    uint64_t cdev[kMaxDW];       // FACTORIAL: n_d!;  CANONICAL: arrangements of device d
    // fast path (single-device blocks only), block types addressed by code = device*4 + symbol
    int32_t  fast_ok;            // the problem fits the fast kernel
    uint32_t info_loc[kMaxK];    // bits 0-5 consumer code (63 none), 6-11 producer code (63 none),
                                 // 12-17 first token slot of the chain, 18-25 memory delta (signed)
    uint32_t chain_tab[kMaxK];   // k-th block type, consumers before producers: bits 0-5 code, 6-11 consumer code
                                 // (63 none), 12-18 dependency number, 19 different device sets, 20 first of its
                                 // chain, 21-26 type id
    uint32_t vtab[24];           // boundary value v: bits 0-5 state slot; 6 device value; 7-12 code of the first block
                                 // of the chain (token values); 13-16 micro-batch offset j; 17 device has blocks
    // sampled leads as sums of per-dependency steps (bit k of the step mask = dependency out of the k-th
    // entry of chain_tab)
    uint32_t cum_code[kMaxK];    // by code: step bits whose sum (capped at N_R-1) is the type's lead
    uint32_t pred_bit[kMaxK];    // by code: step bit of the dependency from its producer (0 = first of its chain)
    uint32_t dep_bit[kMaxK];     // by dependency number: its step bit, 0 if both ends sit on the same device set
    uint32_t mpack[kMaxD];       // memory deltas of the device's 4 types, 8 bits each (signed)
    int32_t  eigen_tries;        // window sweeps a candidate gets at first, and
    int32_t  retry_tries;        // ... from the start again when those found no eigenvector (both: test knobs)
    // blocks on several devices in the fast kernel: such a type has one code on every device it occupies
    int32_t  fast_tp;            // the problem has such blocks (the TP variants of the fast kernel take it)
    int32_t  ntp;                // number of such types
    uint32_t tp_group[kMaxD];    // their codes, one mask per type
    uint32_t slow_mask;          // codes of types that sit on several devices or whose consumer does
    uint32_t grp_code[kMaxK];    // by code: all codes of the same type
    uint8_t  home_code[kMaxK];   // by code: the type's code on its lowest device (63: no such code)
    // Dependency graphs that are not disjoint chains (a block type with several producers or consumers): scored by the
    // general kernel's DAG path, tables by type id
    int32_t  dag;                // the problem takes that path
    int32_t  ndeps;
    int32_t  dag_tries;          // sweeps of the eigenvector search before the bisection takes over (test knob)
    int32_t  ntok;               // rings of 2 N_R end times by micro-batch behind the D device slots: one per unbranched stretch
                                 // of the graph (types joined by dependencies a -> b with a's only consumer b and b's only producer a)
    int32_t  t_type[kMaxKW];
    uint32_t mask_type[kMaxKW];  // devices of the type
    uint64_t predmask[kMaxKW];   // its producers
    uint16_t tokbase[kMaxKW];    // first slot of the ring the type writes its end times to, kNoRing: nobody consumes it
    uint8_t  ring_head[kMaxKW];  // by ring: the first type of its stretch (the largest lead: Property 2)
    uint16_t ring_base[kMaxKW];  // ... its first slot
    uint16_t ring_kept[kMaxKW];  // ... first of the N_R slots that keep what the last window boundary left in its lower half: behind
                                 // the ring for a stretch of several types (the later ones overwrite the entries), the ring's own
                                 // lower half for a single type (which never writes below its lead)
    uint8_t  dsrc[kMaxDeps], ddst[kMaxDeps], dcross[kMaxDeps];   // the dependencies in the caller's order
    uint64_t predmask_of[kMaxDW][kMaxLTW]; // producers of local symbol y of device d
    int32_t  many;               // some device holds more than kMaxLT block types (3-bit symbols; sampled spaces only)
    const int8_t   *leadtab;     // CANONICAL: [nlead][K] in device memory
    const uint64_t *wtab;        // CANONICAL: arrangements by remaining counts, base NR+1 digits
};

// Running best + counters of one search; lives at the start of the caller's workspace.
struct DevResult {
    int32_t  period;             // INT32_MAX = nothing feasible yet
    int32_t  pad;
    uint64_t index;
    uint64_t n_evaluated;
    uint64_t n_status[kNumStatus];   // [kOk] = feasible
    uint64_t n_sweeps;               // window sweeps spent on period computations (fast kernel)
    uint32_t n_retried;              // candidates that needed the longer eigenvector search so far
    uint32_t n_deferred;             // candidates handed to the general kernel so far
    uint32_t overflow;               // a list was too small at some point: results are incomplete
    uint32_t pad1;
    uint32_t defer_count;            // entries of the deferred list of the launch in flight
    uint32_t pad2;
    uint64_t n_blocks;               // blocks placed by the builds of the fast kernel
};

// Decoded best candidate, written by the detail kernel.
struct DevDetail {
    int32_t status, period;
    int32_t peak[kMaxDW];
    int32_t leads[kMaxKW];
    int32_t order_len[kMaxDW];
    int32_t orders[kMaxDW][kMaxPos];
};

// Searched completion (warm-up / cool-down orders as perturbed greedy schedules around the best window):
// what the kernel needs of the problem and of the best candidate, by block type, and the running best.
constexpr int kMaxSeq = kMaxK * kMaxNR;
struct CompParams {
    int32_t  D, K, NR, M, N, J, R, nseq, npaths;
    int32_t  tok_ring;               // slots per chain (graphs: per consumed type; npaths counts them) for the end times of the
                                     // micro-batches in flight: a power of two above (largest - smallest lead) + NR, the most
                                     // two types are ever apart
    uint32_t seed_lo, seed_hi;       // problem seed + kCompletionKey (two words: the kernel's copy of this block in LDS
                                     // is written word by word, and nothing in it is read through a wider type)
    int32_t  t[kMaxK];
    int8_t   m[kMaxK];
    uint8_t  mask[kMaxK];
    int8_t   pred[kMaxK];            // producer type or -1 (chains)
    uint8_t  path[kMaxK];            // dependency chain of the type; graphs: the type's own ring, 0xFF = nobody consumes it
    int32_t  dag;                    // the micro-batch graph is not a set of chains: producers by mask, one ring per consumed type
    uint32_t predmask[kMaxK];        // graphs: bit a = type a is a producer
    uint8_t  lead[kMaxK];
    uint8_t  seq[kMaxSeq];           // the window's blocks (types) in an executable order
    uint8_t  occ[kMaxSeq];           // occurrence number of seq[s] among the earlier entries of its type
};
// The R replayed windows of a completion candidate as one linear map in the (max, +) algebra: every state slot the
// windows write (device free times, end times in the rings) is the largest of (input + longest path) over the slots
// they read before writing them.  The same for every candidate, since the window is; computed on the host.
constexpr int kMatIn = 16, kMatOut = 32;
constexpr int32_t kNoPath = -(1 << 24);
struct CompMatrix {
    int32_t  nin, nout;              // nin = 0: not available (the kernel replays the windows block by block)
    uint16_t in_slot[kMatIn];        // state slots (numbering of the kernel), in the order of the columns
    uint16_t out_slot[kMatOut];
    int32_t  a[kMatOut][kMatIn];     // kNoPath: no path; columns from nin on are kNoPath
};
struct DevCompletion {
    int32_t  makespan;               // INT32_MAX = nothing scheduled yet
    int32_t  pad;
    uint64_t ordinal;
};
struct CompRec { int32_t makespan; int32_t pad; uint64_t ordinal; };

constexpr size_t kWsResultOff = 0;
constexpr size_t kWsCompletionOff = 192;       // DevCompletion
constexpr size_t kWsDetailOff = 256;
constexpr size_t kWsParamsOff = 8192;          // KParams of the bound problem
constexpr size_t kWsTablesOff = 16384;         // lead table, arrangement table
constexpr size_t kWsTablesMax = 1 << 20;
constexpr size_t kWsListOff = kWsTablesOff + kWsTablesMax;     // candidates deferred to the general kernel
constexpr uint32_t kWsListCap = 1u << 20;
constexpr size_t kWsCompParamsOff = kWsListOff + (size_t)kWsListCap * 8;   // CompParams
constexpr size_t kWsCompMatrixOff = kWsCompParamsOff + 1024;              // CompMatrix
constexpr size_t kWsBlockRecOff = kWsCompMatrixOff + 3072;
constexpr int kDeferBlocks = 64;                                // grid of the deferred pass
constexpr int kFirstPassTries = 2;                              // sweeps before a candidate queues for the longer search
constexpr uint64_t kMaxPerLaunch = 1ull << 26;                  // candidates per pass of the kernels
constexpr uint64_t kSafePerLaunch = 1ull << 20;                 // ... at which no list can overflow (<= both list capacities)
constexpr int kRetryTries = 8;                                  // ... and before the general kernel gets it

// queues between the phases of the fast kernel: three rings per wave behind the block records
constexpr uint32_t kRingSlots = 128;                            // a power of two >= 2 * 64 - 1
constexpr int kRingMetaWords = 8;                               // rings 2 and 3: leads (4), index (2), peak (1), unused (1), then the program
constexpr int kStageMetaWords = 12;                             // ring 1: R, HM, X, worst, leads (4), index (2), unused (2), then
                                                                // the device records (4 words each) and the program so far

static_assert(sizeof(CompParams) <= 1024, "completion parameters must fit their workspace slot");
static_assert(sizeof(DevResult) <= kWsCompletionOff && kWsCompletionOff + sizeof(DevCompletion) <= kWsDetailOff, "result records overlap");
static_assert(sizeof(CompParams) <= 1024 && sizeof(CompMatrix) <= 3072, "completion parameters must fit their workspace slots");
static_assert(sizeof(KParams) <= kWsTablesOff - kWsParamsOff, "parameter block must fit its workspace slot");
static_assert(sizeof(DevDetail) <= kWsParamsOff - kWsDetailOff, "detail record must fit its workspace slot");

struct LaunchShape { int blocks, threads; size_t lds_bytes; };

// kernels.hip
// max_blocks: 0, or the most workgroups the workspace has queues for
LaunchShape eval_launch_shape(const KParams &kp, int num_cus, int max_blocks);
size_t eval_workspace_bytes(const KParams &kp, int num_cus, int max_blocks);    // everything launch_eval / launch_score touch
int launch_eval(const KParams &kp, uint64_t first, uint64_t count, void *ws, int num_cus, int max_blocks, void *stream, uint64_t max_piece);
int launch_score(const KParams &kp, uint64_t first, uint64_t count, int32_t *code, int32_t *peak, void *ws, int num_cus,
                 int max_blocks, bool general, void *stream);
// the library's own workspace on the current device (no allocation), and the grid that fits a workspace
constexpr size_t kScratchBytes = (size_t)24 << 20;
int scratch_workspace(void **ptr, size_t *bytes);
int eval_blocks_that_fit(const KParams &kp, int num_cus, size_t bytes);
int launch_detail(const KParams &kp, uint64_t index, void *ws, int num_cus, int max_blocks, void *stream);
int launch_reset(void *ws, void *stream);
// completion search: S = state words per lane; returns 0 or a HIP error (negative: LDS need exceeds the device's)
size_t completion_lds_bytes(const CompParams &cp, const CompMatrix &cm);
int launch_completions(const CompParams &cp, const CompMatrix &cm, uint64_t first, uint64_t count, int32_t *makespan_out, void *ws, int num_cus,
                       void *stream);
int launch_completion_reset(void *ws, void *stream);
int launch_alu_probe(uint32_t *out, int blocks, int rounds, void *stream);
constexpr int kProbeThreads = 256;
constexpr int kProbeLaneOpsPerRound = 32;

}  // namespace tessel
