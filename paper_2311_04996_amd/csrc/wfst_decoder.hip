// WFST token-passing beam search for CTC models on MI355X (gfx950, wave64).
//
// One persistent 1024-thread workgroup owns one channel (utterance / audio stream) and runs
// the whole per-frame iteration of the paper's Section "Algorithm description" on the
// device: ExpandArcs over emitting arcs -> recombination -> Prune (beam + max-active) ->
// epsilon closure -> backpointer store, frame after frame, synchronising only with
// workgroup barriers.  There is no per-frame kernel launch (the overhead the paper removes
// with CUDA graphs) and no per-frame device-to-host copy (the lattice stays in HBM and the
// traceback runs on the device).
//
// Recombination (one token per destination state, lowest (cost, arc id) wins) uses NO global
// atomics: measured on MI355X, random 64-bit global atomics top out near 20 G/s for the whole
// chip, which bounded an earlier global-hash design.  Instead ExpandArcs appends candidates
// {next, cost, source token, arc} to a buffer in four regions (by hash of the destination;
// wave-aggregated, so the stores coalesce); a histogram of a sample of the candidate costs
// selects the few that can survive max-active, and those are reduced in an open-addressing
// table that lives in LDS (160 KB per CU on gfx950) with LDS compare-and-swap, in as many
// passes (a region, or a hash range of it) as the table needs.  After a pass every inserted
// candidate looks at its slot again: the one still there is the recombined token of its
// destination ("winner") and carries its own record on; nobody scans the table.  In the
// epsilon closure "does this state already have a token" is answered the other way round: the
// tokens of the set look their own state up in the round's table, so there is no state -> token
// index in memory at all.
//
// ExpandArcs has no block-wide barrier: every wave takes runs of 64 tokens from a counter in
// LDS and expands them on its own (first arc by the owning lane, the other arcs flattened
// over the wave, very large states shared segment by segment), so the waves drift apart and
// one wave's memory waits overlap another's arithmetic.  A token in a "simple" state (its only
// arc is the graph's most frequent self-loop: in a CTC graph the blank self-loop, where most
// hypotheses sit) is expanded from its queue record alone, and its candidate is never written:
// a bit filter of the buffer's destinations tells which of these tokens can meet another
// candidate at all; the rest are the recombined tokens of their states as they stand.  The hot loops are bound by
// instruction issue (4 waves per SIMD, 4 cycles per wave64 instruction): they are written
// branch-free where it matters.
//
// The graph is stored as one array of 16-byte units, a block per state: a header
// {state id, final cost, emitting degree, both degrees packed in one word}, then the state's
// epsilon arcs, then its emitting arcs, every arc {next, weight, ilabel, olabel}, padded to 32
// bytes.  The packed word sits right before the first arc, so ONE 16-byte load at byte 12 of a
// block brings the degrees and next/weight/ilabel of the first arc.  A state is
// named by its block number (byte offset / 32), which is also the recombination key and grows
// with the state id.  `next` of an arc is the destination's block number plus three flag bits
// (the destination has epsilon arcs / an epsilon arc enters it / it is a simple state), so a token is created from
// the arc alone and the only random graph read per token is the 32-byte header + first arc
// when the token is expanded.  An arc's id is its unit address (epsilon arcs have bit 30 set),
// which orders arcs exactly as (emitting before epsilon, state, position) does.
//
// Per channel, in HBM:
//   token queue   2 x qcap records {key (B state, block number) + flag bits of the state, cost}
//   candidates    cand_cap records {next (block number + flags), cost, source token, arc id}
//   winners       recombined in-beam tokens before the max-active cutoff is known
//   worklists     2 x qcap records {token, block number, cost, first time}
//   lattice       {prev token, arc id} per stored token, frame after frame
// LDS holds, per phase, either the expansion tables (negated log-likelihood row, a slice per
// wave with the prefix sums of its run's arc counts, the list of very large states) or the
// recombination table; beside them the item tables of the epsilon closure, the slot noted for
// every candidate of a table pass, the word-boost table, the 256-bin cost histogram and the
// running best cost.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <string>
#include <unordered_map>
#include <vector>

#include "wfst_decoder.h"

namespace {

#ifndef WFST_BLOCK
#define WFST_BLOCK 1024
#endif
#ifndef WFST_TAB
#define WFST_TAB 8192
#endif
#ifndef WFST_MIN_WAVES
#define WFST_MIN_WAVES 4
#endif
constexpr int kBlock = WFST_BLOCK;            // threads of the workgroup that owns a channel
constexpr int kWaves = kBlock / 64;
#ifndef WFST_U
#define WFST_U 2
#endif
constexpr int kWaveTok = 64;                  // tokens a wave expands at a time (one per lane)
constexpr int kHubCap = 512;                  // listed high-degree tokens per frame (more are expanded by their wave)
constexpr int kHubDeg = 512;                  // arcs beyond which a token is listed there
constexpr int kMaxV = 2048;
constexpr int kU = WFST_U;                    // independent memory requests per lane per phase
#ifndef WFST_UE
#define WFST_UE 2
#endif
#ifndef WFST_UC
#define WFST_UC 2
#endif
constexpr int kUE = WFST_UE;                  // ... in ExpandArcs over emitting arcs
constexpr int kHubSeg = 64 * kUE;             // arcs of a listed state one wave takes at a time
#ifndef WFST_SEL_EVERY
#define WFST_SEL_EVERY 8                      // the selection histogram reads one run of 64 candidates out of this many
#endif
#ifndef WFST_UM
#define WFST_UM 1
#endif
#ifndef WFST_USW
#define WFST_USW 2                            // queue records in flight per lane when the staying tokens are sorted out
#endif
constexpr int kUC = WFST_UC;                  // ... when survivors become tokens
#ifndef WFST_REGION_BITS
#define WFST_REGION_BITS 2
#endif
constexpr int kRegionBits = WFST_REGION_BITS;
constexpr int kRegions = 1 << kRegionBits;    // candidate buffer regions (by destination hash)
constexpr int kTabSlots = WFST_TAB;           // LDS recombination table (power of two)
constexpr unsigned kTabMask = kTabSlots - 1;
#ifndef WFST_GT
#define WFST_GT 12
#endif
constexpr int kGroupTarget = kTabSlots * WFST_GT / 16; // mean candidates reduced per table pass (load 0.75)
#ifndef WFST_BOOST
#define WFST_BOOST 2048
#endif
constexpr int kBoostSlots = WFST_BOOST;       // per-channel table of the boosting acceptor's arcs (open addressing)
constexpr int kBoostMax = kBoostSlots / 2;    // arcs it may hold
constexpr int kBoostStage = 3 * kBoostSlots + 2;   // host staging of one channel's acceptor, in words
constexpr int kBoostStateBits = 12;           // states of a boosting acceptor: at most 4096 (and what the keys have room for)
constexpr int kQueueMax = 65536;              // tokens per closed set
constexpr unsigned long long kValEmpty = ~0ull;
constexpr int kKeyEmpty = -1;
constexpr int kKeyNone = -2;                  // no key at all (a probe sequence that gave up)
constexpr unsigned kOrdNone = 0xFFFFFFFFu;
constexpr int kModeInit = 1, kModeFinal = 2;
constexpr unsigned kKeyMask = 0x1fffffffu;     // block number of a state (32-byte units)
constexpr unsigned kFlagHasEps = 0x80000000u;  // `next` of an arc: the destination has epsilon arcs
constexpr unsigned kFlagEpsIn = 0x40000000u;   //                   an epsilon arc enters the destination
constexpr unsigned kFlagSimple = 0x20000000u;  //                   the destination's only arc is the graph's usual self-loop
                                               // (DevGraph::simple_il, simple_w; no output label): a token there is
                                               // expanded without reading the graph
constexpr unsigned kLoopFirst = 0x80000000u;   // ilabel word of a state's first arc: the state has no epsilon arcs and this arc is
                                               // the usual self-loop (like a simple state's, but other arcs may follow)
constexpr int kLabelMask = 0xffff;             // ... the label itself
constexpr unsigned kArcEps = 0x40000000u;      // arc ids: unit address, plus this bit for epsilon arcs
constexpr unsigned kArcMask = 0x3fffffffu;
constexpr unsigned kPackE = 0xFFFFFu;          // header word 3: emitting degree (20 bits, all ones = see word 2)
constexpr int kPackXShift = 20;                //                epsilon degree (12 bits)
constexpr int kMaxEpsDeg = 4094;
constexpr int kStLattice = WFST_FLAG_LATTICE_OVERFLOW, kStCapacity = WFST_FLAG_CAPACITY;
constexpr int kScratchFrames = 4094;             // most frames a channel may have for wfst_get_lattice_noalloc
constexpr int kHostHead = 24;                    // host staging of the lattice calls: words before the frame offsets
constexpr int kScratchWords = 2 + kScratchFrames + 2;
constexpr int kScratchDevices = 64;

struct ChanState {            // persists between calls (the per-stream decoder state)
  double offset;              // cost offsets: sum of the best costs the token costs were rebased by
  int frame;                  // frames consumed since init
  int n_tok;                  // size of the current closed token set
  int cur;                    // which queue buffer holds it
  int status;                 // sticky WFST_FLAG_* overflow bits
  unsigned lat_used;          // lattice entries in use
  int max_active;
  float beam, scale;          // scale = 256 / beam, computed once on the host
  float sel_ratio;            // candidates taken into recombination per max_active (adaptive)
  int path_frames;            // the traced-path marks of frames 1..path_frames are valid (0: none)
  int boost_n;                // arcs of the channel's boosting acceptor (0 = none); set by the host
  int boost_states;           // its states (1: the paper's one-state acceptor, a table word -> score); set by the host
  int lat_epoch;              // recycled lattice arena: how often the write position has gone back to the start
};

struct DevGraph {
  const int4 *unit;           // state blocks: header {state id, final cost, emitting degree, packed degrees},
                              // epsilon arcs, emitting arcs {next, weight bits, ilabel, olabel}
  unsigned n_blk;             // 32-byte blocks in `unit`
  unsigned start;             // start state: block number + flags, like `next` of an arc
  int has_final;              // 0: every state is final with cost 0
  int S;
  // A token is keyed by (state of the boosting acceptor, graph state): key = (b << blk_bits) | block
  // number, in 29 bits; without an acceptor b = 0 and the key is the block number.
  int blk_bits; unsigned blk_mask;
  // the self-loop that "simple" states have as their only arc (a CTC graph's blank self-loop):
  // the most frequent (ilabel, weight) among states with exactly one arc that is a self-loop
  int simple_il; float simple_w;
  // narrow arc records (an option): for every unit that is an emitting arc, 8 bytes {next, weight as
  // IEEE binary16 << 16 | has-output-label << 12 | ilabel}; the loops over the arcs of states with
  // several arcs read these instead of the 16-byte units.  nullptr: not built.
  const int2 *earc8;
};

struct DevChannels {
  ChanState *st;
  int4 *cand;       int cand_cap, region_cap;  // kRegions x region_cap {next, cost, source token, arc id}
  int4 *win;        int win_cap;               // recombined tokens before the max-active cutoff (their candidate records)
  int2 *queue;      int qcap;                  // 2 buffers {block number, cost}
  int4 *wl;                                    // 2 buffers {token, block number, cost, 1 = new token}
  int2 *lattice;    unsigned lat_cap;          // {prev token, arc id}; lat_cap: entries per channel when shared out equally
  const unsigned long long *lat_start;         // [channels] where the channel's arena begins in `lattice` (and `tokrec`)
  const unsigned *lat_capn;                    // [channels] and how many entries it has
  int recycle;                                 // 1: a channel's arena is a ring over whole frames (streams of any length)
  int *frame_ep;                               // [channels][max_frames + 2] the epoch each frame's tokens were stored in
  int2 *tokrec;                                // nullptr, or beside every backpointer the token's {block number, cost}
  int cost_offset;                             // 1: token costs are rebased to the best cost after every prune step
  int sel_shift;                               // the pre-selection samples one run of 64 candidates out of 2^sel_shift
  // the path of the last traceback, so that the next one can stop where it meets it:
  int *path_tok, *path_nw;                     // [channels][max_frames + 1] per frame: the token the path enters the
                                               // set with (over an emitting arc); words on the path up to and incl. that arc
  int *path_words; int max_words;              // [channels][max_words] its words
  float *frame_best;                           // nullptr, or [channels][max_frames + 1]: the offset every token set was rebased by
  unsigned *frame_off; int max_frames;
  unsigned long long *dig_sum; int *dig_cnt;   // nullptr unless digests are recorded
  long long *counters;                         // [24]: 8 workload counters, 16 phase tick sums
  int *boost_keys; float *boost_vals;          // [channels][kBoostSlots] arcs of the boosting acceptor by output label
  unsigned *boost_from_to;                     //   (key 0 = free slot): score, and from state | to state << 16
};

struct LaunchArgs {
  // device: the launch's lists, n_jobs entries each (the launch may have fewer workgroups): ints
  // [channel id][frames to consume][row in loglikes/outputs][entries of the channel's lattice arena],
  // then the first entry no workgroup has taken yet (starts at the number of workgroups) and a pad,
  // then 64-bit [start of the channel's arena in the lattice pool]
  int *lists; int n_jobs;
  const void *ll; long long ll_stride; int V;   // rows of V elements; fp32, or fp16 / bf16 widened when staged
  int ll_dtype;
  int mode, finalize;
  float beam, scale; int max_active;
  int *words, *nwords; float *cost; int *flags; int max_words;
};

struct EpsLds {               // epsilon expansion: one worklist item per thread, flattened over their arcs
  unsigned pre[kBlock + 1];   // exclusive prefix sums of the items' arc counts
  int abase[kBlock];          // unit address of the item's first arc minus its prefix
  float tcost[kBlock];        // cost of the item's token
  int ttok[kBlock];           // the item's token | its state in the boosting acceptor << 16
};
struct WaveLds {              // ExpandArcs: the work items of one wave (one token per lane)
  unsigned pre[kWaveTok + 1];
  int abase[kWaveTok];
  float tcost[kWaveTok];
  int tb[kWaveTok];           // the token's state in the boosting acceptor (only written when there is one)
  int ttok[kWaveTok];         // the token
  int2 pend[2 * kWaveTok];    // ring: queue records of tokens whose state has to be read from the graph
  int pend_tok[2 * kWaveTok]; //       and which tokens they are
};
struct HubLds {               // ExpandArcs: states with so many arcs that all waves share them
  int first[kHubCap];         // unit address of the first arc to expand
  int deg[kHubCap];           // arcs to expand
  float tcost[kHubCap];
  int ttok[kHubCap];          // token | its state in the boosting acceptor << 16
  int ready[kHubCap];         // set after the entry is written
  int seg_next[kHubCap];      // next segment of kHubSeg arcs nobody has taken yet
};
constexpr int kFilterBits = 1 << 17;           // destinations of a frame's candidates, hashed to one bit each
struct ExpandLds {            // live while arcs are being expanded (and until the first table pass begins)
  float ac[kMaxV];
  WaveLds w[kWaves];
  HubLds hub;
  unsigned filter[kFilterBits / 32];          // bit set: some candidate of the buffer may go to a state with this hash
};
struct TableLds {             // live while candidates are being recombined
  unsigned long long vals[kTabSlots];   // (orderable cost << 32) | candidate index
  int keys[kTabSlots];                  // destination state, kKeyEmpty when free
};
struct Smem {
  union { ExpandLds e; TableLds t; } u;
  EpsLds ek;                  // beside the table: a round's candidates go into the table while its items are
                              // expanded; afterwards the same memory lists the tokens that got better
  unsigned hist[256];
  unsigned hist2[256];        // selection: a sample of the candidates in the buffer
  unsigned hist3[256];        // the self-loop candidates that no candidate of the buffer can meet (exact, all bins)
  float stay_ac;              // this frame's acoustic cost of the simple states' self-loop
  unsigned wave_tot[kWaves];
  unsigned best_ord;
  int n_reg[kRegions];        // candidates per region
  int n_pairs, n_hub, next_run, done_waves;   // improved tokens listed; listed hub states; ExpandArcs run counter; waves done listing
  int n_win, n_next, n_wl_next, status, n_cont;
  int n_in, n_emit, n_back;   // tokens of the emitting step an epsilon arc can enter (they come first), all of them; back counter
  int k_sel, n_sel, n_sel_c, k_keep, redo;
  int overfull;               // a table pass met more destinations than the table takes: the passes are planned again
  int path_frames, trace_from, trace_words;   // traceback: new marks valid up to; where the walk stopped; words before that
  unsigned long long red64, red64b;
  long long ctr[8];
  unsigned short occ[kTabSlots];   // table slot of the candidate at each position of a pass (0xFFFF: not inserted)
  int bk[kBoostSlots]; float bv[kBoostSlots];   // the channel's boosting acceptor, if it has one: per arc its output label,
  unsigned bft[kBoostSlots];                    //   score, and from state | to state << 16
  long long prof[16];         // wall-clock ticks per phase (thread 0)
  long long prof_t0;
  int sel_idx;
  int job;                    // the list entry this workgroup takes next
};

// ------------------------------------------------------------------------------ helpers
// Order-preserving map of float bits to unsigned (negative: all bits flipped, else sign set).
__device__ __forceinline__ unsigned f2ord(float f) {
  const unsigned u = __float_as_uint(f);
  return u ^ ((unsigned)((int)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float ord2f(unsigned o) {
  return __uint_as_float(o ^ ((unsigned)((int)~o >> 31) | 0x80000000u));
}
// -0 becomes +0 (costs are compared by their bits); every other value is unchanged.
__device__ __forceinline__ float canon(float x) { return x + 0.0f; }
__device__ __forceinline__ unsigned hash_state(int s) { return (unsigned)s * 0x9E3779B1u; }
__host__ __device__ inline unsigned boost_slot(int word) { return (((unsigned)word * 0x9E3779B1u) >> 16) & (kBoostSlots - 1); }
__device__ __forceinline__ unsigned long long mix64(unsigned long long x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// Word boosting (paper, Section "Word boosting": the graph composed on the fly with a boosting
// acceptor B): a token in state b of B takes an arc with output label `word` (never 0).  Returns
// the score to add (0 if none) and sets nb to the token's new state in B.
__device__ __forceinline__ float boost_step(const Smem &sm, int b, int word, int &nb);

// Values read from LDS or global memory that are the same in every lane: tell the compiler,
// so that they live in scalar registers and control flow on them is scalar.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned uni(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ float uni(float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); }
__device__ __forceinline__ unsigned long long uni64(unsigned long long v) {
  return ((unsigned long long)uni((unsigned)(v >> 32)) << 32) | uni((unsigned)v);
}
__device__ __forceinline__ double uni(double v) {
  const long long b = __double_as_longlong(v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(b & 0xffffffffll));
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// 16 bytes at byte 12 of a state block: {packed degrees, first unit's next, weight, ilabel}
// (4-byte aligned; one global_load_dwordx4).
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef v4i_t __attribute__((aligned(4))) v4i_unaligned_t;
__device__ __forceinline__ int4 load_block_head(const int4 *unit, int key) {
  const v4i_t q = *reinterpret_cast<const v4i_unaligned_t *>(reinterpret_cast<const char *>(unit + 2 * (size_t)(unsigned)key) + 12);
  return make_int4(q.x, q.y, q.z, q.w);
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive adds: four
// shifts inside each row of 16 lanes, then the last lane of row 0 (2) onto row 1 (3) and lane
// 31 onto rows 2 and 3.  Six vector instructions, no LDS traffic.
__device__ __forceinline__ unsigned wave_scan_add(unsigned v) {
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31
  return v;
}
// Minimum over the 64 lanes (same data-parallel steps; lanes shifted in from outside hold ~0).
__device__ __forceinline__ unsigned wave_min(unsigned v) {
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x111, 0xf, 0xf, false));
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x112, 0xf, 0xf, false));
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x114, 0xf, 0xf, false));
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x118, 0xf, 0xf, false));
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x142, 0xa, 0xf, false));
  v = min(v, (unsigned)__builtin_amdgcn_update_dpp(-1, (int)v, 0x143, 0xc, 0xf, false));
  return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ unsigned wave_sum(unsigned v) {
  return (unsigned)__builtin_amdgcn_readlane((int)wave_scan_add(v), 63);
}

// (Per-lane predicates travel as int arrays: bool arrays get packed into bytes of one register.)
// Indices from an LDS counter for every (lane, u) with pred[u] set: ONE LDS atomic per wave,
// and the lanes of a wave get consecutive indices, so their stores coalesce.  Must be called
// by all 64 lanes of the wave (every call site is inside block-uniform control flow).
template <int N>
__device__ __forceinline__ void wave_alloc_n(int *counter, const int (&pred)[N], int (&idx)[N]) {
  const int lane = threadIdx.x & 63;
  const unsigned long long lt = (1ull << lane) - 1ull;
  unsigned long long m[N]; int off[N], tot = 0;
#pragma unroll
  for (int u = 0; u < N; ++u) { m[u] = __ballot(pred[u]); off[u] = tot; tot += __popcll(m[u]); }
  int base = 0;
  if (lane == 0 && tot) base = atomicAdd(counter, tot);
  base = uni(base);
#pragma unroll
  for (int u = 0; u < N; ++u) idx[u] = pred[u] ? base + off[u] + __popcll(m[u] & lt) : -1;
}

struct Cutoff {
  float best, beam, scale; int k_keep;
  __device__ __forceinline__ int bin(float c) const {
    if (beam == 0.0f) return 0;
    // clamp to [0, 255] without branches; a NaN (inf - inf) lands in bin 0 like every x <= 0
    return (int)fminf(fmaxf(floorf((c - best) * scale), 0.0f), 255.0f);
  }
  __device__ __forceinline__ bool in_beam(float c) const { return (c - best) <= beam; }
  __device__ __forceinline__ bool keep(float c) const { return (int)in_beam(c) & (int)(bin(c) < k_keep); }
};

struct Ctx {                  // block-uniform view of one channel
  const DevGraph &g; const DevChannels &c; Smem &sm;
  int4 *cand; int4 *win;
  int2 *q0; int4 *wl0; int2 *lat; unsigned *frame_off;   // q0/wl0: two buffers of qcap
  unsigned long long *dig_sum; int *dig_cnt;
  ChanState s;
  const int2 *srcq;           // the queue the candidates' source tokens are in (ties between two takes of one arc)
  unsigned lat_cap;           // entries of the channel's lattice arena
  int prof;                   // phase timing is on (a debug hook: reading the clock stalls wave 0 at every mark)
};
// workload counters of this launch, kept in LDS (thread 0 adds the block-uniform ones)
enum { kCtTok = 0, kCtEarc, kCtXarc, kCtKept, kCtStored, kCtMaxAct, kCtBin0, kCtFrames };

// B's arcs are hashed by output label; arcs with the same label (out of different states of B)
// follow each other in the probe sequence.  If state b has an arc on the label, that arc is taken;
// otherwise B's failure arc leads to the root (state 0) at no cost and the label is tried once
// more there: the root's arc on it if there is one, else the token stays in the root and nothing
// is added.  One walk finds both candidates.  With the one-state acceptor of the paper (b is always
// 0) this is the lookup of the word's score in a table.
__device__ __forceinline__ float boost_step(const Smem &sm, int b, int word, int &nb) {
  unsigned h = boost_slot(word);
  float root_score = 0.0f; int root_to = 0;
  for (;;) {
    const int k = sm.bk[h];
    if (k == 0) break;                       // the table is never full (kBoostMax < kBoostSlots)
    if (k == word) {
      const unsigned ft = sm.bft[h];
      const int from = (int)(ft & 0xffffu);
      if (from == b) { nb = (int)(ft >> 16); return sm.bv[h]; }
      if (from == 0) { root_to = (int)(ft >> 16); root_score = sm.bv[h]; }
    }
    h = (h + 1) & (kBoostSlots - 1);
  }
  nb = root_to;
  return root_score;
}

// Phase timing with the constant-rate wall clock (thread 0 only; a few scalar reads per frame).
enum { kPhExpand = 0, kPhSelect, kPhCutoff, kPhEpsExpand, kPhEpsRecombine, kPhFinish, kPhTrace, kPhOther,
       kPhTabClear, kPhTabFill, kPhTabScan, kPhEpsTabFill, kPhEpsTabScan, kPhExpSetup, kPhEpsMeet };
constexpr int kPhStayMeet = kPhTabFill;          // counted with the table fill
__device__ __forceinline__ void prof_mark(const Ctx &x, int phase) {
  if (x.prof && threadIdx.x == 0) {
    const long long now = (long long)wall_clock64();
    x.sm.prof[phase] += now - x.sm.prof_t0;
    x.sm.prof_t0 = now;
  }
}


// Block-wide exclusive scan of N values per thread (thread t owns items N*t ..).
// Returns the total; ex[k] receives the exclusive prefix of the thread's k-th item.
template <int N>
__device__ __forceinline__ unsigned block_scan(Smem &sm, const unsigned (&d)[N], unsigned (&ex)[N]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned s = 0;
#pragma unroll
  for (int k = 0; k < N; ++k) s += d[k];
  const unsigned inc = wave_scan_add(s);
  if (lane == 63) sm.wave_tot[wave] = inc;
  __syncthreads();
  unsigned base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    unsigned t = sm.wave_tot[w];
    if (w < wave) base += t;
    total += t;
  }
  unsigned run = base + inc - s;
#pragma unroll
  for (int k = 0; k < N; ++k) { ex[k] = run; run += d[k]; }
  return uni(total);
}

// The same over a table of exactly kWaveTok items: one compare and one select per step.
__device__ __forceinline__ int wave_owner_of(const unsigned *pre, unsigned f) {
  int j = 0;
#pragma unroll
  for (int step = kWaveTok / 2; step >= 1; step >>= 1)
    if (pre[j + step] <= f) j += step;
  return j;
}

// Which of n work items owns flattened arc f: last j < n with pre[j] <= f (pre[0] = 0).
__device__ __forceinline__ int owner_of(const unsigned *pre, int n, unsigned f) {
  int lo = 0, hi = n;
  const int steps = 32 - __clz(max(n, 1) - 1 | 0);              // ceil(log2(n)), uniform
  for (int it = 0; it < steps; ++it) {
    const int mid = (lo + hi) >> 1;
    if (pre[mid] <= f) lo = mid; else hi = mid;
  }
  return lo;
}

// Owners of the N arcs a lane handles in one step of a block-wide flattened loop: arc u of
// the lane is f0 + u*kBlock + tid, so the 64 lanes of a wave hold 64 consecutive arcs for
// every u.  One full search per wave (2N lanes look up the owners of the first and last arc
// of each run of 64) bounds every lane's own search to the few items its run spans: 0 steps
// inside a high-degree state, a few where degrees are small.
template <int N>
__device__ __forceinline__ void owners_of(const unsigned *pre, int n, unsigned f0, unsigned M, int (&ok)[N], int (&j)[N]) {
  static_assert(2 * N <= 64, "bounds are looked up by 2N lanes");
  const int lane = threadIdx.x & 63;
  const unsigned wave_f = f0 + (threadIdx.x & ~63u);
  unsigned fq = wave_f + (unsigned)(lane >> 1) * kBlock + ((lane & 1) ? 63u : 0u);
  if (lane >= 2 * N || fq >= M) fq = M - 1;
  const int bound = owner_of(pre, n, fq);
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const unsigned f = f0 + u * kBlock + threadIdx.x;
    ok[u] = f < M;
    int lo = __builtin_amdgcn_readlane(bound, 2 * u), hi = __builtin_amdgcn_readlane(bound, 2 * u + 1) + 1;
    const int steps = 32 - __clz(max(hi - lo, 1) - 1 | 0);      // ceil(log2(width)), 0 for width 1
    const unsigned fs = ok[u] ? f : M - 1;
    for (int it = 0; it < steps; ++it) {
      const int mid = (lo + hi) >> 1;
      if (pre[mid] <= fs) lo = mid; else hi = mid;
    }
    j[u] = lo;
  }
}

// Region of the candidate buffer a destination state belongs to (top hash bits).
__device__ __forceinline__ int key_of(int next) { return (int)((unsigned)next & kKeyMask); }
__device__ __forceinline__ int region_of(int key) { return (int)(hash_state(key) >> (32 - kRegionBits)); }

// Append a batch of N candidates per lane to their destinations' regions.  The wave counts
// its candidates per region with ballots, lane 0 reserves one run per region (kRegions
// independent LDS atomics), and every candidate gets a slot in its region's run; lanes
// that hit the same region write consecutive 16-byte records, so the stores coalesce.
// Must be called by all 64 lanes of the wave.
__device__ __forceinline__ unsigned filter_bit(int key) { return (hash_state(key) >> 9) & (kFilterBits - 1); }

template <int N, bool kFilter = false>
__device__ __forceinline__ void push_cands(Ctx &x, const int (&ok)[N], const int (&next)[N], const float (&nc)[N],
                                           const int (&src)[N], const int (&arc)[N]) {
  const int cap = x.c.region_cap;
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const int r = region_of(key_of(next[u]));
    if (ok[u]) {
      if (kFilter) {                           // emitting step: the destination's bit, for the tokens that stay put
        const unsigned fb = filter_bit(key_of(next[u]));
        atomicOr(&x.sm.u.e.filter[fb >> 5], 1u << (fb & 31));
      }
      // one LDS atomic instruction for the whole wave: the hardware serialises the lanes of a
      // region and hands them consecutive slots, in far fewer issue slots than ballots would take
      const int slot = atomicAdd(&x.sm.n_reg[r], 1);
      if (slot < cap) x.cand[r * cap + slot] = make_int4(next[u], __float_as_int(nc[u]), src[u], arc[u]);
      else atomicOr(&x.sm.status, kStCapacity);
    }
  }
}

// Two bit sets over the tokens of the current set live in the closure's item tables, which are idle
// between the end of one frame's closure and the next: bit i of `staybits`: token i's implied
// self-loop candidate is the recombined token of its state; bit i of `hasstay`: token i is in a
// state with other arcs whose first arc is the usual self-loop (set while arcs are expanded).
__device__ __forceinline__ unsigned *staybits_of(Smem &sm) { return reinterpret_cast<unsigned *>(&sm.ek); }
__device__ __forceinline__ unsigned *hasstay_bits(Smem &sm) { return reinterpret_cast<unsigned *>(&sm.ek) + kQueueMax / 32; }
static_assert(sizeof(EpsLds) >= 2 * (kQueueMax / 8), "two bits per token of the set");

// Cost of the self-loop candidate of a token (cost c) in a simple state, in the association of
// every emitting arc: (c + w) + acoustic cost.
__device__ __forceinline__ float stay_cost(const Ctx &x, float c) { return canon((c + x.g.simple_w) + x.sm.stay_ac); }

// ------------------------------------------------------------------ ExpandArcs (emitting)
// For every token of the current set and every emitting arc:
//   cost = (token cost + arc weight) + (-loglike[ilabel-1])      (Expand Arcs pseudo-code)
// Candidates that cannot be in the beam relative to the running best are dropped early;
// the running best is never lower than the final one, so this never drops a survivor.
// Cost, beam test and append for N emitting arcs per lane (all 64 lanes of the wave call it).
template <int N>
__device__ __forceinline__ void emit_arcs(Ctx &x, int (&ok)[N], const int4 (&a)[N], const float (&tc)[N],
                                          const int (&src)[N], const int (&arc)[N], const int (&tb)[N],
                                          float beam, bool boosted) {
  Smem &sm = x.sm;
  const unsigned bo = __hip_atomic_load(&sm.best_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const float rb = bo == kOrdNone ? INFINITY : ord2f(bo);
  unsigned o = kOrdNone;
  float nc[N]; int next[N];
#pragma unroll
  for (int u = 0; u < N; ++u) {
    nc[u] = canon((tc[u] + __int_as_float(a[u].y)) + sm.u.e.ac[a[u].z - 1]);
    next[u] = a[u].x;
    if (boosted) {                             // the destination's key carries the token's state in B
      int nb = tb[u];
      if (a[u].w != 0 && ok[u]) nc[u] = canon(nc[u] + boost_step(sm, tb[u], a[u].w, nb));   // + B's score
      next[u] |= nb << x.g.blk_bits;
    }
    // predicates are combined with & and selects: no short-circuit branches in the hot loop
    ok[u] &= (int)(nc[u] < INFINITY) & (int)!((nc[u] - rb) > beam);
    o = min(o, ok[u] ? f2ord(nc[u]) : kOrdNone);
  }
  // running best: lowered by one lane, and only if some lane of the wave has a lower cost
  // (rare after the first arcs)
  if (__ballot(o < bo) != 0ull) {
    const unsigned m = wave_min(o);
    if ((threadIdx.x & 63) == 0) atomicMin(&sm.best_ord, m);
  }
  push_cands<N, true>(x, ok, next, nc, src, arc);
}

// An emitting arc {next, weight, ilabel, olabel} by its unit address: from the narrow records if
// the graph has them (8 bytes instead of 16; the output label, which only boosting looks at here,
// is then fetched from the full record of the few arcs that have one).
template <bool kNarrow>
__device__ __forceinline__ int4 load_emitting_arc(const DevGraph &g, int arc, bool want_olabel) {
  if (!kNarrow) return g.unit[arc];
  const int2 e = g.earc8[arc];
  const float w = (float)__builtin_bit_cast(_Float16, (unsigned short)((unsigned)e.y >> 16));
  int ol = 0;
  if (want_olabel && ((unsigned)e.y & 0x1000u)) ol = g.unit[arc].w;
  return make_int4(e.x, __float_as_int(w), (int)((unsigned)e.y & 0xfffu), ol);
}

// One step of a wave's flattened loop: arcs f0 + u*64 + lane of its listed work items.
template <int N, bool kNarrow>
__device__ __forceinline__ void wave_arcs(Ctx &x, const WaveLds &wl, unsigned f0, unsigned M, float beam, bool boosted) {
  const int lane = threadIdx.x & 63;
  int ok[N]; int src[N]; int4 a[N]; int arc[N]; float tc[N]; int tb[N];
#pragma unroll
  for (int u = 0; u < N; ++u) {                // arc fetch, N in flight
    const unsigned f = f0 + u * 64 + lane;
    ok[u] = f < M;
    const unsigned fs = ok[u] ? f : M - 1;       // lanes past the end repeat the last arc (no branch)
    const int j = wave_owner_of(wl.pre, fs);
    arc[u] = wl.abase[j] + (int)fs;
    src[u] = wl.ttok[j];
    tc[u] = wl.tcost[j];
    tb[u] = boosted ? wl.tb[j] : 0;
    a[u] = load_emitting_arc<kNarrow>(x.g, arc[u], boosted);
  }
  emit_arcs<N>(x, ok, a, tc, src, arc, tb, beam, boosted);
}

// Arcs [f0, f0 + 64N) of one listed high-degree state (all lanes of the wave call it).
template <int N, bool kNarrow>
__device__ __forceinline__ void hub_arcs(Ctx &x, int first, int deg, float cost, int tok, int f0, float beam, bool boosted) {
  const int lane = threadIdx.x & 63;
  int ok[N], src[N], arc[N], tb[N]; int4 a[N]; float tc[N];
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const int f = f0 + u * 64 + lane;
    ok[u] = f < deg;
    arc[u] = first + (ok[u] ? f : deg - 1);      // lanes past the end repeat the last arc (no branch)
    src[u] = tok & 0xffff; tb[u] = (int)((unsigned)tok >> 16); tc[u] = cost;
    a[u] = load_emitting_arc<kNarrow>(x.g, arc[u], boosted);
  }
  emit_arcs<N>(x, ok, a, tc, src, arc, tb, beam, boosted);
}

// Next run of kWaveTok tokens for this wave (a block-wide counter in LDS; wave-uniform).
__device__ __forceinline__ int next_run(Smem &sm) {
  int r = 0;
  if ((threadIdx.x & 63) == 0) r = atomicAdd(&sm.next_run, 1);
  return uni(r);
}

// The tokens of one wave's list whose state block has to be read: n <= 64 of them, starting at
// `head` of the wave's ring.  A lane reads the 32 bytes at the start of its token's block
// (header + first arc): the first arc is expanded right away by the lane that owns the token, the
// remaining arcs of the batch are flattened over the 64 lanes (prefix sums in the wave's slice of
// LDS, one short search per arc), and states with more than kHubDeg arcs are listed for all waves.
// Returns the emitting arcs expanded (wave-uniform).  All 64 lanes call it.
template <bool kNarrow>
__device__ __forceinline__ unsigned dense_run(Ctx &x, WaveLds &wl, int head, int n, float beam, bool boosted) {
  Smem &sm = x.sm;
  HubLds &hb = sm.u.e.hub;
  const int lane = threadIdx.x & 63;
  const unsigned bm = x.g.blk_mask; const int bbits = x.g.blk_bits;
  const bool valid = lane < n;
  const int at = (head + lane) & (2 * kWaveTok - 1);
  const int2 tk = valid ? wl.pend[at] : make_int2(0, 0);
  const int tok = valid ? wl.pend_tok[at] : 0;
  const int blk = (int)((unsigned)tk.x & bm);
  int4 hd = make_int4(0, 0, 0, 1);                       // no arcs; ilabel 1 keeps the acoustic lookup in range
  if (valid) hd = load_block_head(x.g.unit, blk);
  unsigned n_arcs = 0, deg; int first;
  {
    int has[1], src[1], arc[1], tb[1]; float tc[1]; int4 a0[1];
    tb[0] = (int)(((unsigned)tk.x & kKeyMask) >> bbits);  // 0 without a boosting acceptor
    int ne = (int)((unsigned)hd.x & kPackE); const int nx = (int)((unsigned)hd.x >> kPackXShift);
    if (ne == (int)kPackE) ne = x.g.unit[2 * (size_t)(unsigned)blk].z;        // a very large state: exact degree
    has[0] = (int)(ne > 0) & (int)(nx == 0);            // the unit after the header is an emitting arc
    deg = (unsigned)(ne - has[0]);
    first = 2 * blk + 1 + nx + has[0];                  // unit address of the first arc left
    tc[0] = __int_as_float(tk.y); src[0] = tok; arc[0] = 2 * blk + 1;
    a0[0] = make_int4(hd.y, hd.z, has[0] ? (hd.w & kLabelMask) : 1, 0);
    n_arcs += (unsigned)__popcll(__ballot(has[0]));
    {
      // The first arc is the usual self-loop: its candidate is not made here.  Like the one of a
      // token in a simple state it is implied by the token's queue record (the bit set `hasstay`
      // says for which tokens); here it only lowers the running best.
      const int loop = has[0] & (int)((unsigned)hd.w >> 31);
      const float nc = stay_cost(x, tc[0]);
      const unsigned bo = __hip_atomic_load(&sm.best_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      const unsigned o = (loop && nc < INFINITY) ? f2ord(nc) : kOrdNone;
      if (__ballot(o < bo) != 0ull) {
        const unsigned mo = wave_min(o);
        if (lane == 0) atomicMin(&sm.best_ord, mo);
      }
      if (loop) atomicOr(&hasstay_bits(sm)[tok >> 5], 1u << (tok & 31));
      has[0] &= (int)!loop;
    }
    if (boosted && has[0]) a0[0].w = x.g.unit[2 * (size_t)(unsigned)blk + 1].w;    // the first arc's olabel
    if (deg > (unsigned)kHubDeg) {                      // to the shared list, if it has room
      const int h = atomicAdd(&sm.n_hub, 1);
      if (h < kHubCap) {
        hb.first[h] = first; hb.deg[h] = (int)deg; hb.tcost[h] = tc[0]; hb.ttok[h] = src[0] | (tb[0] << 16);
        __hip_atomic_store(&hb.ready[h], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        deg = 0;
      }
    }
    emit_arcs<1>(x, has, a0, tc, src, arc, tb, beam, boosted);
    if (boosted) wl.tb[lane] = tb[0];
  }
  // exclusive prefix sums of the batch's arc counts (item j = lane)
  const unsigned inc = wave_scan_add(deg);
  const unsigned M = (unsigned)__builtin_amdgcn_readlane((int)inc, 63);
  wl.pre[lane] = inc - deg;
  wl.abase[lane] = first - (int)(inc - deg);
  wl.tcost[lane] = __int_as_float(tk.y);
  wl.ttok[lane] = tok;
  if (lane == 0) wl.pre[kWaveTok] = M;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  n_arcs += M;
  // 64 * kUE arcs per step; a short rest takes the cheaper single-arc step
  unsigned f0 = 0;
  for (; f0 + 64 < M; f0 += 64 * kUE) wave_arcs<kUE, kNarrow>(x, wl, f0, M, beam, boosted);
  if (f0 < M) wave_arcs<1, kNarrow>(x, wl, f0, M, beam, boosted);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  return n_arcs;
}

// On entry sm.next_run == kWaves, sm.done_waves == 0, sm.n_hub == 0 and the hub list's ready
// and seg_next words are zero (the caller sets them before its barrier).
template <bool kNarrow, bool kBoost>
__device__ __forceinline__ void emit_expand(Ctx &x, const int2 *Q, int n_tok) {
  Smem &sm = x.sm;
  ExpandLds &e = sm.u.e;
  HubLds &hb = e.hub;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float beam = x.s.beam;
  const bool boosted = kBoost && x.s.boost_n > 0;
  // Every wave expands runs of kWaveTok tokens at its own pace: it takes the next run from a
  // counter, so no wave waits for another until all tokens are done, and one wave's loads
  // overlap another's arithmetic.  Most tokens sit in "simple" states, whose only arc is the
  // graph's usual self-loop (the queue record says so): their one candidate is made from the
  // token alone, with no graph read at all.  The other tokens of the run go into the wave's
  // list, and whenever 64 of them have come together the wave expands them as one dense batch
  // (dense_run), so that the graph reads and their latency are paid once per 64 such tokens and
  // not once per run.  States with more than kHubDeg arcs are listed instead; when a wave finds
  // no run left it takes segments of listed states until those are done too.  Queue records are
  // loaded two runs ahead.
  static_assert(kWaveTok == 64, "one token per lane");
  WaveLds &wl = e.w[wave];
  const int R = (n_tok + kWaveTok - 1) / kWaveTok;
  int r = wave, rn = next_run(sm);
  const unsigned long long lt = (1ull << lane) - 1ull;
  int2 tk = make_int2(0, 0), tkn = make_int2(0, 0);
  if (r * kWaveTok + lane < n_tok) tk = Q[r * kWaveTok + lane];
  if (rn < R && rn * kWaveTok + lane < n_tok) tkn = Q[rn * kWaveTok + lane];
  int pend_head = 0, pend_n = 0;                       // wave-uniform: the list is ring entries [head, head + n)
  unsigned long long n_arcs = 0;                       // wave-uniform: emitting arcs this wave expanded
  while (r < R) {
    const int base = r * kWaveTok;
    const bool valid = base + lane < n_tok;
    {
      // The self-loop candidate of a token in a simple state is never written anywhere: it is
      // (the token's own key, stay_cost(token cost)) and is made again from the queue record
      // wherever it is needed (selection, recombination, token creation).  Here it only lowers
      // the running best.
      const bool simple = valid && ((unsigned)tk.x & kFlagSimple) != 0;
      const float nc = stay_cost(x, __int_as_float(tk.y));
      const unsigned bo = __hip_atomic_load(&sm.best_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      const unsigned o = (simple && nc < INFINITY) ? f2ord(nc) : kOrdNone;
      if (__ballot(o < bo) != 0ull) {
        const unsigned mo = wave_min(o);
        if (lane == 0) atomicMin(&sm.best_ord, mo);
      }
      n_arcs += (unsigned)__popcll(__ballot(simple));
      const bool other = valid && !simple;
      const unsigned long long m = __ballot(other);
      if (other) {
        const int at = (pend_head + pend_n + __popcll(m & lt)) & (2 * kWaveTok - 1);
        wl.pend[at] = tk; wl.pend_tok[at] = base + lane;
      }
      pend_n += __popcll(m);
    }
    // the queue records of the run after the next
    const int rnn = next_run(sm);
    tk = tkn;
    tkn = make_int2(0, 0);
    if (rnn < R && rnn * kWaveTok + lane < n_tok) tkn = Q[rnn * kWaveTok + lane];
    r = rn; rn = rnn;
    if (pend_n >= kWaveTok) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      n_arcs += dense_run<kNarrow>(x, wl, pend_head, kWaveTok, beam, boosted);
      pend_head = (pend_head + kWaveTok) & (2 * kWaveTok - 1); pend_n -= kWaveTok;
    }
  }
  if (pend_n > 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    n_arcs += dense_run<kNarrow>(x, wl, pend_head, pend_n, beam, boosted);
  }
  // this wave lists no more states
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  if (lane == 0) atomicAdd(&sm.done_waves, 1);
  // ---- listed states, a segment at a time, until every wave is done listing and none is left
  {
    int h = 0, spins = 0;
    while (h < kHubCap) {
      int ready = uni(__hip_atomic_load(&hb.ready[h], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
      if (!ready) {
        const int done = uni(__hip_atomic_load(&sm.done_waves, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
        if (done == kWaves) {                           // nobody lists any more: is the entry really absent?
          ready = uni(__hip_atomic_load(&hb.ready[h], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
          if (!ready) break;
        } else {
          if (++spins > (1 << 22)) { if (lane == 0) atomicOr(&sm.status, kStCapacity); break; }   // never expected
          __builtin_amdgcn_s_sleep(4);
          continue;
        }
      }
      int seg = 0;
      if (lane == 0) seg = atomicAdd(&hb.seg_next[h], 1);
      seg = uni(seg);
      const int deg = uni(hb.deg[h]);
      const int f0 = seg * kHubSeg;
      if (f0 >= deg) { ++h; continue; }
      const int first = uni(hb.first[h]), tok = uni(hb.ttok[h]); const float cost = uni(hb.tcost[h]);
      if (deg - f0 > 64) hub_arcs<kUE, kNarrow>(x, first, deg, cost, tok, f0, beam, boosted);
      else hub_arcs<1, kNarrow>(x, first, deg, cost, tok, f0, beam, boosted);
      n_arcs += (unsigned)min(kHubSeg, deg - f0);
    }
  }
  if (lane == 0 && n_arcs) atomicAdd((unsigned long long *)&sm.ctr[kCtEarc], n_arcs);
  __syncthreads();
  prof_mark(x, kPhExpSetup);
}

// ------------------------------------------------------------------ recombination in LDS
// Probe sequence of a key in the LDS table: double hashing (an odd step from other hash bits visits
// every slot of the power-of-two table).  At the loads the passes run at, an insert then takes
// about half the probes of linear probing, and every probe is an LDS round trip.
#ifndef WFST_STEP_SHIFT
#define WFST_STEP_SHIFT 19
#endif
constexpr int kProbeLimit = 256;
__device__ __forceinline__ unsigned probe_start(int key) { return (hash_state(key) >> 6) & kTabMask; }
__device__ __forceinline__ unsigned probe_step(int key) {
#ifdef WFST_LINEAR
  return 1u;
#else
  return ((hash_state(key) >> WFST_STEP_SHIFT) | 1u) & kTabMask;
#endif
}

// Lower the destination's table entry to this candidate if (cost, arc id) is smaller.
// The value word carries the candidate's index, so the winner's record can be fetched
// afterwards; exact cost ties are decided by the arc ids of the two records.
// With a boosting acceptor two tokens of one graph state can take the same arc into the same
// (graph state, B state) pair; then the lower B state of the source token wins (src = its index).
__device__ __forceinline__ int table_insert(Ctx &x, int dst, float cost, int arc, int src, int idx) {
  TableLds &t = x.sm.u.t;
  unsigned s = probe_start(dst);
  const unsigned step = probe_step(dst);
  // one compare-and-swap per probe: it returns the slot's key, or claims the slot if it was free
  int old;
  for (int probes = 0;; ++probes) {
    old = atomicCAS(&t.keys[s], kKeyEmpty, dst);
    if (old == kKeyEmpty || old == dst) break;
    s = (s + step) & kTabMask;
    if (probes >= kProbeLimit) { old = kKeyNone; break; }
  }
  // a probe sequence this long means that the pass has far more destinations than it was planned
  // for (at the loads passes are planned for, 0.75, one in 10^30 gets here): the caller plans again.
  // (Leaving the loop first and returning here compiles to a faster loop than returning inside it.)
  if (old == kKeyNone) { atomicOr(&x.sm.overfull, 1); return -1; }
  const unsigned oc = f2ord(cost);
  const unsigned long long mine = ((unsigned long long)oc << 32) | (unsigned)idx;
  // a slot this lane has just claimed still holds the empty value (unless another candidate of
  // the same destination was quicker: then the swap below fails once and returns that value)
  unsigned long long cur = kValEmpty;
  if (old != kKeyEmpty) cur = t.vals[s];
  for (;;) {
    const unsigned cc = (unsigned)(cur >> 32);
    bool better = oc < cc;
    if (oc == cc && cur != kValEmpty) {
      // exact tie: lower arc id.  The other record may have been written by another wave just
      // before it published the index (fused closure rounds): acquire pairs with its release
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      const int4 other = x.cand[(unsigned)cur];
      better = (unsigned)arc < (unsigned)other.w;
      if (arc == other.w) better = (unsigned)x.srcq[src].x < (unsigned)x.srcq[other.z].x;   // same graph state: the keys order like the B states
    }
    if (!better) break;
    const unsigned long long prev = atomicCAS(&t.vals[s], cur, mine);
    if (prev == cur) break;
    cur = prev;
  }
  return (int)s;
}

__device__ __forceinline__ void table_clear(Smem &sm) {
  for (int s = threadIdx.x; s < kTabSlots; s += kBlock) { sm.u.t.vals[s] = kValEmpty; sm.u.t.keys[s] = kKeyEmpty; }
}

// Sub-group of a destination state when one region is reduced in G table passes.
__device__ __forceinline__ int group_of(int dst, int G) {
  // the 11 hash bits below the region's, scaled to [0, G)
  return (int)((((hash_state(dst) >> (21 - kRegionBits)) & 0x7ffu) * (unsigned)G) >> 11);
}

// One table pass over regions [r0, r1): every candidate of sub-group g (of G) that is selected
// (inside the beam, cost bin below k_sel) is inserted.  Reads are coalesced 16-byte records.
// The slot every candidate of the pass went to is noted in LDS (sm.occ, by the candidate's
// position in the pass, 0xFFFF = not inserted) for the first kTabSlots positions, so that the
// second sweep finds it without probing again.
template <bool kSelect>
__device__ __forceinline__ void table_fill(Ctx &x, int r0, int r1, int g, int G, const Cutoff &cut, int k_sel) {
  const int tid = threadIdx.x;
  int pos0 = 0;                               // position of the region's first candidate in this pass
  for (int r = r0; r < r1; ++r) {
    const int n = uni(min(x.sm.n_reg[r], x.c.region_cap));
    const int base = r * x.c.region_cap;
    // software pipeline: the next record is in flight while this one goes into the table
    int4 nxt = make_int4(-1, 0, 0, 0);
    if (tid < n) nxt = x.cand[base + tid];
    for (int i = tid; i < n; i += kBlock) {
      const int4 cd = nxt;
      if (i + kBlock < n) nxt = x.cand[base + i + kBlock];
      const float c = __int_as_float(cd.y);
      const int key = key_of(cd.x);
      int take = (int)(G == 1) | (int)(group_of(key, G) == g);
      if (kSelect) take &= (int)cut.in_beam(c) & (int)(cut.bin(c) < k_sel);
      int slot = -1;
      if (take) slot = table_insert(x, key, c, cd.w, cd.z, base + i);
      if (pos0 + i < kTabSlots) x.sm.occ[pos0 + i] = (unsigned short)slot;
    }
    pos0 += (n + kBlock - 1) / kBlock * kBlock;
  }
}

// Slot that candidate `idx` (position `pos` of the pass) was inserted into, or -1.  Positions
// beyond the noted ones repeat the fill's test and probe for the key.
template <bool kSelect>
__device__ __forceinline__ int slot_of_candidate(Ctx &x, int pos, int idx, int g, int G, const Cutoff &cut, int k_sel) {
  TableLds &t = x.sm.u.t;
  if (pos < kTabSlots) {
    const unsigned short sl = x.sm.occ[pos];
    return sl == 0xFFFFu ? -1 : (int)sl;
  }
  const int4 cd = x.cand[idx];
  const float c = __int_as_float(cd.y);
  const int key = key_of(cd.x);
  int take = (int)(G == 1) | (int)(group_of(key, G) == g);
  if (kSelect) take &= (int)cut.in_beam(c) & (int)(cut.bin(c) < k_sel);
  if (!take) return -1;
  unsigned s = probe_start(key);
  const unsigned step = probe_step(key);
  int probes = 0;
  while (t.keys[s] != key && probes < kTabSlots) { s = (s + step) & kTabMask; ++probes; }
  return probes < kTabSlots ? (int)s : -1;
}

// Second sweep of a table pass: every candidate that was inserted looks at its slot again;
// the one whose index is still in the value word is the recombined token of that
// destination.  It is histogrammed and its record is appended to the winners (winners of
// neighbouring lanes are neighbouring records, so the reads coalesce, and nobody has to scan
// the table or fetch records by index afterwards).  Candidates beyond the noted positions
// (more than kTabSlots in one pass) find their slot by probing again.
template <bool kSelect>
__device__ __forceinline__ void table_winners(Ctx &x, int r0, int r1, int g, int G, const Cutoff &cut, int k_sel) {
  TableLds &t = x.sm.u.t;
  const int tid = threadIdx.x;
  constexpr int kW = 2;
  int pos0 = 0;
  for (int r = r0; r < r1; ++r) {
    const int n = uni(min(x.sm.n_reg[r], x.c.region_cap));
    const int base = r * x.c.region_cap;
    for (int i0 = 0; i0 < n; i0 += kBlock * kW) {
      int win[kW], wi[kW]; unsigned long long v[kW];
#pragma unroll
      for (int u = 0; u < kW; ++u) {
        const int i = i0 + u * kBlock + tid;
        int slot = -1;
        if (i < n) slot = slot_of_candidate<kSelect>(x, pos0 + i, base + i, g, G, cut, k_sel);
        v[u] = slot >= 0 ? t.vals[slot] : kValEmpty;
        win[u] = (int)(slot >= 0) & (int)((unsigned)v[u] == (unsigned)(base + i));
        if (win[u]) atomicAdd(&x.sm.hist[cut.bin(ord2f((unsigned)(v[u] >> 32)))], 1u);
      }
      wave_alloc_n<kW>(&x.sm.n_win, win, wi);
#pragma unroll
      for (int u = 0; u < kW; ++u)
        if (win[u]) {
          const int i = i0 + u * kBlock + tid;
          if (wi[u] < x.c.win_cap) x.win[wi[u]] = x.cand[base + i];
          else atomicOr(&x.sm.status, kStCapacity);
        }
    }
    pos0 += (n + kBlock - 1) / kBlock * kBlock;
  }
}

// Tokens in simple states whose self-loop candidate may meet a candidate of the buffer (their
// key's filter bit was set) were listed as {token, queue record}: they look their key up in the
// table of the pass that covers it.  If the table has an entry for the key, the better of the two
// (cost, then arc id) remains: when it is the self-loop, the entry's candidate index is replaced
// by one that no candidate has, so that the winners' sweep finds no winner there.  A self-loop
// candidate that is the best of its key is histogrammed and marked in staybits.  Every listed
// token meets exactly one pass.
__device__ __forceinline__ void stay_meet(Ctx &x, const int4 *CL, int n_cont, unsigned *staybits,
                                          int r0, int r1, int g, int G, const Cutoff &cut, int k_sel) {
  TableLds &t = x.sm.u.t;
  constexpr unsigned kIdxStay = 0xFFFFFFFFu;
  for (int e = threadIdx.x; e < n_cont; e += kBlock) {
    const int4 c = CL[e];                        // {token, key + flags, cost, -}
    const int i = c.x, key = key_of(c.y);
    const int reg = region_of(key);
    if (reg < r0 || reg >= r1 || (G > 1 && group_of(key, G) != g)) continue;
    const float nc = stay_cost(x, __int_as_float(c.z));
    if (!(cut.bin(nc) < k_sel)) continue;        // (it is inside the beam: only those were listed)
    unsigned sl = probe_start(key);
    const unsigned step = probe_step(key);
    int probes = 0, k = t.keys[sl];
    while (k != key && k != kKeyEmpty && probes < kTabSlots) { sl = (sl + step) & kTabMask; ++probes; k = t.keys[sl]; }
    bool win = true;
    if (k == key) {
      const unsigned long long v = t.vals[sl];
      const unsigned oc = f2ord(nc), cc = (unsigned)(v >> 32);
      const unsigned my_arc = 2u * ((unsigned)c.y & x.g.blk_mask) + 1u;
      win = oc < cc;
      if (oc == cc) win = my_arc < (unsigned)x.cand[(unsigned)v].w;          // exact tie: lower arc id
      if (win) t.vals[sl] = ((unsigned long long)oc << 32) | kIdxStay;
    }
    if (win) {
      atomicAdd(&x.sm.hist[cut.bin(nc)], 1u);
      atomicOr(&staybits[i >> 5], 1u << (i & 31));
    }
  }
}

// The table passes that reduce n_sel selected candidates: one pass over everything if they
// fit one table, else every region on its own in as many sub-group passes as it needs.
struct PassPlan {
  int n_pass; bool whole, halves; int per_region[kRegions];
  // every_region: also regions without candidates get a pass (the emitting step, where the self-loop
  // candidates of the tokens meet the table of their region's pass)
  // mult > 1: a plan made from an estimate turned out too small (a pass overfilled the table): every
  // region gets mult times the passes
  __device__ __forceinline__ void make(const Ctx &x, int n_sel, int n_all, bool every_region = false, int mult = 1) {
    static_assert(kRegions == 4, "the halves are regions {0, 1} and {2, 3}");
    whole = n_sel <= kGroupTarget && mult == 1;
    halves = false;
    n_pass = whole ? 1 : 0;
    float est_r[kRegions];
#pragma unroll
    for (int r = 0; r < kRegions; ++r) {
      const int n = uni(min(x.sm.n_reg[r], x.c.region_cap));
      // selected candidates of the region, estimated from its share of all candidates
      est_r[r] = (float)n_sel * (float)n / (float)max(1, n_all) * 1.15f + 64.0f;
      per_region[r] = (whole || (n == 0 && !every_region)) ? 0 : min(2048, ((int)(est_r[r] / (float)kGroupTarget) + 1) * mult);
      n_pass += per_region[r];
    }
    if (!whole && mult == 1 && every_region && est_r[0] + est_r[1] <= (float)kGroupTarget && est_r[2] + est_r[3] <= (float)kGroupTarget) {
      halves = true; n_pass = 2;                  // two regions per pass
    }
  }
  // pass p covers regions [r0, r1) and sub-group g of G
  __device__ __forceinline__ void get(int p, int &r0, int &r1, int &g, int &G) const {
    if (whole) { r0 = 0; r1 = kRegions; g = 0; G = 1; return; }
    if (halves) { r0 = 2 * p; r1 = 2 * p + 2; g = 0; G = 1; return; }
    int r = 0, n = per_region[0];               // no dynamic indexing: the plan stays in registers
#pragma unroll
    for (int q = 0; q < kRegions - 1; ++q) if (r == q && p >= per_region[q]) { p -= per_region[q]; r = q + 1; n = per_region[q + 1]; }
    r0 = r; r1 = r + 1; g = p; G = max(1, n);
  }
};

__device__ __forceinline__ int total_candidates(const Ctx &x) {
  int n = 0;
#pragma unroll
  for (int r = 0; r < kRegions; ++r) n += min(x.sm.n_reg[r], x.c.region_cap);
  return uni(n);
}

// ------------------------------------------------------------------ token creation
// New tokens of the set under construction (N per lane), made from the winning arc alone:
// queue record, backpointer, and an entry in the next epsilon worklist if the state has
// epsilon arcs.  next[] is the arc's destination with its flag bits.  `also[]` appends
// existing tokens (tok[]) that were improved and must be expanded again.  Called by all
// lanes of the wave.
template <int N>
__device__ __forceinline__ void make_tokens(Ctx &x, const int (&make)[N], const int (&ti)[N], const int (&next)[N],
                                            const int (&costbits)[N], const int (&prev)[N], const int (&arc)[N],
                                            const int (&also)[N], const int (&tok)[N],
                                            int2 *NQ, unsigned lat_base, int4 *WLN) {
  int want[2 * N]; int wi[2 * N];
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const int key = key_of(next[u]);
    const bool has_eps = ((unsigned)next[u] & kFlagHasEps) != 0;
    if (make[u]) {
      NQ[ti[u]] = make_int2(next[u], costbits[u]);     // the key and the state's flag bits
      x.lat[lat_base + ti[u]] = make_int2(prev[u], arc[u]);
    }
    want[u] = make[u] & (int)has_eps;
    want[N + u] = also[u] & (int)has_eps;
  }
  wave_alloc_n<2 * N>(&x.sm.n_wl_next, want, wi);
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const int key = key_of(next[u]);
    if (want[u]) WLN[wi[u]] = make_int4(ti[u], key, costbits[u], 1);          // wi < qcap because ti < qcap
    if (want[N + u]) WLN[wi[N + u]] = make_int4(tok[u], key, costbits[u], 0);
  }
}

// ------------------------------------------------------------------ Prune
// 1. select: a histogram of the CANDIDATE costs (before recombination) gives a bin limit
//    k_sel below which a bit more than max_active candidates lie; only those can survive
//    the max-active cutoff, so only those are recombined (k_sel = 256 if everything may).
// 2. recombine the selected candidates in G passes over the LDS table; every occupied
//    slot is the recombined token of one destination; they are histogrammed (256 bins over
//    [best, best+beam]) and parked.
// 3. cutoff: k_keep = first bin where the running count of recombined tokens exceeds
//    max_active (at least 1).  If the selection turns out too small to decide that
//    (duplicate destinations), step 2 is redone with everything selected.
// 4. the survivors become tokens.
__device__ __forceinline__ void recombine_and_prune(Ctx &x, int2 *NQ, unsigned lat_base, int4 *WLN, Cutoff &cut) {
  Smem &sm = x.sm;
  x.srcq = x.q0 + x.s.cur * x.c.qcap;          // the candidates come out of the current token set
  TableLds &t = sm.u.t;
  const int tid = threadIdx.x;
  const unsigned bo = uni(sm.best_ord);
  cut.best = bo == kOrdNone ? INFINITY : ord2f(bo);
  cut.beam = x.s.beam; cut.scale = x.s.scale; cut.k_keep = 256;
  const int n_cand = total_candidates(x);
  const unsigned ma = (unsigned)x.s.max_active;

  const int2 *Q = x.srcq;                      // the current token set: its simple tokens carry implicit candidates
  const int n_tok = x.s.n_tok;
  // bit i of staybits: token i's self-loop candidate is the recombined token of its state (the
  // closure's tables are idle now).  The tokens whose candidate may meet one of the buffer are
  // listed in the second worklist buffer, which nobody uses before the closure's first round ends.
  unsigned *staybits = staybits_of(sm);
  const unsigned *hasstay = hasstay_bits(sm);
  int4 *CL = x.wl0 + x.c.qcap;
  if (tid < 256) { sm.hist2[tid] = 0; sm.hist3[tid] = 0; }
  if (tid == 0) sm.n_cont = 0;
  __syncthreads();

  // ---- 0. the tokens that stay where they are.  One sweep over the token set, while the filter of
  // the buffer's destinations is still there: a self-loop candidate inside the beam whose key's
  // bit is clear meets no other candidate, so it is the recombined token of its state: marked and
  // histogrammed (exactly, in every bin).  The few whose bit is set are left for the table passes.
  constexpr int kS = WFST_USW;                   // queue records in flight per lane
  for (int i0 = 0; i0 < n_tok; i0 += kBlock * kS) {
    int2 q[kS]; int cn[kS], ci[kS];
#pragma unroll
    for (int u = 0; u < kS; ++u) {
      const int i = i0 + u * kBlock + tid;
      q[u] = i < n_tok ? Q[i] : make_int2(0, 0);
    }
#pragma unroll
    for (int u = 0; u < kS; ++u) {
      const int i = i0 + u * kBlock + tid;         // (whole waves beyond the set write words nobody reads)
      const float nc = stay_cost(x, __int_as_float(q[u].y));
      const int stays = (int)(((unsigned)q[u].x & kFlagSimple) != 0) | (int)((hasstay[(i & (kQueueMax - 1)) >> 5] >> (i & 31)) & 1u);
      const int in = (int)(i < n_tok) & stays & (int)(nc < INFINITY) & (int)cut.in_beam(nc);
      const unsigned fb = filter_bit(key_of(q[u].x));
      cn[u] = in & (int)((sm.u.e.filter[fb >> 5] >> (fb & 31)) & 1u);
      const int alone = in & (int)!cn[u];
      if (alone) atomicAdd(&sm.hist3[cut.bin(nc)], 1u);
      const unsigned long long ma_ = __ballot(alone);
      const int lane = tid & 63;                   // the wave's 64 tokens are two words of the bit set
      if (i < kQueueMax) {
        if (lane == 0) staybits[i >> 5] = (unsigned)ma_;
        if (lane == 32) staybits[i >> 5] = (unsigned)(ma_ >> 32);
      }
    }
    wave_alloc_n<kS>(&sm.n_cont, cn, ci);          // at most one entry per token: the list cannot overflow its qcap records
#pragma unroll
    for (int u = 0; u < kS; ++u)
      if (cn[u]) CL[ci[u]] = make_int4(i0 + u * kBlock + tid, q[u].x, q[u].y, 0);
  }

  // ---- 1. select: the exact histogram of the tokens that stay plus a sample of the buffer
  int n_sampled = 0;
  constexpr int kHalf = 2;
  // one run of 64 records in kEvery (a wave reads one run): candidates arrive roughly in the
  // order of the token queue, which is not free of cost trends, so the sample is interleaved finely
  const int sh = x.c.sel_shift, kEvery = 1 << sh;   // one run of 64 records out of kEvery (a power of two)
  const int mine = ((tid >> 6) << (6 + sh)) + (tid & 63);
  for (int r = 0; r < kRegions; ++r) {
    const int n = uni(min(sm.n_reg[r], x.c.region_cap));
    const int4 *cr = x.cand + r * x.c.region_cap;
    for (int i0 = 0; i0 < n; i0 += kEvery * kBlock * kHalf) {
      int cb[kHalf];
#pragma unroll
      for (int u = 0; u < kHalf; ++u) { const int i = i0 + u * kEvery * kBlock + mine; cb[u] = i < n ? cr[i].y : 0; }
#pragma unroll
      for (int u = 0; u < kHalf; ++u) {
        const float c = __int_as_float(cb[u]);
        if (i0 + u * kEvery * kBlock + mine < n && cut.in_beam(c)) atomicAdd(&sm.hist2[cut.bin(c)], 1u);
      }
      const int span = min(n - i0, kEvery * kBlock * kHalf);
      n_sampled += ((span >> (6 + sh)) << 6) + min(span & ((64 << sh) - 1), 64);
    }
  }
  __syncthreads();
  if (tid < 64) {
    // bins of the tokens that stay (exact) plus the buffer's sample scaled up to the whole buffer
    const float up = (float)max(1, n_cand) / (float)max(1, n_sampled);
    float hb[4]; unsigned hs[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { hs[j] = sm.hist3[4 * tid + j]; hb[j] = (float)sm.hist2[4 * tid + j] * up; }
    const unsigned s = hs[0] + hs[1] + hs[2] + hs[3] + (unsigned)(hb[0] + hb[1] + hb[2] + hb[3]);
    const unsigned inc = wave_scan_add(s);
    const unsigned n_in = (unsigned)__builtin_amdgcn_readlane((int)inc, 63);
    const float want = (float)ma * x.s.sel_ratio + 256.0f;
    const unsigned target = want < 2.0e9f ? (unsigned)want : 2000000000u;
    int ks = 256; unsigned nsel = (unsigned)(n_cand + n_tok), nsel_c = (unsigned)n_cand;
    if (n_in > target) {
      float run = (float)(inc - s), run_c = 0.0f;
      int first = 256; float at = 0.0f, at_c = 0.0f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        run += (float)hs[j] + hb[j]; run_c += hb[j];
        if (run >= (float)target && first == 256) { first = 4 * tid + j; at = run; at_c = run_c; }
      }
      int fm = first;
#pragma unroll
      for (int sft = 32; sft > 0; sft >>= 1) fm = min(fm, __shfl_xor(fm, sft, 64));
      const int owner = __ffsll((long long)__ballot(first == fm && fm != 256)) - 1;
      // the buffer's share of the selected: whole lanes before the owner, and the owner's bins up to there
      const float lane_c = hb[0] + hb[1] + hb[2] + hb[3];
      const float before_c = (float)wave_sum((tid & 63) < owner ? (unsigned)lane_c : 0u);
      nsel = (unsigned)__shfl(at, owner, 64);
      nsel_c = min((unsigned)n_cand, (unsigned)(before_c + __shfl(at_c, owner, 64)));
      ks = fm + 1;                                   // bins [0, ks) are selected
    }
    if (tid == 0) { sm.k_sel = ks; sm.n_sel = (int)nsel; sm.n_sel_c = (int)nsel_c; }
  }
  __syncthreads();
  int k_sel = uni(sm.k_sel), n_sel = uni(sm.n_sel), n_sel_c = uni(sm.n_sel_c);
  const int n_cont = uni(sm.n_cont);
  prof_mark(x, kPhSelect);

  // Steps 2 and 3 are done again when the selection turns out wrong: too few distinct destinations
  // among the selected to decide the cutoff -> once more with everything selected; a pass that met
  // far more destinations than the table takes (the number of passes comes from an estimate) ->
  // once more with twice the passes per region.
  int mult = 1;
  for (int attempt = 0;; ++attempt) {
    // ---- 2. recombine the selected candidates, G table passes
    PassPlan plan;
    plan.make(x, n_sel_c, n_cand, true, mult);
    if (tid == 0) sm.overfull = 0;                 // (the first pass begins with a barrier)
    for (int ps = 0; ps < plan.n_pass; ++ps) {
      int r0, r1, g, G;
      plan.get(ps, r0, r1, g, G);
      table_clear(sm);
      __syncthreads();
      prof_mark(x, kPhTabClear);
      table_fill<true>(x, r0, r1, g, G, cut, k_sel);
      __syncthreads();
      prof_mark(x, kPhTabFill);
      stay_meet(x, CL, n_cont, staybits, r0, r1, g, G, cut, k_sel);
      __syncthreads();
      prof_mark(x, kPhStayMeet);
      table_winners<true>(x, r0, r1, g, G, cut, k_sel);
      __syncthreads();
      prof_mark(x, kPhTabScan);
    }
    // ---- 3. cutoff from the histogram of recombined tokens
    if (tid < 64) {
      // recombined tokens in the selected bins: the table passes' winners and the tokens that stay alone
      const unsigned h0 = 4 * tid < k_sel ? sm.hist[4 * tid] + sm.hist3[4 * tid] : 0u;
      const unsigned h1 = 4 * tid + 1 < k_sel ? sm.hist[4 * tid + 1] + sm.hist3[4 * tid + 1] : 0u;
      const unsigned h2 = 4 * tid + 2 < k_sel ? sm.hist[4 * tid + 2] + sm.hist3[4 * tid + 2] : 0u;
      const unsigned h3 = 4 * tid + 3 < k_sel ? sm.hist[4 * tid + 3] + sm.hist3[4 * tid + 3] : 0u;
      unsigned s = h0 + h1 + h2 + h3, inc = s;
      inc = wave_scan_add(inc);
      const unsigned n_u = (unsigned)__builtin_amdgcn_readlane((int)inc, 63);
      int kk = 256, redo = 0;
      if (sm.overfull) {
        redo = 2;                                   // the histogram is worth nothing: more passes
      } else if (n_u > ma) {
        unsigned run = inc - s;
        int first = 256;
        run += h0; if (run > ma && first == 256) first = 4 * tid;
        run += h1; if (run > ma && first == 256) first = 4 * tid + 1;
        run += h2; if (run > ma && first == 256) first = 4 * tid + 2;
        run += h3; if (run > ma && first == 256) first = 4 * tid + 3;
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) first = min(first, __shfl_xor(first, sft, 64));
        kk = first;
        if (tid == 0) { sm.ctr[kCtMaxAct]++; if (kk < 1) sm.ctr[kCtBin0]++; }
        if (kk < 1) kk = 1;
      } else if (k_sel < 256) {
        redo = 1;                                   // too many duplicates among the selected
      }
      {
        // survivors of the cutoff: the recombined tokens in bins below kk
        const unsigned below = (4 * tid < kk ? h0 : 0u) + (4 * tid + 1 < kk ? h1 : 0u) + (4 * tid + 2 < kk ? h2 : 0u) +
                               (4 * tid + 3 < kk ? h3 : 0u);
        const unsigned n_keep = wave_sum(below);
        if (tid == 0) sm.n_emit = (int)min(n_keep, 0x7fffffffu);
      }
      if (tid == 0) {
        sm.k_keep = kk; sm.redo = redo;
        // next frame's selection: enough candidates for max_active distinct destinations
        float r = redo ? x.s.sel_ratio * 2.0f : 1.2f * (float)n_sel / (float)max(1u, n_u);
        sm.red64b = (unsigned long long)__float_as_uint(fminf(fmaxf(r, 1.2f), 16.0f));
      }
    }
    __syncthreads();
    const int redo = uni(sm.redo);
    if (redo != 2) x.s.sel_ratio = uni(__uint_as_float((unsigned)sm.red64b));
    if (!redo) break;
    if (attempt >= 12) { if (tid == 0) atomicOr(&sm.status, kStCapacity); break; }   // never expected: 2048 passes per region
    if (tid == 0) sm.prof[15]++;                   // counted, not timed: re-recombinations
    __syncthreads();
    if (tid < 256) sm.hist[tid] = 0;
    for (int e = tid; e < n_cont; e += kBlock) {   // the listed ones meet the tables again
      const int i = CL[e].x;
      atomicAnd(&staybits[i >> 5], ~(1u << (i & 31)));
    }
    if (tid == 0) { sm.n_win = 0; sm.redo = 0; }
    if (redo == 2) mult *= 2;
    else { k_sel = 256; n_sel = n_cand + n_tok; n_sel_c = n_cand; }
    __syncthreads();
  }
  cut.k_keep = uni(sm.k_keep);
  prof_mark(x, kPhOther);

  // ---- 4. survivors become tokens
  const int n_win = uni(min(sm.n_win, x.c.win_cap));
  const int n_emit = uni(sm.n_emit);
  for (int i0 = 0; i0 < n_win; i0 += kBlock * kUC) {
    int kp[kUC]; int4 cr[kUC];
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      const int i = i0 + u * kBlock + tid;
      cr[u] = x.win[min(i, n_win - 1)];
      kp[u] = (int)(i < n_win) & (int)(cut.bin(__int_as_float(cr[u].y)) < cut.k_keep);
    }
    // tokens an epsilon arc can enter are numbered from the front, the others from the back of
    // the n_emit survivors: the closure then only has to look at the front part
    int ti[kUC], tb[kUC], st[kUC], cb[kUC], pv[kUC], ar[kUC], none[kUC]; int good[kUC], no[kUC], kin[kUC], kout[kUC];
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      kin[u] = kp[u] & (int)(((unsigned)cr[u].x & kFlagEpsIn) != 0);
      kout[u] = kp[u] & (int)!kin[u];
    }
    wave_alloc_n<kUC>(&sm.n_next, kin, ti);
    wave_alloc_n<kUC>(&sm.n_back, kout, tb);
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      if (kout[u]) ti[u] = n_emit - 1 - tb[u];
      good[u] = kp[u]; no[u] = false; none[u] = 0;
      if (kp[u]) {
        if (ti[u] >= x.c.qcap) { atomicOr(&sm.status, kStCapacity); good[u] = false; }
        else if (lat_base + (unsigned)ti[u] >= x.lat_cap) { atomicOr(&sm.status, kStLattice); good[u] = false; }
      }
      st[u] = cr[u].x; cb[u] = cr[u].y; pv[u] = cr[u].z; ar[u] = cr[u].w;
      if (x.c.cost_offset) cb[u] = __float_as_int(canon(__int_as_float(cr[u].y) - cut.best));
    }
    make_tokens<kUC>(x, good, ti, st, cb, pv, ar, no, none, NQ, lat_base, WLN);
  }
  // ... and the tokens that stay where they are: the marked self-loop candidates, made from the
  // queue records of the current set
  for (int i0 = 0; i0 < n_tok; i0 += kBlock * kUC) {
    int kp[kUC]; int2 q[kUC]; float nc[kUC];
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      const int i = i0 + u * kBlock + tid;
      q[u] = Q[min(i, n_tok - 1)];
      nc[u] = stay_cost(x, __int_as_float(q[u].y));
      kp[u] = (int)(i < n_tok) & (int)((staybits[min(i, n_tok - 1) >> 5] >> (i & 31)) & 1u) & (int)(cut.bin(nc[u]) < cut.k_keep);
    }
    int ti[kUC], tb[kUC], st[kUC], cb[kUC], pv[kUC], ar[kUC], none[kUC]; int good[kUC], no[kUC], kin[kUC], kout[kUC];
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      kin[u] = kp[u] & (int)(((unsigned)q[u].x & kFlagEpsIn) != 0);
      kout[u] = kp[u] & (int)!kin[u];
    }
    wave_alloc_n<kUC>(&sm.n_next, kin, ti);
    wave_alloc_n<kUC>(&sm.n_back, kout, tb);
#pragma unroll
    for (int u = 0; u < kUC; ++u) {
      if (kout[u]) ti[u] = n_emit - 1 - tb[u];
      good[u] = kp[u]; no[u] = false; none[u] = 0;
      if (kp[u]) {
        if (ti[u] >= x.c.qcap) { atomicOr(&sm.status, kStCapacity); good[u] = false; }
        else if (lat_base + (unsigned)ti[u] >= x.lat_cap) { atomicOr(&sm.status, kStLattice); good[u] = false; }
      }
      st[u] = q[u].x; cb[u] = __float_as_int(nc[u]); pv[u] = i0 + u * kBlock + tid;
      ar[u] = 2 * (int)((unsigned)q[u].x & x.g.blk_mask) + 1;     // the self-loop: the unit after the header
      if (x.c.cost_offset) cb[u] = __float_as_int(canon(nc[u] - cut.best));
    }
    make_tokens<kUC>(x, good, ti, st, cb, pv, ar, no, none, NQ, lat_base, WLN);
  }
  __syncthreads();
  if (tid == 0) {
    sm.n_in = min(sm.n_next, x.c.qcap);            // the front part
    sm.n_next = n_emit; sm.n_back = 0;
    sm.ctr[kCtKept] += min(n_emit, x.c.qcap);
  }
  if (tid < kRegions) sm.n_reg[tid] = 0;
  if (x.c.frame_best && tid == 0 && x.s.frame + 1 <= x.c.max_frames) {   // the lattice kernel needs it for links across this frame's boundary
    const size_t chan = (size_t)(x.frame_off - x.c.frame_off) / (size_t)(x.c.max_frames + 2);
    x.c.frame_best[chan * (size_t)(x.c.max_frames + 1) + (size_t)x.s.frame + 1] = n_emit > 0 ? cut.best : 0.0f;
  }
  if (x.c.cost_offset && n_emit > 0) {           // the stored costs are relative to this frame's best from here on
    x.s.offset = uni(x.s.offset + (double)cut.best);
    cut.best = 0.0f;
  }
  __syncthreads();
  prof_mark(x, kPhCutoff);
}

// ------------------------------------------------------------------ epsilon closure
// Least fixpoint under the frozen predicate `cut`.  The worklist holds the tokens created
// or improved in the previous round that have epsilon arcs, with their arc ranges.  Each
// round's candidates are recombined in the LDS table; then the tokens the set already has look
// their own state up in the table: a token whose state is there is compared with the
// per-destination best, takes its cost and backpointer if that is better, and removes the entry;
// what is left in the table are destinations without a token, which become new tokens.  Either
// way the token is expanded in the next round.
// On entry WL0 = x.wl0 + sel*qcap holds n_wl entries.
template <bool kBoost>
__device__ __forceinline__ void eps_closure(Ctx &x, int2 *NQ, unsigned lat_base, int sel, const Cutoff &cut) {
  Smem &sm = x.sm;
  EpsLds &ek = sm.ek;
  TableLds &t = sm.u.t;
  const int tid = threadIdx.x;
  const bool boosted = kBoost && x.s.boost_n > 0;
  x.srcq = NQ;                                 // the closure's candidates come out of the set under construction
  int n_wl = uni(min(sm.n_wl_next, x.c.qcap));
  __syncthreads();
  if (tid == 0) sm.n_wl_next = 0;
  __syncthreads();
  for (int round = 0; n_wl > 0; ++round) {
    if (round > (1 << 20)) { if (tid == 0) atomicOr(&sm.status, kStCapacity); break; }
    const int4 *WL = x.wl0 + sel * x.c.qcap; int4 *WLN = x.wl0 + (sel ^ 1) * x.c.qcap;
    // A round whose items fit one chunk and whose arcs fit one table is "fused": the table is
    // cleared up front and every candidate is inserted by the lane that made it, so the
    // candidates are not read back before the winners are known.
    bool fused = false;
    for (int cb = 0; cb < n_wl; cb += kBlock) {
      const int n_items = min(kBlock, n_wl - cb);
      unsigned deg[1], ex[1];
      int4 w = make_int4(0, 0, 0, 0);
      if (tid < n_items) w = WL[cb + tid];
      const unsigned wblk = (unsigned)w.y & x.g.blk_mask;     // w.y is the token's key: (state in B, block)
      deg[0] = tid < n_items ? (unsigned)x.g.unit[2 * (size_t)wblk].w >> kPackXShift : 0u;   // the state's header
      if (n_wl <= kBlock) table_clear(sm);         // while the loads are in flight
      {
        // epsilon arcs out of the set (a counter): every token is listed as new exactly once
        const unsigned xsum = wave_sum(w.w ? deg[0] : 0u);
        if ((tid & 63) == 0 && xsum) atomicAdd((unsigned long long *)&sm.ctr[kCtXarc], (unsigned long long)xsum);
      }
      const unsigned M = block_scan<1>(sm, deg, ex);
      ek.pre[tid] = ex[0];
      ek.abase[tid] = 2 * (int)wblk + 1 - (int)ex[0];
      ek.tcost[tid] = __int_as_float(w.z);         // the token's cost when it was listed
      ek.ttok[tid] = w.x | (int)(((unsigned)w.y >> x.g.blk_bits) << 16);
      if (tid == kBlock - 1) ek.pre[kBlock] = M;
      fused = n_wl <= kBlock && M <= (unsigned)min(kGroupTarget, x.c.region_cap);
      __syncthreads();
      for (unsigned f0 = 0; f0 < M; f0 += kBlock * kU) {
        int ok[kU]; int src[kU]; int4 a[kU]; int arc[kU]; float tc[kU]; int j[kU]; int tb[kU];
        owners_of<kU>(ek.pre, n_items, f0, M, ok, j);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          arc[u] = ek.abase[j[u]] + (int)(f0 + u * kBlock + tid);
          src[u] = ek.ttok[j[u]] & 0xffff;
          tb[u] = (int)((unsigned)ek.ttok[j[u]] >> 16);
          tc[u] = ek.tcost[j[u]];
          a[u] = make_int4(0, 0, 0, 0);
          if (ok[u]) a[u] = x.g.unit[arc[u]];
        }
        int next[kU]; float nc[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          nc[u] = canon(tc[u] + __int_as_float(a[u].y));
          next[u] = a[u].x; arc[u] |= (int)kArcEps;
          if (boosted) {                           // epsilon arcs can carry output labels too
            int nb = tb[u];
            if (ok[u] && a[u].w != 0) nc[u] = canon(nc[u] + boost_step(sm, tb[u], a[u].w, nb));
            next[u] |= nb << x.g.blk_bits;
          }
          ok[u] &= (int)(nc[u] < INFINITY) & (int)cut.keep(nc[u]);
        }
        if (fused) {
          // all into region 0 (at most kGroupTarget <= region_cap records), and into the table
          int ci[kU];
          wave_alloc_n<kU>(&sm.n_reg[0], ok, ci);
#pragma unroll
          for (int u = 0; u < kU; ++u)
            if (ok[u]) x.cand[ci[u]] = make_int4(next[u], __float_as_int(nc[u]), src[u], arc[u]);
          // the records must be visible to the other waves before their indices are published in
          // the table: an exact cost tie makes the other wave read this record's arc id
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
          for (int u = 0; u < kU; ++u)
            if (ok[u]) sm.occ[ci[u]] = (unsigned short)table_insert(x, key_of(next[u]), nc[u], arc[u], src[u], ci[u]);
        } else {
          push_cands<kU>(x, ok, next, nc, src, arc);
        }
      }
      __syncthreads();                             // also keeps ek for this chunk's readers before the next chunk rewrites it
    }
    prof_mark(x, kPhEpsExpand);
    const int n_cand = total_candidates(x);
    PassPlan plan;
    plan.make(x, n_cand, n_cand);
    if (fused) { plan.n_pass = 1; plan.whole = true; }
    for (int ps = 0; ps < plan.n_pass && n_cand > 0; ++ps) {
      int r0, r1, g, G;
      plan.get(ps, r0, r1, g, G);
      if (!fused) {
        table_clear(sm);
        __syncthreads();
        table_fill<false>(x, r0, r1, g, G, cut, 256);
        __syncthreads();
      }
      prof_mark(x, kPhEpsTabFill);
      // the tokens of the set meet the table: each looks its own state up; if the pass has a
      // best candidate for it, the better of the two stays the state's token (cost, then arc id)
      // and the entry is taken out, so that only destinations without a token remain.  The scan
      // itself touches no memory but the (prefetched) queue records: tokens that got better are
      // listed in LDS (the expansion tables are idle) and take their new cost and backpointer
      // afterwards, all candidate records in flight at once.
      {
        // only tokens that an epsilon arc can enter: the front part of the emitting step's tokens
        // [0, n_in) and everything the closure itself has made so far [n_emit, n_next)
        const int n_in = uni(sm.n_in), n_skip = uni(min(sm.n_emit, x.c.qcap)) - n_in;
        const int n_have = n_in + max(0, uni(min(sm.n_next, x.c.qcap)) - n_in - n_skip);
        constexpr int kM = WFST_UM;
        constexpr int kPairs = (int)(sizeof(EpsLds) / sizeof(int2));
        int2 *pairs = reinterpret_cast<int2 *>(&sm.ek);      // {token, candidate index}
        int2 tkn[kM];
#pragma unroll
        for (int k = 0; k < kM; ++k) {
          const int v = min(k * kBlock + tid, max(n_have - 1, 0));
          tkn[k] = NQ[v < n_in ? v : v + n_skip];
        }
        if (tid == 0) sm.n_pairs = 0;
        __syncthreads();
        for (int i0 = 0; i0 < n_have; i0 += kBlock * kM) {
          int2 tk[kM];
#pragma unroll
          for (int k = 0; k < kM; ++k) {
            tk[k] = tkn[k];
            const int v = min(i0 + (kM + k) * kBlock + tid, n_have - 1);
            tkn[k] = NQ[v < n_in ? v : v + n_skip];
          }
#pragma unroll
          for (int k = 0; k < kM; ++k) {
            const int vi = i0 + k * kBlock + tid;
            const int tok = vi < n_in ? vi : vi + n_skip;
            const int tkey = key_of(tk[k].x);
            unsigned sl = probe_start(tkey);
            const unsigned step = probe_step(tkey);
            // (a token that did not fit the lattice arena was never written: the channel stops after
            // this frame, and its queue position must not be looked at)
            const bool real = vi < n_have && lat_base + (unsigned)tok < x.lat_cap;
            int probes = 0, key = real ? t.keys[sl] : kKeyEmpty;
            while (key != tkey && key != kKeyEmpty && probes < kTabSlots) { sl = (sl + step) & kTabMask; ++probes; key = t.keys[sl]; }
            if (key == tkey && real) {
              const unsigned long long v = t.vals[sl];
              t.vals[sl] = kValEmpty;                      // this destination has its token
              const float nc = ord2f((unsigned)(v >> 32)), oc = __int_as_float(tk[k].y);
              bool better = (nc < oc) & (v != kValEmpty);
              if (nc == oc && v != kValEmpty) {              // exact tie: lower arc id, then lower B state of the source
                const int4 cd = x.cand[(unsigned)v]; const int2 bp = x.lat[lat_base + tok];
                better = (unsigned)cd.w < (unsigned)bp.y;
                if (cd.w == bp.y) better = (unsigned)NQ[cd.z].x < (unsigned)NQ[bp.x].x;
              }
              if (better) {
                const int at = atomicAdd(&sm.n_pairs, 1);
                if (at < kPairs) pairs[at] = make_int2(tok, (int)(unsigned)v);
                else {                                       // list full: apply it here
                  const int4 rec = x.cand[(unsigned)v];
                  NQ[tok].y = rec.y;
                  x.lat[lat_base + tok] = make_int2(rec.z, rec.w);
                  if ((unsigned)rec.x & kFlagHasEps) {
                    const int wi = atomicAdd(&sm.n_wl_next, 1);
                    WLN[wi] = make_int4(tok, key_of(rec.x), rec.y, 0);
                  }
                }
              }
            }
          }
        }
        __syncthreads();
        const int n_pairs = uni(min(sm.n_pairs, kPairs));
        for (int i0 = 0; i0 < n_pairs; i0 += kBlock * kU) {
          int improve[kU], tok[kU], none[kU], nx[kU], cb[kU], pv[kU], ar[kU]; int4 rec[kU];
#pragma unroll
          for (int k = 0; k < kU; ++k) {
            const int i = i0 + k * kBlock + tid;
            const int2 pr = pairs[min(i, n_pairs - 1)];
            improve[k] = (int)(i < n_pairs); tok[k] = pr.x; none[k] = 0; pv[k] = 0; ar[k] = 0;
            rec[k] = x.cand[(unsigned)pr.y];
          }
#pragma unroll
          for (int k = 0; k < kU; ++k) {
            nx[k] = rec[k].x; cb[k] = rec[k].y;
            if (improve[k]) {                                // new cost and backpointer in place, expand again
              NQ[tok[k]].y = rec[k].y;
              x.lat[lat_base + tok[k]] = make_int2(rec[k].z, rec[k].w);
            }
          }
          make_tokens<kU>(x, none, tok, nx, cb, pv, ar, improve, tok, NQ, lat_base, WLN);
        }
      }
      __syncthreads();
      prof_mark(x, kPhEpsMeet);
      // the winners left in the table become new tokens
      int pos0 = 0;
      for (int r = r0; r < r1; ++r) {
        const int n = uni(min(sm.n_reg[r], x.c.region_cap));
        const int base = r * x.c.region_cap;
        for (int i0 = 0; i0 < n; i0 += kBlock * kU) {
          int4 rec[kU]; int fresh[kU];
#pragma unroll
          for (int k = 0; k < kU; ++k) {
            const int i = i0 + k * kBlock + tid;
            int slot = -1;
            if (i < n) slot = slot_of_candidate<false>(x, pos0 + i, base + i, g, G, cut, 256);
            fresh[k] = (int)(slot >= 0);
            if (fresh[k]) fresh[k] = (int)((unsigned)t.vals[slot] == (unsigned)(base + i));
            rec[k] = make_int4(0, 0, 0, 0);
            if (fresh[k]) rec[k] = x.cand[base + i];
          }
          int good[kU], no[kU]; int ni[kU], cb[kU], pv[kU], ar[kU], nx[kU];
          wave_alloc_n<kU>(&sm.n_next, fresh, ni);
#pragma unroll
          for (int k = 0; k < kU; ++k) {
            good[k] = fresh[k]; no[k] = 0;
            if (fresh[k]) {
              if (ni[k] >= x.c.qcap) { atomicOr(&sm.status, kStCapacity); good[k] = false; }
              else if (lat_base + (unsigned)ni[k] >= x.lat_cap) { atomicOr(&sm.status, kStLattice); good[k] = false; }
            }
            cb[k] = rec[k].y; pv[k] = rec[k].z; ar[k] = rec[k].w; nx[k] = rec[k].x;
          }
          make_tokens<kU>(x, good, ni, nx, cb, pv, ar, no, ni, NQ, lat_base, WLN);
        }
        pos0 += (n + kBlock - 1) / kBlock * kBlock;
      }
      __syncthreads();
      prof_mark(x, kPhEpsTabScan);
    }
    __syncthreads();
    n_wl = uni(min(sm.n_wl_next, x.c.qcap));
    // (the closure's passes are planned from exact counts: a table that overfills is not expected)
    const bool stop = (uni(sm.status) | uni(sm.overfull)) != 0;
    __syncthreads();
    if (tid == 0 && sm.overfull) { atomicOr(&sm.status, kStCapacity); sm.overfull = 0; }
    if (tid == 0) sm.n_wl_next = 0;
    if (tid < kRegions) sm.n_reg[tid] = 0;
    __syncthreads();
    prof_mark(x, kPhEpsRecombine);
    if (stop) break;
    sel ^= 1;
  }
}

// Publish the closed token set in NQ as A_f (f = x.s.frame).
// Returns true (uniformly) if an overflow was flagged and the channel has to stop.
__device__ __forceinline__ bool finish_set(Ctx &x, int2 *NQ, unsigned lat_base) {
  Smem &sm = x.sm;
  const int tid = threadIdx.x;
  const int n = uni(min(sm.n_next, x.c.qcap));
  const int f = x.s.frame;
  if (x.dig_sum) {
    unsigned long long s = 0;
    for (int i = tid; i < n; i += kBlock) {
      const int2 sc = NQ[i];
      const int state = x.g.unit[2 * (size_t)((unsigned)sc.x & x.g.blk_mask)].x;     // the header names the state
      const unsigned b = ((unsigned)sc.x & kKeyMask) >> x.g.blk_bits;   // the token's state in the boosting acceptor
      s += mix64((((unsigned long long)(unsigned)state << 32) | (unsigned)sc.y) ^ ((unsigned long long)b * 0x9E3779B97F4A7C15ull));
    }
    if (s) atomicAdd(&sm.red64, s);
  }
  if (x.c.tokrec) {                              // lattice output wants the closed set's final records
    int2 *rec = x.c.tokrec + (x.lat - x.c.lattice);
    for (int i = tid; i < n; i += kBlock)
      if (lat_base + (unsigned)i < x.lat_cap) { const int2 q = NQ[i]; rec[lat_base + i] = make_int2((int)((unsigned)q.x & (kKeyMask | kFlagSimple)), q.y); }
  }
  __syncthreads();
  if (tid == 0) {
    const int F = x.c.max_frames + 2;            // the per-frame tables are rings (a recycled channel outlives them)
    x.frame_off[f % F] = lat_base;
    x.frame_off[(f + 1) % F] = lat_base + (unsigned)n;
    x.c.frame_ep[(x.frame_off - x.c.frame_off) + f % F] = x.s.lat_epoch;
    if (x.dig_sum && f <= x.c.max_frames) { x.dig_sum[f] = sm.red64; x.dig_cnt[f] = n; }
    sm.ctr[kCtStored] += n;
    sm.red64 = 0; sm.n_win = 0; sm.n_next = 0; sm.n_wl_next = 0;
    sm.best_ord = kOrdNone;
  }
  if (tid < 256) sm.hist[tid] = 0;
  if (tid < kRegions) sm.n_reg[tid] = 0;
  x.s.lat_used = lat_base + (unsigned)n;
  x.s.n_tok = n;
  x.s.cur ^= 1;
  const bool stop = uni(sm.status) != 0;     // nobody writes status between these two barriers
  __syncthreads();
  return stop;
}

// ------------------------------------------------------------------ final choice + traceback
// Best token by (cost + final cost, state) if any token is final, else by (cost, state)
// (block numbers grow with state ids, so they order the same way);
// then the backpointers are followed to the start token and the non-zero output labels of
// the arcs are written in path order.
__device__ __forceinline__ void select_and_trace(Ctx &x, const LaunchArgs &a, int io) {
  Smem &sm = x.sm;
  const int tid = threadIdx.x;
  const int n = x.s.n_tok;
  const int2 *Q = x.q0 + x.s.cur * x.c.qcap;
  int *words = a.words + (long long)io * a.max_words;
  int flags = x.s.status;
  if (n == 0) {
    if (tid == 0) { a.nwords[io] = 0; a.cost[io] = INFINITY; a.flags[io] = flags | WFST_FLAG_DEAD; }
    return;
  }
  if (tid == 0) { sm.red64 = ~0ull; sm.red64b = ~0ull; sm.sel_idx = -1; }
  __syncthreads();
  // ties go to the lower graph state, then to the lower state of the boosting acceptor: the key
  // (B state, block) is turned round for the comparison
  const int bbits = x.g.blk_bits, sbits = 29 - x.g.blk_bits; const unsigned bm = x.g.blk_mask;
  unsigned long long mf = ~0ull, mr = ~0ull;
  for (int i = tid; i < n; i += kBlock) {
    const int2 t = Q[i];
    const float c = __int_as_float(t.y);
    const unsigned blk = (unsigned)t.x & bm, turned = (blk << sbits) | (((unsigned)t.x & kKeyMask) >> bbits);
    mr = min(mr, ((unsigned long long)f2ord(c) << 32) | turned);
    if (a.finalize) {
      const float fc = x.g.has_final ? __int_as_float(x.g.unit[2 * (size_t)blk].y) : 0.0f;
      const float f = c + fc;
      if (f < INFINITY) mf = min(mf, ((unsigned long long)f2ord(f) << 32) | turned);
    }
  }
  if (mf != ~0ull) atomicMin(&sm.red64, mf);
  atomicMin(&sm.red64b, mr);
  __syncthreads();
  const bool any_final = sm.red64 != ~0ull;
  const unsigned long long best = any_final ? sm.red64 : sm.red64b;
  const unsigned best_turned = (unsigned)(best & 0xffffffffull);
  const int best_key = (int)((best_turned >> sbits) | ((best_turned & ((1u << sbits) - 1u)) << bbits));
  for (int i = tid; i < n; i += kBlock)
    if (key_of(Q[i].x) == best_key) sm.sel_idx = i;
  __syncthreads();
  // One lane follows the backpointers.  The words come out last to first: they go into a ring
  // in LDS (the recombination table is idle now) that keeps the latest max_words of them, i.e.
  // the first max_words of the path, and all lanes then write them out in path order.  Only
  // when max_words exceeds the ring is the chain walked twice (count, then write).
  // The walk is incremental: the previous traceback of the channel left, per frame, the token
  // with which its path entered that frame's set and the number of words up to there, and
  // its words.  Backpointers of stored frames never change, so when the new walk reaches such a
  // token the rest of the path is the old one: the walk stops and the old words are kept.  A
  // partial result after every chunk then costs a walk over the new frames (plus the distance
  // to where the two paths join) instead of over the whole stream.
  int *ring = sm.u.t.keys;
  const bool one_walk = a.max_words <= kTabSlots;
  const bool inc = one_walk && x.c.path_tok != nullptr && a.max_words == x.c.max_words;
  const size_t chan = (size_t)(x.frame_off - x.c.frame_off) / (size_t)(x.c.max_frames + 2);
  int *ptok = inc ? x.c.path_tok + chan * (size_t)(x.c.max_frames + 1) : nullptr;
  int *pnw = inc ? x.c.path_nw + chan * (size_t)(x.c.max_frames + 1) : nullptr;
  int *pwords = inc ? x.c.path_words + chan * (size_t)x.c.max_words : nullptr;
  if (tid == 0) {
    int nw = 0, f_stop = 0, w_stop = 0;
    bool broken = false, gone = false;
    const int F = x.c.max_frames + 2, FM = x.c.max_frames + 1;   // the per-frame tables are rings
    const int *fep = x.c.frame_ep + (x.frame_off - x.c.frame_off);
    for (int pass = one_walk ? 1 : 0; pass < 2; ++pass) {
      int f = x.s.frame, i = sm.sel_idx, k = 0;
      for (unsigned step = 0;; ++step) {
        // every chain ends at the start token; the bounds only guard against a damaged lattice
        if (f < 0 || i < 0 || step > 0x40000000u) { broken = true; break; }
        const unsigned off = x.frame_off[f % F];
        if (x.c.recycle) {
          // is the frame still there?  Its slot of the per-frame tables, and its tokens: stored in
          // this epoch, or in the one before at a place the write position has not reached again
          const int ep = fep[f % F];
          const bool here = x.s.frame - f <= x.c.max_frames &&
                            (ep == x.s.lat_epoch || (ep == x.s.lat_epoch - 1 && off >= x.s.lat_used));
          if (!here) { gone = true; break; }
        } else if (off + (unsigned)i >= x.s.lat_used) { broken = true; break; }
        const unsigned li = off + (unsigned)i;
        if (li >= x.lat_cap) { broken = true; break; }
        const int2 bp = x.lat[li];
        if (bp.y < 0) break;
        const bool emitting = !((unsigned)bp.y & kArcEps);
        if (inc && emitting) {
          if (f <= x.s.path_frames && ptok[f % FM] == i) { f_stop = f; w_stop = pnw[f % FM]; break; }   // the old path from here on
          ptok[f % FM] = i; pnw[f % FM] = k;        // k: words after this arc; turned into words up to it below
        }
        const int ol = x.g.unit[(unsigned)bp.y & kArcMask].w;
        if (ol != 0) {
          if (one_walk) ring[k % a.max_words] = ol;
          else if (pass == 1) { const int pos = nw - 1 - k; if (pos < a.max_words) words[pos] = ol; }
          ++k;
        }
        i = bp.x;
        if (emitting) --f;                                      // an emitting arc consumed a frame
      }
      nw = k;
    }
    nw += w_stop;
    if (any_final) flags |= WFST_FLAG_REACHED_FINAL;
    if (nw > a.max_words) flags |= WFST_FLAG_TRUNCATED;
    if (broken) { flags |= WFST_FLAG_CAPACITY; nw = 0; }
    // a recycled arena no longer holds the frames this path runs through before it meets the path of
    // the previous result (results were asked for too rarely for the arena's size)
    if (gone) { flags |= WFST_FLAG_LATTICE_OVERFLOW; nw = 0; broken = true; }
    a.nwords[io] = min(nw, a.max_words);
    a.cost[io] = x.c.cost_offset ? (float)((double)ord2f((unsigned)(best >> 32)) + x.s.offset) : ord2f((unsigned)(best >> 32));
    a.flags[io] = flags;
    sm.red64 = 0;
    sm.sel_idx = nw;
    sm.trace_from = f_stop; sm.trace_words = w_stop;
    sm.path_frames = (inc && !broken) ? x.s.frame : 0;
  }
  __syncthreads();
  if (one_walk) {
    const int nw = sm.sel_idx, w_stop = sm.trace_words;   // new word k of the walk (0 = last word) sits in ring[k % max_words]
    const int k_new = nw - w_stop;
    if (inc) {
      // marks of the frames walked: words after the arc -> words up to and including it
      const int FM = x.c.max_frames + 1;
      for (int f = sm.trace_from + 1 + tid; f <= x.s.frame; f += kBlock) pnw[f % FM] = nw - pnw[f % FM];
      for (int p = w_stop + tid; p < min(nw, a.max_words); p += kBlock) pwords[p] = ring[(k_new - 1 - (p - w_stop)) % a.max_words];
      __syncthreads();
      for (int p = tid; p < min(nw, a.max_words); p += kBlock) words[p] = pwords[p];
    } else {
      for (int p = tid; p < min(nw, a.max_words); p += kBlock) words[p] = ring[(nw - 1 - p) % a.max_words];
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------ the channel kernel
// kNarrow: the graph has the 8-byte emitting-arc records and the arc loops read them (a variant of
// the kernel of its own, so that the usual one carries none of it).  kBoost: some channel of the
// launch has a boosting table or acceptor; the variant without is smaller, and the frame loop is
// more code than the instruction cache holds, so every kilobyte less of it shows in the time.
// kProf: the phases are timed (a debug hook; an instance of its own because even a skipped
// clock read at every phase boundary costs the frame loop about 1 %).
// kOpt: the decoder has one of its options on (cost offsets, token records for lattices, a recycled
// arena, frame digests); the instance without carries none of their code.
template <bool kNarrow, bool kBoost, bool kProf, bool kOpt, bool kQueue>
__global__ __launch_bounds__(kBlock, WFST_MIN_WAVES) void wfst_channel_kernel(DevGraph g, DevChannels c_arg, LaunchArgs a) {
  __shared__ Smem sm;
  const int tid = threadIdx.x;
  DevChannels c = c_arg;
  if (!kOpt) {                                 // (the host launches this instance only when all of these are off)
    c.cost_offset = 0; c.recycle = 0; c.tokrec = nullptr; c.frame_best = nullptr; c.dig_sum = nullptr; c.dig_cnt = nullptr;
  }
  // A workgroup starts with the list entry of its own number; when that channel is done it takes the
  // first entry nobody has taken yet, until none is left.  (With one workgroup per entry, the usual
  // launch, that is one entry each.)  The host lists long utterances first, so a launch with fewer
  // workgroups than entries ends for all of them at nearly the same time.
  // The channel's pointers are moved from one channel to the next by the difference of the channel
  // numbers, and what else a channel needs comes with the lists: so nothing but the lists has to
  // stay in registers through the frame loop on account of the next channel.
  int job = blockIdx.x;
  int ch = uni(a.lists[job]);
  Ctx x{g, c, sm};
  x.cand = c.cand + (size_t)ch * c.cand_cap;
  x.win = c.win + (size_t)ch * c.win_cap;
  x.q0 = c.queue + (size_t)ch * 2 * c.qcap;
  x.wl0 = c.wl + (size_t)ch * 2 * c.qcap;
  x.lat = c.lattice + uni64(reinterpret_cast<const unsigned long long *>(a.lists + 4 * a.n_jobs + 2)[job]);
  x.prof = kProf ? 1 : 0;
  x.frame_off = c.frame_off + (size_t)ch * (c.max_frames + 2);
  x.dig_sum = c.dig_sum ? c.dig_sum + (size_t)ch * (c.max_frames + 1) : nullptr;
  x.dig_cnt = c.dig_cnt ? c.dig_cnt + (size_t)ch * (c.max_frames + 1) : nullptr;
  ChanState *stp = c.st + ch;
  const int *bkp = c.boost_keys + (size_t)ch * kBoostSlots;
  const float *bvp = c.boost_vals + (size_t)ch * kBoostSlots;
  const unsigned *bfp = c.boost_from_to + (size_t)ch * kBoostSlots;
  for (;;) {
  const int nfr = uni(a.lists[a.n_jobs + job]), io = uni(a.lists[2 * a.n_jobs + job]);
  x.lat_cap = uni((unsigned)a.lists[3 * a.n_jobs + job]);
  x.s = *stp;
  x.s.frame = uni(x.s.frame); x.s.n_tok = uni(x.s.n_tok); x.s.cur = uni(x.s.cur); x.s.status = uni(x.s.status);
  x.s.lat_used = uni(x.s.lat_used); x.s.max_active = uni(x.s.max_active); x.s.beam = uni(x.s.beam);
  x.s.scale = uni(x.s.scale); x.s.sel_ratio = uni(x.s.sel_ratio); x.s.offset = uni(x.s.offset);
  x.s.boost_n = uni(x.s.boost_n); x.s.boost_states = uni(x.s.boost_states); x.s.lat_epoch = uni(x.s.lat_epoch);
  if (kBoost && x.s.boost_n > 0)
    for (int i = tid; i < kBoostSlots; i += kBlock) {
      sm.bk[i] = bkp[i];
      sm.bv[i] = bvp[i];
      sm.bft[i] = bfp[i];
    }

  if (tid == 0) {
    sm.best_ord = kOrdNone; sm.n_pairs = 0; sm.n_hub = 0; sm.n_win = 0; sm.n_next = 0; sm.n_wl_next = 0;
    sm.n_in = 0; sm.n_emit = 0; sm.n_back = 0;
    for (int r = 0; r < kRegions; ++r) sm.n_reg[r] = 0;
    sm.status = 0; sm.red64 = 0; sm.red64b = 0; sm.k_keep = 256; sm.k_sel = 256; sm.n_sel = 0; sm.redo = 0;
    sm.overfull = 0;
    for (int i = 0; i < 16; ++i) sm.prof[i] = 0;
    for (int i = 0; i < 8; ++i) sm.ctr[i] = 0;
    sm.prof_t0 = (long long)wall_clock64();
  }
  if (tid < 256) sm.hist[tid] = 0;
  __syncthreads();

  bool stop = false;
  if (a.mode & kModeInit) {
    // start token, closed over epsilon arcs with best = 0 and no bin limit
    x.s.frame = 0; x.s.n_tok = 0; x.s.cur = 0; x.s.status = 0; x.s.lat_used = 0; x.s.offset = 0.0; x.s.path_frames = 0;
    x.s.lat_epoch = 0;
    x.s.beam = a.beam; x.s.scale = a.scale; x.s.max_active = a.max_active; x.s.sel_ratio = 1.5f;
    int2 *NQ = x.q0 + c.qcap;
    if (tid == 0) { sm.n_next = 1; sm.n_in = 1; sm.n_emit = 1; }
    {
      const int mk[1] = {tid == 0}, no[1] = {false};
      const int z[1] = {0}, st[1] = {(int)g.start}, m1[1] = {-1};
      make_tokens<1>(x, mk, z, st, z, m1, m1, no, z, NQ, 0u, x.wl0);
    }
    __syncthreads();
    Cutoff cut{0.0f, x.s.beam, x.s.scale, 256};
    eps_closure<kBoost>(x, NQ, 0u, 0, cut);
    stop = finish_set(x, NQ, 0u);
  }

  const long long ll0 = (long long)io * a.ll_stride;
  for (int t = 0; t < nfr; ++t) {
    if (stop || x.s.status) break;
    if (x.s.frame >= c.max_frames && !c.recycle) { if (tid == 0) atomicOr(&sm.status, kStCapacity); break; }
    // a recycled arena is a ring over whole frames: a frame's tokens (at most qcap) never straddle
    // its end, the write position goes back to the start instead and the epoch counts that
    if (c.recycle && x.s.lat_used + (unsigned)c.qcap > x.lat_cap) { x.s.lat_used = 0; x.s.lat_epoch++; }
    {
      // the frame's acoustic costs; 16-bit log-likelihoods are widened exactly
      const long long r0 = ll0 + (long long)t * a.V;
      const int vs = g.simple_il - 1;          // the class of the simple states' self-loop: kept beside the table too
      if (a.ll_dtype == WFST_LOGLIKE_F32) {
        const float *row = static_cast<const float *>(a.ll) + r0;
        for (int v = tid; v < a.V; v += kBlock) { const float c = -row[v]; sm.u.e.ac[v] = c; if (v == vs) sm.stay_ac = c; }
      } else if (a.ll_dtype == WFST_LOGLIKE_F16) {
        const _Float16 *row = static_cast<const _Float16 *>(a.ll) + r0;
        for (int v = tid; v < a.V; v += kBlock) { const float c = -(float)row[v]; sm.u.e.ac[v] = c; if (v == vs) sm.stay_ac = c; }
      } else {
        const unsigned short *row = static_cast<const unsigned short *>(a.ll) + r0;
        for (int v = tid; v < a.V; v += kBlock) { const float c = -__uint_as_float((unsigned)row[v] << 16); sm.u.e.ac[v] = c; if (v == vs) sm.stay_ac = c; }
      }
    }
    for (int h = tid; h < kHubCap; h += kBlock) { sm.u.e.hub.ready[h] = 0; sm.u.e.hub.seg_next[h] = 0; }
    for (int h = tid; h < kFilterBits / 32; h += kBlock) sm.u.e.filter[h] = 0u;
    for (int h = tid; h < kQueueMax / 32; h += kBlock) hasstay_bits(sm)[h] = 0u;
    if (tid == 0) { sm.next_run = kWaves; sm.done_waves = 0; sm.n_hub = 0; }
    __syncthreads();
    const int2 *Q = x.q0 + x.s.cur * c.qcap;
    int2 *NQ = x.q0 + (x.s.cur ^ 1) * c.qcap;
    const unsigned lat_base = x.s.lat_used;
    if (tid == 0) { sm.ctr[kCtTok] += x.s.n_tok; sm.ctr[kCtFrames]++; }
    prof_mark(x, kPhOther);
    emit_expand<kNarrow, kBoost>(x, Q, x.s.n_tok);
    prof_mark(x, kPhExpand);
    Cutoff cut;
    recombine_and_prune(x, NQ, lat_base, x.wl0, cut);
    eps_closure<kBoost>(x, NQ, lat_base, 0, cut);
    x.s.frame++;
    stop = finish_set(x, NQ, lat_base);
    prof_mark(x, kPhFinish);
  }
  __syncthreads();
  if (uni(sm.status)) {       // overflow: the channel stops with an empty token set
    x.s.status |= uni(sm.status);
    x.s.n_tok = 0;
  }
  prof_mark(x, kPhOther);
  if (a.mode & kModeFinal) {
    // The traceback works on copies of the context, so that the pointers of the frame loop above
    // never live in memory on its account (only then does the compiler know they are global and
    // keep them in registers).  Inlined: as a called function it cost the frame loop 1 % (the call
    // constrains the registers around it); inlined without the copies was no better.
    const DevGraph g2 = g; const DevChannels c2 = c; const LaunchArgs a2 = a;
    Ctx x2{g2, c2, sm, x.cand, x.win, x.q0, x.wl0, x.lat, x.frame_off, x.dig_sum, x.dig_cnt, x.s, nullptr, x.lat_cap, x.prof};
    if (tid == 0) sm.path_frames = x.s.path_frames;
    select_and_trace(x2, a2, io);
    if (tid == 0) x.s.path_frames = sm.path_frames;      // thread 0's copy is the one that is stored
  }
  prof_mark(x, kPhTrace);
  if (tid == 0) {
    *stp = x.s;
    for (int i = 0; i < 16; ++i) atomicAdd((unsigned long long *)&c.counters[8 + i], (unsigned long long)sm.prof[i]);
    for (int i = 0; i < 8; ++i) atomicAdd((unsigned long long *)&c.counters[i], (unsigned long long)sm.ctr[i]);
    if (kQueue) sm.job = atomicAdd(a.lists + 4 * a.n_jobs, 1);
  }
  if (!kQueue) break;          // (an instance of its own: the loop around the whole kernel costs the one-entry case 1.5 %)
  __syncthreads();             // (also: nobody is still reading this channel's tables when the next one's are set up)
  const int job_done = job;
  job = uni(sm.job);
  if (job >= a.n_jobs) break;
  {
    const int ch2 = uni(a.lists[job]);
    const long long dch = (long long)ch2 - ch;
    ch = ch2;
    const unsigned long long *ls = reinterpret_cast<const unsigned long long *>(a.lists + 4 * a.n_jobs + 2);
    x.lat += (long long)(uni64(ls[job]) - uni64(ls[job_done]));
    x.cand += dch * c.cand_cap;
    x.win += dch * c.win_cap;
    x.q0 += dch * 2 * c.qcap;
    x.wl0 += dch * 2 * c.qcap;
    x.frame_off += dch * (c.max_frames + 2);
    if (x.dig_sum) { x.dig_sum += dch * (c.max_frames + 1); x.dig_cnt += dch * (c.max_frames + 1); }
    stp += dch;
    bkp += dch * kBoostSlots; bvp += dch * kBoostSlots; bfp += dch * kBoostSlots;
  }
  }
}


// ------------------------------------------------------------------ lattice links
// One workgroup per closed token set A_t of one channel, after decoding.  The set's tokens go
// into an LDS hash (block number -> position in A_t); then every epsilon arc of the tokens of
// A_t and every emitting arc of the tokens of A_{t-1} is expanded once more, exactly as the
// decoder did, and its destination looked up: if a token is there and the cost through the arc
// is within the lattice beam of that token's stored cost, the arc is a link.  Sets too large
// for one table are taken in passes over hash groups of their keys.  The kernel runs twice: the
// first run only counts the links of every set, a small scan turns the counts into each set's
// place in the output, and the second run writes the links there (ordered by set; one counter
// in memory for all workgroups would serialise them: measured 3x slower).
constexpr int kLatSlots = 16384;
constexpr int kLatGroup = 11264;              // mean keys per pass (load 0.69)
constexpr int kLatListed = 2048;              // tokens with more than a few arcs: listed, their arcs flattened over the workgroup
constexpr int kLatLightDeg = 3;
constexpr int kLatErrTable = 1;
struct LatLds {
  int keys[kLatSlots];
  unsigned short pos[kLatSlots];
  float ac[kMaxV];
  int bk[kBoostSlots]; float bv[kBoostSlots];
  unsigned short listed[kLatListed];          // position of the token in its set
  int lfirst[kLatListed];                     // unit address of its first arc minus its prefix
  float lcost[kLatListed];
  unsigned lpre[kLatListed + 1];              // arc counts, then their exclusive prefix sums
  unsigned wave_tot[kWaves];
  int n_listed;
  unsigned n_links;                           // links of this set so far
};
struct LatticeArgs {
  int ch, frames;
  const void *ll; int V, ll_dtype;
  float lattice_beam;
  int *tok_state; float *tok_cost; long long tok_cap;
  wfst_lattice_link *links; long long link_cap;
  unsigned long long *ctr;                    // [0] links found (written by the scan), [1] error bits
  unsigned long long *set_links;              // [frames + 1] links per set, then (after the scan) before each set
  int write;                                  // 0: count only; 1: write the links
  // several channels in one launch: workgroup b takes set blocks[b].y of channel blocks[b].x, the
  // blocks[b].z-th channel of the call, whose rows start ll_stride elements after the previous
  // channel's and whose tokens are written from tok_first[blocks[b].z] on; set_links is per workgroup
  const int4 *blocks; const long long *tok_first; long long ll_stride;
};

struct LatPass {                              // block-uniform view of one pass
  const DevGraph &g; LatLds &sm; const LatticeArgs &a;
  const int2 *dst_rec; unsigned dst_base;     // records and first token number of A_t
  int t, p, P; bool boosted;
  unsigned long long links_base;              // where this set's links go
  bool rebase; float set_best;                // cost offsets: the tokens of A_t were rebased by set_best
};

__device__ __forceinline__ int lat_group(int key, int P) {
  return (int)(((hash_state(key) >> 20) * (unsigned)P) >> 12);
}

// One arc (unit address u) out of the token numbered `src` with cost tc.
template <bool kEps>
__device__ __forceinline__ void lat_arc(const LatPass &q, const int4 ar, float tc, unsigned src) {
  const int key = key_of(ar.x);
  if (q.P > 1 && lat_group(key, q.P) != q.p) return;
  const float w = __int_as_float(ar.y);
  float acst = 0.0f, nc;
  if (kEps) nc = canon(tc + w);
  else { acst = q.sm.ac[(ar.z & kLabelMask) - 1]; nc = canon((tc + w) + acst); }
  if (q.boosted && ar.w != 0) {
    unsigned h = boost_slot(ar.w);
    float b = 0.0f;
    for (;;) {
      const int k = q.sm.bk[h];
      if (k == ar.w) { b = q.sm.bv[h]; break; }
      if (k == 0) break;
      h = (h + 1) & (kBoostSlots - 1);
    }
    nc = canon(nc + b);
  }
  if (!kEps && q.rebase) nc = canon(nc - q.set_best);      // into the cost base of A_t, as the decoder did
  if (!(nc < INFINITY)) return;
  unsigned sl = (hash_state(key) >> 6) & (kLatSlots - 1);
  int probes = 0;
  while (q.sm.keys[sl] != key) {
    if (q.sm.keys[sl] == kKeyEmpty || ++probes >= kLatSlots) return;       // no token for that state
    sl = (sl + 1) & (kLatSlots - 1);
  }
  const unsigned j = q.sm.pos[sl];
  const float cj = __int_as_float(q.dst_rec[j].y);
  if (!((nc - cj) <= q.a.lattice_beam)) return;
  const unsigned k = atomicAdd(&q.sm.n_links, 1u);
  const unsigned long long at = q.links_base + k;
  if (q.a.write && at < (unsigned long long)q.a.link_cap) {
    wfst_lattice_link L;
    L.src = (int)src; L.dst = (int)(q.dst_base + j); L.ilabel = kEps ? 0 : (ar.z & kLabelMask); L.olabel = ar.w;
    L.graph_cost = w; L.acoustic_cost = acst; L.cost = nc; L.frame = q.t;
    q.a.links[at] = L;
  }
}

// First arc (unit address) and number of epsilon (kEps) or emitting arcs of a token's state.
template <bool kEps>
__device__ __forceinline__ void lat_arcs_of(const DevGraph &g, int key, int &first, int &deg) {
  const int4 hd = g.unit[2 * (size_t)(unsigned)key];
  const int nx = (int)((unsigned)hd.w >> kPackXShift);
  int ne = (int)((unsigned)hd.w & kPackE);
  if (ne == (int)kPackE) ne = hd.z;
  first = 2 * key + 1 + (kEps ? 0 : nx);
  deg = kEps ? nx : ne;
}

// All epsilon (kEps) or emitting arcs of the n tokens rec[0..n), numbered from `base`.  A token
// in a simple state needs no graph read at all; one with a few arcs is expanded by the lane that
// reads it; the others are listed, and the arcs of all listed tokens are flattened over the
// workgroup (prefix sums over the list, one binary search per arc), so that a state with thousands
// of arcs is shared by all lanes and the arc reads are in flight together.  A token that finds
// the list full is expanded by its own lane.
template <bool kEps>
__device__ __forceinline__ void lat_expand(const LatPass &q, const int2 *rec, unsigned n, unsigned base) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  LatLds &sm = q.sm;
  if (tid == 0) sm.n_listed = 0;
  __syncthreads();
  for (unsigned i = tid; i < n; i += kBlock) {
    int2 tk = rec[i];
    if ((unsigned)tk.x & kFlagSimple) {
      // a simple state: no epsilon arcs, and its one emitting arc is the graph's usual self-loop,
      // known without reading the graph
      tk.x = key_of(tk.x);
      if (!kEps) lat_arc<kEps>(q, make_int4(tk.x, __float_as_int(q.g.simple_w), q.g.simple_il, 0), __int_as_float(tk.y), base + i);
      continue;
    }
    int first, deg;
    lat_arcs_of<kEps>(q.g, tk.x, first, deg);
    bool mine = deg <= kLatLightDeg;
    if (!mine) {
      const int h = atomicAdd(&sm.n_listed, 1);
      if (h < kLatListed) { sm.listed[h] = (unsigned short)i; sm.lfirst[h] = first; sm.lcost[h] = __int_as_float(tk.y); sm.lpre[h] = (unsigned)deg; }
      else mine = true;
    }
    if (mine)
      for (int k = 0; k < deg; ++k) lat_arc<kEps>(q, q.g.unit[first + k], __int_as_float(tk.y), base + i);
  }
  __syncthreads();
  const int nl = min(sm.n_listed, kLatListed);
  // exclusive prefix sums of the listed tokens' arc counts: two entries per thread
  static_assert(kLatListed == 2 * kBlock, "two list entries per thread");
  const unsigned d0 = 2 * tid < nl ? sm.lpre[2 * tid] : 0u, d1 = 2 * tid + 1 < nl ? sm.lpre[2 * tid + 1] : 0u;
  const unsigned inc = wave_scan_add(d0 + d1);
  if (lane == 63) sm.wave_tot[wave] = inc;
  __syncthreads();
  unsigned before = 0, M = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) { const unsigned t = sm.wave_tot[w]; if (w < wave) before += t; M += t; }
  const unsigned ex0 = before + inc - d0 - d1;
  if (2 * tid < nl) { sm.lpre[2 * tid] = ex0; sm.lfirst[2 * tid] -= (int)ex0; }
  if (2 * tid + 1 < nl) { sm.lpre[2 * tid + 1] = ex0 + d0; sm.lfirst[2 * tid + 1] -= (int)(ex0 + d0); }
  if (tid == 0) sm.lpre[nl] = M;
  __syncthreads();
  constexpr int kLU = 2;                         // arc reads in flight per lane
  for (unsigned f0 = 0; f0 < M; f0 += kBlock * kLU) {
    int4 ar[kLU]; int j[kLU]; bool ok[kLU];
#pragma unroll
    for (int u = 0; u < kLU; ++u) {
      const unsigned f = f0 + u * kBlock + tid;
      ok[u] = f < M;
      int lo = 0, hi = nl;                       // last j with lpre[j] <= f
      while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (sm.lpre[mid] <= (ok[u] ? f : 0u)) lo = mid; else hi = mid; }
      j[u] = lo;
      ar[u] = make_int4(0, 0, 1, 0);
      if (ok[u]) ar[u] = q.g.unit[sm.lfirst[lo] + (int)f];
    }
#pragma unroll
    for (int u = 0; u < kLU; ++u)
      if (ok[u]) lat_arc<kEps>(q, ar[u], sm.lcost[j[u]], base + sm.listed[j[u]]);
  }
  __syncthreads();
}

__global__ __launch_bounds__(kBlock) void wfst_lattice_kernel(DevGraph g, DevChannels c, LatticeArgs a) {
  __shared__ LatLds sm;
  const int tid = threadIdx.x;
  int t = blockIdx.x, ch = a.ch;
  long long tok0 = 0, ll0 = 0;
  if (a.blocks) {
    const int4 b = a.blocks[blockIdx.x];
    ch = uni(b.x); t = uni(b.y); tok0 = a.tok_first[uni(b.z)]; ll0 = (long long)uni(b.z) * a.ll_stride;
  }
  const unsigned *off = c.frame_off + (size_t)ch * (c.max_frames + 2);
  const int2 *rec = c.tokrec + c.lat_start[ch];
  const unsigned o1 = off[t], n1 = off[t + 1] - o1;
  const unsigned o0 = t ? off[t - 1] : 0u, n0 = t ? o1 - o0 : 0u;
  // the set's tokens, by state id
  for (unsigned i = tid; i < n1; i += kBlock) {
    const int2 tk = rec[o1 + i];
    if (tok0 + (long long)(o1 + i) < a.tok_cap) {
      a.tok_state[tok0 + o1 + i] = g.unit[2 * (size_t)(unsigned)key_of(tk.x)].x;
      a.tok_cost[tok0 + o1 + i] = __int_as_float(tk.y);
    }
  }
  if (t > 0) {                                  // the acoustic costs the arcs into A_t were taken with
    const long long r0 = ll0 + (long long)(t - 1) * a.V;
    if (a.ll_dtype == WFST_LOGLIKE_F32) {
      const float *row = static_cast<const float *>(a.ll) + r0;
      for (int v = tid; v < a.V; v += kBlock) sm.ac[v] = -row[v];
    } else if (a.ll_dtype == WFST_LOGLIKE_F16) {
      const _Float16 *row = static_cast<const _Float16 *>(a.ll) + r0;
      for (int v = tid; v < a.V; v += kBlock) sm.ac[v] = -(float)row[v];
    } else {
      const unsigned short *row = static_cast<const unsigned short *>(a.ll) + r0;
      for (int v = tid; v < a.V; v += kBlock) sm.ac[v] = -__uint_as_float((unsigned)row[v] << 16);
    }
  }
  const bool boosted = c.st[ch].boost_n > 0;
  if (boosted)
    for (int i = tid; i < kBoostSlots; i += kBlock) {
      sm.bk[i] = c.boost_keys[(size_t)ch * kBoostSlots + i];
      sm.bv[i] = c.boost_vals[(size_t)ch * kBoostSlots + i];
    }
  const int P = max(1, (int)((n1 + kLatGroup - 1) / kLatGroup));
  const unsigned long long links_base = a.write ? a.set_links[blockIdx.x] : 0ull;
  if (tid == 0) sm.n_links = 0;
  for (int p = 0; p < P; ++p) {
    for (int sl = tid; sl < kLatSlots; sl += kBlock) sm.keys[sl] = kKeyEmpty;
    __syncthreads();
    for (unsigned j = tid; j < n1; j += kBlock) {
      const int key = key_of(rec[o1 + j].x);
      if (P > 1 && lat_group(key, P) != p) continue;
      unsigned sl = (hash_state(key) >> 6) & (kLatSlots - 1);
      int probes = 0;
      while (atomicCAS(&sm.keys[sl], kKeyEmpty, key) != kKeyEmpty) {
        if (++probes >= kLatSlots) { atomicOr(&a.ctr[1], (unsigned long long)kLatErrTable); break; }
        sl = (sl + 1) & (kLatSlots - 1);
      }
      if (probes < kLatSlots) sm.pos[sl] = (unsigned short)j;
    }
    __syncthreads();
    const bool rebase = c.frame_best != nullptr && t > 0;
    const float set_best = rebase ? c.frame_best[(size_t)ch * (c.max_frames + 1) + t] : 0.0f;
    const LatPass q{g, sm, a, rec + o1, o1, t, p, P, boosted, links_base, rebase, set_best};
    lat_expand<true>(q, rec + o1, n1, o1);
    if (t > 0) lat_expand<false>(q, rec + o0, n0, o0);
  }
  if (tid == 0 && !a.write) a.set_links[blockIdx.x] = sm.n_links;     // lat_expand ends with a barrier
}

// Exclusive prefix sums of v[0..n) in place, the total into *total (one workgroup).
__global__ __launch_bounds__(kBlock) void wfst_lattice_scan(unsigned long long *v, int n, unsigned long long *total) {
  __shared__ unsigned long long part[kBlock];
  const int tid = threadIdx.x;
  const int per = (n + kBlock - 1) / kBlock, lo = min(n, tid * per), hi = min(n, lo + per);
  unsigned long long s = 0;
  for (int i = lo; i < hi; ++i) s += v[i];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) {
    unsigned long long run = 0;
    for (int i = 0; i < kBlock; ++i) { const unsigned long long x = part[i]; part[i] = run; run += x; }
    *total = run;
  }
  __syncthreads();
  unsigned long long run = part[tid];
  for (int i = lo; i < hi; ++i) { const unsigned long long x = v[i]; v[i] = run; run += x; }
}

}  // namespace

// =================================================================================== host
struct wfst_decoder {
  DevGraph g{};
  DevChannels c{};
  wfst_opts opts{};
  int V = 0;
  std::vector<void *> allocs;
  int64_t dev_bytes = 0;
  // per-launch lists: on the device one area per batch slot (+ one for the calls that name channels); host staging in a ring
  static constexpr int kRing = 8;
  int *d_params = nullptr;  int ring_pos = 0;
  unsigned long long *d_lat_ctr = nullptr;   // lattice kernel: links found, error bits
  unsigned long long *d_set_links = nullptr; // [max_frames + 2] links per token set of the channel being read out
  std::vector<int> h_params[kRing];
  // device staging for host-side outputs
  int *o_words = nullptr, *o_nwords = nullptr, *o_flags = nullptr; float *o_cost = nullptr;
  // word-boost tables: pinned host staging per channel (keys, values, count) + what is on the device
  int *h_boost = nullptr;            // [channels][kBoostStage]: labels, scores, from | to << 16, {arcs, states}
  std::vector<int> boost_on_dev;     // entries of the table each channel currently has on the device
  std::vector<hipEvent_t> boost_ev;  // per channel: recorded after the copies out of its staging area
  std::vector<unsigned> blk_of_state;  // [S + 1] block number of every state (and the block count)
  std::vector<int> state_of_blk;       // inverse, built when a debug call first needs it
  std::vector<unsigned> h_off;         // wfst_get_lattice: channel state, counters and frame offsets on the host
  unsigned *h_pinned = nullptr;        // the same for wfst_get_lattice_noalloc: pinned, allocated at create
  // wfst_get_lattice_batch: which (channel, set) every workgroup takes, where each channel's tokens go
  int4 *d_lat_blocks = nullptr; long long *d_tok_first = nullptr;
  char *h_lat_batch = nullptr; size_t h_lat_batch_bytes = 0;     // pinned staging, allocated by the first such call
  // batch slots: wfst_decode_batch_slot calls on different slots may be in flight together
  int n_slots = 1, slot_channels = 0;
  std::vector<hipEvent_t> ev0, ev1;    // per slot (+ one pair for the calls that name channels): around the last kernel
  std::vector<char> timed;
  // lattice memory: every slot's channels share one pool, shared out equally (streaming) or by
  // utterance length (a batch decode)
  unsigned long long *d_lat_start = nullptr; unsigned *d_lat_capn = nullptr;
  std::vector<unsigned long long> eq_start; std::vector<unsigned> eq_capn;       // the equal shares
  std::vector<unsigned long long> cur_start; std::vector<unsigned> cur_capn;     // where every channel's arena is now (what the device arrays hold)
  std::vector<unsigned long long> h_start[kRing]; std::vector<unsigned> h_capn[kRing];   // staging
  int part_pos = 0, last_timed = -1;
  std::vector<char> slot_by_length;    // the slot's pool is currently shared out by length
  std::vector<char> chan_ready;        // the channel has been initialised since its arena was last moved
  int phase_timing = 0;                // launches time their phases (wfst_debug_set_phase_timing)
  int launch_workgroups = 0;           // most workgroups a launch gets (wfst_set_launch_workgroups); 0: one per list entry
  std::string err;
};

namespace {
std::string g_create_err;

#define HIP_TRY(dec, expr)                                                              \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                             \
      (dec)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                   \
      return e_ == hipErrorOutOfMemory ? WFST_ERR_OOM : WFST_ERR_HIP;                   \
    }                                                                                   \
  } while (0)

template <class T> int dev_alloc(wfst_decoder *d, T **p, size_t n) {
  void *q = nullptr;
  size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) {
    d->err = "hipMalloc of " + std::to_string(bytes) + " bytes: " + hipGetErrorString(e);
    (void)hipGetLastError();
    return WFST_ERR_OOM;
  }
  d->allocs.push_back(q);
  d->dev_bytes += (int64_t)bytes;
  *p = static_cast<T *>(q);
  return WFST_OK;
}

int fail(wfst_decoder *d, int code, const std::string &msg) {
  if (d) d->err = msg; else g_create_err = msg;
  return code;
}

// Graph checks: CSR shape, label and destination ranges, finite weights, acyclic epsilon arcs.
int validate_graph(const wfst_graph_csr *g, std::string &why, int64_t &Ae, int64_t &Ax) {
  const int32_t S = g->num_states;
  if (S <= 0 || g->num_arcs < 0 || g->num_classes <= 0) { why = "empty graph or no classes"; return WFST_ERR_BAD_GRAPH; }
  if (g->start_state < 0 || g->start_state >= S) { why = "start state out of range"; return WFST_ERR_BAD_GRAPH; }
  if (!g->row_offsets || (g->num_arcs && (!g->next_state || !g->ilabel || !g->olabel || !g->weight))) {
    why = "null graph array"; return WFST_ERR_INVALID_ARG;
  }
  if (g->row_offsets[0] != 0 || g->row_offsets[S] != g->num_arcs) { why = "row_offsets must start at 0 and end at num_arcs"; return WFST_ERR_BAD_GRAPH; }
  for (int32_t s = 0; s < S; ++s)
    if (g->row_offsets[s + 1] < g->row_offsets[s]) { why = "row_offsets not monotone at state " + std::to_string(s); return WFST_ERR_BAD_GRAPH; }
  Ae = Ax = 0;
  for (int64_t i = 0; i < g->num_arcs; ++i) {
    if (g->next_state[i] < 0 || g->next_state[i] >= S) { why = "next_state out of range at arc " + std::to_string(i); return WFST_ERR_BAD_GRAPH; }
    if (g->ilabel[i] < 0 || g->ilabel[i] > g->num_classes) { why = "ilabel out of range at arc " + std::to_string(i); return WFST_ERR_BAD_GRAPH; }
    if (g->olabel[i] < 0) { why = "negative olabel at arc " + std::to_string(i); return WFST_ERR_BAD_GRAPH; }
    if (!std::isfinite(g->weight[i])) { why = "non-finite weight at arc " + std::to_string(i); return WFST_ERR_BAD_GRAPH; }
    if (g->ilabel[i] == 0) ++Ax; else ++Ae;
  }
  if (Ae + Ax >= (int64_t)0x7fffffff) { why = "more than 2^31-1 arcs"; return WFST_ERR_BAD_GRAPH; }
  if (g->final_cost)
    for (int32_t s = 0; s < S; ++s)
      if (std::isnan(g->final_cost[s])) { why = "NaN final cost"; return WFST_ERR_BAD_GRAPH; }
  // epsilon sub-graph must be a DAG (the closure is a fixpoint iteration): peel sources
  std::vector<int32_t> indeg(S, 0), ready;
  for (int64_t i = 0; i < g->num_arcs; ++i) if (g->ilabel[i] == 0) indeg[g->next_state[i]]++;
  for (int32_t s = 0; s < S; ++s) if (!indeg[s]) ready.push_back(s);
  int64_t peeled = 0;
  while (!ready.empty()) {
    int32_t s = ready.back(); ready.pop_back(); ++peeled;
    for (int64_t i = g->row_offsets[s]; i < g->row_offsets[s + 1]; ++i)
      if (g->ilabel[i] == 0 && --indeg[g->next_state[i]] == 0) ready.push_back(g->next_state[i]);
  }
  if (peeled != S) { why = "epsilon arcs form a cycle"; return WFST_ERR_BAD_GRAPH; }
  return WFST_OK;
}

// Lay the graph out as state blocks (see the top of this file).
int upload_graph(wfst_decoder *d, const wfst_graph_csr *g) {
  const int32_t S = g->num_states;
  std::vector<char> eps_in(S, 0), has_eps(S, 0);
  std::vector<unsigned> &blk = d->blk_of_state;
  blk.assign((size_t)S + 1, 0);
  uint64_t units = 0;
  for (int32_t s = 0; s < S; ++s) {
    blk[s] = (unsigned)(units / 2);
    uint64_t n = 1 + (uint64_t)(g->row_offsets[s + 1] - g->row_offsets[s]);
    units += n + (n & 1);
    if (units / 2 > (uint64_t)kKeyMask) return fail(d, WFST_ERR_BAD_GRAPH, "graph larger than 2^29 blocks of 32 bytes");
    for (int64_t i = g->row_offsets[s]; i < g->row_offsets[s + 1]; ++i)
      if (g->ilabel[i] == 0) { eps_in[g->next_state[i]] = 1; has_eps[s] = 1; }
  }
  blk[S] = (unsigned)(units / 2);
  // The usual self-loop: the (ilabel, weight) that is most frequent among first arcs that are
  // self-loops without output label, over the states without epsilon arcs (in a CTC graph the
  // blank self-loop).  A state whose first arc is that self-loop is a "loop-first" state; one
  // that has no other arc is "simple".
  std::vector<char> simple(S, 0), loop_first(S, 0);
  int simple_il = 1; float simple_w = 0.0f;
  {
    std::unordered_map<uint64_t, int64_t> freq;
    auto starts_with_loop = [&](int32_t s) {
      const int64_t i = g->row_offsets[s];
      return g->row_offsets[s + 1] > i && !has_eps[s] && g->next_state[i] == s && g->olabel[i] == 0;
    };
    // (with narrow arc records an emitting arc's weight is its binary16 rounding everywhere)
    auto pair_of = [&](int64_t i) {
      const float w = d->opts.narrow_arcs ? (float)(_Float16)g->weight[i] : g->weight[i];
      uint32_t wb; std::memcpy(&wb, &w, 4); return ((uint64_t)(uint32_t)g->ilabel[i] << 32) | wb;
    };
    for (int32_t s = 0; s < S; ++s) if (starts_with_loop(s)) ++freq[pair_of(g->row_offsets[s])];
    uint64_t best = 0; int64_t best_n = 0;
    for (const auto &kv : freq) if (kv.second > best_n || (kv.second == best_n && kv.first < best)) { best = kv.first; best_n = kv.second; }
    if (best_n > 0) {
      simple_il = (int)(best >> 32); const uint32_t wb = (uint32_t)best; std::memcpy(&simple_w, &wb, 4);
      for (int32_t s = 0; s < S; ++s)
        if (starts_with_loop(s) && pair_of(g->row_offsets[s]) == best) {
          loop_first[s] = 1;
          simple[s] = g->row_offsets[s + 1] - g->row_offsets[s] == 1;
        }
    }
  }
  auto named = [&](int32_t s) {
    return blk[s] | (has_eps[s] ? kFlagHasEps : 0u) | (eps_in[s] ? kFlagEpsIn : 0u) | (simple[s] ? kFlagSimple : 0u);
  };
  std::vector<int4> unit(units, make_int4(0, 0, 0, 0));
  const bool narrow = d->opts.narrow_arcs != 0;
  std::vector<int2> earc8(narrow ? units : 0, make_int2(0, 0));
  bool all_zero = true;
  for (int32_t s = 0; s < S; ++s) {
    const int64_t r0 = g->row_offsets[s], r1 = g->row_offsets[s + 1];
    int ne = 0, nx = 0;
    for (int64_t i = r0; i < r1; ++i) if (g->ilabel[i] == 0) ++nx; else ++ne;
    const float fc = g->final_cost ? g->final_cost[s] : 0.0f;
    all_zero = all_zero && fc == 0.0f;
    int fbits; std::memcpy(&fbits, &fc, 4);
    int4 *b = unit.data() + 2 * (size_t)blk[s];
    if (nx > kMaxEpsDeg) return fail(d, WFST_ERR_BAD_GRAPH, "state " + std::to_string(s) + " has more than " + std::to_string(kMaxEpsDeg) + " epsilon arcs");
    const unsigned packed = std::min<unsigned>((unsigned)ne, kPackE) | ((unsigned)nx << kPackXShift);
    b[0] = make_int4(s, fbits, ne, (int)packed);
    int4 *xa = b + 1, *ea = b + 1 + nx;
    for (int64_t i = r0; i < r1; ++i) {
      float w = g->weight[i];
      unsigned short hbits = 0;
      if (narrow && g->ilabel[i] != 0) {
        // the weight of an emitting arc becomes its nearest binary16 value EVERYWHERE (also in the
        // full record), so the decoder is the fp32 decoder on a graph with those weights
        const _Float16 h = (_Float16)w;
        w = (float)h;
        if (!std::isfinite(w)) return fail(d, WFST_ERR_BAD_GRAPH, "narrow_arcs: the weight of arc " + std::to_string(i) + " does not fit binary16");
        std::memcpy(&hbits, &h, 2);
      }
      int wbits; std::memcpy(&wbits, &w, 4);
      int4 arc = make_int4((int)named(g->next_state[i]), wbits, g->ilabel[i], g->olabel[i]);
      if (i == r0 && loop_first[s]) arc.z |= (int)kLoopFirst;       // (the narrow record keeps the plain label)
      if (g->ilabel[i] == 0) *xa++ = arc;
      else {
        if (narrow) earc8[(size_t)(ea - unit.data())] = make_int2(arc.x, (int)(((unsigned)hbits << 16) | (g->olabel[i] != 0 ? 0x1000u : 0u) | (unsigned)g->ilabel[i]));
        *ea++ = arc;
      }
    }
  }
  int4 *d_unit;
  int rc;
  if ((rc = dev_alloc(d, &d_unit, unit.size()))) return rc;
  HIP_TRY(d, hipMemcpy(d_unit, unit.data(), unit.size() * sizeof(int4), hipMemcpyHostToDevice));
  int blk_bits = 1;
  while (blk_bits < 29 && (1u << blk_bits) < blk[S]) ++blk_bits;
  int2 *d_earc8 = nullptr;
  if (narrow) {
    if ((rc = dev_alloc(d, &d_earc8, earc8.size()))) return rc;
    HIP_TRY(d, hipMemcpy(d_earc8, earc8.data(), earc8.size() * sizeof(int2), hipMemcpyHostToDevice));
  }
  d->g = DevGraph{d_unit, blk[S], named(g->start_state), all_zero ? 0 : 1, S, blk_bits, (1u << blk_bits) - 1u,
                  simple_il, simple_w, d_earc8};
  return WFST_OK;
}

int next_pow2(int64_t v) { int64_t p = 1; while (p < v) p <<= 1; return (int)p; }

int alloc_channels(wfst_decoder *d) {
  const wfst_opts &o = d->opts;
  DevChannels &c = d->c;
  const size_t N = (size_t)o.max_channels;
  const int ma = o.max_active_hint > 0 ? o.max_active_hint : 10000;
  // candidates of one frame: ~16 per kept token before the buffer overflows (flagged, not fatal)
  c.cand_cap = o.candidate_capacity > 0 ? o.candidate_capacity : next_pow2(std::max<int64_t>(16384, 16LL * ma));
  c.region_cap = c.cand_cap / kRegions;
  c.win_cap = c.cand_cap;
  c.qcap = std::min(kQueueMax, std::max(8192, next_pow2(4LL * ma)));
  c.max_frames = o.max_frames_per_channel;
  int64_t lat_bytes = o.lattice_bytes_per_channel > 0 ? o.lattice_bytes_per_channel
                                                      : (int64_t)(8.0 * 1.5 * ma * ((double)c.max_frames + 1.0));
  int64_t lat_entries = std::max<int64_t>(lat_bytes / 8, 4096);
  if (lat_entries >= (int64_t)0x7fffffff) lat_entries = 0x7ffffffe;
  c.lat_cap = (unsigned)lat_entries;
  int rc;
  if ((rc = dev_alloc(d, &c.st, N))) return rc;
  if ((rc = dev_alloc(d, &c.cand, N * (size_t)c.cand_cap))) return rc;
  if ((rc = dev_alloc(d, &c.win, N * c.win_cap))) return rc;
  if ((rc = dev_alloc(d, &c.queue, N * 2 * c.qcap))) return rc;
  if ((rc = dev_alloc(d, &c.wl, N * 2 * c.qcap))) return rc;
  c.recycle = o.recycle_lattice ? 1 : 0;
  if (c.recycle && (int64_t)c.lat_cap < 2LL * c.qcap)
    return fail(d, WFST_ERR_INVALID_ARG, "recycle_lattice needs room for two full token sets per channel: at least " +
                                             std::to_string(16LL * c.qcap) + " lattice bytes per channel");
  if ((rc = dev_alloc(d, &c.lattice, N * (size_t)c.lat_cap))) return rc;
  if ((rc = dev_alloc(d, &c.frame_off, N * (size_t)(c.max_frames + 2)))) return rc;
  if ((rc = dev_alloc(d, &c.frame_ep, N * (size_t)(c.max_frames + 2)))) return rc;
  HIP_TRY(d, hipMemset(c.frame_ep, 0, N * (size_t)(c.max_frames + 2) * sizeof(int)));
  if ((rc = dev_alloc(d, &d->d_lat_start, N))) return rc;
  if ((rc = dev_alloc(d, &d->d_lat_capn, N))) return rc;
  d->eq_start.resize(N); d->eq_capn.assign(N, c.lat_cap);
  for (size_t ch = 0; ch < N; ++ch) d->eq_start[ch] = (unsigned long long)ch * c.lat_cap;
  d->cur_start = d->eq_start; d->cur_capn = d->eq_capn;
  HIP_TRY(d, hipMemcpy(d->d_lat_start, d->eq_start.data(), N * sizeof(unsigned long long), hipMemcpyHostToDevice));
  HIP_TRY(d, hipMemcpy(d->d_lat_capn, d->eq_capn.data(), N * sizeof(unsigned), hipMemcpyHostToDevice));
  c.lat_start = d->d_lat_start; c.lat_capn = d->d_lat_capn;
  d->slot_by_length.assign((size_t)d->n_slots, 0);
  d->chan_ready.assign(N, 0);
  if (o.keep_token_records && (rc = dev_alloc(d, &c.tokrec, N * (size_t)c.lat_cap))) return rc;
  c.cost_offset = o.cost_offset ? 1 : 0;
  {
    const int every = o.selection_sample > 0 ? std::min(o.selection_sample, 4096) : WFST_SEL_EVERY;
    c.sel_shift = 0;
    while ((2 << c.sel_shift) <= every) ++c.sel_shift;          // rounded down to a power of two
  }
  c.max_words = o.max_words;
  if ((rc = dev_alloc(d, &c.path_tok, N * (size_t)(c.max_frames + 1)))) return rc;
  if ((rc = dev_alloc(d, &c.path_nw, N * (size_t)(c.max_frames + 1)))) return rc;
  if ((rc = dev_alloc(d, &c.path_words, N * (size_t)o.max_words))) return rc;
  if (o.cost_offset && o.keep_token_records && (rc = dev_alloc(d, &c.frame_best, N * (size_t)(c.max_frames + 1)))) return rc;
  if (o.record_digests) {
    if ((rc = dev_alloc(d, &c.dig_sum, N * (size_t)(c.max_frames + 1)))) return rc;
    if ((rc = dev_alloc(d, &c.dig_cnt, N * (size_t)(c.max_frames + 1)))) return rc;
  }
  if ((rc = dev_alloc(d, &c.counters, (size_t)24))) return rc;
  HIP_TRY(d, hipMemset(c.st, 0, N * sizeof(ChanState)));
  HIP_TRY(d, hipMemset(c.counters, 0, 24 * sizeof(long long)));
  HIP_TRY(d, hipMemset(c.frame_off, 0, N * (size_t)(c.max_frames + 2) * sizeof(unsigned)));
  if ((rc = dev_alloc(d, &c.boost_keys, N * kBoostSlots))) return rc;
  if ((rc = dev_alloc(d, &c.boost_vals, N * kBoostSlots))) return rc;
  if ((rc = dev_alloc(d, &c.boost_from_to, N * kBoostSlots))) return rc;
  HIP_TRY(d, hipMemset(c.boost_keys, 0, N * kBoostSlots * sizeof(int)));
  HIP_TRY(d, hipMemset(c.boost_vals, 0, N * kBoostSlots * sizeof(float)));
  HIP_TRY(d, hipMemset(c.boost_from_to, 0, N * kBoostSlots * sizeof(unsigned)));
  HIP_TRY(d, hipHostMalloc(reinterpret_cast<void **>(&d->h_boost), N * kBoostStage * sizeof(int)));
  d->boost_on_dev.assign(N, 0);
  if ((rc = dev_alloc(d, &d->d_params, ((size_t)d->n_slots + 1) * (6 * N + 2)))) return rc;
  if ((rc = dev_alloc(d, &d->d_lat_ctr, (size_t)2))) return rc;
  if (o.keep_token_records) {                   // one entry per token set of every channel (a call may take them all)
    if ((rc = dev_alloc(d, &d->d_set_links, N * ((size_t)c.max_frames + 1) + 2))) return rc;
    if ((rc = dev_alloc(d, &d->d_lat_blocks, N * ((size_t)c.max_frames + 1)))) return rc;
    if ((rc = dev_alloc(d, &d->d_tok_first, N + 1))) return rc;
  }
  if (o.keep_token_records)
    HIP_TRY(d, hipHostMalloc(reinterpret_cast<void **>(&d->h_pinned), (kHostHead + kScratchFrames + 2) * sizeof(unsigned)));
  if (o.outputs_on_host) {
    if ((rc = dev_alloc(d, &d->o_words, N * (size_t)o.max_words))) return rc;
    if ((rc = dev_alloc(d, &d->o_nwords, N))) return rc;
    if ((rc = dev_alloc(d, &d->o_flags, N))) return rc;
    if ((rc = dev_alloc(d, &d->o_cost, N))) return rc;
  }
  HIP_TRY(d, hipDeviceSynchronize());
  return WFST_OK;
}

// Stage {channel, frames, io row} triples and launch one workgroup per entry.
// `slot`: whose pair of timing events brackets the kernel (n_slots = the calls that name channels).
int launch(wfst_decoder *d, const std::vector<int> &chan, const std::vector<int> &nfr,
           const std::vector<int> &io, LaunchArgs a, hipStream_t st, int slot_id = -1) {
  if (slot_id < 0) slot_id = d->n_slots;
  const int n = (int)chan.size();
  if (n == 0) return WFST_OK;
  const size_t N = (size_t)d->opts.max_channels;
  // workgroups of the launch: one per entry, or at most launch_workgroups, which then take the
  // entries in list order from a counter that travels with the lists
  const int n_wg = d->launch_workgroups > 0 ? std::min(n, d->launch_workgroups) : n;
  // (the lists live on the device until the kernel ends, since its workgroups read them as they go:
  // one area per batch slot, and one for the calls that name channels; calls that share an area do
  // not overlap in time, so the stream orders this copy after the last kernel that read the area)
  int *slot = d->d_params + (size_t)slot_id * (6 * N + 2);
  std::vector<int> &pack = d->h_params[d->ring_pos];
  pack.resize(6 * (size_t)n + 2);
  std::copy(chan.begin(), chan.end(), pack.begin());
  std::copy(nfr.begin(), nfr.end(), pack.begin() + n);
  std::copy(io.begin(), io.end(), pack.begin() + 2 * n);
  for (int i = 0; i < n; ++i) {
    pack[3 * (size_t)n + i] = (int)d->cur_capn[chan[i]];
    std::memcpy(&pack[4 * (size_t)n + 2 + 2 * (size_t)i], &d->cur_start[chan[i]], sizeof(unsigned long long));
  }
  pack[4 * (size_t)n] = n_wg; pack[4 * (size_t)n + 1] = 0;
  d->ring_pos = (d->ring_pos + 1) % wfst_decoder::kRing;
  HIP_TRY(d, hipMemcpyAsync(slot, pack.data(), pack.size() * sizeof(int), hipMemcpyHostToDevice, st));
  a.lists = slot; a.n_jobs = n;
  HIP_TRY(d, hipEventRecord(d->ev0[slot_id], st));
  bool boost = false;                          // does any channel of the launch have a boosting table or acceptor?
  for (int ch : chan) boost = boost || d->boost_on_dev[ch] > 0;
  const bool opt = d->c.cost_offset || d->c.recycle || d->c.tokrec || d->c.frame_best || d->c.dig_sum;
#define WFST_LAUNCH(NARROW, BOOST, PROF, OPT) \
  do { \
    if (n_wg < n) hipLaunchKernelGGL((wfst_channel_kernel<NARROW, BOOST, PROF, OPT, true>), dim3(n_wg), dim3(kBlock), 0, st, d->g, d->c, a); \
    else hipLaunchKernelGGL((wfst_channel_kernel<NARROW, BOOST, PROF, OPT, false>), dim3(n_wg), dim3(kBlock), 0, st, d->g, d->c, a); \
  } while (0)
  if (d->g.earc8) {                            // (no lean instances and no phase timing with narrow arc records)
    if (boost) WFST_LAUNCH(true, true, false, true); else WFST_LAUNCH(true, false, false, true);
  } else if (d->phase_timing) {
    if (boost) { if (opt) WFST_LAUNCH(false, true, true, true); else WFST_LAUNCH(false, true, true, false); }
    else { if (opt) WFST_LAUNCH(false, false, true, true); else WFST_LAUNCH(false, false, true, false); }
  } else {
    if (boost) { if (opt) WFST_LAUNCH(false, true, false, true); else WFST_LAUNCH(false, true, false, false); }
    else { if (opt) WFST_LAUNCH(false, false, false, true); else WFST_LAUNCH(false, false, false, false); }
  }
#undef WFST_LAUNCH
  HIP_TRY(d, hipGetLastError());
  HIP_TRY(d, hipEventRecord(d->ev1[slot_id], st));
  d->timed[slot_id] = 1;
  d->last_timed = slot_id;
  return WFST_OK;
}

// Share out the lattice pool of a slot among its first n channels in proportion to want[] (frames
// each will store) -- or, with want == nullptr, equally among all its channels -- and send the
// new placement to the device on `st`.  The arenas of the slot's channels move: none of them is
// initialised any more.
int partition_slot(wfst_decoder *d, int slot, const int32_t *want, int n, hipStream_t st) {
  const int sc = d->slot_channels, ch0 = slot * sc;
  std::vector<unsigned long long> &hs = d->h_start[d->part_pos]; std::vector<unsigned> &hc = d->h_capn[d->part_pos];
  d->part_pos = (d->part_pos + 1) % wfst_decoder::kRing;
  hs.assign(d->eq_start.begin() + ch0, d->eq_start.begin() + ch0 + sc);
  hc.assign(d->eq_capn.begin() + ch0, d->eq_capn.begin() + ch0 + sc);
  if (want) {
    const unsigned long long pool = (unsigned long long)sc * d->c.lat_cap;
    unsigned long long total = 0, at = d->eq_start[ch0];
    for (int b = 0; b < n; ++b) total += (unsigned long long)want[b] + 2;
    for (int b = 0; b < sc; ++b) {
      unsigned long long cap = b < n ? (unsigned long long)((long double)pool * ((unsigned long long)want[b] + 2) / (long double)total) : 0;
      cap = std::min<unsigned long long>(cap, 0x7ffffffeull);
      hs[b] = at; hc[b] = (unsigned)cap; at += cap;
    }
  }
  std::copy(hs.begin(), hs.end(), d->cur_start.begin() + ch0);
  std::copy(hc.begin(), hc.end(), d->cur_capn.begin() + ch0);
  HIP_TRY(d, hipMemcpyAsync(d->d_lat_start + ch0, hs.data(), sc * sizeof(unsigned long long), hipMemcpyHostToDevice, st));
  HIP_TRY(d, hipMemcpyAsync(d->d_lat_capn + ch0, hc.data(), sc * sizeof(unsigned), hipMemcpyHostToDevice, st));
  d->slot_by_length[slot] = want ? 1 : 0;
  std::fill(d->chan_ready.begin() + ch0, d->chan_ready.begin() + ch0 + sc, 0);
  return WFST_OK;
}

// Before a channel is initialised on its own: its slot's pool must be shared out equally.
int ready_for_init(wfst_decoder *d, int ch, hipStream_t st) {
  const int slot = ch / d->slot_channels;
  if (d->slot_by_length[slot]) { const int rc = partition_slot(d, slot, nullptr, 0, st); if (rc) return rc; }
  d->chan_ready[ch] = 1;
  return WFST_OK;
}

bool valid_prune(float beam, int max_active) { return beam >= 0.0f && max_active >= 1; }

// Give channel `ch` a boosting acceptor before its next init: n arcs (from state, output label, to
// state, score) over n_states states, root 0; from / to may be nullptr for the one-state acceptor
// (the paper's table word -> score).  n == 0: none.  The arcs become an open-addressing hash by
// label (key 0 = free) in the channel's slot; the copies are ordered on `st` before the init kernel.
int set_boost(wfst_decoder *d, int ch, int n_states, int n, const int32_t *from, const int32_t *label,
              const int32_t *to, const float *score, hipStream_t st) {
  if (n == 0 && d->boost_on_dev[ch] == 0) return WFST_OK;
  if (n < 0 || n > kBoostMax) return fail(d, WFST_ERR_INVALID_ARG, "boosting acceptor with more than " + std::to_string(kBoostMax) + " arcs");
  if (n > 0 && (!label || !score)) return fail(d, WFST_ERR_INVALID_ARG, "null boost arrays");
  if (n > 0 && n_states > 1) {
    if (!from || !to) return fail(d, WFST_ERR_INVALID_ARG, "null boost arrays");
    // a token's key holds (state of the acceptor, graph state) in 29 bits
    const int room = std::min(kBoostStateBits, 29 - d->g.blk_bits);
    if (n_states > (1 << room))
      return fail(d, WFST_ERR_INVALID_ARG, "boosting acceptor with " + std::to_string(n_states) + " states: a graph of " +
                                               std::to_string(d->g.n_blk) + " blocks leaves room for " + std::to_string(1 << room));
  }
  if (n > 0 && n_states < 1) return fail(d, WFST_ERR_INVALID_ARG, "a boosting acceptor needs at least its root state");
  int *h = d->h_boost + (size_t)ch * kBoostStage;
  int *keys = h; float *vals = reinterpret_cast<float *>(h + kBoostSlots);
  unsigned *ft = reinterpret_cast<unsigned *>(h + 2 * kBoostSlots); int *cnt = h + 3 * kBoostSlots;
  // the channel's staging area is pinned memory that earlier asynchronous copies may still be
  // reading (a boosted call returns before its copies have run): wait for them before rewriting it
  if (d->boost_ev.empty()) d->boost_ev.assign((size_t)d->opts.max_channels, nullptr);
  if (d->boost_ev[ch]) HIP_TRY(d, hipEventSynchronize(d->boost_ev[ch]));
  else HIP_TRY(d, hipEventCreateWithFlags(&d->boost_ev[ch], hipEventDisableTiming));
  std::memset(h, 0, kBoostStage * sizeof(int));
  for (int i = 0; i < n; ++i) {
    const int w = label[i];
    const int f = n_states > 1 ? from[i] : 0, t = n_states > 1 ? to[i] : 0;
    if (w <= 0) return fail(d, WFST_ERR_INVALID_ARG, "boost labels must be positive output labels");
    if (!std::isfinite(score[i])) return fail(d, WFST_ERR_INVALID_ARG, "non-finite boost score");
    if (f < 0 || f >= n_states || t < 0 || t >= n_states) return fail(d, WFST_ERR_INVALID_ARG, "boosting acceptor: state out of range");
    unsigned s = boost_slot(w);
    while (keys[s] != 0) {
      if (keys[s] == w && (int)(ft[s] & 0xffffu) == f)
        return fail(d, WFST_ERR_INVALID_ARG, n_states > 1 ? "boosting acceptor: two arcs with label " + std::to_string(w) + " out of one state"
                                                          : "word id " + std::to_string(w) + " appears twice in the boost table");
      s = (s + 1) & (kBoostSlots - 1);
    }
    keys[s] = w; vals[s] = score[i]; ft[s] = (unsigned)f | ((unsigned)t << 16);
  }
  cnt[0] = n; cnt[1] = n > 0 ? n_states : 0;
  if (n > 0) {
    HIP_TRY(d, hipMemcpyAsync(d->c.boost_keys + (size_t)ch * kBoostSlots, keys, kBoostSlots * sizeof(int), hipMemcpyHostToDevice, st));
    HIP_TRY(d, hipMemcpyAsync(d->c.boost_vals + (size_t)ch * kBoostSlots, vals, kBoostSlots * sizeof(float), hipMemcpyHostToDevice, st));
    HIP_TRY(d, hipMemcpyAsync(d->c.boost_from_to + (size_t)ch * kBoostSlots, ft, kBoostSlots * sizeof(unsigned), hipMemcpyHostToDevice, st));
  }
  static_assert(offsetof(ChanState, boost_states) == offsetof(ChanState, boost_n) + sizeof(int), "the two are copied together");
  HIP_TRY(d, hipMemcpyAsync(&d->c.st[ch].boost_n, cnt, 2 * sizeof(int), hipMemcpyHostToDevice, st));
  HIP_TRY(d, hipEventRecord(d->boost_ev[ch], st));
  d->boost_on_dev[ch] = n;
  return WFST_OK;
}
int set_boost(wfst_decoder *d, int ch, const wfst_boost_table *t, hipStream_t st) {
  return t ? set_boost(d, ch, 1, t->n, nullptr, t->word_ids, nullptr, t->scores, st)
           : set_boost(d, ch, 1, 0, nullptr, nullptr, nullptr, nullptr, st);
}
int set_boost(wfst_decoder *d, int ch, const wfst_boost_fst *f, hipStream_t st) {
  return f ? set_boost(d, ch, f->n_states, f->n_arcs, f->arc_from, f->arc_label, f->arc_to, f->arc_score, st)
           : set_boost(d, ch, 1, 0, nullptr, nullptr, nullptr, nullptr, st);
}

// ---- scratch of the entry point that allocates nothing
// Device memory for the lattice kernels' counters and per-set link counts that belongs to the
// loaded code object instead of to an allocation: every GPU the library runs on holds its own
// copy for the life of the process.  In host code the array's NAME is only a handle; the address
// each device holds is asked for once per device (scratch_address) and kept.
}  // namespace
static __device__ __align__(256) unsigned long long scratch[kScratchWords];
namespace {
std::mutex g_scratch_mu;
unsigned long long *g_scratch_ptr[kScratchDevices] = {};

// Address of `scratch` on the current device (asked for once per device, with that device current).
int scratch_address(wfst_decoder *d, unsigned long long **out) {
  int dev = -1;
  HIP_TRY(d, hipGetDevice(&dev));
  if (dev < 0 || dev >= kScratchDevices) return fail(d, WFST_ERR_HIP, "device ordinal beyond the scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(d, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(d, WFST_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = static_cast<unsigned long long *>(p);
  }
  *out = g_scratch_ptr[dev];
  return WFST_OK;
}

// Both lattice entry points: `ctr` (2 words) and `set_links` (frames + 2 words) are DEVICE scratch,
// `off` is HOST scratch for frames + 2 offsets; frames_cap is what those hold.
int get_lattice_impl(wfst_decoder *d, int32_t ch, const void *loglikes, float lattice_beam,
                     int32_t *tok_state, float *tok_cost, int64_t tok_cap, int64_t *frame_off,
                     wfst_lattice_link *links, int64_t link_cap, int64_t *n_tokens, int64_t *n_links,
                     hipStream_t st, unsigned long long *ctr_dev, unsigned long long *set_links_dev,
                     unsigned *host, int frames_cap) {
  // `host`: kHostHead words for the channel state and the two counters, then frames_cap + 2 offsets
  static_assert(sizeof(ChanState) + 2 * sizeof(unsigned long long) <= kHostHead * sizeof(unsigned), "head too small");
  ChanState &s = *reinterpret_cast<ChanState *>(host);
  unsigned long long *ctr = reinterpret_cast<unsigned long long *>(host + kHostHead - 4);
  unsigned *off = host + kHostHead;
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  if (!frame_off || !n_tokens || !n_links || tok_cap < 0 || link_cap < 0 || (tok_cap && (!tok_state || !tok_cost)) ||
      (link_cap && !links))
    return fail(d, WFST_ERR_INVALID_ARG, "null output or negative capacity");
  if (!(lattice_beam >= 0.0f)) return fail(d, WFST_ERR_INVALID_ARG, "lattice_beam must be >= 0");
  // first of two synchronisations: the channel's state and its frame offsets (as many as the host
  // buffer holds; which of them are in use is known from the state)
  const int n_off = std::min(d->c.max_frames, frames_cap) + 2;
  HIP_TRY(d, hipMemcpyAsync(&s, d->c.st + ch, sizeof(s), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipMemcpyAsync(off, d->c.frame_off + (size_t)ch * (d->c.max_frames + 2), (size_t)n_off * sizeof(unsigned),
                            hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipStreamSynchronize(st));
  if (s.status & (kStLattice | kStCapacity))
    return fail(d, WFST_ERR_CAPACITY, "the channel stopped on an overflow: its token sets are incomplete");
  if (s.boost_n > 0 && s.boost_states > 1)
    return fail(d, WFST_ERR_INVALID_ARG, "lattices are defined over graph states: not available for a channel decoded "
                                         "with a boosting acceptor of several states");
  const int f = s.frame;
  if (f < 0 || f > frames_cap)
    return fail(d, WFST_ERR_CAPACITY, "the channel has " + std::to_string(f) + " frames; this call takes at most " +
                                          std::to_string(frames_cap));
  if (f > 0 && !loglikes) return fail(d, WFST_ERR_INVALID_ARG, "null loglikes");
  // the counters must start at zero; the per-set counts are all written by the first run
  HIP_TRY(d, hipMemsetAsync(ctr_dev, 0, 2 * sizeof(unsigned long long), st));
  for (int t = 0; t <= f + 1; ++t) frame_off[t] = (int64_t)off[t];
  *n_tokens = (int64_t)off[(size_t)f + 1];
  LatticeArgs a{};
  a.ch = ch; a.frames = f; a.ll = loglikes; a.V = d->V; a.ll_dtype = d->opts.loglike_dtype;
  a.lattice_beam = lattice_beam;
  a.tok_state = tok_state; a.tok_cost = tok_cost; a.tok_cap = tok_cap;
  a.links = links; a.link_cap = link_cap; a.ctr = ctr_dev; a.set_links = set_links_dev;
  a.write = 0;                                  // first run: links per set
  hipLaunchKernelGGL(wfst_lattice_kernel, dim3(f + 1), dim3(kBlock), 0, st, d->g, d->c, a);
  HIP_TRY(d, hipGetLastError());
  hipLaunchKernelGGL(wfst_lattice_scan, dim3(1), dim3(kBlock), 0, st, set_links_dev, f + 1, ctr_dev);
  HIP_TRY(d, hipGetLastError());
  if (link_cap > 0 && *n_tokens <= tok_cap) {
    // second run, queued right behind the scan: every set writes its links at its place; entries
    // beyond link_cap are not written, so nothing has to be known on the host before it starts
    a.write = 1;
    hipLaunchKernelGGL(wfst_lattice_kernel, dim3(f + 1), dim3(kBlock), 0, st, d->g, d->c, a);
    HIP_TRY(d, hipGetLastError());
  }
  ctr[0] = ctr[1] = 0;
  HIP_TRY(d, hipMemcpyAsync(ctr, ctr_dev, 2 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipStreamSynchronize(st));         // second and last synchronisation
  *n_links = (int64_t)ctr[0];
  if (ctr[1]) return fail(d, WFST_ERR_CAPACITY, "lattice kernel: a token set overflowed its lookup table");
  if (*n_tokens > tok_cap || *n_links > link_cap)
    return fail(d, WFST_ERR_CAPACITY, "lattice needs room for " + std::to_string(*n_tokens) + " tokens and " +
                                          std::to_string(*n_links) + " links");
  return WFST_OK;
}

// wfst_get_lattice for n channels at once: one count run, one scan and one write run over all
// their token sets, two synchronisations.
int get_lattice_batch_impl(wfst_decoder *d, const int32_t *channels, int32_t n, const void *loglikes, int32_t T,
                           float lattice_beam, int32_t *tok_state, float *tok_cost, int64_t tok_cap,
                           int64_t *frame_off, wfst_lattice_link *links, int64_t link_cap,
                           int64_t *tok_first, int64_t *link_first, hipStream_t st) {
  const int N = d->opts.max_channels, F = d->c.max_frames;
  if (n < 0 || (n && !channels) || !frame_off || !tok_first || !link_first || tok_cap < 0 || link_cap < 0 ||
      (tok_cap && (!tok_state || !tok_cost)) || (link_cap && !links) || T < 0)
    return fail(d, WFST_ERR_INVALID_ARG, "null argument or negative size");
  if (!(lattice_beam >= 0.0f)) return fail(d, WFST_ERR_INVALID_ARG, "lattice_beam must be >= 0");
  tok_first[0] = link_first[0] = 0;
  if (n == 0) return WFST_OK;
  int lo = N, hi = -1;
  {
    std::vector<char> seen((size_t)N, 0);
    for (int k = 0; k < n; ++k) {
      const int ch = channels[k];
      if (ch < 0 || ch >= N) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
      if (seen[ch]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel " + std::to_string(ch) + " listed twice");
      seen[ch] = 1; lo = std::min(lo, ch); hi = std::max(hi, ch);
    }
  }
  // pinned staging: states and frame offsets of channels lo..hi, the workgroup list, where each channel's
  // tokens start, the scanned links per workgroup, the counters
  const size_t n_blocks_max = (size_t)N * ((size_t)F + 1);
  const size_t b_state = 0, b_off = b_state + (size_t)N * sizeof(ChanState),
               b_blocks = (b_off + (size_t)N * ((size_t)F + 2) * sizeof(unsigned) + 15) / 16 * 16,
               b_first = b_blocks + n_blocks_max * sizeof(int4), b_links = b_first + ((size_t)N + 1) * sizeof(long long),
               b_ctr = b_links + (n_blocks_max + 2) * sizeof(unsigned long long), b_end = b_ctr + 2 * sizeof(unsigned long long);
  if (!d->h_lat_batch) {
    HIP_TRY(d, hipHostMalloc(reinterpret_cast<void **>(&d->h_lat_batch), b_end));
    d->h_lat_batch_bytes = b_end;
  }
  char *H = d->h_lat_batch;
  ChanState *hs = reinterpret_cast<ChanState *>(H + b_state);
  unsigned *hoff = reinterpret_cast<unsigned *>(H + b_off);
  int4 *hblk = reinterpret_cast<int4 *>(H + b_blocks);
  long long *hfirst = reinterpret_cast<long long *>(H + b_first);
  unsigned long long *hlinks = reinterpret_cast<unsigned long long *>(H + b_links);
  unsigned long long *hctr = reinterpret_cast<unsigned long long *>(H + b_ctr);
  // first synchronisation: what the channels hold
  HIP_TRY(d, hipMemcpyAsync(hs + lo, d->c.st + lo, (size_t)(hi - lo + 1) * sizeof(ChanState), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipMemcpyAsync(hoff + (size_t)lo * (F + 2), d->c.frame_off + (size_t)lo * (F + 2),
                            (size_t)(hi - lo + 1) * (F + 2) * sizeof(unsigned), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipStreamSynchronize(st));
  size_t nb = 0; long long ntok = 0;
  for (int k = 0; k < n; ++k) {
    const int ch = channels[k];
    const ChanState &s = hs[ch];
    if (s.status & (kStLattice | kStCapacity))
      return fail(d, WFST_ERR_CAPACITY, "channel " + std::to_string(ch) + " stopped on an overflow: its token sets are incomplete");
    if (s.boost_n > 0 && s.boost_states > 1)
      return fail(d, WFST_ERR_INVALID_ARG, "lattices are defined over graph states: not available for a channel decoded "
                                           "with a boosting acceptor of several states");
    const int f = s.frame;
    if (f < 0 || f > F || f > T)
      return fail(d, WFST_ERR_INVALID_ARG, "channel " + std::to_string(ch) + " has " + std::to_string(f) +
                                               " frames, more than the T = " + std::to_string(T) + " rows per channel");
    if (f > 0 && !loglikes) return fail(d, WFST_ERR_INVALID_ARG, "null loglikes");
    const unsigned *off = hoff + (size_t)ch * (F + 2);
    int64_t *fo = frame_off + (size_t)k * ((size_t)T + 2);
    for (int t = 0; t <= f + 1; ++t) fo[t] = (int64_t)off[t];
    for (int t = f + 2; t < T + 2; ++t) fo[t] = (int64_t)off[f + 1];
    hfirst[k] = ntok; tok_first[k] = ntok;
    for (int t = 0; t <= f; ++t) hblk[nb++] = make_int4(ch, t, k, 0);
    ntok += (long long)off[(size_t)f + 1];
  }
  hfirst[n] = ntok; tok_first[n] = ntok;
  HIP_TRY(d, hipMemcpyAsync(d->d_lat_blocks, hblk, nb * sizeof(int4), hipMemcpyHostToDevice, st));
  HIP_TRY(d, hipMemcpyAsync(d->d_tok_first, hfirst, ((size_t)n + 1) * sizeof(long long), hipMemcpyHostToDevice, st));
  HIP_TRY(d, hipMemsetAsync(d->d_lat_ctr, 0, 2 * sizeof(unsigned long long), st));
  LatticeArgs a{};
  a.ch = 0; a.frames = 0; a.ll = loglikes; a.V = d->V; a.ll_dtype = d->opts.loglike_dtype;
  a.lattice_beam = lattice_beam;
  a.tok_state = tok_state; a.tok_cost = tok_cost; a.tok_cap = tok_cap;
  a.links = links; a.link_cap = link_cap; a.ctr = d->d_lat_ctr; a.set_links = d->d_set_links;
  a.blocks = d->d_lat_blocks; a.tok_first = d->d_tok_first; a.ll_stride = (long long)T * d->V;
  a.write = 0;
  hipLaunchKernelGGL(wfst_lattice_kernel, dim3((unsigned)nb), dim3(kBlock), 0, st, d->g, d->c, a);
  HIP_TRY(d, hipGetLastError());
  hipLaunchKernelGGL(wfst_lattice_scan, dim3(1), dim3(kBlock), 0, st, d->d_set_links, (int)nb, d->d_lat_ctr);
  HIP_TRY(d, hipGetLastError());
  if (link_cap > 0 && ntok <= tok_cap) {
    a.write = 1;
    hipLaunchKernelGGL(wfst_lattice_kernel, dim3((unsigned)nb), dim3(kBlock), 0, st, d->g, d->c, a);
    HIP_TRY(d, hipGetLastError());
  }
  hctr[0] = hctr[1] = 0;
  HIP_TRY(d, hipMemcpyAsync(hlinks, d->d_set_links, nb * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipMemcpyAsync(hctr, d->d_lat_ctr, 2 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
  HIP_TRY(d, hipStreamSynchronize(st));         // second and last synchronisation
  {
    size_t b = 0;
    for (int k = 0; k < n; ++k) { link_first[k] = (int64_t)hlinks[b]; b += (size_t)hs[channels[k]].frame + 1; }
    link_first[n] = (int64_t)hctr[0];
  }
  if (hctr[1]) return fail(d, WFST_ERR_CAPACITY, "lattice kernel: a token set overflowed its lookup table");
  if (ntok > tok_cap || link_first[n] > link_cap)
    return fail(d, WFST_ERR_CAPACITY, "the lattices need room for " + std::to_string(ntok) + " tokens and " +
                                          std::to_string(link_first[n]) + " links");
  return WFST_OK;
}

}  // namespace

namespace {
int decode_batch_impl(wfst_decoder *d, int slot, const void *loglikes, const int32_t *lengths, int32_t B,
                      int32_t T, int32_t V, float beam, int32_t max_active,
                      const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts, void *stream,
                      int32_t *words, int32_t *nwords, float *cost, int32_t *flags);
}

extern "C" {

int32_t wfst_decoder_create(const wfst_graph_csr *graph, const wfst_opts *opts, wfst_decoder **out) {
  if (!graph || !opts || !out) return fail(nullptr, WFST_ERR_INVALID_ARG, "null argument");
  *out = nullptr;
  if (opts->max_channels < 1 || opts->max_frames_per_channel < 1 || opts->max_words < 1)
    return fail(nullptr, WFST_ERR_INVALID_ARG, "max_channels, max_frames_per_channel and max_words must be >= 1");
  if (opts->loglike_dtype < WFST_LOGLIKE_F32 || opts->loglike_dtype > WFST_LOGLIKE_BF16)
    return fail(nullptr, WFST_ERR_INVALID_ARG, "loglike_dtype must be WFST_LOGLIKE_F32, _F16 or _BF16");
  if (opts->candidate_capacity < 0 || (opts->candidate_capacity > 0 && opts->candidate_capacity < 4096))
    return fail(nullptr, WFST_ERR_INVALID_ARG, "candidate_capacity must be 0 or >= 4096");
  if (graph->num_classes > kMaxV)
    return fail(nullptr, WFST_ERR_INVALID_ARG, "num_classes above " + std::to_string(kMaxV));
  std::string why; int64_t Ae = 0, Ax = 0;
  int rc = validate_graph(graph, why, Ae, Ax);
  if (rc) return fail(nullptr, rc, why);
  if (opts->batch_slots < 0 || (opts->batch_slots > 1 && opts->max_channels % opts->batch_slots != 0))
    return fail(nullptr, WFST_ERR_INVALID_ARG, "batch_slots must be >= 0 and divide max_channels");
  if (opts->recycle_lattice && opts->keep_token_records)
    return fail(nullptr, WFST_ERR_INVALID_ARG, "recycle_lattice and keep_token_records exclude each other (a lattice needs every frame)");
  wfst_decoder *d = new wfst_decoder();
  d->opts = *opts; d->V = graph->num_classes;
  d->n_slots = std::max(1, opts->batch_slots); d->slot_channels = opts->max_channels / d->n_slots;
  rc = upload_graph(d, graph);
  if (!rc) rc = alloc_channels(d);
  d->ev0.assign((size_t)d->n_slots + 1, nullptr); d->ev1.assign((size_t)d->n_slots + 1, nullptr);
  d->timed.assign((size_t)d->n_slots + 1, 0);
  for (int i = 0; !rc && i <= d->n_slots; ++i)
    if (hipEventCreate(&d->ev0[i]) != hipSuccess || hipEventCreate(&d->ev1[i]) != hipSuccess) {
      d->err = "hipEventCreate failed"; rc = WFST_ERR_HIP;
    }
  if (rc) { g_create_err = d->err; wfst_decoder_destroy(d); return rc; }
  {
    // learn this device's address of the static scratch now rather than in the first call that needs it
    unsigned long long *p = nullptr;
    if (scratch_address(d, &p) != WFST_OK) { d->err.clear(); (void)hipGetLastError(); }
  }
  *out = d;
  return WFST_OK;
}

int32_t wfst_decoder_destroy(wfst_decoder *d) {
  if (!d) return WFST_OK;
  (void)hipDeviceSynchronize();
  for (void *p : d->allocs) (void)hipFree(p);
  if (d->h_boost) (void)hipHostFree(d->h_boost);
  if (d->h_pinned) (void)hipHostFree(d->h_pinned);
  if (d->h_lat_batch) (void)hipHostFree(d->h_lat_batch);
  for (hipEvent_t e : d->ev0) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : d->ev1) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : d->boost_ev) if (e) (void)hipEventDestroy(e);
  delete d;
  return WFST_OK;
}

int32_t wfst_decode_batch(wfst_decoder *d, const float *loglikes, const int32_t *lengths, int32_t B,
                          int32_t T, int32_t V, float beam, int32_t max_active, void *stream,
                          int32_t *words, int32_t *nwords, float *cost, int32_t *flags) {
  return wfst_decode_batch_boosted(d, loglikes, lengths, B, T, V, beam, max_active, nullptr, stream,
                                   words, nwords, cost, flags);
}

int32_t wfst_decode_batch_boosted(wfst_decoder *d, const float *loglikes, const int32_t *lengths, int32_t B,
                                  int32_t T, int32_t V, float beam, int32_t max_active,
                                  const wfst_boost_table *const *boosts, void *stream,
                                  int32_t *words, int32_t *nwords, float *cost, int32_t *flags) {
  return decode_batch_impl(d, 0, loglikes, lengths, B, T, V, beam, max_active, boosts, nullptr, stream, words, nwords,
                           cost, flags);
}

int32_t wfst_decode_batch_boost_fst(wfst_decoder *d, const float *loglikes, const int32_t *lengths, int32_t B,
                                    int32_t T, int32_t V, float beam, int32_t max_active,
                                    const wfst_boost_fst *const *fsts, void *stream,
                                    int32_t *words, int32_t *nwords, float *cost, int32_t *flags) {
  return decode_batch_impl(d, 0, loglikes, lengths, B, T, V, beam, max_active, nullptr, fsts, stream, words, nwords,
                           cost, flags);
}

int32_t wfst_decode_batch_slot(wfst_decoder *d, int32_t slot, const void *loglikes, const int32_t *lengths, int32_t B,
                               int32_t T, int32_t V, float beam, int32_t max_active,
                               const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts, void *stream,
                               int32_t *words, int32_t *nwords, float *cost, int32_t *flags) {
  if (d && boosts && fsts) return fail(d, WFST_ERR_INVALID_ARG, "give word-boost tables or boosting acceptors, not both");
  return decode_batch_impl(d, slot, loglikes, lengths, B, T, V, beam, max_active, boosts, fsts, stream, words, nwords,
                           cost, flags);
}

int32_t wfst_init_channel_boost_fst(wfst_decoder *d, int32_t ch, float beam, int32_t max_active,
                                    const wfst_boost_fst *fst, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  if (!valid_prune(beam, max_active)) return fail(d, WFST_ERR_INVALID_ARG, "beam must be >= 0 and max_active >= 1");
  const int rcb = set_boost(d, ch, fst, static_cast<hipStream_t>(stream));
  if (rcb) return rcb;
  const int rcr = ready_for_init(d, ch, static_cast<hipStream_t>(stream));
  if (rcr) return rcr;
  LaunchArgs a{};
  a.V = d->V; a.mode = kModeInit;
  a.beam = beam; a.scale = 256.0f / beam; a.max_active = max_active;
  return launch(d, {ch}, {0}, {0}, a, static_cast<hipStream_t>(stream));
}

}  // extern "C"

namespace {
int decode_batch_impl(wfst_decoder *d, int slot, const void *loglikes, const int32_t *lengths, int32_t B,
                      int32_t T, int32_t V, float beam, int32_t max_active,
                      const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts, void *stream,
                      int32_t *words, int32_t *nwords, float *cost, int32_t *flags) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (slot < 0 || slot >= d->n_slots) return fail(d, WFST_ERR_INVALID_ARG, "batch slot out of range");
  const int ch0 = slot * d->slot_channels;
  if (B < 0 || T < 0) return fail(d, WFST_ERR_INVALID_ARG, "negative B or T");
  if (B == 0) return WFST_OK;              // nothing to decode; pointers may be null
  if (!lengths || !words || !nwords || !cost || !flags || (T > 0 && !loglikes))
    return fail(d, WFST_ERR_INVALID_ARG, "null argument");
  if (V != d->V) return fail(d, WFST_ERR_INVALID_ARG, "V differs from the graph's num_classes");
  if (!valid_prune(beam, max_active)) return fail(d, WFST_ERR_INVALID_ARG, "beam must be >= 0 and max_active >= 1");
  if (B > d->slot_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "batch larger than the channels of a slot (max_channels / batch_slots)");
  for (int b = 0; b < B; ++b)
    if (lengths[b] < 0 || lengths[b] > T || lengths[b] > d->opts.max_frames_per_channel)
      return fail(d, WFST_ERR_INVALID_ARG, "lengths[" + std::to_string(b) + "] outside [0, min(T, max_frames_per_channel)]");
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int b = 0; b < B; ++b) {
    const int rcb = fsts ? set_boost(d, ch0 + b, fsts[b], st) : set_boost(d, ch0 + b, boosts ? boosts[b] : nullptr, st);
    if (rcb) return rcb;
  }
  // the slot's lattice memory: in proportion to the utterances' lengths if the decoder was created
  // for that, else the equal shares (put back if a by-length batch left them otherwise)
  if (d->opts.lattice_by_length && !d->c.recycle) {
    const int rcp = partition_slot(d, slot, lengths, B, st);
    if (rcp) return rcp;
  } else if (d->slot_by_length[slot]) {
    const int rcp = partition_slot(d, slot, nullptr, 0, st);
    if (rcp) return rcp;
  }
  for (int b = 0; b < B; ++b) d->chan_ready[ch0 + b] = 1;
  // longest utterances first: workgroups are dispatched in order, so the long ones start
  // at once and the short ones fill in behind them
  std::vector<int> order(B), nfr(B), chan(B);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return lengths[x] > lengths[y]; });
  for (int i = 0; i < B; ++i) { nfr[i] = lengths[order[i]]; chan[i] = ch0 + order[i]; }
  const bool host_out = d->opts.outputs_on_host != 0;
  LaunchArgs a{};
  a.ll = loglikes; a.ll_stride = (long long)T * V; a.V = V; a.ll_dtype = d->opts.loglike_dtype;
  a.mode = kModeInit | kModeFinal; a.finalize = 1;
  a.beam = beam; a.scale = 256.0f / beam; a.max_active = max_active;
  // (host outputs are staged in device memory per channel, so the slots do not share any of it)
  const size_t mw = (size_t)d->opts.max_words;
  a.words = host_out ? d->o_words + ch0 * mw : words; a.nwords = host_out ? d->o_nwords + ch0 : nwords;
  a.cost = host_out ? d->o_cost + ch0 : cost;         a.flags = host_out ? d->o_flags + ch0 : flags;
  a.max_words = d->opts.max_words;
  int rc = launch(d, chan, nfr, order, a, st, slot);
  if (rc) return rc;
  if (host_out) {
    HIP_TRY(d, hipMemcpyAsync(words, d->o_words + ch0 * mw, B * mw * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(nwords, d->o_nwords + ch0, B * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(cost, d->o_cost + ch0, B * sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(flags, d->o_flags + ch0, B * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipStreamSynchronize(st));
    for (int b = 0; b < B; ++b) {
      if (flags[b] & WFST_FLAG_LATTICE_OVERFLOW) return fail(d, WFST_ERR_LATTICE_OVERFLOW, "utterance " + std::to_string(b) + " ran out of lattice memory");
      if (flags[b] & WFST_FLAG_CAPACITY) return fail(d, WFST_ERR_CAPACITY, "utterance " + std::to_string(b) + " overflowed a work buffer");
    }
  }
  return WFST_OK;
}

}  // namespace

extern "C" {

int32_t wfst_init_channel(wfst_decoder *d, int32_t ch, float beam, int32_t max_active,
                          const wfst_boost_table *boost, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  if (!valid_prune(beam, max_active)) return fail(d, WFST_ERR_INVALID_ARG, "beam must be >= 0 and max_active >= 1");
  const int rcb = set_boost(d, ch, boost, static_cast<hipStream_t>(stream));
  if (rcb) return rcb;
  const int rcr = ready_for_init(d, ch, static_cast<hipStream_t>(stream));
  if (rcr) return rcr;
  LaunchArgs a{};
  a.V = d->V; a.mode = kModeInit;
  a.beam = beam; a.scale = 256.0f / beam; a.max_active = max_active;
  return launch(d, {ch}, {0}, {0}, a, static_cast<hipStream_t>(stream));
}

namespace {
int init_channels_impl(wfst_decoder *d, const int32_t *channels, int32_t n, float beam, int32_t max_active,
                       const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts, void *stream);
}

int32_t wfst_init_channels(wfst_decoder *d, const int32_t *channels, int32_t n, float beam, int32_t max_active,
                           const wfst_boost_table *const *boosts, void *stream) {
  return init_channels_impl(d, channels, n, beam, max_active, boosts, nullptr, stream);
}

int32_t wfst_init_channels_boost_fst(wfst_decoder *d, const int32_t *channels, int32_t n, float beam,
                                     int32_t max_active, const wfst_boost_fst *const *fsts, void *stream) {
  return init_channels_impl(d, channels, n, beam, max_active, nullptr, fsts, stream);
}

}  // extern "C"

namespace {
int init_channels_impl(wfst_decoder *d, const int32_t *channels, int32_t n, float beam, int32_t max_active,
                       const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (n < 0 || (n > 0 && !channels)) return fail(d, WFST_ERR_INVALID_ARG, "null or negative argument");
  if (n == 0) return WFST_OK;
  if (!valid_prune(beam, max_active)) return fail(d, WFST_ERR_INVALID_ARG, "beam must be >= 0 and max_active >= 1");
  if (n > d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "more channels than max_channels");
  std::vector<char> seen(d->opts.max_channels, 0);
  std::vector<int> chan(n), zero(n, 0);
  for (int i = 0; i < n; ++i) {
    if (channels[i] < 0 || channels[i] >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
    if (seen[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel listed twice");
    seen[channels[i]] = 1;
    chan[i] = channels[i];
  }
  for (int i = 0; i < n; ++i) {
    const int rcb = fsts ? set_boost(d, chan[i], fsts[i], static_cast<hipStream_t>(stream))
                         : set_boost(d, chan[i], boosts ? boosts[i] : nullptr, static_cast<hipStream_t>(stream));
    if (rcb) return rcb;
    const int rcr = ready_for_init(d, chan[i], static_cast<hipStream_t>(stream));
    if (rcr) return rcr;
  }
  LaunchArgs a{};
  a.V = d->V; a.mode = kModeInit;
  a.beam = beam; a.scale = 256.0f / beam; a.max_active = max_active;
  return launch(d, chan, zero, zero, a, static_cast<hipStream_t>(stream));   // one workgroup per channel, one launch
}
}  // namespace

extern "C" {

int32_t wfst_advance_chunk(wfst_decoder *d, const int32_t *channels, int32_t n, const float *loglikes,
                           const int32_t *nframes, int32_t C, int32_t V, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (n < 0 || C < 0 || !channels || !nframes || (n > 0 && C > 0 && !loglikes))
    return fail(d, WFST_ERR_INVALID_ARG, "null or negative argument");
  if (V != d->V) return fail(d, WFST_ERR_INVALID_ARG, "V differs from the graph's num_classes");
  if (n > d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "more channels than max_channels");
  std::vector<char> seen(d->opts.max_channels, 0);
  std::vector<int> chan(n), nfr(n), io(n);
  for (int i = 0; i < n; ++i) {
    if (channels[i] < 0 || channels[i] >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
    if (seen[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel listed twice");
    seen[channels[i]] = 1;
    if (!d->chan_ready[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel " + std::to_string(channels[i]) + " has not been initialised (or a batch decode has since taken its slot's lattice memory)");
    if (nframes[i] < 0 || nframes[i] > C) return fail(d, WFST_ERR_INVALID_ARG, "nframes outside [0, C]");
    chan[i] = channels[i]; nfr[i] = nframes[i]; io[i] = i;
  }
  LaunchArgs a{};
  a.ll = loglikes; a.ll_stride = (long long)C * V; a.V = V; a.mode = 0; a.ll_dtype = d->opts.loglike_dtype;
  return launch(d, chan, nfr, io, a, static_cast<hipStream_t>(stream));
}

int32_t wfst_advance_chunk_partial(wfst_decoder *d, const int32_t *channels, int32_t n, const float *loglikes,
                                   const int32_t *nframes, int32_t C, int32_t V, int32_t finalize,
                                   int32_t *words, int32_t *nwords, float *cost, int32_t *flags, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (n < 0 || C < 0 || (n > 0 && (!channels || !nframes)) || (n > 0 && C > 0 && !loglikes))
    return fail(d, WFST_ERR_INVALID_ARG, "null or negative argument");
  if (n == 0) return WFST_OK;
  if (!words || !nwords || !cost || !flags) return fail(d, WFST_ERR_INVALID_ARG, "null output");
  if (V != d->V) return fail(d, WFST_ERR_INVALID_ARG, "V differs from the graph's num_classes");
  if (n > d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "more channels than max_channels");
  std::vector<char> seen(d->opts.max_channels, 0);
  std::vector<int> chan(n), nfr(n), io(n);
  for (int i = 0; i < n; ++i) {
    if (channels[i] < 0 || channels[i] >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
    if (seen[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel listed twice");
    seen[channels[i]] = 1;
    if (!d->chan_ready[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel " + std::to_string(channels[i]) + " has not been initialised (or a batch decode has since taken its slot's lattice memory)");
    if (nframes[i] < 0 || nframes[i] > C) return fail(d, WFST_ERR_INVALID_ARG, "nframes outside [0, C]");
    chan[i] = channels[i]; nfr[i] = nframes[i]; io[i] = i;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool host_out = d->opts.outputs_on_host != 0;
  // one launch: every channel's workgroup consumes its frames and then, with the token set still
  // at hand, chooses the best token and walks the new part of its path
  LaunchArgs a{};
  a.ll = loglikes; a.ll_stride = (long long)C * V; a.V = V; a.ll_dtype = d->opts.loglike_dtype;
  a.mode = kModeFinal; a.finalize = finalize ? 1 : 0;
  a.words = host_out ? d->o_words : words; a.nwords = host_out ? d->o_nwords : nwords;
  a.cost = host_out ? d->o_cost : cost;    a.flags = host_out ? d->o_flags : flags;
  a.max_words = d->opts.max_words;
  int rc = launch(d, chan, nfr, io, a, st);
  if (rc) return rc;
  if (host_out) {
    const size_t mw = (size_t)d->opts.max_words;
    HIP_TRY(d, hipMemcpyAsync(words, d->o_words, n * mw * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(nwords, d->o_nwords, n * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(cost, d->o_cost, n * sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(flags, d->o_flags, n * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipStreamSynchronize(st));
  }
  return WFST_OK;
}

int32_t wfst_get_partial(wfst_decoder *d, int32_t ch, int32_t finalize, int32_t *words, int32_t cap,
                         int32_t *nwords, float *cost, int32_t *flags, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (!words || !nwords || !cost || !flags || cap < 1) return fail(d, WFST_ERR_INVALID_ARG, "null output or cap < 1");
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool host_out = d->opts.outputs_on_host != 0;
  if (host_out && cap > d->opts.max_words) cap = d->opts.max_words;
  LaunchArgs a{};
  a.V = d->V; a.mode = kModeFinal; a.finalize = finalize ? 1 : 0;
  a.words = host_out ? d->o_words : words; a.nwords = host_out ? d->o_nwords : nwords;
  a.cost = host_out ? d->o_cost : cost;    a.flags = host_out ? d->o_flags : flags;
  a.max_words = cap;
  int rc = launch(d, {ch}, {0}, {0}, a, st);
  if (rc) return rc;
  if (host_out) {
    HIP_TRY(d, hipMemcpyAsync(nwords, d->o_nwords, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(cost, d->o_cost, sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(flags, d->o_flags, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(words, d->o_words, (size_t)cap * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipStreamSynchronize(st));
  }
  return WFST_OK;
}

int32_t wfst_get_partial_batch(wfst_decoder *d, const int32_t *channels, int32_t n, int32_t finalize,
                               int32_t *words, int32_t *nwords, float *cost, int32_t *flags, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (n < 0) return fail(d, WFST_ERR_INVALID_ARG, "negative n");
  if (n == 0) return WFST_OK;
  if (!channels || !words || !nwords || !cost || !flags) return fail(d, WFST_ERR_INVALID_ARG, "null argument");
  if (n > d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "more channels than max_channels");
  std::vector<int> chan(n), nfr(n, 0), io(n);
  std::vector<char> seen(d->opts.max_channels, 0);
  for (int i = 0; i < n; ++i) {
    if (channels[i] < 0 || channels[i] >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
    // two workgroups on one channel would both rewrite the marks of its traced path
    if (seen[channels[i]]) return fail(d, WFST_ERR_BAD_CHANNEL, "channel listed twice");
    seen[channels[i]] = 1;
    chan[i] = channels[i]; io[i] = i;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool host_out = d->opts.outputs_on_host != 0;
  LaunchArgs a{};
  a.V = d->V; a.mode = kModeFinal; a.finalize = finalize ? 1 : 0;
  a.words = host_out ? d->o_words : words; a.nwords = host_out ? d->o_nwords : nwords;
  a.cost = host_out ? d->o_cost : cost;    a.flags = host_out ? d->o_flags : flags;
  a.max_words = d->opts.max_words;
  int rc = launch(d, chan, nfr, io, a, st);
  if (rc) return rc;
  if (host_out) {
    const size_t mw = (size_t)d->opts.max_words;
    HIP_TRY(d, hipMemcpyAsync(words, d->o_words, n * mw * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(nwords, d->o_nwords, n * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(cost, d->o_cost, n * sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipMemcpyAsync(flags, d->o_flags, n * sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(d, hipStreamSynchronize(st));
  }
  return WFST_OK;
}

int32_t wfst_debug_frame_digests(wfst_decoder *d, int32_t ch, uint64_t *digest, int32_t *count,
                                 int32_t cap, int32_t *n) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (!d->c.dig_sum) return fail(d, WFST_ERR_INVALID_ARG, "decoder was created without record_digests");
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  if (!digest || !count || !n || cap < 0) return fail(d, WFST_ERR_INVALID_ARG, "null output");
  HIP_TRY(d, hipDeviceSynchronize());
  ChanState s;
  HIP_TRY(d, hipMemcpy(&s, d->c.st + ch, sizeof(s), hipMemcpyDeviceToHost));
  *n = s.frame + 1;
  const size_t m = (size_t)std::min(cap, s.frame + 1);
  const size_t base = (size_t)ch * (d->c.max_frames + 1);
  HIP_TRY(d, hipMemcpy(digest, d->c.dig_sum + base, m * sizeof(uint64_t), hipMemcpyDeviceToHost));
  HIP_TRY(d, hipMemcpy(count, d->c.dig_cnt + base, m * sizeof(int), hipMemcpyDeviceToHost));
  return WFST_OK;
}

int32_t wfst_get_lattice(wfst_decoder *d, int32_t ch, const void *loglikes, float lattice_beam,
                         int32_t *tok_state, float *tok_cost, int64_t tok_cap, int64_t *frame_off,
                         wfst_lattice_link *links, int64_t link_cap,
                         int64_t *n_tokens, int64_t *n_links, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (!d->c.tokrec) return fail(d, WFST_ERR_INVALID_ARG, "the decoder was created without keep_token_records");
  // the kernels' scratch (counters, links per token set) is what the decoder allocated at create
  d->h_off.resize((size_t)d->c.max_frames + 2 + kHostHead);
  return get_lattice_impl(d, ch, loglikes, lattice_beam, tok_state, tok_cost, tok_cap, frame_off, links, link_cap,
                          n_tokens, n_links, static_cast<hipStream_t>(stream), d->d_lat_ctr, d->d_set_links,
                          d->h_off.data(), d->c.max_frames);
}

int32_t wfst_get_lattice_batch(wfst_decoder *d, const int32_t *channels, int32_t n, const void *loglikes, int32_t T,
                               float lattice_beam, int32_t *tok_state, float *tok_cost, int64_t tok_cap,
                               int64_t *frame_off, wfst_lattice_link *links, int64_t link_cap,
                               int64_t *tok_first, int64_t *link_first, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (!d->c.tokrec) return fail(d, WFST_ERR_INVALID_ARG, "the decoder was created without keep_token_records");
  return get_lattice_batch_impl(d, channels, n, loglikes, T, lattice_beam, tok_state, tok_cost, tok_cap, frame_off,
                                links, link_cap, tok_first, link_first, static_cast<hipStream_t>(stream));
}

int32_t wfst_get_lattice_noalloc(wfst_decoder *d, int32_t ch, const void *loglikes, float lattice_beam,
                                 int32_t *tok_state, float *tok_cost, int64_t tok_cap, int64_t *frame_off,
                                 wfst_lattice_link *links, int64_t link_cap,
                                 int64_t *n_tokens, int64_t *n_links, void *stream) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (!d->c.tokrec) return fail(d, WFST_ERR_INVALID_ARG, "the decoder was created without keep_token_records");
  unsigned long long *ptr = nullptr;
  const int rc = scratch_address(d, &ptr);      // this device's copy of the static array
  if (rc) return rc;
  // words 0, 1 of the scratch: links found / error bits; from word 2 on: links per token set.
  // The host side of the small copies is pinned memory the decoder got at create, so the runtime
  // needs no staging buffer of its own either.
  return get_lattice_impl(d, ch, loglikes, lattice_beam, tok_state, tok_cost, tok_cap, frame_off, links, link_cap,
                          n_tokens, n_links, static_cast<hipStream_t>(stream), ptr, ptr + 2, d->h_pinned,
                          kScratchFrames);
}

int32_t wfst_debug_get_tokens(wfst_decoder *d, int32_t ch, int32_t *states, float *costs, int32_t cap, int32_t *n) {
  return wfst_debug_get_token_pairs(d, ch, states, nullptr, costs, cap, n);
}

int32_t wfst_debug_get_token_pairs(wfst_decoder *d, int32_t ch, int32_t *states, int32_t *bstates, float *costs,
                                   int32_t cap, int32_t *n) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (ch < 0 || ch >= d->opts.max_channels) return fail(d, WFST_ERR_BAD_CHANNEL, "channel out of range");
  if (!states || !costs || !n || cap < 0) return fail(d, WFST_ERR_INVALID_ARG, "null output");
  HIP_TRY(d, hipDeviceSynchronize());
  ChanState s;
  HIP_TRY(d, hipMemcpy(&s, d->c.st + ch, sizeof(s), hipMemcpyDeviceToHost));
  *n = s.n_tok;
  const int m = std::min(cap, s.n_tok);
  std::vector<int2> q((size_t)m);
  const int2 *src = d->c.queue + ((size_t)ch * 2 + s.cur) * d->c.qcap;
  if (m) HIP_TRY(d, hipMemcpy(q.data(), src, (size_t)m * sizeof(int2), hipMemcpyDeviceToHost));
  if (d->state_of_blk.empty()) {            // tokens name their state by its block number
    d->state_of_blk.assign((size_t)d->g.n_blk + 1, -1);
    for (int32_t st = 0; st < d->g.S; ++st) d->state_of_blk[d->blk_of_state[st]] = st;
  }
  for (int i = 0; i < m; ++i) {
    states[i] = d->state_of_blk[(unsigned)q[i].x & d->g.blk_mask];
    if (bstates) bstates[i] = (int)(((unsigned)q[i].x & kKeyMask) >> d->g.blk_bits);
    std::memcpy(&costs[i], &q[i].y, 4);
  }
  return WFST_OK;
}

int32_t wfst_get_counters(wfst_decoder *d, int64_t counters[8], int32_t reset) {
  if (!d || !counters) return WFST_ERR_INVALID_ARG;
  HIP_TRY(d, hipDeviceSynchronize());
  HIP_TRY(d, hipMemcpy(counters, d->c.counters, 8 * sizeof(int64_t), hipMemcpyDeviceToHost));
  if (reset) HIP_TRY(d, hipMemset(d->c.counters, 0, 8 * sizeof(int64_t)));
  return WFST_OK;
}

int32_t wfst_set_launch_workgroups(wfst_decoder *d, int32_t n) {
  if (!d) return WFST_ERR_INVALID_ARG;
  if (n < 0) return fail(d, WFST_ERR_INVALID_ARG, "launch workgroups must be >= 0");
  d->launch_workgroups = n;
  return WFST_OK;
}

int32_t wfst_debug_set_phase_timing(wfst_decoder *d, int32_t on) {
  if (!d) return WFST_ERR_INVALID_ARG;
  d->phase_timing = on ? 1 : 0;
  return WFST_OK;
}

int32_t wfst_debug_phase_ticks(wfst_decoder *d, int64_t ticks[16], int32_t reset) {
  if (!d || !ticks) return WFST_ERR_INVALID_ARG;
  HIP_TRY(d, hipDeviceSynchronize());
  HIP_TRY(d, hipMemcpy(ticks, d->c.counters + 8, 16 * sizeof(int64_t), hipMemcpyDeviceToHost));
  if (reset) HIP_TRY(d, hipMemset(d->c.counters + 8, 0, 16 * sizeof(int64_t)));
  return WFST_OK;
}

int64_t wfst_device_bytes(const wfst_decoder *d) { return d ? d->dev_bytes : 0; }

float wfst_last_kernel_ms(wfst_decoder *d) {
  if (!d || d->last_timed < 0) return -1.0f;
  const int s = d->last_timed;
  if (hipEventSynchronize(d->ev1[s]) != hipSuccess) return -1.0f;
  float ms = -1.0f;
  if (hipEventElapsedTime(&ms, d->ev0[s], d->ev1[s]) != hipSuccess) return -1.0f;
  return ms;
}

float wfst_slot_kernel_ms(wfst_decoder *d, int32_t slot) {
  if (!d || slot < 0 || slot >= d->n_slots || !d->timed[slot]) return -1.0f;
  if (hipEventSynchronize(d->ev1[slot]) != hipSuccess) return -1.0f;
  float ms = -1.0f;
  if (hipEventElapsedTime(&ms, d->ev0[slot], d->ev1[slot]) != hipSuccess) return -1.0f;
  return ms;
}

const char *wfst_last_error(const wfst_decoder *d) { return d ? d->err.c_str() : g_create_err.c_str(); }

}  // extern "C"
