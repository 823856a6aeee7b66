/*
 * wfst_decoder.h -- C ABI of the MI355X (gfx950) WFST beam-search decoder for CTC models.
 *
 * The library implements the per-frame iteration of the paper's Section "Algorithm
 * description" (ExpandArcs -> Prune -> store tokens and backpointers, then least-cost
 * path from the stored backpointers), with the frame loop, the backpointer lattice and the
 * traceback all resident on the GPU, plus the per-stream saved decoder state of Section
 * "Streaming inference".  All arithmetic on costs is fp32.
 *
 * Conventions
 *   - Every call returns a status (0 = WFST_OK, negative = error).  Nothing throws or aborts
 *     across this boundary.  wfst_last_error() gives a library-owned message for the last
 *     failing call on that decoder (or on creation when passed NULL).
 *   - "host" / "device" on a pointer says where the memory lives.  The library never takes
 *     ownership of caller memory; graph arrays are copied during create.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it; device outputs are valid once the stream has reached the end of the
 *     call's work.  With opts.outputs_on_host != 0 the call copies results to host memory and
 *     synchronises the stream before returning.
 *   - Calls on one decoder must not overlap in time (one stream at a time per decoder), except
 *     wfst_decode_batch_slot calls on different batch slots.  A decoder is not thread-safe on the
 *     host: issue its calls from one thread.
 *   - Labels: ilabel 0 = epsilon; ilabel k >= 1 reads log-likelihood column k-1 (so the CTC
 *     blank, class 0, is ilabel 1); olabel 0 = no output (cf. the olabel != 0 test in the
 *     figure "Pseudo-code of Expand Arcs").
 */
#ifndef WFST_DECODER_H_
#define WFST_DECODER_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  WFST_OK = 0,
  WFST_ERR_INVALID_ARG = -1,
  WFST_ERR_BAD_GRAPH = -2,       /* malformed CSR, label out of range, non-finite weight, epsilon cycle */
  WFST_ERR_OOM = -3,
  WFST_ERR_LATTICE_OVERFLOW = -4,
  WFST_ERR_BAD_CHANNEL = -5,
  WFST_ERR_HIP = -6,
  WFST_ERR_CAPACITY = -7         /* a per-channel work buffer (state map, queues) overflowed */
};

/* bits of the per-utterance `flags` output */
enum {
  WFST_FLAG_REACHED_FINAL = 1,   /* cost includes a final cost */
  WFST_FLAG_TRUNCATED = 2,       /* more than max_words words; the first max_words are returned */
  WFST_FLAG_DEAD = 4,            /* no token survived (no emitting arc could be taken) */
  WFST_FLAG_LATTICE_OVERFLOW = 8,/* the channel ran out of lattice memory and stopped */
  WFST_FLAG_CAPACITY = 16        /* a work buffer overflowed and the channel stopped */
};

typedef struct wfst_decoder wfst_decoder; /* opaque, owned by the library */

/* Decoding graph (the TLG transducer shared by all utterances, Section "Word boosting",
 * first paragraph) as CSR over states.  All arrays are HOST memory, read during create. */
typedef struct {
  int32_t num_states;
  int32_t start_state;
  int32_t num_classes;            /* V: width of a log-likelihood row */
  int64_t num_arcs;
  const int64_t *row_offsets;     /* [num_states+1]; arcs of s are [off[s], off[s+1]) */
  const int32_t *next_state;      /* [num_arcs] */
  const int32_t *ilabel;          /* [num_arcs], 0..V */
  const int32_t *olabel;          /* [num_arcs], 0 = none */
  const float *weight;            /* [num_arcs], finite */
  const float *final_cost;        /* [num_states], +inf = not final; NULL = all final, cost 0 */
} wfst_graph_csr;

typedef struct {
  int32_t max_channels;           /* channel slots (>= largest batch and streaming channel id+1) */
  int32_t max_frames_per_channel; /* frames a channel can consume between two inits */
  int32_t max_words;              /* row width of the `words` output */
  int64_t lattice_bytes_per_channel; /* 0 = 8 B * max_frames * 1.5 * max_active_hint */
  int32_t outputs_on_host;        /* 0: outputs are device pointers; 1: host pointers */
  int32_t max_active_hint;        /* sizes the per-channel work buffers; 0 = 10000 */
  int32_t candidate_capacity;     /* candidate records per channel and frame, 0 = 16 * max_active_hint */
  int32_t record_digests;         /* 1: keep per-frame token-set digests (slower; for tests) */
  int32_t loglike_dtype;          /* element type of every `loglikes` argument of this decoder:
                                     WFST_LOGLIKE_F32 (0), _F16 (1, IEEE binary16) or _BF16 (2).
                                     16-bit rows are widened to fp32 when a frame is staged; all
                                     cost arithmetic stays fp32, so the result is exactly that of
                                     the fp32 decoder fed the widened values */
  int32_t keep_token_records;     /* 1: keep {state, cost} of every stored token beside its
                                     backpointer (as much memory again as the lattice arena), which
                                     wfst_get_lattice needs; 0: only the best path can be read back */
  int32_t cost_offset;            /* 1: after the prune step of every frame the surviving tokens' costs
                                     are rebased to the best cost of that frame (c - best, fp32) and the
                                     offsets are summed in fp64 and added back to every cost that is
                                     reported, so that costs keep their fp32 resolution on streams of any
                                     length (the paper is silent on cost renormalisation; without it a
                                     stream of 40,000 frames loses the exact best path to rounding).
                                     Results can differ from cost_offset = 0 in the last bits of costs
                                     and in near-ties.  Stored token costs, and with them the costs in a
                                     lattice, are the rebased ones (a link's cost is in the base of the
                                     token it enters) */
  int32_t batch_slots;            /* 0 or 1: one.  n > 1: the channels are n equal groups ("slots"), and
                                     wfst_decode_batch_slot calls on DIFFERENT slots may be in flight at the same
                                     time (each on its own stream), sharing the graph: while one batch's long
                                     utterances finish, the next batch's take the free compute units.  max_channels
                                     must be a multiple of n; a batch has at most max_channels / n utterances */
  int32_t recycle_lattice;        /* 1: a channel's backpointer memory is a ring over whole frames, so a stream can
                                     run for any number of frames (the per-stream state is the set of active tokens,
                                     Section "Streaming inference"; backpointers are kept only as far back as results
                                     still need them).  A (partial) result then needs the path of the channel's
                                     previous result: it is exact as long as the new best path joins that path
                                     within the frames the ring still holds (max_frames_per_channel frames and
                                     lattice_bytes_per_channel bytes back); otherwise the call reports
                                     WFST_FLAG_LATTICE_OVERFLOW and no words.  Ask for results at least that often.
                                     Needs lattice_bytes_per_channel >= 16 B x the token queue size (2 full token
                                     sets); excludes keep_token_records.  max_frames_per_channel then bounds only a
                                     single wfst_decode_batch utterance, not a stream */
  int32_t lattice_by_length;      /* 1: wfst_decode_batch* shares a slot's backpointer memory (channels of the slot x
                                     lattice_bytes_per_channel) out among the batch's utterances in proportion to
                                     their lengths instead of equally, so lattice_bytes_per_channel can be sized for
                                     the MEAN utterance.  Such a call takes the memory of every channel of its slot:
                                     channels of that slot used for streaming must be initialised again afterwards */
  int32_t narrow_arcs;            /* 1: beside the full arc records the graph gets 8-byte records of its emitting
                                     arcs {destination, weight as IEEE binary16, ilabel, has-output-label bit},
                                     which ExpandArcs reads for states with several arcs (half the bytes per arc;
                                     the graph itself takes 8 more bytes per arc).  Every emitting arc's weight is
                                     rounded to binary16 (BAD_GRAPH if it does not fit) for ALL uses, so results are
                                     exactly those of this decoder on a graph with the rounded weights; epsilon arcs
                                     keep fp32 weights */
  int32_t selection_sample;       /* 0: default (8).  n > 0: before recombination the decoder looks at one run of 64
                                     candidates out of n (rounded down to a power of two) to estimate which of them can survive
                                     max-active and how many
                                     table passes they need.  A tuning knob: results never depend on it (an estimate
                                     that turns out wrong costs time, the step is then done again) */
} wfst_opts;

#define WFST_LOGLIKE_F32 0
#define WFST_LOGLIKE_F16 1
#define WFST_LOGLIKE_BF16 2

/*
 * Word boosting (paper, Section "Word boosting"): the table of a single-state boosting
 * acceptor B, word id (an output label of the graph, > 0) -> score; boosted words get a
 * NEGATIVE score since the decoder minimises.  The utterance is decoded as if the graph were
 * TLG o B: on every arc, emitting or epsilon, whose olabel is in the table the score is
 * added after the other terms (the green lines of the figure "Pseudo-code of Expand Arcs").
 * Words absent from the graph's output labels have no effect.  HOST arrays, copied during
 * the call; at most 1024 entries, no word twice, finite scores.
 */
typedef struct {
  int32_t n;
  const int32_t *word_ids;        /* [n] */
  const float *scores;            /* [n] */
} wfst_boost_table;

/*
 * Boosting acceptor with several states, for boosting sequences of output labels (phrases); the
 * paper composes the graph on the fly with a boosting acceptor B (Section "Word boosting", TLG o B),
 * draws B with one state, a self-loop per boosted word and a failure arc for every other word
 * (figure "Example word boosting WFSA"), and names phrases as the extension (Conclusions).
 * B is deterministic over the graph's OUTPUT labels: n_arcs arcs (arc_from, arc_label > 0, arc_to,
 * arc_score), states 0..n_states-1, root 0, at most one arc per (state, label).  A hypothesis is a
 * pair (graph state, B state), hypotheses are recombined per pair, and max-active counts pairs.
 * On a graph arc with output label o taken in B state b: if b has an arc on o, its score is added
 * after the other terms and the hypothesis moves to its destination; otherwise the failure arc
 * leads to the root at no cost and o is tried once more there (the root's arc on o if it has one;
 * else the hypothesis stays in the root and nothing is added).  Arcs without output label leave b
 * unchanged.  n_states == 1 is exactly wfst_boost_table.  Typical B: the trie of the target
 * sequences with every node that has no continuation merged into the root.
 * HOST arrays, copied during the call.  Limits: n_arcs <= 1024; n_states <= 4096 and
 * n_states <= 2^(29 - bits needed for the graph's 32-byte block count) (INVALID_ARG otherwise);
 * finite scores.  wfst_get_lattice is not available for a channel decoded with n_states > 1.
 */
typedef struct {
  int32_t n_states;
  int32_t n_arcs;
  const int32_t *arc_from;        /* [n_arcs] */
  const int32_t *arc_label;       /* [n_arcs] */
  const int32_t *arc_to;          /* [n_arcs] */
  const float *arc_score;         /* [n_arcs] */
} wfst_boost_fst;

/*
 * Build a decoder: validates the graph, splits emitting and epsilon arcs (global arc ids:
 * emitting arcs 0..Ae-1 in (state, given order), epsilon arcs Ae.. likewise), uploads it and
 * allocates the per-channel state.  Errors: INVALID_ARG, BAD_GRAPH, OOM, HIP.
 */
int32_t wfst_decoder_create(const wfst_graph_csr *graph, const wfst_opts *opts, wfst_decoder **out);
int32_t wfst_decoder_destroy(wfst_decoder *dec);

/*
 * Offline batch decode (Section "Offline inference"): utterance b uses channel slot b, which
 * is reset first.  For each frame t < lengths[b]:
 *   ExpandArcs over emitting arcs, cost = (token cost + arc weight) + (-loglikes[b][t][ilabel-1])
 *   (figure "Pseudo-code of Expand Arcs"); one token per destination state, lowest (cost,
 *   arc id) wins; Prune: keep tokens with (cost - best) <= beam, and if more than max_active
 *   remain, only those in the lowest bins of a 256-bin histogram over [best, best+beam];
 *   epsilon closure under the same cutoff; backpointers appended to the channel's lattice.
 * Then the best token (with final costs if any token is final) is traced back.
 *   loglikes : DEVICE, [B][T][V] contiguous, float (or the 16-bit type chosen in
 *              opts.loglike_dtype; the parameter is then a pointer to those), V == graph.num_classes; rows t >= lengths[b]
 *              are never read.  Must stay valid until the stream has finished the call.
 *   lengths  : HOST, int32 [B], 0 <= lengths[b] <= min(T, max_frames_per_channel)
 *   words    : [B][max_words] int32, nwords [B] int32, cost [B] float, flags [B] int32
 *              (device or host pointers according to opts.outputs_on_host)
 * Identical in result to wfst_init_channel + wfst_advance_chunk (any chunking) +
 * wfst_get_partial(finalize=1).  Errors: INVALID_ARG, BAD_CHANNEL (B > max_channels), HIP;
 * with host outputs also LATTICE_OVERFLOW / CAPACITY if any utterance hit them (the flags
 * say which).
 */
int32_t wfst_decode_batch(wfst_decoder *dec, const float *loglikes, const int32_t *lengths,
                          int32_t B, int32_t T, int32_t V, float beam, int32_t max_active,
                          void *stream, int32_t *words, int32_t *nwords, float *cost,
                          int32_t *flags);
/* The same with a word-boost table per utterance: boosts is a HOST array of B pointers (a NULL
 * pointer, or NULL for the whole array, means no boosting for that utterance). */
int32_t wfst_decode_batch_boosted(wfst_decoder *dec, const float *loglikes, const int32_t *lengths,
                                  int32_t B, int32_t T, int32_t V, float beam, int32_t max_active,
                                  const wfst_boost_table *const *boosts, void *stream,
                                  int32_t *words, int32_t *nwords, float *cost, int32_t *flags);

/* The same with a boosting acceptor per utterance: fsts is a HOST array of B pointers (NULL entries,
 * or NULL for the whole array: no boosting). */
int32_t wfst_decode_batch_boost_fst(wfst_decoder *dec, const float *loglikes, const int32_t *lengths,
                                    int32_t B, int32_t T, int32_t V, float beam, int32_t max_active,
                                    const wfst_boost_fst *const *fsts, void *stream,
                                    int32_t *words, int32_t *nwords, float *cost, int32_t *flags);

/* wfst_decode_batch on batch slot `slot` (opts.batch_slots): utterance b uses channel
 * slot * (max_channels / batch_slots) + b.  Calls on different slots may overlap in time when they
 * are given different streams; calls on one slot may not.  boosts / fsts: NULL, or one of them a
 * HOST array of B table / acceptor pointers.  loglikes as in wfst_decode_batch (element type
 * opts.loglike_dtype).  With host outputs the call synchronises its stream before returning. */
int32_t wfst_decode_batch_slot(wfst_decoder *dec, int32_t slot, const void *loglikes, const int32_t *lengths,
                               int32_t B, int32_t T, int32_t V, float beam, int32_t max_active,
                               const wfst_boost_table *const *boosts, const wfst_boost_fst *const *fsts,
                               void *stream, int32_t *words, int32_t *nwords, float *cost, int32_t *flags);

/* How many workgroups the launches of this decoder get from now on.  n = 0 (the default): one per
 * utterance (or channel) of the call.  n > 0: at most n; they take the call's utterances, longest
 * first, one after the other from a counter on the device, so that all of them are busy until the
 * call's work runs out and they end at nearly the same time.  This is for several batches in flight
 * (batch slots): the GPU hands the workgroups of a launch to fixed groups of compute units in launch
 * order, so with one workgroup per utterance a compute unit that a short utterance has left can
 * stay idle while the next workgroup in line waits for another group.  With n chosen so that the
 * launches in flight together hold exactly the GPU's compute units (256 on MI355X: n = 128 for
 * two or three slots), and a multiple of 32 (8 dies x 4 groups), every workgroup finds a free
 * compute unit at once.  Results do not depend on n.  Errors: INVALID_ARG (n < 0). */
int32_t wfst_set_launch_workgroups(wfst_decoder *dec, int32_t n);

/*
 * Streaming (Section "Streaming inference": the decoder state kept per audio stream is its
 * set of active tokens; here it lives permanently in the channel's slot in GPU memory, so
 * no gather/scatter is needed between chunks).
 *   wfst_init_channel : reset channel `ch` to the start token closed over epsilon arcs, and
 *                       fix its beam / max_active and its word-boost table (NULL = none).
 *   wfst_init_channels: the same for n channels (HOST int32 channels[n], distinct) in one launch,
 *                       for a burst of new streams; boosts is NULL or a HOST array of n table
 *                       pointers (NULL entries = no table).
 *   wfst_advance_chunk: feed n channels (HOST int32 channels[n], distinct) nframes[i] <= C
 *                       frames each from DEVICE loglikes [n][C][V]; nframes is HOST.
 *   wfst_get_partial  : best hypothesis of channel `ch` so far.  finalize = 0 ignores final
 *                       costs (partial result), 1 applies them.  words [cap], nwords [1],
 *                       cost [1], flags [1] follow opts.outputs_on_host.
 *   wfst_get_partial_batch: the same for n channels (HOST int32 channels[n], distinct) in one launch;
 *                       words [n][max_words], nwords [n], cost [n], flags [n].
 * The traceback behind a (partial) result is incremental: the library remembers the path of the
 * channel's previous traceback and stops where the new one meets it, so a result after every
 * chunk costs a walk over the new frames, not over the whole stream (only with cap ==
 * opts.max_words; another cap takes the full walk).
 */
int32_t wfst_init_channel(wfst_decoder *dec, int32_t ch, float beam, int32_t max_active,
                          const wfst_boost_table *boost, void *stream);
/* wfst_init_channel with a boosting acceptor of several states (NULL = none) for the stream. */
int32_t wfst_init_channel_boost_fst(wfst_decoder *dec, int32_t ch, float beam, int32_t max_active,
                                    const wfst_boost_fst *fst, void *stream);
int32_t wfst_init_channels(wfst_decoder *dec, const int32_t *channels, int32_t n, float beam,
                           int32_t max_active, const wfst_boost_table *const *boosts, void *stream);
/* wfst_init_channels with a boosting acceptor of several states per stream: fsts is a HOST array of
 * n acceptor pointers (an entry may be NULL = that stream is not boosted), or NULL. */
int32_t wfst_init_channels_boost_fst(wfst_decoder *dec, const int32_t *channels, int32_t n, float beam,
                                     int32_t max_active, const wfst_boost_fst *const *fsts, void *stream);
int32_t wfst_advance_chunk(wfst_decoder *dec, const int32_t *channels, int32_t n,
                           const float *loglikes, const int32_t *nframes, int32_t C, int32_t V,
                           void *stream);
/* wfst_advance_chunk followed by wfst_get_partial_batch on the same channels, in ONE launch: every
 * channel consumes its frames and then reports its partial (finalize = 0) or final hypothesis
 * (Section "Streaming inference": the serving loop wants a transcript after every chunk).  Same
 * arguments, outputs, results and errors as the two calls made one after the other. */
int32_t wfst_advance_chunk_partial(wfst_decoder *dec, const int32_t *channels, int32_t n,
                                   const float *loglikes, const int32_t *nframes, int32_t C, int32_t V,
                                   int32_t finalize, int32_t *words, int32_t *nwords, float *cost,
                                   int32_t *flags, void *stream);
int32_t wfst_get_partial(wfst_decoder *dec, int32_t ch, int32_t finalize, int32_t *words,
                         int32_t cap, int32_t *nwords, float *cost, int32_t *flags, void *stream);
int32_t wfst_get_partial_batch(wfst_decoder *dec, const int32_t *channels, int32_t n, int32_t finalize,
                               int32_t *words, int32_t *nwords, float *cost, int32_t *flags,
                               void *stream);

/*
 * Lattice output.  The paper says only that the stored tokens and backpointers let the host
 * construct "a lattice or least cost path" (Section "Algorithm description") and defines no
 * lattice; the definition here is this library's own.  Nodes are the stored tokens of channel
 * `ch`: the closed token sets A_0..A_f (f = frames consumed since its init), numbered
 * consecutively, A_t = [frame_off[t], frame_off[t+1]).  There is a link for every arc of the
 * graph between two stored tokens -- an emitting arc from a token of A_{t-1} to a token of A_t,
 * an epsilon arc between two tokens of the same A_t -- whose cost through the arc (the source
 * token's stored cost plus arc weight, acoustic cost and boost score, added in the decoder's
 * own order and precision) is finite and at most `lattice_beam` above the destination token's
 * stored cost.  The best path's backpointers are links of difference 0, so the lattice's least
 * cost path is the decoder's; lattice_beam = +inf keeps every arc between stored tokens.
 *
 * Needs opts.keep_token_records.  `loglikes`: DEVICE, the utterance's f rows of V elements
 * (dense, element type opts.loglike_dtype) with the values it was decoded with; the decoder
 * does not keep them.  tok_state / tok_cost [tok_cap] and links [link_cap]: DEVICE, caller
 * owned; the links are ordered by `frame`, in no particular order inside a frame.  frame_off [f+2], n_tokens, n_links: HOST.  The
 * call runs on `stream` and returns after it has finished.  If tok_cap or link_cap is too
 * small the call returns WFST_ERR_CAPACITY with *n_tokens and *n_links set to what is needed
 * (entries beyond the capacities are not written).  Other errors: INVALID_ARG (no records
 * kept, null pointer, negative or NaN lattice_beam), BAD_CHANNEL, CAPACITY (the channel
 * itself stopped on an overflow: its token sets are incomplete), HIP.
 */
typedef struct {
  int32_t src, dst;               /* token numbers */
  int32_t ilabel, olabel;         /* of the arc; ilabel 0 = epsilon link */
  float graph_cost;               /* arc weight */
  float acoustic_cost;            /* -loglikes[frame-1][ilabel-1]; 0 for an epsilon link */
  float cost;                     /* cost through the arc (includes the boost score, if any) */
  int32_t frame;                  /* t of the set A_t the destination token is in */
} wfst_lattice_link;

int32_t wfst_get_lattice(wfst_decoder *dec, int32_t ch, const void *loglikes, float lattice_beam,
                         int32_t *tok_state, float *tok_cost, int64_t tok_cap, int64_t *frame_off,
                         wfst_lattice_link *links, int64_t link_cap,
                         int64_t *n_tokens, int64_t *n_links, void *stream);

/*
 * wfst_get_lattice (same definition of the lattice, Section "Algorithm description" as read above)
 * for n DISTINCT channels in one call: all their token sets go through the kernels together -- two
 * launches and two synchronisations in all, instead of per channel.
 *   loglikes   DEVICE [n][T][V] (element type opts.loglike_dtype): the rows of channels[k] start at
 *              element k*T*V; every channel must have consumed at most T frames
 *   tok_state / tok_cost [tok_cap], links [link_cap]   DEVICE, caller owned: the channels' tokens
 *              and links one after the other in the order of `channels`
 *   tok_first, link_first [n + 1]   HOST: channel k's tokens are entries [tok_first[k], tok_first[k+1]),
 *              its links [link_first[k], link_first[k+1])
 *   frame_off  HOST [n][T + 2]: row k as wfst_get_lattice's frame_off for channels[k] (entries after
 *              the channel's last set repeat its token count)
 * Token numbers (frame_off, src and dst of a link) count from 0 within each channel, as in
 * wfst_get_lattice.  If a capacity is too small: WFST_ERR_CAPACITY with tok_first[n] and
 * link_first[n] set to the totals needed (call with capacities 0 to learn them).  Other errors as
 * wfst_get_lattice, plus BAD_CHANNEL for a channel listed twice and INVALID_ARG for a channel with
 * more than T frames.  The first call allocates pinned host staging memory.
 */
int32_t wfst_get_lattice_batch(wfst_decoder *dec, const int32_t *channels, int32_t n, const void *loglikes,
                               int32_t T, float lattice_beam, int32_t *tok_state, float *tok_cost,
                               int64_t tok_cap, int64_t *frame_off, wfst_lattice_link *links,
                               int64_t link_cap, int64_t *tok_first, int64_t *link_first, void *stream);

/*
 * wfst_get_lattice for callers that must not allocate (code between graph captures, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same results, but the call allocates
 * nothing, neither device nor host memory.  The kernels' scratch (two counters and the number of
 * links of every token set) lives in a static device array of 32 KB inside the library instead of
 * in memory the decoder allocated; every GPU the library runs on holds its own copy until the
 * process ends.  Limits: the channel may have consumed at most 4094 frames (else WFST_ERR_CAPACITY).
 * All decoders and calls on one GPU share that array: calls of this entry point that overlap in
 * time on one GPU race with each other (calls of wfst_get_lattice do not use it).
 */
int32_t wfst_get_lattice_noalloc(wfst_decoder *dec, int32_t ch, const void *loglikes, float lattice_beam,
                                 int32_t *tok_state, float *tok_cost, int64_t tok_cap, int64_t *frame_off,
                                 wfst_lattice_link *links, int64_t link_cap,
                                 int64_t *n_tokens, int64_t *n_links, void *stream);

/*
 * Test and measurement hooks.  All outputs are HOST memory; each call synchronises the
 * device first.
 *   wfst_debug_frame_digests: needs opts.record_digests.  For the closed token sets A_0..A_f
 *     of channel ch (f = frames consumed): count[t] = |A_t| and digest[t] = sum over tokens
 *     of mix(state, cost bits) modulo 2^64.  Writes min(f+1, cap) entries, *n = f+1.
 *   wfst_debug_get_tokens: current token set of channel ch (any order).
 *   wfst_debug_get_token_pairs: the same with each token's state in the boosting acceptor
 *     (bstates [cap], may be NULL).
 *   wfst_get_counters: sums over all channels since create or the last reset:
 *     [0] tokens expanded, [1] emitting arcs out of them, [2] epsilon arcs out of every
 *     closed token set, [3] tokens surviving the prune step (before the closure), [4] tokens stored,
 *     [5] frames where max-active pruned, [6] frames where bin 0 alone exceeded max-active,
 *     [7] frames decoded.   reset != 0 zeroes them after reading.
 */
int32_t wfst_debug_frame_digests(wfst_decoder *dec, int32_t ch, uint64_t *digest, int32_t *count,
                                 int32_t cap, int32_t *n);
int32_t wfst_debug_get_tokens(wfst_decoder *dec, int32_t ch, int32_t *states, float *costs,
                              int32_t cap, int32_t *n);
int32_t wfst_debug_get_token_pairs(wfst_decoder *dec, int32_t ch, int32_t *states, int32_t *bstates,
                                   float *costs, int32_t cap, int32_t *n);
int32_t wfst_get_counters(wfst_decoder *dec, int64_t counters[8], int32_t reset);

/*
 * Where the channel workgroups spend their time: sums over all channels of 100 MHz
 * wall-clock ticks per phase since create or the last reset (HOST output, synchronises):
 *   [0] ExpandArcs over emitting arcs, [1] recombination, [2] cutoff + compaction,
 *   [3] epsilon expansion, [4] epsilon recombination, [5] publishing the token set,
 *   [6] final choice + traceback, [7] everything else (row staging, init);
 *   [8..12] split of [1] and [4]: table clear, fill, winners; epsilon table clear+fill, new
 *   tokens out of the table (these are counted instead of, not on top of, [1] and [4]);
 *   [13] the arc loops of [0]; [14] epsilon closure: the set's tokens looking their states up
 *   in the table; [15] is not a time: the number of times a frame's recombination had to be
 *   done again (with every candidate selected, or with more table passes).
 * The times are only taken by launches made while phase timing is on
 * (wfst_debug_set_phase_timing(dec, 1); off by default: the clock reads at every phase boundary
 * cost a launch about 1 %; not available with narrow arc records); [15] is always counted.
 */
int32_t wfst_debug_set_phase_timing(wfst_decoder *dec, int32_t on);
int32_t wfst_debug_phase_ticks(wfst_decoder *dec, int64_t ticks[16], int32_t reset);

/* Device memory the decoder holds, in bytes (graph + channel state). */
int64_t wfst_device_bytes(const wfst_decoder *dec);

/*
 * Time of the most recent decode/advance kernel in milliseconds, measured with HIP events
 * recorded on the stream the kernel was launched on.  Synchronises on the stop event.
 * Returns a negative value if no kernel has been launched.
 */
float wfst_last_kernel_ms(wfst_decoder *dec);
/* The same for the most recent wfst_decode_batch* kernel of one batch slot. */
float wfst_slot_kernel_ms(wfst_decoder *dec, int32_t slot);

const char *wfst_last_error(const wfst_decoder *dec);

#ifdef __cplusplus
}
#endif
#endif /* WFST_DECODER_H_ */
