/*
 * cbd.h -- C ABI of the contextual-biasing beam-search decoder for MI355X (gfx950).
 *
 * The library decodes many audio channels at once over one shared, read-only
 * decoding graph.  Each channel carries its own context: a set of arc indices
 * and a discount offset that is added to a listed arc's weight at the moment
 * the arc is expanded (paper Sec. 1: only a list of arc indices is stored per
 * context and the offset is added during decoding; Sec. 4.1: boosted weight =
 * original weight + discount factor).  The graph is never modified, so
 * contexts can be replaced between calls (Sec. 4.3) and partial best-path
 * hypotheses are read without building lattices (Sec. 1, Sec. 2.2).
 *
 * Conventions
 *   - Every function returns 0 (CBD_OK) or a negative cbd_status.  On error the
 *     out-parameters are left untouched unless a function says otherwise.
 *   - "HOST" pointers are ordinary process memory, "DEVICE" pointers are HIP
 *     device memory on the decoder's GPU.  The caller owns every pointer it
 *     passes; the library owns everything behind its handles and copies what
 *     it needs before returning, except DEVICE inputs of cbd_advance (below).
 *   - Handles are not thread-safe: one host thread per decoder at a time.
 *     A graph may be shared by several decoders.
 *   - All work of a decoder is enqueued on the HIP stream given at creation.
 *   - Arc indices at this boundary are positions in the arrays given to
 *     cbd_graph_load (the caller's numbering).
 *   - No exceptions cross this boundary.  There is no CPU fallback.
 *
 * Decoding rule (fp32, every choice independent of thread order): tokens are
 * (cost, arc) keys per state; lower cost wins, ties go to the arc with the lower
 * source state, then emitting before epsilon-input arcs, then the lower arc
 * index.  Per frame: tokens whose cost exceeds the frame's best by more than
 * `beam` are dropped; if more than `max_active` remain, a 256-bin histogram over
 * (cost - best) * 256 / beam keeps the largest prefix of bins that fits.  Every
 * emitting arc of every survivor is expanded, cand = (cost + w') - loglike, the
 * minimum m over candidates fixes the frame's cutoff (cand - m > beam is
 * dropped), epsilon-input arcs are relaxed to a fixed point under the same
 * cutoff, and the predecessor of a token is the final token of its arc's
 * source state.
 */
#ifndef CBD_H_
#define CBD_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cbd_status {
  CBD_OK = 0,
  CBD_E_INVALID = -1,      /* bad argument, index or shape; checked on the host before any enqueue */
  CBD_E_CAPACITY = -2,     /* a channel overflowed its token table, change log or back-pointer buffer */
  CBD_E_EPS_DIVERGED = -3, /* epsilon closure did not settle within max_eps_iters rounds */
  CBD_E_NO_TOKENS = -4,    /* nothing survived (dead end) or channel never reset */
  CBD_E_BUFFER = -5,       /* caller's output buffer too small */
  CBD_E_HIP = -6,          /* HIP runtime error; text via cbd_last_error() */
  CBD_E_NOMEM = -7
} cbd_status;

typedef struct cbd_graph cbd_graph;     /* opaque; immutable; device resident */
typedef struct cbd_decoder cbd_decoder; /* opaque; owns all per-channel device state */

/*
 * The decoding graph as per-arc vectors grouped into rows by source state (the
 * vectors Sec. 4.1 lists: input labels, output labels, next states, weights;
 * Sec. 2.2: compressed sparse rows).  All pointers HOST.
 */
typedef struct cbd_graph_desc {
  int32_t num_states;
  int32_t num_arcs;
  int32_t num_pdfs;           /* log-likelihood row length, at most 65535 */
  int32_t start_state;
  const int32_t *row_offsets; /* [num_states+1]; arcs of state s are [row_offsets[s], row_offsets[s+1]) */
  const int32_t *dst;         /* [num_arcs] next state */
  const int32_t *ilabel;      /* [num_arcs] 0 = epsilon input, else pdf id + 1 (1..num_pdfs) */
  const int32_t *olabel;      /* [num_arcs] 0 = no word, else word id */
  const float *weight;        /* [num_arcs] cost (-log probability), finite */
  const float *final_cost;    /* [num_states] or NULL = every state final at cost 0 */
} cbd_graph_desc;

/*
 * Copies the graph to the current HIP device (rows are re-packed so that each
 * state's emitting arcs precede its epsilon-input arcs; the caller's numbering
 * stays the one used at this boundary).  CBD_E_INVALID for inconsistent rows,
 * labels outside range, non-finite weights.
 */
int32_t cbd_graph_load(const cbd_graph_desc *desc, cbd_graph **out);
int32_t cbd_graph_free(cbd_graph *g);

/*
 * Which arcs to boost for a biasing list of word sequences (Algorithm 1; host only, no GPU work).
 * words: HOST, the sequences' word ids back to back; sequence i is words[seq_offsets[i] ..
 * seq_offsets[i+1]) (seq_offsets HOST [n_seq+1]).  For each sequence w_1..w_k: every arc that outputs
 * w_1 (the sequence may start anywhere in the graph), and for t > 1 every arc that outputs w_t and
 * leaves a state reached from a w_{t-1} arc of the sequence so far through arcs without output label.
 * The union over the sequences is written to arcs (HOST [capacity]) sorted and without duplicates,
 * ready for cbd_set_context; *n_arcs receives its size.  CBD_E_BUFFER if capacity is too small
 * (*n_arcs = needed size).  Unknown words contribute nothing.  Not thread-safe per graph.
 */
int32_t cbd_context_from_words(cbd_graph *g, const int32_t *words, const int32_t *seq_offsets, int32_t n_seq,
                               int32_t *arcs, int32_t capacity, int32_t *n_arcs);

typedef struct cbd_config {
  int32_t num_channels;       /* >= 1 */
  float beam;                 /* >= 0; may be +inf */
  int32_t max_active;         /* 0 = off (needs 0 < beam < inf to act) */
  int32_t max_frames;         /* frames per utterance the back-pointer buffer is sized for */
  int32_t max_context_arcs;   /* largest context list after de-duplication */
  int32_t lookup_mode;        /* 0 sorted list + binary search (Sec. 4.2); 1 hashed bitmap filter, then the search */
  int32_t hash_capacity_log2; /* device-memory state table slots per channel = 2^this; a frame may hold at most
                                 half as many tokens (frames that fit the LDS tables never touch this table) */
  int32_t max_eps_iters;      /* epsilon-closure limit; 0 = default 64.  Counted in levels of a chain of improving
                                 epsilon-input arcs (and in rounds over the change log): a closure that needs more,
                                 a legitimate acyclic chain that long included, parks the channel with
                                 CBD_E_EPS_DIVERGED; raise the limit for graphs with longer epsilon chains */
  int32_t records_per_frame;  /* average back-pointer records per frame to reserve; 0 = table capacity / 2 */
  int32_t table_location;     /* 0 or 1 = LDS tables, frames that outgrow them are redone in device memory;
                                 2 = device-memory tables only */
  int32_t lds_token_cap;      /* tokens per frame the LDS tables hold; 0 = as many as fit (a log-likelihood row of
                                 up to 1024 pdfs is kept in LDS beside them, a longer one is read from device memory) */
  int32_t max_pool_contexts;  /* pre-loaded contexts the decoder can hold besides one per channel (Sec. 4.3) */
  int32_t workgroups_per_cu;  /* channels decoded side by side on one compute unit (they share its LDS, so each
                                 gets a smaller table): 1, 2 or 4; 0 = chosen by the library (1).  CBD_E_INVALID if
                                 the device cannot hold that many workgroups of the kernel on a compute unit */
  int32_t compact_records_above; /* 0 = records are only compacted on request (cbd_compact_records); N > 0 = a
                                 cbd_advance call first compacts those of its channels that hold more than N records
                                 above the part their paths share, and with them (so that a call is held up once,
                                 not once per channel) those that hold more than N / 2.  While the counts that
                                 recent launches have reported show nothing due, the call does not even look (and
                                 asynchronous result walks keep running beside the decoding); N may therefore be
                                 overshot by the records of a few calls: size the buffer with that room */
  int32_t block_threads;      /* threads per workgroup of the decoding kernel: 256, 512, 960 or 1024; 0 = chosen by
                                 the library from workgroups_per_cu (1024 / 512 / 256 for 1 / 2 / 4) */
  int32_t frame_code;         /* 0 = frames that qualify (tables in LDS, every closure met stored as a list with the
                                 graph) are decoded by the lean frame code, the rest by the general code; 1 = general
                                 code only.  Results are the same either way. */
  int32_t workgroups_per_channel; /* 0 or 1 = one workgroup decodes a channel; 2, 4 or 8 = a team of that many
                                 shares it (for frames with far more tokens than one compute unit's LDS holds: the
                                 states are split over the team, candidates travel between members through device
                                 memory).  Needs num_channels x team <= compute units of the device, a graph whose
                                 epsilon closures are all stored as lists (at most 15 levels and 62 arcs each), and
                                 compact_records_above = 0; members are 1024-thread workgroups, each can hold about 7,000 tokens per frame
                                 (CBD_E_CAPACITY beyond).  Results are the same; token and record numbers differ
                                 (cbd_get_tokens / cbd_get_records then show unused places at infinite cost) */
} cbd_config;

/*
 * Allocates all per-channel state on the graph's device.  `hip_stream` is a
 * hipStream_t (NULL = the null stream); it must outlive the decoder.
 */
int32_t cbd_decoder_create(const cbd_graph *g, const cbd_config *cfg, void *hip_stream, cbd_decoder **out);
int32_t cbd_decoder_free(cbd_decoder *d);

/*
 * Starts a new utterance on the listed channels (HOST, n entries, each in
 * [0, num_channels), no duplicates): one start token at cost 0 followed by
 * the epsilon closure under the channel's current context.  Clears the
 * channel's back-pointers, counters and sticky error status.  Enqueues only.
 */
int32_t cbd_reset_channels(cbd_decoder *d, const int32_t *channels, int32_t n);

/*
 * Replaces one channel's context (Sec. 4.3 dynamic context update).  arc_idx:
 * HOST, n entries, any order, duplicates allowed (the list is a set; Algorithm 1
 * returns a set); n = 0 clears.  Takes effect for arcs expanded by later
 * cbd_advance / cbd_reset_channels calls; existing tokens are never re-scored.
 * CBD_E_INVALID for an index outside [0, num_arcs) or more than
 * max_context_arcs distinct entries.
 */
int32_t cbd_set_context(cbd_decoder *d, int32_t channel, const int32_t *arc_idx, int32_t n, float offset);

/*
 * The same for many channels with one upload.  list_offsets: HOST [n_channels+1],
 * channel i's list is arc_idx[list_offsets[i] .. list_offsets[i+1]); offsets:
 * HOST [n_channels].  Nothing is changed if any list is invalid.
 */
int32_t cbd_set_contexts(cbd_decoder *d, const int32_t *channels, int32_t n_channels, const int32_t *arc_idx,
                         const int32_t *list_offsets, const float *offsets);

/*
 * Pre-loaded contexts (Sec. 4.3: contexts anticipated in advance are loaded before decoding and the
 * decoder switches among them).  cbd_contexts_create uploads n_contexts lists (same layout and rules as
 * cbd_set_contexts) into the decoder's pool and returns their ids in context_ids (HOST [n_contexts]);
 * CBD_E_CAPACITY if the pool (max_pool_contexts) has too few free entries.  cbd_use_contexts switches
 * channels[i] to context_ids[i] (-1 = back to the channel's own list from cbd_set_context) without any
 * upload; many channels may share one context.  It takes effect like cbd_set_context.  A destroyed id may
 * be reused by a later create; channels still bound to it keep decoding with whatever the slot holds.
 */
int32_t cbd_contexts_create(cbd_decoder *d, int32_t n_contexts, const int32_t *arc_idx, const int32_t *list_offsets,
                            const float *offsets, int32_t *context_ids);
int32_t cbd_context_destroy(cbd_decoder *d, int32_t context_id);
int32_t cbd_use_contexts(cbd_decoder *d, const int32_t *channels, const int32_t *context_ids, int32_t n);

/*
 * Decodes n_frames frames on the listed channels (Sec. 2.2, Sec. 3.2: a chunk
 * arrives, every outgoing arc of every queued token is expanded, candidates are
 * pruned and re-queued).  loglikes: DEVICE fp32; the row of channel i (position
 * in `channels`), frame f is at loglikes + i*channel_stride + f*num_pdfs, and
 * holds log-likelihoods already scaled by the caller.  The memory must stay
 * valid and unchanged until the stream has passed this call.  Enqueues only;
 * channels in an error state are skipped on the device.
 */
int32_t cbd_advance(cbd_decoder *d, const int32_t *channels, int32_t n_channels, const float *loglikes,
                    int64_t channel_stride, int32_t n_frames);

/*
 * Drops, on the listed channels (HOST, n entries, no duplicates), the back-pointer records that no token of
 * the current frame has on its path, and renumbers the rest.  Results are read off the best current token's
 * sequence only (Sec. 1, Sec. 3.2), so nothing a later cbd_best_path* call returns changes; what changes is
 * the room left: an utterance as long as the 3-minute recordings of Sec. 5.3, or an endless stream, then
 * needs a buffer (max_frames x records_per_frame) for the stretch between two compactions only, plus what
 * the compactions keep.  Channels that have written at most min_new_records (>= 0) records since their last
 * compaction are left alone, as are channels in an error state.  Records kept by one compaction are never
 * examined again by a later one, so the cost of a call follows the frames since the last one, not the
 * length of the utterance.  Enqueues only; the stream first waits for unfinished cbd_best_paths_begin
 * requests (their walks read the records).  CBD_E_INVALID for a bad channel list or a negative threshold.
 */
int32_t cbd_compact_records(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t min_new_records);

/*
 * Best token of the channel's current frame and its back-pointer path (the
 * partial hypothesis of Sec. 1; with use_final != 0 the state's final cost is
 * added before the minimum is taken).  words: HOST [capacity] word ids in time
 * order; arcs: HOST [capacity] or NULL, the arc path in the caller's numbering.
 * Synchronises the stream.  Returns the channel's sticky error if it has one;
 * CBD_E_BUFFER if the path has more than `capacity` arcs (then *n_arcs and
 * *n_words hold the needed sizes).
 */
int32_t cbd_best_path(cbd_decoder *d, int32_t channel, int32_t use_final, int32_t *words, int32_t *arcs,
                      int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost);

/*
 * The same for many channels with one kernel, which writes words and counts
 * straight into pinned host memory of the library's (arcs, if wanted, come by
 * one copy).  Row i of words / arcs ([n][capacity], HOST) belongs to
 * channels[i]; status[i] (HOST [n]) receives that channel's result code; the
 * function itself fails only for invalid arguments or HIP errors.
 */
int32_t cbd_best_paths(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                       int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                       int32_t *status);

/*
 * cbd_best_paths for callers that cannot allocate device memory while they run (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, same results in the
 * caller's arrays (entries of a row beyond its count are unspecified), but the kernel's device-side result
 * rows live in a fixed 8 MiB array that is part of the library's code object instead of buffers the library
 * sizes on demand: the call allocates and frees nothing, on the device or in pinned memory.  The fixed
 * array bounds the request: CBD_E_CAPACITY unless n * (2 * capacity + 8) <= 2,097,152.  Every GPU the
 * library runs on holds one such array until the process ends, and every call on that GPU shares it:
 * calls that overlap on one GPU (two decoders driven from two threads) race and must be serialised by
 * the caller.  Synchronises the stream.
 */
int32_t cbd_best_paths_static(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                              int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                              int32_t *status);

/*
 * The same in two steps, so that intermediate results leave the GPU without interrupting the
 * decoding (Sec. 2.2).  cbd_best_paths_begin notes the best tokens on the decoder's stream (for the
 * channel list of the latest cbd_advance / cbd_reset_channels call and use_final = 0 the decoding
 * kernel has left them behind already) and enqueues the path walks on a stream of the library's own;
 * it returns at once with a ticket.  Calls enqueued afterwards (cbd_advance, context changes) do not disturb the request;
 * cbd_reset_channels waits on the device for outstanding walks.  cbd_best_paths_finish waits for the
 * request and fills the caller's arrays exactly like cbd_best_paths (same capacity as at begin; arcs
 * only if want_arcs was set).  At most four requests may be in flight (CBD_E_CAPACITY).
 */
int32_t cbd_best_paths_begin(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t capacity,
                             int32_t want_arcs, int32_t *ticket);
int32_t cbd_best_paths_finish(cbd_decoder *d, int32_t ticket, int32_t *words, int32_t *arcs, int32_t capacity,
                              int32_t *n_words, int32_t *n_arcs, float *cost, int32_t *status);

/*
 * Results in two parts, for long utterances.  All paths of a channel's current tokens share their beginning,
 * and the part of it that the compactions (cbd_compact_records) have found so far can no longer change: it is
 * what an online recogniser may show as final while the utterance goes on (Sec. 1, Sec. 3.2: intermediate
 * results are the best current token sequence).  The library keeps that part per channel, in time order.
 *
 * cbd_best_tails / _begin / _finish work like cbd_best_paths / _begin / _finish, but follow each best path only
 * down to that fixed part: words / arcs receive the rest of the path, and n_fixed_words[i] / n_fixed_arcs[i]
 * (HOST [n]) say how many words and arcs of the fixed part precede it.  The whole result is the first
 * n_fixed_words[i] words of the fixed part followed by the returned words (likewise for arcs); cost is the
 * whole path's.  A walk then costs the frames since the paths merged, not the utterance so far.  Without
 * compactions the fixed part is empty and the calls return whole paths.  A request begun by cbd_best_tails_begin
 * is finished by cbd_best_tails_finish (and one begun by cbd_best_paths_begin by cbd_best_paths_finish).
 *
 * cbd_get_fixed copies the fixed part of one channel from word from_word and arc from_arc on (it only ever
 * grows within an utterance, so a caller keeps what it has and asks for the rest): words, arcs HOST [capacity]
 * or NULL; *n_words, *n_arcs receive the counts beyond from_word / from_arc; CBD_E_BUFFER if a wanted array is
 * too small.  Synchronises.  The fixed part is cleared by cbd_reset_channels; its room is that of the
 * back-pointer buffer (when it is full, nothing more is declared fixed).
 *
 * (cbd_best_path* use the fixed part too: they walk down to it and copy it in front of the rest, so whole-path
 * results stay cheap on long utterances once compactions run; what they return is the same either way.)
 */
int32_t cbd_best_tails(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                       int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                       int32_t *status, int32_t *n_fixed_words, int32_t *n_fixed_arcs);
int32_t cbd_best_tails_begin(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t capacity,
                             int32_t want_arcs, int32_t *ticket);
int32_t cbd_best_tails_finish(cbd_decoder *d, int32_t ticket, int32_t *words, int32_t *arcs, int32_t capacity,
                              int32_t *n_words, int32_t *n_arcs, float *cost, int32_t *status,
                              int32_t *n_fixed_words, int32_t *n_fixed_arcs);
int32_t cbd_get_fixed(cbd_decoder *d, int32_t channel, int32_t from_word, int32_t from_arc, int32_t *words,
                      int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs);

/*
 * The channel's current token table (any order): state, cost, arc (caller's
 * numbering, -1 for the start token).  For tests and inspection.  Synchronises.
 * *n receives the table size; at most `capacity` entries are written.
 */
int32_t cbd_get_tokens(cbd_decoder *d, int32_t channel, int32_t *states, float *costs, int32_t *arcs,
                       int32_t capacity, int32_t *n);

typedef struct cbd_stats {
  int64_t frames;         /* frames decoded since reset */
  int64_t active_tokens;  /* tokens that survived pruning and were expanded */
  int64_t emit_arcs;      /* emitting arcs expanded */
  int64_t eps_arcs;       /* epsilon-input arcs expanded (every relaxation round counts) */
  int64_t candidates;     /* candidates that passed the cutoff and reached the state table */
  int64_t improvements;   /* table updates (change-log entries) */
  int64_t tokens;         /* sum over frames of the table size */
  int64_t eps_rounds;     /* per frame the longest run of closure levels any wave made, summed over frames */
  int64_t records;        /* back-pointer records in use */
  int64_t slow_frames;    /* frames decoded with the device-memory tables */
  int64_t records_dropped; /* back-pointer records removed by compactions */
  int64_t lean_frames;    /* frames decoded by the lean frame code */
  int32_t compactions;    /* compactions that ran */
  int32_t status;         /* sticky cbd_status of the channel */
  int32_t max_tokens;     /* largest table so far */
} cbd_stats;

/*
 * Diagnostic: the back-pointer records of one channel as they stand (Sec. 1: the token sequences partial
 * results are read from).  Record i is (arcs[i], prev[i]): the arc that produced the token (caller's
 * numbering; -1 for the start token) and the record of the token it came from (-1: none).  The tokens
 * of the current frame are records [*frame_base, *n_records); records below *kept_base survived a
 * compaction.  arcs, prev: HOST [capacity], or NULL to ask for the sizes only; CBD_E_BUFFER if capacity
 * is too small (*n_records = needed size).  Synchronises.
 */
int32_t cbd_get_records(cbd_decoder *d, int32_t channel, int32_t *arcs, int32_t *prev, int32_t capacity,
                        int32_t *n_records, int32_t *frame_base, int32_t *kept_base);

/* Counters of one channel since its last reset (channel >= 0) or summed over all (-1; status = first error).
 * Synchronises. */
int32_t cbd_get_stats(cbd_decoder *d, int32_t channel, cbd_stats *out);

/* Bytes of device memory the decoder holds; LDS bytes and threads per workgroup of the decode kernel;
 * tokens per frame its LDS tables hold (0 = device-memory tables only).  Any pointer may be NULL. */
int32_t cbd_decoder_info(const cbd_decoder *d, int64_t *device_bytes, int32_t *lds_bytes, int32_t *block_threads,
                         int32_t *lds_token_cap);

int32_t cbd_synchronize(cbd_decoder *d);

/* Runs the kernels' wave-level prefix sum and minimum on the current device against plain host loops.
 * CBD_OK, or CBD_E_HIP with the mismatch in cbd_last_error(). */
int32_t cbd_selftest(void);

const char *cbd_strerror(int32_t status);
/* Text of the last CBD_E_HIP / CBD_E_INVALID on this thread. */
const char *cbd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CBD_H_ */
