/*
 * dblp_agg -- receiver-side bounded-loss gradient aggregation of DBLP
 * (Dynamic Bounded-Loss Protocol) on one AMD MI355X (gfx950).
 *
 * One context models the parameter server of the paper's centralized
 * all-reduce for one communication round at a time: packets from W workers
 * arrive in any order over a lossy channel, are validated and scattered into
 * an accumulator (Alg. "DBLP_RECV"), loss is counted against the current
 * tolerance to decide what must be retransmitted (Sec. "Dynamically Changing
 * Loss Tolerance"), unreceived chunks stay zero and the mean over all workers
 * is formed (Alg. "DBLP_RECV" last statements, Alg. "Server"), and the L2 norm
 * of that mean drives critical-regime detection (Eq. 1).
 *
 * Conventions
 *   - Every call returns DBLP_OK (0) or a negative DBLP_E* code; nothing
 *     throws, aborts or prints.  dblp_last_error() gives a short text.
 *   - d_* arguments are DEVICE pointers owned by the caller; the library never
 *     frees them and does not keep them after the call returns (the kernels
 *     that read them are ordered on the context's stream).  h_* arguments are
 *     HOST pointers.  Anything else is passed by value.
 *   - All work is enqueued on the hipStream_t given at creation (passed as
 *     void*).  Calls are asynchronous except those that return host scalars
 *     (dblp_loss_account, dblp_phase_signal, dblp_get_counters,
 *     dblp_packetize with a slot map, dblp_packetize_list), which synchronise
 *     that stream; dblp_accumulator_copies does too.  dblp_apply_arrivals*
 *     never allocate and never wait, with one exception that the caller opts
 *     into: a context with TWO library-owned accumulator copies under the
 *     policy DBLP_ACC_AUTO times a probe kernel the first time it sees a packet
 *     buffer of 1 GiB or more (see "The accumulator and where it lives").
 *   - dblp_begin_round, dblp_apply_arrivals* (outside the exception above) and
 *     dblp_finalize only launch kernels on the context's stream, so a caller may
 *     record a round of them into a HIP graph by stream capture and replay it
 *     (tested: replays give the bits of the eager run).  The context's host-side
 *     bookkeeping is done when the calls are made, i.e. at capture: replay the
 *     recorded round as a whole, and call the functions that return host scalars
 *     outside the capture, after a replay.
 *   - A context is not thread-safe; use one per host thread.
 *
 * Geometry.  The gradient has N fp32 elements, tiled in order by B buckets
 * (e.g. one per tensor, Sec. "Metadata": layer names and chunk counts are
 * exchanged once before training; here they arrive as the bucket table).  A
 * bucket of c elements is cut into ceil(c / P) packets of P floats, the last
 * one short; packets never straddle buckets.  Sequence numbers run bucket-major
 * from 0 to n_pkts - 1 for every worker.
 *
 * Limits: at most DBLP_MAX_WORKERS (64) workers; fewer than 2^32 - 1 packets per worker and
 * round, slots per packet buffer and arrivals per batch; payloads of 1..65535 floats; a
 * bucket holds fewer than 2^32 elements; N itself is a 64-bit count.  Anything beyond is
 * refused with DBLP_EINVAL at dblp_create or at the call.
 *
 * Wire packet (Sec. "Metadata": sequence number, round counter, data length;
 * field widths are this library's choice), little-endian, `stride` bytes apart
 * with stride = 8 + 4P rounded up to 16:
 *     uint32 seq; uint16 round; uint16 len_floats; float payload[len_floats]; zero padding
 * With P = 366 the stride is 1472 bytes, the UDP payload of a 1500-byte MTU.
 * The worker a packet came from is not in the header (the paper identifies it
 * by the UDP port): it is given per slot in d_src_worker, or per arrival in the
 * descriptors of a receive queue (dblp_apply_arrivals_queue).
 */
#ifndef DBLP_AGG_H
#define DBLP_AGG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DBLP_OK 0
#define DBLP_EINVAL (-1)    /* bad argument (null, out of range, misaligned) */
#define DBLP_ENOMEM (-2)    /* host or device allocation failed */
#define DBLP_ECAPACITY (-3) /* retransmit list longer than the caller's buffer (count still valid) */
#define DBLP_ESTATE (-4)    /* call out of order (e.g. apply before begin_round) */
#define DBLP_EHIP (-5)      /* a HIP call failed; see dblp_last_error() */

#define DBLP_COMP_ZEROFILL_MEAN 0 /* the paper's compensation: missing = 0, divide by all W */

#define DBLP_MAX_WORKERS 64

typedef struct dblp_ctx dblp_ctx;

typedef struct {
    uint64_t elem_offset; /* first element; buckets must tile [0, n_elems) in order */
    uint64_t elem_count;  /* > 0, < 2^32 */
} dblp_bucket;

typedef struct {
    uint32_t n_workers;      /* W, 1..DBLP_MAX_WORKERS */
    uint32_t payload_floats; /* P, 1..65535 */
    uint64_t n_elems;        /* N */
    uint32_t n_buckets;      /* B */
    const dblp_bucket* buckets; /* HOST array of B entries, copied */
    double eta;              /* Eq. 1 threshold; the paper uses 0.5 */
    int device;              /* HIP device ordinal */
    void* stream;            /* hipStream_t; NULL = the null stream */
    /* The accumulator (see "The accumulator and where it lives"); all zero = one copy that the
     * library allocates. */
    int accumulator_mode;        /* DBLP_ACCMODE_SINGLE, _PAIR or _SEARCH */
    float* d_accumulator[2];     /* caller-owned DEVICE buffers of n_elems floats, 256-byte aligned, or
                                    NULL: [0] the accumulator, [1] the second copy (PAIR only).  They stay
                                    the caller's and must outlive the context. */
    double search_free_fraction; /* SEARCH: share of the memory that is FREE when dblp_create runs that the
                                    search may hold at once, 0 < f <= 0.9; 0 = 0.5 */
    double search_seconds;       /* SEARCH: time limit of the search; 0 = 2 seconds */
} dblp_config;

#define DBLP_ACCMODE_SINGLE 0 /* one accumulator */
#define DBLP_ACCMODE_PAIR 1   /* two copies, the second a plain allocation (or d_accumulator[1]) */
#define DBLP_ACCMODE_SEARCH 2 /* two copies, the second searched for in another third of HBM; one copy if none is found */

/* Allocates the context and its device state (bitmap W x ceil(n_pkts/64) words, arrival
 * index W x n_pkts x 8 bytes, accumulator N floats in one or two copies unless the caller
 * supplies them, one byte per packet sequence number, per-bucket counters).  Under
 * DBLP_ACCMODE_SEARCH it also searches for the second accumulator copy (see below) within the
 * limits given in the configuration.  *out is set only on success.  Errors: EINVAL (bad table,
 * W too large, n_pkts >= 2^32, unknown mode, misaligned or inconsistent caller buffers), ENOMEM,
 * EHIP. */
int dblp_create(dblp_ctx** out, const dblp_config* cfg);

/* Frees everything the context owns.  NULL is accepted. */
int dblp_destroy(dblp_ctx* ctx);

/* Sizes a caller needs to allocate buffers: packets per worker per round, wire stride in
 * bytes, bitmap words per worker.  Any output pointer may be NULL. */
int dblp_layout(const dblp_ctx* ctx, uint64_t* n_pkts_per_worker, uint32_t* packet_stride_bytes,
                uint64_t* bitmap_words_per_worker);

/* The accumulator and where it lives.  Not in the paper: a property of this memory system.
 * A payload stream with a few percent of result writes mixed in runs about 15 % slower on
 * MI355X when reads and writes fall into the same third of the HBM address space than when
 * they fall into different thirds.  A context can therefore keep the accumulator (N floats) in
 * two copies: the spans a batch writes for the first time go to one of them, later batches
 * update a span where it lives, and dblp_finalize reads each span from its copy.  Results do
 * not depend on any of this.  The caller decides (dblp_config.accumulator_mode):
 *   DBLP_ACCMODE_SINGLE  one copy (the default).  Nothing is measured, nothing is searched.
 *   DBLP_ACCMODE_PAIR    a second copy, allocated plainly or supplied by the caller.
 *   DBLP_ACCMODE_SEARCH  a second copy in another third than the first: candidates are
 *       allocated 6 GiB apart and a probe kernel is timed writing to each until one differs
 *       from the first copy.  The search holds at most search_free_fraction of the memory that
 *       was free when it started, stops after search_seconds, and releases everything but the
 *       copy it adopts; when it finds none the context has one copy (dblp_accumulator_info
 *       tells).  Both copies are the library's (d_accumulator must be NULL).
 * Caller-owned buffers (d_accumulator): [0] becomes the accumulator, which makes
 * dblp_finalize(d_out = that buffer) an in-place operation; [1] is used under PAIR.  The
 * library never measures caller-owned buffers: with them DBLP_ACC_AUTO behaves as
 * DBLP_ACC_FIRST.
 *
 * dblp_accumulator_copies(copies = 1|2, place) reallocates library-owned copies later: place
 *   = 0 plain allocation, 1 the bounded search described above.  Synchronises the stream and
 *   discards the round in progress (call dblp_begin_round again).  EINVAL on a context with
 *   caller-owned buffers.  ENOMEM if not even one copy fits; the context then has no
 *   accumulator and dblp_begin_round returns ESTATE until a later call succeeds.
 * dblp_accumulator_policy: which copy the spans that a batch writes first go to.
 *   DBLP_ACC_AUTO (default): with two library-owned copies, the first batch seen from each
 *   packet buffer of at least 1 GiB is preceded by a timed probe kernel (about 3 ms once per
 *   buffer, synchronising the stream; it reads d_packets[0 .. n_slots * stride) and writes a
 *   scratch area that the library keeps behind each copy) and the answer is remembered for the
 *   last 32 buffers (the second copy is chosen when the probe finds it faster by 3 %, plus,
 *   while results are left in place, what dblp_finalize spends moving its spans to the first); smaller or thinly used buffers, and contexts with one copy or with
 *   caller-owned copies, use the first copy without measuring.  FIRST / SECOND force a copy,
 *   ALTERNATE switches on every batch (for tests).  Select FIRST or SECOND before calling
 *   dblp_apply_arrivals* on a stream that is being captured.
 * dblp_accumulator_info: number of copies, whether they were measured to lie in different
 *   thirds, the copy the last batch wrote new spans to, and the placement measurement
 *   (placement_ms[0], [1]: probe time in ms writing to the first / second copy, 0 if not
 *   taken; [2]: candidates the search tried; [3]: seconds the search took).  Any pointer may be NULL.
 * dblp_accumulator_ptr: device address of copy `which` (0 or 1; EINVAL if it does not exist).
 *   Copy 0 holds the result after an in-place dblp_finalize. */
#define DBLP_ACC_AUTO 0
#define DBLP_ACC_FIRST 1
#define DBLP_ACC_SECOND 2
#define DBLP_ACC_ALTERNATE 3
int dblp_accumulator_copies(dblp_ctx* ctx, int copies, int place);
int dblp_accumulator_policy(dblp_ctx* ctx, int policy);
int dblp_accumulator_info(const dblp_ctx* ctx, int* copies, int* distinct_thirds, int* last_pick,
                          double placement_ms[4]);
int dblp_accumulator_ptr(const dblp_ctx* ctx, int which, float** d_copy);

/* Alg. "DBLP_RECV", initialisation: empty bitmap, nothing received, counters zero; `round`
 * is the round counter that arriving packets must carry.  The accumulator is not cleared:
 * a packet's first arrival overwrites its span and dblp_finalize writes zeros for spans
 * that never arrived, which gives the same result as a zero-initialised buffer. */
int dblp_begin_round(dblp_ctx* ctx, uint16_t round);

/* Sender side (Alg. "DBLP Send": split data into chunks).  Not part of the timed receiver
 * path.  d_grad holds elements [elem_base, elem_base + n_grad_elems) of worker w's gradient.
 * Packets first_seq .. first_seq + n_pkts - 1 are written; packet i goes to slot
 * d_slot_map[i] (device array, may be NULL: slot_base + i).  Slots must be < n_slots
 * (the capacity of d_packets in packets and of d_src_worker in entries); a slot outside is
 * skipped and the call returns EINVAL.  `round` is written into the headers.
 * Errors: EINVAL if the packets' elements are not inside the gradient window. */
int dblp_packetize(dblp_ctx* ctx, uint32_t w, uint16_t round, const float* d_grad,
                   uint64_t elem_base, uint64_t n_grad_elems, uint64_t first_seq, uint64_t n_pkts,
                   const uint32_t* d_slot_map, uint64_t slot_base, uint64_t n_slots,
                   void* d_packets, uint16_t* d_src_worker);

/* Sender side, retransmission (Alg. "DBLP Send": after a bitmap reply only the lost packets
 * are sent again).  Entry i of d_retx_list, (w << 32) | seq as produced by dblp_loss_account,
 * becomes the packet at slot slot_base + i of d_packets (and d_src_worker[slot_base + i] = w).
 * h_grads: HOST array of n_workers DEVICE pointers, h_grads[w] = worker w's whole gradient
 * (N floats).  n_slots is the capacity of d_packets / d_src_worker.  An entry whose worker or
 * seq is out of range is skipped and the call returns EINVAL.  Synchronises the stream. */
int dblp_packetize_list(dblp_ctx* ctx, uint16_t round, const float* const* h_grads,
                        const uint64_t* d_retx_list, uint64_t n_entries, uint64_t slot_base,
                        uint64_t n_slots, void* d_packets, uint16_t* d_src_worker);

/* Alg. "DBLP_RECV", chunk-arrival branch, for one batch of arrivals (property 1 of the
 * paper: packets are applied as they arrive, in any order).
 *   d_packets     n_slots wire packets, 16-byte aligned, `stride` bytes apart
 *   d_src_worker  n_slots entries: worker each slot's packet arrived from
 *   d_mask_words  ceil(n_slots/64) words, bit s%64 of word s/64 = slot s survived the
 *                 network; a lost slot is never read.  NULL = all survived.
 *   d_order       n_arrivals entries, d_order[k] = slot of the k-th arrival; a slot may
 *                 appear any number of times.  NULL = identity (then n_arrivals <= n_slots).
 * Per arrival: round != current -> stale (Sec. "Bounded-Loss-Tolerant Transmission");
 * worker, seq or length inconsistent with the geometry, or slot >= n_slots -> invalid;
 * already in the bitmap -> duplicate; otherwise accepted: bitmap bit set and payload added
 * to the accumulator.  If two copies of one packet arrive in the same batch the earlier
 * arrival is used.  The sum over workers of one packet is formed in worker order, so the
 * result does not depend on the arrival permutation.  Requires begin_round. */
int dblp_apply_arrivals(dblp_ctx* ctx, const void* d_packets, const uint16_t* d_src_worker,
                        uint64_t n_slots, const uint64_t* d_mask_words, const uint32_t* d_order,
                        uint64_t n_arrivals);

/* The same step (Alg. "DBLP_RECV", chunk-arrival branch) with the batch given as a receive
 * queue: one 8-byte descriptor per datagram that actually arrived, in arrival order, as a
 * receive loop sees them (each datagram comes with the address it was sent from).
 *   d_queue       n_arrivals descriptors, 8-byte aligned:
 *                 bits 0..31 slot of the packet in d_packets, bits 32..47 worker it came
 *                 from, bits 48..63 zero.  Lost packets simply have no descriptor.
 * Equivalent to dblp_apply_arrivals with d_order[k] = slot of descriptor k, d_src_worker taken
 * from the descriptors and no mask, and classifies every arrival the same way (a descriptor
 * with a non-zero reserved field, a worker >= n_workers or a slot >= n_slots is invalid).  It
 * is the faster form: the descriptor is read coalesced, where the per-slot worker table and
 * the mask cost a random access each.  Requires begin_round. */
int dblp_apply_arrivals_queue(dblp_ctx* ctx, const void* d_packets, uint64_t n_slots,
                              const uint64_t* d_queue, uint64_t n_arrivals);

/* One probe (Alg. "DBLP_RECV" probe branch; Sec. "Dynamically Changing Loss Tolerance":
 * retransmission stops once missing/total <= p, and only lost packets are resent).
 * For every (worker w, bucket b): missing = packets of b not in w's bitmap; the pair meets
 * the tolerance iff missing <= floor(bound_ppm * n_b / 10^6).  The retransmit list is every
 * missing (w, seq) of every pair that does not meet it, encoded (w << 32) | seq, ascending.
 *   d_missing      [W*B] counts, index w*B + b; may be NULL
 *   d_retx_list    retx_capacity entries; may be NULL iff retx_capacity == 0
 *   h_retx_count   full list length (even when it exceeds the capacity)
 *   h_all_met      1 iff the list is empty
 * Returns ECAPACITY if the list was truncated to retx_capacity entries. */
int dblp_loss_account(dblp_ctx* ctx, uint32_t bound_ppm, uint32_t* d_missing, uint64_t* d_retx_list,
                      uint64_t retx_capacity, uint64_t* h_retx_count, int* h_all_met);

/* Alg. "DBLP_RECV" last statements + Alg. "Server" mean: d_out[e] = acc[e] / W where
 * unreceived chunks count as zero (a span no worker delivered is exactly 0).  d_out: 16-byte
 * aligned, N floats.  Only DBLP_COMP_ZEROFILL_MEAN is defined by the paper; other values give
 * EINVAL.  When W is a power of two the division is exact and is applied as the payloads are
 * summed, so the first accumulator copy already holds the mean of what arrived; then
 *   d_out == NULL, or d_out == the first accumulator copy (dblp_accumulator_ptr, or the
 *   caller's d_accumulator[0]): IN PLACE.  Only spans that nobody delivered are written (zeros)
 *   and spans that live in the second copy are moved over; the result is read from copy 0.
 *   With W not a power of two this form returns EINVAL.
 *   any other d_out: the mean is written there (one read and one write of N floats).
 * Arrivals may still be applied after a finalize (then finalize again).  The sum of squares of
 * the result is kept for dblp_phase_signal. */
int dblp_finalize(dblp_ctx* ctx, int compensation, float* d_out);

/* Eq. 1: norm = ||G_curr||_2 of the aggregated gradient; rel_delta = | ||G_prev|| - norm | /
 * ||G_prev||; critical = rel_delta >= eta.  With no previous norm (or a zero one) rel_delta
 * is +inf and critical is 1 (training starts in the critical regime).  The stored previous
 * norm is replaced by `norm`.  d_vec == NULL uses the sum of squares produced by the last
 * dblp_finalize of this round (ESTATE if there was none); otherwise d_vec is N floats,
 * 16-byte aligned, and is reduced here. */
int dblp_phase_signal(dblp_ctx* ctx, const float* d_vec, double* h_norm, double* h_rel_delta,
                      int* h_critical);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the reduction of dblp_phase_signal(d_vec) without a context and without
 * any allocation, here or in a library it calls.  *d_sumsq (DEVICE, 8-byte aligned) receives
 * sum(d_vec[i]^2) in double over n_elems floats (DEVICE, 16-byte aligned), enqueued on `stream`
 * of `device`; the caller takes the square root and applies Eq. 1 once the stream has reached
 * that point.  The per-block partial sums live in a static device array of 32 KB that every GPU
 * the library runs on holds until the process ends; all calls on one GPU share it, so calls that
 * overlap on one GPU (different streams, different threads) race: order them.  The array keeps
 * the last call's contents; every call overwrites what it reads.  Limits: n_elems 1..2^36,
 * device 0..15; beyond them EINVAL.  Same arithmetic and block order as dblp_phase_signal, hence
 * the same bits.  dblp_sumsq_static_error() gives the text of this thread's last failure. */
int dblp_sumsq_static(int device, void* stream, const float* d_vec, uint64_t n_elems, double* d_sumsq);
const char* dblp_sumsq_static_error(void);

/* Copies the bitmap, W x bitmap_words_per_worker words, bit seq%64 of word seq/64. */
int dblp_get_bitmap(dblp_ctx* ctx, uint64_t* d_bitmap_out);

/* h_counters = {accepted, duplicate, stale, invalid} since begin_round. */
int dblp_get_counters(dblp_ctx* ctx, uint64_t h_counters[4]);

/* The only state that survives a round: ||G_prev||.  have = 0 means "none yet". */
int dblp_set_prev_norm(dblp_ctx* ctx, double norm, int have);
int dblp_get_prev_norm(const dblp_ctx* ctx, double* h_norm, int* h_have);

/* Optional tracing: `on` is a bit mask of kernel groups (bit DBLP_K_* set = the launches of that
 * group are bracketed by HIP events on the context's stream; 0 = off, 31 = all five; a bracket
 * costs two event records, 10-17 us of the stream's time, which shows on small rounds).  dblp_profile_read synchronises the stream, returns
 * the summed duration (milliseconds) and number of launches recorded for one kernel group
 * since the last read of that group, and forgets them.  At most 16384 brackets are kept between
 * reads; further ones are dropped.  dblp_profile_enable may return ENOMEM. */
#define DBLP_K_INDEX 0    /* header parse / validation / arrival index */
#define DBLP_K_GATHER 1   /* payload gather + accumulate, staged kernel (dense batches) */
#define DBLP_K_PROBE 2    /* loss count + prefix + retransmit list (three launches, one bracket) */
#define DBLP_K_FINALIZE 3 /* zero-fill mean + partial sums of squares */
#define DBLP_K_GATHER_DIRECT 4 /* the same, direct kernel (sparse batches, packets too long to stage) */
#define DBLP_K_COUNT 5
int dblp_profile_enable(dblp_ctx* ctx, int on);
int dblp_profile_read(dblp_ctx* ctx, int kernel, double* h_total_ms, uint64_t* h_launches);

/* Text of the last error on this context (valid until the next call on it). */
const char* dblp_last_error(const dblp_ctx* ctx);

/* Tolerance policies: host scalars that turn the phase signal into the next bound (ppm).
 * two_level is the paper's rule (Sec. "Centralized All-Reduce Architecture", Table 1):
 * critical -> P_low, otherwise P_high = P_low + k; the first iteration is critical.
 * three_level and linear are extensions for workloads that step through more levels:
 *   three_level: delta >= eta -> tight; eta/2 <= delta < eta -> mid; else loose
 *   linear:      hi - (hi - lo) * min(delta/eta, 1), rounded to a multiple of 1000 ppm */
uint32_t dblp_policy_two_level(int critical, uint32_t p_low_ppm, uint32_t p_high_ppm);
uint32_t dblp_policy_three_level(double rel_delta, double eta, uint32_t tight_ppm, uint32_t mid_ppm,
                                 uint32_t loose_ppm);
uint32_t dblp_policy_linear(double rel_delta, double eta, uint32_t lo_ppm, uint32_t hi_ppm);

/* Epoch-level tolerance controller, Alg. "Server" (the tolerance block inside the loop) and Sec.
 * "Centralized All-Reduce Architecture": the threshold starts at P_low; at the first
 * iteration of every epoch it is reset to P_high and, if that iteration's gradient triggers
 * critical-regime detection (Eq. 1), set to P_low; inside an epoch it does not change.
 * The caller owns the state (plain struct, host memory).  dblp_clr_init sets bound_ppm = P_low;
 * dblp_clr_step is called once per iteration, after dblp_phase_signal, with that iteration's
 * `critical` flag, and returns the bound for the following iterations (also left in
 * state->bound_ppm).  iters_per_epoch must be >= 1. */
typedef struct {
    uint32_t p_low_ppm, p_high_ppm, iters_per_epoch;
    uint32_t bound_ppm; /* tolerance currently in force */
    uint64_t step;      /* iterations seen so far */
} dblp_clr_state;
int dblp_clr_init(dblp_clr_state* state, uint32_t p_low_ppm, uint32_t p_high_ppm, uint32_t iters_per_epoch);
uint32_t dblp_clr_step(dblp_clr_state* state, int critical);

#ifdef __cplusplus
}
#endif
#endif /* DBLP_AGG_H */
