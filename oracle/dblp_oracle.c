/*
 * CPU oracle for the receiver side of DBLP (bounded-loss gradient aggregation).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * statement of what the receiver computes; it exists so that the GPU library
 * can be compared against something written independently from the paper.  It
 * shares no code, header, table or helper with the GPU library and must never
 * be called from the product path.
 *
 * What it follows (DBLP paper):
 *   - Sec. "Metadata": every packet carries {sequence number, round counter,
 *     data length}; sequence numbers place out-of-order packets.
 *   - Sec. "Bounded-Loss-Tolerant Transmission": packets whose round counter is
 *     not the current round are dropped.
 *   - Alg. "DBLP_RECV": bitmap starts empty; a valid chunk is accepted and the
 *     bitmap updated; chunks never received stay zero-filled.
 *   - Sec. "Dynamically Changing Loss Tolerance": retransmission stops once the
 *     ratio of missing packets is equal to or less than the tolerance p; the
 *     sender retransmits only the lost packets of the latest bitmap.
 *   - Alg. "Server": the reduced gradient is the mean over all N workers of the
 *     (zero-filled) received gradients.
 *   - Eq. 1: | ||G_prev|| - ||G_curr|| | / ||G_prev|| >= eta  (L2 norm) marks a
 *     critical learning regime; eta = 0.5.
 *   - Sec. "Centralized All-Reduce Architecture" / Table 1: critical => P_low,
 *     otherwise P_high = P_low + k; the threshold starts at P_low.
 *
 * Readings where the paper is silent:
 *   header = little-endian {u32 seq, u16 round, u16 length in floats}, 8 bytes;
 *   the worker a packet came from is side information (the port it arrived on);
 *   loss is accounted per (worker, bucket), one bucket over the whole gradient
 *   reproducing the paper's per-round accounting; packets never straddle
 *   buckets, the last packet of a bucket is short; a second copy of a packet is
 *   ignored; the tolerance is an integer in parts per million and the test is
 *   missing * 10^6 <= bound_ppm * packets_in_bucket; the first iteration (no
 *   previous norm, or a zero one) counts as critical.
 *
 * oracle_apply_arrivals_mt is the same receiver step spread over threads by element range
 * (used only to time the baseline on all cores; pinned equal to the plain walk).
 *
 * Arithmetic: sums, mean and norm in IEEE double.  Parity status: every
 * function here is pinned by tests/test_oracle_*.py (brute force over all
 * masks and permutations, closed forms, the paper's constants) except the
 * three-level and linear tolerance policies, which the paper does not define:
 * those two are "parity unpinned" by the paper and pinned only by the
 * definitions written in their own comments below.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    uint32_t W;          /* workers */
    uint64_t N;          /* gradient elements */
    uint32_t P;          /* payload floats of a full packet */
    uint32_t B;          /* buckets */
    uint64_t* b_off;     /* [B] first element of bucket */
    uint64_t* b_cnt;     /* [B] elements in bucket */
    uint64_t* b_first;   /* [B] sequence number of the bucket's first packet */
    uint64_t* b_npk;     /* [B] packets in bucket */
    uint64_t n_pkts;     /* packets per worker per round */
    uint32_t* bucket_of; /* [n_pkts] bucket of each sequence number */
    uint8_t* received;   /* [W][n_pkts] the bitmap, one byte per bit */
    double* acc;         /* [N] running sum of accepted payloads */
    uint16_t round;
    double eta;
    double prev_norm;
    int have_prev;
    uint64_t accepted, duplicate, stale, invalid;
} oracle_t;

void oracle_destroy(oracle_t* o) {
    if (!o) return;
    free(o->b_off); free(o->b_cnt); free(o->b_first); free(o->b_npk);
    free(o->bucket_of); free(o->received); free(o->acc); free(o);
}

/* Buckets must tile [0, N) in order.  Returns NULL on a bad table or on allocation failure. */
oracle_t* oracle_create(uint32_t W, uint64_t N, uint32_t P, uint32_t B,
                        const uint64_t* bucket_off, const uint64_t* bucket_cnt, double eta) {
    if (W == 0 || N == 0 || P == 0 || P > 65535 || B == 0) return NULL;
    uint64_t expect = 0;
    for (uint32_t b = 0; b < B; ++b) {
        if (bucket_off[b] != expect || bucket_cnt[b] == 0) return NULL;
        expect += bucket_cnt[b];
    }
    if (expect != N) return NULL;
    oracle_t* o = (oracle_t*)calloc(1, sizeof *o);
    if (!o) return NULL;
    o->W = W; o->N = N; o->P = P; o->B = B; o->eta = eta;
    o->b_off = (uint64_t*)malloc(B * sizeof(uint64_t));
    o->b_cnt = (uint64_t*)malloc(B * sizeof(uint64_t));
    o->b_first = (uint64_t*)malloc(B * sizeof(uint64_t));
    o->b_npk = (uint64_t*)malloc(B * sizeof(uint64_t));
    if (!o->b_off || !o->b_cnt || !o->b_first || !o->b_npk) { oracle_destroy(o); return NULL; }
    uint64_t seq = 0;
    for (uint32_t b = 0; b < B; ++b) {
        o->b_off[b] = bucket_off[b];
        o->b_cnt[b] = bucket_cnt[b];
        o->b_first[b] = seq;
        o->b_npk[b] = (bucket_cnt[b] + P - 1) / P;
        seq += o->b_npk[b];
    }
    o->n_pkts = seq;
    if (seq > 0xFFFFFFFFull) { oracle_destroy(o); return NULL; }
    o->bucket_of = (uint32_t*)malloc(seq * sizeof(uint32_t));
    o->received = (uint8_t*)calloc((size_t)W * seq, 1);
    o->acc = (double*)calloc(N, sizeof(double));
    if (!o->bucket_of || !o->received || !o->acc) { oracle_destroy(o); return NULL; }
    for (uint32_t b = 0; b < B; ++b)
        for (uint64_t k = 0; k < o->b_npk[b]; ++k) o->bucket_of[o->b_first[b] + k] = b;
    return o;
}

uint64_t oracle_n_pkts(const oracle_t* o) { return o->n_pkts; }

/* Element offset and float count of the packet with this sequence number. */
static void packet_span(const oracle_t* o, uint64_t seq, uint64_t* elem, uint32_t* len) {
    uint32_t b = o->bucket_of[seq];
    uint64_t k = seq - o->b_first[b];
    uint64_t start = k * o->P;
    uint64_t left = o->b_cnt[b] - start;
    *elem = o->b_off[b] + start;
    *len = (uint32_t)(left < o->P ? left : o->P);
}

/* Alg. DBLP_RECV, first two statements: empty bitmap; the reconstruction buffer is zero. */
void oracle_begin_round(oracle_t* o, uint16_t round) {
    memset(o->received, 0, (size_t)o->W * o->n_pkts);
    memset(o->acc, 0, o->N * sizeof(double));
    o->round = round;
    o->accepted = o->duplicate = o->stale = o->invalid = 0;
}

/*
 * Sender side (Alg. DBLP Send, "split data into chunks"): worker w's gradient,
 * of which grad[0..n_grad) holds elements [elem_base, elem_base + n_grad), is
 * cut into the packets first_seq .. first_seq + n - 1.  Packet i is written at
 * slot slot_map[i] (or slot_base + i when slot_map is NULL) of `packets`
 * (stride bytes apart); src_worker[slot] = w.  `round` goes into the header
 * (a sender may be a round behind).  Returns 0, or -1 if a packet's elements
 * fall outside the supplied gradient window.
 */
int oracle_packetize(const oracle_t* o, uint32_t w, uint16_t round, const float* grad, uint64_t elem_base,
                     uint64_t n_grad, uint64_t first_seq, uint64_t n, const uint32_t* slot_map,
                     uint64_t slot_base, uint8_t* packets, uint64_t stride, uint16_t* src_worker) {
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t seq = first_seq + i, elem; uint32_t len;
        if (seq >= o->n_pkts) return -1;
        packet_span(o, seq, &elem, &len);
        if (elem < elem_base || elem + len > elem_base + n_grad) return -1;
        uint64_t slot = slot_map ? slot_map[i] : slot_base + i;
        uint8_t* p = packets + slot * stride;
        memset(p, 0, stride);
        p[0] = (uint8_t)(seq); p[1] = (uint8_t)(seq >> 8); p[2] = (uint8_t)(seq >> 16); p[3] = (uint8_t)(seq >> 24);
        p[4] = (uint8_t)(round); p[5] = (uint8_t)(round >> 8);
        p[6] = (uint8_t)(len); p[7] = (uint8_t)(len >> 8);
        memcpy(p + 8, grad + (elem - elem_base), (size_t)len * 4);
        src_worker[slot] = (uint16_t)w;
    }
    return 0;
}

/*
 * The headers alone of the same packets (Sec. "Metadata": sequence number, round counter,
 * data length), 8 bytes per slot and nothing else: what a receiver that only keeps the
 * books needs (oracle_apply_arrivals with accumulate == 0 and stride 8).  Same slot rule as
 * oracle_packetize; no gradient is needed because the length of a packet follows from its
 * sequence number.  Returns 0, or -1 if a sequence number is out of range.
 */
int oracle_write_headers(const oracle_t* o, uint32_t w, uint16_t round, uint64_t first_seq, uint64_t n,
                         const uint32_t* slot_map, uint64_t slot_base, uint8_t* headers, uint16_t* src_worker) {
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t seq = first_seq + i, elem; uint32_t len;
        if (seq >= o->n_pkts) return -1;
        packet_span(o, seq, &elem, &len);
        uint64_t slot = slot_map ? slot_map[i] : slot_base + i;
        uint8_t* p = headers + slot * 8;
        p[0] = (uint8_t)(seq); p[1] = (uint8_t)(seq >> 8); p[2] = (uint8_t)(seq >> 16); p[3] = (uint8_t)(seq >> 24);
        p[4] = (uint8_t)(round); p[5] = (uint8_t)(round >> 8);
        p[6] = (uint8_t)(len); p[7] = (uint8_t)(len >> 8);
        src_worker[slot] = (uint16_t)w;
    }
    return 0;
}

/*
 * Receiver (Alg. DBLP_RECV, the chunk-arrival branch), for one batch of
 * arrivals.  order[k] is the slot of the k-th arrival (NULL: k itself);
 * mask bit s (NULL: all ones) says whether slot s survived the network, a lost
 * slot is never looked at.  With accumulate == 0 only headers are read (the
 * bitmap and counters are maintained, payloads are ignored).
 */
void oracle_apply_arrivals(oracle_t* o, const uint8_t* packets, uint64_t stride,
                           const uint16_t* src_worker, uint64_t n_slots, const uint64_t* mask,
                           const uint32_t* order, uint64_t n_arrivals, int accumulate) {
    for (uint64_t k = 0; k < n_arrivals; ++k) {
        uint64_t s = order ? order[k] : k;
        if (s >= n_slots) { o->invalid++; continue; }
        if (mask && !((mask[s >> 6] >> (s & 63)) & 1)) continue;
        const uint8_t* p = packets + s * stride;
        uint32_t seq = (uint32_t)p[0] | (uint32_t)p[1] << 8 | (uint32_t)p[2] << 16 | (uint32_t)p[3] << 24;
        uint16_t rnd = (uint16_t)(p[4] | p[5] << 8);
        uint16_t len = (uint16_t)(p[6] | p[7] << 8);
        uint32_t w = src_worker[s];
        if (rnd != o->round) { o->stale++; continue; }             /* other communication cycle */
        if (w >= o->W || seq >= o->n_pkts) { o->invalid++; continue; }
        uint64_t elem; uint32_t want;
        packet_span(o, seq, &elem, &want);
        if (len != want) { o->invalid++; continue; }                /* integrity check */
        uint8_t* bit = &o->received[(uint64_t)w * o->n_pkts + seq];
        if (*bit) { o->duplicate++; continue; }
        *bit = 1;                                                   /* accept, update bitmap */
        o->accepted++;
        if (accumulate) {
            for (uint32_t j = 0; j < len; ++j) {
                float v; memcpy(&v, p + 8 + 4 * (size_t)j, 4);
                o->acc[elem + j] += (double)v;
            }
        }
    }
}

/*
 * The same batch on several threads, for the all-cores timing of the baseline.  Thread t owns
 * the sequence numbers [t * n_pkts / T, (t + 1) * n_pkts / T), i.e. a disjoint element range of
 * the reconstruction buffer; every thread walks ALL arrivals in arrival order and handles the
 * ones whose header names a sequence number it owns (thread 0 also takes the arrivals whose
 * sequence number or slot is out of range).  Each packet is therefore classified exactly once,
 * by the same tests in the same order as in oracle_apply_arrivals, first copies still win, and
 * every element receives its addends in arrival order: bitmap, counters and sums are identical
 * to the single-threaded walk (pinned in tests/test_oracle_pins.py).  n_threads <= 0: as many as
 * OpenMP offers.  Returns the number of threads used.
 */
int oracle_apply_arrivals_mt(oracle_t* o, const uint8_t* packets, uint64_t stride,
                             const uint16_t* src_worker, uint64_t n_slots, const uint64_t* mask,
                             const uint32_t* order, uint64_t n_arrivals, int accumulate, int n_threads) {
    int used = 1;
    uint64_t accepted = 0, duplicate = 0, stale = 0, invalid = 0;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
#else
    n_threads = 1;
#endif
    #pragma omp parallel num_threads(n_threads) reduction(+ : accepted, duplicate, stale, invalid)
    {
        int T = 1, t = 0;
#ifdef _OPENMP
        T = omp_get_num_threads(); t = omp_get_thread_num();
#endif
        #pragma omp single
        used = T;
        const uint64_t own_lo = o->n_pkts * (uint64_t)t / (uint64_t)T, own_hi = o->n_pkts * (uint64_t)(t + 1) / (uint64_t)T;
        for (uint64_t k = 0; k < n_arrivals; ++k) {
            uint64_t s = order ? order[k] : k;
            if (s >= n_slots) { if (t == 0) invalid++; continue; }
            if (mask && !((mask[s >> 6] >> (s & 63)) & 1)) continue;
            const uint8_t* p = packets + s * stride;
            uint32_t seq = (uint32_t)p[0] | (uint32_t)p[1] << 8 | (uint32_t)p[2] << 16 | (uint32_t)p[3] << 24;
            if (seq < o->n_pkts ? (seq < own_lo || seq >= own_hi) : t != 0) continue;    /* another thread's */
            uint16_t rnd = (uint16_t)(p[4] | p[5] << 8);
            uint16_t len = (uint16_t)(p[6] | p[7] << 8);
            uint32_t w = src_worker[s];
            if (rnd != o->round) { stale++; continue; }
            if (w >= o->W || seq >= o->n_pkts) { invalid++; continue; }
            uint64_t elem; uint32_t want;
            packet_span(o, seq, &elem, &want);
            if (len != want) { invalid++; continue; }
            uint8_t* bit = &o->received[(uint64_t)w * o->n_pkts + seq];
            if (*bit) { duplicate++; continue; }
            *bit = 1;
            accepted++;
            if (accumulate) {
                for (uint32_t j = 0; j < len; ++j) {
                    float v; memcpy(&v, p + 8 + 4 * (size_t)j, 4);
                    o->acc[elem + j] += (double)v;
                }
            }
        }
    }
    o->accepted += accepted; o->duplicate += duplicate; o->stale += stale; o->invalid += invalid;
    return used;
}

/*
 * One probe.  For every (worker, bucket): missing = packets of the bucket not
 * in the bitmap; the bucket meets the tolerance iff missing / packets <= bound,
 * tested in integers as missing * 10^6 <= bound_ppm * packets.  The retransmit
 * list holds every missing (worker, seq) of every bucket that does not meet
 * it, worker ascending then seq ascending, encoded (w << 32) | seq.
 * missing_out ([W*B], may be NULL) gets the counts.  At most `capacity` list
 * entries are written; *count is the full length.
 */
void oracle_loss_account(const oracle_t* o, uint32_t bound_ppm, uint32_t* missing_out,
                         uint64_t* list, uint64_t capacity, uint64_t* count, int* all_met) {
    uint64_t n = 0;
    for (uint32_t w = 0; w < o->W; ++w) {
        for (uint32_t b = 0; b < o->B; ++b) {
            uint64_t miss = 0;
            for (uint64_t k = 0; k < o->b_npk[b]; ++k)
                if (!o->received[(uint64_t)w * o->n_pkts + o->b_first[b] + k]) miss++;
            if (missing_out) missing_out[(uint64_t)w * o->B + b] = (uint32_t)miss;
            int ok = miss * 1000000ull <= (uint64_t)bound_ppm * o->b_npk[b];
            if (ok) continue;
            for (uint64_t k = 0; k < o->b_npk[b]; ++k) {
                uint64_t seq = o->b_first[b] + k;
                if (!o->received[(uint64_t)w * o->n_pkts + seq]) {
                    if (n < capacity) list[n] = ((uint64_t)w << 32) | seq;
                    n++;
                }
            }
        }
    }
    *count = n;
    *all_met = (n == 0);
}

/* Alg. DBLP_RECV last statements + Alg. Server mean: unreceived chunks are zero;
   out = (sum over workers of the zero-filled gradients) / W. */
void oracle_finalize(const oracle_t* o, double* out) {
    for (uint64_t e = 0; e < o->N; ++e) out[e] = o->acc[e] / (double)o->W;
}

/* Eq. 1 on the aggregated gradient.  Updates the stored previous norm. */
void oracle_phase_signal(oracle_t* o, const double* out, double* norm, double* rel_delta, int* critical) {
    double ss = 0.0;
    for (uint64_t e = 0; e < o->N; ++e) ss += out[e] * out[e];
    double cur = sqrt(ss);
    if (!o->have_prev || o->prev_norm == 0.0) {
        *rel_delta = INFINITY;
        *critical = 1;
    } else {
        *rel_delta = fabs(o->prev_norm - cur) / o->prev_norm;
        *critical = (*rel_delta >= o->eta);
    }
    *norm = cur;
    o->prev_norm = cur;
    o->have_prev = 1;
}

void oracle_set_prev_norm(oracle_t* o, double v, int have) { o->prev_norm = v; o->have_prev = have; }

void oracle_get_received(const oracle_t* o, uint8_t* out) { memcpy(out, o->received, (size_t)o->W * o->n_pkts); }
void oracle_get_acc(const oracle_t* o, double* out) { memcpy(out, o->acc, o->N * sizeof(double)); }
void oracle_get_counters(const oracle_t* o, uint64_t c[4]) {
    c[0] = o->accepted; c[1] = o->duplicate; c[2] = o->stale; c[3] = o->invalid;
}

/* ---- tolerance policies (host scalars) ---- */

/* The paper's two-level rule: critical => P_low, else P_high. */
uint32_t oracle_policy_two_level(int critical, uint32_t p_low_ppm, uint32_t p_high_ppm) {
    return critical ? p_low_ppm : p_high_ppm;
}

static uint32_t quantise_1000(double ppm) { return (uint32_t)(floor(ppm / 1000.0 + 0.5) * 1000.0); }

/* Extension (not in the paper): delta >= eta -> tight; eta/2 <= delta < eta -> mid; else loose. */
uint32_t oracle_policy_three_level(double rel_delta, double eta, uint32_t tight_ppm, uint32_t mid_ppm,
                                   uint32_t loose_ppm) {
    if (rel_delta >= eta) return tight_ppm;
    if (rel_delta >= eta / 2) return mid_ppm;
    return loose_ppm;
}

/* Extension (not in the paper): bound = hi - (hi - lo) * min(delta / eta, 1), rounded to 1000 ppm. */
uint32_t oracle_policy_linear(double rel_delta, double eta, uint32_t lo_ppm, uint32_t hi_ppm) {
    double x = rel_delta / eta;
    if (!(x < 1.0)) x = 1.0;
    return quantise_1000((double)hi_ppm - ((double)hi_ppm - (double)lo_ppm) * x);
}

/*
 * Epoch-level controller (Alg. Server, the tolerance block; Sec. "Centralized All-Reduce
 * Architecture").  Written as the paper's loop reads: the threshold is initialised to P_low;
 * for each step, if the step is the beginning of an epoch the threshold is reset to P_high and
 * then, if CLR is detected, set to P_low.  `critical[s]` is the Eq. 1 outcome of step s;
 * bound_after[s] receives the threshold in force once step s has been handled.
 */
void oracle_clr_trace(uint32_t p_low_ppm, uint32_t p_high_ppm, uint32_t iters_per_epoch,
                      const uint8_t* critical, uint64_t n_steps, uint32_t* bound_after) {
    uint32_t threshold = p_low_ppm;
    for (uint64_t step = 0; step < n_steps; ++step) {
        int at_epoch_start = (step % iters_per_epoch) == 0;
        if (at_epoch_start) {
            threshold = p_high_ppm;
            if (critical[step]) threshold = p_low_ppm;
        }
        bound_after[step] = threshold;
    }
}
