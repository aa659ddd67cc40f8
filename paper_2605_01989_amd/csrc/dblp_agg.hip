// Receiver-side bounded-loss gradient aggregation of DBLP on gfx950 (MI355X).
// Kernels and the C-ABI declared in include/dblp_agg.h.
//
// Data flow of one arrival batch (Alg. "DBLP_RECV", chunk-arrival branch):
//   index_arrivals   one thread per arrival: header parse, validation, and an atomicMin of
//                    (arrival rank << 32 | slot) into the arrival index `pending[w][seq]`, so the
//                    earliest copy of a packet in the batch wins; per-block tallies (stale, invalid,
//                    candidates, touched seq range) that every gather block adds up for itself
//   gather_accumulate_staged / gather_accumulate
//                    organised by OUTPUT packet: a block takes a group of consecutive sequence
//                    numbers, reads the index entries of all workers, drops copies of packets
//                    that an earlier batch delivered, sets the bitmap bits, then streams the
//                    payloads of each packet from every delivering worker (16-byte loads,
//                    worker order) into registers and writes the accumulator span once.
// Every payload byte is read exactly once and the accumulator is written once per batch that
// touches it; there are no floating-point atomics, so the sum is independent of the arrival
// permutation.  The accumulator may exist in two copies placed in different thirds of the HBM
// address space (classify_rw measures which copy a packet buffer should be paired with); a
// per-packet byte map records where each span lives.
//
// The probe (Sec. "Dynamically Changing Loss Tolerance"): loss_count (popcount of bitmap words +
// DPP wave reduction), scan_need (exclusive prefix of the per-(worker,bucket) list lengths) and
// emit_retx (ordered compaction).  The mean of Alg. "Server" is formed as the payloads are summed when
// W is a power of two (the division is exact), and the gather kernels keep the sum of squares of
// what they store, so finalize_pass only writes zeros where nothing arrived (and moves or copies
// spans where the result is wanted elsewhere); for other W it divides and squares itself.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include <new>
#include <vector>

#include "../../include/dblp_agg.h"

typedef unsigned long long u64;
typedef uint32_t u32;

#define NONE64 0xFFFFFFFFFFFFFFFFull
#define WAVE 64

// device counters (u64 each)
enum { C_ACCEPTED = 0, C_STALE, C_INVALID, C_CANDIDATES, C_PKT_BAD, C_COUNT };

struct Geo {
    const u32* first_seq;   // [B+1]
    const u64* b_off;       // [B]
    const u64* b_cnt;       // [B]
    u32 B, P, W;
    u32 n_pkts;
    u32 stride;             // bytes
    u32 units;              // stride / 16
    u64 words_pw;           // bitmap words per worker
};

// ------------------------------------------------------------------------------------------
// wave-level primitives (64 lanes): DPP moves, reductions and scans
// ------------------------------------------------------------------------------------------
#define DPP_ROW_SHR(n) (0x110 + (n))
#define DPP_ROW_BCAST15 0x142
#define DPP_ROW_BCAST31 0x143

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ u32 dpp_u32(u32 identity, u32 v) {
    return (u32)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xF, false);
}

struct OpAdd { static __device__ __forceinline__ u32 id() { return 0u; } static __device__ __forceinline__ u32 f(u32 a, u32 b) { return a + b; } };
struct OpMin { static __device__ __forceinline__ u32 id() { return 0xFFFFFFFFu; } static __device__ __forceinline__ u32 f(u32 a, u32 b) { return a < b ? a : b; } };
struct OpMax { static __device__ __forceinline__ u32 id() { return 0u; } static __device__ __forceinline__ u32 f(u32 a, u32 b) { return a > b ? a : b; } };
struct OpOr { static __device__ __forceinline__ u32 id() { return 0u; } static __device__ __forceinline__ u32 f(u32 a, u32 b) { return a | b; } };

// Inclusive scan over the 64 lanes; all lanes must be active.  Lane 63 ends with the total.
template <class Op>
__device__ __forceinline__ u32 wave_scan_incl(u32 v) {
    v = Op::f(v, dpp_u32<DPP_ROW_SHR(1), 0xF>(Op::id(), v));
    v = Op::f(v, dpp_u32<DPP_ROW_SHR(2), 0xF>(Op::id(), v));
    v = Op::f(v, dpp_u32<DPP_ROW_SHR(4), 0xF>(Op::id(), v));
    v = Op::f(v, dpp_u32<DPP_ROW_SHR(8), 0xF>(Op::id(), v));
    v = Op::f(v, dpp_u32<DPP_ROW_BCAST15, 0xA>(Op::id(), v));
    v = Op::f(v, dpp_u32<DPP_ROW_BCAST31, 0xC>(Op::id(), v));
    return v;
}

template <class Op>
__device__ __forceinline__ u32 wave_reduce(u32 v) {
    return (u32)__builtin_amdgcn_readlane((int)wave_scan_incl<Op>(v), 63);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {
    u64 bits = (u64)__double_as_longlong(v);
    u32 lo = dpp_u32<CTRL, ROW_MASK>(0u, (u32)bits);
    u32 hi = dpp_u32<CTRL, ROW_MASK>(0u, (u32)(bits >> 32));
    return __longlong_as_double((long long)(((u64)hi << 32) | lo));   // identity 0.0 = all-zero bits
}

// Sum of a double over the 64 lanes (all active); every lane gets the total.
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<DPP_ROW_SHR(1), 0xF>(v);
    v += dpp_f64<DPP_ROW_SHR(2), 0xF>(v);
    v += dpp_f64<DPP_ROW_SHR(4), 0xF>(v);
    v += dpp_f64<DPP_ROW_SHR(8), 0xF>(v);
    v += dpp_f64<DPP_ROW_BCAST15, 0xA>(v);
    v += dpp_f64<DPP_ROW_BCAST31, 0xC>(v);
    u64 bits = (u64)__double_as_longlong(v);
    u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)bits, 63);
    u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(bits >> 32), 63);
    return __longlong_as_double((long long)(((u64)hi << 32) | lo));
}

// 16-byte load with the non-temporal hint: the payload is read exactly once, so it should not
// displace the accumulator and index lines that are being written in L2 / the memory-side cache
// (measured: 8 % off the payload pass).  Headers are NOT loaded this way in the index pass:
// their lines are read again by the payload pass and are worth keeping.
typedef float f4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld_stream4(const void* p) {
    const f4v t = __builtin_nontemporal_load((const f4v*)p);
    return make_float4(t.x, t.y, t.z, t.w);
}

// 16-byte store with the non-temporal hint (the sender's packets are not read again by the sender).
typedef u32 u4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st_stream4(uint4* p, uint4 v) {
    const u4v t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (u4v*)p);
}

__device__ __forceinline__ u32 lane_id() { return threadIdx.x & (WAVE - 1); }

// ------------------------------------------------------------------------------------------
// geometry helpers
// ------------------------------------------------------------------------------------------
// Largest b with first_seq[b] <= seq (seq < n_pkts).
__device__ __forceinline__ u32 find_bucket(const u32* __restrict__ fs, u32 B, u32 seq) {
    u32 lo = 0, hi = B;
    while (hi - lo > 1) {
        u32 mid = (lo + hi) >> 1;
        if (fs[mid] <= seq) lo = mid; else hi = mid;
    }
    return lo;
}

// First element and float count of packet `seq`, which lies in bucket b.
__device__ __forceinline__ void packet_span(const Geo& g, u32 seq, u32 b, u64* elem, u32* len) {
    u64 start = (u64)(seq - g.first_seq[b]) * g.P;
    u64 left = g.b_cnt[b] - start;
    *elem = g.b_off[b] + start;
    *len = left < g.P ? (u32)left : g.P;
}

// ------------------------------------------------------------------------------------------
// small utility kernels
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_u64(u64* __restrict__ p, u64 n, u64 v) {
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

__global__ void reset_counters(u64* __restrict__ c) {
    u32 t = threadIdx.x;
    if (t >= C_COUNT) return;
    c[t] = 0;
}

// Start of a round in one launch: bitmap and the gather kernels' per-block rows to zero, counters reset.
__global__ __launch_bounds__(256) void reset_round(u64* __restrict__ bitmap, u64 n_bitmap, u64* __restrict__ rows, u64 n_rows,
                                                   u64* __restrict__ counters) {
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n_bitmap + n_rows; i += stride) {
        if (i < n_bitmap) bitmap[i] = 0; else rows[i - n_bitmap] = 0;
    }
    if (blockIdx.x == 0 && threadIdx.x < C_COUNT) counters[threadIdx.x] = 0;
}

// counters[C_ACCEPTED] = sum of the per-block rows written by the gather kernels.  One block.
__global__ __launch_bounds__(256) void fold_accept_rows(const u64* __restrict__ rows, u32 n, u64* __restrict__ counters) {
    __shared__ u64 sh[256];
    u64 a[8] = {0, 0, 0, 0, 0, 0, 0, 0};          // eight loads in flight per thread
    for (u32 i = threadIdx.x; i < n; i += 256 * 8) {
        #pragma unroll
        for (u32 j = 0; j < 8; ++j) {
            const u32 k = i + j * 256;
            a[j] += k < n ? rows[k] : 0;
        }
    }
    sh[threadIdx.x] = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    __syncthreads();
    for (u32 d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) counters[C_ACCEPTED] = sh[0];
}

// ------------------------------------------------------------------------------------------
// sender: gradient -> wire packets
// ------------------------------------------------------------------------------------------
// One wave writes one packet: lane l builds 16-byte units l, l + 64, ... (header in the first 8
// bytes of unit 0, zero padding after the payload) and stores them aligned.  The payload is read
// with 8-byte loads when its first element is even (then every unit's two halves are 8-byte
// aligned in the gradient), else float by float.  All loads of a packet are issued before the
// first store; the stores carry the non-temporal hint (+11 %), the loads do not (with it: -8 %,
// the two halves of a unit share lines).  PK_UNITS = units per lane kept in registers (packets of up to PK_UNITS KB go in
// one pass, longer ones in several).
#define PK_UNITS 5
__device__ __forceinline__ void write_packet(const float* __restrict__ src, u32 len, u32 seq, u32 round, u32 units,
                                             uint4* __restrict__ dst, u32 lane) {
    const bool even = (((uintptr_t)src) & 7) == 0;         // src = address of payload float 0
    const u32 hdr1 = (round & 0xFFFFu) | (len << 16);
    for (u32 u0 = 0; u0 < units; u0 += PK_UNITS * WAVE) {
        uint4 q[PK_UNITS];
        #pragma unroll
        for (int k = 0; k < PK_UNITS; ++k) {
            const u32 u = u0 + k * WAVE + lane;            // packet float positions 4u .. 4u+3 = payload floats 4u-2 .. 4u+1
            q[k] = make_uint4(0u, 0u, 0u, 0u);
            if (u >= units) continue;
            const u32 p0 = 4 * u;
            if (even) {
                if (p0 >= 2 && p0 - 2 + 1 < len) { const uint2 t = *(const uint2*)(src + (p0 - 2)); q[k].x = t.x; q[k].y = t.y; }
                else if (p0 >= 2 && p0 - 2 < len) q[k].x = __float_as_uint(src[p0 - 2]);
                if (p0 + 1 < len) { const uint2 t = *(const uint2*)(src + p0); q[k].z = t.x; q[k].w = t.y; }
                else if (p0 < len) q[k].z = __float_as_uint(src[p0]);
            } else {
                if (p0 >= 2 && p0 - 2 < len) q[k].x = __float_as_uint(src[p0 - 2]);
                if (p0 >= 2 && p0 - 1 < len) q[k].y = __float_as_uint(src[p0 - 1]);
                if (p0 < len) q[k].z = __float_as_uint(src[p0]);
                if (p0 + 1 < len) q[k].w = __float_as_uint(src[p0 + 1]);
            }
            if (u == 0) { q[k].x = seq; q[k].y = hdr1; }
        }
        #pragma unroll
        for (int k = 0; k < PK_UNITS; ++k) {
            const u32 u = u0 + k * WAVE + lane;
            if (u < units) st_stream4(dst + u, q[k]);
        }
    }
}

// Sender, a range of sequence numbers of one worker: packet first_seq + i -> slot slot_map[i] (or
// slot_base + i).  The bucket boundaries are searched in LDS when the table fits (TABLE_IN_LDS).
template <bool TABLE_IN_LDS>
__global__ __launch_bounds__(256) void packetize_kernel(Geo g, u32 w, u32 round, const float* __restrict__ grad,
                                                        u64 elem_base, u32 first_seq, u32 n, const u32* __restrict__ slot_map,
                                                        u64 slot_base, u64 n_slots, uint8_t* __restrict__ packets,
                                                        uint16_t* __restrict__ src_worker, u64* __restrict__ counters) {
    extern __shared__ u32 fs_lds[];
    const u32* fs = g.first_seq;
    if (TABLE_IN_LDS) {
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) fs_lds[i] = g.first_seq[i];
        __syncthreads();
        fs = fs_lds;
    }
    u32 lane = lane_id();
    u32 wave = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    u32 n_waves = gridDim.x * blockDim.x / WAVE;
    for (u32 i = wave; i < n; i += n_waves) {
        u32 seq = first_seq + i;
        u64 slot = slot_map ? (u64)slot_map[i] : slot_base + i;
        if (slot >= n_slots) {
            if (lane == 0) atomicAdd(&counters[C_PKT_BAD], 1ull);
            continue;
        }
        u32 b = find_bucket(fs, g.B, seq);
        const u64 start = (u64)(seq - fs[b]) * g.P;
        const u64 left = g.b_cnt[b] - start;
        const u64 elem = g.b_off[b] + start;
        const u32 len = left < g.P ? (u32)left : g.P;
        write_packet(grad + (elem - elem_base), len, seq, round, g.units, (uint4*)(packets + slot * g.stride), lane);
        if (lane == 0) src_worker[slot] = (uint16_t)w;
    }
}

struct GradPtrs { const float* p[DBLP_MAX_WORKERS]; };

// One wave per list entry (w << 32 | seq): worker w's packet seq -> slot slot_base + i.
template <bool TABLE_IN_LDS>
__global__ __launch_bounds__(256) void packetize_list_kernel(Geo g, GradPtrs grads, u32 round, const u64* __restrict__ list,
                                                             u64 n, u64 slot_base, uint8_t* __restrict__ packets,
                                                             uint16_t* __restrict__ src_worker, u64* __restrict__ counters) {
    extern __shared__ u32 fs_lds[];
    const u32* fs = g.first_seq;
    if (TABLE_IN_LDS) {
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) fs_lds[i] = g.first_seq[i];
        __syncthreads();
        fs = fs_lds;
    }
    const u32 lane = lane_id();
    const u64 wave = ((u64)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const u64 n_waves = (u64)gridDim.x * blockDim.x / WAVE;
    for (u64 i = wave; i < n; i += n_waves) {
        const u64 e = list[i];
        const u32 w = (u32)(e >> 32), seq = (u32)e;
        if (w >= g.W || seq >= g.n_pkts) {
            if (lane == 0) atomicAdd(&counters[C_PKT_BAD], 1ull);
            continue;
        }
        const u32 b = find_bucket(fs, g.B, seq);
        const u64 start = (u64)(seq - fs[b]) * g.P;
        const u64 left = g.b_cnt[b] - start;
        const u64 elem = g.b_off[b] + start;
        const u32 len = left < g.P ? (u32)left : g.P;
        write_packet(grads.p[w] + elem, len, seq, round, g.units, (uint4*)(packets + (slot_base + i) * g.stride), lane);
        if (lane == 0) src_worker[slot_base + i] = (uint16_t)w;
    }
}

// ------------------------------------------------------------------------------------------
// receiver step 1: index the arrivals
// ------------------------------------------------------------------------------------------
// Grid-stride over arrivals.  Per-thread tallies are reduced per wave (DPP) and per block
// (LDS) and written to the block's row of block_tallies; fold_index_tallies adds the rows up.
// No global atomics on shared counters: atomics of many waves (or even of a few thousand
// blocks) on one address serialise in L2 at about 12 ns each.
#ifndef IDX_UNROLL
#define IDX_UNROLL 1     // arrivals in flight per thread of the index kernel
#endif
//
// TABLE_IN_LDS: the block first copies the bucket boundaries (first_seq, B + 1 words of dynamic
// shared memory) into LDS, so the ten dependent steps of the bucket search stay inside the CU.
// FROM_QUEUE: arrival k is the descriptor queue[k] = slot | worker << 32 (one coalesced 8-byte
// load) instead of order[k], mask bit[slot] and src_worker[slot]; the latter two are random
// accesses, and src_worker[slot] alone costs half as much as the header line it sits beside.
template <bool TABLE_IN_LDS, bool FROM_QUEUE>
__global__ __launch_bounds__(256) void index_arrivals(Geo g, const uint8_t* __restrict__ packets,
                                                      const uint16_t* __restrict__ src_worker, u64 n_slots,
                                                      const u64* __restrict__ mask, const u32* __restrict__ order,
                                                      const u64* __restrict__ queue,
                                                      u64 n_arrivals, u32 cur_round, u64* __restrict__ pending,
                                                      u32* __restrict__ block_tallies) {
    __shared__ u32 sh[4][5];    // per wave: stale, invalid, candidates, lowest seq, highest seq + 1
    extern __shared__ u32 fs_lds[];
    const u32* fs = g.first_seq;
    if (TABLE_IN_LDS) {
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) fs_lds[i] = g.first_seq[i];
        __syncthreads();
        fs = fs_lds;
    }
    u32 n_stale = 0, n_inv = 0, n_cand = 0;
    u32 seq_lo = 0xFFFFFFFFu, seq_hi = 0;
    const u64 stride = (u64)gridDim.x * blockDim.x;
    // IDX_UNROLL arrivals per thread and trip: the loads of one stage (order, then mask word,
    // header and worker) are issued for all of them before the first is used.
    for (u64 k0 = (u64)blockIdx.x * blockDim.x + threadIdx.x; k0 < n_arrivals; k0 += IDX_UNROLL * stride) {
        u64 slot[IDX_UNROLL];
        bool live[IDX_UNROLL];
        uint2 hdr[IDX_UNROLL];
        u32 w[IDX_UNROLL];
#pragma unroll
        for (int j = 0; j < IDX_UNROLL; ++j) {
            const u64 k = k0 + j * stride;
            live[j] = k < n_arrivals;
            if (FROM_QUEUE) {
                const u64 e = live[j] ? queue[k] : 0;
                slot[j] = e & 0xFFFFFFFFull;
                w[j] = (u32)(e >> 32);      // bits 48..63 must be zero: w >= W below catches them
            } else {
                slot[j] = live[j] ? (order ? (u64)order[k] : k) : 0;
            }
        }
#pragma unroll
        for (int j = 0; j < IDX_UNROLL; ++j) {
            if (live[j] && slot[j] >= n_slots) { ++n_inv; live[j] = false; }
            // lost packets are never looked at
            if (!FROM_QUEUE && live[j] && mask && !((mask[slot[j] >> 6] >> (slot[j] & 63)) & 1ull)) live[j] = false;
        }
#pragma unroll
        for (int j = 0; j < IDX_UNROLL; ++j) {
            if (live[j]) {
                hdr[j] = *(const uint2*)(packets + slot[j] * g.stride);
                if (!FROM_QUEUE) w[j] = src_worker[slot[j]];
            }
        }
#pragma unroll
        for (int j = 0; j < IDX_UNROLL; ++j) {
            if (!live[j]) continue;
            const u64 k = k0 + j * stride;
            const u32 seq = hdr[j].x, round = hdr[j].y & 0xFFFFu, len = hdr[j].y >> 16;
            if (round != cur_round) { ++n_stale; continue; }
            if (w[j] >= g.W || seq >= g.n_pkts) { ++n_inv; continue; }
            const u32 b = find_bucket(fs, g.B, seq);
            u32 want = g.P;         // every packet of a bucket but its last one is full
            if (seq + 1 == fs[b + 1]) { u64 elem; packet_span(g, seq, b, &elem, &want); }
            if (len != want) { ++n_inv; continue; }
            ++n_cand;
            atomicMin(&pending[(u64)w[j] * g.n_pkts + seq], (k << 32) | slot[j]);
            seq_lo = seq < seq_lo ? seq : seq_lo;
            seq_hi = seq + 1 > seq_hi ? seq + 1 : seq_hi;
        }
    }
    // loops above have lane-dependent trip counts; all 64 lanes are back here
    n_stale = wave_reduce<OpAdd>(n_stale); n_inv = wave_reduce<OpAdd>(n_inv);
    n_cand = wave_reduce<OpAdd>(n_cand);
    seq_lo = wave_reduce<OpMin>(seq_lo); seq_hi = wave_reduce<OpMax>(seq_hi);
    const u32 wave = threadIdx.x / WAVE;
    if (lane_id() == 0) {
        sh[wave][0] = n_stale; sh[wave][1] = n_inv; sh[wave][2] = n_cand;
        sh[wave][3] = seq_lo; sh[wave][4] = seq_hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 t[3] = {0, 0, 0}, lo = 0xFFFFFFFFu, hi = 0;
        for (int i = 0; i < 4; ++i) {
            for (int j = 0; j < 3; ++j) t[j] += sh[i][j];
            lo = sh[i][3] < lo ? sh[i][3] : lo;
            hi = sh[i][4] > hi ? sh[i][4] : hi;
        }
        u32* row = block_tallies + (u64)blockIdx.x * 5;
        row[0] = t[0]; row[1] = t[1]; row[2] = t[2]; row[3] = lo; row[4] = hi;
    }
}

// What the gather kernels need to know about the batch: the touched sequence range and the number
// of candidates.  Every block of a gather launch adds up the index launch's per-block tallies
// itself (n_rows rows of 5 words, read from L2), which saves a launch between the two passes; the
// block that `owner` names also adds the totals to the round's counters (one block of one launch
// per batch).  All threads of the block must call this; sh holds 5 words per wave.
struct BatchInfo { u64 lo, hi, cand; };
__device__ __forceinline__ BatchInfo fold_index_tallies(const u32* __restrict__ block_tallies, u32 n_rows, u64* __restrict__ counters,
                                                        bool owner, u32* sh) {
    u32 t0 = 0, t1 = 0, t2 = 0, lo = 0xFFFFFFFFu, hi = 0;
    for (u32 b = threadIdx.x; b < n_rows; b += blockDim.x) {
        const u32* row = block_tallies + (u64)b * 5;
        t0 += row[0]; t1 += row[1]; t2 += row[2];
        lo = row[3] < lo ? row[3] : lo;
        hi = row[4] > hi ? row[4] : hi;
    }
    t0 = wave_reduce<OpAdd>(t0); t1 = wave_reduce<OpAdd>(t1); t2 = wave_reduce<OpAdd>(t2);
    lo = wave_reduce<OpMin>(lo); hi = wave_reduce<OpMax>(hi);
    const u32 wave = threadIdx.x / WAVE, n_waves = blockDim.x / WAVE;
    if (lane_id() == 0) { sh[wave * 5 + 0] = t0; sh[wave * 5 + 1] = t1; sh[wave * 5 + 2] = t2; sh[wave * 5 + 3] = lo; sh[wave * 5 + 4] = hi; }
    __syncthreads();
    u64 s0 = 0, s1 = 0, s2 = 0;
    u32 l = 0xFFFFFFFFu, h = 0;
    for (u32 i = 0; i < n_waves; ++i) {
        s0 += sh[i * 5 + 0]; s1 += sh[i * 5 + 1]; s2 += sh[i * 5 + 2];
        l = sh[i * 5 + 3] < l ? sh[i * 5 + 3] : l;
        h = sh[i * 5 + 4] > h ? sh[i * 5 + 4] : h;
    }
    __syncthreads();                                // sh may be reused by the caller
    if (owner && threadIdx.x == 0) {
        counters[C_STALE] += s0;
        counters[C_INVALID] += s1;
        counters[C_CANDIDATES] += s2;
    }
    BatchInfo bi;
    bi.cand = s2; bi.lo = s2 ? (u64)l : NONE64; bi.hi = s2 ? (u64)h : 0;
    return bi;
}

// ------------------------------------------------------------------------------------------
// receiver step 2: gather payloads per output packet and accumulate
// ------------------------------------------------------------------------------------------
#ifndef GROUP
#define GROUP 8             // payload loads kept in flight per lane
#endif
#ifndef GA_WAVES
#define GA_WAVES 8          // waves per block
#endif
#ifndef GA_BLOCKS_PER_CU
#define GA_BLOCKS_PER_CU 4
#endif
#define SUB 16              // consecutive sequence numbers a block handles at a time (divides 64)
#define NONE32 0xFFFFFFFFu

// A batch is sparse when it holds fewer than one packet per SPARSE_DIV (worker, seq) pairs of the
// sequence range it touches (retransmission batches).  Sparse batches take the direct kernel
// (independent waves, no staging pipeline to fill per group), dense ones the staged kernel; both
// are launched and the one whose regime it is not returns at once.
#define SPARSE_DIV 8
__device__ __forceinline__ bool batch_is_sparse(const BatchInfo& bi, u32 W) {
    return bi.cand * SPARSE_DIV < (bi.hi - bi.lo) * W;
}

// Sum the payload unit `u` (16 bytes at offset 16u of each packet) over the workers in `sub`
// (bit w set = worker w delivered this packet in this batch), ascending worker order.
// slot32 holds worker w's slot in lane w.
__device__ __forceinline__ float4 sum_unit(const uint8_t* __restrict__ packets, u32 stride, u32 u, bool active,
                                           u64 sub, u32 slot32) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    while (sub) {
        float4 v[GROUP];
        #pragma unroll
        for (int j = 0; j < GROUP; ++j) {
            v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (sub) {
                const u32 w = (u32)__builtin_ctzll(sub);
                sub &= sub - 1;
                const u32 slot = (u32)__builtin_amdgcn_readlane((int)slot32, (int)w);
                if (active) v[j] = *(const float4*)(packets + (u64)slot * stride + 16ull * u);
            }
        }
        #pragma unroll
        for (int j = 0; j < GROUP; ++j) { a.x += v[j].x; a.y += v[j].y; a.z += v[j].z; a.w += v[j].w; }
    }
    return a;
}

// Epilogue of one 16-byte unit of a summed packet: scale, fold in the old accumulator value when the
// span was written before (rmw is uniform over the wave), and keep the running sum of squares of
// what is stored.  Written without per-element branches: positions outside the payload (the two
// header words of unit 0, the tail beyond len) are carried along and masked out of the sum of
// squares only; the writer never reads them.  o points at the accumulator element that packet
// float position 4u corresponds to (only dereferenced where the position is payload).
__device__ __forceinline__ float4 finish_unit(float4 a, float inv_w, bool rmw, const float* o, u32 u, u32 len, double& sq) {
    float qv[4] = {a.x * inv_w, a.y * inv_w, a.z * inv_w, a.w * inv_w};
    bool ok[4];
    #pragma unroll
    for (int c = 0; c < 4; ++c) { const u32 i4 = 4 * u + c; ok[c] = i4 >= 2 && i4 - 2 < len; }
    if (rmw) {                                    // result = old value + this batch's sum
        float ov[4];
        #pragma unroll
        for (int c = 0; c < 4; ++c) ov[c] = ok[c] ? o[c] : 0.f;      // four loads in flight, one wait
        #pragma unroll
        for (int c = 0; c < 4; ++c) {
            sq -= (double)ov[c] * (double)ov[c];
            qv[c] = ov[c] + qv[c];
        }
    }
    #pragma unroll
    for (int c = 0; c < 4; ++c) {
        const double d = (double)(ok[c] ? qv[c] : 0.f);
        sq += d * d;
    }
    return make_float4(qv[0], qv[1], qv[2], qv[3]);
}

// One block per group of SUB consecutive sequence numbers, grid-stride over the groups the
// batch touched.
//   phase A  64 lanes = 4 workers x 16 packets per load of the arrival index: ballot -> new
//            bitmap bits (one atomicOr per worker and group), slots staged in LDS, index
//            entries reset; the 16 packets' element spans are computed by 16 lanes in parallel
//   phase B  the waves split the 16 packets: per packet, 16-byte payload loads from every
//            worker that delivered it, summed in registers in worker order, one write of the span
//
// The accumulator may exist in two copies (acc0, acc1; acc1 == acc0 when there is one): a span
// written for the first time in this round goes to copy `pick` and home[seq] records it; a span
// that earlier batches wrote is read and rewritten where home[seq] says it lives.
__global__ __launch_bounds__(GA_WAVES * WAVE) __attribute__((amdgpu_waves_per_eu(8))) void gather_accumulate(Geo g, const uint8_t* __restrict__ packets,
                                                                    u64* __restrict__ pending, u64* __restrict__ bitmap,
                                                                    float* acc0, float* acc1,
                                                                    uint8_t* __restrict__ home, u32 pick,
                                                                    const u32* __restrict__ block_tallies, u32 n_tally_rows,
                                                                    u64* __restrict__ counters, int tally_owner,
                                                                    u64* __restrict__ accept_rows, double* __restrict__ sumsq_rows,
                                                                    float inv_w, int only_if_sparse, u32 table_in_lds) {
    extern __shared__ u32 sh_slot[];           // [W rounded up to 4][SUB], then the bucket boundaries when table_in_lds
    __shared__ u64 sh_elem[SUB];
    __shared__ u32 sh_len[SUB], sh_home[SUB];
    __shared__ u32 sh_new[GA_WAVES], sh_old[GA_WAVES];
    __shared__ double sh_sq[GA_WAVES];
    __shared__ u32 sh_tally[GA_WAVES * 5];
    __shared__ u32 sh_mask[2][2];
    const BatchInfo bi = fold_index_tallies(block_tallies, n_tally_rows, counters, tally_owner && blockIdx.x == 0, sh_tally);
    const u64 lo = bi.lo, hi = bi.hi;
    if (hi == 0) return;                                    // no candidate in this batch
    if (only_if_sparse && !batch_is_sparse(bi, g.W)) return;
    const u32 lane = lane_id();
    const u32 wave = threadIdx.x / WAVE;
    const u32 W = g.W;
    const u32 s_lane = lane & (SUB - 1), w_sub = lane / SUB;   // packet and worker-within-load of this lane
    const u32 grp_lo = (u32)(lo / SUB), grp_end = (u32)((hi + SUB - 1) / SUB);
    u32 accepted = 0;
    double sq = 0.0;      // change of the sum of squares of the stored values caused by this lane's writes
    // bucket boundaries in LDS when the host made room for them: the span lookup is a chain of
    // dependent loads that every packet of a small batch would wait for
    const u32* fs = g.first_seq;
    if (table_in_lds) {
        u32* tab = sh_slot + (W + 3) / 4 * 4 * SUB;
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) tab[i] = g.first_seq[i];
        fs = tab;
        __syncthreads();
    }

    // Every block walks the groups of the touched range grid-stride.  When most groups hold no
    // arrival at all (a small retransmission batch spread over the round: fewer than one candidate
    // per four groups), the block first looks through the arrival index of up to 64 of its groups at
    // a time, one wave per group and all loads in flight together, and then walks only the groups
    // that hold an entry.
    const bool skim = bi.cand * (4 * SUB) < hi - lo;
    u32 grp_next = grp_lo + blockIdx.x;
    u32 tile_base = 0, tile_no = 0;
    u64 tile_mask = 0;
    for (;;) {
        u32 grp;
        if (skim) {      // block-uniform control flow throughout: the barriers below are reached by all
            while (tile_mask == 0 && grp_next < grp_end) {
                u32* mask = sh_mask[tile_no & 1];      // two buffers: the next look clears one while this one is read
                ++tile_no;
                tile_base = grp_next;                  // group k of the tile is tile_base + k * gridDim.x
                const u32 left = (grp_end - grp_next + gridDim.x - 1) / gridDim.x;
                const u32 n_g = left < 64 ? left : 64;
                grp_next = left <= 64 ? grp_end : grp_next + 64 * gridDim.x;
                if (threadIdx.x < 2) mask[threadIdx.x] = 0;
                __syncthreads();
                u32 m0 = 0, m1 = 0;
                for (u32 k = wave; k < n_g; k += GA_WAVES) {
                    const u32 seq_k = (tile_base + k * gridDim.x) * SUB + s_lane;
                    bool any = false;
                    #pragma unroll 4
                    for (u32 w0 = 0; w0 < W; w0 += 4) {
                        const u32 w = w0 + w_sub;
                        if (w < W && seq_k < g.n_pkts) any |= pending[(u64)w * g.n_pkts + seq_k] != NONE64;
                    }
                    if (__ballot(any)) { if (k < 32) m0 |= 1u << k; else m1 |= 1u << (k - 32); }
                }
                if (lane == 0 && (m0 | m1)) { atomicOr(&mask[0], m0); atomicOr(&mask[1], m1); }
                __syncthreads();
                tile_mask = (u64)mask[0] | ((u64)mask[1] << 32);
            }
            if (tile_mask == 0) break;
            grp = tile_base + (u32)__builtin_ctzll(tile_mask) * gridDim.x;
            tile_mask &= tile_mask - 1;
        } else {
            grp = grp_next;
            if (grp >= grp_end) break;
            grp_next += gridDim.x;
        }
        const u32 seq0 = grp * SUB;
        const u32 seq_l = seq0 + s_lane;
        const u32 word = seq0 >> 6, shift = seq0 & 63;
        u32 new_or = 0, old_or = 0;
        for (u32 w0 = wave * 4; w0 < W; w0 += GA_WAVES * 4) {
            const u32 w = w0 + w_sub;
            const bool valid = w < W && seq_l < g.n_pkts;
            u64 p = NONE64, bits = 0;
            if (valid) {
                p = pending[(u64)w * g.n_pkts + seq_l];
                bits = bitmap[(u64)w * g.words_pw + word];
            }
            const bool has = p != NONE64;
            const bool had = valid && ((bits >> (shift + s_lane)) & 1ull);   // delivered by an earlier batch
            const bool fresh = has && !had;                                  // a copy of a delivered packet is dropped
            const u64 nb = __ballot(fresh);
            sh_slot[w * SUB + s_lane] = fresh ? (u32)p : NONE32;
            if (has) pending[(u64)w * g.n_pkts + seq_l] = NONE64;   // leave the index empty for the next batch
            const u32 mine = (u32)(nb >> (w_sub * SUB)) & 0xFFFFu;  // this lane's worker: new bits of the group
            if (s_lane == 0 && mine) atomicOr(&bitmap[(u64)w * g.words_pw + word], (u64)mine << shift);
            const u64 ob = __ballot(had);
            #pragma unroll
            for (int j = 0; j < 4; ++j) {
                new_or |= (u32)(nb >> (j * SUB)) & 0xFFFFu;
                old_or |= (u32)(ob >> (j * SUB)) & 0xFFFFu;
            }
            accepted += (u32)__popcll(nb);
        }
        if (wave == GA_WAVES - 1 && lane < SUB && seq_l < g.n_pkts) {
            const u32 hm = home[seq_l];                      // only meaningful (and only used) for spans written before
            const u32 b = find_bucket(fs, g.B, seq_l);
            const u64 start = (u64)(seq_l - fs[b]) * g.P;    // packet_span with the boundary from the table at hand
            const u64 left = g.b_cnt[b] - start;
            sh_elem[lane] = g.b_off[b] + start; sh_len[lane] = left < g.P ? (u32)left : g.P; sh_home[lane] = hm;
        }
        if (lane == 0) { sh_new[wave] = new_or; sh_old[wave] = old_or; }
        __syncthreads();
        u32 new_any = 0, old_any = 0;
        #pragma unroll
        for (int i = 0; i < GA_WAVES; ++i) { new_any |= sh_new[i]; old_any |= sh_old[i]; }

        for (u32 t = wave; t < SUB; t += GA_WAVES) {
            if (!((new_any >> t) & 1u)) continue;
            const bool rmw = (old_any >> t) & 1u;            // span already holds earlier arrivals
            const u64 elem = sh_elem[t];
            const u32 len = sh_len[t];
            const u32 slot32 = lane < W ? sh_slot[lane * SUB + t] : NONE32;
            const u64 sub = __ballot(slot32 != NONE32);
            const u32 units = (len + 2 + 3) >> 2;            // 16-byte units holding header + payload
            u32 h = pick;
            if (rmw) h = sh_home[t];
            else if (lane == 0) home[seq0 + t] = (uint8_t)pick;
            float* dst0 = (h ? acc1 : acc0) + elem - 2;      // float position i of the packet -> dst0[i]
            for (u32 u0 = 0; u0 < units; u0 += WAVE) {
                const u32 u = u0 + lane;
                const bool active = u < units;
                const float4 a = sum_unit(packets, g.stride, u, active, sub, slot32);
                if (active) {
                    float* d = dst0 + 4 * u;                 // packet float position 4u+c -> d[c]
                    const float4 r = finish_unit(a, inv_w, rmw, d, u, len, sq);
                    const float q[4] = {r.x, r.y, r.z, r.w};
                    #pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const u32 i4 = 4 * u + c;
                        if (i4 >= 2 && i4 - 2 < len) d[c] = q[c];
                    }
                }
            }
        }
        __syncthreads();                                     // LDS is reused by the next group
    }
    // accepted packets and sum-of-squares change of this block: plain adds to the block's own rows
    // (no shared atomics; kernels on the stream run one after the other)
    sq = wave_sum_f64(sq);
    if (lane == 0) { sh_new[wave] = accepted; sh_sq[wave] = sq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 total = 0;
        double t = 0.0;
        for (int i = 0; i < GA_WAVES; ++i) { total += sh_new[i]; t += sh_sq[i]; }
        if (total) { accept_rows[blockIdx.x] += total; sumsq_rows[blockIdx.x] += t; }
    }
}

// Staged variant of the gather (used whenever two groups of packets fit in LDS).
// Mixing the accumulator stores into the waves that stream the payloads costs far more than the
// stores' bytes (a payload-only loop sustains 6.2 TB/s on this chip, the same loop with its
// 3 % of stores 4.9 TB/s).  Here up to GS_READERS waves only load and add, and hand each summed
// packet to LDS; one extra writer wave drains the previous group from LDS to the accumulator
// while the readers work on the next one (double-buffered).  Because the writer reads LDS at
// arbitrary float offsets, its global accesses are 16-byte aligned float4s whatever the
// alignment of the packet's element span.
#ifndef GS_READERS
#define GS_READERS 8
#endif
#ifndef GS_READERS_SHORT
#define GS_READERS_SHORT 4            // reader waves and blocks per CU for packets of up to 2 KB
#endif
#ifndef GS_MAX_PER_CU_SHORT
#define GS_MAX_PER_CU_SHORT 3
#endif
#ifndef GS_LDS_BUDGET
#define GS_LDS_BUDGET (48u * 1024u)   // bytes for the two packet buffers
#endif
#ifndef GS_WRITER_PREPARES_MAX_W
#define GS_WRITER_PREPARES_MAX_W 16   // up to this many workers the writer wave also prepares the next group (see the kernel)
#endif
#ifndef GS_MAX_PER_CU
#define GS_MAX_PER_CU 2               // blocks per CU for packets longer than 2 KB (more waves in flight
#endif                                // only spread the DRAM accesses over more open rows); see apply_batch

// Sum of one whole packet over the workers in `sub`: lane l holds 16-byte units l, l+64, ...
// (NP of them).  All NP loads of one worker's packet are issued together, so a packet's
// cache lines are requested back to back (a line shared by two 1 KB passes is fetched once),
// and 8/NP workers (at least 2) are in flight at a time.  Same addition order as sum_unit.
template <int NP>
__device__ __forceinline__ void sum_packet(const uint8_t* __restrict__ packets, u32 stride, u32 lane, u32 units,
                                           u64 sub, u32 slot32, float4 (&a)[NP]) {
    constexpr int G = NP <= 2 ? 8 / NP : 2;
    #pragma unroll
    for (int q = 0; q < NP; ++q) a[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    while (sub) {
        float4 v[G][NP];
        #pragma unroll
        for (int j = 0; j < G; ++j) {
            #pragma unroll
            for (int q = 0; q < NP; ++q) v[j][q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (sub) {
                const u32 w = (u32)__builtin_ctzll(sub);
                sub &= sub - 1;
                const u32 slot = (u32)__builtin_amdgcn_readlane((int)slot32, (int)w);
                const uint8_t* base = packets + (u64)slot * stride + 16ull * lane;
                #pragma unroll
                for (int q = 0; q < NP; ++q)
                    if (q * WAVE + lane < units) v[j][q] = ld_stream4(base + 1024ull * q);
            }
        }
        #pragma unroll
        for (int j = 0; j < G; ++j) {
            #pragma unroll
            for (int q = 0; q < NP; ++q) { a[q].x += v[j][q].x; a[q].y += v[j][q].y; a[q].z += v[j][q].z; a[q].w += v[j][q].w; }
        }
    }
}

// NP = 16-byte-unit passes per packet handled in one go (1..5), 0 = generic one pass at a time.
template <int NP>
__global__ __launch_bounds__((GS_READERS + 1) * WAVE) __attribute__((amdgpu_waves_per_eu(NP == 0 ? 7 : NP <= 3 ? 6 : NP == 4 ? 5 : 4))) void gather_accumulate_staged(
    Geo g, const uint8_t* __restrict__ packets, u64* __restrict__ pending, u64* __restrict__ bitmap,
    float* acc0, float* acc1, uint8_t* __restrict__ home, u32 pick,
    const u32* __restrict__ block_tallies, u32 n_tally_rows, u64* __restrict__ counters, int whole_batch,
    u64* __restrict__ accept_rows, double* __restrict__ sumsq_rows, float inv_w,
    u32 sub, u32 sub_log2, u32 n_pass, u32 table_in_lds, u32 writer_prepares) {
    extern __shared__ float4 sh_dyn[];              // buf[2][sub * stride / 16] float4, slots, bucket table
    __shared__ double sh_sq[GS_READERS];
    __shared__ u64 sh_elem[2][SUB];
    __shared__ u32 sh_len[2][SUB];
    __shared__ u32 sh_home[2][SUB];                 // accumulator copy each packet of the group goes to
    __shared__ u32 sh_new[2][GS_READERS], sh_old[2][GS_READERS];   // per preparing wave: packets of the group that arrived in this batch / in an earlier one
    __shared__ u32 sh_accepted[GS_READERS + 1];
    __shared__ u32 sh_tally[(GS_READERS + 1) * 5];
    // this launch is the first of the batch's gather launches: its block 0 books the index pass's tallies
    const BatchInfo bi = fold_index_tallies(block_tallies, n_tally_rows, counters, blockIdx.x == 0, sh_tally);
    const u64 lo = bi.lo, hi = bi.hi;
    if (hi == 0) return;                            // no candidate in this batch (uniform over the grid)
    if (!whole_batch && batch_is_sparse(bi, g.W)) return;     // left to the direct kernel
    const u32 lane = lane_id();
    const u32 wave = threadIdx.x / WAVE;
    const u32 n_readers = blockDim.x / WAVE - 1;      // the last wave of the block is the writer
    const u32 W = g.W;
    const u32 upp = g.stride >> 4;                  // float4 units per packet
    float4* buf0 = sh_dyn;
    float4* buf1 = sh_dyn + sub * upp;
    const u32 wpl = WAVE >> sub_log2;               // workers per 64-lane load of the index
    const u32 slot_words = (W + wpl - 1) / wpl * wpl * sub;
    u32* sh_slot0 = (u32*)(sh_dyn + 2 * sub * upp); // slot tables [W rounded up to a multiple of 64/sub][sub]:
    u32* sh_slot1 = writer_prepares ? sh_slot0 + slot_words : sh_slot0;   // two when the next group is prepared during this one's gather
    // bucket boundaries in LDS when the host made room for them (the span lookup of phase A is ten
    // dependent loads)
    const u32* fs = g.first_seq;
    if (table_in_lds) {
        u32* tab = sh_slot1 + slot_words;
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) tab[i] = g.first_seq[i];
        fs = tab;
        __syncthreads();
    }
    const u32 s_lane = lane & (sub - 1), w_sub = lane >> sub_log2;
    const u32 submask = (1u << sub) - 1;
    const u32 grp0 = (u32)(lo >> sub_log2) + blockIdx.x;
    const u32 grp_end = (u32)((hi + sub - 1) >> sub_log2);
    const u32 n_it = grp0 < grp_end ? (grp_end - grp0 + gridDim.x - 1) / gridDim.x : 0;
    u32 accepted = 0;
    double sq = 0.0;      // change of the sum of squares of the stored values caused by this lane's packets

    // ---- phase A of group `ia`: arrival index -> bitmap bits, slots, spans.  The calling wave takes
    // the index loads w_first, w_first + w_step, ... (wpl workers each) and leaves the group's
    // flags as seen by it in entry `part`; one of the callers also computes the spans.
    const u32 n_parts = writer_prepares ? 1u : n_readers;
    auto phase_a = [&](u32 ia, u32 w_first, u32 w_step, bool spans, u32 part) {
        const u32 nb_buf = ia & 1;
        u32* slot_tab = nb_buf ? sh_slot1 : sh_slot0;
        const u32 seq0 = (grp0 + ia * gridDim.x) << sub_log2;
        const u32 seq_l = seq0 + s_lane;
        const u32 word = seq0 >> 6, shift = seq0 & 63;
        u32 new_or = 0, old_or = 0;
        for (u32 w0 = w_first; w0 < W; w0 += w_step) {
            const u32 w = w0 + w_sub;
            const bool valid = w < W && seq_l < g.n_pkts;
            u64 p = NONE64, bits = 0;
            if (valid) {
                p = pending[(u64)w * g.n_pkts + seq_l];
                bits = bitmap[(u64)w * g.words_pw + word];
            }
            const bool has = p != NONE64;
            const bool had = valid && ((bits >> (shift + s_lane)) & 1ull);   // delivered by an earlier batch
            const bool fresh = has && !had;                     // a copy of a delivered packet is dropped
            const u64 nb = __ballot(fresh);
            slot_tab[w * sub + s_lane] = fresh ? (u32)p : NONE32;
            if (has) pending[(u64)w * g.n_pkts + seq_l] = NONE64;   // leave the index empty
            const u32 mine = (u32)(nb >> (w_sub * sub)) & submask;
            if (s_lane == 0 && mine) atomicOr(&bitmap[(u64)w * g.words_pw + word], (u64)mine << shift);
            const u64 ob = __ballot(had);
            for (u32 j = 0; j < wpl; ++j) {
                new_or |= (u32)(nb >> (j * sub)) & submask;
                old_or |= (u32)(ob >> (j * sub)) & submask;
            }
            accepted += (u32)__popcll(nb);
        }
        if (spans && lane < sub && seq_l < g.n_pkts) {
            const u32 b = find_bucket(fs, g.B, seq_l);
            const u64 start = (u64)(seq_l - fs[b]) * g.P;
            const u64 left = g.b_cnt[b] - start;
            sh_elem[nb_buf][lane] = g.b_off[b] + start;
            sh_len[nb_buf][lane] = left < g.P ? (u32)left : g.P;
        }
        if (lane == 0) { sh_new[nb_buf][part] = new_or; sh_old[nb_buf][part] = old_or; }
    };

    // Turn `it`, two schedules (the host picks by the number of workers; every LDS table exists
    // twice, by turn parity):
    //   writer_prepares   the reader waves gather group it (phase B) while the writer wave drains
    //                     group it - 1 to the accumulator and then prepares group it + 1 (phase A):
    //                     the readers never wait for the arrival index; one barrier per turn
    //   otherwise         the reader waves share phase A of group it while the writer drains group
    //                     it - 1; barrier; phase B; barrier
    if (writer_prepares) {
        if (wave == n_readers && n_it > 0) phase_a(0, 0, wpl, true, 0);
        __syncthreads();
    }
    for (u32 it = 0; it <= n_it; ++it) {            // one extra turn so the writer drains the last group
        const u32 cur = it & 1;
        const u32 seq0 = (grp0 + it * gridDim.x) << sub_log2;
        if (wave < n_readers) {
            if (!writer_prepares && it < n_it) phase_a(it, wave * wpl, n_readers * wpl, wave == n_readers - 1, wave);
        } else {
            if (it > 0) {
            // ---- writer: drain group it-1 from LDS to the accumulator (plain aligned stores; a span
            // that earlier batches had written already has its old value folded in by the readers)
            const u32 prev = cur ^ 1;
            const float* src = (const float*)(prev ? buf1 : buf0);
            u32 nf = 0;
            for (u32 i = 0; i < n_parts; ++i) nf |= sh_new[prev][i];
            for (u32 t = 0; t < sub; ++t) {
                if (!((nf >> t) & 1u)) continue;
                const u64 elem = sh_elem[prev][t];
                const u32 len = sh_len[prev][t];
                const float* pk = src + t * (g.stride >> 2) + 2;   // payload float j at pk[j]
                float* acc = sh_home[prev][t] ? acc1 : acc0;
                const u64 c0 = elem >> 2, c1 = (elem + len - 1) >> 2;
                for (u64 c = c0 + lane; c <= c1; c += WAVE) {
                    const u64 e0 = c << 2;
                    float* d = acc + e0;
                    if (e0 >= elem && e0 + 4 <= elem + len) {
                        const u32 j = (u32)(e0 - elem);
                        *(float4*)d = make_float4(pk[j], pk[j + 1], pk[j + 2], pk[j + 3]);
                    } else {
                        #pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const u64 e = e0 + k;
                            if (e >= elem && e < elem + len) d[k] = pk[(u32)(e - elem)];
                        }
                    }
                }
            }
            }
            // writes the tables of parity (it + 1) & 1, which the drain above has just read
            if (writer_prepares && it + 1 < n_it) phase_a(it + 1, 0, wpl, true, 0);
        }
        if (!writer_prepares) __syncthreads();
        if (wave < n_readers && it < n_it) {
            // ---- phase B: payload gather, worker order, results to LDS
            u32 new_any = 0, old_any = 0;
            for (u32 i = 0; i < n_parts; ++i) { new_any |= sh_new[cur][i]; old_any |= sh_old[cur][i]; }
            const u32* sh_slot = cur ? sh_slot1 : sh_slot0;
            float4* dstbuf = cur ? buf1 : buf0;
            if (NP > 0) {
                for (u32 t = wave; t < sub; t += n_readers) {
                    if (!((new_any >> t) & 1u)) continue;
                    const u32 len = sh_len[cur][t];
                    const u32 units = (len + 2 + 3) >> 2;        // 16-byte units holding header + payload
                    const u32 slot32 = lane < W ? sh_slot[lane * sub + t] : NONE32;
                    const u64 subm = __ballot(slot32 != NONE32);
                    float4 a[NP > 0 ? NP : 1];
                    sum_packet<(NP > 0 ? NP : 1)>(packets, g.stride, lane, units, subm, slot32, a);
                    const bool rmw = (old_any >> t) & 1u;         // earlier batches already wrote this span
                    u32 h = pick;
                    if (rmw) h = home[seq0 + t];
                    else if (lane == 0) home[seq0 + t] = (uint8_t)pick;
                    if (lane == 0) sh_home[cur][t] = h;
                    const float* acc = h ? acc1 : acc0;
                    #pragma unroll
                    for (int q = 0; q < (NP > 0 ? NP : 1); ++q) {
                        const u32 u = q * WAVE + lane;
                        if (u >= units) continue;
                        const float* o = acc + sh_elem[cur][t] - 2 + 4 * u;       // packet float position 4u+c -> o[c]
                        dstbuf[t * upp + u] = finish_unit(a[q], inv_w, rmw, o, u, len, sq);
                    }
                }
            } else {
            const u32 items = n_pass << sub_log2;
            for (u32 i = wave; i < items; i += n_readers) {
                const u32 t = i & (sub - 1), pass = i >> sub_log2;
                if (!((new_any >> t) & 1u)) continue;
                const u32 len = sh_len[cur][t];
                const u32 units = (len + 2 + 3) >> 2;        // 16-byte units holding header + payload
                const u32 u = pass * WAVE + lane;
                if (pass * WAVE >= units) continue;
                const bool active = u < units;
                const u32 slot32 = lane < W ? sh_slot[lane * sub + t] : NONE32;
                const u64 subm = __ballot(slot32 != NONE32);
                float4 a = sum_unit(packets, g.stride, u, active, subm, slot32);
                const bool rmw = (old_any >> t) & 1u;
                u32 h = pick;                       // every pass of packet t derives and records the same value
                if (rmw) h = home[seq0 + t];
                else if (lane == 0) home[seq0 + t] = (uint8_t)pick;
                if (lane == 0) sh_home[cur][t] = h;
                if (active) {
                    const float* o = (h ? acc1 : acc0) + sh_elem[cur][t] - 2 + 4 * u;   // packet float position 4u+c -> o[c]
                    dstbuf[t * upp + u] = finish_unit(a, inv_w, rmw, o, u, len, sq);
                }
            }
            }
        }
        __syncthreads();
    }
    // accepted packets and sum-of-squares change of this block: plain adds to the block's own rows
    sq = wave_sum_f64(sq);
    if (lane == 0) {
        sh_accepted[wave] = accepted;               // counted by whichever waves ran phase A
        if (wave < n_readers) sh_sq[wave] = sq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 total = 0;
        double t = 0.0;
        for (u32 i = 0; i <= n_readers; ++i) total += sh_accepted[i];
        for (u32 i = 0; i < n_readers; ++i) t += sh_sq[i];
        if (total) { accept_rows[blockIdx.x] += total; sumsq_rows[blockIdx.x] += t; }
    }
}

// ------------------------------------------------------------------------------------------
// probe: per-(worker,bucket) loss count, prefix of list lengths, ordered list
// ------------------------------------------------------------------------------------------
// Bits of word index `wd` that belong to sequence range [s0, s1).
__device__ __forceinline__ u64 range_mask(u32 wd, u32 s0, u32 s1) {
    u64 m = NONE64;
    u64 base = (u64)wd * 64;
    if (base < s0) m &= NONE64 << (s0 - base);
    if (base + 64 > s1) m &= NONE64 >> (base + 64 - s1);
    return m;
}

__global__ __launch_bounds__(256) void loss_count(Geo g, const u64* __restrict__ bitmap, u32 bound_ppm,
                                                  u32* __restrict__ missing_out, u32* __restrict__ need) {
    const u32 lane = lane_id();
    const u32 wave = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const u32 n_waves = gridDim.x * blockDim.x / WAVE;
    const u32 pairs = g.W * g.B;
    for (u32 pr = wave; pr < pairs; pr += n_waves) {
        const u32 w = pr / g.B, b = pr - w * g.B;
        const u32 s0 = g.first_seq[b], s1 = g.first_seq[b + 1];
        const u32 wd0 = s0 >> 6, wd1 = (s1 - 1) >> 6;
        u32 cnt = 0;
        for (u32 wd = wd0 + lane; wd <= wd1; wd += WAVE)
            cnt += (u32)__popcll(bitmap[(u64)w * g.words_pw + wd] & range_mask(wd, s0, s1));
        const u32 got = wave_reduce<OpAdd>(cnt);
        if (lane == 0) {
            const u32 n_b = s1 - s0;
            const u32 miss = n_b - got;
            const u64 allowed = ((u64)bound_ppm * n_b) / 1000000ull;
            if (missing_out) missing_out[pr] = miss;
            need[pr] = (u64)miss > allowed ? miss : 0u;
        }
    }
}

// Exclusive prefix of need[0..n) into offs[0..n); total list length to *total (device) and to
// the host mailbox.  Single block of 1024 threads.
__global__ __launch_bounds__(1024) void scan_need(const u32* __restrict__ need, u32 n, u64* __restrict__ offs,
                                                  u64* __restrict__ mailbox) {
    __shared__ u64 part[1024];
    const u32 t = threadIdx.x;
    const u32 per = (n + 1023) / 1024;
    const u32 i0 = t * per, i1 = min(n, i0 + per);
    u64 s = 0;
    for (u32 i = i0; i < i1; ++i) s += need[i];
    part[t] = s;
    __syncthreads();
    for (u32 d = 1; d < 1024; d <<= 1) {
        u64 v = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    u64 run = part[t] - s;     // exclusive prefix of this thread's chunk
    for (u32 i = i0; i < i1; ++i) { offs[i] = run; run += need[i]; }
    if (t == 1023) mailbox[0] = part[1023];
}

__global__ __launch_bounds__(256) void emit_retx(Geo g, const u64* __restrict__ bitmap, const u32* __restrict__ need,
                                                 const u64* __restrict__ offs, u64* __restrict__ list, u64 capacity) {
    const u32 lane = lane_id();
    const u32 wave = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
    const u32 n_waves = gridDim.x * blockDim.x / WAVE;
    const u32 pairs = g.W * g.B;
    for (u32 pr = wave; pr < pairs; pr += n_waves) {
        if (need[pr] == 0) continue;
        const u32 w = pr / g.B, b = pr - w * g.B;
        const u32 s0 = g.first_seq[b], s1 = g.first_seq[b + 1];
        const u32 wd0 = s0 >> 6, wd1 = (s1 - 1) >> 6;
        u64 base = offs[pr];
        for (u32 c0 = wd0; c0 <= wd1; c0 += WAVE) {
            const u32 wd = c0 + lane;
            u64 m = 0;
            if (wd <= wd1) m = ~bitmap[(u64)w * g.words_pw + wd] & range_mask(wd, s0, s1);
            const u32 c = (u32)__popcll(m);
            const u32 incl = wave_scan_incl<OpAdd>(c);
            const u32 total = (u32)__builtin_amdgcn_readlane((int)incl, 63);
            u64 pos = base + (incl - c);
            while (m) {
                const u32 bit = (u32)__builtin_ctzll(m);
                m &= m - 1;
                if (pos < capacity) list[pos] = ((u64)w << 32) | ((u64)wd * 64 + bit);
                ++pos;
            }
            base += total;
        }
    }
}

// ------------------------------------------------------------------------------------------
// finalize (zero-fill + mean over all W) with fused partial sums of squares; norm reduction
// ------------------------------------------------------------------------------------------
#define FIN_TILE 8   // consecutive packets per wave step; divides 64 so a tile sits in one bitmap word

// x / P for x < FIN_TILE * P (fits a float exactly enough to be fixed up by one step).
__device__ __forceinline__ u32 div_small(u32 x, u32 P, float inv_p) {
    u32 t = (u32)((float)x * inv_p);
    if (t * P > x) --t;
    if ((t + 1) * P <= x) ++t;
    return t;
}

// Compensation pass (Alg. "DBLP_RECV" last statements, Alg. "Server" mean).  Per packet span:
//   some worker delivered it   out = src            (scale_mode 0: the gather already divided by W)
//                              out = src / W        (scale_mode 1: W is not a power of two)
//                              where src is the accumulator copy that home[seq] names;
//                              nothing at all when src and out are the same memory and there is
//                              no scaling (in-place form: only moved and missing spans are touched)
//   nobody delivered it        out = 0 exactly
// A tile of 8 packets inside one bucket is one contiguous element range: it is walked in
// 16-byte aligned chunks (float4 load, store); chunks that straddle a packet or the range's
// ends, and tiles that cross a bucket boundary, go element by element.
// home[seq] (padded to a multiple of 8 entries) names the copy that holds the packet's span; with
// move_home set (in-place form) the entries of moved spans are reset to copy 0.
// With scale_mode 1 the per-block sums of out^2 go to partials[blockIdx.x].  Otherwise the sum of
// squares is already known: the gather kernels kept it per block in sumsq_rows, and the one extra
// block of this launch (blockIdx.x == n_work_blocks) adds those rows up in a fixed order (fixed
// for given launch sizes of the round's gather kernels) and writes the total to the host mailbox.
template <bool TABLE_IN_LDS>
__global__ __launch_bounds__(256) void finalize_pass(Geo g, const u64* __restrict__ bitmap, const float* acc0,
                                                     const float* acc1, uint8_t* __restrict__ home,
                                                     float* out, int scale_mode, float wf, int move_home,
                                                     double* __restrict__ partials, u32 n_work_blocks,
                                                     const double* __restrict__ sumsq_rows, const u64* __restrict__ accept_rows,
                                                     u32 rows_staged, u32 rows_direct, u32 row_pitch,
                                                     u64* __restrict__ counters, u64* __restrict__ mailbox) {
    __shared__ double wsum[4];
    __shared__ u64 asum[4];
    extern __shared__ u32 fs_lds[];             // bucket boundaries (B + 1 words) when TABLE_IN_LDS
    const u32 lane = lane_id();
    const u32 wave_in_block = threadIdx.x / WAVE;
    if (blockIdx.x >= n_work_blocks) {
        // the extra block: fixed-order sum of the gather's rows (sum of squares for Eq. 1, accepted
        // packets), and the round's counters mirrored into the host mailbox:
        // mailbox[1] = sum of squares (when the gather kept it), mailbox[8..11] = accepted,
        // candidates, stale, invalid
        // Only the rows that a launch of this round can have written are read: rows_staged of the
        // staged kernel's, rows_direct of the direct kernel's (row_pitch apart); the rest are zero.
        double s = 0.0;
        u64 a = 0;
        for (u32 k = 0; k < 2; ++k) {
            const double* sr = sumsq_rows + (size_t)k * row_pitch;
            const u64* ar = accept_rows + (size_t)k * row_pitch;
            const u32 n = k ? rows_direct : rows_staged;
            for (u32 i0 = 0; i0 < n; i0 += 4 * 256) {      // four independent loads of each kind in flight
                double sv[4]; u64 av[4];
                #pragma unroll
                for (u32 j = 0; j < 4; ++j) {
                    const u32 i = i0 + j * 256 + threadIdx.x;
                    sv[j] = i < n ? sr[i] : 0.0;
                    av[j] = i < n ? ar[i] : 0ull;
                }
                #pragma unroll
                for (u32 j = 0; j < 4; ++j) { s += sv[j]; a += av[j]; }
            }
        }
        s = wave_sum_f64(s);
        const u32 a_lo = wave_reduce<OpAdd>((u32)(a & 0xFFFFFu)), a_hi = wave_reduce<OpAdd>((u32)(a >> 20));   // 64 x 2^20 fits 32 bits
        if (lane == 0) { wsum[wave_in_block] = s; asum[wave_in_block] = ((u64)a_hi << 20) + a_lo; }
        __syncthreads();
        if (threadIdx.x == 0) {
            const u64 accepted = (asum[0] + asum[1]) + (asum[2] + asum[3]);
            counters[C_ACCEPTED] = accepted;
            if (scale_mode == 0) ((double*)mailbox)[1] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
            mailbox[8] = accepted; mailbox[9] = counters[C_CANDIDATES];
            mailbox[10] = counters[C_STALE]; mailbox[11] = counters[C_INVALID];
        }
        return;
    }
    const u32* fs = g.first_seq;
    if (TABLE_IN_LDS) {
        for (u32 i = threadIdx.x; i <= g.B; i += blockDim.x) fs_lds[i] = g.first_seq[i];
        __syncthreads();
        fs = fs_lds;
    }
    const u32 wave = blockIdx.x * (blockDim.x / WAVE) + wave_in_block;
    const u32 n_waves = n_work_blocks * (blockDim.x / WAVE);
    const u32 n_tiles = (g.n_pkts + FIN_TILE - 1) / FIN_TILE;
    const float inv_p = 1.0f / (float)g.P;
    const bool skip_same = scale_mode == 0;     // a span that already sits in `out` needs no copy
    double dsum = 0.0;
    for (u32 tile = wave; tile < n_tiles; tile += n_waves) {
        const u32 seq0 = tile * FIN_TILE;
        const u32 n_t = g.n_pkts - seq0 < FIN_TILE ? g.n_pkts - seq0 : FIN_TILE;
        // OR of the workers' bitmap words: lane w loads worker w's word (one load instruction
        // for the wave, W <= 64), the OR runs across the lanes
        const u64 mine = lane < g.W ? bitmap[(u64)lane * g.words_pw + (seq0 >> 6)] : 0ull;
        u64 any = ((u64)wave_reduce<OpOr>((u32)(mine >> 32)) << 32) | wave_reduce<OpOr>((u32)mine);
        any >>= (seq0 & 63);
        const u64 hm = *(const u64*)(home + seq0);          // byte t = copy of packet seq0 + t (valid where `any` has bit t)
        // which of the tile's packets need work at all (wave-uniform)
        u32 todo = 0;
        for (u32 t = 0; t < n_t; ++t) {
            const bool got = (any >> t) & 1ull;
            const float* src = ((hm >> (8 * t)) & 1ull) ? acc1 : acc0;
            if (!got || !(skip_same && src == out)) todo |= 1u << t;
        }
        if (!todo) continue;
        u32 b = find_bucket(fs, g.B, seq0);
        if (seq0 + n_t <= fs[b + 1]) {
            const u64 elem0 = g.b_off[b] + (u64)(seq0 - fs[b]) * g.P;
            const u64 bucket_end = g.b_off[b] + g.b_cnt[b];
            const u64 end = elem0 + (u64)n_t * g.P < bucket_end ? elem0 + (u64)n_t * g.P : bucket_end;
            const u64 c1 = (end - 1) >> 2;
            for (u64 c = (elem0 >> 2) + lane; c <= c1; c += WAVE) {
                const u64 e0 = c << 2;
                const u64 lo_e = e0 > elem0 ? e0 : elem0, hi_e = e0 + 3 < end - 1 ? e0 + 3 : end - 1;
                const u32 t_lo = div_small((u32)(lo_e - elem0), g.P, inv_p), t_hi = div_small((u32)(hi_e - elem0), g.P, inv_p);
                if (e0 >= elem0 && e0 + 4 <= end && t_lo == t_hi) {
                    if (!((todo >> t_lo) & 1u)) continue;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);      // never received: exactly zero
                    if ((any >> t_lo) & 1ull) {
                        v = *(const float4*)((((hm >> (8 * t_lo)) & 1ull) ? acc1 : acc0) + e0);
                        if (scale_mode) {
                            v.x = v.x / wf; v.y = v.y / wf; v.z = v.z / wf; v.w = v.w / wf;
                            dsum += (double)((v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w));
                        }
                    }
                    *(float4*)(out + e0) = v;
                } else {
                    for (u64 e = lo_e; e <= hi_e; ++e) {
                        const u32 t_e = div_small((u32)(e - elem0), g.P, inv_p);
                        if (!((todo >> t_e) & 1u)) continue;
                        float v = 0.f;
                        if ((any >> t_e) & 1ull) {
                            v = (((hm >> (8 * t_e)) & 1ull) ? acc1 : acc0)[e];
                            if (scale_mode) { v = v / wf; dsum += (double)(v * v); }
                        }
                        out[e] = v;
                    }
                }
            }
        } else {
            for (u32 t = 0; t < n_t; ++t) {
                const u32 seq = seq0 + t;
                while (seq >= fs[b + 1]) ++b;
                if (!((todo >> t) & 1u)) continue;
                u64 elem; u32 len;
                packet_span(g, seq, b, &elem, &len);
                float s = 0.f;
                if ((any >> t) & 1ull) {
                    const float* acc = ((hm >> (8 * t)) & 1ull) ? acc1 : acc0;
                    for (u32 j = lane; j < len; j += WAVE) {
                        float v = acc[elem + j];
                        if (scale_mode) { v = v / wf; s += v * v; }
                        out[elem + j] = v;
                    }
                } else {
                    for (u32 j = lane; j < len; j += WAVE) out[elem + j] = 0.f;
                }
                dsum += (double)s;
            }
        }
        // in-place form: the spans that were moved now live in copy 0
        if (move_home && lane < n_t && ((any >> lane) & 1ull) && ((hm >> (8 * lane)) & 1ull)) home[seq0 + lane] = 0;
    }
    if (scale_mode) {
        dsum = wave_sum_f64(dsum);
        if (lane == 0) wsum[wave_in_block] = dsum;
        __syncthreads();
        if (threadIdx.x == 0) partials[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    }
}

// Sum of squares of a plain vector (16-byte aligned), same partials layout.
__global__ __launch_bounds__(256) void sumsq_vec(const float* __restrict__ v, u64 n, double* __restrict__ partials) {
    __shared__ double wsum[4];
    const u64 n4 = n / 4;
    const float4* v4 = (const float4*)v;
    const u64 stride = (u64)gridDim.x * blockDim.x;
    double dsum = 0.0;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 x = v4[i];
        dsum += (double)((x.x * x.x + x.y * x.y) + (x.z * x.z + x.w * x.w));
    }
    if (blockIdx.x == 0 && threadIdx.x < (u32)(n - 4 * n4)) {
        float x = v[4 * n4 + threadIdx.x];
        dsum += (double)(x * x);
    }
    dsum = wave_sum_f64(dsum);
    if (lane_id() == 0) wsum[threadIdx.x / WAVE] = dsum;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// Fixed-order sum of the per-block partials; the result goes to the host mailbox.
__global__ __launch_bounds__(256) void reduce_partials(const double* __restrict__ partials, u32 n, double* __restrict__ mailbox) {
    __shared__ double wsum[4];
    double s = 0.0;
    for (u32 i = threadIdx.x; i < n; i += 256) s += partials[i];
    s = wave_sum_f64(s);
    if (lane_id() == 0) wsum[threadIdx.x / WAVE] = s;
    __syncthreads();
    if (threadIdx.x == 0) mailbox[0] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// ------------------------------------------------------------------------------------------
// where to write: measuring a buffer against the accumulator copies
// ------------------------------------------------------------------------------------------
// On this chip a stream of payload reads with a few percent of result writes mixed in runs about
// 15 % slower when the reads and the writes fall into the same third of the HBM address space
// than when they fall into different thirds (measured with this very loop: 1.60 vs 1.39 ms per
// 8.5 GB; which third a buffer lies in cannot be asked for, only measured).  The library
// therefore keeps two copies of the accumulator in different thirds when it can, and sends the
// spans a batch writes for the first time to the copy that is faster for that batch's buffer.
//
// The loop below has the access pattern of the gather (CLS_STREAMS streams of 1472-byte pieces,
// each wave sums one piece per stream and stores the 1472-byte result): a plain linear copy does
// not show the effect.  It reads CLS_SAMPLE_BYTES from src and writes CLS_SCRATCH_BYTES.
#define CLS_STREAMS 32u
#define CLS_PIECE 1472u
#define CLS_SEQS 22795u
#define CLS_SAMPLE_BYTES ((u64)CLS_STREAMS * CLS_SEQS * CLS_PIECE)      /* 1.07 GB */
#define CLS_SCRATCH_BYTES ((u64)CLS_SEQS * CLS_PIECE)                    /* 33.6 MB */
__global__ __launch_bounds__(256) void classify_rw(const uint8_t* __restrict__ src, float* __restrict__ scratch) {
    const u32 lane = lane_id();
    const u32 wave = (blockIdx.x * 256 + threadIdx.x) / WAVE, n_waves = gridDim.x * 4;
    const bool second = lane < CLS_PIECE / 16 - WAVE;            // 92 units per piece: lanes 0..27 take two
    for (u32 seq = wave; seq < CLS_SEQS; seq += n_waves) {
        f4v a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0;
        for (u32 w0 = 0; w0 < CLS_STREAMS; w0 += 4) {
            f4v v0[4], v1[4];
            #pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint8_t* b = src + ((u64)(w0 + j) * CLS_SEQS + seq) * CLS_PIECE + 16ull * lane;
                v0[j] = __builtin_nontemporal_load((const f4v*)b);
                v1[j] = f4v{0.f, 0.f, 0.f, 0.f};
                if (second) v1[j] = __builtin_nontemporal_load((const f4v*)(b + 1024));
            }
            #pragma unroll
            for (int j = 0; j < 4; ++j) { a0 += v0[j]; a1 += v1[j]; }
        }
        f4v* d = (f4v*)(scratch + (u64)seq * (CLS_PIECE / 4)) + lane;
        *d = a0;
        if (second) d[WAVE] = a1;
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct dblp_ctx {
    Geo g;
    u64 N;
    double eta;
    int device;
    hipStream_t stream;
    int n_cus;
    // device state
    u32* d_first_seq; u64* d_b_off; u64* d_b_cnt;
    u64* d_bitmap; u64* d_pending; u64* d_counters;
    // accumulator: one or two copies (d_acc[1] == d_acc[0] when there is one); each copy's
    // allocation ends with CLS_SCRATCH_BYTES that classify_rw may overwrite
    void* acc_alloc[2]; float* d_acc[2]; float* d_scratch[2];
    int n_acc;              // 1 or 2
    int acc_caller;         // the copies are the caller's buffers: never measured, never freed
    int acc_distinct;       // the two copies were measured to lie in different thirds of HBM
    float place_ms[2];      // that measurement: probe time writing to copy 0 / copy 1 (0 = not taken)
    int place_steps;        // candidates tried by the placement search
    double place_seconds;   // time the search took
    double search_fraction; // share of the free memory the search may hold
    double search_seconds;  // its time limit
    int fold;               // W is a power of two: the gather stores sum / W
    int norm_in_mailbox;    // the last finalize left the sum of squares in the host mailbox
    int counters_in_mailbox; // ... and the round's counters (until the next batch or round)
    int mailbox_seen;       // the stream has been synchronised since that finalize
    int acc_policy;         // DBLP_ACC_*
    int last_pick;          // copy the last batch wrote new spans to
    u32 batch_no;
    uint8_t* d_home;        // [n_pkts rounded up to 8] copy that holds each packet's span
    struct Picked { const void* p; u64 bytes; int pick; } picked[32];   // measured buffers
    u32 n_picked;
    hipEvent_t cls_ev[2];
    u32* d_need; u32* d_missing; u64* d_offs; double* d_partials;
    u32* d_block_tallies;   // [IDX_BLOCKS_PER_CU * n_cus][5], written by index_arrivals
    u64* d_accept_rows;     // [2][ACCEPT_ROWS] accepted packets per gather block (staged grid, direct grid)
    u32 rows_used[2];       // largest staged / direct gather grid launched in the open round
    int result_in_place;    // the form of the last dblp_finalize (in place until one says otherwise): prices the second copy
    double* d_sumsq_rows;   // [2][ACCEPT_ROWS] sum of squares of what each gather block stored (same allocation)
    u64* h_mailbox;         // pinned host memory, 16 x u64, also mapped into the device
    u64* d_mailbox;         // device address of h_mailbox
    // host copies of the geometry
    u32* h_first_seq; u64* h_b_off; u64* h_b_cnt;
    u32 n_partials;         // blocks of the last finalize / sumsq launch
    // protocol state
    int round_open; int finalized; uint16_t round;
    double prev_norm; int have_prev;
    // optional per-kernel timing (HIP events on the context's stream)
    int profiling;          // bit k set: launches of kernel group k are bracketed by events
    struct Timed { hipEvent_t a, b; int kernel; };
    std::vector<Timed>* timed;        // recorded, not yet read
    std::vector<hipEvent_t>* ev_pool; // free events
    char err[256];
};

static hipEvent_t prof_event(dblp_ctx* c) {
    hipEvent_t e = nullptr;
    if (!c->ev_pool->empty()) { e = c->ev_pool->back(); c->ev_pool->pop_back(); }
    else if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); e = nullptr; }
    return e;
}

// Brackets one kernel launch with events when profiling is on.
struct ProfScope {
    dblp_ctx* c; hipEvent_t a; int kernel;
    ProfScope(dblp_ctx* c_, int kernel_) : c(c_), a(nullptr), kernel(kernel_) {
        if (((c->profiling >> kernel) & 1) && (a = prof_event(c))) (void)hipEventRecord(a, c->stream);
    }
    ~ProfScope() {
        if (!a) return;
        hipEvent_t b = prof_event(c);
        if (!b) { c->ev_pool->push_back(a); return; }
        (void)hipEventRecord(b, c->stream);
        if (c->timed->size() < c->timed->capacity()) c->timed->push_back({a, b, kernel});   // never reallocates
        else { c->ev_pool->push_back(a); c->ev_pool->push_back(b); }                        // buffer full: drop the sample
    }
};

static int fail(dblp_ctx* c, int code, const char* what) {
    if (c) snprintf(c->err, sizeof c->err, "%s", what);
    return code;
}

static int fail_hip(dblp_ctx* c, hipError_t e, const char* what) {
    if (c) snprintf(c->err, sizeof c->err, "%s: %s", what, hipGetErrorString(e));
    return DBLP_EHIP;
}

#define HIP_TRY(c, call)                                            \
    do {                                                            \
        hipError_t e__ = (call);                                    \
        if (e__ != hipSuccess) return fail_hip((c), e__, #call);    \
    } while (0)

#define LAUNCH_CHECK(c, name)                                       \
    do {                                                            \
        hipError_t e__ = hipGetLastError();                         \
        if (e__ != hipSuccess) return fail_hip((c), e__, name);     \
    } while (0)

static u32 grid_for(const dblp_ctx* c, u64 blocks_wanted, u32 blocks_per_cu) {
    u64 cap = (u64)c->n_cus * blocks_per_cu;
    u64 g = blocks_wanted < cap ? blocks_wanted : cap;
    return (u32)(g ? g : 1);
}

extern "C" const char* dblp_last_error(const dblp_ctx* ctx) { return ctx ? ctx->err : "null context"; }

extern "C" int dblp_destroy(dblp_ctx* c) {
    if (!c) return DBLP_OK;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    void* dev[] = {c->d_first_seq, c->d_b_off, c->d_b_cnt, c->d_bitmap, c->d_pending,
                   c->acc_caller ? nullptr : c->acc_alloc[0], c->acc_caller ? nullptr : c->acc_alloc[1], c->d_home, c->d_counters, c->d_need, c->d_missing, c->d_offs, c->d_partials, c->d_block_tallies,
                   c->d_accept_rows};
    for (void* p : dev) if (p) (void)hipFree(p);
    for (hipEvent_t e : c->cls_ev) if (e) (void)hipEventDestroy(e);
    if (c->h_mailbox) (void)hipHostFree(c->h_mailbox);
    if (c->timed) { for (auto& t : *c->timed) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); } delete c->timed; }
    if (c->ev_pool) { for (auto e : *c->ev_pool) (void)hipEventDestroy(e); delete c->ev_pool; }
    free(c->h_first_seq); free(c->h_b_off); free(c->h_b_cnt);
    free(c);
    return DBLP_OK;
}

// Milliseconds of classify_rw reading src and writing scratch (best of two after one untimed run), < 0 on error.
static float time_rw(dblp_ctx* c, const void* src, float* scratch) {
    for (hipEvent_t& e : c->cls_ev)
        if (!e && hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); e = nullptr; return -1.f; }
    float best = -1.f;
    for (int r = 0; r < 3; ++r) {
        if (hipEventRecord(c->cls_ev[0], c->stream) != hipSuccess) return -1.f;
        hipLaunchKernelGGL(classify_rw, dim3(4 * c->n_cus), dim3(256), 0, c->stream, (const uint8_t*)src, scratch);
        if (hipEventRecord(c->cls_ev[1], c->stream) != hipSuccess) return -1.f;
        if (hipEventSynchronize(c->cls_ev[1]) != hipSuccess) return -1.f;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->cls_ev[0], c->cls_ev[1]) != hipSuccess) return -1.f;
        if (r > 0 && (best < 0.f || ms < best)) best = ms;
    }
    return best;
}

// (Re)allocates the library-owned accumulator as `copies` copies.  place != 0: search for a second
// copy in another third of the HBM address space than the first, within the context's limits
// (share of the free memory held at once, seconds), and have no second copy if none is found.
// The contents of the round in progress are lost.
#define PLACE_MAX_STEPS 40
#define PLACE_STRIDE_BYTES (6ull << 30)
static double wall_seconds() {
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (double)ts.tv_sec + 1e-9 * (double)ts.tv_nsec;
}

static int set_accumulator_copies(dblp_ctx* c, int copies, int place) {
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, DBLP_EHIP, "accumulator_copies: synchronize");
    for (int i = 0; i < 2; ++i) { if (c->acc_alloc[i]) (void)hipFree(c->acc_alloc[i]); c->acc_alloc[i] = nullptr; }
    c->n_acc = 1; c->acc_distinct = 0; c->place_ms[0] = c->place_ms[1] = 0.f; c->place_steps = 0; c->place_seconds = 0.0;
    c->n_picked = 0; c->last_pick = 0; c->round_open = 0; c->finalized = 0; c->norm_in_mailbox = 0; c->counters_in_mailbox = 0;
    const size_t bytes = (c->N * sizeof(float) + 255) / 256 * 256;     // the scratch area starts aligned
    const size_t scratch = copies == 2 ? CLS_SCRATCH_BYTES : 0;
    if (hipMalloc(&c->acc_alloc[0], bytes + scratch) != hipSuccess) { (void)hipGetLastError(); return fail(c, DBLP_ENOMEM, "accumulator"); }
    c->d_acc[0] = c->d_acc[1] = (float*)c->acc_alloc[0];
    c->d_scratch[0] = c->d_scratch[1] = (float*)((uint8_t*)c->acc_alloc[0] + bytes);
    if (copies != 2) return DBLP_OK;
    auto adopt = [&](void* p) {
        c->acc_alloc[1] = p; c->n_acc = 2;
        c->d_acc[1] = (float*)p; c->d_scratch[1] = (float*)((uint8_t*)p + bytes);
    };
    if (!place) {
        void* p = nullptr;
        if (hipMalloc(&p, bytes + scratch) == hipSuccess) adopt(p); else (void)hipGetLastError();
        return DBLP_OK;
    }
    // Walk through the free memory: candidate, then a holder allocation that pushes the next
    // candidate further on, until a candidate measures differently from the first copy against
    // the same read buffer, or the share of the free memory that may be held is reached, or time
    // is up.  What the probe reads: a buffer allocated right after the first copy (next to its
    // end, where the scratch area that the reference measurement writes lies).
    const double t_start = wall_seconds();
    void* near0 = nullptr;
    if (hipMalloc(&near0, CLS_SAMPLE_BYTES) != hipSuccess) { (void)hipGetLastError(); return DBLP_OK; }
    const void* rd = near0;
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) { (void)hipGetLastError(); free_b = 0; }
    const size_t may_hold = (size_t)((double)free_b * c->search_fraction);
    const float t_ref = time_rw(c, rd, c->d_scratch[0]);
    c->place_ms[0] = t_ref > 0.f ? t_ref : 0.f;
    void* held[2 * PLACE_MAX_STEPS];
    int n_held = 0;
    size_t held_bytes = 0;
    for (int step = 0; step < PLACE_MAX_STEPS && t_ref > 0.f; ++step) {
        if (held_bytes + bytes + scratch > may_hold) break;
        if (wall_seconds() - t_start > c->search_seconds) break;
        void* cand = nullptr;
        if (hipMalloc(&cand, bytes + scratch) != hipSuccess) { (void)hipGetLastError(); break; }
        // both ends of the candidate must differ from the first copy, and in the same direction
        // (a candidate that straddles two thirds is passed over); its contents are scratch here
        const float t_end = time_rw(c, rd, (float*)((uint8_t*)cand + bytes));
        const float t_beg = bytes >= CLS_SCRATCH_BYTES ? time_rw(c, rd, (float*)cand) : t_end;
        auto differs = [&](float t) { const float hi = t > t_ref ? t : t_ref; return t > 0.f && fabsf(t - t_ref) > 0.07f * hi; };
        c->place_ms[1] = t_end > 0.f ? t_end : 0.f;
        c->place_steps = step + 1;
        if (differs(t_end) && differs(t_beg) && (t_end < t_ref) == (t_beg < t_ref)) { adopt(cand); c->acc_distinct = 1; break; }
        held[n_held++] = cand; held_bytes += bytes + scratch;
        if (held_bytes + PLACE_STRIDE_BYTES > may_hold) break;
        void* holder = nullptr;
        if (hipMalloc(&holder, PLACE_STRIDE_BYTES) != hipSuccess) { (void)hipGetLastError(); break; }
        held[n_held++] = holder; held_bytes += PLACE_STRIDE_BYTES;
    }
    for (int i = 0; i < n_held; ++i) (void)hipFree(held[i]);
    (void)hipFree(near0);
    (void)hipGetLastError();
    c->place_seconds = wall_seconds() - t_start;
    return DBLP_OK;
}

// Which copy the spans that this batch writes first should go to.  Never allocates.  Measures
// (and then waits for its probe kernel) only under the automatic policy on a context with two
// library-owned copies, once per large packet buffer.
static int pick_copy(dblp_ctx* c, const void* d_packets, u64 bytes, u64 n_slots, u64 n_arrivals) {
    if (c->n_acc < 2) return 0;
    switch (c->acc_policy) {
    case DBLP_ACC_FIRST: return 0;
    case DBLP_ACC_SECOND: return 1;
    case DBLP_ACC_ALTERNATE: return (int)(c->batch_no & 1u);
    default: break;
    }
    // automatic: measure the buffer once; small or thinly used buffers are not worth it, and
    // caller-owned copies have no scratch area to write to
    if (c->acc_caller || bytes < CLS_SAMPLE_BYTES || n_arrivals < n_slots / 8) return 0;
    for (u32 i = 0; i < c->n_picked; ++i)
        if (c->picked[i].p == d_packets && c->picked[i].bytes == bytes) return c->picked[i].pick;
    const u64 last = (bytes - CLS_SAMPLE_BYTES) & ~15ull;
    const u64 offs[3] = {0, (last / 2) & ~15ull, last};
    const int n_offs = bytes >= 3 * CLS_SAMPLE_BYTES ? 3 : 1;
    auto measure = [&](float* scratch) {           // summed over the sample positions, < 0 on error
        float sum = 0.f;
        for (int i = 0; i < n_offs; ++i) {
            const float ms = time_rw(c, (const uint8_t*)d_packets + offs[i], scratch);
            if (ms < 0.f) { (void)hipGetLastError(); return -1.f; }
            sum += ms;
        }
        return sum;
    };
    const float t0 = measure(c->d_scratch[0]);
    if (t0 < 0.f) return 0;
    const float t1 = measure(c->d_scratch[1]);
    // The second copy has to be that much faster: 3 % when the result is copied out of the
    // accumulator anyway; when it is left in place, spans written to the second copy are moved to
    // the first by finalize (8 bytes per element, at about two thirds of the gather's rate, against
    // the 4 W (1 + 2/P) + 4 bytes per element that the gather moves).
    float margin = 0.03f;
    if (c->result_in_place) {
        const float gather_bytes = 4.f * (float)c->g.W * (1.f + 2.f / (float)c->g.P) + 4.f;
        margin += 1.5f * 8.f / gather_bytes;
    }
    const int pick = t1 > 0.f && t1 < (1.f - margin) * t0 ? 1 : 0;
    dblp_ctx::Picked& slot = c->picked[c->n_picked < 32 ? c->n_picked++ : c->batch_no % 32];
    slot.p = d_packets; slot.bytes = bytes; slot.pick = pick;
    return pick;
}

#ifndef FIN_BLOCKS_PER_CU
#define FIN_BLOCKS_PER_CU 8
#endif
#define ACCEPT_ROWS 8192   // >= blocks of any gather launch (n_cus * blocks per CU)
#ifndef IDX_BLOCKS_PER_CU
#define IDX_BLOCKS_PER_CU 4   // 2-4 blocks per CU index 3 % faster than 8: its bound is requests to memory, not latency
#endif
// Largest bucket-boundary table (bytes) a kernel copies into LDS; with up to 8 blocks per CU
// (finalize) this keeps all of them resident in the CU's 160 KB.  Larger tables are searched in global memory.
#define IDX_TABLE_LDS_MAX 16384u

extern "C" int dblp_create(dblp_ctx** out, const dblp_config* cfg) {
    if (!out || !cfg || !cfg->buckets) return DBLP_EINVAL;
    if (cfg->n_workers == 0 || cfg->n_workers > DBLP_MAX_WORKERS) return DBLP_EINVAL;
    if (cfg->payload_floats == 0 || cfg->payload_floats > 65535) return DBLP_EINVAL;
    if (cfg->n_buckets == 0 || cfg->n_elems == 0) return DBLP_EINVAL;
    if (!(cfg->eta >= 0.0)) return DBLP_EINVAL;
    if (cfg->accumulator_mode < DBLP_ACCMODE_SINGLE || cfg->accumulator_mode > DBLP_ACCMODE_SEARCH) return DBLP_EINVAL;
    if (cfg->search_free_fraction < 0.0 || cfg->search_free_fraction > 0.9 || !(cfg->search_seconds >= 0.0)) return DBLP_EINVAL;
    for (int i = 0; i < 2; ++i)
        if (cfg->d_accumulator[i] && ((uintptr_t)cfg->d_accumulator[i] & 255) != 0) return DBLP_EINVAL;
    if (cfg->d_accumulator[1] && (!cfg->d_accumulator[0] || cfg->accumulator_mode != DBLP_ACCMODE_PAIR ||
                                  cfg->d_accumulator[1] == cfg->d_accumulator[0])) return DBLP_EINVAL;
    if (cfg->d_accumulator[0] && cfg->accumulator_mode == DBLP_ACCMODE_SEARCH) return DBLP_EINVAL;   // the search owns both copies
    if (cfg->d_accumulator[0] && cfg->accumulator_mode == DBLP_ACCMODE_PAIR && !cfg->d_accumulator[1]) return DBLP_EINVAL;
    const u32 B = cfg->n_buckets, P = cfg->payload_floats;
    u64 expect = 0, n_pkts = 0;
    for (u32 b = 0; b < B; ++b) {
        if (cfg->buckets[b].elem_offset != expect) return DBLP_EINVAL;
        if (cfg->buckets[b].elem_count == 0 || cfg->buckets[b].elem_count >= (1ull << 32)) return DBLP_EINVAL;
        expect += cfg->buckets[b].elem_count;
        n_pkts += (cfg->buckets[b].elem_count + P - 1) / P;
    }
    if (expect != cfg->n_elems) return DBLP_EINVAL;
    if (n_pkts >= 0xFFFFFFFFull) return DBLP_EINVAL;

    dblp_ctx* c = (dblp_ctx*)calloc(1, sizeof *c);
    if (!c) return DBLP_ENOMEM;
    c->N = cfg->n_elems; c->eta = cfg->eta; c->device = cfg->device; c->stream = (hipStream_t)cfg->stream;
    c->search_fraction = cfg->search_free_fraction > 0.0 ? cfg->search_free_fraction : 0.5;
    c->search_seconds = cfg->search_seconds > 0.0 ? cfg->search_seconds : 2.0;
    c->fold = (cfg->n_workers & (cfg->n_workers - 1)) == 0;
    c->result_in_place = c->fold ? 1 : 0;     // the in-place finalize exists for power-of-two worker counts
    c->timed = new (std::nothrow) std::vector<dblp_ctx::Timed>();
    c->ev_pool = new (std::nothrow) std::vector<hipEvent_t>();
    if (!c->timed || !c->ev_pool) { dblp_destroy(c); return DBLP_ENOMEM; }
    c->h_first_seq = (u32*)malloc((B + 1) * sizeof(u32));
    c->h_b_off = (u64*)malloc(B * sizeof(u64));
    c->h_b_cnt = (u64*)malloc(B * sizeof(u64));
    if (!c->h_first_seq || !c->h_b_off || !c->h_b_cnt) { dblp_destroy(c); return DBLP_ENOMEM; }
    u64 seq = 0;
    for (u32 b = 0; b < B; ++b) {
        c->h_first_seq[b] = (u32)seq;
        c->h_b_off[b] = cfg->buckets[b].elem_offset;
        c->h_b_cnt[b] = cfg->buckets[b].elem_count;
        seq += (c->h_b_cnt[b] + P - 1) / P;
    }
    c->h_first_seq[B] = (u32)seq;

    Geo& g = c->g;
    g.B = B; g.P = P; g.W = cfg->n_workers; g.n_pkts = (u32)n_pkts;
    g.stride = (8 + 4 * P + 15) / 16 * 16;
    g.units = g.stride / 16;
    g.words_pw = (n_pkts + 63) / 64;

    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) { dblp_destroy(c); return DBLP_EHIP; }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) { dblp_destroy(c); return DBLP_EHIP; }
    c->n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if ((u64)c->n_cus * 16 > ACCEPT_ROWS) c->n_cus = ACCEPT_ROWS / 16;   // grids are sized n_cus x (<= 16) blocks

    const u64 pairs = (u64)g.W * B;
    const u32 max_partials = (u32)c->n_cus * FIN_BLOCKS_PER_CU;
    bool ok = true;
    ok = ok && hipMalloc(&c->d_first_seq, (B + 1) * sizeof(u32)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_b_off, B * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_b_cnt, B * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_bitmap, g.W * g.words_pw * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_pending, (u64)g.W * n_pkts * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_home, (n_pkts + 7) / 8 * 8 + 8) == hipSuccess;
    ok = ok && hipMalloc(&c->d_counters, C_COUNT * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_need, pairs * sizeof(u32)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_missing, pairs * sizeof(u32)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_offs, pairs * sizeof(u64)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_partials, max_partials * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_accept_rows, 4 * ACCEPT_ROWS * sizeof(u64)) == hipSuccess;   // + the sum-of-squares rows
    ok = ok && hipMalloc(&c->d_block_tallies, (size_t)c->n_cus * IDX_BLOCKS_PER_CU * 5 * sizeof(u32)) == hipSuccess;
    ok = ok && hipHostMalloc((void**)&c->h_mailbox, 16 * sizeof(u64), hipHostMallocMapped) == hipSuccess;
    if (!ok) { (void)hipGetLastError(); dblp_destroy(c); return DBLP_ENOMEM; }
    ok = ok && hipHostGetDevicePointer((void**)&c->d_mailbox, c->h_mailbox, 0) == hipSuccess;
    ok = ok && hipMemcpyAsync(c->d_first_seq, c->h_first_seq, (B + 1) * sizeof(u32), hipMemcpyHostToDevice, c->stream) == hipSuccess;
    ok = ok && hipMemcpyAsync(c->d_b_off, c->h_b_off, B * sizeof(u64), hipMemcpyHostToDevice, c->stream) == hipSuccess;
    ok = ok && hipMemcpyAsync(c->d_b_cnt, c->h_b_cnt, B * sizeof(u64), hipMemcpyHostToDevice, c->stream) == hipSuccess;
    if (!ok) { (void)hipGetLastError(); dblp_destroy(c); return DBLP_EHIP; }
    g.first_seq = c->d_first_seq; g.b_off = c->d_b_off; g.b_cnt = c->d_b_cnt;
    c->d_sumsq_rows = (double*)(c->d_accept_rows + 2 * ACCEPT_ROWS);

    const u64 n_pending = (u64)g.W * n_pkts;
    hipLaunchKernelGGL(fill_u64, dim3(grid_for(c, (n_pending + 255) / 256, 16)), dim3(256), 0, c->stream,
                       c->d_pending, n_pending, NONE64);
    hipLaunchKernelGGL(fill_u64, dim3(grid_for(c, (g.W * g.words_pw + 255) / 256, 16)), dim3(256), 0, c->stream,
                       c->d_bitmap, g.W * g.words_pw, 0ull);
    hipLaunchKernelGGL(reset_counters, dim3(1), dim3(64), 0, c->stream, c->d_counters);
    hipLaunchKernelGGL(fill_u64, dim3(32), dim3(256), 0, c->stream, c->d_accept_rows, (u64)(4 * ACCEPT_ROWS), 0ull);
    hipLaunchKernelGGL(fill_u64, dim3(grid_for(c, (n_pkts + 16 + 2047) / 2048, 16)), dim3(256), 0, c->stream,
                       (u64*)c->d_home, (u64)((n_pkts + 7) / 8 + 1), 0ull);
    e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess || hipGetLastError() != hipSuccess) { dblp_destroy(c); return DBLP_EHIP; }
    // accumulator last
    if (cfg->d_accumulator[0]) {
        c->acc_caller = 1;
        c->acc_alloc[0] = cfg->d_accumulator[0]; c->acc_alloc[1] = cfg->d_accumulator[1];
        c->d_acc[0] = cfg->d_accumulator[0];
        c->d_acc[1] = cfg->d_accumulator[1] ? cfg->d_accumulator[1] : cfg->d_accumulator[0];
        c->n_acc = cfg->d_accumulator[1] ? 2 : 1;
        c->d_scratch[0] = c->d_scratch[1] = nullptr;
    } else {
        const int rc = set_accumulator_copies(c, cfg->accumulator_mode == DBLP_ACCMODE_SINGLE ? 1 : 2,
                                              cfg->accumulator_mode == DBLP_ACCMODE_SEARCH ? 1 : 0);
        if (rc != DBLP_OK) { dblp_destroy(c); return rc; }
    }
    c->err[0] = 0;
    *out = c;
    return DBLP_OK;
}

extern "C" int dblp_layout(const dblp_ctx* c, uint64_t* n_pkts, uint32_t* stride, uint64_t* words_pw) {
    if (!c) return DBLP_EINVAL;
    if (n_pkts) *n_pkts = c->g.n_pkts;
    if (stride) *stride = c->g.stride;
    if (words_pw) *words_pw = c->g.words_pw;
    return DBLP_OK;
}

extern "C" int dblp_accumulator_copies(dblp_ctx* c, int copies, int place) {
    if (!c) return DBLP_EINVAL;
    if (copies != 1 && copies != 2) return fail(c, DBLP_EINVAL, "accumulator_copies: 1 or 2");
    if (place < 0 || place > 1) return fail(c, DBLP_EINVAL, "accumulator_copies: place is 0 or 1");
    if (c->acc_caller) return fail(c, DBLP_EINVAL, "accumulator_copies: the accumulator is the caller's");
    HIP_TRY(c, hipSetDevice(c->device));
    return set_accumulator_copies(c, copies, place);
}

extern "C" int dblp_accumulator_policy(dblp_ctx* c, int policy) {
    if (!c) return DBLP_EINVAL;
    if (policy < DBLP_ACC_AUTO || policy > DBLP_ACC_ALTERNATE) return fail(c, DBLP_EINVAL, "accumulator_policy: unknown policy");
    c->acc_policy = policy;
    return DBLP_OK;
}

extern "C" int dblp_accumulator_info(const dblp_ctx* c, int* copies, int* distinct, int* last_pick, double* placement_ms) {
    if (!c) return DBLP_EINVAL;
    if (placement_ms) { placement_ms[0] = c->place_ms[0]; placement_ms[1] = c->place_ms[1]; placement_ms[2] = c->place_steps; placement_ms[3] = c->place_seconds; }
    if (copies) *copies = c->n_acc;
    if (distinct) *distinct = c->acc_distinct;
    if (last_pick) *last_pick = c->last_pick;
    return DBLP_OK;
}

extern "C" int dblp_accumulator_ptr(const dblp_ctx* c, int which, float** d_copy) {
    if (!c || !d_copy) return DBLP_EINVAL;
    if (which < 0 || which >= c->n_acc || !c->acc_alloc[0]) return DBLP_EINVAL;
    *d_copy = c->d_acc[which];
    return DBLP_OK;
}

extern "C" int dblp_begin_round(dblp_ctx* c, uint16_t round) {
    if (!c) return DBLP_EINVAL;
    if (!c->acc_alloc[0]) return fail(c, DBLP_ESTATE, "begin_round: no accumulator (dblp_accumulator_copies ran out of memory)");
    HIP_TRY(c, hipSetDevice(c->device));
    const u64 n = c->g.W * c->g.words_pw;
    hipLaunchKernelGGL(reset_round, dim3(grid_for(c, (n + 4 * ACCEPT_ROWS + 255) / 256, 16)), dim3(256), 0, c->stream,
                       c->d_bitmap, n, c->d_accept_rows, (u64)(4 * ACCEPT_ROWS), c->d_counters);
    LAUNCH_CHECK(c, "begin_round");
    c->round = round; c->round_open = 1; c->finalized = 0; c->norm_in_mailbox = 0; c->counters_in_mailbox = 0;
    c->rows_used[0] = c->rows_used[1] = 0;
    return DBLP_OK;
}

// Element window [lo, hi) covered by packets first_seq .. first_seq + n - 1 (host geometry).
static void seq_window(const dblp_ctx* c, u64 first_seq, u64 n, u64* lo, u64* hi) {
    const Geo& g = c->g;
    auto span = [&](u64 seq, u64* elem, u64* len) {
        u32 a = 0, b = g.B;
        while (b - a > 1) { u32 m = (a + b) / 2; if (c->h_first_seq[m] <= seq) a = m; else b = m; }
        u64 start = (seq - c->h_first_seq[a]) * g.P;
        u64 left = c->h_b_cnt[a] - start;
        *elem = c->h_b_off[a] + start;
        *len = left < g.P ? left : g.P;
    };
    u64 e0, l0, e1, l1;
    span(first_seq, &e0, &l0);
    span(first_seq + n - 1, &e1, &l1);
    *lo = e0; *hi = e1 + l1;
}

extern "C" int dblp_packetize(dblp_ctx* c, uint32_t w, uint16_t round, const float* d_grad, uint64_t elem_base,
                              uint64_t n_grad, uint64_t first_seq, uint64_t n_pkts, const uint32_t* d_slot_map,
                              uint64_t slot_base, uint64_t n_slots, void* d_packets, uint16_t* d_src_worker) {
    if (!c) return DBLP_EINVAL;
    if (n_pkts == 0) return DBLP_OK;
    if (!d_grad || !d_packets || !d_src_worker) return fail(c, DBLP_EINVAL, "packetize: null pointer");
    if (w >= c->g.W) return fail(c, DBLP_EINVAL, "packetize: worker out of range");
    if (first_seq >= c->g.n_pkts || n_pkts > c->g.n_pkts - first_seq) return fail(c, DBLP_EINVAL, "packetize: seq range");
    if (((uintptr_t)d_packets & 15) != 0) return fail(c, DBLP_EINVAL, "packetize: d_packets must be 16-byte aligned");
    if (!d_slot_map && (slot_base > n_slots || n_pkts > n_slots - slot_base)) return fail(c, DBLP_EINVAL, "packetize: slots exceed buffer");
    u64 lo, hi;
    seq_window(c, first_seq, n_pkts, &lo, &hi);
    if (lo < elem_base || hi > elem_base + n_grad) return fail(c, DBLP_EINVAL, "packetize: packets outside the gradient window");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t table = ((size_t)c->g.B + 1) * sizeof(u32);
    if (table <= IDX_TABLE_LDS_MAX)
        hipLaunchKernelGGL(packetize_kernel<true>, dim3(grid_for(c, (n_pkts + 3) / 4, 8)), dim3(256), table, c->stream, c->g, w,
                           (u32)round, d_grad, (u64)elem_base, (u32)first_seq, (u32)n_pkts, d_slot_map, (u64)slot_base,
                           (u64)n_slots, (uint8_t*)d_packets, d_src_worker, c->d_counters);
    else
        hipLaunchKernelGGL(packetize_kernel<false>, dim3(grid_for(c, (n_pkts + 3) / 4, 8)), dim3(256), 0, c->stream, c->g, w,
                           (u32)round, d_grad, (u64)elem_base, (u32)first_seq, (u32)n_pkts, d_slot_map, (u64)slot_base,
                           (u64)n_slots, (uint8_t*)d_packets, d_src_worker, c->d_counters);
    LAUNCH_CHECK(c, "packetize");
    if (d_slot_map) {   // slots come from device memory: the kernel checks them, report here
        u64 bad = 0;
        HIP_TRY(c, hipMemcpyAsync(c->h_mailbox + 4, c->d_counters + C_PKT_BAD, sizeof(u64), hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        bad = c->h_mailbox[4];
        if (bad) {
            HIP_TRY(c, hipMemsetAsync(c->d_counters + C_PKT_BAD, 0, sizeof(u64), c->stream));
            return fail(c, DBLP_EINVAL, "packetize: slot map entry outside the packet buffer");
        }
    }
    return DBLP_OK;
}

extern "C" int dblp_packetize_list(dblp_ctx* c, uint16_t round, const float* const* h_grads, const uint64_t* d_list,
                                   uint64_t n, uint64_t slot_base, uint64_t n_slots, void* d_packets,
                                   uint16_t* d_src_worker) {
    if (!c) return DBLP_EINVAL;
    if (n == 0) return DBLP_OK;
    if (!h_grads || !d_list || !d_packets || !d_src_worker) return fail(c, DBLP_EINVAL, "packetize_list: null pointer");
    if (((uintptr_t)d_packets & 15) != 0) return fail(c, DBLP_EINVAL, "packetize_list: d_packets must be 16-byte aligned");
    if (slot_base > n_slots || n > n_slots - slot_base) return fail(c, DBLP_EINVAL, "packetize_list: slots exceed buffer");
    GradPtrs gp;
    for (u32 w = 0; w < DBLP_MAX_WORKERS; ++w) gp.p[w] = nullptr;
    for (u32 w = 0; w < c->g.W; ++w) {
        if (!h_grads[w]) return fail(c, DBLP_EINVAL, "packetize_list: null gradient pointer");
        gp.p[w] = h_grads[w];
    }
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t table = ((size_t)c->g.B + 1) * sizeof(u32);
    if (table <= IDX_TABLE_LDS_MAX)
        hipLaunchKernelGGL(packetize_list_kernel<true>, dim3(grid_for(c, (n + 3) / 4, 8)), dim3(256), table, c->stream, c->g, gp,
                           (u32)round, (const u64*)d_list, (u64)n, (u64)slot_base, (uint8_t*)d_packets, d_src_worker,
                           c->d_counters);
    else
        hipLaunchKernelGGL(packetize_list_kernel<false>, dim3(grid_for(c, (n + 3) / 4, 8)), dim3(256), 0, c->stream, c->g, gp,
                           (u32)round, (const u64*)d_list, (u64)n, (u64)slot_base, (uint8_t*)d_packets, d_src_worker,
                           c->d_counters);
    LAUNCH_CHECK(c, "packetize_list");
    HIP_TRY(c, hipMemcpyAsync(c->h_mailbox + 4, c->d_counters + C_PKT_BAD, sizeof(u64), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->h_mailbox[4]) {
        HIP_TRY(c, hipMemsetAsync(c->d_counters + C_PKT_BAD, 0, sizeof(u64), c->stream));
        return fail(c, DBLP_EINVAL, "packetize_list: list entry with worker or seq out of range");
    }
    return DBLP_OK;
}

// Index pass + gather pass over one batch.  Exactly one of (d_src_worker [+ d_mask, d_order]) and
// d_queue describes the arrivals.
static int apply_batch(dblp_ctx* c, const void* d_packets, const uint16_t* d_src_worker, uint64_t n_slots,
                       const uint64_t* d_mask, const uint32_t* d_order, const uint64_t* d_queue, uint64_t n_arrivals) {
    HIP_TRY(c, hipSetDevice(c->device));
    const Geo& g = c->g;
    const int pick = pick_copy(c, d_packets, n_slots * g.stride, n_slots, n_arrivals);
    c->last_pick = pick;
    ++c->batch_no;
    u32 n_tally_rows = 0;
    {
        ProfScope ps(c, DBLP_K_INDEX);
        const u32 grid = grid_for(c, (n_arrivals + 255) / 256, IDX_BLOCKS_PER_CU);
        const size_t table = ((size_t)g.B + 1) * sizeof(u32);
        const bool lds = table <= IDX_TABLE_LDS_MAX;
        void (*idx)(Geo, const uint8_t*, const uint16_t*, u64, const u64*, const u32*, const u64*, u64, u32, u64*, u32*) =
            lds ? (d_queue ? index_arrivals<true, true> : index_arrivals<true, false>)
                : (d_queue ? index_arrivals<false, true> : index_arrivals<false, false>);
        hipLaunchKernelGGL(idx, dim3(grid), dim3(256), lds ? table : 0, c->stream, g,
                           (const uint8_t*)d_packets, d_src_worker, (u64)n_slots, (const u64*)d_mask, d_order,
                           (const u64*)d_queue, (u64)n_arrivals, (u32)c->round, c->d_pending, c->d_block_tallies);
        n_tally_rows = grid;
    }
    const float inv_w = c->fold ? 1.0f / (float)g.W : 1.0f;   // exact for the powers of two it is used with
    {
        u32 sub = SUB, sub_log2 = 4;
        while (sub >= 2 && 2u * sub * g.stride > GS_LDS_BUDGET) { sub >>= 1; --sub_log2; }
        // Which gather kernel: the staged one for dense batches, the direct one for sparse ones
        // (and for packets too long to stage).  Where the number of arrivals settles it, only that
        // one is launched: at least one arrival per SPARSE_DIV (worker, seq) pairs of the whole
        // round is dense whatever range it touches; fewer than one per 8 * SPARSE_DIV pairs is
        // taken as sparse.  In between both are launched and each decides on the device, from the
        // sequence range the index pass found, whether the batch is its own.
        const u64 pairs = (u64)g.W * g.n_pkts;
        const bool can_stage = sub >= 2;
        const bool surely_dense = can_stage && n_arrivals * SPARSE_DIV >= pairs;
        const bool surely_sparse = n_arrivals * SPARSE_DIV * 8 < pairs;
        const bool launch_staged = can_stage && !surely_sparse;
        const bool launch_direct = !surely_dense;
        if (launch_staged) {   // two groups of packets fit in LDS: readers + writer wave
            const u32 wpl = WAVE / sub;
            // Up to GS_WRITER_PREPARES_MAX_W workers the writer wave prepares the next group while the
            // readers gather this one (measured: 4-6 % off the launch with 8 workers, 2 % with 16, but
            // 3.5 % slower with 32, where the readers share the index loads of a group instead).
            const u32 writer_prepares = g.W <= GS_WRITER_PREPARES_MAX_W ? 1u : 0u;
            // two packet buffers, one or two slot tables, and the bucket table when it fits a block's LDS limit
            size_t lds = 2ull * sub * g.stride + (writer_prepares ? 2 : 1) * (size_t)((g.W + wpl - 1) / wpl * wpl) * sub * sizeof(u32);
            const size_t table = ((size_t)g.B + 1) * sizeof(u32);
            const u32 table_in_lds = table <= IDX_TABLE_LDS_MAX && lds + table <= 64u * 1024u ? 1u : 0u;
            if (table_in_lds) lds += table;
            const u64 groups = ((u64)g.n_pkts + sub - 1) / sub;
            const u32 n_pass = (g.units + WAVE - 1) / WAVE;
            // Block shape: packets of up to 2 KB (one or two 1 KB passes) go fastest with 4 reader waves
            // and three blocks per CU (measured: 5 % off the launch with 8 workers, 0.6 % with 32);
            // longer packets with up to 8 reader waves and two blocks per CU (three: 9 % slower at 4 KB).
            const u32 readers_max = n_pass <= 2 ? (u32)GS_READERS_SHORT : (u32)GS_READERS;
            const u32 per_cu_max = n_pass <= 2 ? (u32)GS_MAX_PER_CU_SHORT : (u32)GS_MAX_PER_CU;
            const u32 readers = sub < readers_max ? sub : readers_max;   // a reader wave takes whole packets
            u32 per_cu = (u32)((160u * 1024u) / (lds + 1024));
            if (per_cu > 32 / (readers + 1)) per_cu = 32 / (readers + 1);
            if (per_cu > per_cu_max) per_cu = per_cu_max;
            if (per_cu < 1) per_cu = 1;
            void (*kern)(Geo, const uint8_t*, u64*, u64*, float*, float*, uint8_t*, u32, const u32*, u32, u64*, int, u64*, double*, float, u32, u32, u32, u32, u32) =
                n_pass == 1 ? gather_accumulate_staged<1> : n_pass == 2 ? gather_accumulate_staged<2>
                : n_pass == 3 ? gather_accumulate_staged<3> : n_pass == 4 ? gather_accumulate_staged<4>
                : n_pass == 5 ? gather_accumulate_staged<5> : gather_accumulate_staged<0>;
            const u32 grid = grid_for(c, groups, per_cu);
            if (grid > c->rows_used[0]) c->rows_used[0] = grid;
            ProfScope ps(c, DBLP_K_GATHER);
            hipLaunchKernelGGL(kern, dim3(grid), dim3((readers + 1) * WAVE),
                               lds, c->stream, g, (const uint8_t*)d_packets, c->d_pending, c->d_bitmap, c->d_acc[0],
                               c->d_acc[1], c->d_home, (u32)pick, (const u32*)c->d_block_tallies, n_tally_rows, c->d_counters,
                               surely_dense ? 1 : 0, c->d_accept_rows, c->d_sumsq_rows, inv_w, sub, sub_log2, n_pass, table_in_lds,
                               writer_prepares);
        }
        if (launch_direct) {   // sparse batches, and packets too long to stage: direct stores from the gathering waves
            const u64 groups = ((u64)g.n_pkts + SUB - 1) / SUB;
            size_t lds = (size_t)((g.W + 3) / 4 * 4) * SUB * sizeof(u32);
            const size_t table = ((size_t)g.B + 1) * sizeof(u32);
            const u32 table_in_lds = table <= IDX_TABLE_LDS_MAX ? 1u : 0u;
            if (table_in_lds) lds += table;
            const u32 grid = grid_for(c, groups, GA_BLOCKS_PER_CU);
            if (grid > c->rows_used[1]) c->rows_used[1] = grid;
            ProfScope ps(c, DBLP_K_GATHER_DIRECT);
            hipLaunchKernelGGL(gather_accumulate, dim3(grid), dim3(GA_WAVES * WAVE),
                               lds, c->stream, g, (const uint8_t*)d_packets, c->d_pending, c->d_bitmap, c->d_acc[0],
                               c->d_acc[1], c->d_home, (u32)pick, (const u32*)c->d_block_tallies, n_tally_rows, c->d_counters,
                               launch_staged ? 0 : 1, c->d_accept_rows + ACCEPT_ROWS, c->d_sumsq_rows + ACCEPT_ROWS, inv_w,
                               launch_staged ? 1 : 0, table_in_lds);
        }
    }
    LAUNCH_CHECK(c, "apply_arrivals");
    c->finalized = 0; c->norm_in_mailbox = 0; c->counters_in_mailbox = 0;
    return DBLP_OK;
}

extern "C" int dblp_apply_arrivals(dblp_ctx* c, const void* d_packets, const uint16_t* d_src_worker, uint64_t n_slots,
                                   const uint64_t* d_mask, const uint32_t* d_order, uint64_t n_arrivals) {
    if (!c) return DBLP_EINVAL;
    if (!c->round_open) return fail(c, DBLP_ESTATE, "apply_arrivals before begin_round");
    if (n_arrivals == 0) return DBLP_OK;
    if (!d_packets || !d_src_worker) return fail(c, DBLP_EINVAL, "apply_arrivals: null pointer");
    if (((uintptr_t)d_packets & 15) != 0) return fail(c, DBLP_EINVAL, "apply_arrivals: d_packets must be 16-byte aligned");
    if (n_slots >= 0xFFFFFFFFull || n_arrivals >= 0xFFFFFFFFull) return fail(c, DBLP_EINVAL, "apply_arrivals: too many slots");
    if (!d_order && n_arrivals > n_slots) return fail(c, DBLP_EINVAL, "apply_arrivals: identity order longer than the buffer");
    return apply_batch(c, d_packets, d_src_worker, n_slots, d_mask, d_order, nullptr, n_arrivals);
}

extern "C" int dblp_apply_arrivals_queue(dblp_ctx* c, const void* d_packets, uint64_t n_slots, const uint64_t* d_queue,
                                         uint64_t n_arrivals) {
    if (!c) return DBLP_EINVAL;
    if (!c->round_open) return fail(c, DBLP_ESTATE, "apply_arrivals_queue before begin_round");
    if (n_arrivals == 0) return DBLP_OK;
    if (!d_packets || !d_queue) return fail(c, DBLP_EINVAL, "apply_arrivals_queue: null pointer");
    if (((uintptr_t)d_packets & 15) != 0) return fail(c, DBLP_EINVAL, "apply_arrivals_queue: d_packets must be 16-byte aligned");
    if (((uintptr_t)d_queue & 7) != 0) return fail(c, DBLP_EINVAL, "apply_arrivals_queue: d_queue must be 8-byte aligned");
    if (n_slots >= 0xFFFFFFFFull || n_arrivals >= 0xFFFFFFFFull) return fail(c, DBLP_EINVAL, "apply_arrivals_queue: too many slots");
    return apply_batch(c, d_packets, nullptr, n_slots, nullptr, nullptr, d_queue, n_arrivals);
}

extern "C" int dblp_loss_account(dblp_ctx* c, uint32_t bound_ppm, uint32_t* d_missing, uint64_t* d_retx_list,
                                 uint64_t retx_capacity, uint64_t* h_retx_count, int* h_all_met) {
    if (!c) return DBLP_EINVAL;
    if (!c->round_open) return fail(c, DBLP_ESTATE, "loss_account before begin_round");
    if (!h_retx_count || !h_all_met) return fail(c, DBLP_EINVAL, "loss_account: null host pointer");
    if (!d_retx_list && retx_capacity) return fail(c, DBLP_EINVAL, "loss_account: null list with capacity");
    if (bound_ppm > 1000000u) return fail(c, DBLP_EINVAL, "loss_account: bound above 100%");
    HIP_TRY(c, hipSetDevice(c->device));
    const Geo& g = c->g;
    const u32 pairs = g.W * g.B;
    {
        ProfScope ps(c, DBLP_K_PROBE);
        hipLaunchKernelGGL(loss_count, dim3(grid_for(c, (pairs + 3) / 4, 8)), dim3(256), 0, c->stream, g, c->d_bitmap,
                           bound_ppm, d_missing ? d_missing : c->d_missing, c->d_need);
        hipLaunchKernelGGL(scan_need, dim3(1), dim3(1024), 0, c->stream, c->d_need, pairs, c->d_offs, c->d_mailbox);
        if (retx_capacity)
            hipLaunchKernelGGL(emit_retx, dim3(grid_for(c, (pairs + 3) / 4, 8)), dim3(256), 0, c->stream, g, c->d_bitmap,
                               c->d_need, c->d_offs, (u64*)d_retx_list, (u64)retx_capacity);
    }
    LAUNCH_CHECK(c, "loss_account");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->mailbox_seen = 1;
    const u64 total = c->h_mailbox[0];
    *h_retx_count = total;
    *h_all_met = total == 0;
    if (total > retx_capacity) return fail(c, DBLP_ECAPACITY, "retransmit list truncated");
    return DBLP_OK;
}

extern "C" int dblp_finalize(dblp_ctx* c, int compensation, float* d_out) {
    if (!c) return DBLP_EINVAL;
    if (!c->round_open) return fail(c, DBLP_ESTATE, "finalize before begin_round");
    if (compensation != DBLP_COMP_ZEROFILL_MEAN) return fail(c, DBLP_EINVAL, "finalize: unknown compensation mode");
    const bool in_place = !d_out || d_out == c->d_acc[0];
    if (in_place && !c->fold) return fail(c, DBLP_EINVAL, "finalize: the in-place form needs a power-of-two worker count");
    if (!in_place && c->n_acc == 2 && d_out == c->d_acc[1]) return fail(c, DBLP_EINVAL, "finalize: d_out is the second accumulator copy");
    if (((uintptr_t)d_out & 15) != 0) return fail(c, DBLP_EINVAL, "finalize: d_out must be 16-byte aligned");
    HIP_TRY(c, hipSetDevice(c->device));
    const Geo& g = c->g;
    const u64 tiles = ((u64)g.n_pkts + FIN_TILE - 1) / FIN_TILE;
    const u32 work = grid_for(c, (tiles + 3) / 4, FIN_BLOCKS_PER_CU);
    const u32 grid = work + 1;      // one more block sums the gather's rows: accepted packets, and the sum of squares for Eq. 1
    float* out = in_place ? c->d_acc[0] : d_out;
    {
        ProfScope ps(c, DBLP_K_FINALIZE);
        const size_t table = ((size_t)g.B + 1) * sizeof(u32);
        void (*kern)(Geo, const u64*, const float*, const float*, uint8_t*, float*, int, float, int, double*, u32,
                     const double*, const u64*, u32, u32, u32, u64*, u64*) = table <= IDX_TABLE_LDS_MAX ? finalize_pass<true> : finalize_pass<false>;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), table <= IDX_TABLE_LDS_MAX ? table : 0, c->stream, g, c->d_bitmap,
                           (const float*)c->d_acc[0], (const float*)c->d_acc[1], c->d_home, out, c->fold ? 0 : 1, (float)g.W,
                           in_place ? 1 : 0, c->d_partials, work, (const double*)c->d_sumsq_rows, (const u64*)c->d_accept_rows,
                           c->rows_used[0], c->rows_used[1], (u32)ACCEPT_ROWS, c->d_counters, c->d_mailbox);
    }
    LAUNCH_CHECK(c, "finalize");
    c->result_in_place = in_place ? 1 : 0;
    c->n_partials = work;
    c->finalized = 1;
    c->norm_in_mailbox = c->fold;
    c->counters_in_mailbox = 1;     // valid on the host once the stream has been synchronised (mailbox_seen)
    c->mailbox_seen = 0;
    return DBLP_OK;
}

extern "C" int dblp_phase_signal(dblp_ctx* c, const float* d_vec, double* h_norm, double* h_rel_delta, int* h_critical) {
    if (!c) return DBLP_EINVAL;
    if (!h_norm || !h_rel_delta || !h_critical) return fail(c, DBLP_EINVAL, "phase_signal: null host pointer");
    HIP_TRY(c, hipSetDevice(c->device));
    if (d_vec) {
        if (((uintptr_t)d_vec & 15) != 0) return fail(c, DBLP_EINVAL, "phase_signal: d_vec must be 16-byte aligned");
        const u32 n_partials = grid_for(c, (c->N / 4 + 255) / 256, FIN_BLOCKS_PER_CU);
        hipLaunchKernelGGL(sumsq_vec, dim3(n_partials), dim3(256), 0, c->stream, d_vec, (u64)c->N, c->d_partials);
        hipLaunchKernelGGL(reduce_partials, dim3(1), dim3(256), 0, c->stream, c->d_partials, n_partials,
                           (double*)(c->d_mailbox + 1));
        c->finalized = 0;   // neither the partials nor the mailbox belong to a finalize any more
        c->norm_in_mailbox = 0;
    } else {
        if (!c->finalized) return fail(c, DBLP_ESTATE, "phase_signal without a finalize in this round");
        if (!c->norm_in_mailbox)     // W not a power of two: the finalize pass left per-block partial sums
            hipLaunchKernelGGL(reduce_partials, dim3(1), dim3(256), 0, c->stream, c->d_partials, c->n_partials,
                               (double*)(c->d_mailbox + 1));
    }
    LAUNCH_CHECK(c, "phase_signal");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->mailbox_seen = 1;
    double ss;
    memcpy(&ss, c->h_mailbox + 1, sizeof ss);
    if (ss < 0.0) ss = 0.0;     // the running sum of squares can end a rounding error below zero
    const double norm = sqrt(ss);
    if (!c->have_prev || c->prev_norm == 0.0) {
        *h_rel_delta = INFINITY;
        *h_critical = 1;
    } else {
        *h_rel_delta = fabs(c->prev_norm - norm) / c->prev_norm;
        *h_critical = *h_rel_delta >= c->eta;
    }
    *h_norm = norm;
    c->prev_norm = norm;
    c->have_prev = 1;
    return DBLP_OK;
}

// ------------------------------------------------------------------------------------------
// sum of squares without any allocation: per-block partial sums in a static device array
// ------------------------------------------------------------------------------------------
#define STATIC_PARTIALS 4096                    // blocks of one launch at most; 32 KB per GPU
#define STATIC_MAX_ELEMS (1ull << 36)           // 64 Gi floats: more than any one GPU holds
#define STATIC_MAX_DEVICES 16
static __device__ __align__(256) double static_partials[STATIC_PARTIALS];
static double* static_partials_ptr[STATIC_MAX_DEVICES];     // device address of the array on each GPU
static int static_cus[STATIC_MAX_DEVICES];
static thread_local char static_err[160] = "";

extern "C" const char* dblp_sumsq_static_error(void) { return static_err; }

extern "C" int dblp_sumsq_static(int device, void* stream, const float* d_vec, uint64_t n_elems, double* d_sumsq) {
    if (device < 0 || device >= STATIC_MAX_DEVICES) { snprintf(static_err, sizeof static_err, "sumsq_static: device ordinal outside 0..%d", STATIC_MAX_DEVICES - 1); return DBLP_EINVAL; }
    if (!d_vec || !d_sumsq) { snprintf(static_err, sizeof static_err, "sumsq_static: null pointer"); return DBLP_EINVAL; }
    if (((uintptr_t)d_vec & 15) != 0 || ((uintptr_t)d_sumsq & 7) != 0) { snprintf(static_err, sizeof static_err, "sumsq_static: d_vec must be 16-byte and d_sumsq 8-byte aligned"); return DBLP_EINVAL; }
    if (n_elems == 0 || n_elems > STATIC_MAX_ELEMS) { snprintf(static_err, sizeof static_err, "sumsq_static: n_elems must be 1..2^36"); return DBLP_EINVAL; }
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) { snprintf(static_err, sizeof static_err, "sumsq_static: hipSetDevice: %s", hipGetErrorString(e)); return DBLP_EHIP; }
    if (!static_partials_ptr[device]) {         // once per device: where this GPU keeps its copy of the array
        double* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(static_partials));
        if (e != hipSuccess || !p) { snprintf(static_err, sizeof static_err, "sumsq_static: hipGetSymbolAddress: %s", hipGetErrorString(e)); (void)hipGetLastError(); return DBLP_EHIP; }
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e != hipSuccess || cus <= 0) { (void)hipGetLastError(); cus = 256; }
        static_cus[device] = cus;
        static_partials_ptr[device] = p;
    }
    double* partials = static_partials_ptr[device];
    u64 blocks = (n_elems / 4 + 255) / 256;     // the grid rule of dblp_phase_signal, so the two agree to the bit
    const u64 cap = (u64)static_cus[device] * FIN_BLOCKS_PER_CU < STATIC_PARTIALS ? (u64)static_cus[device] * FIN_BLOCKS_PER_CU : STATIC_PARTIALS;
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(sumsq_vec, dim3((u32)blocks), dim3(256), 0, (hipStream_t)stream, d_vec, (u64)n_elems, partials);
    hipLaunchKernelGGL(reduce_partials, dim3(1), dim3(256), 0, (hipStream_t)stream, (const double*)partials, (u32)blocks, d_sumsq);
    e = hipGetLastError();
    if (e != hipSuccess) { snprintf(static_err, sizeof static_err, "sumsq_static: launch: %s", hipGetErrorString(e)); return DBLP_EHIP; }
    static_err[0] = 0;
    return DBLP_OK;
}

extern "C" int dblp_get_bitmap(dblp_ctx* c, uint64_t* d_out) {
    if (!c || !d_out) return DBLP_EINVAL;
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, hipMemcpyAsync(d_out, c->d_bitmap, c->g.W * c->g.words_pw * sizeof(u64), hipMemcpyDeviceToDevice, c->stream));
    return DBLP_OK;
}

extern "C" int dblp_get_counters(dblp_ctx* c, uint64_t h[4]) {
    if (!c || !h) return DBLP_EINVAL;
    if (c->counters_in_mailbox && c->mailbox_seen) {
        // the last finalize mirrored the counters into the host mailbox and the stream has been
        // synchronised since: nothing to launch, nothing to wait for
        h[0] = c->h_mailbox[8];
        h[1] = c->h_mailbox[9] - c->h_mailbox[8];
        h[2] = c->h_mailbox[10];
        h[3] = c->h_mailbox[11];
        return DBLP_OK;
    }
    HIP_TRY(c, hipSetDevice(c->device));
    u64 tmp[C_COUNT];
    hipLaunchKernelGGL(fold_accept_rows, dim3(1), dim3(256), 0, c->stream, c->d_accept_rows, (u32)(2 * ACCEPT_ROWS),
                       c->d_counters);
    LAUNCH_CHECK(c, "get_counters");
    HIP_TRY(c, hipMemcpyAsync(tmp, c->d_counters, sizeof tmp, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    h[0] = tmp[C_ACCEPTED];
    h[1] = tmp[C_CANDIDATES] - tmp[C_ACCEPTED];   // valid arrivals that were not the first copy of their packet
    h[2] = tmp[C_STALE];
    h[3] = tmp[C_INVALID];
    return DBLP_OK;
}

#define PROF_MAX_RECORDS 16384   // brackets kept between two dblp_profile_read calls; more are dropped

extern "C" int dblp_profile_enable(dblp_ctx* c, int on) {
    if (!c) return DBLP_EINVAL;
    if (on) {
        try {
            c->timed->reserve(PROF_MAX_RECORDS);
            c->ev_pool->reserve(2 * PROF_MAX_RECORDS + 64);
        } catch (...) {
            return fail(c, DBLP_ENOMEM, "profile_enable: out of host memory");
        }
    }
    c->profiling = on & ((1 << DBLP_K_COUNT) - 1);
    return DBLP_OK;
}

extern "C" int dblp_profile_read(dblp_ctx* c, int kernel, double* h_total_ms, uint64_t* h_launches) {
    if (!c || !h_total_ms || !h_launches || kernel < 0 || kernel >= DBLP_K_COUNT) return DBLP_EINVAL;
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    double total = 0.0; u64 n = 0;
    size_t kept = 0;                      // compact in place: no allocation on this path
    for (size_t i = 0; i < c->timed->size(); ++i) {
        const dblp_ctx::Timed t = (*c->timed)[i];
        if (t.kernel != kernel) { (*c->timed)[kept++] = t; continue; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) { total += ms; ++n; } else (void)hipGetLastError();
        c->ev_pool->push_back(t.a); c->ev_pool->push_back(t.b);   // within the reserved capacity
    }
    c->timed->resize(kept);
    *h_total_ms = total; *h_launches = n;
    return DBLP_OK;
}

extern "C" int dblp_set_prev_norm(dblp_ctx* c, double norm, int have) {
    if (!c || !(norm >= 0.0)) return DBLP_EINVAL;
    c->prev_norm = norm; c->have_prev = have != 0;
    return DBLP_OK;
}

extern "C" int dblp_get_prev_norm(const dblp_ctx* c, double* h_norm, int* h_have) {
    if (!c || !h_norm || !h_have) return DBLP_EINVAL;
    *h_norm = c->prev_norm; *h_have = c->have_prev;
    return DBLP_OK;
}

extern "C" uint32_t dblp_policy_two_level(int critical, uint32_t p_low_ppm, uint32_t p_high_ppm) {
    return critical ? p_low_ppm : p_high_ppm;
}

extern "C" uint32_t dblp_policy_three_level(double rel_delta, double eta, uint32_t tight_ppm, uint32_t mid_ppm,
                                            uint32_t loose_ppm) {
    if (rel_delta >= eta) return tight_ppm;
    return rel_delta >= 0.5 * eta ? mid_ppm : loose_ppm;
}

extern "C" uint32_t dblp_policy_linear(double rel_delta, double eta, uint32_t lo_ppm, uint32_t hi_ppm) {
    double x = rel_delta / eta;
    if (!(x < 1.0)) x = 1.0;
    const double ppm = (double)hi_ppm - ((double)hi_ppm - (double)lo_ppm) * x;
    return (uint32_t)(floor(ppm / 1000.0 + 0.5)) * 1000u;
}

extern "C" int dblp_clr_init(dblp_clr_state* st, uint32_t p_low_ppm, uint32_t p_high_ppm, uint32_t iters_per_epoch) {
    if (!st || iters_per_epoch == 0 || p_low_ppm > 1000000u || p_high_ppm > 1000000u) return DBLP_EINVAL;
    st->p_low_ppm = p_low_ppm; st->p_high_ppm = p_high_ppm; st->iters_per_epoch = iters_per_epoch;
    st->bound_ppm = p_low_ppm;      // training starts in the critical regime
    st->step = 0;
    return DBLP_OK;
}

extern "C" uint32_t dblp_clr_step(dblp_clr_state* st, int critical) {
    if (st->step % st->iters_per_epoch == 0)      // first iteration of an epoch: re-decide
        st->bound_ppm = critical ? st->p_low_ppm : st->p_high_ppm;
    st->step += 1;
    return st->bound_ppm;
}
