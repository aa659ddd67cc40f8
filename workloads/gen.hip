/*
 * Seeded synthetic-input generator, device side (gfx950).
 *
 * Device twin of dblp_gen_grad_fill() in gen.c: the same integer recipe
 * (SplitMix64 output function, twelve 16-bit fields, one exact int->float
 * conversion, one IEEE multiply), so the bits match the CPU generator.  It
 * exists because the largest workloads (tens of billions of values) cannot be
 * generated on the host and shipped over PCIe in reasonable time.  Inputs
 * only: none of the protocol's arithmetic lives here.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL
#define TAILSALT 0xD1B54A32D192ED03ULL

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27; x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

__device__ __forceinline__ uint32_t fields16(uint64_t h) {
    return (uint32_t)(h & 0xFFFF) + (uint32_t)((h >> 16) & 0xFFFF) +
           (uint32_t)((h >> 32) & 0xFFFF) + (uint32_t)(h >> 48);
}

__global__ __launch_bounds__(256) void grad_fill_kernel(float* __restrict__ out, uint64_t e0,
                                                        uint64_t n, uint64_t key, float scale,
                                                        uint32_t tail_ppm, float tail_mul) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t e = e0 + i;
        uint32_t s = fields16(mix64(key + (3 * e + 0) * GOLDEN)) +
                     fields16(mix64(key + (3 * e + 1) * GOLDEN)) +
                     fields16(mix64(key + (3 * e + 2) * GOLDEN));
        int32_t z = 2 * (int32_t)s - 12 * 65535;
        float v = (float)z * scale;
        if (tail_ppm) {
            uint64_t t = mix64((key ^ TAILSALT) + e * GOLDEN) >> 32;
            if (((t * 1000000ULL) >> 32) < tail_ppm) v = v * tail_mul;
        }
        out[i] = v;
    }
}

/* d_out: device pointer, n floats, owned by the caller.  Asynchronous on `stream`.
   Returns 0 or the hipError_t of the launch. */
extern "C" int dblp_gen_hip_grad_fill(float* d_out, uint64_t e0, uint64_t n, uint64_t key,
                                      float scale, uint32_t tail_ppm, float tail_mul,
                                      void* stream) {
    if (n == 0) return 0;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(grad_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       d_out, e0, n, key, scale, tail_ppm, tail_mul);
    return (int)hipGetLastError();
}

/* The simulated sender's answer to a retransmit list: entry i = (worker << 32) | seq names a
   packet, slot_of[worker * n_pkts + seq] is where that packet sits in the wire buffer, and the
   resent packet is delivered from there (a retransmitted packet is byte-identical to the
   original).  Input plumbing only. */
__global__ __launch_bounds__(256) void resend_slots_kernel(const uint64_t* __restrict__ list, uint64_t n,
                                                           const uint32_t* __restrict__ slot_of, uint64_t n_pkts,
                                                           uint32_t* __restrict__ out_slots) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t e = list[i];
        out_slots[i] = slot_of[(e >> 32) * n_pkts + (e & 0xFFFFFFFFULL)];
    }
}

extern "C" int dblp_gen_hip_resend_slots(const uint64_t* d_list, uint64_t n, const uint32_t* d_slot_of,
                                         uint64_t n_pkts, uint32_t* d_out_slots, void* stream) {
    if (n == 0) return 0;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(resend_slots_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       d_list, n, d_slot_of, n_pkts, d_out_slots);
    return (int)hipGetLastError();
}
