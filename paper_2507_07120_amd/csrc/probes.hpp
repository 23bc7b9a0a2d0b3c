// Ceiling probes for the benchmark: what the part sustains for the two access patterns the attention
// kernels are built on, measured with kernels that do nothing else.
//   stream_read_kernel   a bare streaming read with the launch shape of the GQA kernels (one workgroup of 4
//                        waves per contiguous chunk, the waves taking alternating blocks of 16 x 16-byte loads
//                        per lane): the HBM read rate a kernel with this grid can reach at all;
//   mfma_lds_kernel      16x16x32 bf16 MFMAs whose A operand is fresh data from LDS at every instruction (B in
//                        registers), 8 waves per CU, optionally with one 1 KB non-temporal global read per wave
//                        and 16 MFMAs (256 flop per byte, the MLA path's ratio of matrix work to HBM bytes): the matrix rate a
//                        streaming contraction fed from LDS can sustain on the data it is given (the part
//                        lowers its clock under the switching power of random operands).
#pragma once
#include "common.hpp"

namespace helix {

constexpr int kProbeLoads = 16;                     // 16-byte loads per lane and block
constexpr size_t kProbeBlock = (size_t)kProbeLoads * 1024;

template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint8_t* __restrict__ p, size_t n_blocks, uint32_t* sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t per = (n_blocks + gridDim.x - 1) / gridDim.x;
    size_t b = (size_t)blockIdx.x * per + wave;
    const size_t b1 = min((size_t)(blockIdx.x + 1) * per, n_blocks);
    u32x4 acc = {0, 0, 0, 0};
    for (; b < b1; b += 4) {
        const u32x4* base = reinterpret_cast<const u32x4*>(p + b * kProbeBlock) + lane;
        u32x4 r[kProbeLoads];
#pragma unroll
        for (int j = 0; j < kProbeLoads; j++) r[j] = NT ? __builtin_nontemporal_load(base + j * 64) : base[j * 64];
#pragma unroll
        for (int j = 0; j < kProbeLoads; j++) acc ^= r[j];
    }
    // the loads must not be optimised away; the value is (practically) never the magic one
    const uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (v == 0x9E3779B9u && sink) sink[0] = v;
}

constexpr int kProbeLds = 64 * 1024;                // bytes of operand data cycled through
constexpr int kProbeWaves = 8;

template <bool STREAM>
__global__ __launch_bounds__(kProbeWaves * 64, 1) void mfma_lds_kernel(int iters, const u32x4* __restrict__ data, float* sink,
                                                                      const u32x4* __restrict__ big, uint32_t big_mask)
{
    __shared__ u32x4 lds[kProbeLds / 16];
    for (int i = threadIdx.x; i < kProbeLds / 16; i += blockDim.x) lds[i] = data[i];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 b[8];
#pragma unroll
    for (int i = 0; i < 8; i++) b[i] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 8 + i + 1777) % (kProbeLds / 16)]);
    f32x4 c[8];
#pragma unroll
    for (int j = 0; j < 8; j++) c[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint32_t pos = wave * 8192;
    // one 1 KB read per wave and 16 MFMAs = 256 flop per byte (the bf16 MLA path needs 242 useful flop per latent byte)
    u32x4 g[4], gx = {0, 0, 0, 0};
    uint32_t gpos = (blockIdx.x * kProbeWaves + wave) * 64 + lane;    // in 16-byte units; a step advances by the whole grid
    const uint32_t gstep = gridDim.x * kProbeWaves * 64;
    if (STREAM) {
#pragma unroll
        for (int j = 0; j < 4; j++) { g[j] = __builtin_nontemporal_load(big + (gpos & big_mask)); gpos += gstep; }
    }
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (STREAM && (j & 1) == 0) { gx ^= g[j >> 1]; g[j >> 1] = __builtin_nontemporal_load(big + (gpos & big_mask)); gpos += gstep; }
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, lds[((pos + i * 1024) & (kProbeLds - 1)) / 16 + lane]);
                c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[i], c[i], 0, 0, 0);
            }
            pos += 8192;
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) s += c[j].x + c[j].y + c[j].z + c[j].w;
    if (STREAM) {
#pragma unroll
        for (int j = 0; j < 4; j++) gx ^= g[j];
        s += (float)(gx.x ^ gx.y ^ gx.z ^ gx.w);
    }
    if (s == 1234.5f && sink) sink[0] = s;
}

}  // namespace helix
