// FP8 form of V for the P~V product (Alg. 1 line 16 with an E4M3 matrix product; the paper credits
// the SageAttention2-based kernel with it and gives no formulas, so the definition is this library's):
//   delta_V[b,h,c] = fp32(max_t |V[b,h,t,c]|) / 448 (fp32 division), 0 for a zero channel;
//   V_hat[t,c]     = e4m3(fp32(V[t,c]) / delta_V[c])   (OCP E4M3, round to nearest even).
// Tiles: per (b,h) and key block j, 64*d bytes in the operand order of v_mfma_f32_32x32x64_f8f6f4:
//   [channel tile dt = c/32][half h2][lane = c%32 + 32 g][16 bytes b],
//   key = 64 j + 32 h2 + 8 (b/4) + 4 g + b%4,
// which is the order in which a lane of the attention kernel holds the scores of a tile.  Keys >= N are 0.
#include "common.hpp"

namespace sparge {

namespace {

__global__ void zero_u32_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

constexpr int AMAX_ROWS = 512;  // tokens per workgroup of the maximum pass

// max_t |V[t,c]|: the 15 magnitude bits of fp16/bf16 order like the values, so the maximum is taken
// on the bit patterns; the winner's fp32 bit pattern (non-negative floats order like integers) goes
// into amax_bits with an atomic max.
template <int D, int DT>
__global__ __launch_bounds__(256) void v_absmax_kernel(const uint16_t* __restrict__ V, Shape s,
                                                       uint32_t* __restrict__ amax_bits) {
    constexpr int CPR = D / 8, RPI = 256 / CPR;  // 16-byte chunks per row, rows per pass
    __shared__ uint16_t part[RPI][D];
    const int h = blockIdx.y, b = blockIdx.z;
    const uint16_t* base = V + b * s.sb + h * s.sh;
    const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
    const int row_begin = blockIdx.x * AMAX_ROWS, row_end = min(row_begin + AMAX_ROWS, s.N);
    uint16_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int row = row_begin + r0; row < row_end; row += RPI) {
        const uint4 v = *reinterpret_cast<const uint4*>(base + (long long)row * s.sn + col * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            m[2 * e] = max(m[2 * e], static_cast<uint16_t>(w[e] & 0x7fffu));
            m[2 * e + 1] = max(m[2 * e + 1], static_cast<uint16_t>((w[e] >> 16) & 0x7fffu));
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[r0][col * 8 + e] = m[e];
    __syncthreads();
    if (threadIdx.x < D) {
        uint16_t best = 0;
        for (int r = 0; r < RPI; ++r) best = max(best, part[r][threadIdx.x]);
        const float f = cvt16<DT>(best);
        atomicMax(&amax_bits[((long long)b * s.H + h) * D + threadIdx.x], __float_as_uint(f));
    }
}

template <int D, int DT>
__global__ __launch_bounds__(256) void v_tiles_fp8_kernel(const uint16_t* __restrict__ V, Shape s,
                                                          const uint32_t* __restrict__ amax_bits,
                                                          unsigned char* __restrict__ tiles,
                                                          float* __restrict__ v_scale) {
    constexpr int PITCH = D + 8;  // 16-bit elements; keeps the column reads spread over LDS banks
    __shared__ uint16_t lds[BK * PITCH];
    __shared__ float delta[D];
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const long long bh = (long long)b * s.H + h;
    const uint16_t* base = V + b * s.sb + h * s.sh;
    constexpr int CPR = D / 8;
    if (threadIdx.x < D) {
        const float dl = __uint_as_float(amax_bits[bh * D + threadIdx.x]) / 448.0f;
        delta[threadIdx.x] = dl;
        if (j == 0) v_scale[bh * D + threadIdx.x] = dl;
    }
    for (int idx = threadIdx.x; idx < BK * CPR; idx += 256) {
        const int row = idx / CPR, col = idx % CPR;
        const int key = j * BK + row;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (key < s.N) v = *reinterpret_cast<const uint4*>(base + (long long)key * s.sn + col * 8);
        *reinterpret_cast<uint4*>(&lds[row * PITCH + col * 8]) = v;
    }
    __syncthreads();
    unsigned char* out = tiles + (bh * s.Tn + j) * (long long)(D * BK);
    for (int q = threadIdx.x; q < D * 4; q += 256) {  // one 16-byte piece each
        const int dt = q / 128, h2 = (q / 64) & 1, lane = q & 63;
        const int c = dt * 32 + (lane & 31), g = lane >> 5;
        const float dl = delta[c];
        uint32_t w[4];
#pragma unroll
        for (int b4 = 0; b4 < 4; ++b4) {
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int key = 32 * h2 + 8 * b4 + 4 * g + e;
                const float v = cvt16<DT>(lds[key * PITCH + c]);
                x[e] = dl > 0.f ? v / dl : 0.f;
            }
            int word = 0;
            word = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], word, false);
            word = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], word, true);
            w[b4] = static_cast<uint32_t>(word);
        }
        *reinterpret_cast<uint4*>(out + q * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

}  // namespace

hipError_t launch_v_tiles_fp8(const void* V, const Shape& s, unsigned char* tiles, float* v_scale,
                              uint32_t* amax_bits, hipStream_t st) {
    const uint16_t* X = static_cast<const uint16_t*>(V);
    const int n = s.B * s.H * s.d;
    hipLaunchKernelGGL(zero_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, amax_bits, n);
    dim3 g1((s.N + AMAX_ROWS - 1) / AMAX_ROWS, s.H, s.B), g2(s.Tn, s.H, s.B);
#define CALL(D, DT)                                                                                          \
    {                                                                                                        \
        hipLaunchKernelGGL((v_absmax_kernel<D, DT>), g1, dim3(256), 0, st, X, s, amax_bits);                \
        hipLaunchKernelGGL((v_tiles_fp8_kernel<D, DT>), g2, dim3(256), 0, st, X, s, amax_bits, tiles, v_scale); \
    }
    if (s.d == 64 && s.dtype == SPARGE_F16) CALL(64, SPARGE_F16)
    else if (s.d == 64 && s.dtype == SPARGE_BF16) CALL(64, SPARGE_BF16)
    else if (s.d == 128 && s.dtype == SPARGE_F16) CALL(128, SPARGE_F16)
    else if (s.d == 128 && s.dtype == SPARGE_BF16) CALL(128, SPARGE_BF16)
    else return hipErrorInvalidValue;
#undef CALL
    return hipGetLastError();
}

}  // namespace sparge
