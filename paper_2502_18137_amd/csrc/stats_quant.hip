// Bandwidth-bound passes over Q and K (Alg. 1 lines 3-5):
//   block_stats  : one read of a 128-row Q block or 64-row K block -> pooled channel sums/means,
//                  block self-similarity CosSim, and (Q only) the per-block INT8 quantization.
//   k_mean       : per-(batch,head) token mean of K from the block sums.
//   quant_k      : second read of K -> INT8 of (K - mean) with per-block scales.
//   v_tiles      : V re-tiled per 64-key block into the operand order of the P~V matrix product.
// Thread mapping: a token row of d 16-bit values is covered by d/8 adjacent lanes holding 16 bytes
// each, so every global load instruction moves whole 128/256-byte rows; a lane keeps the same 8
// channels for all its rows, which makes channel sums per-lane accumulations.
#include "common.hpp"

namespace sparge {

namespace {

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}

// Cross-lane reductions on the vector ALU (DPP row operations and the lane-swap instructions, row_xchg and
// the swaps below) instead of ds_bpermute: the block statistics spend their time in the LDS pipeline otherwise.
// {own, partner's} in some order for the lanes ^16 or ^32: v_permlane16_swap / v_permlane32_swap of a register
// with its copy leave one of the two values in each result, which is all a commutative reduction needs
template <int PARTNER>
__device__ __forceinline__ void swap_pair(uint32_t v, uint32_t& a, uint32_t& b) {
    static_assert(PARTNER == 16 || PARTNER == 32, "no such exchange");
    if constexpr (PARTNER == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        a = r[0], b = r[1];
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        a = r[0], b = r[1];
    }
}
// v + (v of the partner lane)
template <int PARTNER>
__device__ __forceinline__ double add_partner(double v) {
    const uint32_t lo = static_cast<uint32_t>(__double2loint(v)), hi = static_cast<uint32_t>(__double2hiint(v));
    if constexpr (PARTNER == 16 || PARTNER == 32) {
        uint32_t l0, l1, h0, h1;
        swap_pair<PARTNER>(lo, l0, l1);
        swap_pair<PARTNER>(hi, h0, h1);
        return __hiloint2double(static_cast<int>(h0), static_cast<int>(l0)) +
               __hiloint2double(static_cast<int>(h1), static_cast<int>(l1));
    } else {
        return v + __hiloint2double(static_cast<int>(row_xchg<PARTNER>(hi)), static_cast<int>(row_xchg<PARTNER>(lo)));
    }
}
template <int PARTNER>
__device__ __forceinline__ float max_partner(float v) {
    if constexpr (PARTNER == 16 || PARTNER == 32) {
        uint32_t a, b;
        swap_pair<PARTNER>(__float_as_uint(v), a, b);
        return fmaxf(__uint_as_float(a), __uint_as_float(b));
    } else {
        return fmaxf(v, __uint_as_float(row_xchg<PARTNER>(__float_as_uint(v))));
    }
}
// Two values reduced at the price of one: the lanes whose number has bit PARTNER clear end up with
// a + (a of lane ^ PARTNER), the others with b + (b of lane ^ PARTNER).
template <int PARTNER>
__device__ __forceinline__ double scatter_sum(double a, double b) {
    if constexpr (PARTNER == 16 || PARTNER == 32) {
        // the swap moves a's upper half (odd rows) against b's lower half (even rows): no copies, no selects
        uint32_t l0, l1, h0, h1;
        if constexpr (PARTNER == 16) {
            const auto rl = __builtin_amdgcn_permlane16_swap(static_cast<uint32_t>(__double2loint(a)),
                                                             static_cast<uint32_t>(__double2loint(b)), false, false);
            const auto rh = __builtin_amdgcn_permlane16_swap(static_cast<uint32_t>(__double2hiint(a)),
                                                             static_cast<uint32_t>(__double2hiint(b)), false, false);
            l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
        } else {
            const auto rl = __builtin_amdgcn_permlane32_swap(static_cast<uint32_t>(__double2loint(a)),
                                                             static_cast<uint32_t>(__double2loint(b)), false, false);
            const auto rh = __builtin_amdgcn_permlane32_swap(static_cast<uint32_t>(__double2hiint(a)),
                                                             static_cast<uint32_t>(__double2hiint(b)), false, false);
            l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
        }
        return __hiloint2double(static_cast<int>(h0), static_cast<int>(l0)) +
               __hiloint2double(static_cast<int>(h1), static_cast<int>(l1));
    } else {
        static_assert(PARTNER == 1 || PARTNER == 2, "a true lane ^ PARTNER exchange is needed here");
        const bool up = (threadIdx.x & PARTNER) != 0;
        const double keep = up ? b : a, send = up ? a : b;
        return keep + __hiloint2double(static_cast<int>(row_xchg<PARTNER>(static_cast<uint32_t>(__double2hiint(send)))),
                                       static_cast<int>(row_xchg<PARTNER>(static_cast<uint32_t>(__double2loint(send)))));
    }
}
// v summed (maximized) over the aligned group of G lanes, G = 8, 16 or 64; every lane gets the result
template <int G>
__device__ __forceinline__ double group_sum(double v) {
    v = add_partner<1>(v);
    v = add_partner<2>(v);
    v = add_partner<7>(v);  // the quads agree by now: the mirrors do
    if constexpr (G >= 16) v = add_partner<15>(v);
    if constexpr (G == 64) {
        v = add_partner<16>(v);
        v = add_partner<32>(v);
    }
    return v;
}
template <int G>
__device__ __forceinline__ float group_max(float v) {
    v = max_partner<1>(v);
    v = max_partner<2>(v);
    v = max_partner<7>(v);
    if constexpr (G >= 16) v = max_partner<15>(v);
    return v;
}
template <int DT>
__device__ __forceinline__ void unpack8(const uint4& raw, float (&f)[8]) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = cvt16<DT>(static_cast<uint16_t>(w[e] & 0xFFFFu));
        f[2 * e + 1] = cvt16<DT>(static_cast<uint16_t>(w[e] >> 16));
    }
}

// x_hat = rint_half_even(x * r) packed as 8 int8 (fp32 multiply, single rounding, no contraction).
// Adding 1.5 * 2^23 to the rounded product rounds it to an integer, to nearest even, and leaves that
// integer in two's complement in the low mantissa bits (|x * r| <= 127): the low byte is x_hat.
__device__ __forceinline__ uint2 quant8(const float (&f)[8], float r) {
    uint32_t y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = __float_as_uint(f[e] * r + 12582912.0f);
    uint32_t out[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t lo = __builtin_amdgcn_perm(y[4 * h + 1], y[4 * h + 0], 0x0c0c0400u);  // bytes {y0, y1, 0, 0}
        const uint32_t hi = __builtin_amdgcn_perm(y[4 * h + 3], y[4 * h + 2], 0x0c0c0400u);
        out[h] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    }
    return make_uint2(out[0], out[1]);
}

// One workgroup (256 threads) per block of ROWS tokens.
//   STATS: pooled sums + self-similarity are produced.  KSIDE: sums go out transposed and unscaled
//   ([B,H,d,Tn], needed exactly for the K mean), otherwise means go out as [B,H,Tm,d].
//   QUANT: the block is quantized in place from registers (Q side only).
template <int D, int DT, int ROWS, bool KSIDE, bool QUANT>
__global__ __launch_bounds__(256) void block_stats_kernel(const uint16_t* __restrict__ X, Shape s,
                                                           double* __restrict__ pooled,
                                                           double* __restrict__ sim,
                                                           int8_t* __restrict__ Xq,
                                                           float* __restrict__ scale) {
    constexpr int LPR = D / 8;        // lanes per token row
    constexpr int RPW = 64 / LPR;     // rows per wave-wide load
    constexpr int RPS = 4 * RPW;      // rows per sweep of the 4 waves
    constexpr int NL = ROWS / RPS;    // loads per lane
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int T = KSIDE ? s.Tn : s.Tm;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cchunk = lane % LPR, rsub = lane / LPR;
    const int row0 = t * ROWS;
    const uint16_t* base = X + b * s.sb + h * s.sh;

    __shared__ double lds_raw[4][D];
    __shared__ double lds_hat[4][D];
    __shared__ float lds_amax[4];
    __shared__ double lds_sq[4];
    __shared__ double lds_inv[4][NL * RPW];
    static_assert(NL * RPW <= 64, "a wave's rows must fit one lane each");

    uint4 raw[NL];
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        const int r = row0 + n * RPS + wave * RPW + rsub;
        raw[n] = make_uint4(0u, 0u, 0u, 0u);
        if (r < s.N) raw[n] = *reinterpret_cast<const uint4*>(base + (long long)r * s.sn + cchunk * 8);
    }

    double sraw[8], shat[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sraw[e] = shat[e] = 0.0;
    float amax = 0.f;
    // squared norm of every row of this wave (NL * RPW of them), one value per row in LDS
    double nsq[NL];
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        float f[8];
        unpack8<DT>(raw[n], f);
        nsq[n] = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double x = static_cast<double>(f[e]);
            nsq[n] = __builtin_fma(x, x, nsq[n]);  // x * x is exact in fp64 (16-bit inputs): same result as mul + add
            amax = fmaxf(amax, fabsf(f[e]));
        }
    }
    // The LPR lanes of a row are summed with the first steps halving the number of values: after them
    // the lane with bits (p, q) = (lane & 1, lane >> 1 & 1) works on the rows n = i + NQ q + NH p only.
    {
        static_assert(NL == 2 || NL == 4 || NL == 8, "row count per lane");
        constexpr int NH = NL / 2, NQ = NL >= 4 ? NL / 4 : 1;
        double w1[NH];
#pragma unroll
        for (int i = 0; i < NH; ++i) w1[i] = scatter_sum<1>(nsq[i], nsq[i + NH]);
        const int p = lane & 1, q = (lane >> 1) & 1;
        if constexpr (NL >= 4) {
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                double w = scatter_sum<2>(w1[i], w1[i + NQ]);
                w = add_partner<4>(w);  // lanes of a quad hold different rows from here on: true ^4, ^8 only
                if constexpr (LPR == 16) w = add_partner<8>(w);
                if (cchunk < 4) lds_inv[wave][(i + NQ * q + NH * p) * RPW + rsub] = w;
            }
        } else {
            double w = add_partner<2>(w1[0]);
            w = add_partner<4>(w);
            if constexpr (LPR == 16) w = add_partner<8>(w);
            if (cchunk < 2) lds_inv[wave][p * RPW + rsub] = w;
        }
    }
    // 1 / |row|: the fp64 square root and division are the expensive part, so each row's is evaluated by
    // one lane only (a wave owns at most 64 rows) and handed to the lanes of that row through LDS
    // (the exchange stays inside a wave, whose LDS accesses complete in program order: the wave barriers
    // only keep the compiler from moving accesses across the hand-over points)
    __builtin_amdgcn_wave_barrier();
    if (lane < NL * RPW) {
        const double nsq = lds_inv[wave][lane];
        lds_inv[wave][lane] = nsq > 0.0 ? 1.0 / sqrt(nsq) : 0.0;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        float f[8];
        unpack8<DT>(raw[n], f);
        const double inv = lds_inv[wave][n * RPW + rsub];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double x = static_cast<double>(f[e]);
            sraw[e] += x;
            shat[e] = __builtin_fma(x, inv, shat[e]);
        }
    }
    // Combine the lanes that hold the same channels (different rows of the wave-wide load).  Lane bits 5
    // and 4 each halve the 16 sums a lane works on: lane bit 5 selects raw sums / normalized sums, lane
    // bit 4 the channels 0..3 / 4..7 of the lane's chunk.  (d = 64: lane bit 3 is reduced last, in full.)
    {
        double h8[8], h4[4];
#pragma unroll
        for (int e = 0; e < 8; ++e) h8[e] = scatter_sum<32>(sraw[e], shat[e]);
#pragma unroll
        for (int e = 0; e < 4; ++e) h4[e] = scatter_sum<16>(h8[e], h8[e + 4]);
        if constexpr (LPR == 8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) h4[e] = add_partner<8>(h4[e]);
        }
        amax = max_partner<32>(amax);
        amax = max_partner<16>(amax);
        if constexpr (LPR == 8) amax = max_partner<8>(amax);
        amax = group_max<LPR>(amax);
        if (LPR == 16 || (lane & 8) == 0) {
            double* dst = (lane & 32) ? lds_hat[wave] : lds_raw[wave];
            const int c0 = cchunk * 8 + ((lane & 16) ? 4 : 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[c0 + e] = h4[e];
        }
    }
    if (lane == 0) lds_amax[wave] = amax;
    __syncthreads();

    const int cnt = min(ROWS, s.N - row0);
    const long long bh = (long long)b * s.H + h;
    if (threadIdx.x < D) {
        const int c = threadIdx.x;
        const double rsum = ((lds_raw[0][c] + lds_raw[1][c]) + lds_raw[2][c]) + lds_raw[3][c];
        const double hsum = ((lds_hat[0][c] + lds_hat[1][c]) + lds_hat[2][c]) + lds_hat[3][c];
        if (KSIDE) pooled[(bh * D + c) * T + t] = rsum;
        else pooled[(bh * T + t) * D + c] = rsum / static_cast<double>(cnt);
        double sq = hsum * hsum;
        sq = group_sum<64>(sq);
        if (lane == 0) lds_sq[wave] = sq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = lds_sq[0];
        if (D > 64) tot += lds_sq[1];
        sim[bh * T + t] = tot / (static_cast<double>(cnt) * static_cast<double>(cnt));
    }

    if constexpr (QUANT) {
        const float bmax = fmaxf(fmaxf(lds_amax[0], lds_amax[1]), fmaxf(lds_amax[2], lds_amax[3]));
        const float r = bmax > 0.f ? 127.0f / bmax : 0.f;
        if (threadIdx.x == 0) scale[bh * T + t] = bmax > 0.f ? bmax / 127.0f : 0.f;
        int8_t* qbase = Xq + bh * (long long)s.N * D;
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            const int rr = row0 + n * RPS + wave * RPW + rsub;
            if (rr < s.N) {
                float f[8];
                unpack8<DT>(raw[n], f);
                *reinterpret_cast<uint2*>(qbase + (long long)rr * D + cchunk * 8) = quant8(f, r);
            }
        }
    }
}

// One workgroup per (b, h, 4 channels): wave w reduces channel 4*blockIdx.x + w; lanes stride over the
// key blocks and combine in a fixed butterfly, so the sum does not depend on scheduling.
template <int D>
__global__ __launch_bounds__(256) void k_mean_kernel(const double* __restrict__ ksum_t, Shape s,
                                                      float* __restrict__ k_mean) {
    const long long bh = (long long)blockIdx.z * s.H + blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 4 + wave;
    const double* row = ksum_t + (bh * D + c) * s.Tn;
    double acc = 0.0;
    for (int j = lane; j < s.Tn; j += 64) acc += row[j];
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) acc += shfl_xor_f64(acc, m);
    if (lane == 0) k_mean[bh * D + c] = static_cast<float>(acc / static_cast<double>(s.N));
}

// One workgroup per 64-row K block: K' = fp32(K) - mean, per-block amax, INT8.
template <int D, int DT>
__global__ __launch_bounds__(256) void quant_k_kernel(const uint16_t* __restrict__ K, Shape s,
                                                       const float* __restrict__ k_mean,
                                                       int8_t* __restrict__ Kq, float* __restrict__ k_scale) {
    constexpr int LPR = D / 8, RPW = 64 / LPR, RPS = 4 * RPW, NL = BK / RPS;
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cchunk = lane % LPR, rsub = lane / LPR;
    const int row0 = t * BK;
    const long long bh = (long long)b * s.H + h;
    const uint16_t* base = K + b * s.sb + h * s.sh;
    __shared__ float lds_amax[4];

    float mean[8];
    {
        const float4 m0 = *reinterpret_cast<const float4*>(k_mean + bh * D + cchunk * 8);
        const float4 m1 = *reinterpret_cast<const float4*>(k_mean + bh * D + cchunk * 8 + 4);
        mean[0] = m0.x; mean[1] = m0.y; mean[2] = m0.z; mean[3] = m0.w;
        mean[4] = m1.x; mean[5] = m1.y; mean[6] = m1.z; mean[7] = m1.w;
    }
    float x[NL][8];
    float amax = 0.f;
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        const int r = row0 + n * RPS + wave * RPW + rsub;
        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
        const bool ok = r < s.N;
        if (ok) raw = *reinterpret_cast<const uint4*>(base + (long long)r * s.sn + cchunk * 8);
        unpack8<DT>(raw, x[n]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x[n][e] = ok ? x[n][e] - mean[e] : 0.f;
            amax = fmaxf(amax, fabsf(x[n][e]));
        }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m));
    if (lane == 0) lds_amax[wave] = amax;
    __syncthreads();
    const float bmax = fmaxf(fmaxf(lds_amax[0], lds_amax[1]), fmaxf(lds_amax[2], lds_amax[3]));
    const float r = bmax > 0.f ? 127.0f / bmax : 0.f;
    if (threadIdx.x == 0) k_scale[bh * s.Tn + t] = bmax > 0.f ? bmax / 127.0f : 0.f;
    int8_t* qbase = Kq + bh * (long long)s.N * D;
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        const int rr = row0 + n * RPS + wave * RPW + rsub;
        if (rr < s.N) *reinterpret_cast<uint2*>(qbase + (long long)rr * D + cchunk * 8) = quant8(x[n], r);
    }
}

// One workgroup per 64-key block: tile[c][slot] = V[key(slot)][c], 64 slots per channel row.
// Within each group of 16 keys the slot order is {0..3, 8..11, 4..7, 12..15}: the order in which
// the 32x32 MFMA accumulator of S^T hands a lane its keys, so P~ feeds the P~V product from
// registers.  Keys >= N are written as zeros.
template <int D>
__global__ __launch_bounds__(256) void v_tiles_kernel(const uint16_t* __restrict__ V, Shape s,
                                                       uint16_t* __restrict__ tiles) {
    constexpr int PITCH = D + 8;  // 16-bit elements; keeps the column reads spread over LDS banks
    __shared__ uint16_t lds[BK * PITCH];
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const long long bh = (long long)b * s.H + h;
    const uint16_t* base = V + b * s.sb + h * s.sh;
    constexpr int CPR = D / 8;  // 16-byte chunks per key row
    for (int idx = threadIdx.x; idx < BK * CPR; idx += 256) {
        const int row = idx / CPR, col = idx % CPR;
        const int key = j * BK + row;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (key < s.N) v = *reinterpret_cast<const uint4*>(base + (long long)key * s.sn + col * 8);
        *reinterpret_cast<uint4*>(&lds[row * PITCH + col * 8]) = v;
    }
    __syncthreads();
    uint16_t* out = tiles + (bh * s.Tn + j) * (long long)(D * BK);
    for (int idx = threadIdx.x; idx < D * 8; idx += 256) {
        const int c = idx / 8, sc = idx % 8;  // channel row, chunk of 8 slots
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t pair = 0;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int slot = sc * 8 + e2 * 2 + q;
                const int g = slot >> 4, sl = slot & 15;
                const int key = g * 16 + 8 * ((sl & 7) >> 2) + 4 * (sl >> 3) + (sl & 3);
                pair |= static_cast<uint32_t>(lds[key * PITCH + c]) << (16 * q);
            }
            w[e2] = pair;
        }
        *reinterpret_cast<uint4*>(out + c * BK + sc * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

}  // namespace

#define SPARGE_DISPATCH_D_DT(s, CALL)                                              \
    if ((s).d == 64 && (s).dtype == SPARGE_F16) { CALL(64, SPARGE_F16) }           \
    else if ((s).d == 64 && (s).dtype == SPARGE_BF16) { CALL(64, SPARGE_BF16) }    \
    else if ((s).d == 128 && (s).dtype == SPARGE_F16) { CALL(128, SPARGE_F16) }    \
    else if ((s).d == 128 && (s).dtype == SPARGE_BF16) { CALL(128, SPARGE_BF16) }  \
    else return hipErrorInvalidValue;

hipError_t launch_block_stats_q(const void* Q, const Shape& s, double* pooled_q, double* sim_q,
                                int8_t* Qq, float* q_scale, hipStream_t st) {
    dim3 grid(s.Tm, s.H, s.B);
    const uint16_t* X = static_cast<const uint16_t*>(Q);
#define CALL(D, DT)                                                                                   \
    if (Qq) hipLaunchKernelGGL((block_stats_kernel<D, DT, BQ, false, true>), grid, dim3(256), 0, st,  \
                               X, s, pooled_q, sim_q, Qq, q_scale);                                   \
    else hipLaunchKernelGGL((block_stats_kernel<D, DT, BQ, false, false>), grid, dim3(256), 0, st,    \
                            X, s, pooled_q, sim_q, Qq, q_scale);
    SPARGE_DISPATCH_D_DT(s, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_block_stats_k(const void* K, const Shape& s, double* ksum_t, double* sim_k, hipStream_t st) {
    dim3 grid(s.Tn, s.H, s.B);
    const uint16_t* X = static_cast<const uint16_t*>(K);
#define CALL(D, DT)                                                                              \
    hipLaunchKernelGGL((block_stats_kernel<D, DT, BK, true, false>), grid, dim3(256), 0, st, X,  \
                       s, ksum_t, sim_k, (int8_t*)nullptr, (float*)nullptr);
    SPARGE_DISPATCH_D_DT(s, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_k_mean(const double* ksum_t, const Shape& s, float* k_mean, hipStream_t st) {
    dim3 grid(s.d / 4, s.H, s.B);
    if (s.d == 64) hipLaunchKernelGGL((k_mean_kernel<64>), grid, dim3(256), 0, st, ksum_t, s, k_mean);
    else hipLaunchKernelGGL((k_mean_kernel<128>), grid, dim3(256), 0, st, ksum_t, s, k_mean);
    return hipGetLastError();
}

hipError_t launch_quant_k(const void* K, const Shape& s, const float* k_mean, int8_t* Kq, float* k_scale,
                          hipStream_t st) {
    dim3 grid(s.Tn, s.H, s.B);
    const uint16_t* X = static_cast<const uint16_t*>(K);
#define CALL(D, DT) \
    hipLaunchKernelGGL((quant_k_kernel<D, DT>), grid, dim3(256), 0, st, X, s, k_mean, Kq, k_scale);
    SPARGE_DISPATCH_D_DT(s, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_v_tiles(const void* V, const Shape& s, uint16_t* v_tiles, hipStream_t st) {
    dim3 grid(s.Tn, s.H, s.B);
    const uint16_t* X = static_cast<const uint16_t*>(V);
    if (s.d == 64) hipLaunchKernelGGL((v_tiles_kernel<64>), grid, dim3(256), 0, st, X, s, v_tiles);
    else hipLaunchKernelGGL((v_tiles_kernel<128>), grid, dim3(256), 0, st, X, s, v_tiles);
    return hipGetLastError();
}

}  // namespace sparge
