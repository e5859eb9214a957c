// Sparse flash loop with the stage-2 filter (Alg. 1 lines 7-20; Sec. 3.1, 3.3, 3.4) for gfx950.
//
// Work decomposition: one workgroup of 2 waves per Q block (128 rows); a wave owns 64 query rows =
// two 32-row groups I_w, so the stage-2 decision is wave-uniform per group.  Both matrix products
// put the queries on the N side of a 32x32 MFMA:
//     S^T  (keys x queries) = K_hat (A, from LDS)  x  Q_hat^T (B, registers, loaded once)
//     O^T  (d    x queries) = V^T   (A, from LDS)  x  P~^T    (B, registers)
// In the 32x32 accumulator layout a lane then holds one query and 16 keys (or channels), so row
// max / row sum are in-lane reductions plus one exchange with lane^32, every per-row statistic
// (m, l, rescale factor) is a per-lane scalar, and P~ goes from the S accumulator into the P~V
// operand without leaving registers.  The accumulator hands a lane keys {0-3, 8-11} (lanes < 32)
// or {4-7, 12-15} (lanes >= 32) of each group of 16; the V tiles in memory are stored in exactly
// that slot order (see v_tiles_kernel), which is legal because a contraction index may be permuted
// as long as both operands agree.
#include "common.hpp"

namespace sparge {

namespace {

constexpr float LOG2E = 1.4426950408889634f;

template <int DT>
struct PV;
template <>
struct PV<SPARGE_F16> {
    typedef v8h vec;
    static __device__ __forceinline__ v16f mfma(vec a, vec b, v16f c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec pack(const float* p) {
        vec r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = static_cast<_Float16>(p[e]);
        return r;
    }
};
template <>
struct PV<SPARGE_BF16> {
    typedef v8bf vec;
    static __device__ __forceinline__ v16f mfma(vec a, vec b, v16f c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec pack(const float* p) {
        vec r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = static_cast<__bf16>(p[e]);
        return r;
    }
};

// The value held by the lane 32 positions away, combined with the own one (v_permlane32_swap).
__device__ __forceinline__ float max_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16-byte global -> LDS copy that bypasses registers (LDS-DMA): every lane names its own global
// source, the wave's 64 chunks land contiguously at the wave-uniform LDS address in M0 + lane * 16.
// Issued through inline assembly on purpose: the compiler then does not know that the copy writes
// LDS and so does not stall the next LDS read until the copy has landed; the kernel waits for its
// copies itself (dma_wait) right before the barrier that publishes the tile.
__device__ __forceinline__ void dma16(const void* gsrc, const void* lds_base) {
    const uint32_t lds_addr =
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void*)(lds_base)));
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gsrc), "s"(lds_addr)
                 : "memory");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// LDS tiles are unpadded; bank conflicts of the 16-byte operand reads are avoided by XOR-ing the
// 16-byte chunk index of a row with a few row bits (applied on the global side of the copy).
template <int ROW_BYTES>
__device__ __forceinline__ int swz(int row) {
    return ROW_BYTES == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

// NG = 32-row query groups per wave (1 or 2); the workgroup always covers one 128-row Q block.
template <int D, int DT, bool CAUSAL, int NG>
__global__ __launch_bounds__(64 * (4 / NG), 2) void attn_kernel(
    const int8_t* __restrict__ Qq, const int8_t* __restrict__ Kq, const float* __restrict__ q_scale,
    const float* __restrict__ k_scale, const uint16_t* __restrict__ v_tiles, uint16_t* __restrict__ O,
    const uint8_t* __restrict__ mask, Shape s, HeadParams lambda_h, float sm_scale, int n_work, int per_xcd,
    unsigned long long* __restrict__ stats) {
    constexpr int NW = 4 / NG;          // waves per workgroup
    constexpr int NSTEP = D / 32;       // int8 MFMA steps along d
    constexpr int NDT = D / 32;         // 32-channel output tiles
    constexpr int K_BYTES = BK * D;     // K_hat tile
    constexpr int V_BYTES = D * BK * 2; // V^T tile
    constexpr int K_CPR = D / 16;       // 16-byte chunks per K_hat row
    constexpr int K_DMA = K_BYTES / 1024, V_DMA = V_BYTES / 1024;  // wave-wide copies per tile
    typedef PV<DT> pv;

    __shared__ __align__(1024) unsigned char Ks[2][K_BYTES];
    __shared__ __align__(1024) unsigned char Vs[2][V_BYTES];
    __shared__ uint16_t list[SPARGE_MAX_TN];
    __shared__ int list_cnt;

    // XCD-aware work order: consecutive workgroup ids land on different XCDs, so give each XCD a
    // contiguous range of (head, Q block) items and let its L2 serve that head's K/V tiles.
    const int wg = blockIdx.x;
    const int work = (wg % 8) * per_xcd + wg / 8;
    if (work >= n_work) return;
    const int bh = work / s.Tm;
    const int i = CAUSAL ? (s.Tm - 1 - work % s.Tm) : (work % s.Tm);  // causal: longest rows first
    const int b = bh / s.H, h = bh % s.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int l32 = lane & 31, hl = lane >> 5;

    const int jmax = CAUSAL ? min(s.Tn, (i * BQ + BQ - 1) / BK + 1) : s.Tn;
    // ---- kept key blocks of this row, in ascending order -------------------------------------
    if (wave == 0) {
        const uint8_t* mrow = mask ? mask + ((long long)bh * s.Tm + i) * s.Tn : nullptr;
        int cnt = 0;
        for (int base = 0; base < jmax; base += 64) {
            const int j = base + lane;
            const bool keep = j < jmax && (mrow ? mrow[j] != 0 : true);
            const unsigned long long bal = __ballot(keep);
            if (keep) list[cnt + __popcll(bal & ((1ull << lane) - 1ull))] = static_cast<uint16_t>(j);
            cnt += __popcll(bal);
        }
        if (lane == 0) list_cnt = cnt;
    }
    __syncthreads();
    const int cnt = list_cnt;

    const int8_t* kbase = Kq + (long long)bh * s.N * D;
    const uint16_t* vbase = v_tiles + (long long)bh * s.Tn * (D * BK);

    // asynchronous copy of tile j into buffer `buf` (each wave moves its share of 1 KB pieces)
    auto copy_tile = [&](int j, int buf) {
#pragma unroll
        for (int q = wave; q < K_DMA; q += NW) {
            const int p = q * 64 + lane;
            const int row = p / K_CPR, phys = p % K_CPR;
            const int key = min(j * BK + row, s.N - 1);  // rows past N repeat the last key; they are masked
            dma16(kbase + (long long)key * D + ((phys ^ swz<D>(row)) * 16), &Ks[buf][q * 1024]);
        }
        const unsigned char* vt = reinterpret_cast<const unsigned char*>(vbase + (long long)j * (D * BK));
#pragma unroll
        for (int q = wave; q < V_DMA; q += NW) {
            const int p = q * 64 + lane;
            const int row = p / 8, phys = p % 8;
            dma16(vt + row * 128 + ((phys ^ swz<128>(row)) * 16), &Vs[buf][q * 1024]);
        }
    };
    if (cnt > 0) copy_tile(__builtin_amdgcn_readfirstlane(list[0]), 0);

    // ---- Q_hat fragments (B operand), resident for the whole loop ----------------------------
    const int qrow0 = i * BQ + wave * (32 * NG);
    v4i qf[NG][NSTEP];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int row = qrow0 + g * 32 + l32;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            qf[g][st] = v4i{0, 0, 0, 0};
            if (row < s.N)
                qf[g][st] = *reinterpret_cast<const v4i*>(Qq + ((long long)bh * s.N + row) * D + st * 32 + hl * 16);
        }
    }
    // Pin the Q_hat loads' completion here: otherwise the compiler waits for them at their first use
    // inside the loop with vmcnt(0), which would also wait for the tile copy just issued there.
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) asm volatile("" ::"v"(qf[g][st]));
    const float qs = q_scale[(long long)bh * s.Tm + i] * sm_scale * LOG2E;
    const float lam2 = lambda_h.v[h] * LOG2E;
    const float NEG = -__builtin_inff();

    float m_run[NG], l_run[NG];
    v16f acc[NG][NDT];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        m_run[g] = NEG;
        l_run[g] = 0.f;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[g][dt][r] = 0.f;
    }
    int pv_done = 0;

    for (int t = 0; t < cnt; ++t) {
        const int j = __builtin_amdgcn_readfirstlane(list[t]);
        const int buf = t & 1;
        // this wave's share of tile t has landed; after the barrier all of it has, and every wave
        // has left tile t-1, whose buffer the next copy overwrites
        dma_wait();
        __syncthreads();
        if (t + 1 < cnt) copy_tile(__builtin_amdgcn_readfirstlane(list[t + 1]), buf ^ 1);
        const unsigned char* Kt = Ks[buf];
        const unsigned char* Vt = Vs[buf];
        const float sc = qs * k_scale[(long long)bh * s.Tn + j];  // dequantization, log2 domain
        // element masks are needed only on causal diagonal tiles and on the ragged last key block
        const bool ragged = (j * BK + BK > s.N) || (CAUSAL && (j * BK + BK - 1 > i * BQ));

        // ---- S^T = K_hat Q_hat^T, int32: all operand reads first, then the MFMA chains ---------
        v4i kf[2][NSTEP];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            const int row = kh * 32 + l32;
#pragma unroll
            for (int st = 0; st < NSTEP; ++st)
                kf[kh][st] = *reinterpret_cast<const v4i*>(&Kt[row * D + (((st * 2 + hl) ^ swz<D>(row)) * 16)]);
        }
        v16i sacc[NG][2];  // [query group][key half]
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[g][kh][r] = 0;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st)
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    sacc[g][kh] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kh][st], qf[g][st], sacc[g][kh], 0, 0, 0);
        // first half of the V^T operand (key slots 0..31) travels from LDS during the softmax
        typename pv::vec vf[2][NDT];
        auto read_v = [&](int ks0) {
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const int row = dt * 32 + l32;
                    vf[k2][dt] = *reinterpret_cast<const typename pv::vec*>(
                        &Vt[row * 128 + ((((ks0 + k2) * 2 + hl) ^ swz<128>(row)) * 16)]);
                }
        };
        read_v(0);
        __builtin_amdgcn_sched_barrier(0);

#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int qrow = qrow0 + g * 32 + l32;
            float p[2][16];
            float m_loc, m_new, alpha, rs = 0.f;
            if (!ragged) {
                int mx = sacc[g][0][0];
#pragma unroll
                for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = max(mx, sacc[g][kh][r]);
                m_loc = max_across_halves(static_cast<float>(mx) * sc);
                m_new = fmaxf(m_run[g], m_loc);  // finite: an unmasked tile has 64 finite scores per row
                const float nm = -m_new;
#pragma unroll
                for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        p[kh][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(static_cast<float>(sacc[g][kh][r]), sc, nm));
                        rs += p[kh][r];
                    }
                alpha = __builtin_amdgcn_exp2f(m_run[g] - m_new);
            } else {
                m_loc = NEG;
#pragma unroll
                for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = j * BK + kh * 32 + 8 * (r >> 2) + 4 * hl + (r & 3);
                        const bool ok = key < s.N && (!CAUSAL || key <= qrow);
                        p[kh][r] = ok ? static_cast<float>(sacc[g][kh][r]) * sc : NEG;
                        m_loc = fmaxf(m_loc, p[kh][r]);
                    }
                m_loc = max_across_halves(m_loc);
                m_new = fmaxf(m_run[g], m_loc);
                const float m_use = (m_new == NEG) ? 0.f : m_new;
#pragma unroll
                for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        p[kh][r] = __builtin_amdgcn_exp2f(p[kh][r] - m_use);
                        rs += p[kh][r];
                    }
                alpha = (m_new == NEG) ? 1.f : __builtin_amdgcn_exp2f(m_run[g] - m_use);
            }
            l_run[g] = l_run[g] * alpha + rs;  // the row sum is always updated (Alg. 1 line 13)
            m_run[g] = m_new;
            // stage-2 test over the group's valid rows (Alg. 1 line 15)
            const float diff = (m_loc == NEG || qrow >= s.N) ? NEG : m_loc - m_new;
            const bool exec = __any(diff > lam2);
            if (exec) {
                ++pv_done;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[g][dt][r] *= alpha;
                }
                typename pv::vec pb[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) pb[ks] = pv::pack(&p[ks >> 1][8 * (ks & 1)]);
                if (NG > 1 && g > 0) read_v(0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) acc[g][dt] = pv::mfma(vf[k2][dt], pb[k2], acc[g][dt]);
                read_v(2);
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) acc[g][dt] = pv::mfma(vf[k2][dt], pb[2 + k2], acc[g][dt]);
            }
        }
    }

    // ---- O_i = diag(l)^-1 O_i; a lane holds 4 consecutive channels per accumulator quad -------
    uint16_t* obase = O + b * s.sb + h * s.sh;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int qrow = qrow0 + g * 32 + l32;
        const float l_tot = sum_across_halves(l_run[g]);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        if (qrow < s.N) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int c0 = dt * 32 + 8 * q4 + 4 * hl;
                    uint16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = cvt_to16<DT>(acc[g][dt][4 * q4 + e] * inv);
                    uint2 w;
                    w.x = o[0] | (static_cast<uint32_t>(o[1]) << 16);
                    w.y = o[2] | (static_cast<uint32_t>(o[3]) << 16);
                    *reinterpret_cast<uint2*>(obase + (long long)qrow * s.sn + c0) = w;
                }
        }
    }

    if (stats) {
        if (lane == 0 && pv_done) atomicAdd(&stats[bh * 4 + 1], (unsigned long long)pv_done);
        if (tid == 0) {
            atomicAdd(&stats[bh * 4 + 0], (unsigned long long)cnt);
            atomicAdd(&stats[bh * 4 + 2], (unsigned long long)jmax);
            unsigned long long vg = 0;
            const int rows = min(BQ, s.N - i * BQ);
            for (int g0 = 0; g0 < rows; g0 += RG) {
                const int last_row = i * BQ + min(g0 + RG, rows) - 1;
                vg += CAUSAL ? (unsigned long long)min(jmax, last_row / BK + 1) : (unsigned long long)jmax;
            }
            atomicAdd(&stats[bh * 4 + 3], vg);
        }
    }
}

__global__ void zero_stats_kernel(unsigned long long* stats, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) stats[i] = 0ull;
}

}  // namespace

hipError_t launch_zero_stats(unsigned long long* stats, int n, hipStream_t st) {
    hipLaunchKernelGGL(zero_stats_kernel, dim3((n + 255) / 256), dim3(256), 0, st, stats, n);
    return hipGetLastError();
}

// Query groups per wave: d = 128 keeps one group per wave (4 waves, <= 256 registers, two workgroups
// resident per SIMD set so one wave's softmax overlaps another's MFMAs); d = 64 affords two.
template <int D> struct GroupsPerWave { static constexpr int value = 1; };

hipError_t launch_attn(const int8_t* Qq, const int8_t* Kq, const float* q_scale, const float* k_scale,
                       const uint16_t* v_tiles, const Shape& s, const uint8_t* mask, const HeadParams& lambda,
                       float sm_scale, int causal, void* O, unsigned long long* stats, hipStream_t st) {
    const int n_work = s.B * s.H * s.Tm;
    const int per_xcd = (n_work + 7) / 8;
    dim3 grid(per_xcd * 8);
    const float scale = sm_scale > 0.f ? sm_scale : static_cast<float>(1.0 / sqrt(static_cast<double>(s.d)));
    uint16_t* o16 = static_cast<uint16_t*>(O);
#define CALL(D, DT)                                                                                           \
    {                                                                                                         \
        constexpr int NG = GroupsPerWave<D>::value;                                                           \
        dim3 block(64 * (4 / NG));                                                                            \
        if (causal) hipLaunchKernelGGL((attn_kernel<D, DT, true, NG>), grid, block, 0, st, Qq, Kq, q_scale,   \
                                       k_scale, v_tiles, o16, mask, s, lambda, scale, n_work, per_xcd, stats); \
        else hipLaunchKernelGGL((attn_kernel<D, DT, false, NG>), grid, block, 0, st, Qq, Kq, q_scale, k_scale, \
                                v_tiles, o16, mask, s, lambda, scale, n_work, per_xcd, stats);                \
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
