// Internal declarations shared by the HIP translation units of libsparge (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "sparge.h"

namespace sparge {

constexpr int BQ = SPARGE_BQ;         // query rows per block (Alg. 1 line 2; App. A.1)
constexpr int BK = SPARGE_BK;         // key rows per block
constexpr int RG = SPARGE_ROW_GROUP;  // rows per stage-2 row group (b_q / c_w)

struct Shape {
    int B, H, N, d, dtype;
    long long sb, sh, sn;  // element strides of the 16-bit tensors
    int Tm, Tn;
    int pv_fp8;            // P~V product in FP8 (E4M3) instead of the tensors' 16-bit type
    int qk16;              // Q K^T product on the 16-bit tensors themselves instead of their INT8 quantization
};

// Per-head scalars travel to the device inside the kernel argument block.
struct HeadParams {
    float v[SPARGE_MAX_HEADS];
};

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v8f __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// The value another lane of the same row of 16 holds, through a DPP move (vector ALU, no LDS traffic).
//   PARTNER 1, 2, 8: the value of lane ^ PARTNER (quad permutes, rotation by 8 inside a row of 16).
//   PARTNER 4: the value of lane ^ 4 (two shifts by 4, each written to the banks it is right for).
//   PARTNER 7, 15: the value of lane 7 - lane % 8 of the same group of 8, of lane 15 - lane % 16 of the same
//   row (mirrors, one instruction).  They serve as ^4 (^8) ONLY where the lanes of each group of 4 (of 8)
//   already hold the same value.
template <int PARTNER>
__device__ __forceinline__ uint32_t row_xchg(uint32_t v) {
    static_assert(PARTNER == 1 || PARTNER == 2 || PARTNER == 4 || PARTNER == 8 || PARTNER == 7 || PARTNER == 15,
                  "no such exchange");
    if constexpr (PARTNER == 4) {
        // row_shl:4 brings lane + 4 (banks 0 and 2 take it), row_shr:4 brings lane - 4 (banks 1 and 3)
        const int up = __builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x104, 0xF, 0x5, false);
        return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(up, static_cast<int>(v), 0x114, 0xF, 0xA, false));
    } else {
        constexpr int CTRL = PARTNER == 1 ? 0xB1 : PARTNER == 2 ? 0x4E : PARTNER == 7 ? 0x141 : PARTNER == 15 ? 0x140 : 0x128;
        // every lane has a source inside its row; bound_ctrl tells the compiler that the destination's old
        // value is never kept, which saves a register preload and its wait states per exchange
        return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, true));
    }
}

// 16-bit storage -> fp32 (exact).  DT: SPARGE_F16 or SPARGE_BF16.
template <int DT>
__device__ __forceinline__ float cvt16(uint16_t bits) {
    if constexpr (DT == SPARGE_BF16) {
        return __uint_as_float(static_cast<uint32_t>(bits) << 16);
    } else {
        _Float16 h;
        __builtin_memcpy(&h, &bits, 2);
        return static_cast<float>(h);
    }
}

// fp32 -> 16-bit storage, round to nearest even.
template <int DT>
__device__ __forceinline__ uint16_t cvt_to16(float f) {
    uint16_t bits;
    if constexpr (DT == SPARGE_BF16) {
        __bf16 h = static_cast<__bf16>(f);
        __builtin_memcpy(&bits, &h, 2);
    } else {
        _Float16 h = static_cast<_Float16>(f);
        __builtin_memcpy(&bits, &h, 2);
    }
    return bits;
}

// Order of the attention kernel's work items.  Items are numbered g = (b H + h) T_m + q; q counts a head's Q
// blocks from the last one down when the attention is causal (i = T_m - 1 - q: longest rows first), up
// otherwise (i = q).  They are cut into 8 contiguous ranges of `per_range` items, one per XCD, and a range hands
// out its items through a counter: p = 0, 1, ... -> the item returned here, for the range that starts at r0 and
// holds len items.  Non-causal: in index order.  Causal: in two passes over the range's heads, first the longer
// half of every head's rows (q < T_m - T_m / 2), head by head, then the shorter halves -- so that the items a
// range ends with are short whichever head they belong to (with whole heads one after the other the long rows
// of the last head start late and a tenth of the slot time at the causal language shape was an idle tail).
__host__ __device__ inline int range_item(int r0, int len, int p, int Tm, bool causal) {
    if (!causal) return r0 + p;
    const int r1 = r0 + len, longer = Tm - Tm / 2;
    const int h0 = r0 / Tm, h1 = (r1 - 1) / Tm;
    for (int pass = 0; pass < 2; ++pass) {
        const int lo = pass ? longer : 0, hi = pass ? Tm : longer;  // the q of this pass inside a head
        // the range's first head (it may begin inside it), the whole heads after it, its last head
        const int a0 = r0 - h0 * Tm > lo ? r0 - h0 * Tm : lo;
        const int b0 = r1 - h0 * Tm < hi ? r1 - h0 * Tm : hi;
        const int c0 = b0 > a0 ? b0 - a0 : 0;
        if (p < c0) return h0 * Tm + a0 + p;
        p -= c0;
        if (h1 > h0) {
            const int whole = (h1 - h0 - 1) * (hi - lo);
            if (p < whole) return (h0 + 1 + p / (hi - lo)) * Tm + lo + p % (hi - lo);
            p -= whole;
            const int b1 = r1 - h1 * Tm < hi ? r1 - h1 * Tm : hi;
            const int c1 = b1 > lo ? b1 - lo : 0;
            if (p < c1) return h1 * Tm + lo + p;
            p -= c1;
        }
    }
    return -1;  // p >= len
}

// ---- kernel launchers (host functions defined next to their kernels) ----------------------------
// Block statistics of Q (+ optional INT8 quantization of Q): pooled means, self-similarity.
hipError_t launch_block_stats_q(const void* Q, const Shape& s, double* pooled_q, double* sim_q,
                                int8_t* Qq, float* q_scale, hipStream_t st);
// Block statistics of K: per-block channel sums (transposed [B,H,d,Tn]) and self-similarity.
hipError_t launch_block_stats_k(const void* K, const Shape& s, double* ksum_t, double* sim_k, hipStream_t st);
// Token mean of K per (b,h) from the block sums.
hipError_t launch_k_mean(const double* ksum_t, const Shape& s, float* k_mean, hipStream_t st);
// INT8 quantization of K - k_mean.
hipError_t launch_quant_k(const void* K, const Shape& s, const float* k_mean, int8_t* Kq, float* k_scale,
                          hipStream_t st);
// Compressed logits S_hat = sm_scale * q k^T (no masking), fp64 [B,H,Tm,Tn].
hipError_t launch_logits(const double* pooled_q, const double* ksum_t, const Shape& s, float sm_scale,
                         double* logits, hipStream_t st);
// Softmax + TopCdf + overrides per mask row.
hipError_t launch_topcdf(const double* logits, const double* sim_q, const double* sim_k, const Shape& s,
                         const HeadParams& tau, const HeadParams& theta, int causal, uint8_t* mask,
                         hipStream_t st);
// V [B,H,N,d] (strided) -> per key block, d rows of 64 key slots in the order the P~V MFMA consumes.
hipError_t launch_v_tiles(const void* V, const Shape& s, uint16_t* v_tiles, hipStream_t st);
// lut[b,h,i,:] = the j with mask[b,h,i,j] != 0, ascending, then -1; lut_count[b,h,i] = how many.
hipError_t launch_mask_lut(const uint8_t* mask, const Shape& s, int32_t* lut, int32_t* lut_count, hipStream_t st);
// stats[0..n) = 0 (a fill kernel, not a memset node, so callers may capture it in a graph).
hipError_t launch_zero_stats(unsigned long long* stats, int n, hipStream_t st);
// The sparse flash loop (accumulates into stats).  queue: ATTN_QUEUE_BYTES of device memory for the item
// counters of the work distribution, cleared here by a fill kernel in front of the launch; it must not be
// shared with another launch that may run at the same time.
constexpr size_t ATTN_QUEUE_BYTES = 1024;
hipError_t launch_attn(const void* Qp, const void* Kp, const float* q_scale, const float* k_scale,
                       const void* v_tiles, const float* v_scale, const Shape& s, const uint8_t* mask,
                       const HeadParams& lambda, float sm_scale, int causal, void* O, unsigned long long* stats,
                       unsigned int* queue, hipStream_t st);
// FP8 form of V: per-(b,h,channel) |V| maxima (as fp32 bit patterns, zeroed here), scales amax/448, and
// E4M3 tiles in the operand order of the 32x32x64 MFMA.
hipError_t launch_v_tiles_fp8(const void* V, const Shape& s, unsigned char* tiles, float* v_scale,
                              uint32_t* amax_bits, hipStream_t st);

// out[b,h] = {sum|Oref - O|, sum|Oref|} in fp64 (overwritten; fixed summation order), both tensors laid out as the shape says.
hipError_t launch_rel_l1(const void* O, const void* Oref, const Shape& s, double* out, hipStream_t st);

// Order in which a Hilbert curve visits the row-major cells of a T x H x W grid (host; perm has T*H*W entries).
void hilbert_order_host(int T, int H, int W, int32_t* perm);
// Token gather by that order, or its inverse, on [off, off + L); other tokens are copied in place.
hipError_t launch_permute_tokens(const void* src, const Shape& s, const int32_t* perm, int L, int off, int inverse,
                                 void* dst, hipStream_t st);

}  // namespace sparge
