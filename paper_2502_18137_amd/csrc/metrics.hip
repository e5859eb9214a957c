// Relative L1 distance between two attention outputs (Sec. 3.6: L1 = sum|O - O'| / sum|O|), the error
// measure of the hyper-parameter search: per (batch, head) the two sums, in fp64.
#include "common.hpp"

namespace sparge {

namespace {

// One workgroup of 1024 threads per (batch, head): every thread sums a fixed set of elements in a fixed
// order and the partial sums are combined by a fixed tree, so the result does not depend on scheduling
// (the hyper-parameter search compares these sums with its bounds: it must decide the same way every time).
template <int D, int DT>
__global__ __launch_bounds__(1024) void rel_l1_kernel(const uint16_t* __restrict__ O, const uint16_t* __restrict__ Oref,
                                                      Shape s, double* __restrict__ out) {
    constexpr int CPR = D / 8, RPI = 1024 / CPR;
    __shared__ double red[2][1024];
    const int h = blockIdx.x, b = blockIdx.y;
    const long long base = b * s.sb + h * s.sh;
    const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
    double num = 0.0, den = 0.0;
    for (int row = r0; row < s.N; row += RPI) {
        const long long off = base + (long long)row * s.sn + col * 8;
        const uint4 a = *reinterpret_cast<const uint4*>(O + off);
        const uint4 r = *reinterpret_cast<const uint4*>(Oref + off);
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, rw[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const double x = cvt16<DT>(static_cast<uint16_t>(aw[e] >> (16 * q)));
                const double y = cvt16<DT>(static_cast<uint16_t>(rw[e] >> (16 * q)));
                num += fabs(y - x);
                den += fabs(y);
            }
        }
    }
    red[0][threadIdx.x] = num;
    red[1][threadIdx.x] = den;
    __syncthreads();
    for (int st = 512; st > 0; st >>= 1) {
        if (threadIdx.x < st) {
            red[0][threadIdx.x] += red[0][threadIdx.x + st];
            red[1][threadIdx.x] += red[1][threadIdx.x + st];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const long long bh = (long long)b * s.H + h;
        out[bh * 2 + 0] = red[0][0];
        out[bh * 2 + 1] = red[1][0];
    }
}

}  // namespace

hipError_t launch_rel_l1(const void* O, const void* Oref, const Shape& s, double* out, hipStream_t st) {
    dim3 grid(s.H, s.B);
    const uint16_t* a = static_cast<const uint16_t*>(O);
    const uint16_t* r = static_cast<const uint16_t*>(Oref);
#define CALL(D, DT) hipLaunchKernelGGL((rel_l1_kernel<D, DT>), grid, dim3(1024), 0, st, a, r, s, out);
    if (s.d == 64 && s.dtype == SPARGE_F16) CALL(64, SPARGE_F16)
    else if (s.d == 64 && s.dtype == SPARGE_BF16) CALL(64, SPARGE_BF16)
    else if (s.d == 128 && s.dtype == SPARGE_F16) CALL(128, SPARGE_F16)
    else if (s.d == 128 && s.dtype == SPARGE_BF16) CALL(128, SPARGE_BF16)
    else return hipErrorInvalidValue;
#undef CALL
    return hipGetLastError();
}

}  // namespace sparge
