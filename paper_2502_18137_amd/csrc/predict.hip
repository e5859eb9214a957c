// Stage-1 predictor after the block statistics (Alg. 1 lines 5-6; Sec. 3.2):
//   logits : S_hat = sm_scale * q k^T on the pooled tokens, fp64 (tiny next to the attention itself)
//   topcdf : per mask row: -inf columns, softmax, TopCdf(tau) by an in-LDS bitonic sort and a
//            prefix sum, fix-block overrides, causal rules.
// All arithmetic is fp64 so that block decisions agree with an fp64 reference except for
// statistics that sit within ~1e-13 of a threshold.
#include "common.hpp"

namespace sparge {

namespace {

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double shfl_up_f64(double v, int delta) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_up(lo, delta);
    hi = __shfl_up(hi, delta);
    return __hiloint2double(hi, lo);
}

// Compressed logits as an fp64 matrix product on the matrix cores: a wave computes RT x 16 pooled query rows x 64
// key blocks with v_mfma_f64_16x16x4_f64 (operands: lane = row or column + 16 * k; result register r of a
// lane = row 4 r + lane / 16, column lane % 16).  The pooled queries are row-major, the key sums
// transposed ([d][Tn]), so the B operand loads are lane-coalesced; both operands stay L2-resident and go
// straight from the caches into the operands, RT + 4 loads for 4 RT matrix instructions per step of 4 channels
// (RT is chosen at launch).
typedef double v4d __attribute__((ext_vector_type(4)));
template <int D, int RT>
__global__ __launch_bounds__(256) void logits_kernel(const double* __restrict__ pooled_q,
                                                      const double* __restrict__ ksum_t, Shape s,
                                                      double sm_scale, double* __restrict__ logits) {
    const long long bh = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i0 = (blockIdx.y * 4 + wave) * 16 * RT, j0 = blockIdx.x * 64;
    if (i0 >= s.Tm) return;
    const int l16 = lane & 15, kk = lane >> 4;
    const double* qrow[RT];
#pragma unroll
    for (int u = 0; u < RT; ++u)   // rows past Tm: a valid row, not stored
        qrow[u] = pooled_q + (bh * s.Tm + min(i0 + 16 * u + l16, s.Tm - 1)) * D + kk;
    const double* kcol[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) kcol[t] = ksum_t + bh * D * s.Tn + (long long)kk * s.Tn + min(j0 + 16 * t + l16, s.Tn - 1);
    v4d acc[RT][4];
#pragma unroll
    for (int u = 0; u < RT; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[u][t] = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int c = 0; c < D; c += 4) {
        double a[RT], bcol[4];
#pragma unroll
        for (int u = 0; u < RT; ++u) a[u] = qrow[u][c];
#pragma unroll
        for (int t = 0; t < 4; ++t) bcol[t] = kcol[t][(long long)c * s.Tn];
#pragma unroll
        for (int u = 0; u < RT; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                acc[u][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], bcol[t], acc[u][t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = j0 + 16 * t + l16;
        if (j >= s.Tn) continue;
        const double cnt = static_cast<double>(min(BK, s.N - j * BK));
#pragma unroll
        for (int u = 0; u < RT; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = i0 + 16 * u + 4 * r + kk;
                if (i < s.Tm) logits[(bh * s.Tm + i) * s.Tn + j] = sm_scale * (acc[u][t][r] / cnt);
            }
    }
}

__device__ __forceinline__ double block_reduce(double v, bool is_max, double* scratch) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const double o = shfl_xor_f64(v, m);
        v = is_max ? fmax(v, o) : v + o;
    }
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    double r = scratch[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) r = is_max ? fmax(r, scratch[w]) : r + scratch[w];
    return r;
}

// One workgroup per mask row (b, h, i).  npad = power of two >= max(Tn, 2).
__global__ __launch_bounds__(256) void topcdf_kernel(const double* __restrict__ logits,
                                                      const double* __restrict__ sim_q,
                                                      const double* __restrict__ sim_k, Shape s,
                                                      HeadParams tau_h, HeadParams theta_h, int causal,
                                                      int npad, uint8_t* __restrict__ mask) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* keys = reinterpret_cast<double*>(smem);                      // [npad] probabilities by key block
    unsigned long long* skey = reinterpret_cast<unsigned long long*>(keys + npad);  // [npad] sort keys
    uint8_t* flag = reinterpret_cast<uint8_t*>(skey + npad);             // [npad]
    __shared__ double scratch[4];
    __shared__ double wave_tot[4];

    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const long long bh = (long long)b * s.H + h;
    const int tid = threadIdx.x;
    const double tau = static_cast<double>(tau_h.v[h]);
    const double theta = static_cast<double>(theta_h.v[h]);
    const double* row = logits + (bh * s.Tm + i) * s.Tn;
    const double* sk = sim_k + bh * s.Tn;
    const double NEG = -__builtin_inf();

    // A query block that is not self-similar keeps every (visible) key block: nothing to rank.
    if (sim_q[bh * s.Tm + i] < theta) {
        uint8_t* out_row = mask + (bh * s.Tm + i) * s.Tn;
        for (int j = tid; j < s.Tn; j += 256) out_row[j] = (causal && j * BK > i * BQ + (BQ - 1)) ? 0 : 1;
        return;
    }

    // 1. masked logits and their maximum
    double mx = NEG;
    for (int j = tid; j < npad; j += 256) {
        double x = NEG;
        if (j < s.Tn) {
            x = row[j];
            if (sk[j] < theta) x = NEG;
            if (causal && j * BK > i * BQ + (BQ - 1)) x = NEG;
        }
        keys[j] = x;
        mx = fmax(mx, x);
    }
    mx = block_reduce(mx, true, scratch);
    // 2. softmax numerators and their sum
    double z = 0.0;
    for (int j = tid; j < npad; j += 256) {
        const double x = keys[j];
        const double e = (x == NEG) ? 0.0 : exp(x - mx);
        keys[j] = e;
        z += e;
    }
    z = block_reduce(z, false, scratch);
    double tot = 0.0;
    for (int j = tid; j < npad; j += 256) {
        double p = -1.0;  // padding ranks after every probability
        if (j < s.Tn) {
            p = z > 0.0 ? keys[j] / z : 0.0;
            tot += p;
        }
        keys[j] = p;
        // Sort key: the probability's bit pattern (non-negative doubles order like integers) with its low
        // 16 mantissa bits replaced by 0xFFFF - j: one 64-bit comparison ranks by (value descending, index
        // ascending).  Values closer than 2^-36 relative may swap ranks; that moves a prefix mass by less
        // than 2^-36, far inside the band in which a decision counts as a tie.
        skey[j] = p < 0.0 ? 0ull
                          : ((static_cast<unsigned long long>(__double_as_longlong(p)) & ~0xFFFFull) |
                             static_cast<unsigned long long>(0xFFFF - j));
        flag[j] = 0;
    }
    tot = block_reduce(tot, false, scratch);  // also orders the LDS writes before the sort

    // 3. bitonic sort: rank order = (value descending, index ascending).  Each wave owns a quarter of the
    // array: every compare-exchange at a distance inside a quarter touches the wave's own elements only,
    // and a wave's LDS accesses complete in program order, so those stages need no workgroup barrier
    // (the wave barrier only pins the compiler's order).  Only the few stages that reach across quarters
    // are bracketed by barriers.
    auto exchange = [&](int lo, int jj, int k) {
        const int hi = lo + jj;
        const unsigned long long ka = skey[lo], kb = skey[hi];
        const bool a_first = ka > kb;   // keys are distinct except among the padding
        const bool want_a_first = (lo & k) == 0;
        if (a_first != want_a_first && ka != kb) {
            skey[lo] = kb;
            skey[hi] = ka;
        }
    };
    const int epw = npad >> 2;  // elements per wave
    if (epw >= 128) {
        const int lane_ = tid & 63, seg = (tid >> 6) * epw;
        for (int k = 2; k <= npad; k <<= 1) {
            int jj = k >> 1;
            if (jj >= epw) {
                __syncthreads();
                for (; jj >= epw; jj >>= 1) {
                    for (int t = tid; t < (npad >> 1); t += 256) exchange(2 * jj * (t / jj) + (t % jj), jj, k);
                    __syncthreads();
                }
            }
            for (; jj > 0; jj >>= 1) {
                for (int t = lane_; t < (epw >> 1); t += 64) exchange(seg + 2 * jj * (t / jj) + (t % jj), jj, k);
                __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
    } else {
        for (int k = 2; k <= npad; k <<= 1) {
            for (int jj = k >> 1; jj > 0; jj >>= 1) {
                for (int t = tid; t < (npad >> 1); t += 256) exchange(2 * jj * (t / jj) + (t % jj), jj, k);
                __syncthreads();
            }
        }
    }

    // 4. exclusive prefix mass per rank; rank r is kept iff mass before it < tau * total
    const int per = (npad + 255) / 256;  // consecutive ranks per thread
    const int r0 = tid * per;
    double local = 0.0;
    auto rank_index = [&](int r) { return 0xFFFF - static_cast<int>(skey[r] & 0xFFFFull); };
    auto rank_value = [&](int r) { return skey[r] ? keys[rank_index(r)] : 0.0; };   // padding ranks last, mass 0
    for (int r = r0; r < min(r0 + per, npad); ++r) local += rank_value(r);
    // inclusive scan of `local` over the 256 threads
    const int lane = tid & 63, wave = tid >> 6;
    double incl = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double o = shfl_up_f64(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    double before = incl - local;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    const double thresh = tau * tot;
    for (int r = r0; r < min(r0 + per, npad); ++r) {
        const double p = rank_value(r);
        if (p > 0.0 && before < thresh) flag[rank_index(r)] = 1;
        before += p;
    }
    __syncthreads();

    // 5. fix-block overrides and causal rules, then the row goes out
    const bool fix_q = sim_q[bh * s.Tm + i] < theta;
    uint8_t* out = mask + (bh * s.Tm + i) * s.Tn;
    for (int j = tid; j < s.Tn; j += 256) {
        uint8_t m = flag[j];
        if (fix_q || sk[j] < theta) m = 1;
        if (causal) {
            if (j * BK > i * BQ + (BQ - 1)) m = 0;
            if (j == (i * BQ) / BK) m = 1;
        }
        out[j] = m;
    }
}

// v_permlane16_swap (LD = 16: odd rows of 16 lanes of a against even rows of b) or v_permlane32_swap (LD = 32:
// upper half of a against lower half of b); applying it twice restores a and b
template <int LD>
__device__ __forceinline__ void lane_swap(uint32_t a, uint32_t b, uint32_t& a_out, uint32_t& b_out) {
    static_assert(LD == 16 || LD == 32, "no such swap");
    if constexpr (LD == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
        a_out = r[0], b_out = r[1];
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
        a_out = r[0], b_out = r[1];
    }
}

// Bitonic sort, descending, of 64 * EPL keys held EPL consecutive ranks per lane.  The stages are
// instantiated one by one (K: length of the runs being merged, JJ: distance of the pairs), so that every
// register index, DPP control and swap is a compile-time constant.
// max / min of two keys read as fp64 numbers: two instructions for a compare-exchange where the 64-bit integer
// comparison and its four selects take five.  The keys are never NaN or infinite (probabilities <= 1 with an index
// in the low mantissa bits, or 0), fp64 denormals are not flushed, and the instructions are written out so that
// the compiler does not canonicalize their inputs first.
__device__ __forceinline__ void max_min_f64(unsigned long long a, unsigned long long b, unsigned long long& hi,
                                            unsigned long long& lo) {
    const double x = __longlong_as_double(static_cast<long long>(a)), y = __longlong_as_double(static_cast<long long>(b));
    double mx, mn;
    asm("v_max_f64 %0, %1, %2" : "=v"(mx) : "v"(x), "v"(y));
    asm("v_min_f64 %0, %1, %2" : "=v"(mn) : "v"(x), "v"(y));
    hi = static_cast<unsigned long long>(__double_as_longlong(mx));
    lo = static_cast<unsigned long long>(__double_as_longlong(mn));
}

// Runs of K >= EPL ranks ascend or descend by lane.  While such runs are merged, the lanes of ascending runs carry
// their keys with the sign bit set (set_run_sign, once per run length): read as fp64 the keys of every lane then
// descend the same way, and a pair inside a lane is ordered by max / min without a select.  The comparisons
// between lanes keep reading the keys as integers; both keys of such a pair carry the same sign bit, so their
// integer order is the order of the keys themselves.  The last run descends in every lane: the signs end up clear.
template <int EPL, int K>
__device__ __forceinline__ void set_run_sign(unsigned long long (&key)[EPL], int lane) {
    if constexpr (K >= EPL) {
        const unsigned long long sign = (((lane * EPL) & K) == 0) ? 0ull : 0x8000000000000000ull;
#pragma unroll
        for (int e = 0; e < EPL; ++e) key[e] = (key[e] & 0x7FFFFFFFFFFFFFFFull) | sign;
    }
}

template <int EPL, int K, int JJ>
__device__ __forceinline__ void bitonic_stage(unsigned long long (&key)[EPL], int lane) {
    if constexpr (JJ < EPL) {  // both members of a pair in this lane
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            if (e & JJ) continue;
            unsigned long long hi, lo;
            max_min_f64(key[e], key[e | JJ], hi, lo);
            // short runs: the direction is known per register; long runs: the sign bits make every lane descend
            const bool desc = K < EPL ? ((e & K) == 0) : true;
            key[e] = desc ? hi : lo;
            key[e | JJ] = desc ? lo : hi;
        }
    } else {
        constexpr int LD = JJ / EPL;  // partner lane = lane ^ LD
        const bool desc = ((lane * EPL) & K) == 0;
        if constexpr (LD >= 16) {
            // Lanes 16 or 32 apart: the lane swap of the keys of two entries e, e+1 puts both members of a pair
            // into one lane (one half of the lanes gets the pairs of entry e, the other half those of entry
            // e+1, earlier rank first); the pair is ordered there like a pair inside a lane, and the same swap
            // takes the keys home.
#pragma unroll
            for (int e = 0; e < EPL; e += 2) {
                uint32_t al, ah, bl, bh;
                lane_swap<LD>(static_cast<uint32_t>(key[e]), static_cast<uint32_t>(key[e + 1]), al, bl);
                lane_swap<LD>(static_cast<uint32_t>(key[e] >> 32), static_cast<uint32_t>(key[e + 1] >> 32), ah, bh);
                const unsigned long long a = (static_cast<unsigned long long>(ah) << 32) | al;
                const unsigned long long b = (static_cast<unsigned long long>(bh) << 32) | bl;
                const bool exch = (a > b) != desc;
                const unsigned long long first = exch ? b : a, second = exch ? a : b;
                lane_swap<LD>(static_cast<uint32_t>(first), static_cast<uint32_t>(second), al, bl);
                lane_swap<LD>(static_cast<uint32_t>(first >> 32), static_cast<uint32_t>(second >> 32), ah, bh);
                key[e] = (static_cast<unsigned long long>(ah) << 32) | al;
                key[e + 1] = (static_cast<unsigned long long>(bh) << 32) | bl;
            }
        } else {
            // closer lanes: the partner's key comes through DPP moves
            const bool upper = (lane & LD) != 0;  // this lane holds the later ranks of the pairs
            // the earlier rank of a pair keeps the larger key when the run descends, the later rank the smaller:
            // take the partner's key if it is larger and the larger one is wanted, or neither (equal keys are
            // padding, either copy will do)
            const bool want_min = desc == upper;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const unsigned long long mine = key[e];
                const uint32_t plo = row_xchg<LD>(static_cast<uint32_t>(mine));
                const uint32_t phi = row_xchg<LD>(static_cast<uint32_t>(mine >> 32));
                const unsigned long long other = (static_cast<unsigned long long>(phi) << 32) | plo;
                key[e] = ((other > mine) != want_min) ? other : mine;
            }
        }
    }
}
template <int EPL, int K, int JJ>
__device__ __forceinline__ void bitonic_merge(unsigned long long (&key)[EPL], int lane) {
    bitonic_stage<EPL, K, JJ>(key, lane);
    if constexpr (JJ > 1) bitonic_merge<EPL, K, JJ / 2>(key, lane);
}
template <int EPL, int K = 2>
__device__ __forceinline__ void bitonic_sort(unsigned long long (&key)[EPL], int lane) {
    set_run_sign<EPL, K>(key, lane);
    bitonic_merge<EPL, K, K / 2>(key, lane);
    if constexpr (K < 64 * EPL) bitonic_sort<EPL, 2 * K>(key, lane);
}

// TopCdf with one mask row per wave and the sort in registers: lane L holds the EPL consecutive ranks
// L * EPL .. L * EPL + EPL - 1 as 64-bit keys (see topcdf_kernel for the key).  A bitonic stage at a distance
// below EPL exchanges inside a lane (compile-time register indices), a larger one takes the partner
// lane's key with DPP moves or lane swaps (vector ALU: with ds_bpermute the LDS pipeline was the limit);
// nothing but the final flags and the exact probabilities goes through LDS, and no workgroup barrier is needed.  Same comparisons, hence the same order, as the LDS version.
template <int EPL>
__global__ __launch_bounds__(256) void topcdf_wave_kernel(const double* __restrict__ logits,
                                                           const double* __restrict__ sim_q,
                                                           const double* __restrict__ sim_k, Shape s,
                                                           HeadParams tau_h, HeadParams theta_h, int causal,
                                                           int n_rows, uint8_t* __restrict__ mask) {
    constexpr int NPAD = 64 * EPL;
    __shared__ double pval[4][NPAD];
    __shared__ uint8_t flag[4][NPAD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rowid = blockIdx.x * 4 + wave;          // (b, h, i) flattened
    if (rowid >= n_rows) return;
    const int i = rowid % s.Tm;
    const long long bh = rowid / s.Tm;
    const int h = static_cast<int>(bh % s.H);
    const double tau = static_cast<double>(tau_h.v[h]);
    const double theta = static_cast<double>(theta_h.v[h]);
    const double* row = logits + (long long)rowid * s.Tn;
    const double* sk = sim_k + bh * s.Tn;
    uint8_t* out = mask + (long long)rowid * s.Tn;
    const double NEG = -__builtin_inf();
    if (sim_q[rowid] < theta) {   // a query block that is not self-similar keeps every visible key block
        for (int j = lane; j < s.Tn; j += 64) out[j] = (causal && j * BK > i * BQ + (BQ - 1)) ? 0 : 1;
        return;
    }
    auto wave_sum = [&](double v) {
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) v += shfl_xor_f64(v, m);
        return v;
    };
    // 1.-2. masked logits, softmax, probabilities (entries lane * EPL + e: a lane reads one contiguous piece)
    double x[EPL];
    double mx = NEG;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int j = lane * EPL + e;
        x[e] = NEG;
        if (j < s.Tn) {
            x[e] = row[j];
            if (sk[j] < theta) x[e] = NEG;
            if (causal && j * BK > i * BQ + (BQ - 1)) x[e] = NEG;
        }
        mx = fmax(mx, x[e]);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) mx = fmax(mx, shfl_xor_f64(mx, m));
    double z = 0.0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        x[e] = (x[e] == NEG) ? 0.0 : exp(x[e] - mx);
        z += x[e];
    }
    z = wave_sum(z);
    // (one division per lane; x * (1 / z) is within two roundings of x / z, far inside the band in which a
    // TopCdf decision counts as undecided)
    const double rz = z > 0.0 ? 1.0 / z : 0.0;
    double tot = 0.0;
    unsigned long long key[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int j = lane * EPL + e;
        const double p = j < s.Tn ? x[e] * rz : 0.0;
        tot += p;
        pval[wave][j] = p;
        flag[wave][j] = 0;
        key[e] = j < s.Tn ? ((static_cast<unsigned long long>(__double_as_longlong(p)) & ~0xFFFFull) |
                             static_cast<unsigned long long>(0xFFFF - j))
                          : 0ull;   // padding ranks last
    }
    tot = wave_sum(tot);

    // 3. bitonic sort, descending by key
    bitonic_sort<EPL>(key, lane);

    // 4. exclusive prefix mass per rank (exact probabilities by index); rank kept iff mass before it < tau * total
    double pv[EPL];
    double local = 0.0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        pv[e] = key[e] ? pval[wave][0xFFFF - static_cast<int>(key[e] & 0xFFFFull)] : 0.0;
        local += pv[e];
    }
    double incl = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double o = shfl_up_f64(incl, d);
        if (lane >= d) incl += o;
    }
    double before = incl - local;
    const double thresh = tau * tot;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        if (pv[e] > 0.0 && before < thresh) flag[wave][0xFFFF - static_cast<int>(key[e] & 0xFFFFull)] = 1;
        before += pv[e];
    }
    __builtin_amdgcn_wave_barrier();   // the flags are read back by other lanes of this wave only

    // 5. fix-block overrides and causal rules, then the row goes out
    for (int j = lane; j < s.Tn; j += 64) {
        uint8_t m = flag[wave][j];
        if (sk[j] < theta) m = 1;
        if (causal) {
            if (j * BK > i * BQ + (BQ - 1)) m = 0;
            if (j == (i * BQ) / BK) m = 1;
        }
        out[j] = m;
    }
}

// The mask as an index list: one wave per mask row compacts the kept block indices with ballots, 64 entries
// at a time, in ascending order; the rest of the row is -1.
__global__ __launch_bounds__(256) void mask_lut_kernel(const uint8_t* __restrict__ mask, int Tn, int n_rows,
                                                       int32_t* __restrict__ lut, int32_t* __restrict__ lut_count) {
    const int row = blockIdx.x * 4 + static_cast<int>(threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const uint8_t* m = mask + static_cast<long long>(row) * Tn;
    int32_t* out = lut + static_cast<long long>(row) * Tn;
    int n = 0;
    for (int j0 = 0; j0 < Tn; j0 += 64) {
        const int j = j0 + lane;
        const bool keep = j < Tn && m[j] != 0;
        const unsigned long long bal = __ballot(keep);
        if (keep) out[n + __popcll(bal & ((1ull << lane) - 1ull))] = j;
        n += __popcll(bal);
    }
    for (int j = n + lane; j < Tn; j += 64) out[j] = -1;
    if (lane == 0) lut_count[row] = n;
}

}  // namespace

hipError_t launch_mask_lut(const uint8_t* mask, const Shape& s, int32_t* lut, int32_t* lut_count, hipStream_t st) {
    const int n_rows = s.B * s.H * s.Tm;
    hipLaunchKernelGGL(mask_lut_kernel, dim3((n_rows + 3) / 4), dim3(256), 0, st, mask, s.Tn, n_rows, lut, lut_count);
    return hipGetLastError();
}

hipError_t launch_logits(const double* pooled_q, const double* ksum_t, const Shape& s, float sm_scale,
                         double* logits, hipStream_t st) {
    // two row tiles of 16 pooled queries per wave where there are enough rows to fill the chip that way
    // (measured: 55 against 61 us at T_m = 360, 33 against 39 us at T_m = 256 with 32 heads; 18 against 17 us at T_m = 138)
    const int rt = s.Tm >= 192 ? 2 : 1;
    dim3 grid((s.Tn + 63) / 64, (s.Tm + 64 * rt - 1) / (64 * rt), s.B * s.H);
    const double scale = sm_scale > 0.f ? static_cast<double>(sm_scale) : 1.0 / sqrt(static_cast<double>(s.d));
#define CALL(D, RT) hipLaunchKernelGGL((logits_kernel<D, RT>), grid, dim3(256), 0, st, pooled_q, ksum_t, s, scale, logits)
    if (s.d == 64) { if (rt == 2) CALL(64, 2); else CALL(64, 1); }
    else { if (rt == 2) CALL(128, 2); else CALL(128, 1); }
#undef CALL
    return hipGetLastError();
}

hipError_t launch_topcdf(const double* logits, const double* sim_q, const double* sim_k, const Shape& s,
                         const HeadParams& tau, const HeadParams& theta, int causal, uint8_t* mask,
                         hipStream_t st) {
    const int n_rows = s.B * s.H * s.Tm;
#define CALLW(EPL)                                                                                                 \
    hipLaunchKernelGGL((topcdf_wave_kernel<EPL>), dim3((n_rows + 3) / 4), dim3(256), 0, st, logits, sim_q, sim_k, s, \
                       tau, theta, causal, n_rows, mask)
    if (s.Tn <= 256) { CALLW(4); return hipGetLastError(); }
    if (s.Tn <= 512) { CALLW(8); return hipGetLastError(); }
    if (s.Tn <= 1024) { CALLW(16); return hipGetLastError(); }
    if (s.Tn <= 2048) { CALLW(32); return hipGetLastError(); }
#undef CALLW
    // longer rows: one workgroup per row, sorted in LDS
    int npad = 2;
    while (npad < s.Tn) npad <<= 1;
    const size_t smem = static_cast<size_t>(npad) * (sizeof(double) + sizeof(unsigned long long) + 1);
    // 68 KB at the longest rows: more than the 64 KB a launch gets without asking (the CU has 160 KB)
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(topcdf_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
    if (e != hipSuccess) return e;
    dim3 grid(s.Tm, s.H, s.B);
    hipLaunchKernelGGL(topcdf_kernel, grid, dim3(256), smem, st, logits, sim_q, sim_k, s, tau, theta, causal,
                       npad, mask);
    return hipGetLastError();
}

}  // namespace sparge
