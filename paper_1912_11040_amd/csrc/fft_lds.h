// In-place complex FFT of a power-of-two length held in LDS, shared by the
// overlap-save convolution (lengths 256..16384) and the STFT (length nfft/2).
//
// Forward: decimation in frequency, natural order in, digit-reversed order out.
// Inverse: decimation in time, digit-reversed order in, natural order out, no 1/N.
// A convolution multiplies spectra in the permuted order, so no reordering pass is
// ever run; FftPlan<N>::position(k) says where frequency k sits.
//
// Passes use radix 16 (two radix-4 layers in registers) while four or more bits
// remain, then one radix-4 and/or one radix-2 pass.  Twiddles come from a table
// exp(-2 pi i t / N) rounded once from fp64.
//
// LDS addressing is padded by one complex per 16 so that the stride-16 accesses of
// the late passes spread over banks: element i lives at lds_pad(i).
#pragma once

#include <hip/hip_runtime.h>

namespace aug {

__device__ __host__ constexpr int lds_pad(int i) { return i + (i >> 4); }
__device__ __host__ constexpr int lds_padded_size(int n) { return n + (n >> 4); }

__device__ inline float2 cmul(float2 a, float2 b) {
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ inline float2 cmul_conj(float2 a, float2 b) {   // a * conj(b)
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
__device__ inline float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ inline float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ inline float2 cconj(float2 a) { return make_float2(a.x, -a.y); }
// multiply by -i (forward) or +i (inverse)
template <bool INV> __device__ inline float2 rot90(float2 a) {
    return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}

// 4-point DFT, natural order in and out; INV uses exp(+2 pi i / 4).
template <bool INV>
__device__ inline void dft4(float2& a0, float2& a1, float2& a2, float2& a3) {
    const float2 s02 = cadd(a0, a2), d02 = csub(a0, a2);
    const float2 s13 = cadd(a1, a3), d13 = rot90<INV>(csub(a1, a3));
    a0 = cadd(s02, s13);
    a1 = cadd(d02, d13);
    a2 = csub(s02, s13);
    a3 = csub(d02, d13);
}

// R-point DFT of v[0..R) in registers, natural order in and out.
template <int R, bool INV> struct SmallDft;

template <bool INV> struct SmallDft<2, INV> {
    __device__ static inline void run(float2 (&v)[2]) {
        const float2 a = v[0], b = v[1];
        v[0] = cadd(a, b);
        v[1] = csub(a, b);
    }
};

template <bool INV> struct SmallDft<4, INV> {
    __device__ static inline void run(float2 (&v)[4]) { dft4<INV>(v[0], v[1], v[2], v[3]); }
};

template <bool INV> struct SmallDft<16, INV> {
    // m = m2 + 4 m1, r = r1 + 4 r2:
    // y[r1 + 4 r2] = sum_{m2} W4^{m2 r2} W16^{m2 r1} sum_{m1} x[m2 + 4 m1] W4^{m1 r1}
    __device__ static inline void run(float2 (&v)[16]) {
        constexpr float c1 = 0.92387953251128674f, s1 = 0.38268343236508977f;   // cos, sin(pi/8)
        constexpr float h = 0.70710678118654752f;
        // W16^e = exp(-2 pi i e / 16) for e = 0..9 (forward sign)
        const float2 w[10] = {{1.f, 0.f}, {c1, -s1}, {h, -h}, {s1, -c1}, {0.f, -1.f},
                              {-s1, -c1}, {-h, -h}, {-c1, -s1}, {-1.f, 0.f}, {-c1, s1}};
#pragma unroll
        for (int m2 = 0; m2 < 4; ++m2) {
            dft4<INV>(v[m2], v[m2 + 4], v[m2 + 8], v[m2 + 12]);     // now v[m2 + 4 r1]
#pragma unroll
            for (int r1 = 1; r1 < 4; ++r1) {
                if (m2 == 0) continue;
                const float2 t = w[m2 * r1];
                v[m2 + 4 * r1] = INV ? cmul_conj(v[m2 + 4 * r1], t) : cmul(v[m2 + 4 * r1], t);
            }
        }
#pragma unroll
        for (int r1 = 0; r1 < 4; ++r1) {
            // inputs t[m2][r1] sit at v[m2 + 4 r1]; outputs y[r1 + 4 r2] -> gather below
            dft4<INV>(v[4 * r1 + 0], v[4 * r1 + 1], v[4 * r1 + 2], v[4 * r1 + 3]);  // v[4 r1 + r2]
        }
        // v[4 r1 + r2] holds y[r1 + 4 r2]: transpose the 4x4 index to natural order
#pragma unroll
        for (int r1 = 0; r1 < 4; ++r1)
#pragma unroll
            for (int r2 = r1 + 1; r2 < 4; ++r2) {
                const float2 t = v[4 * r1 + r2];
                v[4 * r1 + r2] = v[4 * r2 + r1];
                v[4 * r2 + r1] = t;
            }
    }
};

constexpr int ilog2(int n) { return n <= 1 ? 0 : 1 + ilog2(n >> 1); }

template <int N>
struct FftPlan {
    static constexpr int kLog = ilog2(N);
    static constexpr int kN16 = kLog / 4;          // radix-16 passes
    static constexpr int kRem = kLog % 4;          // remaining bits: 0..3
    static constexpr bool kHas4 = kRem >= 2;
    static constexpr bool kHas2 = (kRem & 1) != 0;

    // Where frequency k sits after the forward transform: digits of k, least
    // significant first in the order the passes ran, become the most significant
    // digits of the position.
    __device__ __host__ static inline int position(int k) {
        int pos = 0, rest = N;
        for (int p = 0; p < kN16; ++p) {
            rest >>= 4;
            pos += (k & 15) * rest;
            k >>= 4;
        }
        if (kHas4) {
            rest >>= 2;
            pos += (k & 3) * rest;
            k >>= 2;
        }
        if (kHas2) {
            rest >>= 1;
            pos += (k & 1) * rest;
        }
        return pos;
    }
};

// One pass over blocks of length S with radix R (sub-block length Q = S / R).
// Forward (DIF):  y_r = W_S^{j r} sum_m x[j + m Q] W_R^{m r}       -> stored at j + r Q
// Inverse (DIT):  x_m = sum_r (conj(W_S^{j r}) y[j + r Q]) W_R^{-m r} -> stored at j + m Q
template <int N, int S, int R, bool INV, int T>
__device__ inline void fft_pass(float2* buf, const float2* __restrict__ tw, int tid) {
    constexpr int Q = S / R;
    constexpr int kStep = N / S;        // W_S = W_N^kStep
    for (int b = tid; b < N / R; b += T) {
        const int blk = b / Q, j = b % Q;
        const int base = blk * S + j;
        float2 v[R];
#pragma unroll
        for (int m = 0; m < R; ++m) v[m] = buf[lds_pad(base + m * Q)];
        if (INV && Q > 1) {
#pragma unroll
            for (int r = 1; r < R; ++r) v[r] = cmul_conj(v[r], tw[(j * r * kStep) & (N - 1)]);
        }
        SmallDft<R, INV>::run(v);
        if (!INV && Q > 1) {
#pragma unroll
            for (int r = 1; r < R; ++r) v[r] = cmul(v[r], tw[(j * r * kStep) & (N - 1)]);
        }
#pragma unroll
        for (int m = 0; m < R; ++m) buf[lds_pad(base + m * Q)] = v[m];
    }
}

template <int N, int S, int P, bool INV, int T>
struct Fft16Chain {     // P radix-16 passes left, current block length S
    __device__ static inline void fwd(float2* buf, const float2* tw, int tid) {
        if constexpr (P > 0) {
            fft_pass<N, S, 16, false, T>(buf, tw, tid);
            __syncthreads();
            Fft16Chain<N, S / 16, P - 1, INV, T>::fwd(buf, tw, tid);
        }
    }
    __device__ static inline void inv(float2* buf, const float2* tw, int tid) {
        if constexpr (P > 0) {
            Fft16Chain<N, S / 16, P - 1, INV, T>::inv(buf, tw, tid);
            fft_pass<N, S, 16, true, T>(buf, tw, tid);
            __syncthreads();
        }
    }
};

// Forward transform of buf[lds_pad(0..N)) by the T threads of the work group (all must call).
// Data must be visible (barrier) before the call; results are visible after it.
template <int N, int T>
__device__ inline void fft_forward(float2* buf, const float2* __restrict__ tw, int tid) {
    using Plan = FftPlan<N>;
    Fft16Chain<N, N, Plan::kN16, false, T>::fwd(buf, tw, tid);
    constexpr int S1 = N >> (4 * Plan::kN16);
    if constexpr (Plan::kHas4) {
        fft_pass<N, S1, 4, false, T>(buf, tw, tid);
        __syncthreads();
    }
    if constexpr (Plan::kHas2) {
        constexpr int S2 = Plan::kHas4 ? S1 / 4 : S1;
        fft_pass<N, S2, 2, false, T>(buf, tw, tid);
        __syncthreads();
    }
}

template <int N, int T>
__device__ inline void fft_inverse(float2* buf, const float2* __restrict__ tw, int tid) {
    using Plan = FftPlan<N>;
    constexpr int S1 = N >> (4 * Plan::kN16);
    if constexpr (Plan::kHas2) {
        constexpr int S2 = Plan::kHas4 ? S1 / 4 : S1;
        fft_pass<N, S2, 2, true, T>(buf, tw, tid);
        __syncthreads();
    }
    if constexpr (Plan::kHas4) {
        fft_pass<N, S1, 4, true, T>(buf, tw, tid);
        __syncthreads();
    }
    Fft16Chain<N, N, Plan::kN16, true, T>::inv(buf, tw, tid);
}

}  // namespace aug
