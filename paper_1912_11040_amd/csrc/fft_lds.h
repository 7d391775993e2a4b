// Complex FFT of a power-of-two length N held in LDS and worked on by T = N/16 threads,
// shared by the overlap-save convolution (N = 256..16384) and the STFT (N = nfft/2).
//
// Stockham autosort passes: a pass of radix R over sub-transforms of length NS reads, for
// butterfly j < N/R, x[j + m N/R] (m < R), multiplies by exp(-+2 pi i (j mod NS) m / (NS R)),
// takes an R-point DFT and writes y[(j div NS) NS R + (j mod NS) + r NS].  Input and output
// are in natural order.  The transform runs in place: every thread keeps its 16 values of a
// pass in registers, so all reads of a pass complete (barrier) before its writes begin.
// Radix 16 while four or more bits remain, then radix 4 and/or 2.
//
// Twiddles: one table value w = exp(-2 pi i t / N) per butterfly; its powers are formed by
// at most four successive complex products.  The inverse uses conjugates and is unscaled.
//
// Synchronisation between the reads and writes of a pass is a work-group barrier, or, when all
// threads of one transform sit in one wavefront, only a wave-level fence (LDS operations of a wave
// complete in order).  Large transforms are split as N = 16 x M: one radix-16 step across the
// group, then 16 independent M-point row transforms of at most 64 lanes each, which need no
// barriers and so overlap each other's LDS and ALU phases (see fft_columns_*).
//
// LDS addressing is padded by one complex per 16 (element i lives at lds_pad(i)) so that both
// the unit-stride reads and the stride-NS writes of every pass spread over all banks.
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

// R-point DFT of v[0..R), natural order in and out.
template <int R, bool INV> struct SmallDft;

template <bool INV> struct SmallDft<2, INV> {
    __device__ static inline void run(float2* v) {
        const float2 a = v[0], b = v[1];
        v[0] = cadd(a, b);
        v[1] = csub(a, b);
    }
};

template <bool INV> struct SmallDft<4, INV> {
    __device__ static inline void run(float2* v) { dft4<INV>(v[0], v[1], v[2], v[3]); }
};

template <bool INV> struct SmallDft<16, INV> {
    // m = m2 + 4 m1, r = r1 + 4 r2:
    // y[r1 + 4 r2] = sum_{m2} W4^{m2 r2} W16^{m2 r1} sum_{m1} x[m2 + 4 m1] W4^{m1 r1}
    __device__ static inline void run(float2* v) {
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
        for (int r1 = 0; r1 < 4; ++r1)
            dft4<INV>(v[4 * r1 + 0], v[4 * r1 + 1], v[4 * r1 + 2], v[4 * r1 + 3]);  // v[4 r1 + r2] = y[r1 + 4 r2]
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

// v[m] *= w^m for m = 1..R-1, powers by products of depth <= 4
template <int R> __device__ inline void twiddle_inputs(float2* v, float2 w1) {
    if constexpr (R == 2) {
        v[1] = cmul(v[1], w1);
    } else if constexpr (R == 4) {
        const float2 w2 = cmul(w1, w1), w3 = cmul(w2, w1);
        v[1] = cmul(v[1], w1);
        v[2] = cmul(v[2], w2);
        v[3] = cmul(v[3], w3);
    } else {
        static_assert(R == 16, "radix");
        // powers are formed and used in an order that keeps few of them alive: w1..w8, then w8 w_m
        const float2 w2 = cmul(w1, w1);
        const float2 w3 = cmul(w2, w1);
        const float2 w4 = cmul(w2, w2);
        v[1] = cmul(v[1], w1);
        v[2] = cmul(v[2], w2);
        v[3] = cmul(v[3], w3);
        v[4] = cmul(v[4], w4);
        const float2 w5 = cmul(w4, w1);
        const float2 w6 = cmul(w4, w2);
        const float2 w7 = cmul(w4, w3);
        const float2 w8 = cmul(w4, w4);
        v[5] = cmul(v[5], w5);
        v[6] = cmul(v[6], w6);
        v[7] = cmul(v[7], w7);
        v[8] = cmul(v[8], w8);
        v[9] = cmul(v[9], cmul(w8, w1));
        v[10] = cmul(v[10], cmul(w8, w2));
        v[11] = cmul(v[11], cmul(w8, w3));
        v[12] = cmul(v[12], cmul(w8, w4));
        v[13] = cmul(v[13], cmul(w8, w5));
        v[14] = cmul(v[14], cmul(w8, w6));
        v[15] = cmul(v[15], cmul(w8, w7));
    }
}

constexpr int ilog2(int n) { return n <= 1 ? 0 : 1 + ilog2(n >> 1); }

template <int N>
struct FftPlan {
    static constexpr int kLog = ilog2(N);
    static constexpr int kN16 = kLog / 4;
    static constexpr int kRem = kLog % 4;
    static constexpr int kPasses = kN16 + (kRem >= 2 ? 1 : 0) + (kRem & 1);
    static constexpr int radix(int p) { return p < kN16 ? 16 : ((p == kN16 && kRem >= 2) ? 4 : 2); }
    static constexpr int ns(int p) {
        int s = 1;
        for (int i = 0; i < p; ++i) s *= radix(i);
        return s;
    }
    static constexpr int kLastRadix = radix(kPasses - 1);
};

// lds_pad(a + b) = lds_pad(a) + lds_pad(b) whenever b is a multiple of 16; the address code below
// uses this to keep one padded base per thread plus compile-time offsets.

// Each thread owns 16 values per pass: 16 / R butterflies j = tid + bi T.
template <int N, int T, int R>
__device__ inline void fft_load(float2 (&v)[16], const float2* buf, int tid) {
    static_assert(N == 16 * T, "sixteen values per thread");
    if constexpr (T % 16 == 0 && (N / R) % 16 == 0) {
        const float2* base = buf + lds_pad(tid);
#pragma unroll
        for (int bi = 0; bi < 16 / R; ++bi)
#pragma unroll
            for (int m = 0; m < R; ++m) v[bi * R + m] = base[lds_pad(bi * T + m * (N / R))];
    } else {
#pragma unroll
        for (int bi = 0; bi < 16 / R; ++bi)
#pragma unroll
            for (int m = 0; m < R; ++m) v[bi * R + m] = buf[lds_pad(tid + bi * T + m * (N / R))];
    }
}

template <int N, int T, int R, int NS>
__device__ inline void fft_store(const float2 (&v)[16], float2* buf, int tid) {
#pragma unroll
    for (int bi = 0; bi < 16 / R; ++bi) {
        const int j = tid + bi * T;
        const int k = j % NS;
        const int j0 = (j / NS) * NS * R + k;
        if constexpr (NS % 16 == 0) {
            float2* base = buf + lds_pad(j0);
#pragma unroll
            for (int r = 0; r < R; ++r) base[lds_pad(r * NS)] = v[bi * R + r];
        } else if constexpr (NS == 1 && R == 16) {
            float2* base = buf + 17 * j;                 // lds_pad(16 j + r) = 17 j + r
#pragma unroll
            for (int r = 0; r < R; ++r) base[r] = v[bi * R + r];
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) buf[lds_pad(j0 + r * NS)] = v[bi * R + r];
        }
    }
}

enum class FftSync { Group, Wave };

template <FftSync S> __device__ inline void fft_sync() {
    if constexpr (S == FftSync::Group) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// TWS: the table holds exp(-2 pi i t / (N TWS)), i.e. it was built for a TWS times longer transform.
template <int N, int T, int R, int NS, bool INV, int TWS>
__device__ inline void fft_compute(float2 (&v)[16], const float2* __restrict__ tw, int tid) {
#pragma unroll
    for (int bi = 0; bi < 16 / R; ++bi) {
        if constexpr (NS > 1) {
            const int k = (tid + bi * T) % NS;
            float2 w1 = tw[k * (N / (NS * R)) * TWS];
            if (INV) w1.y = -w1.y;
            twiddle_inputs<R>(&v[bi * R], w1);
        }
        SmallDft<R, INV>::run(&v[bi * R]);
    }
}

// Natural index of value v[bi R + r] after the last pass, and before the first pass of input v[bi R + m].
template <int N, int T>
__device__ inline int fft_out_index(int tid, int i) {
    constexpr int R = FftPlan<N>::kLastRadix;
    return tid + (i / R) * T + (i % R) * (N / R);
}
template <int N, int T>
__device__ inline int fft_in_index(int tid, int i) {
    constexpr int R = FftPlan<N>::radix(0);
    return tid + (i / R) * T + (i % R) * (N / R);
}

// Run passes P.. of the transform.  On entry v holds the inputs of pass P (fft_in_index order for
// P = 0); on return it holds the outputs of the last pass (fft_out_index order), not yet stored.
// All T threads of the group must call; buf contents are overwritten.
template <int N, int T, bool INV, FftSync S = FftSync::Group, int TWS = 1, int P = 0>
__device__ inline void fft_passes(float2 (&v)[16], float2* buf, const float2* __restrict__ tw, int tid) {
    using Plan = FftPlan<N>;
    constexpr int R = Plan::radix(P), NS = Plan::ns(P);
    fft_compute<N, T, R, NS, INV, TWS>(v, tw, tid);
    if constexpr (P + 1 < Plan::kPasses) {
        fft_store<N, T, R, NS>(v, buf, tid);
        fft_sync<S>();
        fft_load<N, T, Plan::radix(P + 1)>(v, buf, tid);
        fft_sync<S>();
        fft_passes<N, T, INV, S, TWS, P + 1>(v, buf, tw, tid);
    }
}

// The base twiddle of every butterfly a thread computes, fetched once.  A thread that repeats the same
// transform with the same tid (one frame after another) keeps them in registers, which takes the table
// loads, and their latency, out of its loop.
template <int N, int T>
struct FftLaneTwiddles {
    using Plan = FftPlan<N>;
    float2 w[Plan::kPasses][8];
    template <int P = 0> __device__ inline void load(const float2* __restrict__ tw, int tid) {
        if constexpr (P < Plan::kPasses) {
            constexpr int R = Plan::radix(P), NS = Plan::ns(P);
            if constexpr (NS > 1) {
#pragma unroll
                for (int bi = 0; bi < 16 / R; ++bi) w[P][bi] = tw[((tid + bi * T) % NS) * (N / (NS * R))];
            }
            load<P + 1>(tw, tid);
        }
    }
    // Hides the values from the optimiser inside a loop: otherwise every power of every twiddle is also
    // hoisted out of the loop and the register file overflows.
    template <int P = 0> __device__ inline void keep_in_loop() {
        if constexpr (P < Plan::kPasses) {
            if constexpr (Plan::ns(P) > 1) {
#pragma unroll
                for (int bi = 0; bi < 16 / Plan::radix(P); ++bi) asm volatile("" : "+v"(w[P][bi].x), "+v"(w[P][bi].y));
            }
            keep_in_loop<P + 1>();
        }
    }
};

// fft_passes with the thread's twiddles supplied from registers
template <int N, int T, bool INV, FftSync S, int P = 0>
__device__ inline void fft_passes_cached(float2 (&v)[16], float2* buf, const FftLaneTwiddles<N, T>& lt, int tid) {
    using Plan = FftPlan<N>;
    constexpr int R = Plan::radix(P), NS = Plan::ns(P);
#pragma unroll
    for (int bi = 0; bi < 16 / R; ++bi) {
        if constexpr (NS > 1) {
            float2 w1 = lt.w[P][bi];
            if (INV) w1.y = -w1.y;
            twiddle_inputs<R>(&v[bi * R], w1);
        }
        SmallDft<R, INV>::run(&v[bi * R]);
    }
    if constexpr (P + 1 < Plan::kPasses) {
        fft_store<N, T, R, NS>(v, buf, tid);
        fft_sync<S>();
        fft_load<N, T, Plan::radix(P + 1)>(v, buf, tid);
        fft_sync<S>();
        fft_passes_cached<N, T, INV, S, P + 1>(v, buf, lt, tid);
    }
}

// Store the last pass's outputs in natural order.
template <int N, int T>
__device__ inline void fft_store_natural(const float2 (&v)[16], float2* buf, int tid) {
    constexpr int R = FftPlan<N>::kLastRadix;
    if constexpr (T % 16 == 0 && (N / R) % 16 == 0) {
        float2* base = buf + lds_pad(tid);
#pragma unroll
        for (int i = 0; i < 16; ++i) base[lds_pad((i / R) * T + (i % R) * (N / R))] = v[i];
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) buf[lds_pad(fft_out_index<N, T>(tid, i))] = v[i];
    }
}

// Load the first pass's inputs from a natural-order buffer.
template <int N, int T>
__device__ inline void fft_load_natural(float2 (&v)[16], const float2* buf, int tid) {
    constexpr int R = FftPlan<N>::radix(0);
    if constexpr (T % 16 == 0 && (N / R) % 16 == 0) {
        const float2* base = buf + lds_pad(tid);
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = base[lds_pad((i / R) * T + (i % R) * (N / R))];
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = buf[lds_pad(fft_in_index<N, T>(tid, i))];
    }
}

// ---- N = 16 x M split -------------------------------------------------------------------
// X[k1 + 16 k2] = sum_{n2 < M} W_M^{n2 k2} W_N^{n2 k1} sum_{n1 < 16} x[n2 + M n1] W_16^{n1 k1}.
// Thread n2 of the M = N/16 threads holds x[n2 + M n1] in v[n1]; after the column step v[k1] belongs
// to row k1, column n2.  Row k1 lives at buf[lds_pad(k1 M + .)] and is transformed by M/16 lanes of
// one wavefront.  After the forward transform frequency k = k1 + 16 k2 sits at row k1, column k2.

template <int N> __device__ __host__ constexpr int fft_split_pos(int k) { return (k & 15) * (N / 16) + (k >> 4); }

// forward column step on registers: v[n1] -> v[k1] (twiddled), to be stored at row k1, column n2
template <int N>
__device__ inline void fft_columns_forward(float2 (&v)[16], const float2* __restrict__ tw, int n2) {
    SmallDft<16, false>::run(v);
    twiddle_inputs<16>(v, tw[n2]);
}

// inverse column step: v[k1] (row k1, column n2) -> v[n1] = N x[n2 + M n1]
template <int N>
__device__ inline void fft_columns_inverse(float2 (&v)[16], const float2* __restrict__ tw, int n2) {
    float2 w1 = tw[n2];
    w1.y = -w1.y;
    twiddle_inputs<16>(v, w1);
    SmallDft<16, true>::run(v);
}

template <int N, int T>
__device__ inline void fft_columns_store(const float2 (&v)[16], float2* buf, int n2) {
    static_assert((N / 16) % 16 == 0, "rows are whole padding groups");
    float2* base = buf + lds_pad(n2);
#pragma unroll
    for (int k1 = 0; k1 < 16; ++k1) base[lds_pad(k1 * (N / 16))] = v[k1];
}
template <int N, int T>
__device__ inline void fft_columns_load(float2 (&v)[16], const float2* buf, int n2) {
    const float2* base = buf + lds_pad(n2);
#pragma unroll
    for (int k1 = 0; k1 < 16; ++k1) v[k1] = base[lds_pad(k1 * (N / 16))];
}

// ---- row-pass twiddles with their powers, held in LDS ---------------------------------------
// A persistent kernel fills the table once and its row transforms then read every factor they need
// (pass P of radix R and sub-length NS: exp(-2 pi i k m / (NS R)) at [k][m - 1], k < NS, m = 1..R-1) instead of
// loading one factor from global memory and forming its powers by chained products.  That removes the
// products, and it removes global loads from the row transforms, so loads issued ahead of them are not
// waited for there (a wave's global loads complete in order).
template <int M>
struct RowTwiddles {
    using Plan = FftPlan<M>;
    static constexpr int offset(int p) {
        int o = 0;
        for (int q = 1; q < p; ++q) o += Plan::ns(q) * (Plan::radix(q) - 1);
        return o;
    }
    static constexpr int kEntries = offset(Plan::kPasses);
    // tw: exp(-2 pi i t / (M TWS)); all threads of the group call, then synchronise
    template <int TWS, int P = 1>
    __device__ static inline void fill(float2* tab, const float2* __restrict__ tw, int tid, int n_threads) {
        if constexpr (P < Plan::kPasses) {
            constexpr int R = Plan::radix(P), NS = Plan::ns(P);
            for (int e = tid; e < NS * (R - 1); e += n_threads) {
                const int k = e / (R - 1), m = e % (R - 1) + 1;
                tab[offset(P) + e] = tw[k * m * (M / (NS * R)) * TWS];
            }
            fill<TWS, P + 1>(tab, tw, tid, n_threads);
        }
    }
};

// fft_passes with every twiddle factor read from a RowTwiddles table in LDS
template <int M, int T, bool INV, FftSync S, int P = 0>
__device__ inline void fft_passes_table(float2 (&v)[16], float2* buf, const float2* tab, int tid) {
    using Plan = FftPlan<M>;
    constexpr int R = Plan::radix(P), NS = Plan::ns(P);
#pragma unroll
    for (int bi = 0; bi < 16 / R; ++bi) {
        if constexpr (NS > 1) {
            const float2* e = tab + RowTwiddles<M>::offset(P) + ((tid + bi * T) % NS) * (R - 1);
#pragma unroll
            for (int m = 1; m < R; ++m)
                v[bi * R + m] = INV ? cmul_conj(v[bi * R + m], e[m - 1]) : cmul(v[bi * R + m], e[m - 1]);
        }
        SmallDft<R, INV>::run(&v[bi * R]);
    }
    if constexpr (P + 1 < Plan::kPasses) {
        fft_store<M, T, R, NS>(v, buf, tid);
        fft_sync<S>();
        fft_load<M, T, Plan::radix(P + 1)>(v, buf, tid);
        fft_sync<S>();
        fft_passes_table<M, T, INV, S, P + 1>(v, buf, tab, tid);
    }
}

// The 16 row transforms, in place in natural order within each row; wave-level synchronisation only.
// Thread tid works on row tid / (M/16) as lane tid % (M/16).  Rows must be complete (barrier) before.
template <int N, bool INV>
__device__ inline void fft_rows(float2* buf, const float2* __restrict__ tw, int tid) {
    constexpr int M = N / 16, LANES = M / 16;
    static_assert(LANES >= 1 && LANES <= 64, "a row is transformed inside one wavefront");
    float2* row = buf + lds_pad((tid / LANES) * M);
    const int lane = tid % LANES;
    float2 v[16];
    fft_load_natural<M, LANES>(v, row, lane);
    fft_sync<FftSync::Wave>();
    fft_passes<M, LANES, INV, FftSync::Wave, 16>(v, row, tw, lane);
    fft_store_natural<M, LANES>(v, row, lane);
}

// the same with the twiddles of a RowTwiddles<N / 16> table
template <int N, bool INV>
__device__ inline void fft_rows_table(float2* buf, const float2* tab, int tid) {
    constexpr int M = N / 16, LANES = M / 16;
    static_assert(LANES >= 1 && LANES <= 64, "a row is transformed inside one wavefront");
    float2* row = buf + lds_pad((tid / LANES) * M);
    const int lane = tid % LANES;
    float2 v[16];
    fft_load_natural<M, LANES>(v, row, lane);
    fft_sync<FftSync::Wave>();
    fft_passes_table<M, LANES, INV, FftSync::Wave>(v, row, tab, lane);
    fft_store_natural<M, LANES>(v, row, lane);
}

}  // namespace aug
