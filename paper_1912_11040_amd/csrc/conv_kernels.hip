// Reverberation and SNR mixing (acoustic simulator, Sec. 2.3).
//
// y_j[n] = sum_{k < L} h_j[k] x_j[n-k] is evaluated by uniformly partitioned
// overlap-save: the response is cut into partitions of P taps, each transformed once
// (2P-point real FFT); an output block of P samples is the inverse transform of
// sum_p X_{b-p} H_p, X_w the transform of input samples [(w-1)P, (w+1)P).
// A 2P-point real transform is run as a P-point complex FFT of the even/odd packed
// sequence, entirely in LDS, split as 16 x P/16: the radix-16 column step reads its inputs
// straight from HBM (and, inverse, writes the block straight back); the 16 row transforms
// run one per wavefront without work-group barriers.
//
// One work group produces one output block of one (utterance, source) and adds the
// block's energy to E[u][j] (fp64 atomics); with several partitions every partition's product goes
// through its own inverse transform and the outputs are summed in registers.  A small kernel forms the
// gains g_j = sqrt(E_0 / (E_j 10^(snr_j/10))); the mixture y_0 + sum_j g_j y_j is written by mix_kernel
// when the caller wants it, and formed by the front end on the fly otherwise.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int conv_threads(int n) { return n / 16; }

__host__ __device__ constexpr int twiddle_count(int n) { return n + n / 2 + 1 + n / 32; }

__global__ void twiddle_kernel(int n, float2* tw) {
    // tw[t] = exp(-2 pi i t / n), t < n;  tw[n + k] = exp(-i pi k / n), k <= n/2;
    // tw[n + n/2 + 1 + j] = exp(-i pi 16 j / n), j < n/32
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= twiddle_count(n)) return;
    double s, c;
    if (i < n) sincospi(-2.0 * (double)i / (double)n, &s, &c);
    else if (i < n + n / 2 + 1) sincospi(-(double)(i - n) / (double)n, &s, &c);
    else sincospi(-16.0 * (double)(i - n - n / 2 - 1) / (double)n, &s, &c);
    tw[i] = make_float2((float)c, (float)s);
}

// Even/odd split of the packed transform: from A = Z[k] and B = conj(Z[N-k]) give
// W[k] and conj(W[N-k]) of the 2N-point real transform; w = exp(-i pi k / N).
__device__ inline void unpack_pair(float2 A, float2 B, float2 w, float2& Wk, float2& WNk_conj) {
    const float2 E = make_float2(0.5f * (A.x + B.x), 0.5f * (A.y + B.y));
    const float2 d = csub(A, B);
    const float2 O = make_float2(0.5f * d.y, -0.5f * d.x);     // -(i/2)(A - B)
    const float2 wO = cmul(w, O);
    Wk = cadd(E, wO);
    WNk_conj = csub(E, wO);
}

// Bins are visited as k = k1 + 16 k2 (row k1, column k2 of the split transform), k < N/2, each with
// its partner N - k.  Thread tid owns column k2 = tid mod M/2 of rows k1 = 8 (tid div M/2) + i.
template <int N>
struct PairIndex {
    static constexpr int M = N / 16;
    int k, pos, pos_partner, h_partner;     // LDS/spectrum position of k and of N-k (spectrum: H[N] sits at N)
    __device__ inline PairIndex(int k1, int k2) {
        k = k1 + 16 * k2;
        pos = k1 * M + k2;
        pos_partner = k1 ? (16 - k1) * M + (M - 1 - k2) : ((M - k2) & (M - 1));
        h_partner = k ? pos_partner : N;
    }
};

template <int N> __device__ inline float2 pair_twiddle(const float2* __restrict__ tw, int k1, int k2) {
    return cmul(tw[N + k1], tw[N + N / 2 + 1 + k2]);           // exp(-i pi (k1 + 16 k2) / N)
}

// Spectrum of one response partition, stored in the split order (k at fft_split_pos(k), k = N last)
// and scaled by 1/N for the unnormalised inverse.
template <int N, int T>
__global__ __launch_bounds__(T) void rir_spectrum_kernel(
    const float* __restrict__ rir, int rir_len, int n_part, const float2* __restrict__ tw,
    float2* __restrict__ spec, int* __restrict__ first_tap) {
    extern __shared__ float2 buf[];
    constexpr int M = N / 16;
    const int tid = threadIdx.x;
    const int r = blockIdx.x / n_part, p = blockIdx.x % n_part;
    const float* h = rir + (size_t)r * rir_len;
    float2 v[16];
    int first = 0x7fffffff;                          // index of this thread's first non-zero tap
#pragma unroll
    for (int n1 = 15; n1 >= 0; --n1) {
        const int n = tid + M * n1;
        const int t = p * N + 2 * n;                 // taps of this partition: [pN, (p+1)N), then N zeros
        float a = 0.f, b = 0.f;
        if (2 * n < N) {
            if (t < rir_len) a = h[t];
            if (t + 1 < rir_len) b = h[t + 1];
        }
        v[n1] = make_float2(a, b);
        if (b != 0.f) first = t + 1;
        if (a != 0.f) first = t;
    }
    // the response is zero before its first non-zero tap, and so is everything convolved with it
    for (int off = 32; off > 0; off >>= 1) first = min(first, __shfl_down(first, off, 64));
    if ((tid & 63) == 0 && first != 0x7fffffff) atomicMin(&first_tap[r], first);
    fft_columns_forward<N>(v, tw, tid);
    fft_columns_store<N, T>(v, buf, tid);
    __syncthreads();
    fft_rows<N, false>(buf, tw, tid);
    __syncthreads();
    float2* out = spec + ((size_t)r * n_part + p) * (N + 1);
    const float scale = 1.0f / (float)N;             // the inverse transform's normalisation
    const int k2 = tid % (M / 2), half = tid / (M / 2);
#pragma unroll
    for (int i = 0; i <= 8; ++i) {
        if (i == 8 && tid != 0) break;
        const PairIndex<N> ix(i == 8 ? 0 : half * 8 + i, i == 8 ? M / 2 : k2);
        const float2 A = buf[lds_pad(ix.pos)];
        const float2 B = cconj(buf[lds_pad(ix.pos_partner)]);
        const float2 w = i == 8 ? tw[N + N / 2] : pair_twiddle<N>(tw, half * 8 + i, k2);
        float2 Hk, HNk_conj;
        unpack_pair(A, B, w, Hk, HNk_conj);
        out[ix.pos] = make_float2(Hk.x * scale, Hk.y * scale);
        if (i < 8) out[ix.h_partner] = make_float2(HNk_conj.x * scale, -HNk_conj.y * scale);
    }
}

// Z'[k] and Z'[N-k] of the packed output block from Z[k] = A, conj(Z[N-k]) = B and the response
// spectrum: Y = W H on the 2N-point real transform, repacked for the N-point inverse.
__device__ inline void multiply_pair(float2 A, float2 B, float2 w, float2 Hk, float2 HNk, float2& Zk, float2& ZNk) {
    float2 Wk, WNk_conj;
    unpack_pair(A, B, w, Wk, WNk_conj);
    const float2 Yk = cmul(Hk, Wk);
    const float2 YNk_conj = cmul_conj(WNk_conj, HNk);
    const float2 Ye = make_float2(0.5f * (Yk.x + YNk_conj.x), 0.5f * (Yk.y + YNk_conj.y));
    const float2 dY = make_float2(0.5f * (Yk.x - YNk_conj.x), 0.5f * (Yk.y - YNk_conj.y));
    const float2 Yo = cmul_conj(dY, w);              // conj(w) (Y[k] - conj Y[N-k]) / 2
    Zk = make_float2(Ye.x - Yo.y, Ye.y + Yo.x);      // Ye + i Yo
    ZNk = make_float2(Ye.x + Yo.y, Yo.x - Ye.y);     // conj(Ye) + i conj(Yo)
}

constexpr int kXcds = 8;

// two consecutive samples; only their 4-byte alignment is promised (global accesses of two dwords need no more)
struct __attribute__((aligned(4))) SamplePair { float x, y; };

// MULTI: the response has several partitions.
template <int N, int T, bool MULTI>
__global__ __launch_bounds__(T) void convolve_kernel(ConvArgs a, const float2* __restrict__ tw) {
    extern __shared__ float2 buf[];
    __shared__ double red[T / 64];
    constexpr int M = N / 16;
    static_assert(T == M, "one thread per column of the split transform");
    const int tid = threadIdx.x;
    // Groups are dealt to the eight XCDs in turn, each with an L2 of its own.  Group ids that share an XCD
    // take one contiguous eighth of the work, so that the blocks of an utterance, which read the same response
    // spectrum and overlapping input windows, meet in one L2.
    const unsigned per_xcd = gridDim.x / kXcds;
    const int64_t work = (int64_t)(blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (work >= a.n_items * a.n_src) return;
    const int64_t item = work / a.n_src;
    const int j = (int)(work % a.n_src);
    const int u = a.items[item].x, b = a.items[item].y;
    const int64_t start = a.offsets[u];
    const int len = (int)(a.offsets[u + 1] - start);      // utterances are shorter than 2^30 samples (checked on the host)
    const float* x = (j == 0 ? a.speech : a.noise + (size_t)(j - 1) * a.total) + start;
    const float2* H = a.spec + ((size_t)u * a.n_src + j) * a.n_part * (size_t)(N + 1);
    const int first = a.first_tap[(size_t)u * a.n_src + j];   // first non-zero tap of the response

    // Responses longer than N taps: every partition p convolves the window p blocks back with its own
    // spectrum and the N output samples are summed in registers (eight complex values per thread), which
    // keeps each pass on the register budget of the single-partition path.
    float2 out[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = make_float2(0.f, 0.f);

    float2 v[16];
    const int n_part = MULTI ? a.n_part : 1;
    for (int p = 0; p < n_part; ++p) {
        const int wb = b - p;                        // input window [(wb-1)N, (wb+1)N)
        if (wb < 0) break;
        // The thread index is made opaque in every round so that twiddle powers and addresses are not
        // hoisted out of the partition loop, where they would sit on top of the transforms' registers.
        int tid_p = tid;
        asm volatile("" : "+v"(tid_p));
        const int k2 = tid_p % (M / 2), half = tid_p / (M / 2);
        const int w0 = (wb - 1) * N + 2 * tid_p;           // first sample of this thread in the window (may be < 0)
        // The window is block wb - 1 followed by block wb.  The first is a whole block of the utterance or
        // (wb = 0) lies before its start; the second is whole except at the utterance's end.  Whole blocks
        // are read with two-sample loads and nothing to test, the same for every thread of the group.
        const float* xw = x + w0;
        if (wb >= 1) {
#pragma unroll
            for (int n1 = 0; n1 < 8; ++n1) {
                const SamplePair s2 = *reinterpret_cast<const SamplePair*>(xw + 2 * M * n1);
                v[n1] = make_float2(s2.x, s2.y);
            }
        } else {
#pragma unroll
            for (int n1 = 0; n1 < 8; ++n1) v[n1] = make_float2(0.f, 0.f);
        }
        if ((wb + 1) * (int64_t)N <= len) {
#pragma unroll
            for (int n1 = 8; n1 < 16; ++n1) {
                const SamplePair s2 = *reinterpret_cast<const SamplePair*>(xw + 2 * M * n1);
                v[n1] = make_float2(s2.x, s2.y);
            }
        } else {
#pragma unroll
            for (int n1 = 8; n1 < 16; ++n1) {
                const int g = w0 + 2 * M * n1;                     // >= 0 in this half
                const float x0 = g < len ? x[g] : 0.f;
                const float x1 = g + 1 < len ? x[g + 1] : 0.f;
                v[n1] = make_float2(x0, x1);
            }
        }
        fft_columns_forward<N>(v, tw, tid_p);
        if (MULTI && p > 0) __syncthreads();         // the previous partition's column loads are done
        fft_columns_store<N, T>(v, buf, tid_p);
        __syncthreads();
        fft_rows<N, false>(buf, tw, tid_p);
        __syncthreads();
        const float2* Hp = H + (size_t)p * (N + 1);
        auto pair = [&](int i) {
            const PairIndex<N> ix(i == 8 ? 0 : half * 8 + i, i == 8 ? M / 2 : k2);
            const float2 A = buf[lds_pad(ix.pos)];
            const float2 B = cconj(buf[lds_pad(ix.pos_partner)]);
            const float2 w = i == 8 ? tw[N + N / 2] : pair_twiddle<N>(tw, half * 8 + i, k2);
            float2 Zk, ZNk;
            multiply_pair(A, B, w, Hp[ix.pos], Hp[ix.h_partner], Zk, ZNk);
            buf[lds_pad(ix.pos)] = Zk;               // both positions belong to this thread alone
            if (ix.k != 0 && i < 8) buf[lds_pad(ix.pos_partner)] = ZNk;
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) pair(i);
        if (tid_p == 0) pair(8);
        __syncthreads();
        fft_rows<N, true>(buf, tw, tid_p);
        __syncthreads();
        fft_columns_load<N, T>(v, buf, tid_p);
        fft_columns_inverse<N>(v, tw, tid_p);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = cadd(out[i], v[8 + i]);
    }

    // the last N real samples of the 2N-sample window are this block's outputs: n = tid + M n1 >= N/2
    float* y = a.reverb + (size_t)j * a.reverb_stride + start;
    // Before the response's first non-zero tap the exact result is zero; the transforms leave rounding noise
    // there, which the power law of the front end would turn into a visible feature value.
    const int out0 = b * N + 2 * tid;
    float e = 0.f;
    if ((b + 1) * (int64_t)N <= len) {               // a full block: eight two-sample stores, nothing to test
        float* yb = y + out0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = out0 + 2 * M * i;
            SamplePair s2;
            s2.x = g >= first ? out[i].x : 0.f;
            s2.y = g + 1 >= first ? out[i].y : 0.f;
            *reinterpret_cast<SamplePair*>(yb + 2 * M * i) = s2;
            e += s2.x * s2.x + s2.y * s2.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = out0 + 2 * M * i;
            const float s0 = g >= first ? out[i].x : 0.f, s1 = g + 1 >= first ? out[i].y : 0.f;
            if (g < len) { y[g] = s0; e += s0 * s0; }
            if (g + 1 < len) { y[g + 1] = s1; e += s1 * s1; }
        }
    }
    double es = (double)e;
    for (int off = 32; off > 0; off >>= 1) es += __shfl_down(es, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = es;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int i = 0; i < T / 64; ++i) tot += red[i];
        atomicAdd(&a.energy[(size_t)u * a.n_src + j], tot);
    }
}

// One thread per (utterance, noise source): the gain that puts the reverberated noise at its target
// SNR against the reverberated speech; zero energy on either side gives gain 0.  (A source whose direct
// path arrives after the utterance has ended has exactly zero energy: the convolution writes exact zeros
// before the response's first non-zero tap.)
__global__ void gain_kernel(int n_utt, int n_src, const double* __restrict__ energy, const float* __restrict__ snr_db,
                            float* __restrict__ gains, float* __restrict__ gains_out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int n_noise = n_src - 1;
    if (i >= n_utt * n_noise) return;
    const int u = i / n_noise, j = 1 + i % n_noise;
    const double e0 = energy[(size_t)u * n_src], ej = energy[(size_t)u * n_src + j];
    const double snr = (double)snr_db[i];
    const float gain = (e0 > 0.0 && ej > 0.0) ? (float)sqrt(e0 / (ej * pow(10.0, snr / 10.0))) : 0.f;
    gains[i] = gain;
    if (gains_out) gains_out[i] = gain;
}

__global__ __launch_bounds__(256) void mix_kernel(
    const int64_t* __restrict__ offsets, int64_t stride, int n_src, const float* __restrict__ reverb,
    const float* __restrict__ gains, float* __restrict__ mixed) {
    const int u = blockIdx.y;
    const int64_t start = offsets[u];
    const int64_t len = offsets[u + 1] - start;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x * 4;
    if (first >= len) return;
    const float* g = gains + (size_t)u * (n_src - 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t n = first + (int64_t)i * blockDim.x + threadIdx.x;
        if (n < len) {
            float acc = reverb[start + n];
            for (int j = 1; j < n_src; ++j) acc += g[j - 1] * reverb[(size_t)j * stride + start + n];
            mixed[start + n] = acc;
        }
    }
}

template <int N>
hipError_t spectrum_n(hipStream_t s, int n_rir, const float* rir, int rir_len, const float2* tw,
                      float2* spec, int* first_tap) {
    constexpr int T = conv_threads(N);
    const int n_part = (rir_len + N - 1) / N;
    const size_t lds = sizeof(float2) * lds_padded_size(N);
    auto k = &rir_spectrum_kernel<N, T>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    k<<<dim3((unsigned)(n_rir * n_part)), dim3(T), lds, s>>>(rir, rir_len, n_part, tw, spec, first_tap);
    return hipGetLastError();
}

template <int N>
hipError_t convolve_n(hipStream_t s, const float2* tw, const ConvArgs& a) {
    constexpr int T = conv_threads(N);
    const size_t lds = sizeof(float2) * lds_padded_size(N);
    auto k = a.n_part > 1 ? &convolve_kernel<N, T, true> : &convolve_kernel<N, T, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int64_t per_xcd = (a.n_items * a.n_src + kXcds - 1) / kXcds;
    k<<<dim3((unsigned)(per_xcd * kXcds)), dim3(T), lds, s>>>(a, tw);
    return hipGetLastError();
}

}  // namespace

int conv_fft_size(int rir_len) {
    int n = 1024;                       // at least one full wave of sixteen-point butterflies
    while (n < rir_len && n < 16384) n <<= 1;
    return n;
}

int twiddle_entries(int n) { return twiddle_count(n); }

hipError_t launch_twiddle(hipStream_t s, int n, float2* tw) {
    const int count = twiddle_count(n);
    twiddle_kernel<<<dim3((count + 255) / 256), dim3(256), 0, s>>>(n, tw);
    return hipGetLastError();
}

#define AUG_FFT_DISPATCH(n, CALL)                                  \
    switch (n) {                                                   \
        case 1024: return CALL(1024);                              \
        case 2048: return CALL(2048);                              \
        case 4096: return CALL(4096);                              \
        case 8192: return CALL(8192);                              \
        case 16384: return CALL(16384);                            \
        default: return hipErrorInvalidValue;                      \
    }

hipError_t launch_rir_spectrum(hipStream_t s, int n_rir, const float* rir, int rir_len, int fft_n,
                               const float2* twiddle, float2* spec, int* first_tap) {
    if (n_rir <= 0) return hipSuccess;
#define CALL(NN) spectrum_n<NN>(s, n_rir, rir, rir_len, twiddle, spec, first_tap)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_convolve(hipStream_t s, int fft_n, const float2* twiddle, const ConvArgs& a) {
    if (a.n_items <= 0) return hipSuccess;
#define CALL(NN) convolve_n<NN>(s, twiddle, a)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_gains(hipStream_t s, int n_utt, int n_src, const double* energy, const float* snr_db, float* gains,
                        float* gains_out) {
    const int n = n_utt * (n_src - 1);
    if (n <= 0) return hipSuccess;
    gain_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(n_utt, n_src, energy, snr_db, gains,
                                                                         gains_out);
    return hipGetLastError();
}

hipError_t launch_mix(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t stride, int n_src,
                      const float* reverb, const float* gains, float* mixed_out, int64_t max_len) {
    if (n_utt <= 0) return hipSuccess;
    int64_t chunks = (max_len + 1023) / 1024;
    if (chunks < 1) chunks = 1;
    mix_kernel<<<dim3((unsigned)chunks, (unsigned)n_utt), dim3(256), 0, s>>>(
        d_offsets, stride, n_src, reverb, gains, mixed_out);
    return hipGetLastError();
}

}  // namespace aug
