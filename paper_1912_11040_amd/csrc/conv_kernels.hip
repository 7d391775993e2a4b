// Reverberation and SNR mixing (acoustic simulator, Sec. 2.3).
//
// y_j[n] = sum_{k < L} h_j[k] x_j[n-k] is evaluated by uniformly partitioned
// overlap-save: the response is cut into partitions of P taps, each transformed once
// (2P-point real FFT); an output block of P samples is the inverse transform of
// sum_p X_{b-p} H_p, X_w the transform of input samples [(w-1)P, (w+1)P).
// A 2P-point real transform is run as a P-point complex FFT of the even/odd packed
// sequence, entirely in LDS; spectra stay in the FFT's digit-reversed order.
//
// One work group produces one output block of one (utterance, source), adds the
// block's energy to E[u][j] (fp64 atomics), and a second kernel forms the gains
// g_j = sqrt(E_0 / (E_j 10^(snr_j/10))) and the mixture y_0 + sum_j g_j y_j.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int conv_threads(int n) { return n / 16 > 1024 ? 1024 : (n / 16 < 64 ? 64 : n / 16); }

__global__ void twiddle_kernel(int n, float2* tw) {
    // tw[t] = exp(-2 pi i t / n), t < n;  tw[n + k] = exp(-i pi k / n), k <= n/2
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n + n / 2 + 1) return;
    double s, c;
    if (i < n) sincospi(-2.0 * (double)i / (double)n, &s, &c);
    else sincospi(-(double)(i - n) / (double)n, &s, &c);
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

template <int N, int T>
__global__ __launch_bounds__(T) void rir_spectrum_kernel(
    const float* __restrict__ rir, int rir_len, int n_part, const float2* __restrict__ tw,
    float2* __restrict__ spec) {
    extern __shared__ float2 buf[];
    const int tid = threadIdx.x;
    const int r = blockIdx.x / n_part, p = blockIdx.x % n_part;
    const float* h = rir + (size_t)r * rir_len;
    for (int n = tid; n < N; n += T) {
        const int i = p * N + 2 * n;                 // taps of this partition: [pN, (p+1)N)
        float a = 0.f, b = 0.f;
        if (2 * n < N) {
            if (i < rir_len) a = h[i];
            if (i + 1 < rir_len) b = h[i + 1];
        }
        buf[lds_pad(n)] = make_float2(a, b);
    }
    __syncthreads();
    fft_forward<N, T>(buf, tw, tid);
    float2* out = spec + ((size_t)r * n_part + p) * (N + 1);
    const float scale = 1.0f / (float)N;             // the inverse transform's normalisation
    for (int k = tid; k <= N / 2; k += T) {
        const float2 A = buf[lds_pad(FftPlan<N>::position(k))];
        const float2 B = cconj(buf[lds_pad(FftPlan<N>::position((N - k) & (N - 1)))]);
        float2 Hk, HNk_conj;
        unpack_pair(A, B, tw[N + k], Hk, HNk_conj);
        out[k] = make_float2(Hk.x * scale, Hk.y * scale);
        out[N - k] = make_float2(HNk_conj.x * scale, -HNk_conj.y * scale);
    }
}

template <int N, int T>
__global__ __launch_bounds__(T) void convolve_kernel(ConvArgs a, const float2* __restrict__ tw) {
    extern __shared__ float2 buf[];
    __shared__ double red[T / 64];
    constexpr int PAIRS = (N / 2) / T;               // bins k = tid + i T, k < N/2, each with N-k
    static_assert(PAIRS >= 1 && PAIRS * T == N / 2, "thread count must divide N/2");
    const int tid = threadIdx.x;
    const int64_t item = blockIdx.x / a.n_src;
    const int j = blockIdx.x % a.n_src;
    const int u = a.items[item].x, b = a.items[item].y;
    const int64_t start = a.offsets[u];
    const int64_t len = a.offsets[u + 1] - start;
    const float* x = (j == 0 ? a.speech : a.noise + (size_t)(j - 1) * a.total) + start;
    const float2* H = a.spec + ((size_t)u * a.n_src + j) * a.n_part * (size_t)(N + 1);

    float2 accK[PAIRS + 1], accN[PAIRS];             // Z'[k], Z'[N-k]; last accK is k = N/2
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) accK[i] = accN[i] = make_float2(0.f, 0.f);
    accK[PAIRS] = make_float2(0.f, 0.f);

    for (int p = 0; p < a.n_part; ++p) {
        const int wb = b - p;                        // input window [(wb-1)N, (wb+1)N)
        if (wb < 0) break;
        const int64_t w0 = ((int64_t)wb - 1) * N;
        for (int n = tid; n < N; n += T) {
            const int64_t g = w0 + 2 * n;
            const float x0 = (g >= 0 && g < len) ? x[g] : 0.f;
            const float x1 = (g + 1 >= 0 && g + 1 < len) ? x[g + 1] : 0.f;
            buf[lds_pad(n)] = make_float2(x0, x1);
        }
        __syncthreads();
        fft_forward<N, T>(buf, tw, tid);
        const float2* Hp = H + (size_t)p * (N + 1);
#pragma unroll
        for (int i = 0; i <= PAIRS; ++i) {
            if (i == PAIRS && tid != 0) break;
            const int k = i == PAIRS ? N / 2 : tid + i * T;
            const float2 A = buf[lds_pad(FftPlan<N>::position(k))];
            const float2 B = cconj(buf[lds_pad(FftPlan<N>::position((N - k) & (N - 1)))]);
            const float2 w = tw[N + k];
            float2 Wk, WNk_conj;
            unpack_pair(A, B, w, Wk, WNk_conj);
            const float2 Yk = cmul(Hp[k], Wk);
            const float2 YNk_conj = cmul_conj(WNk_conj, Hp[N - k]);
            const float2 Ye = make_float2(0.5f * (Yk.x + YNk_conj.x), 0.5f * (Yk.y + YNk_conj.y));
            const float2 dY = make_float2(0.5f * (Yk.x - YNk_conj.x), 0.5f * (Yk.y - YNk_conj.y));
            const float2 Yo = cmul_conj(dY, w);      // conj(w) (Y[k] - conj Y[N-k]) / 2
            accK[i].x += Ye.x - Yo.y;                // Ye + i Yo
            accK[i].y += Ye.y + Yo.x;
            if (i < PAIRS) {                         // conj(Ye) + i conj(Yo)
                accN[i].x += Ye.x + Yo.y;
                accN[i].y += Yo.x - Ye.y;
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
        const int k = tid + i * T;
        buf[lds_pad(FftPlan<N>::position(k))] = accK[i];
        if (k != 0) buf[lds_pad(FftPlan<N>::position(N - k))] = accN[i];
    }
    if (tid == 0) buf[lds_pad(FftPlan<N>::position(N / 2))] = accK[PAIRS];
    __syncthreads();
    fft_inverse<N, T>(buf, tw, tid);

    // the last N real samples of the 2N-sample window are this block's outputs
    float* y = a.reverb + (size_t)j * a.total + start;
    const int64_t out0 = (int64_t)b * N;
    float e = 0.f;
    for (int n = tid; n < N / 2; n += T) {
        const float2 v = buf[lds_pad(N / 2 + n)];
        const int64_t g = out0 + 2 * n;
        if (g < len) { y[g] = v.x; e += v.x * v.x; }
        if (g + 1 < len) { y[g + 1] = v.y; e += v.y * v.y; }
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

__global__ __launch_bounds__(256) void mix_kernel(
    const int64_t* __restrict__ offsets, int64_t total, int n_src, const float* __restrict__ reverb,
    const double* __restrict__ energy, const float* __restrict__ snr_db, float* __restrict__ mixed,
    float* __restrict__ gains_out) {
    __shared__ float g[AUG_MAX_NOISE + 1];
    const int u = blockIdx.y;
    const int64_t start = offsets[u];
    const int64_t len = offsets[u + 1] - start;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x * 4;
    if (first >= len && !(blockIdx.x == 0)) return;
    if (threadIdx.x < n_src) {
        float gain = 1.f;
        if (threadIdx.x > 0) {
            const double e0 = energy[(size_t)u * n_src];
            const double ej = energy[(size_t)u * n_src + threadIdx.x];
            const double snr = (double)snr_db[(size_t)u * (n_src - 1) + threadIdx.x - 1];
            gain = (e0 > 0.0 && ej > 0.0) ? (float)sqrt(e0 / (ej * pow(10.0, snr / 10.0))) : 0.f;
            if (blockIdx.x == 0 && gains_out) gains_out[(size_t)u * (n_src - 1) + threadIdx.x - 1] = gain;
        }
        g[threadIdx.x] = gain;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t n = first + (int64_t)i * blockDim.x + threadIdx.x;
        if (n < len) {
            float acc = reverb[start + n];
            for (int j = 1; j < n_src; ++j) acc += g[j] * reverb[(size_t)j * total + start + n];
            mixed[start + n] = acc;
        }
    }
}

template <int N>
hipError_t spectrum_n(hipStream_t s, int n_rir, const float* rir, int rir_len, const float2* tw,
                      float2* spec) {
    constexpr int T = conv_threads(N);
    const int n_part = (rir_len + N - 1) / N;
    const size_t lds = sizeof(float2) * lds_padded_size(N);
    auto k = &rir_spectrum_kernel<N, T>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    k<<<dim3((unsigned)(n_rir * n_part)), dim3(T), lds, s>>>(rir, rir_len, n_part, tw, spec);
    return hipGetLastError();
}

template <int N>
hipError_t convolve_n(hipStream_t s, const float2* tw, const ConvArgs& a) {
    constexpr int T = conv_threads(N);
    const size_t lds = sizeof(float2) * lds_padded_size(N);
    auto k = &convolve_kernel<N, T>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    k<<<dim3((unsigned)(a.n_items * a.n_src)), dim3(T), lds, s>>>(a, tw);
    return hipGetLastError();
}

}  // namespace

int conv_fft_size(int rir_len) {
    int n = 256;
    while (n < rir_len && n < 16384) n <<= 1;
    return n;
}

hipError_t launch_twiddle(hipStream_t s, int n, float2* tw) {
    const int count = n + n / 2 + 1;
    twiddle_kernel<<<dim3((count + 255) / 256), dim3(256), 0, s>>>(n, tw);
    return hipGetLastError();
}

#define AUG_FFT_DISPATCH(n, CALL)                                  \
    switch (n) {                                                   \
        case 256: return CALL(256);                                \
        case 512: return CALL(512);                                \
        case 1024: return CALL(1024);                              \
        case 2048: return CALL(2048);                              \
        case 4096: return CALL(4096);                              \
        case 8192: return CALL(8192);                              \
        case 16384: return CALL(16384);                            \
        default: return hipErrorInvalidValue;                      \
    }

hipError_t launch_rir_spectrum(hipStream_t s, int n_rir, const float* rir, int rir_len, int fft_n,
                               const float2* twiddle, float2* spec) {
    if (n_rir <= 0) return hipSuccess;
#define CALL(NN) spectrum_n<NN>(s, n_rir, rir, rir_len, twiddle, spec)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_convolve(hipStream_t s, int fft_n, const float2* twiddle, const ConvArgs& a) {
    if (a.n_items <= 0) return hipSuccess;
#define CALL(NN) convolve_n<NN>(s, twiddle, a)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_mix(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t total, int n_src,
                      const float* reverb, const double* energy, const float* snr_db,
                      float* mixed_out, float* gains_out, int64_t max_len) {
    if (n_utt <= 0) return hipSuccess;
    int64_t chunks = (max_len + 1023) / 1024;
    if (chunks < 1) chunks = 1;
    mix_kernel<<<dim3((unsigned)chunks, (unsigned)n_utt), dim3(256), 0, s>>>(
        d_offsets, total, n_src, reverb, energy, snr_db, mixed_out, gains_out);
    return hipGetLastError();
}

}  // namespace aug
