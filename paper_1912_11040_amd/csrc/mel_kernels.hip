// Front end (Sec. 2.3): framed power spectrum, VTLP-warped mel filterbank, power law.
//
// P_t[k] = |DFT_K(hamming * x[t hop .. t hop + win))[k]|^2, k = 0..K/2;
// E_t[m] = sum_k Tri_m(f'_k) P_t[k] with f'_k the Eq. (1) bilinear warp of bin k;
// feature = E^(power).
//
// Adjacent unit-peak triangles share their edges, so a bin whose warped frequency
// falls between band edges c and c+1 feeds only filter c (rising side, weight w) and
// filter c-1 (falling side, weight 1-w).  A small kernel writes (c, w) per bin and
// utterance; the main kernel runs each K-point real transform as a K/2-point complex
// FFT in LDS (16 lanes per frame, two radix-16 passes), then scatters the power of
// each bin into its two mel channels.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int kMelThreads = 256;
constexpr int kFramesPerGroup = 64;

__global__ void window_kernel(int win, float* w) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= win) return;
    double s, c;
    sincospi(2.0 * (double)i / (double)(win - 1), &s, &c);
    w[i] = (float)(0.54 - 0.46 * c);
}

__global__ void mel_table_kernel(int n_utt, const float* __restrict__ alpha, aug_frontend_cfg cfg,
                                 float2* __restrict__ tab) {
    const int bins = cfg.nfft / 2 + 1;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_utt * bins) return;
    const int u = i / bins, k = i % bins;
    const double a = 1.0 - (double)alpha[u];
    double sn, cs;
    sincospi(2.0 * (double)k / (double)cfg.nfft, &sn, &cs);
    const double omega = 2.0 * M_PI * (double)k / (double)cfg.nfft;
    const double warped = omega + 2.0 * atan(a * sn / (1.0 - a * cs));          // Eq. (1)
    const double f = warped * (double)cfg.fs / (2.0 * M_PI);
    const double mel_lo = 2595.0 * log10(1.0 + (double)cfg.f_lo / 700.0);
    const double mel_hi = 2595.0 * log10(1.0 + (double)cfg.f_hi / 700.0);
    const double step = (mel_hi - mel_lo) / (double)(cfg.n_mel + 1);
    const double mel = 2595.0 * log10(1.0 + f / 700.0);
    float ch = -2.f, wgt = 0.f;
    if (f >= (double)cfg.f_lo && f <= (double)cfg.f_hi) {
        int c = (int)floor((mel - mel_lo) / step);
        c = c < 0 ? 0 : (c > cfg.n_mel ? cfg.n_mel : c);
        const double e0 = 700.0 * (pow(10.0, (mel_lo + c * step) / 2595.0) - 1.0);
        const double e1 = 700.0 * (pow(10.0, (mel_lo + (c + 1) * step) / 2595.0) - 1.0);
        double w = (f - e0) / (e1 - e0);
        w = w < 0.0 ? 0.0 : (w > 1.0 ? 1.0 : w);
        ch = (float)c;
        wgt = (float)w;
    }
    tab[i] = make_float2(ch, wgt);
}

// K = 512: 256-point complex FFT per frame, 16 lanes per frame, 16 frames per pass of the group.
template <int NC>
__global__ __launch_bounds__(kMelThreads) void mel_kernel(MelArgs a, const float2* __restrict__ tw) {
    constexpr int kLanes = NC / 16;                      // lanes per frame
    constexpr int kSlots = kMelThreads / kLanes;         // frames in flight
    constexpr int kBinsPerLane = NC / kLanes;            // contiguous bins per lane (16)
    __shared__ float2 fft_buf[kSlots][lds_padded_size(NC)];
    __shared__ float mel_acc[kSlots][AUG_MAX_MEL];

    const int tid = threadIdx.x;
    const int slot = tid / kLanes, sub = tid % kLanes;
    const int u = a.items[blockIdx.x].x;
    const int first = a.items[blockIdx.x].y;
    const int64_t start = a.offsets[u];
    const int64_t n_frames_u = a.frame_offsets[u + 1] - a.frame_offsets[u];
    const float* x = a.wave + start;
    const float2* tab = a.mel_tab + (size_t)u * (NC + 1);
    const int win = a.cfg.win, hop = a.cfg.hop, n_mel = a.cfg.n_mel;
    float* feats = a.feats + (size_t)a.frame_offsets[u] * n_mel;
    float2* buf = fft_buf[slot];
    float* acc = mel_acc[slot];

    // this lane's window samples never change: z[n] = w[2n] x[2n] + i w[2n+1] x[2n+1], n = sub + 16 m
    float2 wnd[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int i0 = 2 * fft_in_index<NC, kLanes>(sub, i);
        wnd[i] = make_float2(i0 < win ? a.window[i0] : 0.f, i0 + 1 < win ? a.window[i0 + 1] : 0.f);
    }

    for (int it = 0; it < a.frames_per_group / kSlots; ++it) {
        const int64_t t = (int64_t)first + it * kSlots + slot;
        const bool live = t < n_frames_u;
        float2 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int i0 = 2 * fft_in_index<NC, kLanes>(sub, i);
            float re = 0.f, im = 0.f;
            if (live) {
                if (i0 < win) re = x[t * hop + i0] * wnd[i].x;
                if (i0 + 1 < win) im = x[t * hop + i0 + 1] * wnd[i].y;
            }
            v[i] = make_float2(re, im);
        }
        for (int m = sub; m < n_mel; m += kLanes) acc[m] = 0.f;
        fft_passes<NC, kLanes, false>(v, buf, tw, sub);
        fft_store_natural<NC, kLanes>(v, buf, sub);
        __syncthreads();

        // bins sub*16 .. sub*16+15, and bin NC on the last lane
        for (int i = 0; i < kBinsPerLane + 1; ++i) {
            if (i == kBinsPerLane && sub != kLanes - 1) break;
            const int k = i == kBinsPerLane ? NC : sub * kBinsPerLane + i;
            const int kk = k & (NC - 1);
            const float2 A = buf[lds_pad(kk)];
            const float2 Bc = buf[lds_pad((NC - kk) & (NC - 1))];
            const float2 w = k <= NC / 2 ? tw[NC + k]
                                         : make_float2(-tw[NC + (NC - k)].x, tw[NC + (NC - k)].y);
            // X[k] = E + w O,  E = (A + conj B)/2,  O = -(i/2)(A - conj B)
            const float2 E = make_float2(0.5f * (A.x + Bc.x), 0.5f * (A.y - Bc.y));
            const float2 d = make_float2(A.x - Bc.x, A.y + Bc.y);
            const float2 O = make_float2(0.5f * d.y, -0.5f * d.x);
            const float2 X = cadd(E, cmul(w, O));
            const float p = X.x * X.x + X.y * X.y;
            const float2 cw = tab[k];
            const int c = (int)cw.x;
            if (c >= 0 && c < n_mel) atomicAdd(&acc[c], cw.y * p);
            if (c >= 1 && c <= n_mel) atomicAdd(&acc[c - 1], (1.f - cw.y) * p);
        }
        __syncthreads();
        if (live) {
            for (int m = sub; m < n_mel; m += kLanes) {
                const float e = acc[m];
                feats[t * n_mel + m] = e > 0.f ? powf(e, a.cfg.power) : 0.f;
            }
        }
        __syncthreads();
    }
}

}  // namespace

int mel_frames_per_group() { return kFramesPerGroup; }

hipError_t launch_window(hipStream_t s, int win, float* w) {
    window_kernel<<<dim3((win + 255) / 256), dim3(256), 0, s>>>(win, w);
    return hipGetLastError();
}

hipError_t launch_mel_table(hipStream_t s, int n_utt, const float* alpha, const aug_frontend_cfg& cfg,
                            float2* tab) {
    const int64_t n = (int64_t)n_utt * (cfg.nfft / 2 + 1);
    if (n <= 0) return hipSuccess;
    mel_table_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(n_utt, alpha, cfg, tab);
    return hipGetLastError();
}

hipError_t launch_mel(hipStream_t s, const MelArgs& a) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.cfg.nfft != 512) return hipErrorInvalidValue;
    mel_kernel<256><<<dim3((unsigned)a.n_items), dim3(kMelThreads), 0, s>>>(a, a.twiddle);
    return hipGetLastError();
}

}  // namespace aug
