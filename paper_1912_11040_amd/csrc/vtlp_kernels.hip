// Vocal tract length perturbation on the waveform (Sec. 2.3): the utterance is analysed in short
// frames, each frame's spectrum is moved along the frequency axis by the bilinear rule of Eq. (1)
// with the utterance's warp factor, and the frames are overlap-added back into a waveform that the
// acoustic simulator then takes as its input.
//
// What the paper leaves to a cited work is fixed as follows.  Frames of 800 samples (50 ms, the best
// window length of Sec. 3) under the periodic Hann window, every 400 samples, frame t centred on sample
// 400 t, so that each sample lies in two frames whose weights add up to one.  The frame is laid out
// around time zero of a 2048-point transform.  Output bin k' reads the input spectrum, by linear
// interpolation between the two nearest bins, at the frequency that Eq. (1) maps onto k':
//     omega = omega' - 2 atan(a sin omega' / (1 + a cos omega')),  a = 1 - alpha, omega' = 2 pi k' / 2048.
// All 2048 samples of the inverse transform are added at the frame's position.  alpha = 1 returns the input.
//
// One wavefront per frame.  The 2048-point real transform is a 1024-point complex one of the even/odd
// packing, done by 64 lanes with 16 values each in LDS (wave-level fences only); the frame's samples go
// from HBM straight into the first butterflies' registers and the last butterflies' outputs go straight
// to the overlap-add, which uses float atomics in HBM (about five frames meet on a sample).
// Per utterance a table holds, for every output bin, the lower source bin and the interpolation weight;
// both come from fp64 arithmetic so that the choice of the bin pair matches a double-precision evaluation.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int kWin = 800, kHop = 400, kFft = 2048;
constexpr int kN = kFft / 2;                       // complex transform length
constexpr int kBins = kN + 1;                      // real-spectrum bins 0..1024
constexpr int kWaves = 4, kThreads = 64 * kWaves;
constexpr int kFramesPerGroup = 16;
constexpr int kSlot = lds_padded_size(kN) + 2;     // a wavefront's transform buffer plus the slot of bin 1024

// One thread per (utterance, output bin): lower source bin j (as a float, exact) and weight f of bin j + 1.
__global__ void vtlp_table_kernel(int n_utt, const float* __restrict__ alpha, float2* __restrict__ tab) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_utt * kBins) return;
    const int u = i / kBins, k = i % kBins;
    const double a = 1.0 - (double)alpha[u];
    const double w = M_PI * (double)k / (double)kN;
    const double src = w - 2.0 * atan(a * sin(w) / (1.0 + a * cos(w)));
    // fmin/fmax drop a NaN operand, so a warp factor that is not a number cannot produce an index out of range
    const double kappa = fmin(fmax(src * (double)kN / M_PI, 0.0), (double)kN);
    int j = (int)floor(kappa);
    if (j > kN - 1) j = kN - 1;
    tab[i] = make_float2((float)j, (float)(kappa - (double)j));
}

__device__ inline int frame_count(int len) { return len > 0 ? (len - 1) / kHop + 2 : 0; }

// value of output bin q of the warped spectrum; X is in natural order in buf, bin 1024 in the extra slot
__device__ inline float2 warped_bin(const float2* buf, const float2* s_tab, int q) {
    const float2 jf = s_tab[q];
    const int j = (int)jf.x;
    const float2 lo = buf[lds_pad(j)], hi = buf[lds_pad(j + 1)];
    return make_float2(lo.x + jf.y * (hi.x - lo.x), lo.y + jf.y * (hi.y - lo.y));
}

// grid: (frame groups of the longest utterance, utterances); `out` must be zero on entry
__global__ __launch_bounds__(kThreads) void vtlp_resynth_kernel(
    const int64_t* __restrict__ offsets, const float* __restrict__ wave, const float2* __restrict__ tab,
    const float2* __restrict__ tw, float* __restrict__ out) {
    extern __shared__ float2 smem[];
    const int tid = threadIdx.x, wv = tid / 64, lane = tid % 64;
    const int u = blockIdx.y;
    const int64_t start = offsets[u];
    const int len = (int)(offsets[u + 1] - start);      // utterances are shorter than 2^30 samples (checked on the host)
    const int n_frames = frame_count(len);
    const int first = blockIdx.x * kFramesPerGroup;
    if (first >= n_frames) return;                       // the whole group leaves together
    float2* buf = smem + wv * kSlot;
    float2* s_tab = smem + kWaves * kSlot;
    for (int k = tid; k < kBins; k += kThreads) s_tab[k] = tab[(size_t)u * kBins + k];

    // Lane l holds packed inputs m = l + 64 i, i.e. frame offsets tau = 2m, 2m + 1 for m < 200 and
    // tau = 2m - 2048, 2m - 2047 for m >= 824; everything else in the 2048-point buffer is zero.
    // Slots 0..3 are i = 0..3, slots 4..7 are i = 12..15.  The window weight of offset tau is
    // 0.5 + 0.5 cos(pi tau / 400).
    int tau0[8];
    float2 wnd[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int m = lane + 64 * (s < 4 ? s : s + 8);
        const bool used = s < 4 ? m < kHop / 2 : m >= kN - kHop / 2;
        tau0[s] = s < 4 ? 2 * m : 2 * m - kFft;
        wnd[s] = used ? make_float2(0.5f + 0.5f * cospif((float)tau0[s] / (float)kHop),
                                    0.5f + 0.5f * cospif((float)(tau0[s] + 1) / (float)kHop))
                      : make_float2(0.f, 0.f);
    }
    __syncthreads();

    const float* x = wave + start;
    float* y = out + start;
    for (int it = 0; it < kFramesPerGroup / kWaves; ++it) {
        const int t = first + it * kWaves + wv;
        if (t >= n_frames) break;                        // later rounds of this wavefront are past the end too
        const int centre = t * kHop;
        float2 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = make_float2(0.f, 0.f);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int g = centre + tau0[s];
            // a zero window weight marks the inputs this lane does not have; unsigned compares fold g >= 0 in
            const float x0 = (wnd[s].x != 0.f || wnd[s].y != 0.f) && (unsigned)g < (unsigned)len ? x[g] : 0.f;
            const float x1 = (wnd[s].x != 0.f || wnd[s].y != 0.f) && (unsigned)(g + 1) < (unsigned)len ? x[g + 1] : 0.f;
            v[s < 4 ? s : s + 8] = make_float2(x0 * wnd[s].x, x1 * wnd[s].y);
        }
        fft_passes<kN, 64, false, FftSync::Wave>(v, buf, tw, lane);
        fft_store_natural<kN, 64>(v, buf, lane);
        fft_sync<FftSync::Wave>();

        // Packed transform Z -> real spectrum X, in place: with A = Z[k], B = conj Z[N-k], E = (A + B)/2,
        // O = -(i/2)(A - B), w = exp(-i pi k / N):  X[k] = E + w O,  X[N-k] = conj(E - w O).
        // A lane owns the pair (k, N-k); k = 0 yields X[0] and X[N], the latter kept in the extra slot.
        auto unpack = [&](int k) {
            const int kn = (kN - k) & (kN - 1);
            const float2 A = buf[lds_pad(k)], B = cconj(buf[lds_pad(kn)]);
            const float2 w = tw[kN + k];
            const float2 E = make_float2(0.5f * (A.x + B.x), 0.5f * (A.y + B.y));
            const float2 O = make_float2(0.5f * (A.y - B.y), -0.5f * (A.x - B.x));
            const float2 wO = cmul(w, O);
            buf[lds_pad(k)] = cadd(E, wO);
            buf[lds_pad(k ? kn : kN)] = cconj(csub(E, wO));
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) unpack(lane + 64 * i);
        if (lane == 0) unpack(kN / 2);
        fft_sync<FftSync::Wave>();

        // Warped spectrum Y (two interpolated bins per pair), packed for the inverse transform:
        // Ye = (Y[k] + conj Y[N-k])/2, Yo = conj(w) (Y[k] - conj Y[N-k])/2, Z'[k] = Ye + i Yo,
        // Z'[N-k] = conj(Ye) + i conj(Yo).  All reads of X finish before the buffer is overwritten.
        float2 zk[9], zn[9];
        auto pack = [&](int k, int slot) {
            const float2 Yk = warped_bin(buf, s_tab, k), Yn = cconj(warped_bin(buf, s_tab, kN - k));
            const float2 w = tw[kN + k];
            const float2 Ye = make_float2(0.5f * (Yk.x + Yn.x), 0.5f * (Yk.y + Yn.y));
            const float2 dY = make_float2(0.5f * (Yk.x - Yn.x), 0.5f * (Yk.y - Yn.y));
            const float2 Yo = cmul_conj(dY, w);
            zk[slot] = make_float2(Ye.x - Yo.y, Ye.y + Yo.x);
            zn[slot] = make_float2(Ye.x + Yo.y, Yo.x - Ye.y);
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) pack(lane + 64 * i, i);
        if (lane == 0) pack(kN / 2, 8);
        fft_sync<FftSync::Wave>();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = lane + 64 * i;
            buf[lds_pad(k)] = zk[i];
            if (k) buf[lds_pad(kN - k)] = zn[i];
        }
        if (lane == 0) buf[lds_pad(kN / 2)] = zk[8];
        fft_sync<FftSync::Wave>();

        fft_load_natural<kN, 64>(v, buf, lane);
        fft_sync<FftSync::Wave>();
        fft_passes<kN, 64, true, FftSync::Wave>(v, buf, tw, lane);
        // v[i] is packed output m = fft_out_index(lane, i) times N: samples at offsets 2m, 2m + 1 (m < N/2)
        // or 2m - 2048, 2m - 2047 from the frame centre
        const float scale = 1.0f / (float)kN;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = fft_out_index<kN, 64>(lane, i);
            const int g = centre + (m < kN / 2 ? 2 * m : 2 * m - kFft);
            if ((unsigned)g < (unsigned)len) atomicAdd(&y[g], v[i].x * scale);
            if ((unsigned)(g + 1) < (unsigned)len) atomicAdd(&y[g + 1], v[i].y * scale);
        }
        fft_sync<FftSync::Wave>();                       // the next frame reuses the buffer
    }
}

}  // namespace

int vtlp_table_entries() { return kBins; }
int vtlp_fft_size() { return kN; }
bool vtlp_supported(int win, int hop, int nfft) { return win == kWin && hop == kHop && nfft == kFft; }

hipError_t launch_vtlp_table(hipStream_t s, int n_utt, const float* alpha, float2* tab) {
    const int64_t n = (int64_t)n_utt * kBins;
    if (n <= 0) return hipSuccess;
    vtlp_table_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(n_utt, alpha, tab);
    return hipGetLastError();
}

hipError_t launch_vtlp_resynth(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t max_len,
                               const float* wave, const float2* tab, const float2* twiddle, float* out) {
    if (n_utt <= 0 || max_len <= 0) return hipSuccess;
    const int64_t frames = (max_len - 1) / kHop + 2;
    const int64_t groups = (frames + kFramesPerGroup - 1) / kFramesPerGroup;
    const size_t lds = sizeof(float2) * (size_t)(kWaves * kSlot + kBins);
    vtlp_resynth_kernel<<<dim3((unsigned)groups, (unsigned)n_utt), dim3(kThreads), lds, s>>>(
        d_offsets, wave, tab, twiddle, out);
    return hipGetLastError();
}

}  // namespace aug
