// Vocal tract length perturbation on the waveform (Sec. 2.3): the utterance is analysed in short
// frames, each frame's spectrum is moved along the frequency axis by the bilinear rule of Eq. (1)
// with the utterance's warp factor, and the frames are overlap-added back into a waveform that the
// acoustic simulator then takes as its input.
//
// What the paper leaves to a cited work is fixed as follows.  Frames of 800 samples (50 ms, the best
// window length of Sec. 4, Table 2) under the periodic Hann window, every 400 samples, frame t centred on sample
// 400 t, so that each sample lies in two frames whose weights add up to one.  The frame is laid out
// around time zero of a 2048-point transform.  Output bin k' reads the input spectrum, by linear
// interpolation between the two nearest bins, at the frequency that Eq. (1) maps onto k':
//     omega = omega' - 2 atan(a sin omega' / (1 + a cos omega')),  a = 1 - alpha, omega' = 2 pi k' / 2048.
// All 2048 samples of the inverse transform are added at the frame's position.  alpha = 1 returns the input.
//
// One wavefront per frame.  The 2048-point real transform is a 1024-point complex one of the even/odd
// packing, done by 64 lanes with 16 values each in LDS (wave-level fences only); the frame's samples go
// from HBM straight into the first butterflies' registers.  A wavefront works through a run of consecutive
// frames and overlap-adds them in a 2048-sample sliding window of its own in LDS (plain read-modify-write,
// no atomics); the 400 samples that leave the window after each frame are written out.  Only the ends of
// a run, where the frames of the neighbouring runs also land, go to HBM with float atomics; measured on
// the chip, sending every sample through HBM atomics more than doubled the kernel's time.
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
constexpr int kRun = 16;                           // consecutive frames overlap-added by one wavefront
constexpr int kFramesPerGroup = kRun * kWaves;
constexpr int kSlot = lds_padded_size(kN) + 2;     // a wavefront's transform buffer plus the slot of bin 1024
constexpr int kReach = kFft / 2;                   // a frame adds to [centre - kReach, centre + kReach)

// two consecutive output samples; only their 4-byte alignment is promised
struct __attribute__((aligned(4))) SamplePair { float x, y; };

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

// Write positions [p0, p0 + 2 count) of the wavefront's window to the output and clear them.  Positions in
// [excl_lo, excl_hi) receive nothing from other runs and are stored; the rest is added atomically.
// p0, excl_lo and excl_hi are even, so a pair never straddles a boundary.
__device__ inline void flush_window(float* acc, float* y, int len, int p0, int count, int excl_lo, int excl_hi, int lane) {
    for (int i = lane; i < count; i += 64) {
        const int p = p0 + 2 * i;
        float2* slot = reinterpret_cast<float2*>(acc + (p & (kFft - 1)));
        const float2 s = *slot;
        *slot = make_float2(0.f, 0.f);
        if (p >= excl_lo && p < excl_hi) {
            if (p >= 0 && p + 1 < len) {
                *reinterpret_cast<SamplePair*>(y + p) = SamplePair{s.x, s.y};
            } else {
                if ((unsigned)p < (unsigned)len) y[p] = s.x;
                if ((unsigned)(p + 1) < (unsigned)len) y[p + 1] = s.y;
            }
        } else {
            if ((unsigned)p < (unsigned)len) atomicAdd(&y[p], s.x);
            if ((unsigned)(p + 1) < (unsigned)len) atomicAdd(&y[p + 1], s.y);
        }
    }
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
    if (blockIdx.x * kFramesPerGroup >= n_frames) return;    // the whole group leaves together
    float2* buf = smem + wv * kSlot;
    float2* s_tab = smem + kWaves * kSlot;
    float* acc = reinterpret_cast<float*>(s_tab + kBins + 1) + wv * kFft;     // [waves][2048], 8-byte aligned
    for (int k = tid; k < kBins; k += kThreads) s_tab[k] = tab[(size_t)u * kBins + k];
    for (int k = lane; k < kFft / 2; k += 64) reinterpret_cast<float2*>(acc)[k] = make_float2(0.f, 0.f);

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
    // twiddles of this lane's butterflies and of its bin pairs are the same for every frame
    FftLaneTwiddles<kN, 64> lane_tw;
    lane_tw.load(tw, lane);
    float2 pair_tw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pair_tw[i] = tw[kN + lane + 64 * i];     // exp(-i pi k / N), k = lane + 64 i
    const float2 quarter_tw = make_float2(0.f, -1.f);                   // k = N/2
    __syncthreads();

    // this wavefront's run of frames, and the positions that only its frames reach
    const int t_first = blockIdx.x * kFramesPerGroup + wv * kRun;
    if (t_first >= n_frames) return;                     // no barriers below
    const int t_last = min(t_first + kRun, n_frames) - 1;
    const int excl_lo = t_first == 0 ? -(1 << 30) : t_first * kHop + (kReach - kHop);
    const int excl_hi = t_last == n_frames - 1 ? (1 << 30) : t_last * kHop - (kReach - kHop);

    const float* x = wave + start;
    float* y = out + start;
    // the lane's eight sample pairs of frame t (unweighted); a zero window weight marks inputs the lane does
    // not have, and unsigned compares fold the test for positions before the utterance in
    auto load_frame = [&](float2 (&xs)[8], int t) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int g = t * kHop + tau0[s];
            const bool used = wnd[s].x != 0.f || wnd[s].y != 0.f;
            xs[s] = make_float2(used && (unsigned)g < (unsigned)len ? x[g] : 0.f,
                                used && (unsigned)(g + 1) < (unsigned)len ? x[g + 1] : 0.f);
        }
    };
    float2 next_x[8];
    load_frame(next_x, t_first);
    for (int t = t_first; t <= t_last; ++t) {
        const int centre = t * kHop;
        lane_tw.keep_in_loop();
        float2 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = make_float2(0.f, 0.f);
#pragma unroll
        for (int s = 0; s < 8; ++s) v[s < 4 ? s : s + 8] = make_float2(next_x[s].x * wnd[s].x, next_x[s].y * wnd[s].y);
        if (t < t_last) load_frame(next_x, t + 1);       // arrives while this frame is transformed
        fft_passes_cached<kN, 64, false, FftSync::Wave>(v, buf, lane_tw, lane);
        fft_store_natural<kN, 64>(v, buf, lane);
        fft_sync<FftSync::Wave>();

        // Packed transform Z -> real spectrum X, in place: with A = Z[k], B = conj Z[N-k], E = (A + B)/2,
        // O = -(i/2)(A - B), w = exp(-i pi k / N):  X[k] = E + w O,  X[N-k] = conj(E - w O).
        // A lane owns the pair (k, N-k); k = 0 yields X[0] and X[N], the latter kept in the extra slot.
        auto unpack = [&](int k, float2 w) {
            const int kn = (kN - k) & (kN - 1);
            const float2 A = buf[lds_pad(k)], B = cconj(buf[lds_pad(kn)]);
            const float2 E = make_float2(0.5f * (A.x + B.x), 0.5f * (A.y + B.y));
            const float2 O = make_float2(0.5f * (A.y - B.y), -0.5f * (A.x - B.x));
            const float2 wO = cmul(w, O);
            buf[lds_pad(k)] = cadd(E, wO);
            buf[lds_pad(k ? kn : kN)] = cconj(csub(E, wO));
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) unpack(lane + 64 * i, pair_tw[i]);
        if (lane == 0) unpack(kN / 2, quarter_tw);
        fft_sync<FftSync::Wave>();

        // Warped spectrum Y (two interpolated bins per pair), packed for the inverse transform:
        // Ye = (Y[k] + conj Y[N-k])/2, Yo = conj(w) (Y[k] - conj Y[N-k])/2, Z'[k] = Ye + i Yo,
        // Z'[N-k] = conj(Ye) + i conj(Yo).  All reads of X finish before the buffer is overwritten.
        float2 zk[9], zn[9];
        auto pack = [&](int k, int slot, float2 w) {
            const float2 Yk = warped_bin(buf, s_tab, k), Yn = cconj(warped_bin(buf, s_tab, kN - k));
            const float2 Ye = make_float2(0.5f * (Yk.x + Yn.x), 0.5f * (Yk.y + Yn.y));
            const float2 dY = make_float2(0.5f * (Yk.x - Yn.x), 0.5f * (Yk.y - Yn.y));
            const float2 Yo = cmul_conj(dY, w);
            zk[slot] = make_float2(Ye.x - Yo.y, Ye.y + Yo.x);
            zn[slot] = make_float2(Ye.x + Yo.y, Yo.x - Ye.y);
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) pack(lane + 64 * i, i, pair_tw[i]);
        if (lane == 0) pack(kN / 2, 8, quarter_tw);
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
        fft_passes_cached<kN, 64, true, FftSync::Wave>(v, buf, lane_tw, lane);
        // v[i] is packed output m = fft_out_index(lane, i) times N: samples at offsets 2m, 2m + 1 (m < N/2)
        // or 2m - 2048, 2m - 2047 from the frame centre; position p lives at window slot p mod 2048, and the
        // centre is even, so a pair is one aligned float2 of the window
        const float scale = 1.0f / (float)kN;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = fft_out_index<kN, 64>(lane, i);
            float2* slot = reinterpret_cast<float2*>(acc + ((centre + 2 * m) & (kFft - 1)));
            float2 a = *slot;
            a.x += v[i].x * scale;
            a.y += v[i].y * scale;
            *slot = a;
        }
        fft_sync<FftSync::Wave>();
        // the next frame starts kHop later: the first kHop positions of the window are complete for this run
        flush_window(acc, y, len, centre - kReach, kHop / 2, excl_lo, excl_hi, lane);
        fft_sync<FftSync::Wave>();                       // also: the next frame reuses the transform buffer
    }
    flush_window(acc, y, len, t_last * kHop - kReach + kHop, (kFft - kHop) / 2, excl_lo, excl_hi, lane);
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
    const size_t lds = sizeof(float2) * (size_t)(kWaves * kSlot + kBins + 1) + sizeof(float) * kWaves * kFft;
    vtlp_resynth_kernel<<<dim3((unsigned)groups, (unsigned)n_utt), dim3(kThreads), lds, s>>>(
        d_offsets, wave, tab, twiddle, out);
    return hipGetLastError();
}

}  // namespace aug
