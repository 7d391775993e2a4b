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
// FFT in LDS (16 lanes per frame, two radix-16 passes).  The bins are cut into 16 contiguous ranges that
// end where the band changes, one per lane, so a lane owns every band sum it forms (no atomics); channel m
// is the rising side of band m plus the falling side of band m + 1.  Other epilogues of the same
// energies (log-mel, MFCC) and the on-the-fly mixture of reverberated sources are options of the kernel.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int kMelThreads = 256;
constexpr int kFramesPerGroup = 64;        // smallest target of output rows per work group (the host picks up to 8 times as many)

__global__ void window_kernel(int win, float* w) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= win) return;
    double s, c;
    sincospi(2.0 * (double)i / (double)(win - 1), &s, &c);
    w[i] = (float)(0.54 - 0.46 * c);
}

// (band, weight) of bin k for one utterance: where Eq. (1) puts the bin on the mel scale
__device__ inline float2 mel_bin_entry(const aug_frontend_cfg& cfg, float alpha_u, int k) {
    const double a = 1.0 - (double)alpha_u;
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
    return make_float2(ch, wgt);
}

// Cut the bins of one utterance into 16 contiguous lane ranges that end on changes of the band
// index c, so that every (c, utterance) sum is formed by one lane alone.  Range i ends at the band
// change nearest to (i + 1) bins / 16; the ends are non-decreasing because the targets are.
// One work group per utterance writes the utterance's table, then threads 0..14 each place one boundary.
// An entry is a chain of double-precision library calls: with few utterances a group has a thread per bin
// (K = 512) so that the chains run side by side, with many a single wavefront, which fills the chip anyway
// and measured twice as fast there.
constexpr int kMelTableThreads = 320;
__global__ __launch_bounds__(kMelTableThreads) void mel_table_kernel(int n_utt, const float* __restrict__ alpha, aug_frontend_cfg cfg,
                                                       int stride, float2* __restrict__ tab) {
    __shared__ float band[2050];
    const int bins = cfg.nfft / 2 + 1;
    const int u = blockIdx.x;
    float2* t = tab + (size_t)u * stride;
    int* kstart = reinterpret_cast<int*>(tab + (size_t)u * stride + bins);
    const float alpha_u = alpha[u];
    for (int k = threadIdx.x; k < bins; k += (int)blockDim.x) {
        const float2 e = mel_bin_entry(cfg, alpha_u, k);
        t[k] = e;
        band[k] = e.x;
    }
    __syncthreads();
    const int lane = threadIdx.x;
    if (lane == 0) { kstart[0] = 0; kstart[16] = bins; }
    if (lane < 15) {
        const int ideal = ((lane + 1) * bins + 8) / 16;
        int end = bins;                               // no change found: everything up to the end
        for (int d = 0; d < bins; ++d) {
            const int lo = ideal - d, hi = ideal + d;
            if (lo >= 1 && lo < bins && band[lo] != band[lo - 1]) { end = lo; break; }
            if (hi >= 1 && hi < bins && band[hi] != band[hi - 1]) { end = hi; break; }
        }
        kstart[lane + 1] = end;
    }
}

constexpr int kMelLanes = 16;                            // lanes per frame
constexpr int kProg = 32;                                // steps of a lane's band-sum list, at most
constexpr int kProgStride = kProg + 1;                   // lists start four banks apart
// A frame's transform buffer in LDS, in complex values: one more than the padded transform, so that the
// frames of a wavefront start two banks apart.
template <int NC> constexpr int mel_slot_stride() { return lds_padded_size(NC) + 1; }
constexpr int kMelSlots = kMelThreads / kMelLanes;       // frames in flight per work group

// K = 512: 256-point complex FFT per frame, 16 lanes per frame, 16 frames per pass of the group.
// WIN: the window length when it is known at compile time (the paper's front end uses 400), else 0.
// two consecutive samples; only their 4-byte alignment is promised (global loads of two dwords need no more)
struct __attribute__((aligned(4))) SamplePair { float x, y; };

// e^power for e > 0 as exp2(power log2 e) on the hardware's base-2 logarithm and exponential (about one
// unit in the last place each; the library's pow spends some 150 instructions on its last bit).  The
// logarithm instruction does not take denormal inputs, so tiny energies are scaled into range first.
__device__ inline float power_law(float e, float power) {
    const bool tiny = e < 0x1p-100f;
    const float l = __builtin_amdgcn_logf(tiny ? e * 0x1p+64f : e) - (tiny ? 64.f : 0.f);
    return __builtin_amdgcn_exp2f(power * l);
}

template <int NC, int WIN, bool MIX>
__global__ __launch_bounds__(kMelThreads, 3) void mel_kernel(MelArgs a, const float2* __restrict__ tw, int tab_stride) {
    static_assert(NC == 256 && NC / 16 == kMelLanes, "two radix-16 passes, sixteen lanes per frame");
    extern __shared__ __align__(16) unsigned char smem[];
    const int n_mel = a.cfg.n_mel;
    const int feature = a.cfg.feature;
    const int n_out = feature == AUG_FEAT_MFCC ? a.cfg.n_ceps : n_mel;     // values per output row
    const int n_seg = n_mel + 3;                         // band sums (A, B)[c + 1] for c = -1..n_mel (+1 pad)
    float2* fft_buf = reinterpret_cast<float2*>(smem);                       // [slots][mel_slot_stride]
    float4* s_prog = reinterpret_cast<float4*>(fft_buf + kMelSlots * mel_slot_stride<NC>());   // [16][kProgStride]
    float2* s_tab = reinterpret_cast<float2*>(s_prog + kMelLanes * kProgStride);   // [NC + 1]: (c, w) per bin
    float2* s_tw = s_tab + (NC + 1);                                         // [NC + 1]: exp(-i pi k / NC)
    float2* s_ab = s_tw + (NC + 1);                                          // [slots][n_seg]
    int* s_kstart = reinterpret_cast<int*>(s_ab + kMelSlots * n_seg);        // [17]

    const int tid = threadIdx.x;
    const int slot = tid / kMelLanes, sub = tid % kMelLanes;
    // Group ids are dealt round-robin to the eight XCDs.  XCD x takes the x-th contiguous eighth of the item
    // list, so that every XCD gets the same mix of full and nearly empty groups whatever the period of the
    // list (equal utterances of four groups each would otherwise leave two XCDs with the short groups only),
    // and groups that read neighbouring frames of an utterance share an L2.
    const unsigned int xcd = blockIdx.x % 8u, nth = blockIdx.x / 8u;
    const unsigned int item = xcd * (gridDim.x / 8u) + min(xcd, gridDim.x % 8u) + nth;
    const int u = a.items[item].x;
    const int64_t start = a.offsets[u];
    const float* x = a.wave + start;
    const int win = WIN ? WIN : a.cfg.win, hop = a.cfg.hop;
    // The utterance owns rows_u rows of the output; the first n_frames_u hold its frames and the rest,
    // if the caller reserved more (padded batches), are set to zero.
    const int64_t len = a.offsets[u + 1] - start;
    const int64_t rows_u = a.frame_offsets[u + 1] - a.frame_offsets[u];
    const int64_t n_frames_u = len >= win ? 1 + (len - win) / hop : 0;
    // The utterance's rows are shared evenly among its groups, ceil(rows / frames_per_group) of them (as the
    // item table counts them), in multiples of the frames a group has in flight: no group is left with a few rows.
    const int groups_u = (int)((rows_u + a.frames_per_group - 1) / a.frames_per_group);
    const int rows_per_group = (int)(((rows_u + groups_u - 1) / groups_u + kMelSlots - 1) / kMelSlots) * kMelSlots;
    const int first = (a.items[item].y / a.frames_per_group) * rows_per_group;
    const float power = a.cfg.power;
    float* feats = a.feats + (size_t)a.frame_offsets[u] * n_out;
    float2* buf = fft_buf + slot * mel_slot_stride<NC>();
    float* pw = reinterpret_cast<float*>(buf);           // the frame's bin powers P[0..NC], once they are formed
    float2* AB = s_ab + slot * n_seg;                    // (A, B)[c + 1]; entry 0 takes what belongs to no band

    const float2* g_tab = a.mel_tab + (size_t)u * tab_stride;
    for (int k = tid; k <= NC; k += kMelThreads) {
        s_tab[k] = g_tab[k];
        s_tw[k] = k <= NC / 2 ? tw[NC + k] : make_float2(-tw[NC + (NC - k)].x, tw[NC + (NC - k)].y);
    }
    if (tid < 17) s_kstart[tid] = reinterpret_cast<const int*>(g_tab + (NC + 1))[tid];

    // this lane's window samples never change: z[n] = w[2n] x[2n] + i w[2n+1] x[2n+1], n = sub + 16 m
    float2 wnd[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int i0 = 2 * (sub + kMelLanes * i);
        wnd[i] = make_float2(i0 < win ? a.window[i0] : 0.f, i0 + 1 < win ? a.window[i0 + 1] : 0.f);
    }
    // twiddles of the second pass, exp(-2 pi i sub m / NC), are the same for every frame of this lane
    float2 twp[16];
#pragma unroll
    for (int m = 1; m < 16; ++m) twp[m] = tw[(sub * m) & (NC - 1)];
    __syncthreads();
    const int k_lo = s_kstart[sub], k_hi = s_kstart[sub + 1];
    // Each lane sums the bins of its own bands by a fixed list of steps, one per bin, that is the same for
    // every frame of the utterance: (keep, w, 1 - w, where the running sums go).  keep is 0 where a new band
    // begins, else 1.  The running sums are stored after every bin, so a band's entry ends up holding its
    // whole sum without any test on the way.  Lists are padded to a common length (a multiple of four,
    // the same for all lanes) by steps that add nothing; with more than kProg bins in one lane's range
    // (very wide bands) the plain loop further down is used instead.
    int n_steps = 0;
#pragma unroll
    for (int l = 0; l < kMelLanes; ++l) n_steps = max(n_steps, s_kstart[l + 1] - s_kstart[l]);
    n_steps = (n_steps + 3) & ~3;
    const bool listed = n_steps <= kProg;
    if (listed) {
        for (int e = tid; e < kMelLanes * kProg; e += kMelThreads) {
            const int l = e / kProg, i = e - l * kProg;
            const int lo = s_kstart[l], k = lo + i;
            float4 step = make_float4(1.f, 0.f, 0.f, __int_as_float(0));      // adds nothing, stores to entry 0
            if (k < s_kstart[l + 1]) {
                const float2 cw = s_tab[k];
                const int c = (int)cw.x;
                const bool same = i > 0 && (int)s_tab[k - 1].x == c;
                if (c >= 0) step = make_float4(same ? 1.f : 0.f, cw.y, 1.f - cw.y, __int_as_float(8 * (c + 1)));
                else step.x = same ? 1.f : 0.f;
            }
            s_prog[l * kProgStride + i] = step;
        }
        __syncthreads();
    }
    // Band sums are stored, never added to: an entry that some bin's band owns is rewritten for every frame,
    // and the others (bands without a bin, the padding) keep the zero they get here.
    for (int m = sub; m < n_seg; m += kMelLanes) AB[m] = make_float2(0.f, 0.f);
    const bool even_win = (win & 1) == 0;
    const float* extra = MIX ? a.extra + start : nullptr;
    const float* gains = MIX ? a.gains + (size_t)u * a.n_extra : nullptr;

    for (int it = 0; it < rows_per_group / kMelSlots; ++it) {
        const int64_t t = (int64_t)first + it * kMelSlots + slot;
        if ((int64_t)first + it * kMelSlots >= n_frames_u) {      // only padding rows are left in this group
            if (t < rows_u)
                for (int m = sub; m < n_out; m += kMelLanes) feats[t * n_out + m] = 0.f;
            continue;
        }
        const bool live = t < n_frames_u;
        float2 v[16];
        // Loads are unconditional: a slot past the utterance's last frame recomputes that last frame (its
        // result is dropped) and inputs past the window are read from the frame's last samples and meet a
        // zero window weight.  With MIX the analysed signal is formed here, in source order:
        // x + sum_j gains[j] extra_j.
        const int x0 = (int)(live ? t : n_frames_u - 1) * hop;
        if (even_win) {                                   // one 8-byte load per complex input
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int i0 = min(2 * (sub + kMelLanes * i), win - 2);
                const SamplePair s2 = *reinterpret_cast<const SamplePair*>(x + (x0 + i0));
                v[i] = make_float2(s2.x, s2.y);
            }
            if (MIX) {
                for (int j = 0; j < a.n_extra; ++j) {
                    const float g = gains[j];
                    const float* xj = extra + (size_t)j * a.extra_stride;
                    // all sixteen loads of a source are issued before the first of them is used (the
                    // scheduler may otherwise pair every load with its wait to save registers)
                    SamplePair s2[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int i0 = min(2 * (sub + kMelLanes * i), win - 2);
                        s2[i] = *reinterpret_cast<const SamplePair*>(xj + (x0 + i0));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        v[i].x += g * s2[i].x;
                        v[i].y += g * s2[i].y;
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int i0 = 2 * (sub + kMelLanes * i);
                v[i] = make_float2(x[x0 + min(i0, win - 1)], x[x0 + min(i0 + 1, win - 1)]);
            }
            if (MIX) {
                for (int j = 0; j < a.n_extra; ++j) {
                    const float g = gains[j];
                    const float* xj = extra + (size_t)j * a.extra_stride;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int i0 = 2 * (sub + kMelLanes * i);
                        v[i].x += g * xj[x0 + min(i0, win - 1)];
                        v[i].y += g * xj[x0 + min(i0 + 1, win - 1)];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = make_float2(v[i].x * wnd[i].x, v[i].y * wnd[i].y);
        // 256 = 16 x 16: first pass without twiddles (inputs past the window are zero and fold away when
        // WIN is known), exchange through LDS, second pass with this lane's fixed twiddles
        SmallDft<16, false>::run(v);
        fft_store<NC, kMelLanes, 16, 1>(v, buf, sub);
        fft_sync<FftSync::Wave>();
        fft_load<NC, kMelLanes, 16>(v, buf, sub);
        fft_sync<FftSync::Wave>();
#pragma unroll
        for (int m = 1; m < 16; ++m) v[m] = cmul(v[m], twp[m]);
        SmallDft<16, false>::run(v);
        fft_store_natural<NC, kMelLanes>(v, buf, sub);
        fft_sync<FftSync::Wave>();                       // a frame's 16 lanes share a wavefront

        // Bin powers, two at a time: with E = (Z[k] + conj Z[N-k])/2, O = -(i/2)(Z[k] - conj Z[N-k]) and
        // w = exp(-i pi k / N):  X[k] = E + w O and conj(X[N-k]) = E - w O.
        // The powers go back into the frame's buffer as a plain array P[0..N] of floats, so every lane reads
        // all its bins before any lane writes.
        constexpr int kPairs = NC / 2 / kMelLanes + 1;    // the last one (bin N/2) only for lane 0
        float p_lo[kPairs], p_hi[kPairs];
#pragma unroll
        for (int i = 0; i < kPairs; ++i) {
            const int k = min(sub + kMelLanes * i, NC / 2);   // 0..N/2 (lanes past it repeat bin N/2, unused)
            const int kn = (NC - k) & (NC - 1);
            const float2 Zk = buf[lds_pad(k)];
            const float2 Zn = buf[lds_pad(kn)];
            const float2 w = s_tw[k];
            const float2 E = make_float2(0.5f * (Zk.x + Zn.x), 0.5f * (Zk.y - Zn.y));
            const float2 O = make_float2(0.5f * (Zk.y + Zn.y), -0.5f * (Zk.x - Zn.x));
            const float2 wO = cmul(w, O);
            // sums first, then squares: a weak bin next to a strong mirror bin keeps its relative accuracy
            const float2 Xk = cadd(E, wO), Xn = csub(E, wO);
            p_lo[i] = Xk.x * Xk.x + Xk.y * Xk.y;
            p_hi[i] = Xn.x * Xn.x + Xn.y * Xn.y;
        }
        fft_sync<FftSync::Wave>();
#pragma unroll
        for (int i = 0; i < kPairs; ++i) {
            if (i == kPairs - 1 && sub != 0) break;
            const int k = sub + kMelLanes * i;
            pw[k] = p_lo[i];
            pw[NC - k] = p_hi[i];                         // k = 0: P[N] (it comes from Z[0] too); k = N/2: itself
        }
        fft_sync<FftSync::Wave>();

        // bins [k_lo, k_hi) -> per-band sums; this lane owns every band it meets
        if (listed) {
            const float4* step = s_prog + sub * kProgStride;
            const float* p = pw + k_lo;
            char* dst = reinterpret_cast<char*>(AB);
            float run_a = 0.f, run_b = 0.f;
            for (int i = 0; i < n_steps; i += 4) {
                float4 s4[4];
                float pk[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {             // all reads of the four steps before their stores
                    s4[j] = step[i + j];
                    pk[j] = p[i + j];                     // (past k_hi: some finite value, times zero)
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    run_a = fmaf(s4[j].y, pk[j], run_a * s4[j].x);
                    run_b = fmaf(s4[j].z, pk[j], run_b * s4[j].x);
                    *reinterpret_cast<float2*>(dst + __float_as_int(s4[j].w)) = make_float2(run_a, run_b);
                }
            }
        } else {
            float run_a = 0.f, run_b = 0.f;
            int cur = -100;
            for (int k = k_lo; k < k_hi; ++k) {
                const float pk = pw[k];
                const float2 cw = s_tab[k];
                const int c = (int)cw.x;
                if (c != cur) {
                    if (cur >= 0) AB[cur + 1] = make_float2(run_a, run_b);
                    cur = c;
                    run_a = 0.f;
                    run_b = 0.f;
                }
                run_a += cw.y * pk;
                run_b += (1.f - cw.y) * pk;
            }
            if (cur >= 0) AB[cur + 1] = make_float2(run_a, run_b);
        }
        fft_sync<FftSync::Wave>();

        // channel m collects the rising side of band m and the falling side of band m + 1
        if (feature == AUG_FEAT_POWER_LAW) {
            if (live) {
                for (int m = sub; m < n_mel; m += kMelLanes) {
                    const float e = AB[m + 1].x + AB[m + 2].y;
                    feats[t * n_mel + m] = e > 0.f ? power_law(e, power) : 0.f;
                }
            }
        } else {
            // log-mel; for cepstra the log energies go to the front of the frame's buffer (the bin powers are
            // no longer needed), then every lane takes the dot products of its coefficients with the whole vector
            for (int m = sub; m < n_mel; m += kMelLanes) {
                const float le = logf(fmaxf(AB[m + 1].x + AB[m + 2].y, a.cfg.log_floor));
                if (feature == AUG_FEAT_LOG) {
                    if (live) feats[t * n_mel + m] = le;
                } else {
                    pw[m] = le;
                }
            }
            if (feature == AUG_FEAT_MFCC) {
                fft_sync<FftSync::Wave>();
                for (int q = sub; q < n_out; q += kMelLanes) {
                    const float* row = a.dct + q * n_mel;
                    float acc = 0.f;
                    for (int m = 0; m < n_mel; ++m) acc += row[m] * pw[m];
                    if (live) feats[t * n_out + q] = acc;
                }
            }
        }
        if (!live && t < rows_u)
            for (int m = sub; m < n_out; m += kMelLanes) feats[t * n_out + m] = 0.f;
        fft_sync<FftSync::Wave>();                       // sums are read before the next frame clears them
    }
}

__global__ void dct_table_kernel(int n_ceps, int n_mel, float* dct) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_ceps * n_mel) return;
    const int q = i / n_mel, m = i % n_mel;
    const double s = q == 0 ? sqrt(1.0 / (double)n_mel) : sqrt(2.0 / (double)n_mel);
    dct[i] = (float)(s * cos(M_PI * (double)q * ((double)m + 0.5) / (double)n_mel));
}

}  // namespace

hipError_t launch_dct_table(hipStream_t s, int n_ceps, int n_mel, float* dct) {
    const int n = n_ceps * n_mel;
    if (n <= 0) return hipSuccess;
    dct_table_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(n_ceps, n_mel, dct);
    return hipGetLastError();
}

int mel_frames_per_group() { return kFramesPerGroup; }

hipError_t launch_window(hipStream_t s, int win, float* w) {
    window_kernel<<<dim3((win + 255) / 256), dim3(256), 0, s>>>(win, w);
    return hipGetLastError();
}

int mel_table_stride(int nfft) { return nfft / 2 + 1 + 9; }   // (c, w) per bin, then 17 lane starts (+ pad)

hipError_t launch_mel_table(hipStream_t s, int n_utt, const float* alpha, const aug_frontend_cfg& cfg,
                            float2* tab) {
    if (n_utt <= 0) return hipSuccess;
    const int threads = n_utt >= 1024 ? 64 : kMelTableThreads;
    mel_table_kernel<<<dim3((unsigned)n_utt), dim3(threads), 0, s>>>(n_utt, alpha, cfg, mel_table_stride(cfg.nfft), tab);
    return hipGetLastError();
}

hipError_t launch_mel(hipStream_t s, const MelArgs& a) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.cfg.nfft != 512) return hipErrorInvalidValue;
    constexpr int NC = 256;
    const size_t lds = sizeof(float2) * (kMelSlots * mel_slot_stride<NC>() + 2 * (NC + 1)) +
                       sizeof(float4) * kMelLanes * kProgStride +
                       sizeof(float2) * kMelSlots * (a.cfg.n_mel + 3) + sizeof(int) * 20;
    const bool mix = a.n_extra > 0;
    auto k = a.cfg.win == 400 ? (mix ? &mel_kernel<NC, 400, true> : &mel_kernel<NC, 400, false>)
                              : (mix ? &mel_kernel<NC, 0, true> : &mel_kernel<NC, 0, false>);
    // (launched by address, not called through the pointer: see the convolution's launcher)
    MelArgs by_value = a;
    const float2* tw = a.twiddle;
    int tab_stride = mel_table_stride(a.cfg.nfft);
    void* args[] = {&by_value, &tw, &tab_stride};
    return hipLaunchKernel(reinterpret_cast<const void*>(k), dim3((unsigned)a.n_items), dim3(kMelThreads), args, lds, s);
}

}  // namespace aug
