// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <utility>
#include <vector>

#include "aug.h"

namespace aug {

// A grow-only device buffer owned by the context.
struct DeviceBuffer {
    void* ptr = nullptr;
    size_t bytes = 0;
    hipError_t reserve(size_t need);
    void release();
    template <class T> T* as() const { return static_cast<T*>(ptr); }
};

// Host-side description of how the packed utterances are cut into work items;
// rebuilt only when the offsets of a call differ from the cached ones.
struct Packing {
    std::vector<int64_t> offsets;        // n_utt + 1
    std::vector<int64_t> frame_offsets;  // n_utt + 1 (empty if not a front-end call)
    int conv_block = 0;                  // output samples per convolution block the tables were built for
    int frames_per_group = 0;            // frames per front-end work group the tables were built for
    int64_t n_conv_blocks = 0;           // sum over utterances of ceil(len / conv_block)
    int64_t n_frame_groups = 0;
};

// Pinned host staging for the offset arrays: a call copies its arrays into the next slot and enqueues an
// asynchronous copy from there, so the caller's arrays are free when the call returns and nothing waits for
// the stream.  A slot is reused only after the copy that read it has completed (its event).
struct HostRing {
    static constexpr int kSlots = 4;
    int64_t* slot[kSlots] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t done[kSlots] = {nullptr, nullptr, nullptr, nullptr};
    size_t cap = 0;                      // int64 entries per slot
    int next = 0;
};

}  // namespace aug

struct aug_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string last_error;

    // device copies of the host offset arrays and the work-item tables derived from them
    aug::Packing packing;
    aug::DeviceBuffer d_offsets;         // int64 [n_utt+1]
    aug::DeviceBuffer d_frame_offsets;   // int64 [n_utt+1]
    aug::DeviceBuffer d_conv_items;      // int2 [n_conv_blocks]: (utterance, block)
    aug::DeviceBuffer d_frame_items;     // int2 [n_frame_groups]: (utterance, first frame)
    aug::DeviceBuffer d_conv_first;      // int [n_utt+1]: blocks of the utterances before u
    aug::DeviceBuffer d_frame_first;     // int [n_utt+1]: frame groups of the utterances before u
    aug::HostRing ring;
    unsigned char* scratch = nullptr;    // this device's copy of the library's static scratch array

    // image-method work list
    int n_cu = 0;                        // compute units of the device
    aug::DeviceBuffer rir_items;         // Item [n_rir * items_per_response]
    aug::DeviceBuffer rir_ctrl;          // int [rir_ctrl_ints()]: item count, next item, class counters
    aug::DeviceBuffer visits;            // one 64-bit counter (aug_rir_visited_images)
    aug::DeviceBuffer mic_rows;          // float [n_rir * n_mic][10]: one geometry row per microphone

    // intermediate results
    aug::DeviceBuffer rir;               // float [n_rir][rir_len]            (pipeline only)
    aug::DeviceBuffer rir_spec;          // float2 [n_rir][n_part][P+1]
    aug::DeviceBuffer reverb;            // float [1+n_noise][total rounded up to even]
    aug::DeviceBuffer energy;            // double [n_utt][1+n_noise]: energies of the reverberated signals
    aug::DeviceBuffer gains;             // float [n_utt][n_noise]
    aug::DeviceBuffer first_tap;         // int [n_utt][1+n_noise]
    aug::DeviceBuffer mel_tab;           // float2 [n_utt][nfft/2+1]: (channel, weight) per bin
    aug::DeviceBuffer twiddle[16];       // per log2(n): float2 [n + n/2 + 1] FFT twiddles
    aug::DeviceBuffer window;            // float [win]
    aug::DeviceBuffer dct;               // float [n_ceps][n_mel]
    int dct_ceps = 0, dct_mel = 0;       // shape the table was built for
    aug::DeviceBuffer vtlp_tab;          // float2 [n_utt][vtlp_table_entries()]: (source bin, weight) per output bin
    int window_n = 0;

    // stage timing: events recorded in stream order, each tagged with the stage it ends (-1 = a start mark)
    bool profiling = false;
    std::vector<std::pair<hipEvent_t, int>> marks;
};

namespace aug {

// ---- kernels' host launchers (each checks nothing; arguments are validated by the API layer) ----

// Image-method impulse responses.  launch_rir_plan cuts every response into items (tap ranges of
// about equal image count) ordered heaviest first and resets ctrl (item count,
// next item, class counters: rir_ctrl_ints() ints); `items` needs room for 2 n_rir rir_items_per_response items;
// launch_rir then runs n_groups persistent work groups over the items (restart: once more over the
// same plan), writing either
// rir_out float [n_rir][rir_len] or, if rir_out is null, tap counts cnt_out int32 [n_rir][rir_len].
// With `visits` (device, one 64-bit counter, zero on entry) the amplitude pass runs in a measuring
// instantiation that adds the number of images it walked.
int rir_items_per_response(int rir_len);
size_t rir_item_bytes();
int rir_ctrl_ints();
hipError_t launch_rir_plan(hipStream_t s, int n_groups, int n_rir, const float* geom, int rir_len, double fs_over_c,
                           void* items, int* ctrl);
hipError_t launch_rir(hipStream_t s, int n_groups, int n_rir, const float* geom, int rir_len, double fs_over_c,
                      const void* items, int* ctrl, float* rir_out, int32_t* cnt_out,
                      bool restart, unsigned long long* visits = nullptr);

// rows float [n_rir * n_mic][10]: geometry row r / n_mic with microphone mics[r] (float [n_rir][n_mic][3]).
hipError_t launch_rir_mic_rows(hipStream_t s, int n_rir, int n_mic, const float* geom, const float* mics, float* rows);

// Largest complex FFT size the convolution kernels are built for, and the size chosen for a response length.
int conv_fft_size(int rir_len);

// Spectra of the zero-padded partitions of each response: spec float2 [n_rir][n_part][P+1], P = fft_n;
// the index of every response's first non-zero tap is taken into first_tap[n_rir] (INT_MAX on entry).
hipError_t launch_rir_spectrum(hipStream_t s, int n_rir, const float* rir, int rir_len, int fft_n,
                               const float2* twiddle, float2* spec, int* first_tap, int n_cu);

// Overlap-save convolution of every (utterance, source) with its response; adds the block's energy
// to energy[u][j] (double, must be zero on entry).  src_base[j] points at source j's packed signal.
struct ConvArgs {
    const int64_t* offsets;      // device
    const int2* items;           // device (utterance, block)
    const int* first;            // device [n_utt+1]: blocks of the utterances before u
    int64_t n_items;             // blocks of one source, all utterances
    int n_src;
    const float* speech;
    const float* noise;          // [n_src-1][total]
    int64_t total;
    const float2* spec;          // [n_utt][n_src][n_part][P+1]
    int n_part;
    float* reverb;               // [n_src][reverb_stride]
    int64_t reverb_stride;
    double* energy;              // [n_utt][n_src] of the reverberated signals
    const int* first_tap;        // [n_utt][n_src] first non-zero tap of each response
};
// n_cu: compute units of the device (the kernel runs as persistent work groups)
hipError_t launch_convolve(hipStream_t s, int fft_n, const float2* twiddle, const ConvArgs& a, int n_cu);

// gains [n_utt][n_src - 1] from the energies and the target SNRs (also copied to gains_out when given)
// energy: [n_utt][n_src] energies of the reverberated signals
hipError_t launch_gains(hipStream_t s, int n_utt, int n_src, const double* energy, const float* snr_db, float* gains,
                        float* gains_out);
// mixed = reverb[0] + sum_j gains[j - 1] reverb[j]; source j of the reverberated signals starts at j * stride
hipError_t launch_mix(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t stride, int n_src,
                      const float* reverb, const float* gains, float* mixed_out, int64_t max_len);

// Per-utterance (band, weight) table of the warped mel bank followed by the lane partition of the
// bins: tab float2 [n_utt][mel_table_stride(nfft)].
int mel_table_stride(int nfft);
hipError_t launch_mel_table(hipStream_t s, int n_utt, const float* alpha, const aug_frontend_cfg& cfg,
                            float2* tab);

// Hamming window, float [win].
hipError_t launch_window(hipStream_t s, int win, float* w);

// tw[t] = exp(-2 pi i t / n), t < n, then tw[n + k] = exp(-i pi k / n), k <= n/2, then
// exp(-i pi 16 j / n), j < n/32; each computed in fp64 and rounded once.
int twiddle_entries(int n);
hipError_t launch_twiddle(hipStream_t s, int n, float2* tw);

// STFT power -> warped mel -> power law.
struct MelArgs {
    const int64_t* offsets;        // device
    const int64_t* frame_offsets;  // device
    const int2* items;             // device (utterance, first frame of the group)
    int64_t n_items;
    int frames_per_group;
    const float* wave;
    // Mixing on the fly: when n_extra > 0 the analysed signal is
    // wave[n] + sum_j gains[u][j] * extra[j * extra_stride + n], j < n_extra.
    const float* extra;
    int64_t extra_stride;
    const float* gains;            // [n_utt][n_extra]
    int n_extra;
    const float2* mel_tab;
    const float* dct;              // [n_ceps][n_mel] orthonormal DCT-II rows (AUG_FEAT_MFCC), else null
    const float* window;
    const float2* twiddle;         // table for the nfft/2-point complex transform
    aug_frontend_cfg cfg;
    float* feats;
};
int mel_frames_per_group();
// dct float [n_ceps][n_mel]: s_q cos(pi q (m + 1/2) / n_mel), computed in fp64
hipError_t launch_dct_table(hipStream_t s, int n_ceps, int n_mel, float* dct);
hipError_t launch_mel(hipStream_t s, const MelArgs& a);

// Waveform VTLP: per-utterance table of (lower source bin, interpolation weight) for every output bin,
// then analysis, warp and overlap-add, one wavefront per frame; `out` must be zero on entry.
int vtlp_table_entries();
int vtlp_fft_size();                 // length of the complex transform whose twiddle table the kernel needs
bool vtlp_supported(int win, int hop, int nfft);
hipError_t launch_vtlp_table(hipStream_t s, int n_utt, const float* alpha, float2* tab);
hipError_t launch_vtlp_resynth(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t max_len,
                               const float* wave, const float2* tab, const float2* twiddle, float* out);

// Exclusive prefix sums of the per-utterance item counts (blocks of conv_block samples; groups of
// frames_per_group output rows) and the item tables (utterance, block) / (utterance, first row), all from the
// device copies of the offsets.  A null `*_first` skips that table.  The item counts are the host's.
hipError_t launch_pack(hipStream_t s, int n_utt, const int64_t* d_offsets, const int64_t* d_frame_offsets,
                       int conv_block, int frames_per_group, int* conv_first, int2* conv_items, int64_t n_conv_items,
                       int* frame_first, int2* frame_items, int64_t n_frame_items);

// fill n 32-bit words with a value (used instead of memset so that calls stay graph-capturable)
hipError_t launch_fill_u32(hipStream_t s, void* p, uint32_t v, int64_t n);
// the same for two arrays in one launch
hipError_t launch_fill2_u32(hipStream_t s, void* p, uint32_t v, int64_t n, void* q, uint32_t w, int64_t m);

}  // namespace aug
