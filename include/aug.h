/*
 * aug.h -- C ABI of the on-the-fly speech augmentation + power-mel front end
 * for AMD MI355X (gfx950).
 *
 * The library runs, on one GPU, the per-utterance work that the paper's
 * example servers do before features reach the trainer (Sec. 2.3, "Data
 * augmentation and feature extraction"): room impulse responses computed on
 * the fly by the image method, reverberation of the speech and of every noise
 * source with its own response, additive mixing at a drawn SNR, and
 * power-mel filterbank features with the vocal-tract-length-perturbation
 * warp of Eq. (1) and the (.)^(1/15) power law.
 *
 * Conventions (all entry points)
 *   - Pointers marked DEVICE are HBM addresses on the context's GPU, owned by
 *     the caller; the library reads inputs, writes outputs and never frees or
 *     keeps them.  Pointers marked HOST are ordinary host memory, read before
 *     the call returns.
 *   - Work is enqueued on the context's HIP stream and the call returns
 *     without waiting for it, also when the batch's offsets differ from the
 *     previous call's (they reach the device through pinned staging and
 *     asynchronous copies, and the work-item tables are rebuilt there by small
 *     kernels); the caller synchronises that stream before reading outputs.
 *     HOST arrays are free for reuse as soon as the call returns.  Calls on one
 *     context must not overlap in time from several host threads.
 *   - The context owns a private device workspace (impulse-response spectra,
 *     reverberated signals, energies, warp tables); it grows on demand and is
 *     released by aug_destroy.  Growing frees the old allocation, which waits
 *     for the work that uses it: only calls larger than any before them wait.
 *   - HIP graphs: a call whose sizes and offsets equal those of the previous
 *     call on the context consists of kernel launches only and may be captured
 *     from the context's stream into a graph.  Capture it only after one
 *     identical, uncaptured call.  The graph holds addresses of the workspace:
 *     destroy it before any call with larger sizes or other offsets (which may
 *     move or rewrite the workspace) and before aug_destroy.  A call that would
 *     have to allocate, copy offsets or rebuild tables while its stream is
 *     being captured returns AUG_ERR_UNSUPPORTED instead.
 *   - Every function returns AUG_OK (0) or a negative aug_status; nothing is
 *     thrown across the boundary.  aug_last_error gives the message of the
 *     last failure on that context.  Arguments are checked on the host, and the
 *     workspace is sized, before the first kernel of a call: a call that fails
 *     a check or runs out of memory has launched nothing.
 *   - A pointer to an array that has no elements in this call (a batch with no
 *     utterances or no samples, an output with no rows) may be NULL; any other
 *     NULL that the argument lists below do not allow is AUG_ERR_INVALID_ARG.
 *   - All random draws (rooms, positions, SNRs, warp factors) are inputs.
 */
#ifndef AUG_H_
#define AUG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum aug_status {
    AUG_OK = 0,
    AUG_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, offsets not ascending, ... */
    AUG_ERR_UNSUPPORTED = -2,   /* a size outside what the kernels are built for */
    AUG_ERR_NOMEM = -3,         /* workspace allocation failed */
    AUG_ERR_HIP = -4            /* a HIP runtime call failed */
} aug_status;

typedef struct aug_ctx aug_ctx;

/* Largest impulse response, in taps, that aug_rir_batch / aug_convolve_mix_batch accept. */
#define AUG_MAX_RIR_LEN 32768
/* Largest number of noise sources per utterance. */
#define AUG_MAX_NOISE 8
/* Largest number of mel channels. */
#define AUG_MAX_MEL 128
/* Largest number of microphones per room in aug_rir_mics_batch. */
#define AUG_MAX_MIC 16
#define AUG_MAX_UTT 65535        /* utterances per call */
#define AUG_MAX_UTT_SAMPLES ((1 << 30) - 1)   /* samples per utterance */

/*
 * Create a context bound to GPU `device_id` and to `hip_stream` (a hipStream_t
 * passed as void*; NULL = the device's default stream).  *out receives the
 * context.  The stream must outlive the context.
 */
int aug_create(aug_ctx** out, int device_id, void* hip_stream);

/* Wait for the context's stream, free the workspace and the context. NULL is accepted. */
int aug_destroy(aug_ctx* ctx);

/* Message of the last failed call on `ctx` ("" if none); valid until the next call on it. */
const char* aug_last_error(const aug_ctx* ctx);

/*
 * Number of analysis frames of an `n_samples` long signal: frames lie wholly
 * inside the signal (no padding), 1 + (n_samples - win) / hop, or 0 when
 * n_samples < win.  Host helper; returns -1 for win <= 0 or hop <= 0.
 */
int64_t aug_frame_count(int64_t n_samples, int win, int hop);

/*
 * Room impulse responses by the image method (the acoustic simulator of
 * Sec. 2.3 computes them on the fly for every example).
 *
 *   geom           DEVICE float [n_rir][10]: room Lx,Ly,Lz (m), source x,y,z,
 *                  microphone x,y,z, wall reflection coefficient beta.  The box
 *                  is [0,Lx]x[0,Ly]x[0,Lz]; source and microphone must lie
 *                  inside it and not coincide (not checked on the device).
 *                  beta must lie in [0, 1].  A room with a side under 0.1 m, a
 *                  beta outside [0, 1], or either not a number, yields an
 *                  all-zero response (and zero counts) instead of an unbounded
 *                  image lattice or an overflowing sum.
 *   rir_len        taps per response, 1..AUG_MAX_RIR_LEN.
 *   fs, c          sample rate (Hz) and speed of sound (m/s), both > 0.
 *   rir_out        DEVICE float [n_rir][rir_len], overwritten:
 *                  h[n] = sum over image sources with round(d fs / c) == n of
 *                  beta^(reflections) / (4 pi d), d = image-to-microphone
 *                  distance.  The tap index is evaluated in fp64 as
 *                  floor(sqrt((dx*dx + dy*dy) + dz*dz) * (fs / c) + 0.5).
 *   tap_count_out  DEVICE int32 [n_rir][rir_len] or NULL: number of images
 *                  that landed on each tap (exact, order independent).
 *
 * n_rir == 0 is a no-op.
 */
int aug_rir_batch(aug_ctx* ctx, int n_rir, const float* geom, int rir_len,
                  float fs, float c, float* rir_out, int32_t* tap_count_out);

/*
 * Responses from each source to several microphones in its room: the device
 * that records the far-field test sets of Sec. 4 carries two microphones
 * 6.8 cm apart, and simulating such a device needs one response per
 * microphone for the same room, source and walls.
 *
 *   n_mic          microphones per room, 1..AUG_MAX_MIC.
 *   geom           DEVICE float [n_rir][10] as for aug_rir_batch; its microphone
 *                  columns (6..8) are not read.
 *   mics           DEVICE float [n_rir][n_mic][3]: microphone x,y,z, inside the
 *                  room and away from the source like the single one.
 *   rir_out        DEVICE float [n_rir][n_mic][rir_len], overwritten: slice
 *                  [r][m] is what aug_rir_batch gives for row r with microphone
 *                  mics[r][m], bit for bit.
 *   tap_count_out  DEVICE int32 [n_rir][n_mic][rir_len] or NULL.
 *
 * The image sources of a room are the same for every microphone, but the
 * kernels visit them in shells of distance around the microphone, so each
 * microphone is summed as a response of its own: the cost is n_mic times that
 * of aug_rir_batch.  n_rir == 0 is a no-op.
 */
int aug_rir_mics_batch(aug_ctx* ctx, int n_rir, int n_mic, const float* geom, const float* mics,
                       int rir_len, float fs, float c, float* rir_out, int32_t* tap_count_out);

/*
 * Reverberation and additive noise (acoustic simulator, Sec. 2.3): every
 * source is convolved with its own impulse response, then each noise is scaled
 * to its SNR against the reverberated speech and added.
 *
 *   offsets     HOST int64 [n_utt+1], ascending, offsets[0] == 0: utterance u
 *               occupies samples offsets[u] .. offsets[u+1]-1 of every packed
 *               signal array.  Empty utterances are allowed; n_utt <=
 *               AUG_MAX_UTT and every utterance <= AUG_MAX_UTT_SAMPLES samples
 *               (AUG_ERR_UNSUPPORTED otherwise).
 *   speech      DEVICE float [total], total = offsets[n_utt].
 *   n_noise     0..AUG_MAX_NOISE noise sources per utterance.
 *   noise       DEVICE float [n_noise][total] (NULL iff n_noise == 0).
 *   rir         DEVICE float [n_utt][1+n_noise][rir_len]; source 0 is the speech.
 *   snr_db      DEVICE float [n_utt][n_noise] (NULL iff n_noise == 0).
 *   mixed_out   DEVICE float [total], overwritten:
 *               y_j[n] = sum_{k<=n, k<rir_len} h_j[k] x_j[n-k]  (causal, input
 *               length kept, the tail past the end is dropped),
 *               E_j = sum_n y_j[n]^2,  g_j = sqrt(E_0 / (E_j 10^(snr_j/10)))
 *               (0 if E_0 or E_j is 0),  mixed = y_0 + sum_j g_j y_j.
 *               Samples before the first non-zero tap of h_j are exact
 *               zeros (the transforms alone would leave rounding noise
 *               there), so a source whose direct path arrives after the
 *               utterance has ended has energy 0 and gain 0.
 *   gains_out   DEVICE float [n_utt][n_noise] or NULL: the g_j.
 */
int aug_convolve_mix_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets,
                           const float* speech, int n_noise, const float* noise,
                           const float* rir, int rir_len, const float* snr_db,
                           float* mixed_out, float* gains_out);

/* What is kept of the mel energies E[m] of a frame (Sec. 2.3 names all three). */
enum {
    AUG_FEAT_POWER_LAW = 0,   /* E^power: the paper's power-mel filterbank coefficients; 0 -> 0 */
    AUG_FEAT_LOG = 1,         /* ln max(E, log_floor): conventional log-mel */
    AUG_FEAT_MFCC = 2         /* first n_ceps coefficients of the orthonormal DCT-II of the log-mel vector:
                                 c[q] = s_q sum_m ln max(E[m], log_floor) cos(pi q (m + 1/2) / n_mel),
                                 s_0 = sqrt(1/n_mel), s_q = sqrt(2/n_mel) */
};

/* Front-end constants.  win <= nfft, nfft a power of two in 64..2048 (kernels
 * are built for 512), hop >= 1, 1 <= n_mel <= AUG_MAX_MEL, 0 <= f_lo < f_hi <= fs/2. */
typedef struct aug_frontend_cfg {
    float fs;       /* sample rate, Hz */
    int   win;      /* window length in samples (symmetric Hamming) */
    int   hop;      /* frame shift in samples */
    int   nfft;     /* DFT size K of Eq. (1) */
    int   n_mel;    /* mel channels */
    float f_lo;     /* lowest band edge, Hz */
    float f_hi;     /* highest band edge, Hz */
    float power;    /* power-law exponent, 1/15 in the paper (AUG_FEAT_POWER_LAW) */
    int   feature;  /* AUG_FEAT_* */
    int   n_ceps;   /* AUG_FEAT_MFCC: coefficients kept, 1..n_mel; ignored otherwise */
    float log_floor;/* AUG_FEAT_LOG / AUG_FEAT_MFCC: energies are raised to it before the logarithm, > 0 */
} aug_frontend_cfg;

/* Values per output row: n_ceps for AUG_FEAT_MFCC, else n_mel (host helper; 0 if cfg is NULL). */
int aug_feature_dim(const aug_frontend_cfg* cfg);

/*
 * Power-mel features with the VTLP warp (Sec. 2.3, Eq. (1)).
 *
 *   offsets        HOST int64 [n_utt+1] as above.
 *   wave           DEVICE float [total].
 *   alpha          DEVICE float [n_utt]: warp factor of each utterance
 *                  (1 = no warp; the paper's best range is [0.8, 1.2]).
 *   frame_offsets  HOST int64 [n_utt+1]: first output row of each utterance;
 *                  frame_offsets[0] = 0 and utterance u owns rows
 *                  frame_offsets[u] .. frame_offsets[u+1], at least
 *                  aug_frame_count(length_u, win, hop) of them (checked).  The
 *                  prefix sum of the frame counts gives the packed layout; rows
 *                  an utterance owns beyond its frames are set to zero, so
 *                  frame_offsets[u] = u * Tmax gives the padded batch
 *                  [n_utt][Tmax][n_mel] that the paper's padded_batch step
 *                  produces (Sec. 2.2).
 *   feats_out      DEVICE float [frame_offsets[n_utt]][aug_feature_dim(cfg)], row
 *                  major, overwritten.  With AUG_FEAT_POWER_LAW:
 *                  frame t of utterance u = (sum_k W[m][k] P_t[k])^power with
 *                  P_t[k] = |DFT_nfft(hamming * x[t hop .. t hop + win))[k]|^2,
 *                  k = 0..nfft/2, and W[m][k] the unit-peak triangular mel
 *                  filter m (mel = 2595 log10(1 + f/700), n_mel + 2 edges
 *                  equally spaced in mel on [f_lo, f_hi]) read at the warped
 *                  frequency of bin k,
 *                  w' = w + 2 atan((1-alpha) sin w / (1 - (1-alpha) cos w)),
 *                  w = 2 pi k / nfft.  Zero energy gives zero.
 */
int aug_vtlp_mel_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave,
                       const float* alpha, const aug_frontend_cfg* cfg,
                       const int64_t* frame_offsets, float* feats_out);

/*
 * aug_vtlp_mel_batch for callers that cannot allocate device memory: serving
 * loops, harnesses that forbid hipMalloc, code that must not trigger an
 * allocation at an awkward moment.  Arguments, output and errors are those of
 * aug_vtlp_mel_batch, and so are the kernels; what differs is where the
 * tables of the call live (device copies of the offsets, the frame-group
 * table, the per-utterance warped mel tables, twiddles, window, cosine
 * table): in a fixed array of AUG_STATIC_SCRATCH_BYTES that is part of the
 * library's device image, one copy per GPU, held from the moment the library
 * is loaded on that GPU until the process ends.  The call makes no hipMalloc,
 * hipFree or other allocating call (the pinned staging it copies the offsets
 * through is set up by aug_create).
 *
 * Limits: n_utt <= AUG_STATIC_MAX_UTT, and the output rows, counted in groups
 * of 64 per utterance (sum over u of ceil(rows_u / 64)), at most
 * AUG_STATIC_MAX_ROW_GROUPS; a larger batch is refused with
 * AUG_ERR_UNSUPPORTED and nothing is launched.
 *
 * Every call on a GPU, from any context, uses that GPU's one array and
 * rewrites all of it that it reads: nothing of an earlier call's contents is
 * relied on.  Calls that overlap in time on one GPU (two contexts on two
 * streams, two threads) race on the array; the caller must order them.
 */
#define AUG_STATIC_MAX_UTT 4096
#define AUG_STATIC_MAX_ROW_GROUPS 65536
#define AUG_STATIC_SCRATCH_BYTES (10u << 20)
int aug_vtlp_mel_batch_static(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave,
                              const float* alpha, const aug_frontend_cfg* cfg,
                              const int64_t* frame_offsets, float* feats_out);

/* Analysis constants of the waveform VTLP.  Kernels are built for 800 / 400 / 2048. */
typedef struct aug_vtlp_cfg {
    int win;        /* frame length in samples (periodic Hann), 50 ms in the paper's best setting */
    int hop;        /* frame shift, win / 2 */
    int nfft;       /* DFT size K of Eq. (1), a power of two >= 2 win */
} aug_vtlp_cfg;

/*
 * VTLP on the waveform by resynthesis, the step the paper places before the
 * acoustic simulator (Sec. 2.3, Eq. (1); window length from Sec. 4, Table 2).
 *
 *   offsets   HOST int64 [n_utt+1] as above.
 *   wave      DEVICE float [total].
 *   alpha     DEVICE float [n_utt]: warp factor of each utterance (1 returns
 *             the input; the paper's best range is [0.8, 1.2]).
 *   wave_out  DEVICE float [total], overwritten; must not overlap wave.
 *
 * Per utterance of N samples: frame t = 0 .. (N-1)/hop + 1 is centred on sample
 * t hop, covers win samples (zeros outside the utterance) under
 * w[i] = 0.5 - 0.5 cos(2 pi i / win), and is placed around time zero of an
 * nfft-point DFT X.  The warped spectrum is Y[k'] = (1-f) X[j] + f X[j+1] with
 * j + f = nfft/(2 pi) (w' - 2 atan(a sin w' / (1 + a cos w'))), w' = 2 pi k'/nfft,
 * a = 1 - alpha, k' = 0..nfft/2: the frequency that Eq. (1) maps onto w'.
 * All nfft samples of the inverse DFT of Y are added at the frame's position.
 * Sums of overlapping frames use floating-point atomics, so the last bits of
 * wave_out can differ between runs.
 * Errors: AUG_ERR_UNSUPPORTED for any cfg other than 800 / 400 / 2048.
 */
int aug_vtlp_resynth_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave,
                           const float* alpha, const aug_vtlp_cfg* cfg, float* wave_out);

/*
 * The whole path in one call: aug_rir_batch on geom, aug_convolve_mix_batch
 * with those responses, aug_vtlp_mel_batch on the mixture.  Arguments as in
 * the three calls above; geom is DEVICE float [n_utt][1+n_noise][10].
 * Responses and the mixture stay in the context's workspace unless asked for:
 *   rir_out    DEVICE float [n_utt][1+n_noise][rir_len] or NULL
 *   mixed_out  DEVICE float [total] or NULL
 *   gains_out  DEVICE float [n_utt][n_noise] or NULL
 */
int aug_pipeline_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* speech,
                       int n_noise, const float* noise, const float* geom, int rir_len,
                       float fs, float c, const float* snr_db, const float* alpha,
                       const aug_frontend_cfg* cfg, const int64_t* frame_offsets,
                       float* feats_out, float* rir_out, float* mixed_out, float* gains_out);

/*
 * Per-stage device timing, for measurement (the stages are those of Sec. 2.3's path).
 * While enabled, every call records HIP events on the context's stream around each
 * stage's kernels.  aug_profile_read waits for the stream, adds up the elapsed
 * milliseconds of every stage recorded since the last read into
 * ms_out[AUG_N_STAGES] (HOST float) and the number of times each stage ran into
 * launches_out[AUG_N_STAGES] (HOST int32, may be NULL), then forgets them.
 */
enum {
    AUG_STAGE_RIR = 0,        /* image-sum kernel */
    AUG_STAGE_RIR_SPECTRUM,   /* transforms of the response partitions */
    AUG_STAGE_CONVOLVE,       /* overlap-save reverberation + energies */
    AUG_STAGE_MIX,            /* SNR gains and mixture */
    AUG_STAGE_MEL,            /* STFT power, warped mel, power law */
    AUG_STAGE_OTHER,          /* clears and small tables */
    AUG_STAGE_VTLP,           /* waveform VTLP (aug_vtlp_resynth_batch) */
    AUG_N_STAGES
};
/*
 * Measurement helper for the image sum: runs aug_rir_batch's amplitude pass in an instrumented
 * instantiation, waits for it, and returns in *visited_out (HOST) how many image sources the kernel
 * actually walked.  That is fewer than the images the definition sums over (those are what
 * tap_count_out adds up to): images whose amplitude beta^k / (4 pi d) is too small to change the sum
 * are skipped.  rir_out (DEVICE float [n_rir][rir_len]) receives the responses as usual.
 */
int aug_rir_visited_images(aug_ctx* ctx, int n_rir, const float* geom, int rir_len, float fs, float c,
                           float* rir_out, uint64_t* visited_out);

int aug_profile_enable(aug_ctx* ctx, int on);
int aug_profile_read(aug_ctx* ctx, float* ms_out, int32_t* launches_out);

#ifdef __cplusplus
}
#endif
#endif /* AUG_H_ */
