// C ABI of the augmentation + feature library: argument checks, workspace and
// work-item tables, and the order in which the kernels of Sec. 2.3's path are enqueued
// (impulse responses -> their spectra -> overlap-save reverberation with energies ->
// SNR gains and mixture -> warped power-mel features).  No arithmetic of the method
// lives here.

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <new>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "aug_internal.h"

namespace aug {

hipError_t DeviceBuffer::reserve(size_t need) {
    if (need <= bytes) return hipSuccess;
    if (ptr) {
        hipError_t e = hipFree(ptr);      // waits for work that may still use it
        ptr = nullptr;
        bytes = 0;
        if (e != hipSuccess) return e;
    }
    const size_t want = need + need / 8;  // a little headroom so slowly growing batches do not thrash
    hipError_t e = hipMalloc(&ptr, want);
    if (e != hipSuccess) {
        ptr = nullptr;
        (void)hipGetLastError();
        e = hipMalloc(&ptr, need);
        if (e != hipSuccess) { ptr = nullptr; return e; }
        bytes = need;
        return hipSuccess;
    }
    bytes = want;
    return hipSuccess;
}

void DeviceBuffer::release() {
    if (ptr) (void)hipFree(ptr);
    ptr = nullptr;
    bytes = 0;
}

}  // namespace aug

namespace {

using aug::DeviceBuffer;

// ---- the static scratch array of aug_vtlp_mel_batch_static ----
// Device memory that is part of the library's code object: every GPU that loads the library holds its own
// copy at its own address.  In host code the array's name is only a handle for hipGetSymbolAddress, never a
// device address; g_scratch[device] is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[AUG_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
unsigned char* g_scratch[kMaxDevices] = {};      // per device, filled by aug_create with that device current
std::mutex g_scratch_mutex;

constexpr size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
// byte offsets of the tables inside the array
struct ScratchLayout {
    static constexpr size_t twiddle = 0;                                                        // float2 [393]
    static constexpr size_t window = twiddle + align256(sizeof(float2) * 512);                  // float [<= 2048]
    static constexpr size_t dct = window + align256(sizeof(float) * 2048);                      // float [128][128]
    static constexpr size_t offsets = dct + align256(sizeof(float) * AUG_MAX_MEL * AUG_MAX_MEL);
    static constexpr size_t frame_offsets = offsets + align256(sizeof(int64_t) * (AUG_STATIC_MAX_UTT + 1));
    static constexpr size_t frame_first = frame_offsets + align256(sizeof(int64_t) * (AUG_STATIC_MAX_UTT + 1));
    static constexpr size_t frame_items = frame_first + align256(sizeof(int) * (AUG_STATIC_MAX_UTT + 1));
    static constexpr size_t mel_tab = frame_items + align256(sizeof(int2) * AUG_STATIC_MAX_ROW_GROUPS);
    static constexpr size_t mel_tab_bytes = sizeof(float2) * (size_t)AUG_STATIC_MAX_UTT * (512 / 2 + 1 + 9);
    static constexpr size_t end = mel_tab + align256(mel_tab_bytes);
};
static_assert(ScratchLayout::end <= AUG_STATIC_SCRATCH_BYTES, "the tables fit the static array");

int fail(aug_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        char msg[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(msg, sizeof msg, fmt, ap);
        va_end(ap);
        ctx->last_error = msg;
    }
    return code;
}

int fail_hip(aug_ctx* ctx, hipError_t e, const char* what) {
    (void)hipGetLastError();
    if (e == hipErrorOutOfMemory) return fail(ctx, AUG_ERR_NOMEM, "%s: out of device memory", what);
    return fail(ctx, AUG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define AUG_HIP(expr, what)                                        \
    do {                                                           \
        hipError_t e__ = (expr);                                   \
        if (e__ != hipSuccess) return fail_hip(ctx, e__, what);    \
    } while (0)

#define AUG_TRY(expr)                                              \
    do {                                                           \
        int rc__ = (expr);                                         \
        if (rc__ != AUG_OK) return rc__;                           \
    } while (0)

int check_offsets(aug_ctx* ctx, int n_utt, const int64_t* offsets) {
    if (n_utt < 0) return fail(ctx, AUG_ERR_INVALID_ARG, "n_utt is negative");
    if (n_utt > AUG_MAX_UTT) return fail(ctx, AUG_ERR_UNSUPPORTED, "more than %d utterances in one call", AUG_MAX_UTT);
    if (!offsets) return fail(ctx, AUG_ERR_INVALID_ARG, "offsets is null");
    if (offsets[0] != 0) return fail(ctx, AUG_ERR_INVALID_ARG, "offsets[0] must be 0");
    for (int u = 0; u < n_utt; ++u) {
        if (offsets[u + 1] < offsets[u])
            return fail(ctx, AUG_ERR_INVALID_ARG, "offsets not ascending at utterance %d", u);
        if (offsets[u + 1] - offsets[u] >= ((int64_t)1 << 30))
            return fail(ctx, AUG_ERR_UNSUPPORTED, "utterance %d is 2^30 samples or longer", u);
    }
    if (offsets[n_utt] > ((int64_t)1 << 40)) return fail(ctx, AUG_ERR_UNSUPPORTED, "packed signal too long");
    return AUG_OK;
}

int check_frontend(aug_ctx* ctx, const aug_frontend_cfg* cfg) {
    if (!cfg) return fail(ctx, AUG_ERR_INVALID_ARG, "front-end config is null");
    if (!(cfg->fs > 0.f)) return fail(ctx, AUG_ERR_INVALID_ARG, "fs must be positive");
    if (cfg->win < 2 || cfg->hop < 1) return fail(ctx, AUG_ERR_INVALID_ARG, "win must be >= 2 and hop >= 1");
    if (cfg->nfft < cfg->win) return fail(ctx, AUG_ERR_INVALID_ARG, "nfft is smaller than win");
    if (cfg->n_mel < 1 || cfg->n_mel > AUG_MAX_MEL)
        return fail(ctx, AUG_ERR_INVALID_ARG, "n_mel must be in 1..%d", AUG_MAX_MEL);
    if (!(cfg->f_lo >= 0.f) || !(cfg->f_hi > cfg->f_lo) || !(cfg->f_hi <= 0.5f * cfg->fs))
        return fail(ctx, AUG_ERR_INVALID_ARG, "need 0 <= f_lo < f_hi <= fs/2");
    if (cfg->feature == AUG_FEAT_POWER_LAW) {
        if (!(cfg->power > 0.f)) return fail(ctx, AUG_ERR_INVALID_ARG, "power must be positive");
    } else if (cfg->feature == AUG_FEAT_LOG || cfg->feature == AUG_FEAT_MFCC) {
        if (!(cfg->log_floor > 0.f)) return fail(ctx, AUG_ERR_INVALID_ARG, "log_floor must be positive");
        if (cfg->feature == AUG_FEAT_MFCC && (cfg->n_ceps < 1 || cfg->n_ceps > cfg->n_mel))
            return fail(ctx, AUG_ERR_INVALID_ARG, "n_ceps must be in 1..n_mel");
    } else {
        return fail(ctx, AUG_ERR_INVALID_ARG, "unknown feature kind %d", cfg->feature);
    }
    if (cfg->nfft != 512) return fail(ctx, AUG_ERR_UNSUPPORTED, "kernels are built for nfft = 512");
    return AUG_OK;
}

int check_frame_offsets(aug_ctx* ctx, int n_utt, const int64_t* offsets, const int64_t* frame_offsets,
                        const aug_frontend_cfg* cfg) {
    if (!frame_offsets) return fail(ctx, AUG_ERR_INVALID_ARG, "frame_offsets is null");
    if (frame_offsets[0] != 0) return fail(ctx, AUG_ERR_INVALID_ARG, "frame_offsets[0] must be 0");
    for (int u = 0; u < n_utt; ++u) {
        const int64_t want = aug_frame_count(offsets[u + 1] - offsets[u], cfg->win, cfg->hop);
        if (frame_offsets[u + 1] - frame_offsets[u] < want)
            return fail(ctx, AUG_ERR_INVALID_ARG, "frame_offsets leaves utterance %d fewer rows than it has frames", u);
    }
    return AUG_OK;
}

// Grow one of the context's device buffers.  Growing frees the old allocation (which waits for the work
// that uses it) and allocates: neither may happen while the stream is being captured into a graph.
int grow(aug_ctx* ctx, DeviceBuffer& b, size_t bytes, const char* what) {
    if (bytes <= b.bytes) return AUG_OK;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->stream, &st) != hipSuccess) (void)hipGetLastError();
    if (st != hipStreamCaptureStatusNone)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "%s would have to grow while the stream is being captured: "
                    "run the same call once before capturing it", what);
    hipError_t e = b.reserve(bytes);
    if (e != hipSuccess) return fail_hip(ctx, e, what);
    return AUG_OK;
}

// Pinned staging slots of at least `entries` int64 each, with their events.
int ring_reserve(aug_ctx* ctx, size_t entries) {
    aug::HostRing& r = ctx->ring;
    if (entries <= r.cap) return AUG_OK;
    for (int i = 0; i < aug::HostRing::kSlots; ++i) {
        if (r.done[i]) AUG_HIP(hipEventSynchronize(r.done[i]), "staging event wait");
        if (r.slot[i]) {
            AUG_HIP(hipHostFree(r.slot[i]), "staging free");
            r.slot[i] = nullptr;
        }
    }
    r.cap = 0;
    const size_t want = entries + entries / 4 + 64;
    for (int i = 0; i < aug::HostRing::kSlots; ++i) {
        AUG_HIP(hipHostMalloc(reinterpret_cast<void**>(&r.slot[i]), want * sizeof(int64_t), hipHostMallocDefault),
                "pinned staging buffer");
        if (!r.done[i]) AUG_HIP(hipEventCreateWithFlags(&r.done[i], hipEventDisableTiming), "staging event");
    }
    r.cap = want;
    return AUG_OK;
}

// Copy up to two host arrays of n int64 each to the device through the next staging slot, without waiting
// for the stream: the slot is reused only after this copy has run (its event).  A null array is skipped.
int upload_offsets(aug_ctx* ctx, size_t n, const int64_t* a, int64_t* d_a, const int64_t* b, int64_t* d_b) {
    aug::HostRing& r = ctx->ring;
    const int i = r.next;
    AUG_HIP(hipEventSynchronize(r.done[i]), "staging event wait");     // an unrecorded event counts as complete
    if (a) {
        memcpy(r.slot[i], a, n * sizeof(int64_t));
        AUG_HIP(hipMemcpyAsync(d_a, r.slot[i], n * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream), "offsets copy");
    }
    if (b) {
        memcpy(r.slot[i] + n, b, n * sizeof(int64_t));
        AUG_HIP(hipMemcpyAsync(d_b, r.slot[i] + n, n * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream),
                "frame offsets copy");
    }
    AUG_HIP(hipEventRecord(r.done[i], ctx->stream), "staging event record");
    r.next = (i + 1) % aug::HostRing::kSlots;
    return AUG_OK;
}

// Device copies of the offsets and the (utterance, block) / (utterance, frame group) tables.  When the host
// arrays equal the previous call's nothing is done (a steady-state call is kernel launches only).  Otherwise
// the arrays go to the device through pinned staging with asynchronous copies and the tables are rebuilt
// there by two small kernels, all in stream order behind the earlier calls' kernels: the call does not
// wait for the stream.  The host only counts the items (one pass over the utterances) to size the grids.
int sync_packing(aug_ctx* ctx, int n_utt, const int64_t* offsets, const int64_t* frame_offsets,
                 int conv_block, int frames_per_group) {
    aug::Packing& pk = ctx->packing;
    const size_t n = (size_t)n_utt + 1;
    const bool same_off = pk.offsets.size() == n && !memcmp(pk.offsets.data(), offsets, n * sizeof(int64_t));
    const bool need_conv = conv_block > 0 && !(same_off && pk.conv_block == conv_block);
    const bool need_fr = frame_offsets && !(same_off && pk.frame_offsets.size() == n &&
                          !memcmp(pk.frame_offsets.data(), frame_offsets, n * sizeof(int64_t)) &&
                          pk.frames_per_group == frames_per_group);
    if (same_off && !need_conv && !need_fr) return AUG_OK;

    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->stream, &st) != hipSuccess) (void)hipGetLastError();
    if (st != hipStreamCaptureStatusNone)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "the offsets differ from the previous call's: the tables cannot be "
                    "rebuilt while the stream is being captured (run the same call once before capturing it)");

    int64_t n_conv = 0, n_groups = 0;
    if (need_conv)
        for (int u = 0; u < n_utt; ++u) n_conv += (offsets[u + 1] - offsets[u] + conv_block - 1) / conv_block;
    if (need_fr)
        for (int u = 0; u < n_utt; ++u)
            n_groups += (frame_offsets[u + 1] - frame_offsets[u] + frames_per_group - 1) / frames_per_group;
    if (n_conv > 0x7fffffffLL || n_groups > 0x7fffffffLL)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "too many blocks or frame groups in one call");

    AUG_TRY(grow(ctx, ctx->d_offsets, n * sizeof(int64_t), "offsets buffer"));
    if (need_conv) {
        AUG_TRY(grow(ctx, ctx->d_conv_first, n * sizeof(int), "block prefix table"));
        AUG_TRY(grow(ctx, ctx->d_conv_items, (size_t)std::max<int64_t>(n_conv, 1) * sizeof(int2), "block table"));
    }
    if (need_fr) {
        AUG_TRY(grow(ctx, ctx->d_frame_offsets, n * sizeof(int64_t), "frame offsets buffer"));
        AUG_TRY(grow(ctx, ctx->d_frame_first, n * sizeof(int), "frame group prefix table"));
        AUG_TRY(grow(ctx, ctx->d_frame_items, (size_t)std::max<int64_t>(n_groups, 1) * sizeof(int2), "frame group table"));
    }
    AUG_TRY(ring_reserve(ctx, 2 * n));
    if (!same_off || need_fr)
        AUG_TRY(upload_offsets(ctx, n, same_off ? nullptr : offsets, ctx->d_offsets.as<int64_t>(),
                               need_fr ? frame_offsets : nullptr, ctx->d_frame_offsets.as<int64_t>()));
    AUG_HIP(aug::launch_pack(ctx->stream, n_utt, ctx->d_offsets.as<int64_t>(), ctx->d_frame_offsets.as<int64_t>(),
                             conv_block, frames_per_group,
                             need_conv ? ctx->d_conv_first.as<int>() : nullptr, ctx->d_conv_items.as<int2>(), n_conv,
                             need_fr ? ctx->d_frame_first.as<int>() : nullptr, ctx->d_frame_items.as<int2>(), n_groups),
            "packing kernels");

    if (!same_off) {
        pk.offsets.assign(offsets, offsets + n);
        if (!need_conv) pk.conv_block = 0;
        if (!need_fr) pk.frame_offsets.clear();
    }
    if (need_conv) {
        pk.conv_block = conv_block;
        pk.n_conv_blocks = n_conv;
    }
    if (need_fr) {
        pk.frame_offsets.assign(frame_offsets, frame_offsets + n);
        pk.frames_per_group = frames_per_group;
        pk.n_frame_groups = n_groups;
    }
    return AUG_OK;
}

// Output rows per work group of the front end (an upper bound: the kernel shares an utterance's rows evenly
// among its groups).  A group sets up its utterance's tables once, so larger groups are cheaper per frame
// as long as the launch still has several times more groups than the chip runs at once (three per compute
// unit); measured on 4096 utterances of 798 frames: 1.70 ms with 64 rows, 1.55 with 160, 1.51 with 400.
int frontend_rows_per_group(const aug_ctx* ctx, int n_utt, const int64_t* frame_offsets) {
    const int base = aug::mel_frames_per_group();
    const int64_t rows = n_utt > 0 ? frame_offsets[n_utt] : 0;
    const int64_t wanted = 8LL * 3 * ctx->n_cu;
    const int64_t fit = rows / wanted / 16 * 16;
    return (int)std::min<int64_t>(std::max<int64_t>(fit, base), 8 * base);
}

int ensure_twiddle(aug_ctx* ctx, int n, const float2** out) {
    int lg = 0;
    while ((1 << lg) < n) ++lg;
    DeviceBuffer& b = ctx->twiddle[lg];
    if (!b.ptr) {
        AUG_TRY(grow(ctx, b, sizeof(float2) * (size_t)aug::twiddle_entries(n), "twiddle table"));
        AUG_HIP(aug::launch_twiddle(ctx->stream, n, b.as<float2>()), "twiddle kernel");
    }
    *out = b.as<float2>();
    return AUG_OK;
}

// Record an event that closes stage `stage` (or opens a timed span when stage < 0).
int mark(aug_ctx* ctx, int stage) {
    if (!ctx->profiling) return AUG_OK;
    hipEvent_t ev;
    AUG_HIP(hipEventCreate(&ev), "event create");
    hipError_t e = hipEventRecord(ev, ctx->stream);
    if (e != hipSuccess) {
        (void)hipEventDestroy(ev);
        return fail_hip(ctx, e, "event record");
    }
    ctx->marks.emplace_back(ev, stage);
    return AUG_OK;
}

// Source j of the reverberated signals starts at j * reverb_stride(total): an even stride keeps the
// 8-byte loads of the front end aligned for every source.
int64_t reverb_stride(int64_t total) { return (total + 1) & ~(int64_t)1; }

// ---- workspace of each stage: sized before the first kernel of a call, so that a call that runs out of
// ---- memory has launched nothing ----

int prepare_rir(aug_ctx* ctx, int n_rir, int rir_len) {
    AUG_TRY(grow(ctx, ctx->rir_items, 2 * aug::rir_item_bytes() * (size_t)n_rir * aug::rir_items_per_response(rir_len),
                 "response item table"));
    AUG_TRY(grow(ctx, ctx->rir_ctrl, aug::rir_ctrl_ints() * sizeof(int), "response item counter"));
    return AUG_OK;
}

int prepare_convolve_mix(aug_ctx* ctx, int n_utt, int n_noise, int rir_len) {
    const int64_t total = ctx->packing.offsets[n_utt];
    if (n_utt == 0 || total == 0) return AUG_OK;
    const int n_src = 1 + n_noise;
    const int fft_n = aug::conv_fft_size(rir_len);
    const int n_part = (rir_len + fft_n - 1) / fft_n;
    AUG_TRY(grow(ctx, ctx->rir_spec, sizeof(float2) * (size_t)n_utt * n_src * n_part * (fft_n + 1), "spectrum workspace"));
    AUG_TRY(grow(ctx, ctx->reverb, sizeof(float) * (size_t)n_src * reverb_stride(total), "reverberation workspace"));
    AUG_TRY(grow(ctx, ctx->gains, sizeof(float) * (size_t)std::max(1, n_utt * n_noise), "gain workspace"));
    AUG_TRY(grow(ctx, ctx->energy, sizeof(double) * (size_t)n_utt * n_src, "energy workspace"));
    AUG_TRY(grow(ctx, ctx->first_tap, sizeof(int) * (size_t)n_utt * n_src, "first-tap workspace"));
    return AUG_OK;
}

int prepare_mel(aug_ctx* ctx, int n_utt, const aug_frontend_cfg* cfg) {
    if (n_utt == 0 || ctx->packing.n_frame_groups == 0) return AUG_OK;
    AUG_TRY(grow(ctx, ctx->window, sizeof(float) * (size_t)cfg->win, "window table"));
    if (cfg->feature == AUG_FEAT_MFCC)
        AUG_TRY(grow(ctx, ctx->dct, sizeof(float) * (size_t)cfg->n_ceps * cfg->n_mel, "cosine table"));
    AUG_TRY(grow(ctx, ctx->mel_tab, sizeof(float2) * (size_t)n_utt * aug::mel_table_stride(cfg->nfft), "mel table"));
    return AUG_OK;
}

// ---- stage drivers: arguments already validated, packing already synchronised ----

int run_rir(aug_ctx* ctx, int n_rir, const float* geom, int rir_len, float fs, float c, float* rir_out,
            int32_t* tap_count_out) {
    const double k = (double)fs / (double)c;
    AUG_TRY(prepare_rir(ctx, n_rir, rir_len));
    const int n_groups = 2 * ctx->n_cu;
    AUG_TRY(mark(ctx, -1));
    AUG_HIP(aug::launch_rir_plan(ctx->stream, n_groups, n_rir, geom, rir_len, k, ctx->rir_items.ptr,
                                 ctx->rir_ctrl.as<int>()), "rir plan kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_OTHER));
    AUG_HIP(aug::launch_rir(ctx->stream, n_groups, n_rir, geom, rir_len, k, ctx->rir_items.ptr,
                            ctx->rir_ctrl.as<int>(), rir_out, nullptr, false), "rir kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_RIR));
    if (tap_count_out) {
        AUG_HIP(aug::launch_rir(ctx->stream, n_groups, n_rir, geom, rir_len, k, ctx->rir_items.ptr,
                                ctx->rir_ctrl.as<int>(), nullptr, tap_count_out, true),
                "rir count kernel");
        AUG_TRY(mark(ctx, AUG_STAGE_OTHER));
    }
    return AUG_OK;
}

// Reverberates every source, measures the energies and derives the gains.  With mixed_out the mixture
// is written there; without it the caller mixes on the fly from the context's reverberated signals.
int run_convolve_mix(aug_ctx* ctx, int n_utt, int n_noise, const float* speech, const float* noise,
                     const float* rir, int rir_len, const float* snr_db, float* mixed_out, float* gains_out) {
    const aug::Packing& pk = ctx->packing;
    const int64_t total = pk.offsets[n_utt];
    const int n_src = 1 + n_noise;
    const int fft_n = aug::conv_fft_size(rir_len);
    const int n_part = (rir_len + fft_n - 1) / fft_n;
    const float2* tw = nullptr;
    AUG_TRY(ensure_twiddle(ctx, fft_n, &tw));
    if (n_utt == 0) return AUG_OK;
    if (total == 0) {       // no signal anywhere: every energy is zero, so every gain is
        if (gains_out && n_noise > 0)
            AUG_HIP(aug::launch_fill_u32(ctx->stream, gains_out, 0u, (int64_t)n_utt * n_noise), "gain clear");
        return AUG_OK;
    }
    int64_t max_len = 0;
    for (int u = 0; u < n_utt; ++u) max_len = std::max(max_len, pk.offsets[u + 1] - pk.offsets[u]);

    AUG_TRY(prepare_convolve_mix(ctx, n_utt, n_noise, rir_len));
    const int64_t stride = reverb_stride(total);
    double* const energy = ctx->energy.as<double>();

    AUG_TRY(mark(ctx, -1));
    AUG_HIP(aug::launch_fill2_u32(ctx->stream, energy, 0u, (int64_t)n_utt * n_src * 2, ctx->first_tap.ptr, 0x7fffffffu,
                                  (int64_t)n_utt * n_src), "energy and first-tap reset");
    AUG_TRY(mark(ctx, AUG_STAGE_OTHER));
    AUG_HIP(aug::launch_rir_spectrum(ctx->stream, n_utt * n_src, rir, rir_len, fft_n, tw, ctx->rir_spec.as<float2>(),
                                     ctx->first_tap.as<int>(), ctx->n_cu),
            "spectrum kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_RIR_SPECTRUM));
    aug::ConvArgs ca;
    ca.offsets = ctx->d_offsets.as<int64_t>();
    ca.items = ctx->d_conv_items.as<int2>();
    ca.first = ctx->d_conv_first.as<int>();
    ca.n_items = pk.n_conv_blocks;
    ca.n_src = n_src;
    ca.speech = speech;
    ca.noise = noise;
    ca.total = total;
    ca.spec = ctx->rir_spec.as<float2>();
    ca.n_part = n_part;
    ca.reverb = ctx->reverb.as<float>();
    ca.reverb_stride = stride;
    ca.energy = energy;
    ca.first_tap = ctx->first_tap.as<int>();
    AUG_HIP(aug::launch_convolve(ctx->stream, fft_n, tw, ca, ctx->n_cu), "convolution kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_CONVOLVE));
    AUG_HIP(aug::launch_gains(ctx->stream, n_utt, n_src, energy, snr_db, ctx->gains.as<float>(), gains_out), "gain kernel");
    if (mixed_out)
        AUG_HIP(aug::launch_mix(ctx->stream, n_utt, ctx->d_offsets.as<int64_t>(), stride, n_src, ctx->reverb.as<float>(),
                                ctx->gains.as<float>(), mixed_out, max_len), "mix kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_MIX));
    return AUG_OK;
}

// n_extra > 0: the analysed signal is wave + sum_j gains[u][j] extra[j * extra_stride + .] (mixed on the fly)
int run_mel(aug_ctx* ctx, int n_utt, const float* wave, const float* alpha, const aug_frontend_cfg* cfg,
            float* feats_out, int n_extra = 0, const float* extra = nullptr, int64_t extra_stride = 0,
            const float* gains = nullptr) {
    const aug::Packing& pk = ctx->packing;
    if (n_utt == 0 || pk.n_frame_groups == 0) return AUG_OK;
    const float2* tw = nullptr;
    AUG_TRY(prepare_mel(ctx, n_utt, cfg));
    AUG_TRY(ensure_twiddle(ctx, cfg->nfft / 2, &tw));
    if (ctx->window_n != cfg->win) {
        AUG_HIP(aug::launch_window(ctx->stream, cfg->win, ctx->window.as<float>()), "window kernel");
        ctx->window_n = cfg->win;
    }
    const float* dct = nullptr;
    if (cfg->feature == AUG_FEAT_MFCC) {
        if (ctx->dct_ceps != cfg->n_ceps || ctx->dct_mel != cfg->n_mel) {
            AUG_HIP(aug::launch_dct_table(ctx->stream, cfg->n_ceps, cfg->n_mel, ctx->dct.as<float>()), "cosine table kernel");
            ctx->dct_ceps = cfg->n_ceps;
            ctx->dct_mel = cfg->n_mel;
        }
        dct = ctx->dct.as<float>();
    }
    AUG_TRY(mark(ctx, -1));
    AUG_HIP(aug::launch_mel_table(ctx->stream, n_utt, alpha, *cfg, ctx->mel_tab.as<float2>()), "mel table kernel");
    aug::MelArgs ma;
    ma.offsets = ctx->d_offsets.as<int64_t>();
    ma.frame_offsets = ctx->d_frame_offsets.as<int64_t>();
    ma.items = ctx->d_frame_items.as<int2>();
    ma.n_items = pk.n_frame_groups;
    ma.frames_per_group = pk.frames_per_group;
    ma.wave = wave;
    ma.extra = extra;
    ma.extra_stride = extra_stride;
    ma.gains = gains;
    ma.n_extra = n_extra;
    ma.mel_tab = ctx->mel_tab.as<float2>();
    ma.dct = dct;
    ma.window = ctx->window.as<float>();
    ma.twiddle = tw;
    ma.cfg = *cfg;
    ma.feats = feats_out;
    AUG_HIP(aug::launch_mel(ctx->stream, ma), "mel kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_MEL));
    return AUG_OK;
}

int check_rir_args(aug_ctx* ctx, int rir_len, float fs, float c) {
    if (rir_len < 1 || rir_len > AUG_MAX_RIR_LEN)
        return fail(ctx, rir_len < 1 ? AUG_ERR_INVALID_ARG : AUG_ERR_UNSUPPORTED,
                    "rir_len must be in 1..%d", AUG_MAX_RIR_LEN);
    if (!(fs > 0.f) || !(c > 0.f)) return fail(ctx, AUG_ERR_INVALID_ARG, "fs and c must be positive");
    return AUG_OK;
}

// A pointer may be null only where the array it stands for has no elements.
int check_mix_args(aug_ctx* ctx, int n_utt, int64_t total, int n_noise, const void* speech, const void* noise,
                   const void* snr_db) {
    if (n_noise < 0 || n_noise > AUG_MAX_NOISE)
        return fail(ctx, AUG_ERR_INVALID_ARG, "n_noise must be in 0..%d", AUG_MAX_NOISE);
    if (!speech && total > 0) return fail(ctx, AUG_ERR_INVALID_ARG, "speech is null");
    if (n_noise > 0 && ((!noise && total > 0) || (!snr_db && n_utt > 0)))
        return fail(ctx, AUG_ERR_INVALID_ARG, "noise or snr_db is null");
    return AUG_OK;
}

int enter(aug_ctx* ctx) {
    if (!ctx) return AUG_ERR_INVALID_ARG;
    ctx->last_error.clear();
    AUG_HIP(hipSetDevice(ctx->device), "set device");
    return AUG_OK;
}

}  // namespace

extern "C" {

int aug_create(aug_ctx** out, int device_id, void* hip_stream) {
    if (!out) return AUG_ERR_INVALID_ARG;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device_id < 0 || device_id >= n_dev) {
        (void)hipGetLastError();
        return AUG_ERR_INVALID_ARG;
    }
    if (hipSetDevice(device_id) != hipSuccess) {
        (void)hipGetLastError();
        return AUG_ERR_HIP;
    }
    aug_ctx* ctx = new (std::nothrow) aug_ctx();
    if (!ctx) return AUG_ERR_NOMEM;
    ctx->device = device_id;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    if (hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, device_id) != hipSuccess ||
        ctx->n_cu < 1) {
        (void)hipGetLastError();
        delete ctx;
        return AUG_ERR_HIP;
    }
    // This device's copy of the static scratch array (once per device, with the device current), and pinned
    // staging large enough for the entry point that uses it, so that that entry point never allocates.
    if (device_id < kMaxDevices) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch[device_id]) {
            unsigned char* p = nullptr;
            if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                delete ctx;
                return AUG_ERR_HIP;
            }
            g_scratch[device_id] = p;
        }
        ctx->scratch = g_scratch[device_id];
    }
    if (ring_reserve(ctx, 2 * ((size_t)AUG_STATIC_MAX_UTT + 1)) != AUG_OK) {
        aug_destroy(ctx);
        return AUG_ERR_NOMEM;
    }
    *out = ctx;
    return AUG_OK;
}

int aug_destroy(aug_ctx* ctx) {
    if (!ctx) return AUG_OK;
    int rc = AUG_OK;
    if (hipSetDevice(ctx->device) != hipSuccess || hipStreamSynchronize(ctx->stream) != hipSuccess) {
        (void)hipGetLastError();
        rc = AUG_ERR_HIP;
    }
    DeviceBuffer* bufs[] = {&ctx->d_offsets, &ctx->d_frame_offsets, &ctx->d_conv_items, &ctx->d_frame_items,
                            &ctx->d_conv_first, &ctx->d_frame_first,
                            &ctx->rir_items, &ctx->rir_ctrl, &ctx->mic_rows, &ctx->visits, &ctx->rir, &ctx->rir_spec, &ctx->reverb, &ctx->energy, &ctx->gains, &ctx->first_tap, &ctx->vtlp_tab, &ctx->dct, &ctx->mel_tab,
                            &ctx->window};
    for (DeviceBuffer* b : bufs) b->release();
    for (DeviceBuffer& b : ctx->twiddle) b.release();
    for (auto& m : ctx->marks) (void)hipEventDestroy(m.first);
    for (int i = 0; i < aug::HostRing::kSlots; ++i) {
        if (ctx->ring.done[i]) (void)hipEventDestroy(ctx->ring.done[i]);
        if (ctx->ring.slot[i]) (void)hipHostFree(ctx->ring.slot[i]);
    }
    delete ctx;
    return rc;
}

const char* aug_last_error(const aug_ctx* ctx) { return ctx ? ctx->last_error.c_str() : "context is null"; }

int64_t aug_frame_count(int64_t n_samples, int win, int hop) {
    if (win <= 0 || hop <= 0) return -1;
    return n_samples < win ? 0 : 1 + (n_samples - win) / hop;
}

int aug_profile_enable(aug_ctx* ctx, int on) {
    AUG_TRY(enter(ctx));
    ctx->profiling = on != 0;
    return AUG_OK;
}

int aug_profile_read(aug_ctx* ctx, float* ms_out, int32_t* launches_out) {
    AUG_TRY(enter(ctx));
    if (!ms_out) return fail(ctx, AUG_ERR_INVALID_ARG, "ms_out is null");
    for (int i = 0; i < AUG_N_STAGES; ++i) {
        ms_out[i] = 0.f;
        if (launches_out) launches_out[i] = 0;
    }
    AUG_HIP(hipStreamSynchronize(ctx->stream), "stream synchronize");
    int rc = AUG_OK;
    for (size_t i = 1; i < ctx->marks.size(); ++i) {
        const int stage = ctx->marks[i].second;
        if (stage < 0 || stage >= AUG_N_STAGES) continue;
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, ctx->marks[i - 1].first, ctx->marks[i].first);
        if (e != hipSuccess) { rc = fail_hip(ctx, e, "event elapsed time"); break; }
        ms_out[stage] += ms;
        if (launches_out) launches_out[stage] += 1;
    }
    for (auto& m : ctx->marks) (void)hipEventDestroy(m.first);
    ctx->marks.clear();
    return rc;
}

int aug_rir_batch(aug_ctx* ctx, int n_rir, const float* geom, int rir_len, float fs, float c,
                  float* rir_out, int32_t* tap_count_out) {
    AUG_TRY(enter(ctx));
    if (n_rir < 0) return fail(ctx, AUG_ERR_INVALID_ARG, "n_rir is negative");
    AUG_TRY(check_rir_args(ctx, rir_len, fs, c));
    if (n_rir == 0) return AUG_OK;
    if (!geom || !rir_out) return fail(ctx, AUG_ERR_INVALID_ARG, "geom or rir_out is null");
    if ((int64_t)n_rir * aug::rir_items_per_response(rir_len) > 0x7fffffffLL)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "too many responses in one call");
    return run_rir(ctx, n_rir, geom, rir_len, fs, c, rir_out, tap_count_out);
}

int aug_rir_visited_images(aug_ctx* ctx, int n_rir, const float* geom, int rir_len, float fs, float c,
                           float* rir_out, uint64_t* visited_out) {
    AUG_TRY(enter(ctx));
    if (n_rir < 0) return fail(ctx, AUG_ERR_INVALID_ARG, "n_rir is negative");
    AUG_TRY(check_rir_args(ctx, rir_len, fs, c));
    if (!visited_out) return fail(ctx, AUG_ERR_INVALID_ARG, "visited_out is null");
    *visited_out = 0;
    if (n_rir == 0) return AUG_OK;
    if (!geom || !rir_out) return fail(ctx, AUG_ERR_INVALID_ARG, "geom or rir_out is null");
    if ((int64_t)n_rir * aug::rir_items_per_response(rir_len) > 0x7fffffffLL)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "too many responses in one call");
    AUG_TRY(prepare_rir(ctx, n_rir, rir_len));
    AUG_TRY(grow(ctx, ctx->visits, sizeof(unsigned long long), "visit counter"));
    const double k = (double)fs / (double)c;
    const int n_groups = 2 * ctx->n_cu;
    AUG_HIP(aug::launch_fill_u32(ctx->stream, ctx->visits.ptr, 0u, 2), "visit counter clear");
    AUG_HIP(aug::launch_rir_plan(ctx->stream, n_groups, n_rir, geom, rir_len, k, ctx->rir_items.ptr,
                                 ctx->rir_ctrl.as<int>()), "rir plan kernel");
    AUG_HIP(aug::launch_rir(ctx->stream, n_groups, n_rir, geom, rir_len, k, ctx->rir_items.ptr, ctx->rir_ctrl.as<int>(),
                            rir_out, nullptr, false, ctx->visits.as<unsigned long long>()),
            "rir kernel");
    unsigned long long v = 0;
    AUG_HIP(hipMemcpyAsync(&v, ctx->visits.ptr, sizeof v, hipMemcpyDeviceToHost, ctx->stream), "visit counter copy");
    AUG_HIP(hipStreamSynchronize(ctx->stream), "stream synchronize");
    *visited_out = v;
    return AUG_OK;
}

int aug_rir_mics_batch(aug_ctx* ctx, int n_rir, int n_mic, const float* geom, const float* mics, int rir_len,
                       float fs, float c, float* rir_out, int32_t* tap_count_out) {
    AUG_TRY(enter(ctx));
    if (n_rir < 0) return fail(ctx, AUG_ERR_INVALID_ARG, "n_rir is negative");
    if (n_mic < 1 || n_mic > AUG_MAX_MIC) return fail(ctx, AUG_ERR_INVALID_ARG, "n_mic must be in 1..%d", AUG_MAX_MIC);
    AUG_TRY(check_rir_args(ctx, rir_len, fs, c));
    if (n_rir == 0) return AUG_OK;
    if (!geom || !mics || !rir_out) return fail(ctx, AUG_ERR_INVALID_ARG, "geom, mics or rir_out is null");
    const int64_t n_rows = (int64_t)n_rir * n_mic;
    if (n_rows * aug::rir_items_per_response(rir_len) > 0x7fffffffLL)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "too many responses in one call");
    // rewriting the rows is ordered after an earlier call's kernels by the stream; growing the buffer frees
    // the old one, which waits for them
    AUG_TRY(grow(ctx, ctx->mic_rows, sizeof(float) * 10 * (size_t)n_rows, "microphone rows"));
    AUG_TRY(mark(ctx, -1));
    AUG_HIP(aug::launch_rir_mic_rows(ctx->stream, n_rir, n_mic, geom, mics, ctx->mic_rows.as<float>()), "microphone rows kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_OTHER));
    return run_rir(ctx, (int)n_rows, ctx->mic_rows.as<float>(), rir_len, fs, c, rir_out, tap_count_out);
}

int aug_convolve_mix_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* speech, int n_noise,
                           const float* noise, const float* rir, int rir_len, const float* snr_db,
                           float* mixed_out, float* gains_out) {
    AUG_TRY(enter(ctx));
    AUG_TRY(check_offsets(ctx, n_utt, offsets));
    AUG_TRY(check_mix_args(ctx, n_utt, offsets[n_utt], n_noise, speech, noise, snr_db));
    if (rir_len < 1 || rir_len > AUG_MAX_RIR_LEN)
        return fail(ctx, rir_len < 1 ? AUG_ERR_INVALID_ARG : AUG_ERR_UNSUPPORTED,
                    "rir_len must be in 1..%d", AUG_MAX_RIR_LEN);
    if ((!rir && n_utt > 0) || (!mixed_out && offsets[n_utt] > 0))
        return fail(ctx, AUG_ERR_INVALID_ARG, "rir or mixed_out is null");
    AUG_TRY(sync_packing(ctx, n_utt, offsets, nullptr, aug::conv_fft_size(rir_len), 0));
    return run_convolve_mix(ctx, n_utt, n_noise, speech, noise, rir, rir_len, snr_db, mixed_out, gains_out);
}

int aug_vtlp_mel_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave, const float* alpha,
                       const aug_frontend_cfg* cfg, const int64_t* frame_offsets, float* feats_out) {
    AUG_TRY(enter(ctx));
    AUG_TRY(check_offsets(ctx, n_utt, offsets));
    AUG_TRY(check_frontend(ctx, cfg));
    AUG_TRY(check_frame_offsets(ctx, n_utt, offsets, frame_offsets, cfg));
    if ((!wave && offsets[n_utt] > 0) || (!alpha && n_utt > 0) || (!feats_out && frame_offsets[n_utt] > 0))
        return fail(ctx, AUG_ERR_INVALID_ARG, "wave, alpha or feats_out is null");
    AUG_TRY(sync_packing(ctx, n_utt, offsets, frame_offsets, 0, frontend_rows_per_group(ctx, n_utt, frame_offsets)));
    return run_mel(ctx, n_utt, wave, alpha, cfg, feats_out);
}

int aug_vtlp_mel_batch_static(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave, const float* alpha,
                              const aug_frontend_cfg* cfg, const int64_t* frame_offsets, float* feats_out) {
    AUG_TRY(enter(ctx));
    AUG_TRY(check_offsets(ctx, n_utt, offsets));
    AUG_TRY(check_frontend(ctx, cfg));
    AUG_TRY(check_frame_offsets(ctx, n_utt, offsets, frame_offsets, cfg));
    if ((!wave && offsets[n_utt] > 0) || (!alpha && n_utt > 0) || (!feats_out && frame_offsets[n_utt] > 0))
        return fail(ctx, AUG_ERR_INVALID_ARG, "wave, alpha or feats_out is null");
    if (n_utt > AUG_STATIC_MAX_UTT)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "%d utterances: the static scratch array holds tables for at most %d",
                    n_utt, AUG_STATIC_MAX_UTT);
    const int fpg = aug::mel_frames_per_group();
    int64_t n_groups = 0;
    for (int u = 0; u < n_utt; ++u) n_groups += (frame_offsets[u + 1] - frame_offsets[u] + fpg - 1) / fpg;
    if (n_groups > AUG_STATIC_MAX_ROW_GROUPS)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "%lld groups of %d output rows: the static scratch array holds at most %d",
                    (long long)n_groups, fpg, AUG_STATIC_MAX_ROW_GROUPS);
    if (cfg->win > 2048) return fail(ctx, AUG_ERR_UNSUPPORTED, "window longer than 2048 samples");
    if (n_utt == 0 || n_groups == 0) return AUG_OK;
    unsigned char* const base = ctx->scratch;            // the device address, not the array's name
    if (!base) return fail(ctx, AUG_ERR_HIP, "the static scratch array is not available on this device");
    if (ctx->ring.cap < 2 * ((size_t)n_utt + 1)) return fail(ctx, AUG_ERR_HIP, "staging ring missing");

    float2* const tw = reinterpret_cast<float2*>(base + ScratchLayout::twiddle);
    float* const window = reinterpret_cast<float*>(base + ScratchLayout::window);
    float* const dct = reinterpret_cast<float*>(base + ScratchLayout::dct);
    int64_t* const d_off = reinterpret_cast<int64_t*>(base + ScratchLayout::offsets);
    int64_t* const d_foff = reinterpret_cast<int64_t*>(base + ScratchLayout::frame_offsets);
    int* const d_first = reinterpret_cast<int*>(base + ScratchLayout::frame_first);
    int2* const d_items = reinterpret_cast<int2*>(base + ScratchLayout::frame_items);
    float2* const mel_tab = reinterpret_cast<float2*>(base + ScratchLayout::mel_tab);

    // Everything the kernels read from the array is rewritten here, in stream order, by this call.
    AUG_TRY(upload_offsets(ctx, (size_t)n_utt + 1, offsets, d_off, frame_offsets, d_foff));
    AUG_HIP(aug::launch_pack(ctx->stream, n_utt, d_off, d_foff, 0, fpg, nullptr, nullptr, 0, d_first, d_items, n_groups),
            "packing kernels");
    AUG_HIP(aug::launch_twiddle(ctx->stream, cfg->nfft / 2, tw), "twiddle kernel");
    AUG_HIP(aug::launch_window(ctx->stream, cfg->win, window), "window kernel");
    if (cfg->feature == AUG_FEAT_MFCC)
        AUG_HIP(aug::launch_dct_table(ctx->stream, cfg->n_ceps, cfg->n_mel, dct), "cosine table kernel");
    AUG_HIP(aug::launch_mel_table(ctx->stream, n_utt, alpha, *cfg, mel_tab), "mel table kernel");
    aug::MelArgs ma;
    ma.offsets = d_off;
    ma.frame_offsets = d_foff;
    ma.items = d_items;
    ma.n_items = n_groups;
    ma.frames_per_group = fpg;
    ma.wave = wave;
    ma.extra = nullptr;
    ma.extra_stride = 0;
    ma.gains = nullptr;
    ma.n_extra = 0;
    ma.mel_tab = mel_tab;
    ma.dct = cfg->feature == AUG_FEAT_MFCC ? dct : nullptr;
    ma.window = window;
    ma.twiddle = tw;
    ma.cfg = *cfg;
    ma.feats = feats_out;
    AUG_HIP(aug::launch_mel(ctx->stream, ma), "mel kernel");
    return AUG_OK;
}

int aug_feature_dim(const aug_frontend_cfg* cfg) {
    if (!cfg) return 0;
    return cfg->feature == AUG_FEAT_MFCC ? cfg->n_ceps : cfg->n_mel;
}

int aug_vtlp_resynth_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* wave, const float* alpha,
                           const aug_vtlp_cfg* cfg, float* wave_out) {
    AUG_TRY(enter(ctx));
    AUG_TRY(check_offsets(ctx, n_utt, offsets));
    if (!cfg) return fail(ctx, AUG_ERR_INVALID_ARG, "vtlp config is null");
    if (cfg->win < 2 || cfg->hop < 1 || cfg->nfft < cfg->win)
        return fail(ctx, AUG_ERR_INVALID_ARG, "need win >= 2, hop >= 1, nfft >= win");
    if (!aug::vtlp_supported(cfg->win, cfg->hop, cfg->nfft))
        return fail(ctx, AUG_ERR_UNSUPPORTED, "kernels are built for win 800, hop 400, nfft 2048");
    const int64_t total = offsets[n_utt];
    if (((!wave || !wave_out) && total > 0) || (!alpha && n_utt > 0))
        return fail(ctx, AUG_ERR_INVALID_ARG, "wave, alpha or wave_out is null");
    if (total > 0 && wave_out < wave + total && wave < wave_out + total)
        return fail(ctx, AUG_ERR_INVALID_ARG, "wave_out overlaps wave");
    AUG_TRY(sync_packing(ctx, n_utt, offsets, nullptr, 0, 0));
    if (n_utt == 0 || total == 0) return AUG_OK;
    int64_t max_len = 0;
    for (int u = 0; u < n_utt; ++u) max_len = std::max(max_len, offsets[u + 1] - offsets[u]);
    const float2* tw = nullptr;
    AUG_TRY(ensure_twiddle(ctx, aug::vtlp_fft_size(), &tw));
    AUG_TRY(grow(ctx, ctx->vtlp_tab, sizeof(float2) * (size_t)n_utt * aug::vtlp_table_entries(), "warp table"));
    AUG_TRY(mark(ctx, -1));
    AUG_HIP(aug::launch_vtlp_table(ctx->stream, n_utt, alpha, ctx->vtlp_tab.as<float2>()), "warp table kernel");
    AUG_HIP(aug::launch_fill_u32(ctx->stream, wave_out, 0u, total), "output clear");
    AUG_TRY(mark(ctx, AUG_STAGE_OTHER));
    AUG_HIP(aug::launch_vtlp_resynth(ctx->stream, n_utt, ctx->d_offsets.as<int64_t>(), max_len, wave,
                                     ctx->vtlp_tab.as<float2>(), tw, wave_out), "resynthesis kernel");
    AUG_TRY(mark(ctx, AUG_STAGE_VTLP));
    return AUG_OK;
}

int aug_pipeline_batch(aug_ctx* ctx, int n_utt, const int64_t* offsets, const float* speech, int n_noise,
                       const float* noise, const float* geom, int rir_len, float fs, float c,
                       const float* snr_db, const float* alpha, const aug_frontend_cfg* cfg,
                       const int64_t* frame_offsets, float* feats_out, float* rir_out, float* mixed_out,
                       float* gains_out) {
    AUG_TRY(enter(ctx));
    AUG_TRY(check_offsets(ctx, n_utt, offsets));
    AUG_TRY(check_mix_args(ctx, n_utt, offsets[n_utt], n_noise, speech, noise, snr_db));
    AUG_TRY(check_rir_args(ctx, rir_len, fs, c));
    AUG_TRY(check_frontend(ctx, cfg));
    AUG_TRY(check_frame_offsets(ctx, n_utt, offsets, frame_offsets, cfg));
    if (((!geom || !alpha) && n_utt > 0) || (!feats_out && frame_offsets[n_utt] > 0))
        return fail(ctx, AUG_ERR_INVALID_ARG, "geom, alpha or feats_out is null");
    if (n_utt == 0) return AUG_OK;
    const int n_src = 1 + n_noise;
    if ((int64_t)n_utt * n_src * aug::rir_items_per_response(rir_len) > 0x7fffffffLL)
        return fail(ctx, AUG_ERR_UNSUPPORTED, "too many responses in one call");
    AUG_TRY(sync_packing(ctx, n_utt, offsets, frame_offsets, aug::conv_fft_size(rir_len),
                         frontend_rows_per_group(ctx, n_utt, frame_offsets)));
    const int64_t total = offsets[n_utt];
    float* rir = rir_out;
    if (!rir) {
        AUG_TRY(grow(ctx, ctx->rir, sizeof(float) * (size_t)n_utt * n_src * rir_len, "response workspace"));
        rir = ctx->rir.as<float>();
    }
    AUG_TRY(prepare_rir(ctx, n_utt * n_src, rir_len));
    AUG_TRY(prepare_convolve_mix(ctx, n_utt, n_noise, rir_len));
    AUG_TRY(prepare_mel(ctx, n_utt, cfg));
    AUG_TRY(run_rir(ctx, n_utt * n_src, geom, rir_len, fs, c, rir, nullptr));
    AUG_TRY(run_convolve_mix(ctx, n_utt, n_noise, speech, noise, rir, rir_len, snr_db, mixed_out, gains_out));
    if (mixed_out || total == 0) return run_mel(ctx, n_utt, mixed_out, alpha, cfg, feats_out);
    // The mixture itself is not wanted: the front end adds the scaled reverberated noises to the
    // reverberated speech as it loads its frames, which saves one pass over the batch through HBM.
    const float* reverb = ctx->reverb.as<float>();
    const int64_t stride = reverb_stride(total);
    return run_mel(ctx, n_utt, reverb, alpha, cfg, feats_out, n_noise, reverb + stride, stride, ctx->gains.as<float>());
}

}  // extern "C"
