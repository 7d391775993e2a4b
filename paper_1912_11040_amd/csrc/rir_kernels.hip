// Image-method room impulse responses (the acoustic simulator of Sec. 2.3 computes
// them on the fly for every training example).
//
// h[n] = sum over image sources with floor(d fs/c + 0.5) == n of beta^k / (4 pi d),
// d = distance image -> microphone, k = number of wall reflections of that image.
// Along one axis the images of a source at s between walls at 0 and L are
// (1 - 2q) s + 2 n L, q in {0,1}, n integer, reflected |n - q| + |n| times.
//
// The tap index is integer work decided by floating point, so it follows one fixed
// fp64 recipe with no contraction:
//     d2 = (dx*dx + dy*dy) + dz*dz;  idx = floor(sqrt(d2) * (fs/c) + 0.5)
// A cheap estimate of sqrt (fp32 rsq + one fp64 Newton step) decides the index
// whenever the result is farther from a rounding boundary than the estimate's error
// bound; the rare remaining images take the exact correctly-rounded sqrt.
//
// Layout of the work
//   * plan kernel: one thread per response cuts its taps into shells [n0, n1) of about
//     equal image count (equal volume of the spherical shell) and at most kMaxTaps taps,
//     and appends them to an item table.
//   * image kernel: persistent work groups fetch items from a counter.  An item owns its
//     taps, so sums live in LDS and are stored once, without global atomics.
//     A wave takes 64 (x image, y image) columns at a time; each column contributes up to
//     four runs of consecutive z images inside the shell.  Runs are cut into pieces of at
//     most kPiece images, the pieces are dealt to lanes, and each lane walks its piece.
//   * amplitudes accumulate as 64-bit fixed point (2^-56) with integer LDS atomics:
//     gfx950 executes float LDS atomics about thirty times slower than integer ones, and
//     integer sums do not depend on the order of arrival.

#include "aug_internal.h"

namespace aug {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxTaps = 6016;            // taps owned by one item (LDS: 8 bytes each)
constexpr int kMinTaps = 64;
constexpr int kPow = 1024;                // beta^k table entries held in LDS
constexpr int kZCap = 320;                // z images per q held in LDS; more than that: computed in the loop
constexpr int kPiece = 16;                // images per piece
constexpr float kTargetImages = 800000.f; // images per item aimed for (before reflection cuts)
constexpr int kMaxShells = 96;            // volume-balanced shells per response, at most

#pragma clang fp contract(off)

struct Axis {
    double room, src, mic;
};

// delta of image (q, n) to the microphone along one axis, in the reference operation order
__device__ inline double axis_delta(const Axis& a, int q, int n) {
    const double sgn = q ? -1.0 : 1.0;
    const double coord = __dadd_rn(__dmul_rn(sgn, a.src), __dmul_rn(__dmul_rn(2.0, (double)n), a.room));
    return __dsub_rn(coord, a.mic);
}

__device__ inline int iabs(int v) { return v < 0 ? -v : v; }

__device__ inline bool room_ok(const float* g) {
    return (g[0] >= 0.1f) && (g[1] >= 0.1f) && (g[2] >= 0.1f) && (g[0] * g[1] * g[2] < 1e30f);
}

struct Item { int rir, n0, n1; };

// ctrl[0] = number of items, ctrl[1] = next item to hand out
__global__ void rir_plan_kernel(int n_rir, const float* __restrict__ geom, int rir_len, double k_fs_c,
                                Item* __restrict__ items, int items_per_rir, int* __restrict__ ctrl) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rir) return;
    const float* g = geom + (size_t)r * 10;
    const double radius = (double)rir_len / k_fs_c;
    float shells = 1.f;
    if (room_ok(g)) {
        const float est = 4.18879f * (float)(radius * radius * radius) / (g[0] * g[1] * g[2]);
        shells = fminf(fmaxf(ceilf(est / kTargetImages), 1.f), (float)kMaxShells);
    }
    const double L3 = (double)rir_len * rir_len * rir_len;
    const double step = L3 / (double)shells;
    int bounds[kMaxShells + AUG_MAX_RIR_LEN / kMaxTaps + 4];
    int count = 0, b = 0;
    while (b < rir_len && count < items_per_rir - 1) {
        int nb = (int)cbrt((double)b * b * b + step);
        nb = max(nb, b + kMinTaps);
        nb = min(min(nb, b + kMaxTaps), rir_len);
        bounds[count++] = nb;
        b = nb;
    }
    if (b < rir_len) {          // out of table space: cannot happen with the sizes chosen by the host
        while (b < rir_len && count < items_per_rir) {
            const int nb = min(b + kMaxTaps, rir_len);
            bounds[count++] = nb;
            b = nb;
        }
    }
    const int base = atomicAdd(&ctrl[0], count);
    int lo = 0;
    for (int i = 0; i < count; ++i) {
        items[base + i] = Item{r, lo, bounds[i]};
        lo = bounds[i];
    }
}

__global__ void rir_pow_kernel(int n_rir, const float* __restrict__ geom, float* __restrict__ table) {
    const int r = blockIdx.y;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= kPow) return;
    table[(size_t)r * kPow + k] = (float)pow((double)geom[(size_t)r * 10 + 9], (double)k);
}

// per-column record shared through LDS between the lane that built it and the lanes that walk its pieces
struct __align__(16) Column {
    double a;            // dx*dx + dy*dy
    int kxy;             // reflections along x and y
    int pfx;             // inclusive prefix of piece counts within the wave's batch
    short start[4];      // first n of runs (q=0: runs 0,1; q=1: runs 2,3)
    short len[4];
};

__device__ inline int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}

struct __align__(16) ZEntry {
    double dz2;          // squared z distance of image (q, n), reference operation order
    float bz;            // beta^(|n-q| + |n|)
    float pad;
};

struct WalkCtx {
    double k_fs_c;
    double guard;        // estimates closer than this to a rounding boundary are redone exactly
    double beta;
    int n0, n_taps;
};

// Largest reflection count k whose amplitude beta^k / (4 pi d) can still reach one unit of the
// 2^-56 fixed point at distance d_min or beyond, with a factor-of-two margin and one count of slack;
// "no limit" when beta is 0, >= 1 (log2_beta == 0 encodes both) or d_min is tiny.
__device__ inline int reflection_cut(float log2_beta, float d_min) {
    if (!(log2_beta < 0.f) || !(d_min > 1e-3f)) return 1 << 20;
    // beta^k >= 4 pi d 2^-57  <=>  k <= (log2(4 pi d) - 57) / log2(beta)
    const float k = (__log2f(12.566371f * d_min) - 57.f) / log2_beta;
    return k > 1.0e6f ? (1 << 20) : (int)k + 2;
}

// the reference recipe, kept out of line so that the estimate's loop stays short
__device__ __attribute__((noinline)) int exact_tap(double d2, double k_fs_c) {
    const double d = __dsqrt_rn(d2);
    return (int)__dadd_rn(__dmul_rn(d, k_fs_c), 0.5);     // positive: truncation is floor
}

// Tap index of an image at squared distance d2, and y ~ 1/sqrt(d2) for its amplitude.
__device__ inline int tap_index(const WalkCtx& w, double d2, float& y) {
    const float d2f = (float)d2;
    y = __frsqrt_rn(d2f);
    const double s0 = (double)(d2f * y);                   // sqrt(d2) to ~2e-7
    const double res = fma(-s0, s0, d2);                   // exact residual
    const double s1 = fma(res, (double)(0.5f * y), s0);    // one Newton step: ~1e-13 relative
    const double t = fma(s1, w.k_fs_c, 0.5);
    const double frac = __builtin_amdgcn_fract(t);
    int idx = (int)t;
    if (fabs(frac - 0.5) > 0.5 - w.guard) idx = exact_tap(d2, w.k_fs_c);
    return idx;
}

template <bool COUNT>
__device__ inline void deposit(const WalkCtx& w, int idx, float x, unsigned long long* hist, unsigned int* hist32) {
    const unsigned int rel = (unsigned int)(idx - w.n0);
    if (rel >= (unsigned int)w.n_taps) return;
    if (COUNT) {
        atomicAdd(&hist32[rel], 1u);
    } else {
        // x = amplitude * 2^24; amplitude * 2^56 as a 64-bit integer from two exact fp32 scalings
        const float fr = __builtin_amdgcn_fractf(x);
        const unsigned int hi = (unsigned int)x;
        const unsigned int lo = (unsigned int)(fr * 4294967296.0f);
        atomicAdd(&hist[rel], ((unsigned long long)hi << 32) | lo);
    }
}

template <bool COUNT>
__device__ inline void walk_piece_table(const WalkCtx& w, double a, float cxy, const ZEntry* z, int len,
                                        unsigned long long* hist, unsigned int* hist32) {
    for (int i = 0; i < len; ++i) {
        const ZEntry e = z[i];
        const double d2 = __dadd_rn(a, e.dz2);
        float y;
        const int idx = tap_index(w, d2, y);
        deposit<COUNT>(w, idx, (e.bz * y) * cxy, hist, hist32);
    }
}

template <bool COUNT>
__device__ inline void walk_piece_direct(const WalkCtx& w, const Axis& az, double a, float cxy, int q, int first,
                                         int len, unsigned long long* hist, unsigned int* hist32) {
    for (int i = 0; i < len; ++i) {
        const int n = first + i;
        const double dz = axis_delta(az, q, n);
        const double d2 = __dadd_rn(a, __dmul_rn(dz, dz));
        float y;
        const int idx = tap_index(w, d2, y);
        float bz = 0.f;
        if (!COUNT) bz = (float)pow(w.beta, (double)(iabs(n - q) + iabs(n)));
        deposit<COUNT>(w, idx, (bz * y) * cxy, hist, hist32);
    }
}

template <bool COUNT>
__global__ __launch_bounds__(kThreads, 4) void rir_image_kernel(
    const float* __restrict__ geom, int rir_len, double k_fs_c, const Item* __restrict__ items,
    int* __restrict__ ctrl, const float* __restrict__ pow_table, float* __restrict__ rir_out,
    int32_t* __restrict__ cnt_out) {
    __shared__ unsigned long long hist[COUNT ? kMaxTaps / 2 : kMaxTaps];
    __shared__ float bpow[COUNT ? 1 : kPow];
    __shared__ ZEntry ztab[2 * kZCap];
    __shared__ Column cols[kWaves][64];
    __shared__ int s_item;
    unsigned int* hist32 = reinterpret_cast<unsigned int*>(hist);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_items = ctrl[0];

    for (;;) {
        if (tid == 0) s_item = atomicAdd(&ctrl[1], 1);
        __syncthreads();
        const int it = s_item;
        if (it >= n_items) break;
        const Item item = items[it];
        const int n0 = item.n0, n1 = item.n1, n_taps = n1 - n0;
        const float* g = geom + (size_t)item.rir * 10;

        if (COUNT) {
            for (int i = tid; i < n_taps; i += kThreads) hist32[i] = 0u;
        } else {
            for (int i = tid; i < n_taps; i += kThreads) hist[i] = 0ull;
            for (int i = tid; i < kPow; i += kThreads) bpow[i] = pow_table[(size_t)item.rir * kPow + i];
        }
        __syncthreads();

        if (room_ok(g)) {
            const Axis ax{(double)g[0], (double)g[3], (double)g[6]};
            const Axis ay{(double)g[1], (double)g[4], (double)g[7]};
            const Axis az{(double)g[2], (double)g[5], (double)g[8]};
            const double beta = (double)g[9];
            // every image of this item lies in r_in <= d < r_out (half a tap of slack on either side)
            const double r_out = (double)n1 / k_fs_c;
            const double r_in = n0 > 0 ? (double)(n0 - 1) / k_fs_c : 0.0;
            const double r_out2 = r_out * r_out, r_in2 = r_in * r_in;
            // An image reflected k times adds beta^k / (4 pi d) * 2^56, truncated to an integer, to its
            // tap; once beta^k < 2 pi d 2^-56 that is exactly zero, so such images are never visited.
            // log2_beta < 0 enables the cut (amplitude sums only; tap counts visit every image).
            const float log2_beta = (!COUNT && g[9] > 0.f && g[9] < 1.f) ? __log2f(g[9]) : 0.f;
            const int k_cut_item = reflection_cut(log2_beta, (float)r_in);
            int nmx = (int)ceil(r_out / (2.0 * ax.room)) + 1;
            int nmy = (int)ceil(r_out / (2.0 * ay.room)) + 1;
            const int nmz = (int)ceil(r_out / (2.0 * az.room)) + 1;
            nmx = min(nmx, k_cut_item / 2 + 1);          // |n - q| + |n| >= 2 |n| - 1
            nmy = min(nmy, k_cut_item / 2 + 1);
            const int nix = 2 * (2 * nmx + 1), niy = 2 * (2 * nmy + 1);
            const int n_cand = nix * niy;
            const float inv_two_lzf = (float)(1.0 / (2.0 * az.room));
            const float z0qf[2] = {(float)(az.src - az.mic), (float)(-az.src - az.mic)};
            const int n_batch = (n_cand + 63) / 64;
            Column* wc = cols[wave];
            WalkCtx wctx;
            wctx.k_fs_c = k_fs_c;
            wctx.guard = 1e-12 * (double)(n1 + 1) + 1e-13;
            wctx.n0 = n0;
            wctx.n_taps = n_taps;
            wctx.beta = beta;

            // z images of this response: (dz*dz, beta^reflections) per (q, n), shared by every column
            const bool use_table = 2 * nmz + 1 <= kZCap;
            if (use_table) {
                const int per_q = 2 * nmz + 1;
                for (int i = tid; i < 2 * per_q; i += kThreads) {
                    const int q = i >= per_q, n = i - q * per_q - nmz;
                    const double dz = axis_delta(az, q, n);
                    ZEntry e;
                    e.dz2 = __dmul_rn(dz, dz);
                    e.bz = 0.f;
                    if (!COUNT) {
                        const int k = iabs(n - q) + iabs(n);
                        e.bz = k < kPow ? bpow[k] : (float)pow(beta, (double)k);
                    }
                    e.pad = 0.f;
                    ztab[q * kZCap + n + nmz] = e;
                }
            }
            __syncthreads();

            for (int batch = wave; batch < n_batch; batch += kWaves) {
                // ---- each lane describes one candidate column ----
                const int cand = batch * 64 + lane;
                Column col;
                col.a = 0.0; col.kxy = 0;
                int pieces = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) { col.start[i] = 0; col.len[i] = 0; }
                if (cand < n_cand) {
                    const int ix = cand / niy, iy = cand - ix * niy;
                    const int qx = ix & 1, nx = (ix >> 1) - nmx;
                    const int qy = iy & 1, ny = (iy >> 1) - nmy;
                    const double dx = axis_delta(ax, qx, nx);
                    const double dy = axis_delta(ay, qy, ny);
                    col.a = __dadd_rn(__dmul_rn(dx, dx), __dmul_rn(dy, dy));
                    col.kxy = iabs(nx - qx) + iabs(nx) + iabs(ny - qy) + iabs(ny);
                    // reflections left for the z axis before this column's images vanish
                    const int kz_max = reflection_cut(log2_beta, fmaxf((float)r_in, sqrtf((float)col.a))) - col.kxy;
                    if (col.a < r_out2 && kz_max >= 0) {
                        // z reach of the shell in this column; fp32 is enough because the shell radii carry
                        // half a tap (about a centimetre) of slack and the exact tap test decides anyway
                        const float zout = sqrtf((float)(r_out2 - col.a));
                        const float zin = col.a < r_in2 ? sqrtf((float)(r_in2 - col.a)) : 0.f;
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const float z0 = z0qf[q];
                            // |n - q| + |n| <= kz_max  <=>  cut_lo <= n <= cut_hi
                            const int cut_lo = q ? -((kz_max - 1) >> 1) : -(kz_max >> 1);
                            const int cut_hi = q ? ((kz_max + 1) >> 1) : (kz_max >> 1);
                            const int lo_n = max((int)ceilf((-zout - z0) * inv_two_lzf - 1e-4f), cut_lo);
                            const int hi_n = min((int)floorf((-zin - z0) * inv_two_lzf + 1e-4f), cut_hi);
                            const int lo_p = max((int)ceilf((zin - z0) * inv_two_lzf - 1e-4f), cut_lo);
                            const int hi_p = min((int)floorf((zout - z0) * inv_two_lzf + 1e-4f), cut_hi);
                            if (hi_n >= lo_p - 1) {            // the two sides touch: one run
                                col.start[2 * q] = (short)lo_n;
                                col.len[2 * q] = (short)max(hi_p - lo_n + 1, 0);
                            } else {
                                col.start[2 * q] = (short)lo_n;
                                col.len[2 * q] = (short)max(hi_n - lo_n + 1, 0);
                                col.start[2 * q + 1] = (short)lo_p;
                                col.len[2 * q + 1] = (short)max(hi_p - lo_p + 1, 0);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) pieces += (col.len[i] + kPiece - 1) / kPiece;
                    }
                }
                col.pfx = wave_inclusive_scan(pieces, lane);
                const int n_pieces = __shfl(col.pfx, 63, 64);
                wc[lane] = col;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

                // ---- pieces are dealt to lanes ----
                for (int p = lane; p < n_pieces; p += 64) {
                    int slot = 0;                               // smallest slot with pfx > p
#pragma unroll
                    for (int s = 32; s > 0; s >>= 1)
                        if (wc[slot + s - 1].pfx <= p) slot += s;
                    const Column c = wc[slot];
                    int local = p - (slot ? wc[slot - 1].pfx : 0);
                    // which of the four runs holds piece `local` (selects only: no register indexing)
                    int run = 0, r_start = c.start[0], r_len = c.len[0];
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        const int np = ((int)c.len[i] + kPiece - 1) / kPiece;
                        if (run == i && local >= np) {
                            local -= np;
                            run = i + 1;
                            r_start = c.start[i + 1];
                            r_len = c.len[i + 1];
                        }
                    }
                    const int q = run >> 1;
                    const int first = r_start + local * kPiece;
                    const int len = min(kPiece, r_len - local * kPiece);
                    float cxy = 0.f;       // beta^kxy / (4 pi) * 2^24
                    if (!COUNT)
                        cxy = (c.kxy < kPow ? bpow[c.kxy] : (float)pow(beta, (double)c.kxy)) * (0.07957747154594767f * 16777216.0f);
                    if (use_table)
                        walk_piece_table<COUNT>(wctx, c.a, cxy, ztab + q * kZCap + first + nmz, len, hist, hist32);
                    else
                        walk_piece_direct<COUNT>(wctx, az, c.a, cxy, q, first, len, hist, hist32);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        __syncthreads();

        if (COUNT) {
            int32_t* out = cnt_out + (size_t)item.rir * rir_len + n0;
            for (int i = tid; i < n_taps; i += kThreads) out[i] = (int32_t)hist32[i];
        } else {
            float* out = rir_out + (size_t)item.rir * rir_len + n0;
            for (int i = tid; i < n_taps; i += kThreads) {
                const unsigned long long v = hist[i];
                const double d = (double)(unsigned int)(v >> 32) * 4294967296.0 + (double)(unsigned int)v;
                out[i] = (float)(d * 1.3877787807814457e-17);       // 2^-56
            }
        }
        __syncthreads();
    }
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

}  // namespace

hipError_t launch_fill_u32(hipStream_t s, void* p, uint32_t v, int64_t n) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    fill_u32_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<uint32_t*>(p), v, n);
    return hipGetLastError();
}

int rir_items_per_response(int rir_len) { return kMaxShells + rir_len / kMaxTaps + 2; }
size_t rir_item_bytes() { return sizeof(Item); }
int rir_pow_entries() { return kPow; }

hipError_t launch_rir_plan(hipStream_t s, int n_rir, const float* geom, int rir_len, double fs_over_c,
                           void* items, int* ctrl, float* pow_table) {
    if (n_rir <= 0) return hipSuccess;
    hipError_t e = launch_fill_u32(s, ctrl, 0u, 2);
    if (e != hipSuccess) return e;
    rir_plan_kernel<<<dim3((n_rir + 127) / 128), dim3(128), 0, s>>>(
        n_rir, geom, rir_len, fs_over_c, static_cast<Item*>(items), rir_items_per_response(rir_len), ctrl);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    rir_pow_kernel<<<dim3(kPow / 256, (unsigned)n_rir), dim3(256), 0, s>>>(n_rir, geom, pow_table);
    return hipGetLastError();
}

hipError_t launch_rir(hipStream_t s, int n_groups, int n_rir, const float* geom, int rir_len, double fs_over_c,
                      const void* items, int* ctrl, const float* pow_table, float* rir_out, int32_t* cnt_out) {
    if (n_rir <= 0) return hipSuccess;
    hipError_t e = launch_fill_u32(s, ctrl + 1, 0u, 1);      // restart the item counter
    if (e != hipSuccess) return e;
    const Item* it = static_cast<const Item*>(items);
    if (rir_out)
        rir_image_kernel<false><<<dim3((unsigned)n_groups), dim3(kThreads), 0, s>>>(
            geom, rir_len, fs_over_c, it, ctrl, pow_table, rir_out, nullptr);
    else
        rir_image_kernel<true><<<dim3((unsigned)n_groups), dim3(kThreads), 0, s>>>(
            geom, rir_len, fs_over_c, it, ctrl, pow_table, nullptr, cnt_out);
    return hipGetLastError();
}

}  // namespace aug
