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
// A cheap estimate of sqrt (the hardware's double-precision rsq + one Newton step) decides
// the index whenever the result is farther from a rounding boundary than the estimate's
// error bound; the rare remaining images take the exact correctly-rounded sqrt.
//
// Layout of the work
//   * plan kernels: one thread per response cuts its taps into shells [n0, n1) of about
//     equal image count (equal volume of the spherical shell) and at most kMaxTaps taps; the shell size
//     follows the batch's estimated work per persistent group.  Every shell gets an estimate of its work
//     and a counting sort orders the items heaviest first.
//   * image kernel: persistent work groups fetch items from a counter.  An item owns its
//     taps, so sums live in LDS and are stored once, without global atomics.
//     The z images of the response (both q, both signs) are merged into one LDS table sorted by
//     dz*dz, so the images of an (x image, y image) column that can fall inside the shell are one
//     contiguous range of that table between r_in^2 - a and r_out^2 - a, whose ends are counted from the
//     two arithmetic progressions that the axis's images form rather than searched for.
//     The y images are sorted the same way, so the live columns of an x image are a prefix of the
//     y table; a prefix sum over the x images numbers the live columns and dead ones are never seen.
//     A wave takes 64 live columns at a time; their z ranges are cut into pieces of at most kPiece
//     images, a wave scan numbers the pieces, and lanes take pieces 64 at a time (a piece finds its column by
//     counting bits in a map of the columns' first pieces) and walk them, two images side by side.
//     Rooms so flat or narrow that an axis has more images than the tables hold take a plain path
//     (all columns of the bounding box, every z image of a live column).
//   * amplitudes accumulate as 64-bit fixed point (2^-56, each increment rounded to the nearest unit)
//     with integer LDS atomics: gfx950 executes float LDS atomics about thirty times slower than integer
//     ones, and integer sums do not depend on the order of arrival nor on how a batch is cut into items.

#include "aug_internal.h"

namespace aug {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxTaps = 5632;            // taps owned by one item (LDS: 8 bytes each)
constexpr int kMinTaps = 64;
constexpr int kPow = 1024;                // beta^k table entries held in LDS
constexpr int kAxisCap = 320;             // y or z images per q held in the sorted LDS tables 
constexpr int kPiece = 12;                // images per piece
constexpr int kWalkGroup = 2;             // images a lane works on side by side (three or four measured no better)
constexpr int kStartWords = 32;           // pieces are dealt in chunks of 32 * kStartWords (one bit each in LDS)
// Work per item, in image visits (see item_cost): the batch's estimated work divided by the number of
// persistent groups and by kItemsPerGroup, within limits.  Thick shells visit fewer (x, y) columns per image
// (every shell sets up all columns inside its outer radius), thin ones even out the groups' finishing
// times; every response yields at least one item, so the groups still get several items each.  Measured:
// 16000-tap batch 0.89 -> 0.80 ms, 32768-tap batch 12.8 -> 7.6 ms against a fixed 600000.
constexpr float kItemsPerGroup = 1.25f;
// (the lower limit matters for small batches only, where items must be small for all groups to get one:
// 64 utterances with 8000-tap responses take 0.122 ms at 300000, 0.080 ms at 50000)
constexpr float kMinTargetWork = 50000.f, kMaxTargetWork = 8000000.f;
constexpr float kWorkUnit = 4096.f;       // the batch total is summed in integers of this many visits
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

// A value that every lane of the wavefront has computed alike, moved to scalar registers: what an item's
// geometry determines is the same in all lanes and would otherwise occupy vector registers for the whole item.
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline float uni(float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); }
__device__ inline double uni(double v) { return __hiloint2double(uni(__double2hiint(v)), uni(__double2loint(v))); }

// A usable room has sides of at least 10 cm (else the image lattice is unbounded) and a reflection
// coefficient in [0, 1] (amplitudes are summed as unsigned fixed point and must not grow with the
// reflection count); the comparisons are false for values that are not numbers.
__device__ inline bool room_ok(const float* g) {
    return (g[0] >= 0.1f) && (g[1] >= 0.1f) && (g[2] >= 0.1f) && (g[0] * g[1] * g[2] < 1e30f) &&
           (g[9] >= 0.f) && (g[9] <= 1.f);
}

struct Item { int rir, n0, n1, cls; };

__device__ inline void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}


constexpr int kClasses = 32;            // cost classes for the order in which items are handed out
// ctrl: [0] number of items, [1] next item to hand out, [2 .. 2+kClasses) items per class,
// [2+kClasses .. 2+2 kClasses) next free slot of each class in the sorted table, then the batch's
// estimated work in units of kWorkUnit
constexpr int kCtrlWork = 2 + 2 * kClasses;
constexpr int kCtrlInts = kCtrlWork + 1;

// Fraction of the images at distance d that the reflection cut keeps: an image in direction u has
// about d (|ux|/Lx + |uy|/Ly + |uz|/Lz) reflections, so this is the share of directions whose
// reflections per metre stay under cut / d, counted on a fixed 8 x 8 equal-area lattice of an octant.
__device__ inline float kept_fraction(const float* g, float log2_beta, float d) {
    if (!(log2_beta < 0.f) || !(d > 1e-3f)) return 1.f;
    const float per_metre = (__log2f(12.566371f * d) - 57.f) / (log2_beta * d);
    const float ix = 1.f / g[0], iy = 1.f / g[1], iz = 1.f / g[2];
    int kept = 0;
    for (int i = 0; i < 8; ++i) {
        const float uz = (i + 0.5f) * 0.125f, rho = sqrtf(1.f - uz * uz);
        for (int j = 0; j < 8; ++j) {
            float sn, cs;
            __sincosf((j + 0.5f) * 0.19634954f, &sn, &cs);
            kept += (rho * cs * ix + rho * sn * iy + uz * iz) <= per_metre;
        }
    }
    return fmaxf((float)kept * (1.f / 64.f), 1.f / 128.f);
}

// Work of one item in units of one image visit: the images it keeps plus about twelve visits' worth
// of set-up for every live (x image, y image) column inside its outer radius.
__device__ inline float item_cost(const float* g, float log2_beta, float est_images, float rir_len, float n0, float n1,
                                  float metres_per_tap) {
    const float share = (n1 * n1 * n1 - n0 * n0 * n0) / (rir_len * rir_len * rir_len);
    const float f = kept_fraction(g, log2_beta, 0.5f * (n0 + n1) * metres_per_tap);
    const float r_out = n1 * metres_per_tap;
    const float columns = 3.14159265f * r_out * r_out / (g[0] * g[1]);
    return est_images * share * f + 12.f * columns * __powf(f, 0.6667f);
}

// estimated work of a whole response (0 for a room that is not usable)
__device__ inline float response_work(const float* g, int rir_len, double k_fs_c) {
    if (!room_ok(g)) return 0.f;
    const double radius = (double)rir_len / k_fs_c;
    const float log2_beta = (g[9] > 0.f && g[9] < 1.f) ? __log2f(g[9]) : 0.f;
    const float est = 4.18879f * (float)(radius * radius * radius) / (g[0] * g[1] * g[2]);
    return item_cost(g, log2_beta, est, (float)rir_len, 0.f, (float)rir_len, (float)(1.0 / k_fs_c));
}

// one thread per response: the batch's estimated work (an integer sum, so it does not depend on the order)
__global__ void rir_work_kernel(int n_rir, const float* __restrict__ geom, int rir_len, double k_fs_c,
                                int* __restrict__ ctrl) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    int units = 0;
    if (r < n_rir) units = (int)fminf(response_work(geom + (size_t)r * 10, rir_len, k_fs_c) / kWorkUnit, 500000.f) + 1;
    for (int off = 32; off > 0; off >>= 1) units += __shfl_down(units, off, 64);      // one atomic per wavefront
    if ((threadIdx.x & 63) == 0 && units) atomicAdd(&ctrl[kCtrlWork], units);
}

// Work per item that a batch of `units` work units (kWorkUnit visits each) aims at.
__device__ inline float item_target(int units, int n_groups) {
    return fminf(fmaxf(kWorkUnit * (float)units / ((float)n_groups * kItemsPerGroup), kMinTargetWork), kMaxTargetWork);
}

constexpr int kMaxBounds = kMaxShells + AUG_MAX_RIR_LEN / kMaxTaps + 4;

// Cut the taps of a response of estimated work `work` into shells of about equal image count (equal volume), at most kMaxTaps wide:
// bounds[i] is the lower bound of shell i, outermost shell first; returns their number.
// Shells are cut from the outside in: every shell sets up all (x, y) columns inside its outer radius, so
// where the tap limit, not the work, decides the width it is the inner shells, with few columns, that
// should be the many and the narrow ones, and the left-over sliver belongs at the centre.
__device__ inline int cut_shells(float work, int rir_len, float target, int items_per_rir, int (&bounds)[kMaxBounds]) {
    const float shells = fminf(fmaxf(ceilf(work / target), 1.f), (float)kMaxShells);
    const double L3 = (double)rir_len * rir_len * rir_len;
    const double step = L3 / (double)shells;
    int count = 0, hi = rir_len;
    while (hi > 0 && count < items_per_rir - 1) {
        const double h3 = (double)hi * hi * hi;
        int lo = h3 > step ? (int)cbrt(h3 - step) : 0;
        lo = min(lo, hi - kMinTaps);
        lo = max(max(lo, hi - kMaxTaps), 0);
        if (lo < kMinTaps && hi <= kMaxTaps) lo = 0;              // no sliver at the centre
        bounds[count++] = lo;
        hi = lo;
    }
    while (hi > 0 && count < items_per_rir) {                       // out of table space: cannot happen with the
        const int lo = max(hi - kMaxTaps, 0);                       // sizes chosen by the host
        bounds[count++] = lo;
        hi = lo;
    }
    return count;
}

// cost class of an item (0 = heaviest)
__device__ inline int item_class(const float* g, int rir_len, double k_fs_c, int n0, int n1) {
    if (!room_ok(g)) return kClasses - 1;
    const double radius = (double)rir_len / k_fs_c;
    const float est = 4.18879f * (float)(radius * radius * radius) / (g[0] * g[1] * g[2]);
    const float log2_beta = (g[9] > 0.f && g[9] < 1.f) ? __log2f(g[9]) : 0.f;
    const float cost = item_cost(g, log2_beta, est, (float)rir_len, (float)n0, (float)n1, (float)(1.0 / k_fs_c));
    return min(max((int)(2.5f * __log2f(3.2e7f / fmaxf(cost, 1.f))), 0), kClasses - 1);
}

// One thread per response: cut its taps into shells and append them to the unsorted item table.
__global__ void rir_plan_kernel(int n_rir, const float* __restrict__ geom, int rir_len, double k_fs_c,
                                Item* __restrict__ unsorted, int items_per_rir, int* __restrict__ ctrl, int n_groups) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rir) return;
    const float* g = geom + (size_t)r * 10;
    int bounds[kMaxBounds];
    const int count = cut_shells(response_work(g, rir_len, k_fs_c), rir_len, item_target(ctrl[kCtrlWork], n_groups),
                                 items_per_rir, bounds);
    const int base = atomicAdd(&ctrl[0], count);
    int top = rir_len;
    for (int i = 0; i < count; ++i) {
        unsorted[base + i] = Item{r, bounds[i], top, kClasses - 1};
        top = bounds[i];
    }
}

// The whole plan in one work group, for batches of at most kPlanThreads responses (four launches and a clear
// cost more than the work there): a thread per response for the batch's work and the shells (their places in
// the table by a scan, not by atomics), then all threads over the items for their classes and the counting
// sort.  Leaves ctrl[0] = number of items, ctrl[1] = 0.
constexpr int kPlanThreads = 1024;
__global__ __launch_bounds__(kPlanThreads) void rir_plan_all_kernel(
    int n_rir, const float* __restrict__ geom, int rir_len, double k_fs_c, Item* __restrict__ sorted,
    Item* __restrict__ unsorted, int items_per_rir, int* __restrict__ ctrl, int n_groups) {
    __shared__ int part[kPlanThreads / 64];
    __shared__ int census[kClasses], first_slot[kClasses], cursor[kClasses];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < kClasses) census[tid] = cursor[tid] = 0;
    const int r = tid;                                 // this thread's response, if any
    const float* g = geom + (size_t)min(r, n_rir - 1) * 10;

    const float work = r < n_rir ? response_work(g, rir_len, k_fs_c) : 0.f;
    int units = r < n_rir ? (int)fminf(work / kWorkUnit, 500000.f) + 1 : 0;
    for (int off = 32; off > 0; off >>= 1) units += __shfl_down(units, off, 64);
    if (lane == 0) part[wave] = units;
    __syncthreads();
    int total_units = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) total_units += part[w];
    const float target = item_target(total_units, n_groups);
    __syncthreads();

    int bounds[kMaxBounds];
    const int count = r < n_rir ? cut_shells(work, rir_len, target, items_per_rir, bounds) : 0;
    const int incl = wave_inclusive_scan(count, lane);
    if (lane == 63) part[wave] = incl;
    __syncthreads();
    int before = 0, n_items = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) {
        if (w < wave) before += part[w];
        n_items += part[w];
    }
    {
        const int base = before + incl - count;
        int top = rir_len;
        for (int i = 0; i < count; ++i) {
            unsorted[base + i] = Item{r, bounds[i], top, kClasses - 1};
            top = bounds[i];
        }
    }
    __syncthreads();                                   // the group's writes to `unsorted` are visible to it
    for (int i = tid; i < n_items; i += kPlanThreads) {
        const Item it = unsorted[i];
        const int cls = item_class(geom + (size_t)it.rir * 10, rir_len, k_fs_c, it.n0, it.n1);
        unsorted[i].cls = cls;                         // (read back by this same thread below)
        atomicAdd(&census[cls], 1);
    }
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int c = 0; c < kClasses; ++c) {
            first_slot[c] = at;
            at += census[c];
        }
        ctrl[0] = n_items;
        ctrl[1] = 0;
    }
    __syncthreads();
    for (int i = tid; i < n_items; i += kPlanThreads) {
        const Item it = unsorted[i];
        sorted[first_slot[it.cls] + atomicAdd(&cursor[it.cls], 1)] = it;
    }
}

// one thread per item: its cost class (0 = heaviest), and the class census
__global__ void rir_classify_kernel(const float* __restrict__ geom, int rir_len, double k_fs_c,
                                    Item* __restrict__ unsorted, int* __restrict__ ctrl) {
    // (the census is taken per work group in LDS first: one global atomic per class and group, not per item)
    __shared__ int census[kClasses];
    if (threadIdx.x < kClasses) census[threadIdx.x] = 0;
    __syncthreads();
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < ctrl[0]) {
        const Item it = unsorted[i];
        const int cls = item_class(geom + (size_t)it.rir * 10, rir_len, k_fs_c, it.n0, it.n1);
        unsorted[i].cls = cls;
        atomicAdd(&census[cls], 1);
    }
    __syncthreads();
    if (threadIdx.x < kClasses && census[threadIdx.x]) atomicAdd(&ctrl[2 + threadIdx.x], census[threadIdx.x]);
}

// Items move to their class's stretch of the sorted table, heaviest class first: persistent groups then take
// the heaviest items first and finish on the light ones, which evens out their finishing times.
// ctrl[2 + c] is the census of class c, ctrl[2 + kClasses + c] the cursor within its stretch.
__global__ void rir_sort_items_kernel(const Item* __restrict__ unsorted, Item* __restrict__ sorted, int* __restrict__ ctrl) {
    // (a work group numbers its items of a class in LDS and takes their places in the class's stretch with
    // one global atomic per class)
    __shared__ int first_slot[kClasses], mine[kClasses];
    if (threadIdx.x < kClasses) mine[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        int at = 0;
        for (int c = 0; c < kClasses; ++c) {
            first_slot[c] = at;
            at += ctrl[2 + c];
        }
    }
    __syncthreads();
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool have = i < ctrl[0];
    Item it;
    int rank = 0;
    if (have) {
        it = unsorted[i];
        rank = atomicAdd(&mine[it.cls], 1);
    }
    __syncthreads();
    if (threadIdx.x < kClasses && mine[threadIdx.x])
        first_slot[threadIdx.x] += atomicAdd(&ctrl[2 + kClasses + threadIdx.x], mine[threadIdx.x]);
    __syncthreads();
    if (have) sorted[first_slot[it.cls] + rank] = it;
}

// per-column record shared through LDS between the lane that built it and the lanes that walk its pieces
// (16 bytes: reflection counts stay below 2^16 for every room the interface accepts, and a batch of 64
// columns has at most 64 * 2 kAxisCap / kPiece pieces)
struct __align__(8) Column {
    double a;                    // dx*dx + dy*dy
    unsigned short kxy;          // reflections along x and y
    unsigned short pfx;          // the column's first piece within the wave's batch
    unsigned short start, len;   // range of the sorted z table that can fall inside the shell
};
static_assert(sizeof(Column) == 16, "column records are packed");

// One image along an axis, as stored in the sorted tables: key = squared distance to the microphone
// along that axis (reference operation order); aux = beta^reflections (z axis) or the reflection count
// (y axis).  Sixteen bytes: one LDS read per entry.
struct __align__(16) AxisImage {
    double key;
    double aux;
};

struct WalkCtx {
    double k_fs_c;
    double shift;        // 0.5 + guard - (n0 - 1): added to d fs/c, it gives slot = tap - n0 + 1 by truncation
    double guard2;       // estimates whose fraction (after the shift) is below this are redone exactly
    double beta;
    int n0m1;            // n0 - 1
    unsigned int n_slots;   // taps of the item + 2: slot 0 takes what belongs below the item, the last slot what
                            // belongs above it; neither is read
};

// the reference recipe, kept out of line so that the estimate's loop stays short
__device__ __attribute__((noinline)) int exact_tap(double d2, double k_fs_c) {
    const double d = __dsqrt_rn(d2);
    return (int)__dadd_rn(__dmul_rn(d, k_fs_c), 0.5);     // positive: truncation is floor
}

// Largest reflection count k whose amplitude beta^k / (4 pi d) can still add to a sum in the 2^-56 fixed
// point at distance d_min or beyond.  Increments are rounded to the nearest unit (or truncated, in the
// innermost item), so an amplitude below half a unit adds exactly zero; the cut is taken at 2^-57.5, a
// margin of a factor 1.41 under that, plus one count of slack, which covers the rounding of this estimate
// for every beta that the limit of 10^6 counts lets through.  "No limit" when beta is 0, >= 1
// (log2_beta == 0 encodes both) or d_min is tiny.
__device__ inline int reflection_cut(float log2_beta, float d_min) {
    if (!(log2_beta < 0.f) || !(d_min > 1e-3f)) return 1 << 20;
    // beta^k >= 4 pi d 2^-57.5  <=>  k <= (log2(4 pi d) - 57.5) / log2(beta)
    const float k = (__log2f(12.566371f * d_min) - 57.5f) / log2_beta;
    return k > 1.0e6f ? (1 << 20) : (int)k + 2;
}

// Slot (tap - n0 + 1) of an image at squared distance d2, and y ~ 1/sqrt(d2) (the hardware's
// double-precision estimate, good to 2^-24: enough for the amplitude) for its amplitude.
// One Newton step on the root leaves d fs/c good to ~1e-10 taps; shifted up by the guard, its fraction
// falls below 2 guard exactly when the true value may lie within the guard of a rounding boundary, and only
// then is the reference recipe evaluated.
// (in two parts, so that a caller with several images in hand can run their estimates side by side
// before any of the rare exact evaluations)
__device__ inline double tap_estimate(const WalkCtx& w, double d2, double& y) {
    y = __builtin_amdgcn_rsq(d2);
    const double s0 = __dmul_rn(d2, y);                    // sqrt(d2) to 2^-24
    const double res = fma(-s0, s0, d2);                   // exact residual
    const double s1 = fma(__dmul_rn(res, y), 0.5, s0);     // one Newton step: ~4e-15 relative
    return fma(s1, w.k_fs_c, w.shift);
}
__device__ inline int tap_settle(const WalkCtx& w, double d2, double t) {
    int slot = (int)t;
    if (__builtin_amdgcn_fract(t) < w.guard2) slot = exact_tap(d2, w.k_fs_c) - w.n0m1;
    return slot;
}
__device__ inline int tap_slot(const WalkCtx& w, double d2, double& y) {
    return tap_settle(w, d2, tap_estimate(w, d2, y));
}

// amp2 = amplitude * 2^56, rounded to an integer, goes to the tap's 64-bit integer sum.  Below 2^51 (every
// image farther than 2.55 m) adding 1.5 * 2^52 rounds the exact product to an integer in the sum's own
// mantissa, whose low 51 bits are then the increment; larger ones are rounded and split in two exact steps
// (amp2 < 2^64: images at least a third of a millimetre away).  Which of the two an image takes depends on
// its own amplitude only, so a response does not depend on how the batch was cut into items.
// FAR: every image of the item lies beyond 2.6 m, the test is not needed.
// CHECKED: the caller may pass slots outside the item (they are dropped); the table walk never does.
template <bool COUNT, bool FAR, bool CHECKED>
__device__ inline void deposit(const WalkCtx& w, int slot, double a, double y, unsigned long long* hist,
                               unsigned int* hist32) {
    if (CHECKED && (unsigned int)slot >= w.n_slots) return;
    if (COUNT) {
        atomicAdd(&hist32[slot], 1u);
        return;
    }
    unsigned int hi, lo;
    if (FAR || __dmul_rn(a, y) < 0x1p51) {
        const double m = fma(a, y, 0x1.8p52);
        hi = (unsigned int)__double2hiint(m) & 0x7ffffu;
        lo = (unsigned int)__double2loint(m);
    } else {
        const double amp2 = rint(__dmul_rn(a, y));
        hi = (unsigned int)__dmul_rn(amp2, 0x1p-32);
        lo = (unsigned int)fma(-(double)hi, 0x1p32, amp2);
    }
    atomicAdd(&hist[slot], ((unsigned long long)hi << 32) | lo);
}

// Every entry of a piece lies inside the item's shell up to the slack of the closed-form table positions
// (a relative 1e-9: a few 1e-5 taps), so its slot is one of 0 .. taps + 1 and needs no test.
template <bool COUNT, bool FAR>
__device__ inline void walk_piece_table(const WalkCtx& w, double a, double cxy, const AxisImage* z, int len,
                                        unsigned long long* hist, unsigned int* hist32) {
    // walked from the far end so that one register is both the address and the loop condition
    // (the sums are integers: the order does not matter)
    // (the LDS address itself is the loop variable, opaque to the compiler so that it is not split into
    // a counter plus an offset)
    typedef const AxisImage __attribute__((address_space(3))) * LdsImages;
    // kGroup images at a time, so that each lane has as many independent chains of arithmetic in flight; the
    // group of the next round is requested before the current one is worked on.  A piece whose length is
    // not a multiple of kGroup takes the entries above it as partners whose distance is made not-a-number:
    // every comparison on them fails and they land in slot 0, which is never read.  The last round requests
    // the kGroup entries below the piece, and a ragged piece reads up to kGroup - 1 entries above it: the
    // table has spare entries in front and behind.
    constexpr int kGroup = kWalkGroup;
    constexpr unsigned int kE = (unsigned int)sizeof(AxisImage);
    const unsigned int first = (unsigned int)(uintptr_t)(LdsImages)z;
    const int groups = (len + kGroup - 1) / kGroup;
    unsigned int cur = first + (unsigned int)((groups - 1) * kGroup) * kE;      // lowest entry of the top group
    auto entry_at = [](unsigned int lds_address) {
        const LdsImages p = (LdsImages)(uintptr_t)lds_address;
        AxisImage e;
        e.key = p->key;
        e.aux = p->aux;
        return e;
    };
    struct Group { AxisImage e[kGroup]; };
    auto load = [&](unsigned int at) {
        Group g;
#pragma unroll
        for (int i = 0; i < kGroup; ++i) g.e[i] = entry_at(at + (unsigned int)i * kE);
        return g;
    };
    auto step = [&](const Group& g) {
        double d2[kGroup], y[kGroup], t[kGroup];
        int slot[kGroup];
        bool redo = false;
#pragma unroll
        for (int i = 0; i < kGroup; ++i) {
            d2[i] = __dadd_rn(a, g.e[i].key);
            t[i] = tap_estimate(w, d2[i], y[i]);
            slot[i] = (int)t[i];
            redo |= __builtin_amdgcn_fract(t[i]) < w.guard2;
        }
        if (redo) {       // (one test for all, so that the estimates are complete before the branch)
#pragma unroll
            for (int i = 0; i < kGroup; ++i) slot[i] = tap_settle(w, d2[i], t[i]);
        }
#pragma unroll
        for (int i = 0; i < kGroup; ++i)
            deposit<COUNT, FAR, false>(w, slot[i], COUNT ? 0.0 : __dmul_rn(g.e[i].aux, cxy), y[i], hist, hist32);
    };
    Group g0 = load(cur), g1;
    {
        const int top = len - 1 - (groups - 1) * kGroup;       // index of the piece's last entry within the top group
        const double nan = __longlong_as_double(0x7ff8000000000000ll);
#pragma unroll
        for (int i = 1; i < kGroup; ++i) if (i > top) g0.e[i].key = nan;
    }
    for (;;) {
        const bool last0 = cur == first;
        cur -= (unsigned int)kGroup * kE;
        asm("" : "+v"(cur));
        g1 = load(cur);
        step(g0);
        if (last0) break;
        const bool last1 = cur == first;
        cur -= (unsigned int)kGroup * kE;
        asm("" : "+v"(cur));
        g0 = load(cur);
        step(g1);
        if (last1) break;
    }
}

// beta^k for reflection counts past the LDS table; out of line so that the double-precision pow does not
// weigh on the register allocation of the loops that call it once in a long while
__device__ __attribute__((noinline)) float beta_pow_slow(double beta, int k) { return (float)pow(beta, (double)k); }

// (out of line for the same reason: only rooms too flat or narrow for the tables come here)
template <bool COUNT>
__device__ __attribute__((noinline)) void walk_column_direct(const WalkCtx w, const Axis az, double a, double cxy, int nmz,
                                                             unsigned long long* hist, unsigned int* hist32) {
    for (int q = 0; q < 2; ++q)
        for (int n = -nmz; n <= nmz; ++n) {
            const double dz = axis_delta(az, q, n);
            const double d2 = __dadd_rn(a, __dmul_rn(dz, dz));
            double y;
            const int slot = tap_slot(w, d2, y);
            double bz = 0.0;
            if (!COUNT) bz = (double)beta_pow_slow(w.beta, iabs(n - q) + iabs(n));
            deposit<COUNT, false, true>(w, slot, __dmul_rn(bz, cxy), y, hist, hist32);
        }
}

// All images (1 - 2q) s + 2 n L - m, q in {0,1}, |n| <= nm, of one axis, written to `out` in order of
// squared distance.  For each q the signed distance grows with n, so the images with negative
// distance (walked towards smaller n) and those with non-negative distance are two sorted lists;
// an image's place in the merged order is its place in its own list plus, by binary search, the
// number of images of the other three lists that sort before it (ties go to the lower list).
// All threads of the group must call; aux(q, n) supplies the entry's second field.
template <class Aux>
__device__ inline void build_sorted_images(const Axis& ax, int nm, int* s_split, AxisImage* out, int tid, Aux aux) {
    const int per_q = 2 * nm + 1, n_all = 2 * per_q;
    if (tid < 2) s_split[tid] = per_q;
    __syncthreads();
    for (int i = tid; i < n_all; i += kThreads) {
        const int q = i >= per_q, n = i - q * per_q - nm;
        if (axis_delta(ax, q, n) >= 0.0 && (n == -nm || axis_delta(ax, q, n - 1) < 0.0)) s_split[q] = n + nm;
    }
    __syncthreads();
    auto key_at = [&](int l, int pos) {           // list l = 2 q + side, position pos in walking order
        const int sp = s_split[l >> 1];
        const double d = axis_delta(ax, l >> 1, ((l & 1) ? sp + pos : sp - 1 - pos) - nm);
        return __dmul_rn(d, d);
    };
    for (int i = tid; i < n_all; i += kThreads) {
        const int q = i >= per_q, t = i - q * per_q, sp = s_split[q];
        const int side = t >= sp, own = 2 * q + side;
        const double d = axis_delta(ax, q, t - nm);
        const double key = __dmul_rn(d, d);
        int rank = side ? t - sp : sp - 1 - t;
#pragma unroll
        for (int l = 0; l < 4; ++l) {
            if (l == own) continue;
            int lo = 0, hi = (l & 1) ? per_q - s_split[l >> 1] : s_split[l >> 1];
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                const double km = key_at(l, mid);
                if (km < key || (km == key && l < own)) lo = mid + 1; else hi = mid;
            }
            rank += lo;
        }
        AxisImage e;
        e.key = key;
        e.aux = aux(q, t - nm);
        out[rank] = e;
    }
    __syncthreads();
}

// Position in an axis's sorted table without searching it.  The table holds the images c_q + 2 n L,
// q in {0,1}, |n| <= nm, ordered by squared distance, so the number of entries within distance s of the
// microphone is the number of terms of the two arithmetic progressions that lie in [-s, s].
struct AxisCount {
    double k0, k1;       // -c_q / (2 L), c_q = (1 - 2q) src - mic
    double inv2l;        // 1 / (2 L)
    double nm;
};

__device__ inline AxisCount axis_count(const Axis& a, int nm) {
    const double inv2l = 1.0 / (2.0 * a.room);
    return AxisCount{uni(-(a.src - a.mic) * inv2l), uni(-(-a.src - a.mic) * inv2l), uni(inv2l), uni((double)nm)};
}

// terms n of c_q + 2 n L, |n| <= nm, within [-s, s]: (-s - c_q) / 2L <= n <= (s - c_q) / 2L
__device__ inline int count_within(const AxisCount& a, double s) {
    int total = 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const double k = q ? a.k1 : a.k0;
        const double hi = fmin(floor(fma(s, a.inv2l, k)), a.nm);
        const double lo = fmax(ceil(fma(-s, a.inv2l, k)), -a.nm);
        total += max((int)hi - (int)lo + 1, 0);
    }
    return total;
}

// sqrt(b) to a few 1e-15 relative for b > 0 (the hardware's estimate of 1/sqrt and one Newton step), 0 for b <= 0
__device__ inline double quick_sqrt(double b) {
    if (!(b > 1e-30)) return 0.0;
    const double y = __builtin_amdgcn_rsq(b);
    const double s0 = __dmul_rn(b, y);
    return fma(__dmul_rn(fma(-s0, s0, b), y), 0.5, s0);
}

// The table's keys and these counts round differently, so a bound is widened (or narrowed) by far more
// than either rounding error before counting.  An entry that close to a bound is then visited although
// it may lie outside; every visited image is tested against the item's taps anyway.
// number of entries with key <= bound, or a few more
__device__ inline int count_not_above(const AxisCount& a, int n, double bound) {
    if (!(bound >= 0.0)) return 0;
    const double s = quick_sqrt(bound);
    return min(count_within(a, s * (1.0 + 1e-9) + 1e-9), n);
}
// number of entries with key < bound, or a few fewer
__device__ inline int count_below(const AxisCount& a, double bound) {
    const double s = quick_sqrt(bound) * (1.0 - 1e-9) - 1e-9;
    return s > 0.0 ? count_within(a, s) : 0;
}

// VISITS: a measuring instantiation that also adds the number of images it walked to *visits.
template <bool COUNT, bool VISITS = false>
__global__ __launch_bounds__(kThreads, 4) void rir_image_kernel(
    const float* __restrict__ geom, int rir_len, double k_fs_c, const Item* __restrict__ items,
    int* __restrict__ ctrl, float* __restrict__ rir_out,
    int32_t* __restrict__ cnt_out, unsigned long long* __restrict__ visits = nullptr) {
    __shared__ unsigned long long hist[(COUNT ? kMaxTaps / 2 : kMaxTaps) + 2];     // first and last slot are never read
    __shared__ float bpow[COUNT ? 1 : kPow];
    __shared__ AxisImage ztab_store[2 * kAxisCap + 2 * kWalkGroup - 1];
    AxisImage* const ztab = ztab_store + kWalkGroup;       // z images sorted by dz*dz (spare entries in front and behind)
    __shared__ AxisImage ytab[2 * kAxisCap];       // y images sorted by dy*dy
    __shared__ int row_pfx[2 * kAxisCap];          // per x image: inclusive prefix of live column counts
    __shared__ int s_split[2];
    __shared__ Column cols[kWaves][64];
    __shared__ __align__(8) unsigned int piece_starts[kWaves][kStartWords];
    __shared__ int s_item;
    unsigned int* hist32 = reinterpret_cast<unsigned int*>(hist);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_items = ctrl[0];
    unsigned long long walked = 0;

    for (;;) {
        if (tid == 0) s_item = atomicAdd(&ctrl[1], 1);
        __syncthreads();
        const int it = uni(s_item);
        if (it >= n_items) break;
        const Item item = items[it];
        const int n0 = item.n0, n1 = item.n1, n_taps = n1 - n0;
        const float* g = geom + (size_t)item.rir * 10;

        if (COUNT) {
            for (int i = tid; i <= n_taps + 1; i += kThreads) hist32[i] = 0u;
        } else {
            for (int i = tid; i <= n_taps + 1; i += kThreads) hist[i] = 0ull;
            // beta^k by squaring (k < 1024: ten steps, a few units in the last place of the double, far inside
            // the float it is kept as; the library pow is some ten times the instructions)
            for (int i = tid; i < kPow; i += kThreads) {
                double b = (double)g[9], acc = 1.0;
#pragma unroll
                for (int bit = 0; bit < 10; ++bit) {
                    if ((i >> bit) & 1) acc *= b;
                    b *= b;
                }
                bpow[i] = (float)acc;
            }
        }
        __syncthreads();

        if (room_ok(g)) {
            const Axis ax{uni((double)g[0]), uni((double)g[3]), uni((double)g[6])};
            const Axis ay{uni((double)g[1]), uni((double)g[4]), uni((double)g[7])};
            const Axis az{uni((double)g[2]), uni((double)g[5]), uni((double)g[8])};
            const double beta = uni((double)g[9]);
            // every image of this item lies in r_in <= d < r_out (half a tap of slack on either side)
            const double r_out = uni((double)n1 / k_fs_c);
            const double r_in = n0 > 0 ? uni((double)(n0 - 1) / k_fs_c) : 0.0;
            const double r_out2 = uni(r_out * r_out), r_in2 = uni(r_in * r_in);
            // An image reflected k times adds beta^k / (4 pi d) * 2^56, rounded to an integer, to its
            // tap; once beta^k < 2 pi d 2^-56 that is exactly zero, so such images are never visited.
            // log2_beta < 0 enables the cut (amplitude sums only; tap counts visit every image).
            const float log2_beta = (!COUNT && g[9] > 0.f && g[9] < 1.f) ? uni(__log2f(g[9])) : 0.f;
            const int k_cut_item = uni(reflection_cut(log2_beta, (float)r_in));
            int nmx = uni((int)ceil(r_out / (2.0 * ax.room)) + 1);
            int nmy = uni((int)ceil(r_out / (2.0 * ay.room)) + 1);
            const int nmz = uni((int)ceil(r_out / (2.0 * az.room)) + 1);
            nmx = min(nmx, k_cut_item / 2 + 1);          // |n - q| + |n| >= 2 |n| - 1
            nmy = min(nmy, k_cut_item / 2 + 1);
            const int nix = 2 * (2 * nmx + 1), niy = 2 * (2 * nmy + 1), niz = 2 * (2 * nmz + 1);
            const AxisCount cy = axis_count(ay, nmy), cz = axis_count(az, nmz);
            Column* wc = cols[wave];
            WalkCtx wctx;
            wctx.k_fs_c = k_fs_c;
            const double guard = 1e-12 * (double)(n1 + 1) + 1e-13;
            wctx.shift = (0.5 + guard) - (double)(n0 - 1);      // (a vector register: the index step's other factor is scalar)
            wctx.guard2 = uni(2.0 * guard);
            wctx.n0m1 = n0 - 1;
            wctx.n_slots = (unsigned int)n_taps + 2u;
            // beyond 2.6 m every amplitude is below 2^-5 (see deposit)
            const bool far_item = r_in >= 2.6;
            wctx.beta = beta;
            const float y0_max = uni(fmaxf(fabsf((float)(ay.src - ay.mic)), fabsf((float)(ay.src + ay.mic))));
            const float z0_max = uni(fmaxf(fabsf((float)(az.src - az.mic)), fabsf((float)(az.src + az.mic))));
            const float lyf = uni((float)ay.room), lzf = uni((float)az.room);
            // every image with at most k reflections along an axis lies within max|c_q| + (k + 1) L of the
            // microphone on that axis; squared, with a little slack, this bounds the table range to visit
            auto reach2 = [](float c_max, float room, int k) {
                const float r = c_max + (float)(k + 1) * room;
                return (double)(r * r * 1.0001f + 1e-3f);
            };

            // fast path: the y and z images fit the LDS tables and so do the x rows
            const bool fast = nix <= 2 * kAxisCap && niy <= 2 * kAxisCap && niz <= 2 * kAxisCap;
            int n_cand;
            if (fast) {
                build_sorted_images(az, nmz, s_split, ztab, tid, [&](int q, int n) {
                    if (COUNT) return 0.0;
                    const int k = iabs(n - q) + iabs(n);
                    return (double)(k < kPow ? bpow[k] : beta_pow_slow(beta, k));
                });
                build_sorted_images(ay, nmy, s_split, ytab, tid, [&](int q, int n) { return (double)(iabs(n - q) + iabs(n)); });
                // live columns of x image ix: the y images with dy^2 <= r_out^2 - dx^2 that the reflection
                // cut can still reach -- a prefix of the sorted y table
                for (int ix = tid; ix < nix; ix += kThreads) {
                    const int qx = ix & 1, nx = (ix >> 1) - nmx;
                    const double dx = axis_delta(ax, qx, nx);
                    double bound = r_out2 - __dmul_rn(dx, dx);
                    const int ky_max = k_cut_item - (iabs(nx - qx) + iabs(nx));
                    if (ky_max < (1 << 18)) bound = fmin(bound, reach2(y0_max, lyf, ky_max));
                    row_pfx[ix] = (bound >= 0.0 && ky_max >= 0) ? count_not_above(cy, niy, bound) : 0;
                }
                __syncthreads();
                if (wave == 0) {                              // inclusive scan over the rows, 64 at a time
                    int carry = 0;
                    for (int base = 0; base < nix; base += 64) {
                        const int i = base + lane;
                        const int v = wave_inclusive_scan(i < nix ? row_pfx[i] : 0, lane) + carry;
                        if (i < nix) row_pfx[i] = v;
                        carry = __shfl(v, 63, 64);
                    }
                }
                __syncthreads();
                n_cand = row_pfx[nix - 1];
            } else {
                n_cand = nix * niy;
            }
            const int n_batch = (n_cand + 63) / 64;

            int row_lo = 0;          // row of the batch's first candidate: it only moves up from batch to batch
            for (int batch = wave; batch < n_batch; batch += kWaves) {
                // ---- each lane describes one candidate column ----
                const int cand = batch * 64 + lane;
                if (fast)
                    while (row_pfx[row_lo] <= batch * 64) ++row_lo;       // (the same in every lane; batch * 64 < n_cand)
                Column col;
                col.a = 0.0; col.kxy = 0; col.start = 0; col.len = 0;
                int pieces = 0;
                if (cand < n_cand) {
                    if (fast) {
                        // smallest row with row_pfx > cand: a short walk from the row of the batch's first
                        // column, since 64 consecutive columns span few rows
                        int lo = row_lo;
                        while (row_pfx[lo] <= cand) ++lo;
                        const int ix = lo, qx = ix & 1, nx = (ix >> 1) - nmx;
                        const AxisImage ye = ytab[cand - (ix ? row_pfx[ix - 1] : 0)];
                        const double dx = axis_delta(ax, qx, nx);
                        col.a = __dadd_rn(__dmul_rn(dx, dx), ye.key);
                        col.kxy = (unsigned short)(iabs(nx - qx) + iabs(nx) + (int)ye.aux);
                    } else {
                        const int ix = cand / niy, iy = cand - ix * niy;
                        const int qx = ix & 1, nx = (ix >> 1) - nmx;
                        const int qy = iy & 1, ny = (iy >> 1) - nmy;
                        const double dx = axis_delta(ax, qx, nx);
                        const double dy = axis_delta(ay, qy, ny);
                        col.a = __dadd_rn(__dmul_rn(dx, dx), __dmul_rn(dy, dy));
                        col.kxy = (unsigned short)(iabs(nx - qx) + iabs(nx) + iabs(ny - qy) + iabs(ny));
                    }
                    // reflections left for the z axis before this column's images vanish
                    // (beyond the first shell the shell's own inner radius bounds the distance well enough)
                    const int kz_max = (n0 > 0 ? k_cut_item : reflection_cut(log2_beta, sqrtf((float)col.a))) - (int)col.kxy;
                    if (col.a < r_out2 && kz_max >= 0) {
                        if (fast) {
                            // images with r_in^2 - a <= dz^2 <= r_out^2 - a within reach of the reflection cut:
                            // one contiguous range of the sorted z table (the few images past the cut that it
                            // keeps add exactly zero)
                            double hi2 = r_out2 - col.a;
                            if (kz_max < (1 << 18)) hi2 = fmin(hi2, reach2(z0_max, lzf, kz_max));
                            const double lo2 = r_in2 - col.a;
                            const int first = lo2 > 0.0 ? count_below(cz, lo2) : 0;     // entries with dz2 < lo2
                            const int last = count_not_above(cz, niz, hi2);
                            if (last > first) {
                                col.start = (unsigned short)first;
                                col.len = (unsigned short)(last - first);
                                pieces = (last - first + kPiece - 1) / kPiece;
                            }
                        } else {
                            pieces = 1;                        // one lane walks every z image of the column
                        }
                    }
                }
                const int pfx = wave_inclusive_scan(pieces, lane);
                const int my_first = pfx - pieces;             // this column's first piece
                col.pfx = (unsigned short)my_first;
                const int n_pieces = __shfl(pfx, 63, 64);
                // columns with pieces, packed in order
                const unsigned long long live = __ballot(pieces > 0);
                if (pieces > 0)
                    wc[__builtin_amdgcn_mbcnt_hi((unsigned int)(live >> 32), __builtin_amdgcn_mbcnt_lo((unsigned int)live, 0u))] = col;

                // ---- pieces are dealt to lanes ----
                // Piece p belongs to the last column that starts at or before it.  Every column sets the bit of
                // its first piece in a bit map; a piece's column is then a count of bits, not a search.
                unsigned int* starts = piece_starts[wave];
                constexpr int kChunk = 32 * kStartWords;
                for (int chunk = 0; chunk < n_pieces; chunk += kChunk) {
                    if (lane < kStartWords) starts[lane] = 0u;
                    wave_sync_lds();
                    if (pieces > 0 && my_first >= chunk && my_first < chunk + kChunk)
                        atomicOr(&starts[(my_first - chunk) >> 5], 1u << (my_first & 31));
                    int before = __popcll(__ballot(pieces > 0 && my_first < chunk));     // columns begun in earlier chunks
                    wave_sync_lds();
                    const int chunk_end = min(n_pieces, chunk + kChunk);
                    for (int p0 = chunk; p0 < chunk_end; p0 += 64) {
                        const uint2 m = *reinterpret_cast<const uint2*>(&starts[(p0 - chunk) >> 5]);   // pieces p0 .. p0 + 63
                        // starts in [p0, p0 + lane]: bit 0, and the bits below this lane of the map moved down by one
                        const unsigned int s_lo = (m.x >> 1) | (m.y << 31), s_hi = m.y >> 1;
                        const int upto = (int)(m.x & 1u) + (int)__builtin_amdgcn_mbcnt_hi(s_hi, __builtin_amdgcn_mbcnt_lo(s_lo, 0u));
                        const int p = p0 + lane;
                        if (p < chunk_end) {
                            const Column c = wc[before + upto - 1];
                            const int local = p - (int)c.pfx;
                            double cxy = 0.0;      // beta^kxy / (4 pi) * 2^56
                            if (!COUNT)
                                cxy = (double)(c.kxy < kPow ? bpow[c.kxy] : beta_pow_slow(beta, c.kxy)) * (0.07957747154594767 * 0x1p56);
                            if (fast) {
                                const int first = (int)c.start + local * kPiece;
                                const int len = min(kPiece, (int)c.len - local * kPiece);
                                if (far_item) walk_piece_table<COUNT, true>(wctx, c.a, cxy, ztab + first, len, hist, hist32);
                                else walk_piece_table<COUNT, false>(wctx, c.a, cxy, ztab + first, len, hist, hist32);
                                if (VISITS) walked += (unsigned long long)len;
                            } else {
                                walk_column_direct<COUNT>(wctx, az, c.a, cxy, nmz, hist, hist32);
                                if (VISITS) walked += (unsigned long long)niz;
                            }
                        }
                        before += __popc(m.x) + __popc(m.y);
                    }
                    wave_sync_lds();
                }
            }
        }
        __syncthreads();

        if (COUNT) {
            int32_t* out = cnt_out + (size_t)item.rir * rir_len + n0;
            for (int i = tid; i < n_taps; i += kThreads) out[i] = (int32_t)hist32[i + 1];
        } else {
            float* out = rir_out + (size_t)item.rir * rir_len + n0;
            for (int i = tid; i < n_taps; i += kThreads) {
                const unsigned long long v = hist[i + 1];
                const double d = (double)(unsigned int)(v >> 32) * 4294967296.0 + (double)(unsigned int)v;
                out[i] = (float)(d * 1.3877787807814457e-17);       // 2^-56
            }
        }
        __syncthreads();
    }
    if (VISITS) {
        for (int off = 32; off > 0; off >>= 1) walked += __shfl_down(walked, off, 64);
        if (lane == 0 && walked) atomicAdd(visits, walked);
    }
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

__global__ void fill2_u32_kernel(uint32_t* p, uint32_t v, int64_t n, uint32_t* q, uint32_t w, int64_t m) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n + m; i += stride) {
        if (i < n) p[i] = v; else q[i - n] = w;
    }
}

}  // namespace

hipError_t launch_fill_u32(hipStream_t s, void* p, uint32_t v, int64_t n) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    fill_u32_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<uint32_t*>(p), v, n);
    return hipGetLastError();
}

hipError_t launch_fill2_u32(hipStream_t s, void* p, uint32_t v, int64_t n, void* q, uint32_t w, int64_t m) {
    if (n + m <= 0) return hipSuccess;
    int64_t blocks = (n + m + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    fill2_u32_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<uint32_t*>(p), v, n,
                                                                  static_cast<uint32_t*>(q), w, m);
    return hipGetLastError();
}

// One geometry row per (response, microphone): the row of the response with its microphone columns replaced.
__global__ void rir_mic_rows_kernel(int n_rows, int n_mic, const float* __restrict__ geom, const float* __restrict__ mics,
                                    float* __restrict__ rows) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;       // one thread per output value
    if (i >= n_rows * 10) return;
    const int row = i / 10, col = i - row * 10;
    rows[i] = (col >= 6 && col < 9) ? mics[(size_t)row * 3 + (col - 6)] : geom[(size_t)(row / n_mic) * 10 + col];
}

hipError_t launch_rir_mic_rows(hipStream_t s, int n_rir, int n_mic, const float* geom, const float* mics, float* rows) {
    const int n_rows = n_rir * n_mic;
    if (n_rows <= 0) return hipSuccess;
    rir_mic_rows_kernel<<<dim3((unsigned)((n_rows * 10 + 255) / 256)), dim3(256), 0, s>>>(n_rows, n_mic, geom, mics, rows);
    return hipGetLastError();
}

int rir_items_per_response(int rir_len) { return kMaxShells + rir_len / kMaxTaps + 2; }
size_t rir_item_bytes() { return sizeof(Item); }

int rir_ctrl_ints() { return kCtrlInts; }

hipError_t launch_rir_plan(hipStream_t s, int n_groups, int n_rir, const float* geom, int rir_len, double fs_over_c,
                           void* items, int* ctrl) {
    if (n_rir <= 0) return hipSuccess;
    // `items` holds the sorted table followed by the unsorted one
    const int per_rir = rir_items_per_response(rir_len);
    Item* sorted = static_cast<Item*>(items);
    Item* unsorted = sorted + (size_t)n_rir * per_rir;
    if (n_rir <= kPlanThreads) {                             // one launch instead of five
        rir_plan_all_kernel<<<dim3(1), dim3(kPlanThreads), 0, s>>>(n_rir, geom, rir_len, fs_over_c, sorted, unsorted,
                                                                    per_rir, ctrl, n_groups);
        return hipGetLastError();
    }
    hipError_t e = launch_fill_u32(s, ctrl, 0u, kCtrlInts);
    if (e != hipSuccess) return e;
    rir_work_kernel<<<dim3((n_rir + 127) / 128), dim3(128), 0, s>>>(n_rir, geom, rir_len, fs_over_c, ctrl);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    rir_plan_kernel<<<dim3((n_rir + 127) / 128), dim3(128), 0, s>>>(n_rir, geom, rir_len, fs_over_c, unsorted, per_rir, ctrl,
                                                                    n_groups);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t max_items = (size_t)n_rir * per_rir;
    const int item_groups = (int)((max_items + 255) / 256);
    rir_classify_kernel<<<dim3((unsigned)item_groups), dim3(256), 0, s>>>(geom, rir_len, fs_over_c, unsorted, ctrl);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    rir_sort_items_kernel<<<dim3((unsigned)item_groups), dim3(256), 0, s>>>(unsorted, sorted, ctrl);
    return hipGetLastError();
}

hipError_t launch_rir(hipStream_t s, int n_groups, int n_rir, const float* geom, int rir_len, double fs_over_c,
                      const void* items, int* ctrl, float* rir_out, int32_t* cnt_out,
                      bool restart, unsigned long long* visits) {
    if (n_rir <= 0) return hipSuccess;
    hipError_t e = hipSuccess;
    if (restart) {                                           // another pass over the same plan
        e = launch_fill_u32(s, ctrl + 1, 0u, 1);
        if (e != hipSuccess) return e;
    }
    const Item* it = static_cast<const Item*>(items);
    if (rir_out && visits)
        rir_image_kernel<false, true><<<dim3((unsigned)n_groups), dim3(kThreads), 0, s>>>(
            geom, rir_len, fs_over_c, it, ctrl, rir_out, nullptr, visits);
    else if (rir_out)
        rir_image_kernel<false><<<dim3((unsigned)n_groups), dim3(kThreads), 0, s>>>(
            geom, rir_len, fs_over_c, it, ctrl, rir_out, nullptr);
    else
        rir_image_kernel<true><<<dim3((unsigned)n_groups), dim3(kThreads), 0, s>>>(
            geom, rir_len, fs_over_c, it, ctrl, nullptr, cnt_out);
    return hipGetLastError();
}

}  // namespace aug
