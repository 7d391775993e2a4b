// Image-method room impulse responses (the acoustic simulator of Sec. 2.3 computes
// them on the fly for every training example).
//
// h[n] = sum over image sources with floor(d fs/c + 0.5) == n of beta^k / (4 pi d),
// d = distance image -> microphone, k = number of wall reflections of that image.
// Along one axis the images of a source at s between walls at 0 and L are
// (1 - 2q) s + 2 n L, q in {0,1}, n integer, reflected |n - q| + |n| times.
//
// The tap index is integer work decided by floating point, so it is evaluated in
// fp64 with a fixed operation order and no contraction:
//     d2 = (dx*dx + dy*dy) + dz*dz;  idx = floor(sqrt(d2) * (fs/c) + 0.5)
// Amplitudes are fp32 and accumulate through LDS float atomics (order free).
//
// Work split: one response is cut over `n_split` work groups by striding the
// (x image, y image) columns; each thread walks the z images of its columns that can
// fall inside the sphere of radius rir_len * c / fs.  Every group keeps a private
// tap histogram in LDS and adds it to the zero-initialised output at the end.

#include "aug_internal.h"

namespace aug {
namespace {

constexpr int kRirThreads = 1024;
constexpr int kPowTable = 4096;          // beta^k table entries held in LDS
constexpr int kMaxSplit = 64;            // most work groups one response is cut into
constexpr float kImagesPerGroup = 262144.0f;

#pragma clang fp contract(off)

struct AxisGeom {
    double room, src, mic;
    int n_max;       // images use n in [-n_max, n_max]
    int n_img;       // 2 * (2 n_max + 1)
};

__device__ inline AxisGeom make_axis(float room, float src, float mic, double radius) {
    AxisGeom a;
    a.room = (double)room;
    a.src = (double)src;
    a.mic = (double)mic;
    a.n_max = (int)ceil(radius / (2.0 * a.room)) + 1;
    a.n_img = 2 * (2 * a.n_max + 1);
    return a;
}

// image index i -> (q, n): q = i & 1, n = (i >> 1) - n_max
__device__ inline double axis_delta(const AxisGeom& a, int q, int n) {
    const double sgn = q ? -1.0 : 1.0;
    const double coord = __dadd_rn(__dmul_rn(sgn, a.src), __dmul_rn(__dmul_rn(2.0, (double)n), a.room));
    return __dsub_rn(coord, a.mic);
}

__device__ inline int iabs(int v) { return v < 0 ? -v : v; }

template <bool COUNT>
__global__ __launch_bounds__(kRirThreads) void rir_image_kernel(
    const float* __restrict__ geom, int rir_len, double k_fs_c, float* __restrict__ rir_out,
    int32_t* __restrict__ cnt_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* hist_f = reinterpret_cast<float*>(smem);
    int* hist_i = reinterpret_cast<int*>(smem);
    float* bpow = reinterpret_cast<float*>(smem + sizeof(float) * (size_t)rir_len);

    const int r = blockIdx.x / kMaxSplit;
    const int part = blockIdx.x % kMaxSplit;
    const float* g = geom + (size_t)r * 10;

    // Images beyond this distance cannot round to a tap below rir_len.
    const double radius = (double)rir_len / k_fs_c;
    // a degenerate room (a side under 10 cm, or not a number) has no images: the output stays zero
    if (!(g[0] >= 0.1f) || !(g[1] >= 0.1f) || !(g[2] >= 0.1f) || !(g[0] * g[1] * g[2] < 1e30f)) return;
    const float volume = g[0] * g[1] * g[2];
    const float est_images = 4.18879f * (float)(radius * radius * radius) / volume;
    int n_split = (int)ceilf(est_images / kImagesPerGroup);
    n_split = n_split < 1 ? 1 : (n_split > kMaxSplit ? kMaxSplit : n_split);
    if (part >= n_split) return;

    const AxisGeom ax = make_axis(g[0], g[3], g[6], radius);
    const AxisGeom ay = make_axis(g[1], g[4], g[7], radius);
    const AxisGeom az = make_axis(g[2], g[5], g[8], radius);
    const double beta = (double)g[9];

    for (int i = threadIdx.x; i < rir_len; i += kRirThreads) {
        if (COUNT) hist_i[i] = 0; else hist_f[i] = 0.0f;
    }
    if (!COUNT) {
        for (int i = threadIdx.x; i < kPowTable; i += kRirThreads)
            bpow[i] = (float)pow(beta, (double)i);
    }
    __syncthreads();

    const double r2_cut = radius * radius * (1.0 + 1e-9) + 1e-9;
    const double two_lz = 2.0 * az.room;
    const double inv_two_lz = 1.0 / two_lz;
    const float inv_4pi = 0.07957747154594767f;

    const int64_t n_col = (int64_t)ax.n_img * ay.n_img;
    for (int64_t col = (int64_t)part * kRirThreads + threadIdx.x; col < n_col;
         col += (int64_t)n_split * kRirThreads) {
        const int ix = (int)(col / ay.n_img), iy = (int)(col % ay.n_img);
        const int qx = ix & 1, nx = (ix >> 1) - ax.n_max;
        const int qy = iy & 1, ny = (iy >> 1) - ay.n_max;
        const double dx = axis_delta(ax, qx, nx);
        const double dy = axis_delta(ay, qy, ny);
        const double a = __dadd_rn(__dmul_rn(dx, dx), __dmul_rn(dy, dy));
        if (a >= r2_cut) continue;
        const int kxy = iabs(nx - qx) + iabs(nx) + iabs(ny - qy) + iabs(ny);
        const double z_reach = sqrt(r2_cut - a);
#pragma unroll
        for (int qz = 0; qz < 2; ++qz) {
            // images with |dz| <= z_reach, padded by one on either side; the exact
            // idx < rir_len test below decides.
            const double z0 = __dsub_rn(__dmul_rn(qz ? -1.0 : 1.0, az.src), az.mic);
            int n_lo = (int)floor((-z_reach - z0) * inv_two_lz) - 1;
            int n_hi = (int)ceil((z_reach - z0) * inv_two_lz) + 1;
            n_lo = n_lo < -az.n_max ? -az.n_max : n_lo;
            n_hi = n_hi > az.n_max ? az.n_max : n_hi;
            for (int n = n_lo; n <= n_hi; ++n) {
                const double dz = axis_delta(az, qz, n);
                const double d2 = __dadd_rn(a, __dmul_rn(dz, dz));
                const double d = __dsqrt_rn(d2);
                const double t = __dadd_rn(__dmul_rn(d, k_fs_c), 0.5);
                if (!(t < (double)rir_len)) continue;
                const int idx = (int)t;            // t >= 0.5 > 0: truncation is floor
                if (COUNT) {
                    atomicAdd(&hist_i[idx], 1);
                } else {
                    const int k = kxy + iabs(n - qz) + iabs(n);
                    const float b = k < kPowTable ? bpow[k] : (float)pow(beta, (double)k);
                    atomicAdd(&hist_f[idx], b * inv_4pi / (float)d);
                }
            }
        }
    }
    __syncthreads();

    if (COUNT) {
        int32_t* out = cnt_out + (size_t)r * rir_len;
        for (int i = threadIdx.x; i < rir_len; i += kRirThreads) {
            const int v = hist_i[i];
            if (n_split == 1) out[i] = v; else if (v) atomicAdd(&out[i], v);
        }
    } else {
        float* out = rir_out + (size_t)r * rir_len;
        for (int i = threadIdx.x; i < rir_len; i += kRirThreads) {
            const float v = hist_f[i];
            if (n_split == 1) out[i] = v; else if (v != 0.0f) atomicAdd(&out[i], v);
        }
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

hipError_t launch_rir(hipStream_t s, int n_rir, const float* geom, int rir_len, double fs_over_c,
                      float* rir_out, int32_t* cnt_out) {
    if (n_rir <= 0) return hipSuccess;
    hipError_t e = hipSuccess;
    const size_t lds_f = sizeof(float) * (size_t)rir_len + sizeof(float) * kPowTable;
    const size_t lds_i = sizeof(int) * (size_t)rir_len;
    static bool attr_set = false;
    if (!attr_set) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rir_image_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rir_image_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((unsigned)n_rir * kMaxSplit), block(kRirThreads);
    // Outputs must be zero on entry: a response cut over several groups is accumulated with atomics.
    if (rir_out) {
        rir_image_kernel<false><<<grid, block, lds_f, s>>>(geom, rir_len, fs_over_c, rir_out, nullptr);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (cnt_out) {
        rir_image_kernel<true><<<grid, block, lds_i, s>>>(geom, rir_len, fs_over_c, nullptr, cnt_out);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace aug
