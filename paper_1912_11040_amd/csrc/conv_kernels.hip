// Reverberation and SNR mixing (acoustic simulator, Sec. 2.3).
//
// y_j[n] = sum_{k < L} h_j[k] x_j[n-k] is evaluated by uniformly partitioned
// overlap-save: the response is cut into partitions of P taps, each transformed once
// (2P-point real FFT); an output block of P samples is the inverse transform of
// sum_p X_{b-p} H_p, X_w the transform of input samples [(w-1)P, (w+1)P).
// A 2P-point real transform is run as a P-point complex FFT of the even/odd packed
// sequence, entirely in LDS, split as 16 x P/16: the radix-16 column step reads its inputs
// straight from HBM (and, inverse, writes the block straight back); the 16 row transforms
// run one per wavefront without work-group barriers.
//
// Work groups are persistent and walk along the reverberated signals block after block (see
// convolve_kernel); each block's energy is added to E[u][j] (fp64 atomics).  A response of two partitions
// costs one forward and one inverse transform per block as well: the previous window's spectrum stays in
// registers.  A small kernel forms the gains g_j = sqrt(E_0 / (E_j 10^(snr_j/10))) (zero where an energy is
// zero); the mixture y_0 + sum_j g_j y_j is written by mix_kernel when the caller wants it, and formed by
// the front end on the fly otherwise.

#include "aug_internal.h"
#include "fft_lds.h"

namespace aug {
namespace {

constexpr int conv_threads(int n) { return n / 16; }

__host__ __device__ constexpr int twiddle_count(int n) { return n + n / 2 + 1 + n / 32; }

__global__ void twiddle_kernel(int n, float2* tw) {
    // tw[t] = exp(-2 pi i t / n), t < n;  tw[n + k] = exp(-i pi k / n), k <= n/2;
    // tw[n + n/2 + 1 + j] = exp(-i pi 16 j / n), j < n/32
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= twiddle_count(n)) return;
    double s, c;
    if (i < n) sincospi(-2.0 * (double)i / (double)n, &s, &c);
    else if (i < n + n / 2 + 1) sincospi(-(double)(i - n) / (double)n, &s, &c);
    else sincospi(-16.0 * (double)(i - n - n / 2 - 1) / (double)n, &s, &c);
    tw[i] = make_float2((float)c, (float)s);
}

// Even/odd split of the packed transform: from A = Z[k] and B = conj(Z[N-k]) give
// W[k] and conj(W[N-k]) of the 2N-point real transform; w = exp(-i pi k / N).
__device__ inline void unpack_pair(float2 A, float2 B, float2 w, float2& Wk, float2& WNk_conj) {
    const float2 E = make_float2(0.5f * (A.x + B.x), 0.5f * (A.y + B.y));
    const float2 d = csub(A, B);
    const float2 O = make_float2(0.5f * d.y, -0.5f * d.x);     // -(i/2)(A - B)
    const float2 wO = cmul(w, O);
    Wk = cadd(E, wO);
    WNk_conj = csub(E, wO);
}

// Bins are visited as k = k1 + 16 k2 (row k1, column k2 of the split transform), k < N/2, each with
// its partner N - k.  Thread tid owns column k2 = tid mod M/2 of rows k1 = 8 (tid div M/2) + i.
template <int N>
struct PairIndex {
    static constexpr int M = N / 16;
    int k, pos, pos_partner, h_partner;     // LDS/spectrum position of k and of N-k (spectrum: H[N] sits at N)
    __device__ inline PairIndex(int k1, int k2) {
        k = k1 + 16 * k2;
        pos = k1 * M + k2;
        pos_partner = k1 ? (16 - k1) * M + (M - 1 - k2) : ((M - k2) & (M - 1));
        h_partner = k ? pos_partner : N;
    }
};

template <int N> __device__ inline float2 pair_twiddle(const float2* __restrict__ tw, int k1, int k2) {
    return cmul(tw[N + k1], tw[N + N / 2 + 1 + k2]);           // exp(-i pi (k1 + 16 k2) / N)
}

// Spectra of the response partitions, stored in the split order (k at fft_split_pos(k), k = N last)
// and scaled by 1/(4N): 1/N for the unnormalised inverse, 1/4 for the halves that multiply_pair leaves out.
// Work groups are persistent: each takes every gridDim.x-th partition and requests the taps of its next one
// before the row transforms of the current one, whose twiddles come from a table in LDS (no global load of
// theirs then stands between the requested taps and the arithmetic).
template <int N>
__device__ inline int load_taps(float2 (&v)[8], const float* __restrict__ h, int rir_len, int p, int tid) {
    constexpr int M = N / 16;
    int first = 0x7fffffff;                          // index of this thread's first non-zero tap
#pragma unroll
    for (int n1 = 7; n1 >= 0; --n1) {                // taps of this partition: [pN, (p+1)N), then N zeros
        const int t = p * N + 2 * (tid + M * n1);
        const float a = t < rir_len ? h[t] : 0.f, b = t + 1 < rir_len ? h[t + 1] : 0.f;
        v[n1] = make_float2(a, b);
        if (b != 0.f) first = t + 1;
        if (a != 0.f) first = t;
    }
    return first;
}

template <int N, int T>
__global__ __launch_bounds__(T) void rir_spectrum_kernel(
    const float* __restrict__ rir, int rir_len, int n_part, int n_work, const float2* __restrict__ tw,
    float2* __restrict__ spec, int* __restrict__ first_tap) {
    extern __shared__ float2 buf[];
    constexpr int M = N / 16;
    float2* const row_tw = buf + lds_padded_size(N);
    RowTwiddles<M>::template fill<16>(row_tw, tw, threadIdx.x, T);
    const int tid0 = threadIdx.x;
    int work = blockIdx.x;
    if (work >= n_work) return;
    float2 taps[8];
    int first = load_taps<N>(taps, rir + (size_t)(work / n_part) * rir_len, rir_len, work % n_part, tid0);
    __syncthreads();                                 // the twiddle table is complete
    for (;;) {
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int r = work / n_part, p = work % n_part;
        // the response is zero before its first non-zero tap, and so is everything convolved with it
        for (int off = 32; off > 0; off >>= 1) first = min(first, __shfl_down(first, off, 64));
        if ((tid & 63) == 0 && first != 0x7fffffff) atomicMin(&first_tap[r], first);
        float2 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = i < 8 ? taps[i] : make_float2(0.f, 0.f);
        fft_columns_forward<N>(v, tw, tid);
        fft_columns_store<N, T>(v, buf, tid);
        __syncthreads();
        const int next = work + (int)gridDim.x;
        if (next < n_work)
            first = load_taps<N>(taps, rir + (size_t)(next / n_part) * rir_len, rir_len, next % n_part, tid);
        fft_rows_table<N, false>(buf, row_tw, tid);
        __syncthreads();
        asm volatile("" : "+v"(tid));
        float2* out = spec + ((size_t)r * n_part + p) * (N + 1);
        const float scale = 0.25f / (float)N;
        const int k2 = tid % (M / 2), half = tid / (M / 2);
#pragma unroll
        for (int i = 0; i <= 8; ++i) {
            if (i == 8 && tid != 0) break;
            const PairIndex<N> ix(i == 8 ? 0 : half * 8 + i, i == 8 ? M / 2 : k2);
            const float2 A = buf[lds_pad(ix.pos)];
            const float2 B = cconj(buf[lds_pad(ix.pos_partner)]);
            const float2 w = i == 8 ? tw[N + N / 2] : pair_twiddle<N>(tw, half * 8 + i, k2);
            float2 Hk, HNk_conj;
            unpack_pair(A, B, w, Hk, HNk_conj);
            out[ix.pos] = make_float2(Hk.x * scale, Hk.y * scale);
            if (i < 8) out[ix.h_partner] = make_float2(HNk_conj.x * scale, -HNk_conj.y * scale);
        }
        if (next >= n_work) break;
        work = next;
        __syncthreads();                             // every bin is read before the next column store
    }
}

// Z'[k] and Z'[N-k] of the packed output block from Z[k] = A, conj(Z[N-k]) = B and the response
// spectrum: Y = W H on the 2N-point real transform, repacked for the N-point inverse.  The halves of the
// even/odd split (two on the way in, two on the way out) are left out here: the stored response spectrum
// carries the factor 1/4 for them (powers of two: the result is the same bit for bit).
__device__ inline void multiply_pair(float2 A, float2 B, float2 w, float2 Hk, float2 HNk, float2& Zk, float2& ZNk) {
    const float2 E = cadd(A, B);
    const float2 d = csub(A, B);
    const float2 O = make_float2(d.y, -d.x);         // -i (A - B)
    const float2 wO = cmul(w, O);
    const float2 Yk = cmul(Hk, cadd(E, wO));
    const float2 YNk_conj = cmul_conj(csub(E, wO), HNk);
    const float2 Ye = cadd(Yk, YNk_conj);
    const float2 Yo = cmul_conj(csub(Yk, YNk_conj), w);      // conj(w) (Y[k] - conj Y[N-k])
    Zk = make_float2(Ye.x - Yo.y, Ye.y + Yo.x);      // Ye + i Yo
    ZNk = make_float2(Ye.x + Yo.y, Yo.x - Ye.y);     // conj(Ye) + i conj(Yo)
}

// two consecutive samples; only their 4-byte alignment is promised (global accesses of two dwords need no more)
struct __attribute__((aligned(4))) SamplePair { float x, y; };

// Accesses at a per-lane 32-bit byte offset from a wave-uniform base: the address is then a scalar register
// pair plus one vector register, with no 64-bit vector arithmetic per access.
__device__ inline SamplePair load_pair(const float* base, uint32_t byte_off) {
    return *reinterpret_cast<const SamplePair*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ inline float load_sample(const float* base, uint32_t byte_off) {
    return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ inline float2 load_bin(const float2* base, uint32_t byte_off) {
    return *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(base) + byte_off);
}

// One block of one (utterance, source): everything here is the same for all lanes.
struct ConvBlock {
    const float* x;          // the source's signal, first sample of the utterance
    const float2* H;         // the response's spectra, partition 0
    float* y;                // reverberated signal, first sample of the utterance
    double* energy;          // E[u][j]
    int len;                 // samples of the utterance
    int first;               // first non-zero tap of the response
    int b;                   // block index: outputs [b N, (b+1) N)
};

// The window of block wb, samples [(wb-1) N, (wb+1) N) of the utterance, as the inputs of the column step:
// v[n1] = (x[2n], x[2n+1]), n = tid + M n1.  Block wb - 1 is a whole block of the utterance or (wb = 0) lies
// before its start; block wb is whole except at the utterance's end.  Whole blocks are read with two-sample
// loads and nothing to test, the same for every thread of the group.
template <int N>
__device__ inline void load_window(float2 (&v)[16], const float* x, int len, int wb, int tid) {
    constexpr int M = N / 16;
    const uint32_t lane_off = 8u * (uint32_t)tid;
    if (wb >= 1) {
        const float* blk = x + (size_t)(wb - 1) * N;
#pragma unroll
        for (int n1 = 0; n1 < 8; ++n1) {
            const SamplePair s2 = load_pair(blk + 2 * M * n1, lane_off);
            v[n1] = make_float2(s2.x, s2.y);
        }
    } else {
#pragma unroll
        for (int n1 = 0; n1 < 8; ++n1) v[n1] = make_float2(0.f, 0.f);
    }
    const float* blk = x + (size_t)wb * N;
    if ((wb + 1) * (int64_t)N <= len) {
#pragma unroll
        for (int n1 = 8; n1 < 16; ++n1) {
            const SamplePair s2 = load_pair(blk + 2 * M * (n1 - 8), lane_off);
            v[n1] = make_float2(s2.x, s2.y);
        }
    } else {
        // the utterance ends inside this block: addresses are clamped to its last sample, values past it are zero
        const int left = len - wb * N;                     // 1 .. N - 1 samples of this block exist
#pragma unroll
        for (int n1 = 8; n1 < 16; ++n1) {
            const int g = 2 * tid + 2 * M * (n1 - 8);
            const float x0 = load_sample(blk, 4u * (uint32_t)min(g, left - 1));
            const float x1 = load_sample(blk, 4u * (uint32_t)min(g + 1, left - 1));
            v[n1] = make_float2(g < left ? x0 : 0.f, g + 1 < left ? x1 : 0.f);
        }
    }
}

// The outputs of a block, v[8 + i] = (y[n], y[n+1]) with n = b N + 2 tid + 2 M i, go to HBM; returns the
// lane's share of the block's energy.  Samples before the response's first non-zero tap are exact zeros
// (the transforms leave rounding noise there, which the power law of the front end would magnify).
template <int N>
__device__ inline float store_block(const float2 (&v)[16], const ConvBlock& c, int tid) {
    constexpr int M = N / 16;
    float* yb = c.y + (size_t)c.b * N;
    const int first = c.first - c.b * N;                   // first live sample of this block (may be <= 0)
    const int left = c.len - c.b * N;                      // samples of this block inside the utterance
    float e = 0.f;
    if (left >= N && first <= 0) {                         // whole and live: eight two-sample stores
        char* dst = reinterpret_cast<char*>(yb) + 8u * (uint32_t)tid;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            SamplePair s2;
            s2.x = v[8 + i].x;
            s2.y = v[8 + i].y;
            *reinterpret_cast<SamplePair*>(dst + 8 * M * i) = s2;
            e += s2.x * s2.x + s2.y * s2.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = 2 * tid + 2 * M * i;
            const float s0 = g >= first ? v[8 + i].x : 0.f, s1 = g + 1 >= first ? v[8 + i].y : 0.f;
            if (g < left) { yb[g] = s0; e += s0 * s0; }
            if (g + 1 < left) { yb[g + 1] = s1; e += s1 * s1; }
        }
    }
    return e;
}

// Work groups are persistent and take their blocks from the list of all blocks ordered by (utterance,
// source, block), either a contiguous share or every 32nd block of an eighth of the list (see the kernel).  While a block's
// inverse transform runs, the inputs of the next block are already on their way from HBM, and the response
// spectrum is requested before the forward row transforms that precede its use: the loads' latency is
// hidden behind arithmetic instead of being paid at either end of a short-lived group.
// MULTI: the response has two partitions.  Block b is then the inverse transform of
// H_0 W_b + H_1 W_{b-1}; W_{b-1} is the window spectrum of the block this group finished just before, and
// each thread keeps its sixteen bins of it in registers, so a block still costs one forward and one inverse
// transform (plus one forward transform at the start of a group's share).
template <int N, int T, bool MULTI>
__global__ __launch_bounds__(T) void convolve_kernel(ConvArgs a, const float2* __restrict__ tw) {
    extern __shared__ float2 buf[];
    __shared__ double red[T / 64];
    constexpr int M = N / 16;
    static_assert(T == M, "one thread per column of the split transform");
    // behind the transform buffer: the row transforms' twiddles with their powers, and the two factors of
    // the even/odd split's twiddle exp(-i pi (k1 + 16 k2) / N) = split_lo[k1] split_hi[k2]
    float2* const row_tw = buf + lds_padded_size(N);
    float2* const split_lo = row_tw + RowTwiddles<M>::kEntries;
    float2* const split_hi = split_lo + 16;
    RowTwiddles<M>::template fill<16>(row_tw, tw, threadIdx.x, T);
    for (int i = threadIdx.x; i < 16 + M / 2; i += T) split_lo[i] = i < 16 ? tw[N + i] : tw[N + N / 2 + 1 + (i - 16)];
    // (the first barrier of the loop below comes before any of these is read)
    // With two partitions the kept spectrum takes the registers that the single-partition kernel spends on
    // loads issued ahead of time; the inputs and the response spectrum are then loaded where they are used.
    constexpr bool AHEAD = !MULTI;
    const int tid0 = threadIdx.x;
    const int total = (int)(a.n_items * a.n_src);          // (the launcher refuses lists of 2^31 blocks or more)
    // Shares.  With two partitions a group needs consecutive blocks of a signal, so it takes one contiguous
    // range of the list.  Otherwise the groups that share an L2 (the hardware deals group ids round-robin to
    // the eight XCDs) take one contiguous eighth of the list together and go through it side by side, group
    // s of the 32 on blocks s, s + 32, ...: at any time they are on a few neighbouring signals, so a
    // response spectrum and the halves that neighbouring windows have in common are fetched from HBM once
    // and found in L2 by the other groups, not re-read by one group a whole block later.
    constexpr bool STRIDED = !MULTI;
    int w_begin, w_end, w_step;
    if (STRIDED) {
        const int teams = gridDim.x % 8 == 0 ? 8 : 1;
        const int team = blockIdx.x % teams, slot = blockIdx.x / teams;
        w_begin = (int)((int64_t)total * team / teams) + slot;
        w_end = (int)((int64_t)total * (team + 1) / teams);
        w_step = (int)gridDim.x / teams;
    } else {
        w_begin = (int)((int64_t)total * blockIdx.x / gridDim.x);
        w_end = (int)((int64_t)total * (blockIdx.x + 1) / gridDim.x);
        w_step = 1;
    }
    if (w_begin >= w_end) return;

    // block w of the list: utterance u (the one that holds item w / n_src), source j, block b
    int u, nb, j, b;
    auto locate = [&](int at) {
        u = a.items[(unsigned int)at / (unsigned int)a.n_src].x;
        nb = a.first[u + 1] - a.first[u];
        const unsigned int r = (unsigned int)(at - a.first[u] * a.n_src);
        j = (int)(r / (unsigned int)nb);
        b = (int)r - j * nb;
    };
    locate(w_begin);
    auto describe = [&](int uu, int jj, int bb) {
        ConvBlock c;
        const int64_t start = a.offsets[uu];
        const size_t uj = (size_t)uu * a.n_src + jj;
        c.len = (int)(a.offsets[uu + 1] - start);          // utterances are shorter than 2^30 samples (checked on the host)
        c.x = (jj == 0 ? a.speech : a.noise + (size_t)(jj - 1) * a.total) + start;
        c.H = a.spec + uj * a.n_part * (size_t)(N + 1);
        c.y = a.reverb + (size_t)jj * a.reverb_stride + start;
        c.energy = a.energy + uj;
        c.first = a.first_tap[uj];
        c.b = bb;
        return c;
    };
    ConvBlock cur = describe(u, j, b);

    float2 v[16];
    float2 prev_a[MULTI ? 8 : 1], prev_b[MULTI ? 8 : 1], prev_mid = make_float2(0.f, 0.f);
    bool have_prev = false;         // prev_* hold the window spectrum of block cur.b - 1 of this signal
    if (MULTI) {
#pragma unroll
        for (int i = 0; i < 8; ++i) prev_a[i] = prev_b[i] = make_float2(0.f, 0.f);
        have_prev = cur.b == 0;     // the window before the first block is all zeros, and so is its spectrum
    }
    if (AHEAD) load_window<N>(v, cur.x, cur.len, cur.b, tid0);

    for (int w = w_begin;;) {
        // The thread index is made opaque in every round so that twiddle powers and addresses are not
        // hoisted out of the loop, where they would sit on top of the transforms' registers.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const bool warm_up = MULTI && !have_prev;          // this pass only produces the spectrum of window b - 1
        if (!AHEAD) load_window<N>(v, cur.x, cur.len, warm_up ? cur.b - 1 : cur.b, tid);

        fft_columns_forward<N>(v, tw, tid);
        fft_columns_store<N, T>(v, buf, tid);
        __syncthreads();

        // the response spectrum of this thread's bins, requested now, used after the row transforms
        float2 hk[8], hn[8];
        if (AHEAD) {
            const int k2 = tid % (M / 2), half = tid / (M / 2);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const PairIndex<N> ix(half * 8 + i, k2);
                hk[i] = load_bin(cur.H, 8u * (uint32_t)ix.pos);
                hn[i] = load_bin(cur.H, 8u * (uint32_t)ix.h_partner);
            }
        }
        fft_rows_table<N, false>(buf, row_tw, tid);
        __syncthreads();
        // (opaque again: bin positions are recomputed here rather than kept in registers across the transform)
        asm volatile("" : "+v"(tid));
        const int k2 = tid % (M / 2), half = tid / (M / 2);

        if (warm_up) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const PairIndex<N> ix(half * 8 + i, k2);
                prev_a[i] = buf[lds_pad(ix.pos)];
                prev_b[i] = cconj(buf[lds_pad(ix.pos_partner)]);
            }
            prev_mid = buf[lds_pad(M / 2)];
            have_prev = true;
            __syncthreads();                               // all bins are read before the next column store
            continue;
        }

        const float2* H1 = cur.H + (N + 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const PairIndex<N> ix(half * 8 + i, k2);
            const float2 A = buf[lds_pad(ix.pos)];
            const float2 B = cconj(buf[lds_pad(ix.pos_partner)]);
            const float2 wk = cmul(split_lo[half * 8 + i], split_hi[k2]);
            if (!AHEAD) {
                hk[i] = load_bin(cur.H, 8u * (uint32_t)ix.pos);
                hn[i] = load_bin(cur.H, 8u * (uint32_t)ix.h_partner);
            }
            float2 Zk, ZNk;
            multiply_pair(A, B, wk, hk[i], hn[i], Zk, ZNk);
            if (MULTI) {
                float2 Zk1, ZNk1;
                multiply_pair(prev_a[i], prev_b[i], wk, load_bin(H1, 8u * (uint32_t)ix.pos),
                              load_bin(H1, 8u * (uint32_t)ix.h_partner), Zk1, ZNk1);
                Zk = cadd(Zk, Zk1);
                ZNk = cadd(ZNk, ZNk1);
                prev_a[i] = A;
                prev_b[i] = B;
            }
            buf[lds_pad(ix.pos)] = Zk;                     // both positions belong to this thread alone
            if (ix.k != 0) buf[lds_pad(ix.pos_partner)] = ZNk;
        }
        if (tid == 0) {                                    // the bin in the middle, k = N / 2, is its own partner
            const PairIndex<N> ix(0, M / 2);
            const float2 A = buf[lds_pad(ix.pos)];
            const float2 wk = tw[N + N / 2];
            float2 Zk, ZNk;
            multiply_pair(A, cconj(A), wk, cur.H[ix.pos], cur.H[ix.h_partner], Zk, ZNk);
            if (MULTI) {
                float2 Zk1, ZNk1;
                multiply_pair(prev_mid, cconj(prev_mid), wk, H1[ix.pos], H1[ix.h_partner], Zk1, ZNk1);
                Zk = cadd(Zk, Zk1);
                prev_mid = A;
            }
            buf[lds_pad(ix.pos)] = Zk;
        }
        __syncthreads();

        // the next block of the share: its inputs are requested now and arrive during the inverse transform
        const bool more = w + w_step < w_end;
        ConvBlock nxt = cur;
        asm volatile("" : "+v"(tid));
        if (more) {
            if (STRIDED) {
                locate(w + w_step);
            } else if (++b == nb) {
                b = 0;
                if (++j == a.n_src) {
                    j = 0;
                    do {
                        ++u;
                        nb = a.first[u + 1] - a.first[u];
                    } while (nb == 0);
                }
            }
            nxt = describe(u, j, b);
            if (AHEAD) load_window<N>(v, nxt.x, nxt.len, nxt.b, tid);
        } else if (AHEAD) {
            // (assigned on this path too, so that the old inputs do not stay alive in registers up to here)
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = make_float2(0.f, 0.f);
        }

        fft_rows_table<N, true>(buf, row_tw, tid);
        __syncthreads();
        float2 o[16];
        fft_columns_load<N, T>(o, buf, tid);
        fft_columns_inverse<N>(o, tw, tid);
        const float e = store_block<N>(o, cur, tid);

        float es = e;                                      // a wave's 1024 squares in fp32, the rest in fp64
        for (int off = 32; off > 0; off >>= 1) es += __shfl_down(es, off, 64);
        if ((tid & 63) == 0) red[tid >> 6] = (double)es;
        __syncthreads();                                   // also: every thread has read its columns from LDS
        if (tid == 0) {
            double tot = 0.0;
            for (int i = 0; i < T / 64; ++i) tot += red[i];
            atomicAdd(cur.energy, tot);
        }
        if (!more) break;
        if (MULTI && nxt.b == 0) {                         // a new signal starts: nothing precedes its first window
#pragma unroll
            for (int i = 0; i < 8; ++i) prev_a[i] = prev_b[i] = make_float2(0.f, 0.f);
            prev_mid = make_float2(0.f, 0.f);
        }
        cur = nxt;
        w += w_step;
    }
}

// One thread per (utterance, noise source): the gain that puts the reverberated noise at its target
// SNR against the reverberated speech; zero energy on either side gives gain 0.  (A source whose direct
// path arrives after the utterance has ended has exactly zero energy: the convolution writes exact zeros
// before the response's first non-zero tap.)
__global__ void gain_kernel(int n_utt, int n_src, const double* __restrict__ energy, const float* __restrict__ snr_db,
                            float* __restrict__ gains, float* __restrict__ gains_out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int n_noise = n_src - 1;
    if (i >= n_utt * n_noise) return;
    const int u = i / n_noise, j = 1 + i % n_noise;
    const double e0 = energy[(size_t)u * n_src], ej = energy[(size_t)u * n_src + j];
    const double snr = (double)snr_db[i];
    const float gain = (e0 > 0.0 && ej > 0.0) ? (float)sqrt(e0 / (ej * pow(10.0, snr / 10.0))) : 0.f;
    gains[i] = gain;
    if (gains_out) gains_out[i] = gain;
}

__global__ __launch_bounds__(256) void mix_kernel(
    const int64_t* __restrict__ offsets, int64_t stride, int n_src, const float* __restrict__ reverb,
    const float* __restrict__ gains, float* __restrict__ mixed) {
    const int u = blockIdx.y;
    const int64_t start = offsets[u];
    const int64_t len = offsets[u + 1] - start;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x * 4;
    if (first >= len) return;
    const float* g = gains + (size_t)u * (n_src - 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t n = first + (int64_t)i * blockDim.x + threadIdx.x;
        if (n < len) {
            float acc = reverb[start + n];
            for (int j = 1; j < n_src; ++j) acc += g[j - 1] * reverb[(size_t)j * stride + start + n];
            mixed[start + n] = acc;
        }
    }
}

template <int N>
hipError_t spectrum_n(hipStream_t s, int n_rir, const float* rir, int rir_len, const float2* tw,
                      float2* spec, int* first_tap, int n_cu) {
    constexpr int T = conv_threads(N);
    int n_part = (rir_len + N - 1) / N;
    int n_work = n_rir * n_part;
    const size_t lds = sizeof(float2) * (lds_padded_size(N) + RowTwiddles<N / 16>::kEntries);
    auto k = &rir_spectrum_kernel<N, T>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // as many persistent groups as the chip holds at once (see convolve_n)
    const int by_lds = (int)((160 * 1024) / (lds + 256));
    const int by_waves = 16 / ((T + 63) / 64);
    const int per_cu = by_lds < 1 ? 1 : (by_lds < by_waves ? by_lds : by_waves);
    int groups = n_cu * per_cu;
    if (groups > n_work) groups = n_work;
    // (launched by address, not called through the pointer: the call form is what undefined-behaviour
    // sanitizers of the host code instrument, and with them it was seen to launch nothing)
    void* args[] = {&rir, &rir_len, &n_part, &n_work, &tw, &spec, &first_tap};
    return hipLaunchKernel(reinterpret_cast<const void*>(k), dim3((unsigned)groups), dim3(T), args, lds, s);
}

template <int N>
hipError_t convolve_n(hipStream_t s, const float2* tw, const ConvArgs& a, int n_cu) {
    constexpr int T = conv_threads(N);
    const size_t lds = sizeof(float2) * (lds_padded_size(N) + RowTwiddles<N / 16>::kEntries + 16 + N / 32);
    // responses longer than one partition exist only at the largest transform size (conv_fft_size)
    void (*k)(ConvArgs, const float2*) = &convolve_kernel<N, T, false>;
    if (a.n_part > 1) {
        if constexpr (N == 16384) k = &convolve_kernel<N, T, true>;
        else return hipErrorInvalidValue;
        if (a.n_part != 2) return hipErrorInvalidValue;
    }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // as many persistent groups as the chip holds at once: per compute unit, what the 160 KB of LDS and
    // sixteen wavefronts (128 registers each) allow
    const int by_lds = (int)((160 * 1024) / (lds + 256));
    const int by_waves = 16 / ((T + 63) / 64);
    const int per_cu = by_lds < 1 ? 1 : (by_lds < by_waves ? by_lds : by_waves);
    int64_t groups = (int64_t)n_cu * per_cu;
    const int64_t total = a.n_items * a.n_src;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    if (groups > total) groups = total;
    ConvArgs by_value = a;
    void* args[] = {&by_value, &tw};
    return hipLaunchKernel(reinterpret_cast<const void*>(k), dim3((unsigned)groups), dim3(T), args, lds, s);
}

}  // namespace

int conv_fft_size(int rir_len) {
    int n = 1024;                       // at least one full wave of sixteen-point butterflies
    while (n < rir_len && n < 16384) n <<= 1;
    return n;
}

int twiddle_entries(int n) { return twiddle_count(n); }

hipError_t launch_twiddle(hipStream_t s, int n, float2* tw) {
    const int count = twiddle_count(n);
    twiddle_kernel<<<dim3((count + 255) / 256), dim3(256), 0, s>>>(n, tw);
    return hipGetLastError();
}

#define AUG_FFT_DISPATCH(n, CALL)                                  \
    switch (n) {                                                   \
        case 1024: return CALL(1024);                              \
        case 2048: return CALL(2048);                              \
        case 4096: return CALL(4096);                              \
        case 8192: return CALL(8192);                              \
        case 16384: return CALL(16384);                            \
        default: return hipErrorInvalidValue;                      \
    }

hipError_t launch_rir_spectrum(hipStream_t s, int n_rir, const float* rir, int rir_len, int fft_n,
                               const float2* twiddle, float2* spec, int* first_tap, int n_cu) {
    if (n_rir <= 0) return hipSuccess;
#define CALL(NN) spectrum_n<NN>(s, n_rir, rir, rir_len, twiddle, spec, first_tap, n_cu)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_convolve(hipStream_t s, int fft_n, const float2* twiddle, const ConvArgs& a, int n_cu) {
    if (a.n_items <= 0) return hipSuccess;
#define CALL(NN) convolve_n<NN>(s, twiddle, a, n_cu)
    AUG_FFT_DISPATCH(fft_n, CALL)
#undef CALL
}

hipError_t launch_gains(hipStream_t s, int n_utt, int n_src, const double* energy, const float* snr_db, float* gains,
                        float* gains_out) {
    const int n = n_utt * (n_src - 1);
    if (n <= 0) return hipSuccess;
    gain_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(n_utt, n_src, energy, snr_db, gains,
                                                                         gains_out);
    return hipGetLastError();
}

hipError_t launch_mix(hipStream_t s, int n_utt, const int64_t* d_offsets, int64_t stride, int n_src,
                      const float* reverb, const float* gains, float* mixed_out, int64_t max_len) {
    if (n_utt <= 0) return hipSuccess;
    int64_t chunks = (max_len + 1023) / 1024;
    if (chunks < 1) chunks = 1;
    mix_kernel<<<dim3((unsigned)chunks, (unsigned)n_utt), dim3(256), 0, s>>>(
        d_offsets, stride, n_src, reverb, gains, mixed_out);
    return hipGetLastError();
}

}  // namespace aug
