// Weight-streaming GEMM for M <= 128 activation rows:  part[s][m][n] = sum_{k in split s} X[m][k] W[n][k].
//
// The round is bound by reading every weight once (the verify pass reads the whole target, each
// draft pass one specialist and the shared LM head; sections 3.3 and 6.2 of the paper discuss the
// cost of switching specialist parameters, which is exactly this stream).  Design:
//   * weights pre-packed in MFMA B-operand order: each lane issues 16-byte loads, a wave reads
//     GEMM_NT KiB contiguous per k-step straight into registers (no LDS hop for the big operand);
//   * a ring of PF k-steps of weight loads stays in flight per wave across LDS chunk boundaries;
//   * the (small, L2-resident) activation slice is staged in LDS in A-operand order, double
//     buffered, its global loads issued one chunk ahead so they are older than the weight loads
//     they overlap and never force the weight ring to drain;
//   * K is split across workgroups (fixed order, summed by the consumer kernel: bitwise
//     repeatable, no atomics).
#include "common.h"

namespace poss {

typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef f16_t  f16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Mfma;
template <> struct Mfma<bf16_t> {
    static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<f16_t> {
    static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

constexpr int KCS = GEMM_KCHUNK / GEMM_KSTEP;   // k-steps per LDS chunk (8)
constexpr int PF  = 4;                          // weight k-steps in flight per wave

// ------------------------------------------------------------------------------------------
template <typename T, int MT>
__global__ __launch_bounds__(GEMM_WPB * 64) void gemm_stream_kernel(
    const u32x4 *__restrict__ Wp, const T *__restrict__ X, int ldx, float *__restrict__ part,
    int M, int K, int Npad, int ksteps_total, int chunks_per_split) {
    static_assert(KCS % PF == 0, "ring index must be static");
    constexpr int XUNITS = KCS * MT * 64;                 // 16-byte units of one staged chunk
    constexpr int XPT    = XUNITS / (GEMM_WPB * 64);      // units per thread (2*MT)
    __shared__ u32x4 xs[2][XUNITS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int chunk0 = blockIdx.y * chunks_per_split;
    const int n_chunks_total = ksteps_total / KCS;
    const int chunk1 = min(n_chunks_total, chunk0 + chunks_per_split);
    const int ks_end = chunk1 * KCS;
    const int ngroup = blockIdx.x * GEMM_WPB + wave;
    const u32x4 *wp = Wp + ((size_t)ngroup * ksteps_total + (size_t)chunk0 * KCS) * (GEMM_NT * 64) + lane;

    // Global->LDS staging map: unit u of a chunk covers row m = u / 32, 8 consecutive k starting at
    // (u % 32) * 8 (coalesced along k); it lands at A-operand position [k_step][m_tile][lane].
    int x_m[XPT], x_k8[XPT], x_dst[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int u = tid + i * (GEMM_WPB * 64);
        const int m = u >> 5, k8 = u & 31;
        x_m[i] = m; x_k8[i] = k8;
        x_dst[i] = ((k8 >> 2) * MT + (m >> 4)) * 64 + ((k8 & 3) << 4) + (m & 15);
    }
    auto load_x = [&](int chunk, u32x4 (&xr)[XPT]) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int k = chunk * GEMM_KCHUNK + x_k8[i] * 8;
            xr[i] = (x_m[i] < M && k < K)
                        ? *reinterpret_cast<const u32x4 *>(X + (size_t)x_m[i] * ldx + k)
                        : u32x4{0u, 0u, 0u, 0u};
        }
    };

    f32x4 acc[MT][GEMM_NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 xr[XPT];
    load_x(chunk0, xr);
    u32x4 wr[PF][GEMM_NT];
    int ks_issue = chunk0 * KCS;                     // next k-step whose weights get requested
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        if (ks_issue < ks_end) {
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt) wr[p][nt] = __builtin_nontemporal_load(wp + nt * 64);
            wp += GEMM_NT * 64;
        }
        ++ks_issue;
    }
#pragma unroll
    for (int i = 0; i < XPT; ++i) xs[0][x_dst[i]] = xr[i];
    __syncthreads();

    int buf = 0;
    for (int chunk = chunk0; chunk < chunk1; ++chunk) {
        const bool more = chunk + 1 < chunk1;
        if (more) load_x(chunk + 1, xr);             // older than every weight load issued below
#pragma unroll
        for (int i = 0; i < KCS; ++i) {
            u32x4 a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = xs[buf][(i * MT + mt) * 64 + lane];
            u32x4 w[GEMM_NT];
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt) w[nt] = wr[i % PF][nt];
            if (ks_issue < ks_end) {
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) wr[i % PF][nt] = __builtin_nontemporal_load(wp + nt * 64);
                wp += GEMM_NT * 64;
            }
            ++ks_issue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = Mfma<T>::run(a[mt], w[nt], acc[mt][nt]);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < XPT; ++i) xs[buf ^ 1][x_dst[i]] = xr[i];
        }
        __syncthreads();
        buf ^= 1;
    }

    // D tile: lane -> column n = lane % 16, register r -> row m = 4 * (lane / 16) + r
    float *out = part + (size_t)blockIdx.y * (MT * 16) * Npad;
    const int n0 = ngroup * (GEMM_NT * 16) + (lane & 15);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = mt * 16 + 4 * (lane >> 4) + r;
                out[(size_t)m * Npad + n0 + nt * 16] = acc[mt][nt][r];
            }
}

// ------------------------------------------------------------------------------------------
// float32 storage (reference-precision mode of the small test shape): plain FMA loop, weights
// kept row-major.  One thread per output element, k ascending.
__global__ void gemm_f32_kernel(const float *__restrict__ W, const float *__restrict__ X, int ldx,
                                float *__restrict__ part, int M, int N, int Npad, int K) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= Npad) return;
    float acc = 0.f;
    if (n < N && m < M) {
        const float *w = W + (size_t)n * K, *x = X + (size_t)m * ldx;
        for (int k = 0; k < K; ++k) acc = fmaf(x[k], w[k], acc);
    }
    part[(size_t)m * Npad + n] = acc;
}

// ------------------------------------------------------------------------------------------
// Row count of a partial plane as the kernel instantiation writes it.
static int gemm_rows_written(int mpad) {
    const int mt = mpad / 16;
    return (mt <= 2 ? mt : mt <= 4 ? 4 : mt <= 6 ? 6 : 8) * 16;
}

GemmShape gemm_plan(int dt, int M, int N, int K, int target_wgs) {
    GemmShape g;
    g.M = M; g.N = N; g.K = K;
    g.Npad = gemm_npad(N);
    g.Kpad = gemm_kpad(dt, K);
    g.Mpad = round_up(M < 1 ? 1 : M, 16);
    if (dt == DT_F32) { g.S = 1; g.chunks_per_split = 0; return g; }
    g.Mpad = gemm_rows_written(g.Mpad);       // the kernel is instantiated for 1, 2, 4, 6 or 8 row tiles
    const int n_blocks = g.Npad / GEMM_BLOCK_N;
    const int n_chunks = g.Kpad / GEMM_KCHUNK;
    if (target_wgs <= 0) target_wgs = 512;
    int S = (target_wgs + n_blocks - 1) / n_blocks;
    int max_s = n_chunks / 2; if (max_s < 1) max_s = 1;          // at least 512 of K per split
    if (S > max_s) S = max_s;
    if (S < 1) S = 1;
    g.chunks_per_split = (n_chunks + S - 1) / S;
    g.S = (n_chunks + g.chunks_per_split - 1) / g.chunks_per_split;
    return g;
}

template <typename T>
static void launch_gemm_t(const GemmShape &g, const void *Wp, const void *X, int ldx, float *part,
                          hipStream_t st) {
    dim3 grid(g.Npad / GEMM_BLOCK_N, g.S), block(GEMM_WPB * 64);
    const int ksteps = g.Kpad / GEMM_KSTEP;
    const u32x4 *w = static_cast<const u32x4 *>(Wp);
    const T *x = static_cast<const T *>(X);
#define POSS_GEMM_CASE(MT)                                                                        \
    hipLaunchKernelGGL((gemm_stream_kernel<T, MT>), grid, block, 0, st, w, x, ldx, part, g.M, g.K, \
                       g.Npad, ksteps, g.chunks_per_split)
    switch (g.Mpad / 16) {
        case 1: POSS_GEMM_CASE(1); break;
        case 2: POSS_GEMM_CASE(2); break;
        case 4: POSS_GEMM_CASE(4); break;
        case 6: POSS_GEMM_CASE(6); break;
        default: POSS_GEMM_CASE(8); break;
    }
#undef POSS_GEMM_CASE
}

void launch_gemm(int dt, const GemmShape &g, const void *Wp, const void *X, int ldx, float *part,
                 hipStream_t st) {
    if (dt == DT_F32) {
        dim3 grid((g.Npad + 127) / 128, g.Mpad), block(128);
        hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, st, static_cast<const float *>(Wp),
                           static_cast<const float *>(X), ldx, part, g.M, g.N, g.Npad, g.K);
    } else if (dt == DT_BF16) {
        launch_gemm_t<bf16_t>(g, Wp, X, ldx, part, st);
    } else {
        launch_gemm_t<f16_t>(g, Wp, X, ldx, part, st);
    }
}

// ------------------------------------------------------------------------------------------
// Repack up to three row-major [rows_i, K] matrices, stacked along N, into B-operand order.
__global__ void pack16_kernel(PackSrc src, int K, int Kpad, int Npad, u32x4 *__restrict__ dst) {
    const size_t unit = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte unit of dst
    const size_t total = (size_t)Npad * Kpad / 8;
    if (unit >= total) return;
    const int ksteps = Kpad / GEMM_KSTEP;
    const int lane = unit & 63;
    size_t r = unit >> 6;
    const int nt = r % GEMM_NT; r /= GEMM_NT;
    const int ks = r % ksteps;
    const int ngroup = r / ksteps;
    int n = (ngroup * GEMM_NT + nt) * 16 + (lane & 15);
    const int k = ks * GEMM_KSTEP + (lane >> 4) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (k < K) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            if (n >= 0 && n < src.rows[i]) {
                v = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(src.ptr[i]) + (size_t)n * K + k);
                n = -1;
            } else if (n >= 0) {
                n -= src.rows[i];
            }
        }
    }
    dst[unit] = v;
}

__global__ void pack32_kernel(PackSrc src, int K, int Npad, float *__restrict__ dst) {
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)Npad * K) return;
    int n = e / K;
    const int k = e % K;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        if (n >= 0 && n < src.rows[i]) {
            v = static_cast<const float *>(src.ptr[i])[(size_t)n * K + k];
            n = -1;
        } else if (n >= 0) {
            n -= src.rows[i];
        }
    }
    dst[e] = v;
}

void launch_pack(int dt, const PackSrc &src, int K, void *dst, hipStream_t st) {
    const int N = src.rows[0] + src.rows[1] + src.rows[2];
    const int Npad = gemm_npad(N), Kpad = gemm_kpad(dt, K);
    if (dt == DT_F32) {
        const size_t total = (size_t)Npad * K;
        hipLaunchKernelGGL(pack32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, K, Npad,
                           static_cast<float *>(dst));
    } else {
        const size_t total = (size_t)Npad * Kpad / 8;
        hipLaunchKernelGGL(pack16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, K, Kpad,
                           Npad, static_cast<u32x4 *>(dst));
    }
}

}  // namespace poss
