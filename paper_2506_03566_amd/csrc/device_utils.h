// Device-side helpers: storage conversions, block reductions, cache addressing.
#pragma once
#include "common.h"

namespace poss {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v) { return (T)v; }   // round to nearest even

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a workgroup of up to 1024 threads, identical in every thread; fixed order.
__device__ __forceinline__ float block_sum(float v, float *red /* >= 17 floats of LDS */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    __syncthreads();                      // red may still be read from an earlier call
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i];
    return s;
}

// One 16-byte LDS-direct load per lane: lane l's 16 bytes from `g` land at LDS byte address lds_base + 16 l
// (lds_base wave-uniform).  Written as assembly because the compiler, which cannot tell which LDS reads a
// load it knows of may alias, would wait for ALL such loads before every LDS read; counted waits
// (dma_wait) are placed by hand instead.  M0 is set in the same statement and nothing else in these kernels uses it.
__device__ __forceinline__ void lds_dma16(unsigned lds_base, const void *g) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(g) : "memory");
}
// Wait until at most N of this wave's vector-memory loads are outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void dma_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// A token id that came out of arithmetic indexes the embedding table only through this: an argmax over a row of
// logits that are all NaN finds no entry that compares and leaves the id of "no entry" (0x7fffffff) - a bad number
// must not become a bad address.  Such a row reads token 0.
__device__ __forceinline__ int embedding_row(int token, int vocab) { return (unsigned)token < (unsigned)vocab ? token : 0; }

// (value, index) ordering used by every argmax / top-k here: larger value first, then lower index.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
    return (v > bv) || (v == bv && i < bi);
}

__device__ __forceinline__ void wave_argmax(float &v, int &i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(i, o, 64);
        if (better(ov, oi, v, i)) { v = ov; i = oi; }
    }
}

// Workgroup-wide argmax; result valid in every thread.  red_v/red_i: >= 17 entries of LDS each.
__device__ __forceinline__ void block_argmax(float &v, int &i, float *red_v, int *red_i) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    wave_argmax(v, i);
    __syncthreads();
    if (lane == 0) { red_v[wave] = v; red_i[wave] = i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float bv = red_v[0]; int bi = red_i[0];
        for (int w = 1; w < nw; ++w)
            if (better(red_v[w], red_i[w], bv, bi)) { bv = red_v[w]; bi = red_i[w]; }
        red_v[16] = bv; red_i[16] = bi;
    }
    __syncthreads();
    v = red_v[16]; i = red_i[16];
}

// Maximum over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48), left in every lane.  The two
// row-swap instructions of gfx950 stay in the vector ALU (v_permlane16_swap: [A.r0 B.r0 A.r2 B.r2] and
// [A.r1 B.r1 A.r3 B.r3] from rows r0..r3 of registers A and B; v_permlane32_swap: [A.lo B.lo] and
// [A.hi B.hi]); a shuffle would go through the LDS crossbar and wait for it.  Written as assembly with both
// registers as in/out operands: through the builtin, this compiler reads the second result from the first
// register.  (The s_nop covers the wait states a swap needs behind the VALU write of its operands.)
// Every lane of the wave must be active.
__device__ __forceinline__ float rows_max(float x) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    x = fmaxf(a, b);
    a = x; b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return fmaxf(a, b);
}

// Rotary table of one row, by `half` threads of the row's workgroup starting at first_thread:
// cs[i] = (cos, sin)(pos * theta^(-2i/dh)).  The angle is formed in float64 so that positions in the
// thousands keep float32-accurate sines; one table serves every layer of the pass.
__device__ __forceinline__ void rope_table_row(int pos, const double *__restrict__ inv_freq, int half,
                                               float2 *__restrict__ cs_row, int first_thread = 0) {
    const int i = (int)threadIdx.x - first_thread;
    if (i < 0 || i >= half) return;
    double s, c;
    sincos((double)pos * inv_freq[i], &s, &c);
    cs_row[i] = make_float2((float)c, (float)s);
}

// Element offsets into the paged caches.
__device__ __forceinline__ size_t k_offset(const KVCache &kv, int slot, int head, int hkv, int dh) {
    const int P = 1 << kv.page_shift;
    const int pg = kv.page_table[slot >> kv.page_shift];
    return ((size_t)(pg * hkv + head) * P + (slot & (P - 1))) * dh;
}
__device__ __forceinline__ size_t vt_offset(const KVCache &kv, int slot, int head, int hkv, int dh, int row) {
    const int P = 1 << kv.page_shift;
    const int pg = kv.page_table[slot >> kv.page_shift];
    return ((size_t)(pg * hkv + head) * dh + row) * P + (slot & (P - 1));
}

}  // namespace poss
