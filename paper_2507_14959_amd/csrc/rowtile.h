// Building blocks shared by the kernels that keep a tile of 64 token rows on chip (rowlin.hip, mlp.hip).
#pragma once
#include "poly_dev.h"

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_byte_addr + 16 * i.  Issued as
// inline assembly on purpose: when the compiler sees LDS-bound loads it makes every later LDS read wait for
// all of them (it cannot tell the ring stages apart), which would serialise the W stream below.  The waits are
// counted by hand instead; a compiler-inserted vmcnt wait that does not know about these loads can only be
// stricter than intended, never too weak, because loads complete in issue order.
__device__ __forceinline__ void glds16(const void *gptr, unsigned lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte_addr), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_addr_of(const void *p)
{
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void *)p;
}

// LDS tile of [rows][64] bf16: 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7)
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3); }

// wait until at most N of this wave's vector-memory loads are pending, then a bare workgroup barrier (a fenced
// __syncthreads() would wait for every pending load and so drain a stream that is meant to stay in flight)
template <int N> __device__ __forceinline__ void rl_wait_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// LayerNorm (fp32 statistics) of the 64 rows t0 .. t0 + 63 of one block of fp32 rows with K = 64 * KT elements,
// written as bf16 into KT swizzled [64][64] tiles at As.  512 threads, 8 per row, K / 8 contiguous elements
// each; gain and shift are requested together with the rows (one latency, not two).  Rows past T repeat row
// T - 1: whatever is computed from them is never stored.
template <int KT>
__device__ __forceinline__ void ln_rows_to_lds(const float *xblock, int T, int t0, const float *ln_g, const float *ln_b, float eps,
                                               bf16_t *As, int tid)
{
    constexpr int K = 64 * KT, PER = K / 8, NV = PER / 4;
    const int row = tid >> 3, part = tid & 7;
    const float *xr = xblock + (size_t)min(t0 + row, T - 1) * K + part * PER;
    const float *gp = ln_g + part * PER, *bp = ln_b + part * PER;
    f32x4 v[NV], gv[NV], bv[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = *(const f32x4 *)(xr + 4 * i);
#pragma unroll
    for (int i = 0; i < NV; ++i) { gv[i] = *(const f32x4 *)(gp + 4 * i); bv[i] = *(const f32x4 *)(bp + 4 * i); }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    s += __shfl_xor(s, 1, 64); s += __shfl_xor(s, 2, 64); s += __shfl_xor(s, 4, 64);
    const float mean = s * (1.0f / K);
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int z = 0; z < 4; ++z) { const float d = v[i][z] - mean; q = fmaf(d, d, q); }
    q += __shfl_xor(q, 1, 64); q += __shfl_xor(q, 2, 64); q += __shfl_xor(q, 4, 64);
    const float inv = rsqrtf(q * (1.0f / K) + eps);
#pragma unroll
    for (int c = 0; c < PER / 8; ++c) {
        bf16x8 o;
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            o[z] = (bf16_t)((v[2 * c][z] - mean) * inv * gv[2 * c][z] + bv[2 * c][z]);
            o[4 + z] = (bf16_t)((v[2 * c + 1][z] - mean) * inv * gv[2 * c + 1][z] + bv[2 * c + 1][z]);
        }
        const int k = part * PER + 8 * c;   // first of 8 consecutive k: tile k / 64, chunk (k % 64) / 8
        *(bf16x8 *)(As + (k >> 6) * (64 * 64) + tile_off(row, (k & 63) >> 3)) = o;
    }
}
