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
// same, address given as a uniform base (scalar registers) plus a 32-bit per-lane byte offset: no vector
// arithmetic at the point of issue
__device__ __forceinline__ void glds16_s(const void *sbase, unsigned voff, unsigned lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_addr_of(const void *p)
{
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void *)p;
}

// 4 bytes per lane, same path: lane i lands at lds_byte_addr + 4 * i
__device__ __forceinline__ void glds4(const void *gptr, unsigned lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_byte_addr), "v"(gptr) : "memory", "m0");
}

// Pull [base, base + bytes) into the L2 of the XCD this workgroup runs on, ahead of the stream that will read it.
// Every workgroup of a launch streams the same weights at about the same pace, so without this each piece of
// the stream is a first touch in its L2 and pays the latency of a miss while the LDS ring (a few pieces deep)
// runs dry.  Workgroups are dealt to the 8 XCDs round-robin; the workgroups of one XCD split the lines of the
// range among them, one 4-byte load per 128-byte line, data dumped into 256 spare bytes of LDS (dump_lds, a
// byte address).  The loads count in vmcnt like the stream's: issue them before a point that drains it.
__device__ __forceinline__ void l2_warm(const void *base, long bytes, unsigned dump_lds, int tid, int nthreads)
{
    const int xcd_wgs = ((int)gridDim.x - (int)(blockIdx.x & 7) + 7) >> 3, j = blockIdx.x >> 3;
    const long lines = (bytes + 127) >> 7;
    for (long L = (long)tid * xcd_wgs + j; L < lines; L += (long)nthreads * xcd_wgs) glds4((const char *)base + L * 128, dump_lds);
}

// LDS tile of [rows][64] bf16: 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7)
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3); }

// wait until at most N of this wave's vector-memory loads are pending (and its LDS accesses are done), then a
// bare workgroup barrier (a fenced
// __syncthreads() would wait for every pending load and so drain a stream that is meant to stay in flight)
template <int N> __device__ __forceinline__ void rl_wait_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// LayerNorm (fp32 statistics) of the 64 rows t0 .. t0 + 63 of one block of fp32 rows with K = 64 * KT elements,
// written as bf16 into KT swizzled [64][64] tiles at As.  64 * TPR threads (tid 0 .. 64 TPR - 1), TPR = 4 or 8 per
// row, K / TPR contiguous elements each; gain and shift are requested together with the rows (one latency,
// not two).  Rows past T repeat row T - 1: whatever is computed from them is never stored.
template <int KT, int TPR>
__device__ __forceinline__ void ln_rows_to_lds(const float *xblock, int T, int t0, const float *ln_g, const float *ln_b, float eps,
                                               bf16_t *As, int tid)
{
    constexpr int K = 64 * KT, PER = K / TPR, NV = PER / 4;
    const int row = tid / TPR, part = tid % TPR;
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
#pragma unroll
    for (int m = 1; m < TPR; m <<= 1) s += __shfl_xor(s, m, 64);
    const float mean = s * (1.0f / K);
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int z = 0; z < 4; ++z) { const float d = v[i][z] - mean; q = fmaf(d, d, q); }
#pragma unroll
    for (int m = 1; m < TPR; m <<= 1) q += __shfl_xor(q, m, 64);
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
