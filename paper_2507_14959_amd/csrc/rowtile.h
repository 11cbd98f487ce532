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
// eight such loads in a row, one wave filling a whole [64][64] bf16 tile: load g takes the per-lane byte offset voff[g]
// from the uniform base and lands at lds_byte_addr + 1024 g + 16 * lane.  Three instructions per load (the LDS
// position advances inside M0), for a wave whose only job is to keep the stream going.
__device__ __forceinline__ void glds16_tile8(const void *sbase, unsigned lds_byte_addr, unsigned v0, unsigned v1, unsigned v2, unsigned v3,
                                             unsigned v4, unsigned v5, unsigned v6, unsigned v7)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %8, %1\n\t"
                 "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %9, %1" ::"s"(lds_byte_addr),
                 "s"(sbase), "v"(v0), "v"(v1), "v"(v2), "v"(v3), "v"(v4), "v"(v5), "v"(v6), "v"(v7)
                 : "memory", "m0", "scc");
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
// row.  A thread takes the 16-byte pieces part, part + TPR, part + 2 TPR, ... of its row, so that the TPR lanes of
// a row read 16 TPR contiguous bytes per instruction (with one contiguous stretch per thread every lane of an
// instruction would touch a cache line of its own).  Rows past T repeat row T - 1: whatever is computed from
// them is never stored.  Two halves, so that the caller can put a barrier between them: ln_load requests the
// rows; ln_finish reads gain and shift from LDS (gb_s: g[K] then b[K], staged by ln_gb_load / ln_gb_store before that
// barrier -- fetching them from global memory per thread would triple the number of loads of the prologue).
template <int KT, int TPR>
__device__ __forceinline__ void ln_load(const float *xblock, int T, int t0, int tid, f32x4 (&v)[64 * KT / TPR / 4])
{
    constexpr int K = 64 * KT, NV = K / TPR / 4;
    const int row = tid / TPR, part = tid % TPR;
    const float *xr = xblock + (size_t)min(t0 + row, T - 1) * K + 4 * part;
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = *(const f32x4 *)(xr + 4 * TPR * i);
}
// gain and shift: requested early (ln_gb_load), written to LDS later by threads 0 .. K/2 - 1 (ln_gb_store)
template <int KT> __device__ __forceinline__ f32x4 ln_gb_load(const float *ln_g, const float *ln_b, int tid)
{
    // every thread loads (a load under a per-lane condition makes the compiler wait for it on the spot); the
    // threads past K/2 repeat the last piece and drop it in ln_gb_store
    constexpr int K = 64 * KT;
    const int i = min(tid, K / 2 - 1);
    const float *src = i < K / 4 ? ln_g + 4 * i : ln_b + 4 * (i - K / 4);
    return *(const f32x4 *)src;
}
template <int KT> __device__ __forceinline__ void ln_gb_store(f32x4 v, float *gb_s, int tid)
{
    if (tid < 32 * KT) *(f32x4 *)(gb_s + 4 * tid) = v;
}
// Lanes l and l + 32 each hold two 8-byte pieces p0, p1.  Returns, in lane l < 32, (own p0, the other lane's p0) and, in lane
// l + 32, (the other lane's p1, own p1): with p = four consecutive bf16 columns at offset 4 * (lane / 32) of an 8-column
// group, lane l gets all eight columns of the first group and lane l + 32 all eight of the second.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 pair_halves(bf16x4 p0, bf16x4 p1)
{
    const u32x2 a = __builtin_bit_cast(u32x2, p0), b = __builtin_bit_cast(u32x2, p1);
    // v_permlane32_swap: lanes 32-63 of the first operand trade places with lanes 0-31 of the second
    const auto r0 = __builtin_amdgcn_permlane32_swap(a[0], b[0], false, false);
    const auto r1 = __builtin_amdgcn_permlane32_swap(a[1], b[1], false, false);
    return u32x4{r0[0], r1[0], r0[1], r1[1]};
}

// sum over the TPR (4 or 8) adjacent lanes that share a row, in every one of them: data-parallel-primitive moves inside
// the quad (lane ^ 1, lane ^ 2) and across the two quads of eight lanes (mirror: every lane of a quad holds the quad's sum by
// then) -- a shuffle through the LDS crossbar costs a hundred-odd cycles per step
template <int CTRL> __device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int TPR> __device__ __forceinline__ float row_group_sum(float s)
{
    static_assert(TPR == 4 || TPR == 8, "threads per row");
    s += dpp_move<0xB1>(s);                      // quad_perm [1, 0, 3, 2]
    s += dpp_move<0x4E>(s);                      // quad_perm [2, 3, 0, 1]
    if (TPR == 8) s += dpp_move<0x141>(s);       // row_half_mirror
    return s;
}
// sum over the 16 lanes of a DPP row, in every one of them
__device__ __forceinline__ float row16_sum(float s)
{
    s += dpp_move<0xB1>(s);                      // quad_perm [1, 0, 3, 2]
    s += dpp_move<0x4E>(s);                      // quad_perm [2, 3, 0, 1]
    s += dpp_move<0x141>(s);                     // row_half_mirror: the other quad of eight lanes
    s += dpp_move<0x140>(s);                     // row_mirror: the other eight lanes
    return s;
}
template <int KT, int TPR>
__device__ __forceinline__ void ln_finish(const f32x4 (&v)[64 * KT / TPR / 4], const float *gb_s, float eps, bf16_t *As, int tid)
{
    constexpr int K = 64 * KT, NV = K / TPR / 4;
    const int row = tid / TPR, part = tid % TPR;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    s = row_group_sum<TPR>(s);
    const float mean = s * (1.0f / K);
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int z = 0; z < 4; ++z) { const float d = v[i][z] - mean; q = fmaf(d, d, q); }
    q = row_group_sum<TPR>(q);
    const float inv = rsqrtf(q * (1.0f / K) + eps), nmi = -mean * inv;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = 4 * (TPR * i + part);          // first of this piece's 4 elements
        const f32x4 g = *(const f32x4 *)(gb_s + k), b = *(const f32x4 *)(gb_s + K + k);
        bf16x4 o;
#pragma unroll
        for (int z = 0; z < 4; ++z) o[z] = (bf16_t)fmaf(fmaf(v[i][z], inv, nmi), g[z], b[z]);   // ((x - mean) inv) g + b
        // tile k / 64, 16-byte chunk (k % 64) / 8, first or second half of it
        *(bf16x4 *)(As + (k >> 6) * (64 * 64) + tile_off(row, (k & 63) >> 3) + (k & 4)) = o;
    }
}
