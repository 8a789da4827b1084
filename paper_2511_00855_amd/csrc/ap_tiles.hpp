// Building blocks of the construction kernels: a 128x128 MFMA tile product of
// gathered dense rows, an exact radix selection of the K best keys of a row,
// and a bitonic sort of keys in LDS.
#pragma once
#include "ap_common.hpp"

#ifdef __HIPCC__
typedef float ap_f32x16 __attribute__((ext_vector_type(16)));

#define AP_TILE 128
#define AP_BK 32
#define AP_LDS_STRIDE (AP_BK + 1)   // odd stride: the 32 rows read by one MFMA operand fall in distinct banks

// Columns [k0, k0+32) of 128 rows (row id -1 = zeros) as f32: thread t holds 4 consecutive columns of rows
// t/8 + 32*pass, whose ids it keeps in row[] for the whole product.  Loading (global memory -> registers) and
// storing (registers -> lds[128][33]) are separate steps so that the loads of the next chunk can be in flight while
// the current one is multiplied.  The loads are unconditional (a hole reads row 0, a column past the end re-reads
// the row's last group) so that four loads issue back to back; what they brought is zeroed when it is stored.
template <int DT>
__device__ __forceinline__ void ap_tile_load(const void *dense, int32_t dim, const int32_t row[4], int32_t k0, float4 v[4]) {
    const int c = (threadIdx.x & 7) * 4;
    const bool inside = k0 + c < dim;              // dim is a multiple of 4: a group of 4 is all inside or all outside
    const int32_t col = inside ? k0 + c : dim - 4;
#pragma unroll
    for (int pass = 0; pass < 4; pass++) {
        const int64_t at = (int64_t)(row[pass] < 0 ? 0 : row[pass]) * dim + col;
        float4 x;
        if (DT == AP_F32) {
            x = *reinterpret_cast<const float4 *>(static_cast<const float *>(dense) + at);
        } else {
            const uint2 y = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(dense) + at);
            x = make_float4(__uint_as_float(y.x << 16), __uint_as_float(y.x & 0xffff0000u), __uint_as_float(y.y << 16),
                            __uint_as_float(y.y & 0xffff0000u));
        }
        v[pass] = x;
    }
}

// k0: the chunk v[] was loaded for.
__device__ __forceinline__ void ap_tile_store(const float4 v[4], const int32_t row[4], int32_t dim, int32_t k0, float *lds) {
    const int t = threadIdx.x;
    const bool inside = k0 + (t & 7) * 4 < dim;
#pragma unroll
    for (int pass = 0; pass < 4; pass++) {
        float *d = lds + ((t >> 3) + 32 * pass) * AP_LDS_STRIDE + (t & 7) * 4;
        const bool keep = row[pass] >= 0 && inside;
        d[0] = keep ? v[pass].x : 0.f; d[1] = keep ? v[pass].y : 0.f; d[2] = keep ? v[pass].z : 0.f; d[3] = keep ? v[pass].w : 0.f;
    }
}

// acc[a][b] (a, b in {0,1}) accumulate the 32x32 sub-tiles of this wave's
// 64x64 quadrant: rows wm*64 + a*32 .., columns wn*64 + b*32 ..
// C[i][j] = sum_k A[i][k] * B[j][k]   (both operands row-major: a Gram-type product).
// v_mfma_f32_32x32x2_f32: lane l feeds A[l%32][l/32] and B[l/32][l%32]; the
// result element (row, col) = (8*(r/4) + 4*(l/32) + r%4, l%32) sits in register r of lane l.
template <int DT>
__device__ __forceinline__ void ap_tile_gemm(const void *dense, int32_t dim, const int32_t *a_rows, const int32_t *b_rows,
                                             float *lA, float *lB, ap_f32x16 acc[2][2]) {
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[a][b][r] = 0.f;
    float4 va[4], vb[4];
    int32_t ra[4], rb[4];
    __syncthreads();                // the row lists were just written by the caller's threads
#pragma unroll
    for (int pass = 0; pass < 4; pass++) {
        ra[pass] = a_rows[(threadIdx.x >> 3) + 32 * pass];
        rb[pass] = b_rows[(threadIdx.x >> 3) + 32 * pass];
    }
    ap_tile_load<DT>(dense, dim, ra, 0, va);
    ap_tile_load<DT>(dense, dim, rb, 0, vb);
    for (int32_t k0 = 0; k0 < dim; k0 += AP_BK) {
        __syncthreads();            // everyone is done with the previous chunk in LDS
        ap_tile_store(va, ra, dim, k0, lA);
        ap_tile_store(vb, rb, dim, k0, lB);
        __syncthreads();
        if (k0 + AP_BK < dim) {     // the next chunk travels while this one is multiplied
            ap_tile_load<DT>(dense, dim, ra, k0 + AP_BK, va);
            ap_tile_load<DT>(dense, dim, rb, k0 + AP_BK, vb);
        }
        const float *pa0 = lA + (wm * 64 + li) * AP_LDS_STRIDE + lk;
        const float *pa1 = pa0 + 32 * AP_LDS_STRIDE;
        const float *pb0 = lB + (wn * 64 + li) * AP_LDS_STRIDE + lk;
        const float *pb1 = pb0 + 32 * AP_LDS_STRIDE;
#pragma unroll
        for (int kk = 0; kk < AP_BK; kk += 2) {
            const float a0 = pa0[kk], a1 = pa1[kk], b0 = pb0[kk], b1 = pb1[kk];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
}

// bf16 rows: the same 128x128 tile product on v_mfma_f32_32x32x16_bf16 (8x the
// rate of the f32 instruction).  Rows are staged as bf16, 64 columns a chunk;
// lane l feeds A[l%32][8*(l/32) .. +8] and B[8*(l/32) .. +8][l%32] per 16-wide
// step; the result layout is that of the f32 instruction.
typedef __bf16 ap_bf16x8 __attribute__((ext_vector_type(8)));
#define AP_BK16 64
#define AP_LDS_STRIDE16 (AP_BK16 + 8)   // in bf16 elements: 144-byte rows keep the 16-byte operand reads spread over the banks

// thread t holds 8 consecutive columns (16 bytes) of rows t / AP_TPR16 + AP_RPP16 * pass
#define AP_TPR16 (AP_BK16 / 8)            // threads per row of a chunk
#define AP_RPP16 (256 / AP_TPR16)         // rows per pass
#define AP_NP16 (AP_TILE / AP_RPP16)      // passes
// row[]: the ids of this thread's rows, kept in registers for the whole product; unconditional loads, zeroed when
// stored, as above.
__device__ __forceinline__ void ap_tile_load_bf16(const void *dense, int32_t dim, const int32_t row[AP_NP16], int32_t k0, uint4 v[AP_NP16]) {
    const int c = (threadIdx.x % AP_TPR16) * 8;
    const int32_t col = k0 + c < dim ? k0 + c : dim - 8;   // dim is a multiple of 8: a 16-byte group is all inside or all outside
#pragma unroll
    for (int pass = 0; pass < AP_NP16; pass++)
        v[pass] = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(dense) + (int64_t)(row[pass] < 0 ? 0 : row[pass]) * dim + col);
}

__device__ __forceinline__ void ap_tile_store_bf16(const uint4 v[AP_NP16], const int32_t row[AP_NP16], int32_t dim, int32_t k0, uint16_t *lds) {
    const int t = threadIdx.x;
    const bool inside = k0 + (t % AP_TPR16) * 8 < dim;
#pragma unroll
    for (int pass = 0; pass < AP_NP16; pass++)
        *reinterpret_cast<uint4 *>(lds + (t / AP_TPR16 + AP_RPP16 * pass) * AP_LDS_STRIDE16 + (t % AP_TPR16) * 8) =
            (row[pass] >= 0 && inside) ? v[pass] : make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ void ap_tile_gemm_bf16(const void *dense, int32_t dim, const int32_t *a_rows, const int32_t *b_rows,
                                                  uint16_t *lA, uint16_t *lB, ap_f32x16 acc[2][2]) {
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lk = (lane >> 5) * 8;
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[a][b][r] = 0.f;
    uint4 va[AP_NP16], vb[AP_NP16];
    int32_t ra[AP_NP16], rb[AP_NP16];
    __syncthreads();                // the row lists were just written by the caller's threads
#pragma unroll
    for (int pass = 0; pass < AP_NP16; pass++) {
        ra[pass] = a_rows[threadIdx.x / AP_TPR16 + AP_RPP16 * pass];
        rb[pass] = b_rows[threadIdx.x / AP_TPR16 + AP_RPP16 * pass];
    }
    ap_tile_load_bf16(dense, dim, ra, 0, va);
    ap_tile_load_bf16(dense, dim, rb, 0, vb);
    for (int32_t k0 = 0; k0 < dim; k0 += AP_BK16) {
        __syncthreads();            // everyone is done with the previous chunk in LDS
        ap_tile_store_bf16(va, ra, dim, k0, lA);
        ap_tile_store_bf16(vb, rb, dim, k0, lB);
        __syncthreads();
        if (k0 + AP_BK16 < dim) {   // the next chunk travels while this one is multiplied
            ap_tile_load_bf16(dense, dim, ra, k0 + AP_BK16, va);
            ap_tile_load_bf16(dense, dim, rb, k0 + AP_BK16, vb);
        }
        const uint16_t *pa0 = lA + (wm * 64 + li) * AP_LDS_STRIDE16 + lk;
        const uint16_t *pa1 = pa0 + 32 * AP_LDS_STRIDE16;
        const uint16_t *pb0 = lB + (wn * 64 + li) * AP_LDS_STRIDE16 + lk;
        const uint16_t *pb1 = pb0 + 32 * AP_LDS_STRIDE16;
#pragma unroll
        for (int kk = 0; kk < AP_BK16; kk += 16) {
            const ap_bf16x8 a0 = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const uint4 *>(pa0 + kk));
            const ap_bf16x8 a1 = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const uint4 *>(pa1 + kk));
            const ap_bf16x8 b0 = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const uint4 *>(pb0 + kk));
            const ap_bf16x8 b1 = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const uint4 *>(pb1 + kk));
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
}

// The large bf16 product: a 256x256 tile by WM x WN waves, each a (256/WM) x (256/WN) block of 32x32 MFMA tiles,
// twice the multiply-adds per byte fetched of the 128x128 tile, and fewer LDS reads per MFMA the larger a wave's
// block is.  Chunks of 64 columns alternate between two LDS stages, so a chunk costs one barrier: while chunk k is
// multiplied out of one stage, chunk k+1 (already in registers) is written to the other and chunks k+2 and k+3 are
// on their way from memory.  Same instruction, operand layout and chunk order as the 128x128 product: every element
// gets the same bits.
#define AP_BIG 256
#define AP_BIG_STAGE (2 * AP_BIG * AP_LDS_STRIDE16)               // bf16 elements of one stage (A then B)
#define AP_BIG_LDS_BYTES (2 * AP_BIG_STAGE * 2)
typedef uint32_t ap_u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte group as a plain vector value
template <int WM, int WN> struct ApBig {
    static constexpr int THREADS = WM * WN * 64;
    static constexpr int NP = AP_BIG * AP_TPR16 / THREADS;        // 16-byte groups per thread, operand and chunk
    static constexpr int RPP = THREADS / AP_TPR16;                // rows per pass of the staging
    static constexpr int FA = AP_BIG / WM / 32, FB = AP_BIG / WN / 32;   // 32x32 tiles of a wave's block
};
template <int NP>
__device__ __forceinline__ void ap_big_load(const void *dense, int32_t dim, const int32_t row[NP], int32_t k0, ap_u32x4 v[NP]) {
    const int c = (threadIdx.x % AP_TPR16) * 8;
    const int32_t col = k0 + c < dim ? k0 + c : dim - 8;
#pragma unroll
    for (int pass = 0; pass < NP; pass++)
        v[pass] = *reinterpret_cast<const ap_u32x4 *>(static_cast<const uint16_t *>(dense) + (int64_t)(row[pass] < 0 ? 0 : row[pass]) * dim + col);
}
template <int NP, int RPP>
__device__ __forceinline__ void ap_big_store(const ap_u32x4 v[NP], const int32_t row[NP], int32_t dim, int32_t k0, uint16_t *lds) {
    const int t = threadIdx.x;
    const bool inside = k0 + (t % AP_TPR16) * 8 < dim;
#pragma unroll
    for (int pass = 0; pass < NP; pass++)
        *reinterpret_cast<ap_u32x4 *>(lds + (t / AP_TPR16 + RPP * pass) * AP_LDS_STRIDE16 + (t % AP_TPR16) * 8) =
            (row[pass] >= 0 && inside) ? v[pass] : ap_u32x4{0u, 0u, 0u, 0u};
}
template <int NP, int RPP>
__device__ __forceinline__ void ap_big_load_run(const char *run, uint32_t off0, uint32_t pass_stride, int32_t k0, ap_u32x4 (&v)[NP]) {
#pragma unroll
    for (int pass = 0; pass < NP; pass++) v[pass] = *reinterpret_cast<const ap_u32x4 *>(run + (off0 + pass * pass_stride + (uint32_t)k0 * 2u));
}
template <int NP, int RPP>
__device__ __forceinline__ void ap_big_store_run(const ap_u32x4 (&v)[NP], uint16_t *lds) {
#pragma unroll
    for (int pass = 0; pass < NP; pass++)
        *reinterpret_cast<ap_u32x4 *>(lds + (threadIdx.x / AP_TPR16 + RPP * pass) * AP_LDS_STRIDE16 + (threadIdx.x % AP_TPR16) * 8) = v[pass];
}
#define AP_BIG_LOAD(run, row, k0, v)                                  \
    do {                                                              \
        if constexpr (RUN) ap_big_load_run<NP, RPP>(run, run_off, run_stride, k0, v); \
        else ap_big_load<NP>(dense, dim, row, k0, v);                 \
    } while (0)
#define AP_BIG_STORE(v, row, k0, to)                                  \
    do {                                                              \
        if constexpr (RUN) ap_big_store_run<NP, RPP>(v, to);          \
        else ap_big_store<NP, RPP>(v, row, dim, k0, to);              \
    } while (0)
// RUN: both operands are runs of 256 consecutive documents (first ids a_first / b_first; a_rows / b_rows unused), all
// inside the corpus, and dim is a multiple of 64 -- the case of every tile of a sweep but those on its edges.  Then an
// address is a uniform base plus a 32-bit offset that is fixed for the whole product, nothing needs zeroing, and a
// chunk costs no vector instruction besides its loads, stores and MFMAs.
template <int WM, int WN, bool RUN>
__device__ __forceinline__ void ap_big_gemm_bf16(const void *dense, int32_t dim, const int32_t *a_rows, const int32_t *b_rows,
                                                 int32_t a_first, int32_t b_first, uint16_t *lds,
                                                 ap_f32x16 acc[ApBig<WM, WN>::FA][ApBig<WM, WN>::FB]) {
    using B = ApBig<WM, WN>;
    constexpr int NP = B::NP, RPP = B::RPP, FA = B::FA, FB = B::FB;
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lk = (lane >> 5) * 8;
    const char *run_a = static_cast<const char *>(dense) + (int64_t)a_first * dim * 2;   // uniform
    const char *run_b = static_cast<const char *>(dense) + (int64_t)b_first * dim * 2;
    const uint32_t run_off = (uint32_t)(threadIdx.x / AP_TPR16) * (uint32_t)dim * 2u + (threadIdx.x % AP_TPR16) * 16u;
    const uint32_t run_stride = (uint32_t)RPP * (uint32_t)dim * 2u;   // from one of a thread's rows to the next (uniform)
#pragma unroll
    for (int a = 0; a < FA; a++)
#pragma unroll
        for (int b = 0; b < FB; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[a][b][r] = 0.f;
    ap_u32x4 va0[NP], vb0[NP], va1[NP], vb1[NP];   // two chunks on their way from memory
    int32_t ra[NP], rb[NP];
    __syncthreads();                // the row lists were just written by the caller's threads
#pragma unroll
    for (int pass = 0; pass < NP; pass++) {
        ra[pass] = RUN ? 0 : a_rows[threadIdx.x / AP_TPR16 + RPP * pass];
        rb[pass] = RUN ? 0 : b_rows[threadIdx.x / AP_TPR16 + RPP * pass];
    }
    const int32_t nch = (dim + AP_BK16 - 1) / AP_BK16;
    AP_BIG_LOAD(run_a, ra, 0, va0);
    AP_BIG_LOAD(run_b, rb, 0, vb0);
    AP_BIG_STORE(va0, ra, 0, lds);
    AP_BIG_STORE(vb0, rb, 0, lds + AP_BIG * AP_LDS_STRIDE16);
    if (nch > 1) {
        AP_BIG_LOAD(run_a, ra, AP_BK16, va0);
        AP_BIG_LOAD(run_b, rb, AP_BK16, vb0);
    }
    if (nch > 2) {
        AP_BIG_LOAD(run_a, ra, 2 * AP_BK16, va1);
        AP_BIG_LOAD(run_b, rb, 2 * AP_BK16, vb1);
    }
    __syncthreads();
    // Round k multiplies chunk k out of stage k & 1.  Register set k & 1 holds chunk k+1: it goes to the other stage
    // (last read before the barrier that ended round k-1) and is then filled with chunk k+3, so two chunks travel
    // while two are multiplied.
#define AP_BIG_ROUND(k, sa, sb)                                                                                                                       \
    do {                                                                                                                                              \
        uint16_t *cur = lds + ((k) & 1) * AP_BIG_STAGE, *nxt = lds + (((k) + 1) & 1) * AP_BIG_STAGE;                                                  \
        if ((k) + 1 < nch) {                                                                                                                          \
            AP_BIG_STORE(sa, ra, ((k) + 1) * AP_BK16, nxt);                                                                                           \
            AP_BIG_STORE(sb, rb, ((k) + 1) * AP_BK16, nxt + AP_BIG * AP_LDS_STRIDE16);                                                                \
        }                                                                                                                                             \
        if ((k) + 3 < nch) {                                                                                                                          \
            AP_BIG_LOAD(run_a, ra, ((k) + 3) * AP_BK16, sa);                                                                                          \
            AP_BIG_LOAD(run_b, rb, ((k) + 3) * AP_BK16, sb);                                                                                          \
        }                                                                                                                                             \
        const uint16_t *pa = cur + (wm * (AP_BIG / WM) + li) * AP_LDS_STRIDE16 + lk;                                                                  \
        const uint16_t *pb = cur + AP_BIG * AP_LDS_STRIDE16 + (wn * (AP_BIG / WN) + li) * AP_LDS_STRIDE16 + lk;                                       \
_Pragma("unroll")                                                                                                                                     \
        for (int kk = 0; kk < AP_BK16; kk += 16) {                                                                                                    \
            ap_bf16x8 fa[FA], fb[FB];                                                                                                                 \
_Pragma("unroll")                                                                                                                                     \
            for (int a = 0; a < FA; a++) fa[a] = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const ap_u32x4 *>(pa + a * 32 * AP_LDS_STRIDE16 + kk)); \
_Pragma("unroll")                                                                                                                                     \
            for (int b = 0; b < FB; b++) fb[b] = __builtin_bit_cast(ap_bf16x8, *reinterpret_cast<const ap_u32x4 *>(pb + b * 32 * AP_LDS_STRIDE16 + kk)); \
_Pragma("unroll")                                                                                                                                     \
            for (int a = 0; a < FA; a++)                                                                                                              \
_Pragma("unroll")                                                                                                                                     \
                for (int b = 0; b < FB; b++) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);                   \
        }                                                                                                                                             \
        __syncthreads();                                                                                                                              \
    } while (0)

    for (int32_t k = 0; k < nch; k += 2) {
        AP_BIG_ROUND(k, va0, vb0);
        if (k + 1 < nch) AP_BIG_ROUND(k + 1, va1, vb1);
    }
#undef AP_BIG_ROUND
}
#undef AP_BIG_LOAD
#undef AP_BIG_STORE

// Calls f(i, j, value) for every element this lane holds of the 256x256 tile.
template <int WM, int WN, typename F>
__device__ __forceinline__ void ap_big_foreach(const ap_f32x16 acc[ApBig<WM, WN>::FA][ApBig<WM, WN>::FB], F f) {
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int wm = wave / WN, wn = wave % WN;
#pragma unroll
    for (int a = 0; a < ApBig<WM, WN>::FA; a++)
#pragma unroll
        for (int b = 0; b < ApBig<WM, WN>::FB; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int i = wm * (AP_BIG / WM) + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int j = wn * (AP_BIG / WN) + b * 32 + (lane & 31);
                f(i, j, acc[a][b][r]);
            }
}

// LDS bytes the tile product needs (both operands) for a storage type.
template <int DT> struct ApTileLds {
    static constexpr int BYTES = DT == AP_BF16 ? 2 * AP_TILE * AP_LDS_STRIDE16 * 2 : 2 * AP_TILE * AP_LDS_STRIDE * 4;
};

// Tile product for storage type DT out of one raw LDS area of ApTileLds<DT>::BYTES bytes.
template <int DT>
__device__ __forceinline__ void ap_tile_product(const void *dense, int32_t dim, const int32_t *a_rows, const int32_t *b_rows,
                                                void *lds, ap_f32x16 acc[2][2]) {
    if (DT == AP_BF16) {
        uint16_t *l = static_cast<uint16_t *>(lds);
        ap_tile_gemm_bf16(dense, dim, a_rows, b_rows, l, l + AP_TILE * AP_LDS_STRIDE16, acc);
    } else {
        float *l = static_cast<float *>(lds);
        ap_tile_gemm<AP_F32>(dense, dim, a_rows, b_rows, l, l + AP_TILE * AP_LDS_STRIDE, acc);
    }
}

// Calls f(i, j, value) for every element this lane holds of the 128x128 tile.
template <typename F>
__device__ __forceinline__ void ap_tile_foreach(const ap_f32x16 acc[2][2], F f) {
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int i = wm * 64 + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int j = wn * 64 + b * 32 + (lane & 31);
                f(i, j, acc[a][b][r]);
            }
}

// Sorts keys[0..n) (n a power of two, <= 2*blockDim.x) in LDS, descending.
__device__ __forceinline__ void ap_bitonic_desc(uint64_t *keys, int32_t n) {
    for (int32_t size = 2; size <= n; size <<= 1)
        for (int32_t stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int32_t t = threadIdx.x; t < (n >> 1); t += blockDim.x) {
                const int32_t lo = 2 * t - (t & (stride - 1));
                const int32_t hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
        }
    __syncthreads();
}

// Exact selection of the K largest of the n keys key_of(j), j in [0, n) (a key
// of 0 means "no candidate here"): radix selection on the 64-bit keys, eight
// bits a pass from the top, stopping as soon as the digit bucket that holds
// the K-th key is taken whole.  The selected keys land in sel[] (unordered);
// returns their number (min(K, number of non-zero keys)).  `valid` = number of
// non-zero keys, known to the caller.  hist: 256 words of LDS.
template <typename KeyOf>
__device__ __forceinline__ int32_t ap_radix_select_keys(KeyOf key_of, int64_t n, int64_t valid, int32_t K, uint32_t *hist,
                                                        uint64_t *sel, int32_t *s_misc /* 4 ints */, uint64_t *s_prefix /* 1 */) {
    int32_t krem = (int64_t)K < valid ? K : (int32_t)valid;
    const int32_t ktotal = krem;
    uint64_t prefix = 0, mask = 0;
    if (ktotal > 0 && (int64_t)ktotal < valid) {
        for (int pass = 0; pass < 8; pass++) {
            const int shift = 56 - 8 * pass;
            for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
            __syncthreads();
            for (int64_t j = threadIdx.x; j < n; j += blockDim.x) {
                const uint64_t key = key_of(j);
                if (key != 0 && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                int32_t cum = 0, b = 255;
                for (; b > 0; b--) {
                    if (cum + (int32_t)hist[b] >= krem) break;
                    cum += (int32_t)hist[b];
                }
                s_misc[0] = krem - cum;
                s_misc[1] = ((int32_t)hist[b] == krem - cum) ? 1 : 0;
                *s_prefix = prefix | ((uint64_t)b << shift);
            }
            __syncthreads();
            krem = s_misc[0];
            prefix = *s_prefix;
            mask |= 0xffull << shift;
            const int done = s_misc[1];
            __syncthreads();
            if (done) break;
        }
    }
    if (threadIdx.x == 0) s_misc[2] = 0;
    __syncthreads();
    if (ktotal > 0) {
        for (int64_t j = threadIdx.x; j < n; j += blockDim.x) {
            const uint64_t key = key_of(j);
            if (key != 0 && (key & mask) >= prefix) {
                const int32_t pos = atomicAdd(&s_misc[2], 1);
                if (pos < ktotal) sel[pos] = key;
            }
        }
    }
    __syncthreads();
    return ktotal;
}

// The K best of a row of scores: key(j) = ap_make_key(row[j], j), j != exclude.
__device__ __forceinline__ int32_t ap_radix_select(const float *row, int64_t n, int32_t exclude, int32_t K,
                                                   uint32_t *hist, uint64_t *sel, int32_t *s_misc, uint64_t *s_prefix) {
    const int64_t valid = n - ((exclude >= 0 && exclude < n) ? 1 : 0);
    return ap_radix_select_keys([&](int64_t j) -> uint64_t { return j == exclude ? 0ull : ap_make_key(row[j], (int32_t)j, 1u); },
                                n, valid, K, hist, sel, s_misc, s_prefix);
}

#endif
