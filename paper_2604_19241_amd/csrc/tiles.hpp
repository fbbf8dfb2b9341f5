// bf16 MFMA tile machinery for gfx950 (CDNA4), shared by forward and backward.
//
// A workgroup is 4 waves (256 threads) and owns an output tile of BM = 128*FM
// rows by BN = 256 columns; wave w owns rows [w*32*FM, (w+1)*32*FM) and all 256
// columns (FM x 8 accumulators of v_mfma_f32_32x32x16_bf16, 16 fp32 each).
// Both operands are staged through LDS as [row][k] with k contiguous, 64 k per
// stage, rows padded to 144 bytes so that 16-byte fragment reads of
// consecutive rows fall in distinct banks.  Two LDS stages: global loads of
// stage s+1 are in flight while stage s feeds the matrix cores.
//
// Column mapping of the B operand: the 256 tile columns are 32 chunks of 8
// consecutive columns.  Column (chunk nb, j) lives in LDS row j*32 + nb, so B
// fragment f of lane c is column c*8 + f: after the main loop a lane holds 8
// consecutive output columns of each of its rows and stores them as one
// 16-byte vector, and a loader thread that transposed an 8x8 block writes 8
// rows that are consecutive across lanes (bank-conflict free).
#pragma once
#include "common.hpp"

namespace uniep {

constexpr int BK = 64;
constexpr int BN = 256;
constexpr int kRowBytes = (BK + 8) * 2;   // 144
constexpr int kTileThreads = 256;

template <int FM>
struct Geom {
    static constexpr int BM = 128 * FM;
    static constexpr int A_BYTES = BM * kRowBytes;
    static constexpr int B_BYTES = BN * kRowBytes;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int SMEM = 2 * STAGE;
};

// Row inside a 32-row fragment that accumulator element v of this lane holds.
__device__ __forceinline__ int frag_row(int v, int lane) {
    return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

__device__ __forceinline__ u32x4_t zero4() { return u32x4_t{0u, 0u, 0u, 0u}; }

// ------------------------------------------------------------------ loaders
// Every loader has  gload(s): fetch K-stage s into registers, and
// sstore(base): write those registers into the operand's LDS region.

// Rows with k contiguous in memory (activations).  Thread (mrow = tid/8,
// kc = tid%8) moves the 16-byte piece kc of rows mrow, mrow+32, ...: eight
// neighbouring lanes read 128 contiguous bytes of one row.  rp[p] points at
// that piece for stage 0 and must always be readable: rows beyond the tile
// alias a valid row (their products land in output rows that are never stored).
// SCALE: multiply the row by a per-row fp32 factor and round to bf16 once.
template <int NROWS32, bool SCALE>
struct RowLoader {
    const char* rp[NROWS32];
    float sc[NROWS32];
    u32x4_t reg[NROWS32];
    int lds_off;   // (tid/8)*144 + (tid%8)*16

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x >> 3) * kRowBytes + (threadIdx.x & 7) * 16;
    }
    __device__ __forceinline__ void gload(int s) {
#pragma unroll
        for (int p = 0; p < NROWS32; ++p)
            reg[p] = *(const u32x4_t*)(rp[p] + (size_t)s * (BK * 2));
    }
    __device__ __forceinline__ void sstore(char* base) {
#pragma unroll
        for (int p = 0; p < NROWS32; ++p) {
            u32x4_t r = reg[p];
            if (SCALE) {
                const float f = sc[p];
#pragma unroll
                for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(bf16_lo(r[q]) * f, bf16_hi(r[q]) * f);
            }
            *(u32x4_t*)(base + lds_off + p * 32 * kRowBytes) = r;
        }
    }
};

// 8x8 bf16 transpose in registers: in[r] = 8 consecutive columns of k-row r;
// out[j] = the 8 k-values of column j, k ascending.
__device__ __forceinline__ void transpose8x8(const u32x4_t (&in)[8], u32x4_t (&out)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t lo = in[2 * p][j >> 1], hi = in[2 * p + 1][j >> 1];
            out[j][p] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
        }
    }
}

// Operand whose k runs along memory rows (row pitch ld_bytes) and whose tile
// "rows" (the M or N index) are contiguous in memory: weights [K,N] in the
// forward pass.  Thread (kb = tid/32, nb = tid%32) fetches the 8x8 block
// k in [kb*8, kb*8+8) x chunk nb, transposes it in registers and writes 8
// LDS rows j*32 + nb.  bp = address of (k = kb*8 of stage 0, first column of
// chunk nb); chunks outside the matrix alias a valid chunk (their output
// columns are never stored).
struct StridedLoader {
    const char* bp;
    size_t ld_bytes;
    u32x4_t reg[8];
    int lds_off;   // nb*144 + kb*16

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x & 31) * kRowBytes + (threadIdx.x >> 5) * 16;
    }
    __device__ __forceinline__ void gload(int s) {
        const char* p = bp + (size_t)s * BK * ld_bytes;
#pragma unroll
        for (int r = 0; r < 8; ++r) reg[r] = *(const u32x4_t*)(p + r * ld_bytes);
    }
    __device__ __forceinline__ void sstore(char* base) {
        u32x4_t out[8];
        transpose8x8(reg, out);
#pragma unroll
        for (int j = 0; j < 8; ++j) *(u32x4_t*)(base + lds_off + j * 32 * kRowBytes) = out[j];
    }
};

// RowLoader whose k axis is the concatenation of two matrices with identical
// layout (W_gate then W_up along k): stages >= switch_stage read from the
// second matrix, which sits `delta` bytes after the first.
template <int NROWS32>
struct SplitRowLoader {
    const char* rp[NROWS32];
    u32x4_t reg[NROWS32];
    long long delta;
    int switch_stage;
    int lds_off;

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x >> 3) * kRowBytes + (threadIdx.x & 7) * 16;
    }
    __device__ __forceinline__ void gload(int s) {
        const long long off = (s < switch_stage) ? (long long)s * (BK * 2)
                                                 : delta + (long long)(s - switch_stage) * (BK * 2);
#pragma unroll
        for (int p = 0; p < NROWS32; ++p) reg[p] = *(const u32x4_t*)(rp[p] + off);
    }
    __device__ __forceinline__ void sstore(char* base) {
#pragma unroll
        for (int p = 0; p < NROWS32; ++p) *(u32x4_t*)(base + lds_off + p * 32 * kRowBytes) = reg[p];
    }
};

// StridedLoader for a reduction over K memory rows where K is not a multiple
// of 64 (the rows of one expert): rows at and beyond K are zero-filled.
// bp = address of (k = 0, first column of chunk nb).
struct StridedLoaderK {
    const char* bp;
    size_t ld_bytes;
    int K;
    u32x4_t reg[8];
    int lds_off, kb8;

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x & 31) * kRowBytes + (threadIdx.x >> 5) * 16;
        kb8 = (threadIdx.x >> 5) * 8;
    }
    __device__ __forceinline__ void gload(int s) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int k = s * BK + kb8 + r;
            const u32x4_t v = *(const u32x4_t*)(bp + (size_t)min(k, K - 1) * ld_bytes);
            reg[r] = (k < K) ? v : zero4();
        }
    }
    __device__ __forceinline__ void sstore(char* base) {
        u32x4_t out[8];
        transpose8x8(reg, out);
#pragma unroll
        for (int j = 0; j < 8; ++j) *(u32x4_t*)(base + lds_off + j * 32 * kRowBytes) = out[j];
    }
};

// The same with a gather: memory row of reduction index k is row_tok[row0+k]
// of a [T, ld] matrix (the token that sits in that expert row), optionally
// scaled by row_w[row0+k] and rounded to bf16 once (dO = gate * dY).
// src = matrix base + byte offset of the first column of chunk nb.
template <bool SCALE>
struct GatherStridedLoader {
    const char* src;
    size_t ld_bytes;
    const int32_t* row_tok;
    const float* row_w;
    int row0, K;
    u32x4_t reg[8];
    float sc[8];
    int lds_off, kb8;

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x & 31) * kRowBytes + (threadIdx.x >> 5) * 16;
        kb8 = (threadIdx.x >> 5) * 8;
    }
    __device__ __forceinline__ void gload(int s) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int k = s * BK + kb8 + r;
            const int row = row0 + min(k, K - 1);
            const int tok = row_tok[row];
            if (SCALE) sc[r] = row_w[row];
            const u32x4_t v = *(const u32x4_t*)(src + (size_t)tok * ld_bytes);
            reg[r] = (k < K) ? v : zero4();
        }
    }
    __device__ __forceinline__ void sstore(char* base) {
        if (SCALE) {
#pragma unroll
            for (int r = 0; r < 8; ++r)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    reg[r][q] = pack_bf16x2(bf16_lo(reg[r][q]) * sc[r], bf16_hi(reg[r][q]) * sc[r]);
        }
        u32x4_t out[8];
        transpose8x8(reg, out);
#pragma unroll
        for (int j = 0; j < 8; ++j) *(u32x4_t*)(base + lds_off + j * 32 * kRowBytes) = out[j];
    }
};

// ---------------------------------------------------------------- main loop
// acc[i][f] += A-fragment i  x  B-fragment f over nk stages of 64.
template <int FM, class AL, class BL>
__device__ __forceinline__ void mma_mainloop(AL& al, BL& bl, int nk, char* smem,
                                             f32x16_t (&acc)[FM][8]) {
    typedef Geom<FM> G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int f = 0; f < 8; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;
    if (nk <= 0) return;   // empty reduction (an expert without rows): the tile is all zeros

    al.gload(0);
    bl.gload(0);
    al.sstore(smem);
    bl.sstore(smem + G::A_BYTES);
    __syncthreads();
    const int a_off = (wave * FM * 32 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;
    const int b_off = G::A_BYTES + (lane & 31) * kRowBytes + (lane >> 5) * 16;
    for (int s = 0; s < nk; ++s) {
        char* cur = smem + (s & 1) * G::STAGE;
        char* nxt = smem + ((s + 1) & 1) * G::STAGE;
        const bool more = (s + 1 < nk);
        if (more) {
            al.gload(s + 1);
            bl.gload(s + 1);
        }
        // fragments of sub-step kk+1 are read while the MFMAs of kk run
        bf16x8_t a[2][FM], b[2][8];
#pragma unroll
        for (int i = 0; i < FM; ++i) a[0][i] = *(const bf16x8_t*)(cur + a_off + i * 32 * kRowBytes);
#pragma unroll
        for (int f = 0; f < 8; ++f) b[0][f] = *(const bf16x8_t*)(cur + b_off + f * 32 * kRowBytes);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int c = kk & 1, n = c ^ 1;
            __builtin_amdgcn_sched_barrier(0);
            if (kk + 1 < BK / 16) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    a[n][i] = *(const bf16x8_t*)(cur + a_off + i * 32 * kRowBytes + (kk + 1) * 32);
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    b[n][f] = *(const bf16x8_t*)(cur + b_off + f * 32 * kRowBytes + (kk + 1) * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][f], acc[i][f], 0, 0, 0);
        }
        if (more) {
            al.sstore(nxt);
            bl.sstore(nxt + G::A_BYTES);
        }
        __syncthreads();
    }
}

// Pack the 8 consecutive columns a lane holds for (fragment row i, element v).
template <int FM>
__device__ __forceinline__ u32x4_t pack_row8(const f32x16_t (&acc)[FM][8], int i, int v) {
    u32x4_t r;
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(acc[i][2 * q][v], acc[i][2 * q + 1][v]);
    return r;
}

__device__ __forceinline__ float dpp_swap_pair(float x) {   // value of lane ^ 1
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true));
}

__device__ __forceinline__ float sigmoid_f(float z) { return __frcp_rn(1.f + __expf(-z)); }

}  // namespace uniep
