// bf16 MFMA tile machinery for gfx950 (CDNA4), shared by forward and backward.
//
// A workgroup is NW waves (NW = 8: two waves per SIMD, or NW = 4) and owns an
// output tile of BM = 32*NW rows by BN = 256 columns; wave w owns rows
// [32w, 32w+32) and all 256 columns: 8 accumulators of
// v_mfma_f32_32x32x16_bf16 (16 fp32 each, kept in AGPRs).  With NW = 8 the two
// waves of a SIMD hide each other's LDS and global latency.
// The B operand (and, in the weight-gradient GEMMs, the A operand too) is staged
// through LDS as [row][k] with k contiguous, 64 k per stage, rows padded to
// 144 bytes so that the 16-byte fragment reads of consecutive rows fall in
// distinct banks; the A operand of the row-tile GEMMs goes straight from global
// memory into registers (DirectRowLoader).  Two LDS stages: global loads of
// stage s+1 are in flight while stage s feeds the matrix cores.
//
// Column mapping of the B operand: the 256 tile columns are 32 chunks of 8
// consecutive columns.  Column (chunk nb, j) lives in LDS row j*32 + nb, so B
// fragment f of lane c is column c*8 + f: after the main loop a lane holds 8
// consecutive output columns of each of its rows and stores them as one
// 16-byte vector, and a loader thread that transposed a block of k-rows x 8
// columns writes LDS rows that are consecutive across lanes (conflict free).
#pragma once
#include "common.hpp"

namespace uniep {

constexpr int BK = 64;
constexpr int BN = 256;
constexpr int kRowBytes = (BK + 8) * 2;   // 144

template <int NW>
struct Geom {
    static constexpr int NT = 64 * NW;        // threads
    static constexpr int BM = 32 * NW;        // tile rows
    static constexpr int A_BYTES = BM * kRowBytes;
    static constexpr int B_BYTES = BN * kRowBytes;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    // NW = 8: one workgroup per CU with two LDS stages.  NW = 4: one LDS stage (55 KB) so that
    // two workgroups share a CU and each hides the other's barriers, prologue and epilogue.
    static constexpr int NSTAGE = (NW == 8) ? 2 : 1;
    static constexpr int SMEM = (NSTAGE * STAGE > 2 * B_BYTES) ? NSTAGE * STAGE : 2 * B_BYTES;
    static constexpr int WAVES_PER_SIMD = 2;
};

// Row inside a 32-row fragment that accumulator element v of this lane holds.
__device__ __forceinline__ int frag_row(int v, int lane) {
    return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

__device__ __forceinline__ u32x4_t zero4() { return u32x4_t{0u, 0u, 0u, 0u}; }

// ------------------------------------------------------------------ loaders
// Every loader has  gload(s): fetch K-stage s into registers, and
// sstore(base): write those registers into the operand's LDS region.

// Rows with k contiguous in memory.  Thread (tid/8, tid%8) moves the 16-byte
// piece tid%8 of LDS rows tid/8 + p*NT/8: eight neighbouring lanes read 128
// contiguous bytes of one row.  rp[p] points at that piece for stage 0 and must
// always be readable: rows beyond the tile alias a valid row (their products
// land in outputs that are never stored).
// SCALE: multiply the row by a per-row fp32 factor and round to bf16 once.
template <int NT, int NROWS, bool SCALE>
struct RowLoader {
    static constexpr bool kNeedsPrime = false;
    __device__ __forceinline__ void prime() {}
    static constexpr int RPP = NT / 8;         // rows per pass
    static constexpr int NP = NROWS / RPP;     // passes
    const char* rp[NP];
    float sc[NP];
    u32x4_t reg[NP];
    int lds_off;

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x >> 3) * kRowBytes + (threadIdx.x & 7) * 16;
    }
    // LDS row that pass p of this thread fills
    static __device__ __forceinline__ int row(int p) { return (threadIdx.x >> 3) + p * RPP; }
    // The whole stage moves in part 0, right behind the stage barrier: measured faster than
    // a quarter of it ahead of every k-sub-step.
    __device__ __forceinline__ void gload_part(int s, int part) {
        if (part != 0) return;
#pragma unroll
        for (int p = 0; p < NP; ++p)
            reg[p] = *(const u32x4_t*)(rp[p] + (size_t)s * (BK * 2));
    }
    __device__ __forceinline__ void sstore_part(char* base, int part) {
        if (part != 0) return;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            u32x4_t r = reg[p];
            if (SCALE) {
                const float f = sc[p];
#pragma unroll
                for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(bf16_lo(r[q]) * f, bf16_hi(r[q]) * f);
            }
            *(u32x4_t*)(base + lds_off + p * RPP * kRowBytes) = r;
        }
    }
};

// RowLoader whose k axis is the concatenation of two matrices with identical
// layout (W_gate then W_up along k): stages >= switch_stage read from the
// second matrix, which sits `delta` bytes after the first.
template <int NT, int NROWS>
struct SplitRowLoader {
    static constexpr bool kNeedsPrime = false;
    __device__ __forceinline__ void prime() {}
    static constexpr int RPP = NT / 8;
    static constexpr int NP = NROWS / RPP;
    const char* rp[NP];
    u32x4_t reg[NP];
    long long delta;
    int switch_stage;
    int lds_off;

    __device__ __forceinline__ void init() {
        lds_off = (threadIdx.x >> 3) * kRowBytes + (threadIdx.x & 7) * 16;
    }
    static __device__ __forceinline__ int row(int p) { return (threadIdx.x >> 3) + p * RPP; }
    __device__ __forceinline__ void gload_part(int s, int part) {
        const long long off = (s < switch_stage) ? (long long)s * (BK * 2)
                                                 : delta + (long long)(s - switch_stage) * (BK * 2);
        if (part != 0) return;
#pragma unroll
        for (int p = 0; p < NP; ++p) reg[p] = *(const u32x4_t*)(rp[p] + off);
    }
    __device__ __forceinline__ void sstore_part(char* base, int part) {
        if (part != 0) return;
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *(u32x4_t*)(base + lds_off + p * RPP * kRowBytes) = reg[p];
    }
};

// Transposing loaders: the operand's k runs along memory rows and its tile
// rows (the M or N index) are contiguous in memory, e.g. weights [K,N] in the
// forward pass.  The tile has NCH chunks of 8 consecutive tile rows; thread
// (kq = tid / NCH, chunk = tid % NCH) fetches KR = 64*NCH/NT consecutive k-rows
// of its chunk (16 bytes each), transposes the KR x 8 block in registers and
// writes, for j = 0..7, the KR k-values of tile row chunk*8 + j to LDS row
// j*NCH + chunk.  Chunks outside the matrix alias a valid chunk.
template <int KR>
__device__ __forceinline__ void transpose_store(const u32x4_t (&in)[KR], char* dst, int row_stride) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int p = 0; p < KR / 2; ++p) {
            const uint32_t lo = in[2 * p][j >> 1], hi = in[2 * p + 1][j >> 1];
            // one byte permute per word: {lo.hi16, hi.hi16} or {lo.lo16, hi.lo16}
            o[p] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        char* d = dst + j * row_stride;
        if (KR == 8) *(u32x4_t*)d = u32x4_t{o[0], o[1], o[2], o[3]};
        else if (KR == 4) *(u32x2_t*)d = u32x2_t{o[0], o[1]};
        else *(uint32_t*)d = o[0];
    }
}

template <int NT, int NCH>
struct TrGeom {
    static constexpr int KQ = NT / NCH;    // threads along k
    static constexpr int KR = BK / KQ;     // k-rows per thread
    static_assert(KR == 8 || KR == 4 || KR == 2, "unsupported transposing loader shape");
    static __device__ __forceinline__ int chunk() { return threadIdx.x % NCH; }
    static __device__ __forceinline__ int k0() { return (threadIdx.x / NCH) * KR; }
    static __device__ __forceinline__ int lds_off() { return chunk() * kRowBytes + k0() * 2; }
};

// Dense matrix, K a multiple of 64.  bp = address of (k = k0() of stage 0,
// first element of this thread's chunk).
template <int NT, int NCH>
struct StridedLoader {
    typedef TrGeom<NT, NCH> TG;
    static constexpr bool kNeedsPrime = false;
    __device__ __forceinline__ void prime() {}
    const char* bp;
    size_t ld_bytes;
    u32x4_t reg[TG::KR];
    int lds_off;

    __device__ __forceinline__ void init() { lds_off = TG::lds_off(); }
    // the transpose needs all k-rows of the block: the whole stage moves in part 0
    __device__ __forceinline__ void gload_part(int s, int part) {
        if (part != 0) return;
        const char* p = bp + (size_t)s * BK * ld_bytes;
#pragma unroll
        for (int r = 0; r < TG::KR; ++r) reg[r] = *(const u32x4_t*)(p + r * ld_bytes);
    }
    __device__ __forceinline__ void sstore_part(char* base, int part) {
        if (part != 0) return;
        transpose_store<TG::KR>(reg, base + lds_off, NCH * kRowBytes);
    }
};

// Reduction over K memory rows where K is not a multiple of 64 (the rows of one
// expert): k-rows at and beyond K are zero-filled.  bp = address of (k = 0,
// first element of this thread's chunk).
template <int NT, int NCH>
struct StridedLoaderK {
    typedef TrGeom<NT, NCH> TG;
    static constexpr bool kNeedsPrime = false;
    __device__ __forceinline__ void prime() {}
    const char* bp;
    size_t ld_bytes;
    int K;
    u32x4_t reg[TG::KR];
    int lds_off, k0;

    __device__ __forceinline__ void init() { lds_off = TG::lds_off(); k0 = TG::k0(); }
    __device__ __forceinline__ void gload_part(int s, int part) {
        if (part != 0) return;
#pragma unroll
        for (int r = 0; r < TG::KR; ++r) {
            const int k = s * BK + k0 + r;
            const u32x4_t v = *(const u32x4_t*)(bp + (size_t)min(k, K - 1) * ld_bytes);
            reg[r] = (k < K) ? v : zero4();
        }
    }
    __device__ __forceinline__ void sstore_part(char* base, int part) {
        if (part != 0) return;
        transpose_store<TG::KR>(reg, base + lds_off, NCH * kRowBytes);
    }
};

// The same with a gather: memory row of reduction index k is row_tok[row0+k]
// of a [T, ld] matrix (the token that sits in that expert row), optionally
// scaled by row_w[row0+k] and rounded to bf16 once (dO = gate * dY).
// src = matrix base + byte offset of the first element of this thread's chunk.
//
// The tokens and gates of a stage's 64 rows are the same for every thread that
// loads from those rows, and a vector-memory instruction per row and thread
// costs more issue time than the data loads themselves.  So one wave fetches
// them (one row per lane, two stages ahead of their use) and hands them to the
// workgroup through a ring of kIdxRing stages in LDS, from which every thread
// reads its KR consecutive entries with one LDS read per array.
// Protocol: prime() fills ring slots 0..3 with stages 0..3 (threads 0..255, one
// stage per 64 threads) and leaves stage 4 in the first wave's registers; the
// caller then runs a workgroup barrier.  gload_part(s, 0) with s >= 2, which the
// main loop calls once per stage ahead of that stage's barrier, writes the held
// stage to its slot and fetches the next one; the entries a thread reads for
// stage s were therefore written at least two barriers earlier.  Row indices are
// clamped to the expert's last row, so stages past the end stay readable.
constexpr int kIdxRing = 8;
constexpr int kIdxRingBytes = kIdxRing * BK * 8;   // tokens (int32) then gates (fp32)

template <int NT, int NCH, bool SCALE>
struct GatherStridedLoader {
    typedef TrGeom<NT, NCH> TG;
    static_assert(TG::KR % 4 == 0, "the index ring is read four entries at a time");
    static constexpr bool kNeedsPrime = true;
    const char* src;
    size_t ld_bytes;
    const int32_t* row_tok;
    const float* row_w;
    int row0, K;
    char* ring;        // LDS, kIdxRingBytes
    u32x4_t reg[TG::KR];
    float sc[TG::KR];
    int32_t held_tok;  // first wave: entry `lane` of stage held_stage
    float held_w;
    int held_stage;
    int lds_off, k0;

    __device__ __forceinline__ void init() {
        lds_off = TG::lds_off();
        k0 = TG::k0();
    }
    __device__ __forceinline__ int32_t* ring_tok(int s) const {
        return (int32_t*)(ring + (s & (kIdxRing - 1)) * BK * 4);
    }
    __device__ __forceinline__ float* ring_w(int s) const {
        return (float*)(ring + kIdxRing * BK * 4 + (s & (kIdxRing - 1)) * BK * 4);
    }
    __device__ __forceinline__ void fetch_held(int s) {   // first wave only
        const int row = row0 + min(s * BK + (int)(threadIdx.x & 63), K - 1);
        held_tok = row_tok[row];
        if (SCALE) held_w = row_w[row];
        held_stage = s;
    }
    __device__ __forceinline__ void prime() {
        const int tid = threadIdx.x;
        if (tid < 256) {
            const int s = tid >> 6, l = tid & 63;
            const int row = row0 + min(s * BK + l, K - 1);
            ring_tok(s)[l] = row_tok[row];
            if (SCALE) ring_w(s)[l] = row_w[row];
        }
        if (tid < 64) fetch_held(4);
    }
    __device__ __forceinline__ void gload_part(int s, int part) {
        if (part != 0) return;
        if (s >= 2 && threadIdx.x < 64) {   // wave-uniform
            ring_tok(held_stage)[threadIdx.x] = held_tok;
            if (SCALE) ring_w(held_stage)[threadIdx.x] = held_w;
            fetch_held(held_stage + 1);
        }
        int32_t tok[TG::KR];
#pragma unroll
        for (int r = 0; r < TG::KR; r += 4) {
            const u32x4_t t4 = *(const u32x4_t*)(ring_tok(s) + k0 + r);
#pragma unroll
            for (int q = 0; q < 4; ++q) tok[r + q] = (int32_t)t4[q];
            if (SCALE) {
                const u32x4_t w4 = *(const u32x4_t*)(ring_w(s) + k0 + r);
#pragma unroll
                for (int q = 0; q < 4; ++q) sc[r + q] = __uint_as_float(w4[q]);
            }
        }
#pragma unroll
        for (int r = 0; r < TG::KR; ++r) {
            const int k = s * BK + k0 + r;
            const u32x4_t v = *(const u32x4_t*)(src + (size_t)tok[r] * ld_bytes);
            reg[r] = (k < K) ? v : zero4();
        }
    }
    __device__ __forceinline__ void sstore_part(char* base, int part) {
        if (part != 0) return;
        if (SCALE) {
#pragma unroll
            for (int r = 0; r < TG::KR; ++r)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    reg[r][q] = pack_bf16x2(bf16_lo(reg[r][q]) * sc[r], bf16_hi(reg[r][q]) * sc[r]);
        }
        transpose_store<TG::KR>(reg, base + lds_off, NCH * kRowBytes);
    }
};

// Tile row (0..32*NW) that LDS row rho of an A operand staged by a transposing
// loader with NCH = 4*NW chunks holds: LDS row j*NCH + chunk <-> chunk*8 + j.
template <int NW>
__device__ __forceinline__ int tr_tile_row(int rho) {
    return (rho % (4 * NW)) * 8 + rho / (4 * NW);
}

// ---------------------------------------------------------------- main loop
// acc[f] += A-fragment (this wave's 32 rows) x B-fragment f over nk stages.
//
// Pipeline: while stage t is multiplied out of LDS buffer t%2, the registers
// that hold stage t+1 (fetched during stage t-1) are written to the other
// buffer and immediately refilled with stage t+2, right behind the stage
// barrier (the loaders take a part index 0..3, one per k-sub-step, and all of
// them move the whole stage in part 0: spreading it over the sub-steps measured
// slower), so every load has a whole stage of matrix work to arrive and every
// LDS write a whole stage before the barrier that publishes it.  One barrier per
// stage.  Stage indices past the end are clamped (a harmless re-read; the
// extra LDS image is never consumed).
// `active` = false lets a wave whose rows are all outside the tile skip the
// matrix work while still taking part in the loads and barriers.
template <int NW, class AL, class BL>
__device__ __forceinline__ void mma_mainloop(AL& al, BL& bl, int nk, char* smem, bool active,
                                             f32x16_t (&acc)[8]) {
    typedef Geom<NW> G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
    if (nk <= 0) return;   // empty reduction (an expert without rows): the tile is all zeros
    // wave-uniform, so the branch below is a scalar branch
    const bool active_u = __builtin_amdgcn_readfirstlane((int)active) != 0;
    al.prime();
    bl.prime();
    if (AL::kNeedsPrime || BL::kNeedsPrime) __syncthreads();

#pragma unroll
    for (int part = 0; part < 4; ++part) {
        al.gload_part(0, part);
        bl.gload_part(0, part);
    }
#pragma unroll
    for (int part = 0; part < 4; ++part) {
        al.sstore_part(smem, part);
        bl.sstore_part(smem + G::A_BYTES, part);
    }
    const int s1 = min(1, nk - 1);
#pragma unroll
    for (int part = 0; part < 4; ++part) {
        al.gload_part(s1, part);
        bl.gload_part(s1, part);
    }
    __syncthreads();
    const int a_off = (wave * 32 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;
    const int b_off = G::A_BYTES + (lane & 31) * kRowBytes + (lane >> 5) * 16;
    if (G::NSTAGE == 1) {
        // single LDS stage: multiply, barrier, refill from the prefetch registers, barrier
        if (!active_u) {
            for (int t = 0; t + 1 < nk; ++t) {
                __syncthreads();
                const int s2 = min(t + 2, nk - 1);
#pragma unroll
                for (int part = 0; part < 4; ++part) {
                    al.sstore_part(smem, part);
                    bl.sstore_part(smem + G::A_BYTES, part);
                    al.gload_part(s2, part);
                    bl.gload_part(s2, part);
                }
                __syncthreads();
            }
            __syncthreads();
            return;
        }
        for (int t = 0; t < nk; ++t) {
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                __builtin_amdgcn_sched_barrier(0);
                bf16x8_t a, b[8];
                a = *(const bf16x8_t*)(smem + a_off + kk * 32);
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    b[f] = *(const bf16x8_t*)(smem + b_off + f * 32 * kRowBytes + kk * 32);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[f], acc[f], 0, 0, 0);
            }
            if (t + 1 < nk) {
                __syncthreads();
                const int s2 = min(t + 2, nk - 1);
#pragma unroll
                for (int part = 0; part < 4; ++part) {
                    al.sstore_part(smem, part);
                    bl.sstore_part(smem + G::A_BYTES, part);
                    al.gload_part(s2, part);
                    bl.gload_part(s2, part);
                }
                __syncthreads();
            }
        }
        __syncthreads();   // the tile's epilogue may not overtake slower waves' last reads
        return;
    }
    if (!active_u) {
        for (int t = 0; t < nk; ++t) {
            char* nxt = smem + ((t + 1) & 1) * G::STAGE;
            const int s2 = min(t + 2, nk - 1);
#pragma unroll
            for (int part = 0; part < 4; ++part) {
                al.sstore_part(nxt, part);
                bl.sstore_part(nxt + G::A_BYTES, part);
                al.gload_part(s2, part);
                bl.gload_part(s2, part);
            }
            __syncthreads();
        }
        return;
    }
    for (int t = 0; t < nk; ++t) {
        char* cur = smem + (t & 1) * G::STAGE;
        char* nxt = smem + ((t + 1) & 1) * G::STAGE;
        const int s2 = min(t + 2, nk - 1);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            __builtin_amdgcn_sched_barrier(0);
            al.sstore_part(nxt, kk);
            bl.sstore_part(nxt + G::A_BYTES, kk);
            al.gload_part(s2, kk);
            bl.gload_part(s2, kk);
            __builtin_amdgcn_sched_barrier(0);
            bf16x8_t a, b[8];
            a = *(const bf16x8_t*)(cur + a_off + kk * 32);
#pragma unroll
            for (int f = 0; f < 8; ++f)
                b[f] = *(const bf16x8_t*)(cur + b_off + f * 32 * kRowBytes + kk * 32);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < 8; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[f], acc[f], 0, 0, 0);
        }
        __syncthreads();
    }
}

// ------------------------------------------------- A operand straight to registers
// In the row-tile GEMMs every wave owns its 32 rows alone, so the A operand need
// not pass through LDS: lane (row = lane%32, g = lane/32) fetches its fragments
// directly, 16 bytes per k-sub-step.  The order of k inside a stage is free as
// long as both operands agree, so lane half g takes the k-range [32g, 32g+32) of
// the stage (64 contiguous bytes per lane and stage); the B fragment reads use the
// same k offsets.  Four rolling fragment registers: fragment kk of stage t+1 is
// requested right after fragment kk of stage t was consumed.
// rp = address of (this lane's row, k = 32*g) of stage 0; rows outside the tile
// alias a valid row.  SCALE: multiply by a per-row fp32 factor, round to bf16.
template <bool SCALE>
struct DirectRowLoader {
    const char* rp;
    float sc;
    u32x4_t frag[BK / 16];

    __device__ __forceinline__ void load(int s, int kk) {
        frag[kk] = *(const u32x4_t*)(rp + (size_t)s * (BK * 2) + kk * 16);
    }
    __device__ __forceinline__ bf16x8_t get(int kk) const {
        u32x4_t r = frag[kk];
        if (SCALE) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(bf16_lo(r[q]) * sc, bf16_hi(r[q]) * sc);
        }
        return __builtin_bit_cast(bf16x8_t, r);
    }
};

// Main loop with the A operand in registers and only B in LDS (two stages of
// B_BYTES at the start of smem).  Same pipeline as mma_mainloop for B.
template <int NW, bool SCALE, class BL>
__device__ __forceinline__ void mma_mainloop_direct(DirectRowLoader<SCALE>& al, BL& bl, int nk,
                                                    char* smem, bool active, f32x16_t (&acc)[8]) {
    typedef Geom<NW> G;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
    if (nk <= 0) return;
    const bool active_u = __builtin_amdgcn_readfirstlane((int)active) != 0;

#pragma unroll
    for (int part = 0; part < 4; ++part) bl.gload_part(0, part);
    if (active_u) {
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) al.load(0, kk);
    }
#pragma unroll
    for (int part = 0; part < 4; ++part) bl.sstore_part(smem, part);
    const int s1 = min(1, nk - 1);
#pragma unroll
    for (int part = 0; part < 4; ++part) bl.gload_part(s1, part);
    __syncthreads();
    // B fragment f of this lane: LDS row f*32 + lane%32, k bytes (lane/32)*64 + kk*16
    const int b_off = (lane & 31) * kRowBytes + (lane >> 5) * 64;
    if (!active_u) {
        for (int t = 0; t < nk; ++t) {
            char* nxt = smem + ((t + 1) & 1) * G::B_BYTES;
            const int s2 = min(t + 2, nk - 1);
#pragma unroll
            for (int part = 0; part < 4; ++part) {
                bl.sstore_part(nxt, part);
                bl.gload_part(s2, part);
            }
            __syncthreads();
        }
        return;
    }
    for (int t = 0; t < nk; ++t) {
        char* cur = smem + (t & 1) * G::B_BYTES;
        char* nxt = smem + ((t + 1) & 1) * G::B_BYTES;
        const int s2 = min(t + 2, nk - 1);
        const int sa = min(t + 1, nk - 1);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            __builtin_amdgcn_sched_barrier(0);
            bl.sstore_part(nxt, kk);
            bl.gload_part(s2, kk);
            __builtin_amdgcn_sched_barrier(0);
            bf16x8_t b[8];
#pragma unroll
            for (int f = 0; f < 8; ++f)
                b[f] = *(const bf16x8_t*)(cur + b_off + f * 32 * kRowBytes + kk * 16);
            const bf16x8_t a = al.get(kk);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < 8; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[f], acc[f], 0, 0, 0);
            al.load(sa, kk);
        }
        __syncthreads();
    }
}

// Pack the 8 consecutive columns a lane holds for accumulator element v.
__device__ __forceinline__ u32x4_t pack_row8(const f32x16_t (&acc)[8], int v) {
    u32x4_t r;
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(acc[2 * q][v], acc[2 * q + 1][v]);
    return r;
}

__device__ __forceinline__ float dpp_swap_pair(float x) {   // value of lane ^ 1
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true));
}

// v_exp_f32 and v_rcp_f32 (1 ulp each): far inside the bf16 rounding of the results
__device__ __forceinline__ float sigmoid_f(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

}  // namespace uniep
