// bf16 MFMA tile machinery for gfx950 (CDNA4): operands by global->LDS DMA, fragments by
// LDS reads that run one k-sub-step ahead of the matrix instructions.
//
// A workgroup is 8 waves (two per SIMD) and owns an output tile of 256 x 256: 256 "row"
// indices (the B role of the MFMA: one index per lane) by 256 "column" indices (the A role:
// 16 values per lane and accumulator, arranged so that a lane ends with runs of 8 consecutive
// columns and stores 16 bytes).  Wave w = 4 wm + wn owns rows [128 wm, +128) as 4 fragments
// of 32 and columns [64 wn, +64) as 2 fragments of 32: 8 accumulators of
// v_mfma_f32_32x32x16_bf16, 6 fragment reads per 8 matrix instructions.
//
// K advances in stages of 64.  A stage of an operand is a 32 KB LDS image in one of two forms:
//   KC  the operand's k runs along its memory rows (activations [rows, k]; weights read
//       "transposed"): image [256 rows][128 B], the 16-byte chunk c of row r at chunk position
//       c ^ ((r >> 1) & 7), fragments by ds_read_b128;
//   KS  the operand's k is its memory row index (weights [k, n]; both operands of the
//       weight-gradient GEMMs): image [64 k][512 B], the 16-byte chunk c of k row k at chunk
//       position c ^ ((k & 3) << 2), fragments by ds_read_b64_tr_b16, which hands lane l of a
//       group of 16 the element l % 4 of the 8-byte pieces that lanes 4e + l / 4 addressed
//       (e = 0..3): four k rows of one column.
// Both swizzles make the fragment reads bank-conflict free, and both are applied by the DMA
// side through the choice of the global address each lane fetches: a DMA instruction writes
// lane p's 16 bytes to (LDS base) + 16 p, so nothing is staged in registers and no LDS
// write instruction or register transpose exists.
//
// Two stage buffers (128 KB of LDS).  Stage t+2 is requested right behind the barrier that
// ends the fragment reads of stage t, so it has a whole stage of matrix work to land; one
// workgroup barrier per stage.  The fragment reads are inline assembly: the compiler would put
// a full vmcnt(0) in front of every LDS read it knows about while a DMA load is in flight.
// The waits that make their results usable are therefore written by hand (lgkmcnt counts,
// LDS operations complete in order) and tie the fragment registers, so that no matrix
// instruction can be scheduled ahead of them.
#pragma once
#include "common.hpp"

namespace uniep {

constexpr int BK = 64;
constexpr int BN = 256;                 // tile columns (A role)
constexpr int BMAX = 256;               // tile rows (B role)
constexpr int kOperandBytes = 32768;    // one operand, one stage
constexpr int kStageBytes = 2 * kOperandBytes;   // rows (B role) first, columns (A role) second
constexpr int kMmaSmem = 2 * kStageBytes;
constexpr int kMmaThreads = 512;

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void glb_void_t;

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ u32x4_t zero4() { return u32x4_t{0u, 0u, 0u, 0u}; }

// This thread's coordinates, derived from an opaque copy of threadIdx.x.  Address arithmetic
// that depends only on threadIdx.x is loop-invariant for the persistent task loop, so the
// compiler computes all of it once at kernel start, runs out of registers and reloads it from
// scratch next to the stores (each reload waits for the previous store to complete).  A task
// makes its own Lane before its main loop and another one for its epilogue.
struct Lane {
    int tid, l, l31, hf, w, wm, wn;
    __device__ __forceinline__ Lane() {
        unsigned t = threadIdx.x;
        asm volatile("" : "+v"(t));
        tid = (int)t;
        l = tid & 63;
        l31 = tid & 31;
        hf = (tid >> 5) & 1;
        w = tid >> 6;
        wm = tid >> 8;
        wn = (tid >> 6) & 3;
    }
    __device__ __forceinline__ int wave_uniform() const { return __builtin_amdgcn_readfirstlane(w); }
};

// MFMA row index i (0..31) -> position of that column inside the 32 columns of an A-role
// fragment: accumulator element v of lane half hf holds MFMA row 8 (v / 4) + 4 hf + v % 4, and
// this bit swap turns v = 0..7 into 8 consecutive columns (16 hf' ... see acc_col()).
__device__ __forceinline__ int swap23(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// Tile row / column of accumulator (tf, af) element v of this lane.
__device__ __forceinline__ int acc_row(const Lane& ln, int tf) { return 128 * ln.wm + 32 * tf + ln.l31; }
// first of the 8 consecutive columns that elements v = 8 vg .. 8 vg + 7 hold
__device__ __forceinline__ int acc_col8(const Lane& ln, int af, int vg) {
    return 64 * ln.wn + 32 * af + 16 * vg + 8 * ln.hf;
}

// ------------------------------------------------------------------ fragment addresses
struct FragAddr {
    uint32_t b[4];   // B role: KC -> per k-sub-step (+ tf * 4096); KS -> b[0] + ((tf << 6) ^ b[1]) per row fragment (+ kk * 8192 + hr * 2048)
    uint32_t a[4];   // A role: KC -> per k-sub-step (+ af * 4096); KS -> a[0..1] per column fragment (+ kk * 8192 + hr * 2048)
};

template <bool A_KS, bool B_KS>
__device__ __forceinline__ void frag_addresses(FragAddr& fa, uint32_t lds0, const Lane& ln) {
    const int l = ln.l;
    const int wm = ln.wm, wn = ln.wn;
    const int kh = ln.hf, l31 = ln.l31;
    const int g = (l >> 4) & 1, jj = l & 15, e = jj >> 2, q = jj & 3;
    if (B_KS) {
        // chunk of row fragment tf = (16 wm + 2 g + q / 2) | ((tf ^ e) << 2): the swizzle only touches the
        // fragment bits, so one base and the lane's e << 6 describe all four addresses
        fa.b[0] = lds0 + (8 * kh + e) * 512 + ((16 * wm + 2 * g + (q >> 1)) << 4) + (q & 1) * 8;
        fa.b[1] = e << 6;
        fa.b[2] = fa.b[3] = 0;
    } else {
        const int x0 = (l >> 1) & 7;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            fa.b[kk] = lds0 + (128 * wm + l31) * 128 + (((2 * kk + kh) ^ x0) << 4);
    }
    const uint32_t a0 = lds0 + kOperandBytes;
    if (A_KS) {
        const int sq = ((q & 1) << 1) | (q >> 1);   // piece -> position of its 4 columns inside the 16
#pragma unroll
        for (int af = 0; af < 2; ++af) {
            const int c = 8 * wn + 4 * af + 2 * g + (sq >> 1);
            fa.a[af] = a0 + (8 * kh + e) * 512 + ((c ^ (e << 2)) << 4) + (sq & 1) * 8;
        }
        fa.a[2] = fa.a[3] = 0;
    } else {
        const int n = swap23(l31);
        const int x1 = (n >> 1) & 7;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            fa.a[kk] = a0 + (64 * wn + n) * 128 + (((2 * kk + kh) ^ x1) << 4);
    }
}

// ------------------------------------------------------------------ fragments
struct Frags {
    u32x4_t b[4];   // B role, one per row fragment
    u32x4_t a[2];   // A role, one per column fragment
};

// The two halves of a transposing read land in the low and high register pair of one
// 128-bit fragment: the pair is addressed through a 64-bit view of the same registers.
#define UNIEP_TR2(dst, addr, off)                                                                  \
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:" #off "\n ds_read_b64_tr_b16 %1, %2 offset:" #off "+2048" \
                 : "=&v"(lo_), "=&v"(hi_) : "v"(addr) : "memory");                                   \
    dst = u32x4_t{lo_[0], lo_[1], hi_[0], hi_[1]}

template <int KK>
__device__ __forceinline__ void read_ks(u32x4_t& dst, uint32_t addr) {
    u32x2_t lo_, hi_;
    if (KK == 0) { UNIEP_TR2(dst, addr, 0); }
    else if (KK == 1) { UNIEP_TR2(dst, addr, 8192); }
    else if (KK == 2) { UNIEP_TR2(dst, addr, 16384); }
    else { UNIEP_TR2(dst, addr, 24576); }
}
#undef UNIEP_TR2

template <int F>
__device__ __forceinline__ void read_kc(u32x4_t& dst, uint32_t addr) {
    if (F == 0) asm volatile("ds_read_b128 %0, %1" : "=&v"(dst) : "v"(addr) : "memory");
    else if (F == 1) asm volatile("ds_read_b128 %0, %1 offset:4096" : "=&v"(dst) : "v"(addr) : "memory");
    else if (F == 2) asm volatile("ds_read_b128 %0, %1 offset:8192" : "=&v"(dst) : "v"(addr) : "memory");
    else asm volatile("ds_read_b128 %0, %1 offset:12288" : "=&v"(dst) : "v"(addr) : "memory");
}

// LDS read instructions of one call of read_frags
template <int NTF, bool A_KS, bool B_KS>
constexpr int reads_per_step() { return (B_KS ? 2 : 1) * NTF + (A_KS ? 2 : 1) * 2; }

// Fragments of k-sub-step KK of the stage at byte offset `boff`.
template <int NTF, bool A_KS, bool B_KS, int KK>
__device__ __forceinline__ void read_frags(Frags& f, const FragAddr& fa, uint32_t boff) {
    if (A_KS) {
        read_ks<KK>(f.a[0], fa.a[0] + boff);
        read_ks<KK>(f.a[1], fa.a[1] + boff);
    } else {
        const uint32_t ad = fa.a[KK] + boff;
        read_kc<0>(f.a[0], ad);
        read_kc<1>(f.a[1], ad);
    }
    if (B_KS) {
        const uint32_t bd = fa.b[0] + boff;
        if (NTF > 0) read_ks<KK>(f.b[0], bd + fa.b[1]);
        if (NTF > 1) read_ks<KK>(f.b[1], bd + (fa.b[1] ^ 64u));
        if (NTF > 2) read_ks<KK>(f.b[2], bd + (fa.b[1] ^ 128u));
        if (NTF > 3) read_ks<KK>(f.b[3], bd + (fa.b[1] ^ 192u));
    } else {
        const uint32_t bd = fa.b[KK] + boff;
        if (NTF > 0) read_kc<0>(f.b[0], bd);
        if (NTF > 1) read_kc<1>(f.b[1], bd);
        if (NTF > 2) read_kc<2>(f.b[2], bd);
        if (NTF > 3) read_kc<3>(f.b[3], bd);
    }
}

// Wait until at most N LDS operations are outstanding; ties the fragment registers.
template <int N>
__device__ __forceinline__ void wait_frags(Frags& f) {
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3]), "+v"(f.a[0]), "+v"(f.a[1])
                 : "n"(N) : "memory");
}

template <int NTF>
__device__ __forceinline__ void mfma_step(const Frags& f, f32x16_t (&acc)[4][2]) {
#pragma unroll
    for (int tf = 0; tf < NTF; ++tf)
#pragma unroll
        for (int af = 0; af < 2; ++af)
            acc[tf][af] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, f.a[af]),
                                                                  __builtin_bit_cast(bf16x8_t, f.b[tf]),
                                                                  acc[tf][af], 0, 0, 0);
}

// The matrix instructions of one k-sub-step (fragments `cur`) with the fragment reads of sub-step KK
// (into `nxt`) between the first three of them: a wave issues in order, and a matrix instruction
// keeps its pipe busy for 32 clocks during which the same wave may issue other instructions, so
// the reads cost no matrix issue slot, and the LDS sees them spread out instead of in bursts of
// six to twelve from every wave at once.
template <int NTF, bool A_KS, bool B_KS, int KK>
__device__ __forceinline__ void mfma_step_reading(const Frags& cur, Frags& nxt, const FragAddr& fa, uint32_t boff,
                                                  f32x16_t (&acc)[4][2], bool rd = true) {
    auto mm = [&](int tf, int af) {
        acc[tf][af] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, cur.a[af]),
                                                              __builtin_bit_cast(bf16x8_t, cur.b[tf]), acc[tf][af], 0, 0, 0);
    };
    const uint32_t ad = (A_KS ? 0u : fa.a[KK]) + boff, bd = (B_KS ? fa.b[0] : fa.b[KK]) + boff;
    auto rb = [&](int tf) {
        if (!rd) return;
        if (B_KS) {
            if (tf == 0) read_ks<KK>(nxt.b[0], bd + fa.b[1]);
            if (tf == 1) read_ks<KK>(nxt.b[1], bd + (fa.b[1] ^ 64u));
            if (tf == 2) read_ks<KK>(nxt.b[2], bd + (fa.b[1] ^ 128u));
            if (tf == 3) read_ks<KK>(nxt.b[3], bd + (fa.b[1] ^ 192u));
        } else {
            if (tf == 0) read_kc<0>(nxt.b[0], bd);
            if (tf == 1) read_kc<1>(nxt.b[1], bd);
            if (tf == 2) read_kc<2>(nxt.b[2], bd);
            if (tf == 3) read_kc<3>(nxt.b[3], bd);
        }
    };
    auto ra = [&](int af) {
        if (!rd) return;
        if (A_KS) {
            if (af == 0) read_ks<KK>(nxt.a[0], fa.a[0] + boff);
            else read_ks<KK>(nxt.a[1], fa.a[1] + boff);
        } else {
            if (af == 0) read_kc<0>(nxt.a[0], ad);
            else read_kc<1>(nxt.a[1], ad);
        }
    };
    if (NTF > 0) mm(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    ra(0);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 0) mm(0, 1);
    __builtin_amdgcn_sched_barrier(0);
    ra(1);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 1) mm(1, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 0) rb(0);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 1) mm(1, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 1) rb(1);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 2) mm(2, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 2) rb(2);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 2) mm(2, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 3) rb(3);
    __builtin_amdgcn_sched_barrier(0);
    if (NTF > 3) {
        mm(3, 0);
        mm(3, 1);
    }
}

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ------------------------------------------------------------------ DMA sources
// Every loader moves one operand: issue(dst) requests the next stage into the 32 KB image at
// `dst` (4 DMA instructions per wave, 1 KB each) and advances; DMA instruction i of wave w
// fills the 1 KB block u = 4 w + i of the image.
__device__ __forceinline__ void dma16(const char* src, char* dst) {
    __builtin_amdgcn_global_load_lds((glb_void_t*)src, (lds_void_t*)dst, 16, 0, 0);
}
// this wave's first 1 KB block of an operand image, as a wave-uniform byte offset
__device__ __forceinline__ int wave_block_off() {
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * 4096;
}
__device__ __forceinline__ int wave_block_off(const Lane& ln) { return ln.wave_uniform() * 4096; }

// KC image: block u holds rows 8u .. 8u+7; lane p moves the chunk of row 8u + p/8 that belongs
// at chunk position p%8.  row_of(i) / chunk_of(i) tell a task which (row, chunk) this lane
// fetches with instruction i; p[i] = address of that chunk in stage 0.
struct KcGeom {
    static __device__ __forceinline__ int row(const Lane& ln, int i) { return 8 * (4 * ln.w + i) + (ln.l >> 3); }
    static __device__ __forceinline__ int chunk(const Lane& ln, int i) { return (ln.l & 7) ^ ((row(ln, i) >> 1) & 7); }
};
// Rows whose k runs on: every stage is 128 bytes further along each row.  Only the first
// `n` of the wave's four 8-row blocks are moved: blocks whose rows all lie beyond the tile's
// rows are skipped (nothing reads them except row fragments whose outputs are never stored).
struct KcLoader {
    const char* p[4];
    int n = 4;   // wave-uniform
    __device__ __forceinline__ void sync() {}
    // blocks of this wave that hold rows of a tile with `rows` rows
    __device__ __forceinline__ void prepare() {}
    static __device__ __forceinline__ int blocks_for(const Lane& ln, int rows) {
        return min(4, max(0, (rows - 32 * ln.wave_uniform() + 7) >> 3));
    }
    __device__ __forceinline__ void issue(char* dst) {
        char* d = dst + wave_block_off();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i < n) dma16(p[i], d + i * 1024);
            p[i] += BK * 2;
        }
    }
};
// The same with the k axis being the concatenation of two matrices of identical layout (W_gate
// then W_up along k): after `left` more stages every pointer jumps by `delta` bytes.
struct KcSplitLoader {
    const char* p[4];
    long long delta;   // (second matrix) - (first matrix) - (bytes walked in the first)
    int left;
    __device__ __forceinline__ void prepare() {}
    __device__ __forceinline__ void sync() {}
    __device__ __forceinline__ void issue(char* dst) {
        char* d = dst + wave_block_off();
        if (left == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) p[i] += delta;
        }
        --left;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(p[i], d + i * 1024);
            p[i] += BK * 2;
        }
    }
};

// KS image: block u holds k rows 2u, 2u+1 (512 B = 32 chunks each); lane p moves the chunk of
// k row 2u + p/32 that belongs at chunk position p%32.
struct KsGeom {
    static __device__ __forceinline__ int krow(const Lane& ln, int i) { return 2 * (4 * ln.w + i) + ln.hf; }
    static __device__ __forceinline__ int chunk(const Lane& ln, int i) { return ln.l31 ^ ((krow(ln, i) & 3) << 2); }
};
// Dense matrix [K, n], K a multiple of 64: p[i] = address of (k row krow(i), this lane's chunk).
struct KsLoader {
    const char* p[4];
    long long step;   // 64 memory rows
    __device__ __forceinline__ void prepare() {}
    __device__ __forceinline__ void sync() {}
    __device__ __forceinline__ void issue(char* dst) {
        char* d = dst + wave_block_off();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(p[i], d + i * 1024);
            p[i] += step;
        }
    }
};
// Reduction over K memory rows with K not a multiple of 64 (the rows of one expert): k rows at
// and beyond K are written as zeros instead of fetched.  The four k rows a lane moves are
// krow(0) + 2i, and its chunk depends on i only through i % 2, so two addresses describe them:
// p[j] = address of (k row krow(j), chunk(j)) of stage 0, j = 0, 1; instructions 2, 3 are 4
// memory rows further.
__device__ __forceinline__ void lds_zero16(char* dst) {
    const uint32_t ad = lds_addr(dst) + (threadIdx.x & 63) * 16;   // (cheap; recomputed where it is used)
    asm volatile("ds_write_b128 %0, %1" : : "v"(ad), "v"(zero4()) : "memory");
}
__device__ __forceinline__ int rfl(int v) { return __builtin_amdgcn_readfirstlane(v); }

struct KsTailLoader {
    const char* p[2];
    long long ld_bytes;   // one memory row (wave-uniform)
    int k0;               // reduction index of instruction 0's k row in the stage to come
    int K;
    __device__ __forceinline__ void prepare() {}
    __device__ __forceinline__ void sync() {}
    __device__ __forceinline__ void issue(char* dst) {
        char* d = dst + wave_block_off();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (k0 + 2 * i < K) dma16(p[i & 1] + (i >> 1) * 4 * ld_bytes, d + i * 1024);
            else lds_zero16(d + i * 1024);
        }
        p[0] += BK * ld_bytes;
        p[1] += BK * ld_bytes;
        k0 += BK;
    }
};
// The same with a gather: reduction index k is memory row rows[k] of a [T, ld] matrix.  The
// row indices of a stage are fetched (plain loads) right behind the DMA of the stage before
// it and are complete by the barrier in between.  init() is called once per tile, after
// coloff[] is filled.
// prepare() turns the fetched indices into the four source addresses, and the main loop calls
// it for both loaders before either requests anything: while a DMA is pending the compiler puts
// a full vmcnt(0) in front of every use of a register that an ordinary load filled (it cannot
// order the two kinds of operation), so address arithmetic between the DMA instructions would
// make every request wait for the one before it to land.
struct KsGatherLoader {
    const char* src;          // matrix base
    uint32_t coloff[2];       // byte offset, inside a memory row, of the chunk instructions i, i % 2 = j move
    long long ld_bytes;       // wave-uniform
    const int32_t* rows;      // row_tok + first row of the expert (wave-uniform)
    int32_t tok[4];           // memory rows of the stage whose DMA goes out next
    const char* a[4];         // their addresses (prepare)
    int k0;                   // reduction index of instruction 0's k row in that stage
    int K;
    __device__ __forceinline__ void fetch() {
#pragma unroll
        for (int i = 0; i < 4; ++i) tok[i] = rows[min(k0 + 2 * i, K - 1)];
    }
    __device__ __forceinline__ void init(const Lane& ln, const char* src_, long long ld_bytes_, const int32_t* rows_, int K_) {
        src = src_;
        ld_bytes = ld_bytes_;
        rows = rows_;
        K = K_;
        k0 = KsGeom::krow(ln, 0);
        fetch();
    }
    __device__ __forceinline__ void prepare() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = src + (long long)tok[i] * ld_bytes + coloff[i & 1];
            asm volatile("" : "+v"(a[i]));   // the address exists before the first request
        }
    }
    __device__ __forceinline__ void issue(char* dst) {
        char* d = dst + wave_block_off();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (k0 + 2 * i < K) dma16(a[i], d + i * 1024);
            else lds_zero16(d + i * 1024);
        }
        k0 += BK;
        fetch();
    }
};

// ------------------------------------------------------------------ main loop
// acc[tf][af] += (column fragment af) x (row fragment tf) over nk stages (nk >= 1).
// NTF = row fragments of this wave that hold rows of the tile (0..4): the others are neither
// read nor multiplied.  Every wave takes part in the DMA and in the barriers whatever its NTF.
// Pipeline per stage t (buffer t % 2), k-sub-steps 0..3 of 16:
//   sub-step s < 3: wait for the fragments of s, 8 matrix instructions with the fragment reads
//                   of s+1 between the first three of them (mfma_step_reading);
//   sub-step 3:     wait for its fragments (the last reads of the buffer), wait for this wave's
//                   DMA of stage t+1, barrier, request the row operand of stage t+2 into the
//                   buffer just freed, request the fragments of (t+1, 0), 8 matrix instructions,
//                   request the column operand of stage t+2 (a CU takes about 64 DMA requests
//                   before issue blocks, which is what one stage has: the second half goes out
//                   behind a burst of matrix work instead of in front of it; 1 % on the step).
template <int NTF, bool A_KS, bool B_KS, class LB, class LA>
__device__ __forceinline__ void mma_loop(LB& lb, LA& la, int nk, char* smem, const FragAddr& fa,
                                         f32x16_t (&acc)[4][2]) {
    lb.prepare();
    la.prepare();
    __builtin_amdgcn_sched_barrier(0);
    lb.issue(smem);
    la.issue(smem + kOperandBytes);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (nk > 1) {
        lb.prepare();
        la.prepare();
        __builtin_amdgcn_sched_barrier(0);
        lb.issue(smem + kStageBytes);
        la.issue(smem + kStageBytes + kOperandBytes);
    }
    Frags f0, f1;
    if (NTF > 0) read_frags<NTF, A_KS, B_KS, 0>(f0, fa, 0);
    for (int t = 0; t < nk; ++t) {
        const uint32_t boff = (t & 1) * kStageBytes, noff = kStageBytes - boff;
        __builtin_amdgcn_sched_barrier(0);
        if (NTF > 0) {
            wait_frags<0>(f0);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step_reading<NTF, A_KS, B_KS, 1>(f0, f1, fa, boff, acc);
            __builtin_amdgcn_sched_barrier(0);
            wait_frags<0>(f1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step_reading<NTF, A_KS, B_KS, 2>(f1, f0, fa, boff, acc);
            __builtin_amdgcn_sched_barrier(0);
            wait_frags<0>(f0);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step_reading<NTF, A_KS, B_KS, 3>(f0, f1, fa, boff, acc);
            __builtin_amdgcn_sched_barrier(0);
            wait_frags<0>(f1);
        }
        if (t + 1 < nk) {
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            if (t + 2 < nk) {
                lb.prepare();
                la.prepare();
                __builtin_amdgcn_sched_barrier(0);
                lb.issue(smem + boff);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // the matrix instructions of sub-step 3, with the first fragment reads of stage t+1 (if there is one) between them
        if (NTF > 0) mfma_step_reading<NTF, A_KS, B_KS, 0>(f1, f0, fa, noff, acc, t + 1 < nk);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < nk) la.issue(smem + boff + kOperandBytes);   // the second operand's requests behind a burst of matrix work
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();   // every wave has read its last fragments: the buffers may be refilled
}

// Row fragments of this wave that hold rows when the tile has `rows` of them.
__device__ __forceinline__ int active_row_frags(int rows) {
    const int mine = rows - 128 * __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8));
    return __builtin_amdgcn_readfirstlane(mine <= 0 ? 0 : (mine >= 128 ? 4 : (mine + 31) >> 5));
}

// Runs mma_loop with the wave's NTF (a scalar branch: every wave runs exactly one instance, and all
// instances execute the same barriers).
template <bool A_KS, bool B_KS, class LB, class LA>
__device__ __forceinline__ void mma_tile(LB& lb, LA& la, int nk, int rows, char* smem, const FragAddr& fa,
                                         f32x16_t (&acc)[4][2]) {
#pragma unroll
    for (int tf = 0; tf < 4; ++tf)
#pragma unroll
        for (int af = 0; af < 2; ++af)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tf][af][v] = 0.f;
    if (nk <= 0) return;   // empty reduction (an expert without rows): the tile is all zeros
    const int ntf = active_row_frags(rows);
    if (ntf == 4) mma_loop<4, A_KS, B_KS>(lb, la, nk, smem, fa, acc);
    else if (ntf == 3) mma_loop<3, A_KS, B_KS>(lb, la, nk, smem, fa, acc);
    else if (ntf == 2) mma_loop<2, A_KS, B_KS>(lb, la, nk, smem, fa, acc);
    else if (ntf == 1) mma_loop<1, A_KS, B_KS>(lb, la, nk, smem, fa, acc);
    else mma_loop<0, A_KS, B_KS>(lb, la, nk, smem, fa, acc);
}

// ------------------------------------------------------------------ epilogue helpers
// The 8 consecutive columns of accumulator elements 8 vg .. 8 vg + 7, packed to bf16.
__device__ __forceinline__ u32x4_t pack8(const f32x16_t& a, int vg) {
    u32x4_t r;
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = pack_bf16x2(a[8 * vg + 2 * q], a[8 * vg + 2 * q + 1]);
    return r;
}

// Stores that cover whole 128-byte lines.  After the main loop a lane holds, per row fragment,
// 16-byte pieces of 32 different rows, so a store instruction straight from the accumulators
// touches 32 rows with 32 contiguous bytes each: four times the write requests of a row-major
// store, as partial lines, and the next tile's first loads queue behind them.  Instead every
// wave passes its 128 x 64 sub-tile through its own 16 KB of the (now idle) stage buffers:
// put() writes a lane's 16-byte pieces, get() hands lane l the piece l % NP of row
// (64 / NP) j + l / NP, so NP neighbouring lanes store one contiguous run of NP * 16 bytes.
// Rows are NP * 16 bytes apart and the piece position is XORed with row bits so that both
// directions are bank-conflict free.  Wave-private: LDS operations of a wave execute in
// order, no barrier is involved.  NP = 8: 64 bf16 columns per row (or 32 fp32); NP = 4: 32 bf16 columns.
template <int NP>
struct WaveRepack {
    char* base;   // this wave's 16 KB
    int l;        // lane
    __device__ __forceinline__ WaveRepack(char* smem, const Lane& ln) : base(smem + ln.w * 16384), l(ln.l) {}
    // eight neighbouring lanes of a put() hold eight consecutive rows: their 16-byte slots must differ
    static __device__ __forceinline__ int swz(int row) { return NP == 8 ? (row & 7) : ((row >> 1) & 3); }
    // piece pi (0..NP-1) of sub-tile row `row` (0..127)
    __device__ __forceinline__ void put(int row, int pi, u32x4_t v) {
        *(u32x4_t*)(base + row * (NP * 16) + ((pi ^ swz(row)) << 4)) = v;
    }
    __device__ __forceinline__ int get_row(int j) const { return (64 / NP) * j + l / NP; }
    __device__ __forceinline__ int get_piece() const { return l % NP; }
    __device__ __forceinline__ u32x4_t get(int j) const {
        const int row = get_row(j);
        return *(const u32x4_t*)(base + row * (NP * 16) + ((get_piece() ^ swz(row)) << 4));
    }
    // The same in 8-byte pieces (2 NP per row), for outputs that leave through 8-byte write-through
    // stores: lane l gets piece l % (2 NP) of row (32 / NP) j + l / (2 NP).
    __device__ __forceinline__ int get8_row(int j) const { return (32 / NP) * j + l / (2 * NP); }
    __device__ __forceinline__ int get8_piece() const { return l % (2 * NP); }
    __device__ __forceinline__ u32x2_t get8(int j) const {
        const int row = get8_row(j), p8 = get8_piece();
        return *(const u32x2_t*)(base + row * (NP * 16) + (((p8 >> 1) ^ swz(row)) << 4) + (p8 & 1) * 8);
    }
};

// The wave's 128 x 64 bf16 sub-tile of the accumulators, handed to store(tile row, tile column,
// 8 columns as 16 bytes) with 8 neighbouring lanes on one row (128 contiguous bytes); rows at
// and beyond `rows` and 8-column pieces at and beyond `cols` (tile coordinates) are left out.
template <class StoreFn>
__device__ __forceinline__ void store_subtile_bf16(const f32x16_t (&acc)[4][2], char* smem, int rows, int cols,
                                                   StoreFn store) {
    const Lane ln;
    WaveRepack<8> rp(smem, ln);
    const int l31 = ln.l31, hf = ln.hf;
    const int wm = ln.wm, wn = ln.wn;
#pragma unroll
    for (int tf = 0; tf < 4; ++tf)
#pragma unroll
        for (int af = 0; af < 2; ++af)
#pragma unroll
            for (int vg = 0; vg < 2; ++vg) rp.put(32 * tf + l31, 4 * af + 2 * vg + hf, pack8(acc[tf][af], vg));
    const int col = 64 * wn + 8 * rp.get_piece();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int row = 128 * wm + rp.get_row(j);
        const u32x4_t v = rp.get(j);
        if (row < rows && col < cols) store(row, col, v);
    }
}

// v_exp_f32 and v_rcp_f32 (1 ulp each): far inside the bf16 rounding of the results
__device__ __forceinline__ float sigmoid_f(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

}  // namespace uniep
