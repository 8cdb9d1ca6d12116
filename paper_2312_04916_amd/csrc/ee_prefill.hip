// HIP kernels (gfx950) for the prompt phase: the full-depth causal forward of many positions at once
// (the "prefilling phase" of Section 4), where the projections are true GEMMs and the matrix cores, not
// HBM, are the bound; and the exit heads scored on every position (the per-position token / confidence
// view of Table 4).
//
// Operand layout.  Weights keep the decode layout: 16-row tiles, [tile][K/32][64 lanes][8 bf16], which is
// the register image of one 16x32 MFMA operand.  Activations of this path use THE SAME layout with rows =
// positions: [row/16][K/32][64][8], one array for the hi term and one for the lo term (two-term bf16,
// see ee_kernels.hip).  A workgroup therefore stages both operands with plain 1 KB global->LDS copies
// (no register round trip, no swizzle, no bank conflicts) and every wave reads ready-made operands back.
//
// The product is formed transposed, D[n][m] (weights as the A operand): a lane then holds four
// consecutive output features of one position, which is exactly an 8-byte piece of the next GEMM's
// activation operand, of a K-cache row, or of a packed q row.
#include "ee_internal.h"

#include "ee_lanes.h"
#include "ee_launch.h"

namespace ee {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define EE_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
#define EE_GLB_PTR(p) ((const void __attribute__((address_space(1)))*)(p))

namespace {

constexpr int PF_NTL = 16;  // 16-column weight tiles per workgroup (256 output features)

// element index of (row m, feature k) in a packed activation array with KT = K/32 tiles per row group
__device__ __forceinline__ size_t pk_index(int m, int k, int KT) {
    return (((size_t)(m >> 4) * KT + (k >> 5)) * 64 + (((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7);
}

// stores four consecutive features (k % 4 == 0) of row m as two bf16 terms
__device__ __forceinline__ void pk_store4(__bf16* hi, __bf16* lo, int m, int k, int KT, const float v[4]) {
    const size_t o = pk_index(m, k, KT);
    bf16x4 h, l;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const __bf16 t = (__bf16)v[r];
        h[r] = t;
        l[r] = (__bf16)(v[r] - (float)t);
    }
    *(bf16x4*)(hi + o) = h;
    *(bf16x4*)(lo + o) = l;
}

// ... and two consecutive features (k % 2 == 0)
__device__ __forceinline__ void pk_store2(__bf16* hi, __bf16* lo, int m, int k, int KT, float v0, float v1) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const size_t o = pk_index(m, k, KT);
    const __bf16 h0 = (__bf16)v0, h1 = (__bf16)v1;
    bf16x2 h, l;
    h[0] = h0;
    h[1] = h1;
    l[0] = (__bf16)(v0 - (float)h0);
    l[1] = (__bf16)(v1 - (float)h1);
    *(bf16x2*)(hi + o) = h;
    *(bf16x2*)(lo + o) = l;
}

struct PfArgs {
    const u32x4* W;   // packed weights [n_tiles][KT][64]
    const u32x4* Xh;  // packed activations [m_tiles][KT][64], hi and lo terms
    const u32x4* Xl;
    int KT, n_tiles, m_tiles;  // valid 16-wide tiles of W and X (loads of tiles beyond them are clamped)
    int n_wgN, n_wgM;
    int M, N;
    const float* ssq;  // [rows][ssq_n] partial sums of squares of the rows of X before their gain, or NULL
    int ssq_n;
    float inv_d, eps;
};

// ---------------------------------------------------------------------------------------------------
// main loop: acc[i][j] (+)= W tile i of this wave x activation tile j (MTL/2 of them), for both terms of the
// activations.  Tile = 256 features x MTL*16 rows; K advances 32 per stage; the stages are filled by direct
// global->LDS copies that run ahead of the MFMAs.
// ---------------------------------------------------------------------------------------------------
// NWAVE waves per workgroup, arranged (NWAVE/2) along the features x 2 along the rows: a wave owns
// WNF = 32/NWAVE weight tiles and MTL/2 row tiles.  A single wave per SIMD cannot issue 16x16x32 MFMAs back to
// back fast enough to keep the matrix core busy, and the more waves share a SIMD the better it is fed: the QKV and
// gate|up GEMMs run 8 waves with two workgroups per CU (four waves per SIMD), and so does the head GEMM; the residual
// GEMMs (a grid of one workgroup per CU at 1024 rows, and an epilogue that needs more registers) run 8 waves with one
// workgroup per CU and a deeper ring.
template <int MTL>
struct PfTile {
    int nt0, mt0, n_wg, wn, wm;
};

template <int MTL, int NWAVE>
__device__ __forceinline__ bool pf_tile_of(const PfArgs& a, PfTile<MTL>& t) {
    // Workgroups are dealt round-robin to the 8 XCDs: give each XCD whole column panels, all row tiles of
    // a panel back to back, so that a weight panel is fetched from HBM once and then served by that XCD's L2.
    const int w = blockIdx.x, xcd = w & 7, j = w >> 3;
    t.n_wg = (j / a.n_wgM) * 8 + xcd;
    const int m_wg = j % a.n_wgM;
    if (t.n_wg >= a.n_wgN) return false;
    t.nt0 = t.n_wg * PF_NTL;
    t.mt0 = m_wg * MTL;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    t.wn = wave % (NWAVE / 2);
    t.wm = wave / (NWAVE / 2);
    return true;
}

// Two ways to keep the matrix cores fed, chosen per kernel (WIDE):
//  - WIDE: two workgroups of 8 waves share a CU (four waves per SIMD, at most 128 registers each): the other
//    workgroup's MFMAs cover this one's barriers and copy waits, so few stages suffice (2 for the 128-row tile, 3
//    for the 64-row tile, which also has room for a second operand set in registers);
//  - otherwise one workgroup per CU with four stages and two operand sets (the residual epilogue needs the registers).
// The head GEMM (4 waves, two workgroups per CU, 2 stages) is its own case.
// (LO = false: the activations' hi term only, 24 KB instead of 32 KB per stage of the 128-row tile, so three stages fit twice)
template <int MTL, int NWAVE, bool WIDE, bool LO = true>
constexpr int pf_stages() {
    return NWAVE == 4 ? 2 : (WIDE ? (MTL == 8 && LO ? 2 : 3) : 4);
}
template <int MTL, int NWAVE, bool WIDE>
constexpr bool pf_pipe() {  // (the residual epilogue overrides this for its two-workgroups-per-CU variant)
    return NWAVE == 8 && MTL == 4;
}

// The operand reads and the wait counts are written by hand: the compiler would make every LDS read wait
// for ALL outstanding global->LDS copies (it cannot tell which buffer a copy targets), which would
// serialise the stages.  vmcnt counts this wave's copies in issue order: stage kt has landed once at most
// (stages - 2) * FPW younger copies are still in flight.
#define PF_DSR(dst, base, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(base), "n"(off))

template <int N>
__device__ __forceinline__ void pf_wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int MTL, int NWAVE, bool WIDE, bool PIPE = pf_pipe<MTL, NWAVE, WIDE>(), bool LO = true>
__device__ __forceinline__ void pf_mainloop(const PfArgs& a, const PfTile<MTL>& t, u32x4* lds, float* rs,
                                            f32x4 (&acc)[32 / NWAVE][MTL / 2]) {
    constexpr int WNF = 32 / NWAVE;
    constexpr int NF = PF_NTL + (LO ? 2 : 1) * MTL;  // fragments (1 KB each) per stage
    constexpr int FPW = NF / NWAVE;                  // copied per wave
    constexpr int NST = pf_stages<MTL, NWAVE, WIDE, LO>();
    static_assert(LO || !PIPE, "the single-term loop has one operand set");
    static_assert(NF % NWAVE == 0, "fragments must divide over the waves");
    static_assert((NST - 2) * FPW < 64, "vmcnt range");
    constexpr int STAGE = NF * 64;        // u32x4 per stage
    constexpr int MW = MTL / 2;
    static_assert(MW == 2 || MW == 4, "row tiles per wave");
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int KT = a.KT;
    const u32x4* src[FPW];
#pragma unroll
    for (int i = 0; i < FPW; ++i) {
        const int f = wave * FPW + i;
        if (f < PF_NTL) {
            int tt = t.nt0 + f;
            if (tt >= a.n_tiles) tt = a.n_tiles - 1;
            src[i] = a.W + (size_t)tt * KT * 64 + lane;
        } else {
            const int g = f - PF_NTL;  // (g < MTL always in the single-term loop)
            int mt = t.mt0 + (g < MTL ? g : g - MTL);
            if (mt >= a.m_tiles) mt = a.m_tiles - 1;
            src[i] = (g < MTL ? a.Xh : a.Xl) + (size_t)mt * KT * 64 + lane;
        }
    }
    auto issue = [&](int st, int kt) {
#pragma unroll
        for (int i = 0; i < FPW; ++i)
            __builtin_amdgcn_global_load_lds(EE_GLB_PTR(src[i] + (size_t)kt * 64), EE_LDS_PTR(lds + st * STAGE + (wave * FPW + i) * 64), 16,
                                             0, 0);
    };
    // r[m] = 1/sqrt(mean(x^2)+eps) of this tile's rows, from the producers' partial sums (fixed order)
    for (int ml = threadIdx.x; ml < MTL * 16; ml += blockDim.x) {
        const int m = t.mt0 * 16 + ml;
        float r = 1.f;
        if (a.ssq != nullptr && m < a.M) {
            const float* p = a.ssq + (size_t)m * a.ssq_n;
            float s = 0.f;
            for (int i = 0; i < a.ssq_n; ++i) s += p[i];
            r = 1.0f / sqrtf(s * a.inv_d + a.eps);
        }
        rs[ml] = r;
    }
#pragma unroll
    for (int i = 0; i < WNF; ++i)
#pragma unroll
        for (int j = 0; j < MW; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    // (the copy count per iteration is kept uniform: beyond the last stage the last one is fetched again
    // into a buffer nobody reads any more)
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) issue(p, p < KT ? p : KT - 1);
    const unsigned lds0 = (unsigned)(size_t)EE_LDS_PTR(lds) + lane * 16;
    const unsigned woff = t.wn * WNF * 1024, xoff = (PF_NTL + t.wm * MW) * 1024;
    int st_r = 0, st_w = NST - 1;
    struct Frags {
        u32x4 wf[WNF], xh[MW], xl[MW];
    };
    // front half of a k-tile: wait until its stage has landed for everybody, start the operand reads of this wave
    // and refill the buffer that was read one k-tile earlier
    auto fetch = [&](Frags& f, int kt) {
        pf_wait_vm<(NST - 2) * FPW>();     // this wave's copies of stage kt have landed
        __builtin_amdgcn_s_barrier();      // ... and everybody else's; the buffer refilled below is no longer read
        const unsigned wb = lds0 + st_r * (STAGE * 16) + woff, xb = lds0 + st_r * (STAGE * 16) + xoff;
        PF_DSR(f.wf[0], wb, 0); PF_DSR(f.wf[1], wb, 1024); PF_DSR(f.wf[2], wb, 2048); PF_DSR(f.wf[3], wb, 3072);
        if constexpr (WNF == 8) {
            PF_DSR(f.wf[4], wb, 4096); PF_DSR(f.wf[5], wb, 5120); PF_DSR(f.wf[6], wb, 6144); PF_DSR(f.wf[7], wb, 7168);
        }
        PF_DSR(f.xh[0], xb, 0); PF_DSR(f.xh[1], xb, 1024);
        if constexpr (MW == 4) {
            PF_DSR(f.xh[2], xb, 2048); PF_DSR(f.xh[3], xb, 3072);
        }
        if constexpr (LO) {
            PF_DSR(f.xl[0], xb, MTL * 1024); PF_DSR(f.xl[1], xb, MTL * 1024 + 1024);
            if constexpr (MW == 4) {
                PF_DSR(f.xl[2], xb, MTL * 1024 + 2048); PF_DSR(f.xl[3], xb, MTL * 1024 + 3072);
            }
        }
        issue(st_w, kt + NST - 1 < KT ? kt + NST - 1 : KT - 1);
        st_r = st_r + 1 == NST ? 0 : st_r + 1;
        st_w = st_w + 1 == NST ? 0 : st_w + 1;
    };
    // the operands are in registers after this (and the MFMAs that use them may not move above it)
    auto landed = [&](Frags& f) {
        if constexpr (!LO) {
            static_assert(LO || (WNF == 4 && MW == 4), "single-term loop: 8 waves on the 128-row tile");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.xh[0]), "+v"(f.xh[1]),
                         "+v"(f.xh[2]), "+v"(f.xh[3]));
        } else if constexpr (WNF == 8 && MW == 4)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.wf[4]), "+v"(f.wf[5]),
                         "+v"(f.wf[6]), "+v"(f.wf[7]), "+v"(f.xh[0]), "+v"(f.xh[1]), "+v"(f.xh[2]), "+v"(f.xh[3]), "+v"(f.xl[0]),
                         "+v"(f.xl[1]), "+v"(f.xl[2]), "+v"(f.xl[3]));
        else if constexpr (WNF == 8)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.wf[4]), "+v"(f.wf[5]),
                         "+v"(f.wf[6]), "+v"(f.wf[7]), "+v"(f.xh[0]), "+v"(f.xh[1]), "+v"(f.xl[0]), "+v"(f.xl[1]));
        else if constexpr (MW == 4)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.xh[0]), "+v"(f.xh[1]),
                         "+v"(f.xh[2]), "+v"(f.xh[3]), "+v"(f.xl[0]), "+v"(f.xl[1]), "+v"(f.xl[2]), "+v"(f.xl[3]));
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.xh[0]), "+v"(f.xh[1]),
                         "+v"(f.xl[0]), "+v"(f.xl[1]));
    };
    auto multiply_lo = [&](const Frags& f) {
#pragma unroll
        for (int i = 0; i < WNF; ++i)
#pragma unroll
            for (int j = 0; j < MW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.wf[i]), __builtin_bit_cast(bf16x8, f.xl[j]),
                                                                    acc[i][j], 0, 0, 0);
    };
    auto multiply_hi = [&](const Frags& f) {
#pragma unroll
        for (int i = 0; i < WNF; ++i)
#pragma unroll
            for (int j = 0; j < MW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.wf[i]), __builtin_bit_cast(bf16x8, f.xh[j]),
                                                                    acc[i][j], 0, 0, 0);
    };
    if constexpr (PIPE) {
        // One workgroup per CU: its eight waves pass the barrier together, so with reads and MFMAs of the same k-tile
        // back to back the LDS and the matrix cores would take turns.  Two register sets instead: the operand reads of
        // k-tile kt+1 are in flight while the MFMAs of k-tile kt run, and the barrier that guards them sits in the
        // middle of that MFMA stream (after the lo-term half), so the matrix core has queued work while the waves meet.
        Frags fa, fb;
        fetch(fa, 0);
        landed(fa);
        for (int kt = 0; kt < KT; kt += 2) {
            multiply_lo(fa);
            __builtin_amdgcn_sched_barrier(0);
            if (kt + 1 < KT) fetch(fb, kt + 1);
            __builtin_amdgcn_sched_barrier(0);
            multiply_hi(fa);
            __builtin_amdgcn_sched_barrier(0);
            if (kt + 1 >= KT) break;
            landed(fb);
            multiply_lo(fb);
            __builtin_amdgcn_sched_barrier(0);
            if (kt + 2 < KT) fetch(fa, kt + 2);
            __builtin_amdgcn_sched_barrier(0);
            multiply_hi(fb);
            __builtin_amdgcn_sched_barrier(0);
            if (kt + 2 < KT) landed(fa);
        }
    } else {
        // two workgroups per CU: the other workgroup's MFMAs cover this one's reads (also taken where the second
        // register set would not fit)
        for (int kt = 0; kt < KT; ++kt) {
            Frags f;
            fetch(f, kt);
            landed(f);
            if constexpr (LO) multiply_lo(f);
            multiply_hi(f);
        }
    }
    pf_wait_vm<0>();  // the surplus copies too, before the epilogue reuses the stage buffers
    __syncthreads();  // (also makes rs[] visible)
}

constexpr int PFK_NF = 2 * (PF_NTL + 8);  // fragments per stage: two k-tiles of 16 weight and 4 + 4 activation fragments
constexpr int PFK_NST = 3;
constexpr size_t pfk_lds_bytes() { return (size_t)PFK_NST * PFK_NF * 1024 + 64 * 4 * 8; }
__device__ __forceinline__ float* pfk_rs_ptr(u32x4* lds) { return (float*)(lds + PFK_NST * PFK_NF * 64); }

// ---------------------------------------------------------------------------------------------------
// Main loop for a 64-row tile on a grid of one workgroup per CU: 16 waves, i.e. four per SIMD like the wide
// kernels, as 4 (features) x 2 (rows) x 2 (halves of K).  A stage holds two k-tiles; wave group kh works on k-tile
// 2s + kh with the wave tile of the plain main loop (4 weight tiles x 2 row tiles).  At the end the upper group
// hands its accumulators to the lower one through LDS (fixed order: lower half of K first); only waves 0..7 leave
// with sums, in the layout of the plain main loop with 8 waves.  KT must be even.
// ---------------------------------------------------------------------------------------------------
constexpr int PF16_FPW = PFK_NF / 16;

__device__ __forceinline__ void pf_mainloop_k16(const PfArgs& a, const PfTile<4>& t, int kh, u32x4* lds, float* rs, f32x4 (&acc)[4][2]) {
    constexpr int MTL = 4, NST = PFK_NST, FPW = PF16_FPW, HALF = PFK_NF / 2;
    constexpr int STAGE = PFK_NF * 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int KT = a.KT, KS = KT >> 1;
    const u32x4* src[FPW];
#pragma unroll
    for (int i = 0; i < FPW; ++i) {
        const int f = wave * FPW + i, fh = f / HALF, g = f % HALF;
        if (g < PF_NTL) {
            int tt = t.nt0 + g;
            if (tt >= a.n_tiles) tt = a.n_tiles - 1;
            src[i] = a.W + ((size_t)tt * KT + fh) * 64 + lane;
        } else {
            const int r = g - PF_NTL;
            int mt = t.mt0 + (r < MTL ? r : r - MTL);
            if (mt >= a.m_tiles) mt = a.m_tiles - 1;
            src[i] = (r < MTL ? a.Xh : a.Xl) + ((size_t)mt * KT + fh) * 64 + lane;
        }
    }
    auto issue = [&](int st, int s) {
#pragma unroll
        for (int i = 0; i < FPW; ++i)
            __builtin_amdgcn_global_load_lds(EE_GLB_PTR(src[i] + (size_t)s * 128), EE_LDS_PTR(lds + st * STAGE + (wave * FPW + i) * 64), 16,
                                             0, 0);
    };
    for (int ml = threadIdx.x; ml < MTL * 16; ml += blockDim.x) {
        const int m = t.mt0 * 16 + ml;
        float r = 1.f;
        if (a.ssq != nullptr && m < a.M) {
            const float* p = a.ssq + (size_t)m * a.ssq_n;
            float sum = 0.f;
            for (int i = 0; i < a.ssq_n; ++i) sum += p[i];
            r = 1.0f / sqrtf(sum * a.inv_d + a.eps);
        }
        rs[ml] = r;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) issue(p, p < KS ? p : KS - 1);
    const unsigned lds0 = (unsigned)(size_t)EE_LDS_PTR(lds) + lane * 16;
    const unsigned woff = (kh * HALF + t.wn * 4) * 1024, xoff = (kh * HALF + PF_NTL + t.wm * 2) * 1024;
    int st_r = 0, st_w = NST - 1;
    for (int s = 0; s < KS; ++s) {
        u32x4 wf[4], xh[2], xl[2];
        pf_wait_vm<(NST - 2) * FPW>();
        __builtin_amdgcn_s_barrier();
        const unsigned wb = lds0 + st_r * (STAGE * 16) + woff, xb = lds0 + st_r * (STAGE * 16) + xoff;
        PF_DSR(wf[0], wb, 0); PF_DSR(wf[1], wb, 1024); PF_DSR(wf[2], wb, 2048); PF_DSR(wf[3], wb, 3072);
        PF_DSR(xh[0], xb, 0); PF_DSR(xh[1], xb, 1024);
        PF_DSR(xl[0], xb, 4096); PF_DSR(xl[1], xb, 5120);
        issue(st_w, s + NST - 1 < KS ? s + NST - 1 : KS - 1);
        st_r = st_r + 1 == NST ? 0 : st_r + 1;
        st_w = st_w + 1 == NST ? 0 : st_w + 1;
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[0]), "+v"(wf[1]), "+v"(wf[2]), "+v"(wf[3]), "+v"(xh[0]), "+v"(xh[1]), "+v"(xl[0]),
                     "+v"(xl[1]));
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, xl[j]),
                                                                    acc[i][j], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i]), __builtin_bit_cast(bf16x8, xh[j]),
                                                                    acc[i][j], 0, 0, 0);
    }
    pf_wait_vm<0>();
    __syncthreads();  // every copy has landed and every operand read is done: the stage buffers are free (rs[] is visible)
    f32x4* xch = (f32x4*)lds;  // [wave 0..7][8][64 lanes]
    if (kh == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) xch[(((wave & 7) * 8) + i * 2 + j) * 64 + lane] = acc[i][j];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] += xch[((wave * 8) + i * 2 + j) * 64 + lane];
    }
    __syncthreads();  // before the epilogue reuses the buffers
}

template <int MTL, int NWAVE, bool WIDE, bool LO = true>
constexpr size_t pf_lds_bytes() {  // the stages + rs[] + up to seven reduction rows
    return pf_stages<MTL, NWAVE, WIDE, LO>() * (size_t)(PF_NTL + (LO ? 2 : 1) * MTL) * 1024 + (size_t)MTL * 16 * 4 * 8;
}

template <int MTL, int NWAVE, bool WIDE, bool LO = true>
__device__ __forceinline__ float* pf_rs_ptr(u32x4* lds) {
    return (float*)(lds + pf_stages<MTL, NWAVE, WIDE, LO>() * (PF_NTL + (LO ? 2 : 1) * MTL) * 64);
}

// ---- epilogue 1: RMS scale, rotary embedding, q (packed), k and v into the paged cache
struct PfQkv {
    __bf16 *q_hi, *q_lo;  // packed [rows][d]
    int d, H, hd;
    const float2* rope_cs;
    __bf16* kv_layer;
    size_t blk_stride;
    int BT;
    const int32_t* bt;  // block table of the sequence
    int p0;             // position of row 0 (multiple of 16)
};

template <int MTL, int NWAVE>
__global__ __launch_bounds__(NWAVE * 64, NWAVE == 8 ? 4 : 2) void pf_qkv_kernel(PfArgs a, PfQkv e) {
    extern __shared__ u32x4 pf_lds[];
    PfTile<MTL> t;
    if (!pf_tile_of<MTL, NWAVE>(a, t)) return;
    constexpr int WNF = 32 / NWAVE;
    constexpr int MW = MTL / 2;
    float* rs = pf_rs_ptr<MTL, NWAVE, true>(pf_lds);
    const int tiles_per_part = e.d / 16, per_head = e.hd / 16, half = e.hd / 2;
    f32x4 acc[WNF][MW];
    pf_mainloop<MTL, NWAVE, true>(a, t, pf_lds, rs, acc);
    const int lane = threadIdx.x & 63, li = lane & 15, rg = lane >> 4;
    const int KTd = e.d / 32;
    // (row tiles outside, weight tiles inside: what depends on the position alone, its cache block, its place in the
    // block and its RMS scale, is formed once per row instead of once per tile)
#pragma unroll
    for (int j = 0; j < MW; ++j) {
        const int ml = (t.wm * MW + j) * 16 + li, m = t.mt0 * 16 + ml;
        if (m >= a.M) continue;
        const float r = rs[ml];
        const int pos = e.p0 + m;
        const int blk = e.bt[pos / e.BT], pin = pos % e.BT;
        const bool is_hi = rg >= 2;
#pragma unroll
        for (int i = 0; i < WNF; ++i) {
            const int T = t.nt0 + t.wn * WNF + i;
            if (T >= a.n_tiles) continue;  // (uniform over the wave)
            const int part = T / tiles_per_part, rem = T % tiles_per_part;
            const int h = rem / per_head, c = rem % per_head;
            if (part < 2) {
                // lane: features rg*4..rg*4+3 of the tile (rows 0-7 = features c*8.., rows 8-15 = their rotary
                // partners) for position m
                f32x4 v = acc[i][j] * r;
                f32x4 o;
                // (a lane swap instead of this shuffle costs the kernel eight more live registers, which it does not have:
                // 48 spilled, four times the run time)
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = __shfl_xor(v[q], 32);
                const int fi = c * 8 + (rg & 1) * 4;
                const f32x4 cs0 = *(const f32x4*)(e.rope_cs + (size_t)pos * half + fi);
                const f32x4 cs1 = *(const f32x4*)(e.rope_cs + (size_t)pos * half + fi + 2);
                const float cx[4] = {cs0[0], cs0[2], cs1[0], cs1[2]}, sx[4] = {cs0[1], cs0[3], cs1[1], cs1[3]};
                float res[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) res[q] = is_hi ? v[q] * cx[q] + o[q] * sx[q] : v[q] * cx[q] - o[q] * sx[q];
                const int f = fi + (is_hi ? half : 0);
                if (part == 0) {
                    pk_store4(e.q_hi, e.q_lo, m, h * e.hd + f, KTd, res);
                } else {
                    __bf16* kp = e.kv_layer + (size_t)blk * e.blk_stride + ((size_t)h * e.BT + pin) * e.hd + f;
                    bf16x4 kb;
#pragma unroll
                    for (int q = 0; q < 4; ++q) kb[q] = (__bf16)res[q];
                    *(bf16x4*)kp = kb;
                }
            } else {
                // V block, transposed [head][position / 32][feature][position % 32]: four 2-byte stores per lane; the
                // 16 lanes of a group cover 16 consecutive positions of one feature
                const int f = c * 8 + (rg & 1) * 4 + (is_hi ? half : 0);
                __bf16* vp = e.kv_layer + (size_t)blk * e.blk_stride + (size_t)e.H * e.BT * e.hd + (size_t)h * e.hd * e.BT +
                             (size_t)(pin >> 5) * (e.hd * 32) + f * 32 + (pin & 31);
#pragma unroll
                for (int q = 0; q < 4; ++q) vp[q * 32] = (__bf16)(acc[i][j][q] * r);
            }
        }
    }
}

// ---- epilogue 2: residual add; operand(s) of what follows; sum-of-squares partial per (row, workgroup)
struct PfResid {
    float* x;  // [rows][d] fp32
    __bf16 *xg_hi, *xg_lo, *xgh_hi, *xgh_lo;  // packed [rows][d]; xgh optional
    const float *g_next, *g_head;
    float* ssq_out;  // [rows][ssq_n_out]
    int ssq_n_out, d;
};

// (waves with active == false hold no sums: they only keep the barriers company)
template <int MTL, int NWAVE>
__device__ __forceinline__ void pf_resid_epilogue(const PfArgs& a, const PfResid& e, const PfTile<MTL>& t, const float* rs, float* red,
                                                  const f32x4 (&acc)[32 / NWAVE][MTL / 2], bool active = true) {
    constexpr int WNF = 32 / NWAVE;
    constexpr int MW = MTL / 2;
    const int lane = threadIdx.x & 63, li = lane & 15, rg = lane >> 4;
    const int KTd = e.d / 32;
    float sq[MW];
#pragma unroll
    for (int j = 0; j < MW; ++j) sq[j] = 0.f;
#pragma unroll
    for (int i = 0; i < WNF; ++i) {
        const int T = t.nt0 + t.wn * WNF + i;
        if (T >= a.n_tiles || !active) continue;
        const int n = T * 16 + rg * 4;
        const f32x4 gn = *(const f32x4*)(e.g_next + n);
        f32x4 gh = f32x4{0.f, 0.f, 0.f, 0.f};
        if (e.g_head) gh = *(const f32x4*)(e.g_head + n);
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            const int ml = (t.wm * MW + j) * 16 + li, m = t.mt0 * 16 + ml;
            if (m >= a.M) continue;
            float* xp = e.x + (size_t)m * e.d + n;
            f32x4 v = *(const f32x4*)xp;
            const float r = a.ssq ? rs[ml] : 1.f;
            v += acc[i][j] * r;
            *(f32x4*)xp = v;
            float o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o[q] = v[q] * gn[q];
                sq[j] += v[q] * v[q];
            }
            pk_store4(e.xg_hi, e.xg_lo, m, n, KTd, o);
            if (e.g_head) {
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = v[q] * gh[q];
                pk_store4(e.xgh_hi, e.xgh_lo, m, n, KTd, o);
            }
        }
    }
    // sum of squares of this workgroup's 256 columns per row: over the four lane groups, then the waves along the features
#pragma unroll
    for (int j = 0; j < MW; ++j) {
        float s = sq[j];
        s = rows4_sum(s);
        if (rg == 0 && active) red[t.wn * (MTL * 16) + (t.wm * MW + j) * 16 + li] = s;
    }
    __syncthreads();
    for (int ml = threadIdx.x; ml < MTL * 16; ml += blockDim.x) {
        const int m = t.mt0 * 16 + ml;
        if (m < a.M) {
            float sum = red[ml];
#pragma unroll
            for (int wv = 1; wv < NWAVE / 2; ++wv) sum += red[wv * (MTL * 16) + ml];
            e.ssq_out[(size_t)m * e.ssq_n_out + t.n_wg] = sum;
        }
    }
}

template <int MTL, int NWAVE, bool WIDE = false>
__global__ __launch_bounds__(NWAVE * 64, WIDE ? 4 : 2) void pf_resid_kernel(PfArgs a, PfResid e) {
    extern __shared__ u32x4 pf_lds[];
    PfTile<MTL> t;
    if (!pf_tile_of<MTL, NWAVE>(a, t)) return;
    float* rs = pf_rs_ptr<MTL, NWAVE, WIDE>(pf_lds);
    float* red = rs + MTL * 16;  // [NWAVE/2][MTL*16]
    f32x4 acc[32 / NWAVE][MTL / 2];
    pf_mainloop<MTL, NWAVE, WIDE, (!WIDE && MTL == 4)>(a, t, pf_lds, rs, acc);  // (two operand sets need 152 registers here)
    pf_resid_epilogue<MTL, NWAVE>(a, e, t, rs, red, acc);
}

// 64-row tile, one workgroup of 16 waves per CU, the contraction split over two wave groups
__global__ __launch_bounds__(1024, 4) void pf_resid_k16_kernel(PfArgs a, PfResid e) {
    extern __shared__ u32x4 pf_lds[];
    PfTile<4> t;
    if (!pf_tile_of<4, 8>(a, t)) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kh = wave >> 3;
    t.wn = (wave & 7) % 4;
    t.wm = (wave & 7) / 4;
    float* rs = pfk_rs_ptr(pf_lds);
    float* red = rs + 64;
    f32x4 acc[4][2];
    pf_mainloop_k16(a, t, kh, pf_lds, rs, acc);
    pf_resid_epilogue<4, 8>(a, e, t, rs, red, acc, kh == 0);
}

// ---- epilogue 3: SwiGLU.  Tile j of the packed gate|up matrix: rows 0-7 gate features 8j.., rows 8-15 the up features
template <int MTL, int NWAVE>
__global__ __launch_bounds__(NWAVE * 64, NWAVE == 8 ? 4 : 2) void pf_swiglu_kernel(PfArgs a, __bf16* act_hi, __bf16* act_lo, int F) {
    extern __shared__ u32x4 pf_lds[];
    PfTile<MTL> t;
    if (!pf_tile_of<MTL, NWAVE>(a, t)) return;
    constexpr int WNF = 32 / NWAVE;
    constexpr int MW = MTL / 2;
    float* rs = pf_rs_ptr<MTL, NWAVE, true>(pf_lds);
    f32x4 acc[WNF][MW];
    pf_mainloop<MTL, NWAVE, true>(a, t, pf_lds, rs, acc);
    const int lane = threadIdx.x & 63, li = lane & 15, rg = lane >> 4;
    const int KTf = F / 32;
#pragma unroll
    for (int i = 0; i < WNF; ++i) {
        const int T = t.nt0 + t.wn * WNF + i;
        if (T >= a.n_tiles) continue;
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            const int ml = (t.wm * MW + j) * 16 + li, m = t.mt0 * 16 + ml;
            const f32x4 v = acc[i][j] * rs[ml];
            // The gate features sit in the lower 32 lanes, their up partners in the upper 32.  Both halves get both
            // (a lane swap each) and share the work: the lower half forms features 0 and 1 of its four, the upper
            // half 2 and 3.  Hardware exponential and reciprocal (a few 1e-7 relative: the results are kept to 16
            // mantissa bits); with the library routines and one half idle this epilogue was 8 % of the kernel.
            float gq[4], uq[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) halves_of(v[q], gq[q], uq[q]);
            const bool upper = rg >= 2;
            const float g0 = upper ? gq[2] : gq[0], g1 = upper ? gq[3] : gq[1];
            const float u0 = upper ? uq[2] : uq[0], u1 = upper ? uq[3] : uq[1];
            if (m < a.M)
                pk_store2(act_hi, act_lo, m, T * 8 + (rg & 1) * 4 + (upper ? 2 : 0), KTf, __fdividef(g0, 1.0f + __expf(-g0)) * u0,
                          __fdividef(g1, 1.0f + __expf(-g1)) * u1);
        }
    }
}

// ---- epilogue 4: a head on every row: per (row, workgroup) max, arg max and sum of exponentials of its 256 logits
struct PfHead {
    HeadPartial* partials;  // [rows][n_wgN]
    int V;
    const int32_t* target;  // per row: the token whose logit is wanted (negative: none), or NULL
    float* target_logit;    // per row: that logit
};

__device__ __forceinline__ void pf_merge(float& m, float& s, int& i, float m2, float s2, int i2) {
    if (m2 > m || (m2 == m && i2 < i)) {
        s = s * __expf(m - m2) + s2;
        m = m2;
        i = i2;
    } else if (m2 > -INFINITY) {
        s = s + s2 * __expf(m2 - m);
    }
}

template <int MTL, int NWAVE, bool LO>
__global__ __launch_bounds__(NWAVE * 64, NWAVE == 8 ? 4 : 2) void pf_head_kernel(PfArgs a, PfHead e) {
    extern __shared__ u32x4 pf_lds[];
    PfTile<MTL> t;
    if (!pf_tile_of<MTL, NWAVE>(a, t)) return;
    constexpr int WNF = 32 / NWAVE;
    constexpr int MW = MTL / 2;
    float* rs = pf_rs_ptr<MTL, NWAVE, (NWAVE == 8), LO>(pf_lds);
    constexpr int WN = NWAVE / 2;        // waves along the features
    float* red = rs + MTL * 16;          // waves wn > 0 hand (max, sum) over here: [2 * (wn - 1) + {0, 1}][MTL * 16]
    f32x4 acc[WNF][MW];
    pf_mainloop<MTL, NWAVE, (NWAVE == 8), false, LO>(a, t, pf_lds, rs, acc);
    int* redi = (int*)pf_lds;            // ... and the index here (the stage buffers are free now): [wn - 1][MTL * 16]
    const int lane = threadIdx.x & 63, li = lane & 15, rg = lane >> 4;
    float mxs[MW], sms[MW];
    int ixs[MW];
#pragma unroll
    for (int j = 0; j < MW; ++j) {
        const int ml = (t.wm * MW + j) * 16 + li;
        const float r = rs[ml];
        float mx = -INFINITY, sm = 0.f;
        int ix = 0x7fffffff;
        const int m_row = t.mt0 * 16 + ml;
        const int tgt = (e.target != nullptr && m_row < a.M) ? e.target[m_row] : -1;
#pragma unroll
        for (int i = 0; i < WNF; ++i) {
            const int n = (t.nt0 + t.wn * WNF + i) * 16 + rg * 4;
            if (n >= e.V) continue;
            acc[i][j] = acc[i][j] * r;  // the logits, in place
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float z = acc[i][j][q];
                if (z > mx) {
                    mx = z;
                    ix = n + q;
                }
            }
            if ((unsigned)(tgt - n) < 4u) {  // (exactly one lane of one workgroup holds the wanted token's logit)
                const int q = tgt - n;
                e.target_logit[m_row] = q == 0 ? acc[i][j][0] : q == 1 ? acc[i][j][1] : q == 2 ? acc[i][j][2] : acc[i][j][3];
            }
        }
        // (hardware exponential: relative error about 1e-6, far inside what the logits themselves carry; the library
        // routine made this epilogue a ninth of the kernel)
#pragma unroll
        for (int i = 0; i < WNF; ++i) {
            const int n = (t.nt0 + t.wn * WNF + i) * 16 + rg * 4;
            if (n >= e.V) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) sm += __expf(acc[i][j][q] - mx);
        }
        // the four lane groups of a row, in a fixed order (even row then odd row, lower half then upper half: every
        // lane forms the same merge, so all four groups end up equal)
        {
            float m0, m1, s0, s1, i0, i1;
            row_pair_of(mx, m0, m1);
            row_pair_of(sm, s0, s1);
            row_pair_of(__int_as_float(ix), i0, i1);
            int ia = __float_as_int(i0);
            pf_merge(m0, s0, ia, m1, s1, __float_as_int(i1));
            halves_of(m0, mx, m1);
            halves_of(s0, sm, s1);
            halves_of(__int_as_float(ia), i0, i1);
            ix = __float_as_int(i0);
            pf_merge(mx, sm, ix, m1, s1, __float_as_int(i1));
        }
        if (t.wn > 0 && rg == 0) {
            red[(2 * (t.wn - 1)) * (MTL * 16) + ml] = mx;
            red[(2 * (t.wn - 1) + 1) * (MTL * 16) + ml] = sm;
            redi[(t.wn - 1) * (MTL * 16) + ml] = ix;
        }
        mxs[j] = mx, sms[j] = sm, ixs[j] = ix;
    }
    __syncthreads();  // (one hand-over for all row tiles: their slots are disjoint)
    if (t.wn == 0 && rg == 0) {
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            const int ml = (t.wm * MW + j) * 16 + li;
            float mx = mxs[j], sm = sms[j];
            int ix = ixs[j];
#pragma unroll
            for (int wv = 1; wv < WN; ++wv)
                pf_merge(mx, sm, ix, red[(2 * (wv - 1)) * (MTL * 16) + ml], red[(2 * (wv - 1) + 1) * (MTL * 16) + ml],
                         redi[(wv - 1) * (MTL * 16) + ml]);
            const int m = t.mt0 * 16 + ml;
            if (m < a.M) {
                HeadPartial p;
                p.max = mx;
                p.sum = sm;
                p.idx = ix;
                p.pad = 0;
                e.partials[(size_t)m * a.n_wgN + t.n_wg] = p;
            }
        }
    }
}

// one wave per row: merges the row's partials in workgroup order; token = arg max, confidence = 1 / sum exp(z - max)
// and, where a target token is given, nll = log sum exp(z) - z[target]
__global__ __launch_bounds__(64) void pf_head_merge_kernel(const HeadPartial* __restrict__ partials, int n_wg, int M,
                                                           int32_t* __restrict__ tok, float* __restrict__ conf,
                                                           const int32_t* __restrict__ target, const float* __restrict__ target_logit,
                                                           float* __restrict__ nll) {
    const int m = blockIdx.x, lane = threadIdx.x;
    if (m >= M) return;
    float mx = -INFINITY, sm = 0.f;
    int ix = 0x7fffffff;
    for (int w = lane; w < n_wg; w += 64) {
        const HeadPartial p = partials[(size_t)m * n_wg + w];
        pf_merge(mx, sm, ix, p.max, p.sum, p.idx);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float m2 = __shfl_xor(mx, o), s2 = __shfl_xor(sm, o);
        const int i2 = __shfl_xor(ix, o);
        if (lane & o) {
            float m1 = m2, s1 = s2;
            int i1 = i2;
            pf_merge(m1, s1, i1, mx, sm, ix);
            mx = m1;
            sm = s1;
            ix = i1;
        } else {
            pf_merge(mx, sm, ix, m2, s2, i2);
        }
    }
    if (lane == 0) {
        tok[m] = ix;
        conf[m] = 1.0f / sm;
        if (nll != nullptr) nll[m] = (target != nullptr && target[m] >= 0) ? (logf(sm) + mx) - target_logit[m] : 0.f;
    }
}

// ---- embedding rows -> residual stream, operand of layer 1, sum-of-squares partials (one per 256 columns)
__global__ __launch_bounds__(256) void pf_embed_kernel(const __bf16* __restrict__ embed, const int32_t* __restrict__ tokens, int d,
                                                       const float* __restrict__ g_next, float* __restrict__ x,
                                                       __bf16* __restrict__ xg_hi, __bf16* __restrict__ xg_lo,
                                                       float* __restrict__ ssq, int ssq_n) {
    __shared__ float red[4];
    const int m = blockIdx.x, KTd = d / 32;
    const __bf16* er = embed + (size_t)tokens[m] * d;
    for (int c0 = 0, part = 0; c0 < d; c0 += 256, ++part) {
        const int col = c0 + threadIdx.x;
        float v = 0.f;
        if (col < d) {
            v = (float)er[col];
            x[(size_t)m * d + col] = v;
            const float o = v * g_next[col];
            const __bf16 h = (__bf16)o;
            const size_t pi = pk_index(m, col, KTd);
            xg_hi[pi] = h;
            xg_lo[pi] = (__bf16)(o - (float)h);
        }
        float s = v * v;
        s = wave_sum(s);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
        __syncthreads();
        if (threadIdx.x == 0) ssq[(size_t)m * ssq_n + part] = (red[0] + red[1]) + (red[2] + red[3]);
        __syncthreads();
    }
}

// ---- one row of the residual stream handed to the decode-side residual store (row-major operands, one
// sum-of-squares entry holding the whole sum), so that the decode heads can run on it
__global__ __launch_bounds__(256) void pf_export_row_kernel(const float* __restrict__ x, int d, const float* __restrict__ g_a,
                                                            const float* __restrict__ g_b, float* __restrict__ dx,
                                                            __bf16* __restrict__ dxg, __bf16* __restrict__ dxgh, size_t lo_off,
                                                            float* __restrict__ dssq, int ssq_stride) {
    __shared__ float red[4];
    float s = 0.f;
    for (int col = threadIdx.x; col < d; col += 256) {
        const float v = x[col];
        dx[col] = v;
        float o = v * g_a[col];
        __bf16 h = (__bf16)o;
        dxg[col] = h;
        dxg[lo_off + col] = (__bf16)(o - (float)h);
        if (g_b) {
            o = v * g_b[col];
            h = (__bf16)o;
            dxgh[col] = h;
            dxgh[lo_off + col] = (__bf16)(o - (float)h);
        }
        s += v * v;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    for (int i = threadIdx.x; i < ssq_stride; i += 256) dssq[i] = i == 0 ? (red[0] + red[1]) + (red[2] + red[3]) : 0.f;
}

// ---------------------------------------------------------------------------------------------------
// causal attention over many query rows of one sequence.  A block of 64 consecutive query positions of one
// head (16 per wave, four waves) walks the keys 0 .. its last position in tiles of 32.  The work of a block
// grows with its position, so a workgroup takes two: waves 0-3 the j-th block from the end, waves 4-7 the
// j-th from the start, which makes every workgroup (and, a wave of each block per SIMD, every SIMD) carry the
// same number of key tiles; the lighter block's keys are a prefix of the heavier one's, so both read the
// same tiles.  Each K / V^T tile is copied once per workgroup from the paged cache into LDS, already permuted
// into MFMA operand order by the copy's source addressing (so that the reads back are plain 1 KB wave reads
// without bank conflicts), through a ring of stages that keeps several tiles in flight; the arithmetic is the
// decode kernel's (S^T = K Q^T so that P^T is already a B operand; q and P as two bf16 terms).
// ---------------------------------------------------------------------------------------------------
constexpr int PFA_STAGES = 4;

template <int HD>
__global__ __launch_bounds__(512) void pf_attn_kernel(const u32x4* __restrict__ q_hi, const u32x4* __restrict__ q_lo,
                                                      __bf16* __restrict__ out_hi, __bf16* __restrict__ out_lo,
                                                      const __bf16* __restrict__ layer_base, KvGeom kv,
                                                      const int32_t* __restrict__ bt, int p0, int M, int d) {
    constexpr int KK = HD / 32, CG = HD / 16;
    constexpr int NCH = 2 * KK + CG;     // 1 KB chunks per tile: K score halves x k-steps, then V feature groups
    constexpr int NCW = NCH >= 8 ? 8 : 4;  // waves that copy
    constexpr int FPW = NCH / NCW;       // copied per such wave
    constexpr int STAGE = NCH * 64;      // u32x4
    static_assert(NCH % NCW == 0, "chunks must divide over the copying waves");
    extern __shared__ u32x4 pfa_lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, li = lane & 15, lg = lane >> 4;
    // Heads along x: workgroup ids go round-robin to the XCDs, and all blocks of a head share an XCD's L2 when the head
    // count is a multiple of 8.
    const int nb = (M + 63) >> 6, h = blockIdx.x;
    const int qb_far = nb - 1 - (int)blockIdx.y, qb_near = (int)blockIdx.y;  // (the middle block of an odd count has no partner)
    const int qb = wave < 4 ? qb_far : qb_near;
    const int qt = qb * 4 + (wave & 3);
    const int r0 = qt * 16;
    const int nq = (wave >= 4 && qb_near >= qb_far) ? 0 : max(0, min(16, M - r0));
    const int pos0 = p0 + r0, ctx = pos0 + nq;
    const int my_tiles = nq > 0 ? (ctx + 31) >> 5 : 0;
    const int wg_last = min(M, qb_far * 64 + 64);             // rows of this workgroup end here
    const int wg_tiles = (p0 + wg_last + 31) >> 5;            // >= my_tiles of every wave
    const int KTd = d / 32;
    const bool qvalid = li < nq;
    const int krow0 = (li >> 2) * 8 + (li & 3);  // see attn_mfma_kernel: row permutation of the score tile
    bf16x8 qh[KK], ql[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const size_t qi = ((size_t)(nq > 0 ? qt : 0) * KTd + h * KK + kk) * 64 + lane;
        qh[kk] = __builtin_bit_cast(bf16x8, q_hi[qi]);
        ql[kk] = __builtin_bit_cast(bf16x8, q_lo[qi]);
    }
    // copy of tile t into stage st: chunk c = wave*FPW + i; this lane's 16 bytes of it
    auto issue = [&](int st, int t) {
        if (wave >= NCW) return;  // (head size 32: a tile is four chunks)
        const int tb = t << 5;
        const int blk = bt[tb / kv.BT];
        const int tin = tb % kv.BT;
        const __bf16* kbase = layer_base + (size_t)blk * kv.blk_stride + ((size_t)h * kv.BT + tin) * HD;
        const __bf16* vbase = layer_base + (size_t)blk * kv.blk_stride + (size_t)kv.H * kv.BT * HD + (size_t)h * HD * kv.BT +
                              (size_t)(tin >> 5) * (HD * 32);
#pragma unroll
        for (int i = 0; i < FPW; ++i) {
            const int c = wave * FPW + i;
            const __bf16* src;
            if (c < 2 * KK) {
                const int sub = c / KK, kk = c % KK;
                src = kbase + (size_t)(krow0 + sub * 4) * HD + kk * 32 + lg * 8;
            } else {
                src = vbase + ((c - 2 * KK) * 16 + li) * 32 + lg * 8;
            }
            __builtin_amdgcn_global_load_lds(EE_GLB_PTR(src), EE_LDS_PTR(pfa_lds + st * STAGE + c * 64), 16, 0, 0);
        }
    };
    const float scale = 1.0f / sqrtf((float)HD);
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[CG];
#pragma unroll
    for (int c = 0; c < CG; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < PFA_STAGES - 1; ++p) issue(p, p < wg_tiles ? p : wg_tiles - 1);
    const unsigned lds0 = (unsigned)(size_t)EE_LDS_PTR(pfa_lds) + lane * 16;
    int st_r = 0, st_w = PFA_STAGES - 1;
    for (int t = 0; t < wg_tiles; ++t) {
        pf_wait_vm<(PFA_STAGES - 2) * FPW>();
        __builtin_amdgcn_s_barrier();
        const unsigned sb = lds0 + st_r * (STAGE * 16);
        u32x4 kf[2 * KK], vf_[CG];
        PF_DSR(kf[0], sb, 0);
        PF_DSR(kf[1], sb, 1024);
        if constexpr (KK >= 2) {
            PF_DSR(kf[2], sb, 2048);
            PF_DSR(kf[3], sb, 3072);
        }
        if constexpr (KK == 4) {
            PF_DSR(kf[4], sb, 4096);
            PF_DSR(kf[5], sb, 5120);
            PF_DSR(kf[6], sb, 6144);
            PF_DSR(kf[7], sb, 7168);
        }
        PF_DSR(vf_[0], sb, 2 * KK * 1024);
        PF_DSR(vf_[1], sb, 2 * KK * 1024 + 1024);
        if constexpr (CG >= 4) {
            PF_DSR(vf_[2], sb, 2 * KK * 1024 + 2048);
            PF_DSR(vf_[3], sb, 2 * KK * 1024 + 3072);
        }
        if constexpr (CG == 8) {
            PF_DSR(vf_[4], sb, 2 * KK * 1024 + 4096);
            PF_DSR(vf_[5], sb, 2 * KK * 1024 + 5120);
            PF_DSR(vf_[6], sb, 2 * KK * 1024 + 6144);
            PF_DSR(vf_[7], sb, 2 * KK * 1024 + 7168);
        }
        issue(st_w, t + PFA_STAGES - 1 < wg_tiles ? t + PFA_STAGES - 1 : wg_tiles - 1);
        st_r = st_r + 1 == PFA_STAGES ? 0 : st_r + 1;
        st_w = st_w + 1 == PFA_STAGES ? 0 : st_w + 1;
        if constexpr (HD == 128)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]),
                         "+v"(kf[7]), "+v"(vf_[0]), "+v"(vf_[1]), "+v"(vf_[2]), "+v"(vf_[3]), "+v"(vf_[4]), "+v"(vf_[5]), "+v"(vf_[6]),
                         "+v"(vf_[7]));
        else if constexpr (HD == 64)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(vf_[0]), "+v"(vf_[1]), "+v"(vf_[2]),
                         "+v"(vf_[3]));
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(vf_[0]), "+v"(vf_[1]));
        if (t >= my_tiles) continue;  // (uniform over the wave) keys beyond this wave's rows
        const int tb = t << 5;
        // four independent accumulation chains (score half x term of q), so that no MFMA waits for the one before it
        f32x4 sacc[2], s_lo[2], s_hi[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) s_lo[sub] = s_hi[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const bf16x8 kfr = __builtin_bit_cast(bf16x8, kf[sub * KK + kk]);
                s_lo[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr, ql[kk], s_lo[sub], 0, 0, 0);
                s_hi[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr, qh[kk], s_hi[sub], 0, 0, 0);
            }
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) sacc[sub] = s_lo[sub] + s_hi[sub];
        float pv[8];
        float tmax = -INFINITY;
        if (tb + 31 <= pos0) {
            // every key of the tile lies at or before the first query of this wave: no causal mask (rows past the end of
            // the prompt then carry finite numbers that are never stored)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = sacc[e >> 2][e & 3] * scale;
                tmax = fmaxf(tmax, pv[e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int pa = tb + lg * 8 + e;
                const float val = (qvalid && pa <= pos0 + li) ? sacc[e >> 2][e & 3] * scale : -INFINITY;
                pv[e] = val;
                tmax = fmaxf(tmax, val);
            }
        }
        tmax = rows4_max(tmax);
        const float m_new = fmaxf(m_run, tmax);
        float corr = 1.f, psum = 0.f;
        if (m_new == -INFINITY) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[e] = 0.f;
        } else {
            // (hardware exponential: relative error about 1e-6 over the range that matters, far inside the bf16 contract)
            corr = __expf(m_run - m_new);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = __expf(pv[e] - m_new);
                psum += pv[e];
            }
        }
        psum = rows4_sum(psum);
        l_run = l_run * corr + psum;
        m_run = m_new;
        bf16x8 ph, pl;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const __bf16 hi = (__bf16)pv[e];
            ph[e] = hi;
            pl[e] = (__bf16)(pv[e] - (float)hi);
        }
        // the running maximum seldom moves once a few tiles have been seen: the accumulator is rescaled only when some
        // query of this wave needs it
        const bool rescale = __builtin_amdgcn_ballot_w64(corr != 1.f) != 0;
        const bool ragged = tb + 32 > ctx;  // positions beyond this wave's context may hold unknown bits: zero them
        if (ragged) {
#pragma unroll
            for (int c = 0; c < CG; ++c) {
                bf16x8 vf = __builtin_bit_cast(bf16x8, vf_[c]);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (tb + lg * 8 + e >= ctx) vf[e] = (__bf16)0.f;
                vf_[c] = __builtin_bit_cast(u32x4, vf);
            }
        }
        if (rescale) {
#pragma unroll
            for (int c = 0; c < CG; ++c) o[c] = o[c] * corr;
        }
        // (one pass per term of P over all feature groups: the two MFMAs on an accumulator are CG instructions apart)
#pragma unroll
        for (int c = 0; c < CG; ++c) o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf_[c]), pl, o[c], 0, 0, 0);
#pragma unroll
        for (int c = 0; c < CG; ++c) o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf_[c]), ph, o[c], 0, 0, 0);
    }
    pf_wait_vm<0>();  // surplus copies of the ring
    // O^T: lane (query li, group lg) holds features c*16 + lg*4 .. +3
    if (qvalid) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            float res[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) res[r] = o[c][r] * inv;
            pk_store4(out_hi, out_lo, r0 + li, h * HD + c * 16 + lg * 4, KTd, res);
        }
    }
}

template <int MTL>
int pf_grid(const PfArgs& a) {
    return ((a.n_wgN + 7) / 8) * 8 * a.n_wgM;
}

PfArgs pf_args(const PfGemm& g, int MTL) {
    PfArgs a;
    a.W = (const u32x4*)g.W;
    a.Xh = (const u32x4*)g.A_hi;
    a.Xl = (const u32x4*)g.A_lo;
    a.KT = g.K / 32;
    a.n_tiles = g.N / 16;
    a.m_tiles = (g.M + 15) / 16;
    a.n_wgN = (g.N + 255) / 256;
    a.n_wgM = (g.M + MTL * 16 - 1) / (MTL * 16);
    a.M = g.M;
    a.N = g.N;
    a.ssq = g.ssq;
    a.ssq_n = g.ssq_n;
    a.inv_d = g.inv_d;
    a.eps = g.eps;
    return a;
}

// Rows per workgroup tile, 128 or 64.  A CU works through about ceil(workgroups / 256) tiles (whether one after
// another or two side by side), each for a time proportional to its rows: take the cheaper, 128 on a tie
// (half the activation traffic from L2).
int pf_mtl(const PfGemm& g) {
    const long n_wgN = (g.N + 255) / 256;
    const long r8 = (n_wgN * ((g.M + 127) / 128) + 255) / 256 * 8;
    const long r4 = (n_wgN * ((g.M + 63) / 64) + 255) / 256 * 4;
    return r4 < r8 ? 4 : 8;
}

template <typename K>
hipError_t pf_set_lds(K kernel, size_t bytes) {
    return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

#define PF_DISPATCH(KERNEL, WIDE, ...)                                                                        \
    do {                                                                                                  \
        if (pf_mtl(g) == 8) {                                                                             \
            PfArgs a = pf_args(g, 8);                                                                     \
            constexpr size_t lds_b = pf_lds_bytes<8, 8, WIDE>();                                              \
            static hipError_t once = pf_set_lds(KERNEL<8, 8>, lds_b);                                     \
            if (once != hipSuccess) return once;                                                          \
            EE_LAUNCH_SM((KERNEL<8, 8>), dim3(pf_grid<8>(a)), dim3(512), lds_b, s, a, __VA_ARGS__);       \
        } else {                                                                                          \
            PfArgs a = pf_args(g, 4);                                                                     \
            constexpr size_t lds_b = pf_lds_bytes<4, 8, WIDE>();                                              \
            static hipError_t once = pf_set_lds(KERNEL<4, 8>, lds_b);                                     \
            if (once != hipSuccess) return once;                                                          \
            EE_LAUNCH_SM((KERNEL<4, 8>), dim3(pf_grid<4>(a)), dim3(512), lds_b, s, a, __VA_ARGS__);       \
        }                                                                                                 \
        return hipGetLastError();                                                                         \
    } while (0)

hipError_t launch_pf_qkv(const PfGemm& g, void* q_hi, void* q_lo, const float* rope_cs, const KvGeom& kv, int layer, const int32_t* bt,
                         int p0, hipStream_t s) {
    const int d = g.N / 3;
    PfQkv e{(__bf16*)q_hi, (__bf16*)q_lo, d, kv.H, kv.hd, (const float2*)rope_cs, (__bf16*)kv.pool + (size_t)layer * kv.layer_stride,
            kv.blk_stride, kv.BT, bt, p0};
    PF_DISPATCH(pf_qkv_kernel, true, e);
}

hipError_t launch_pf_resid(const PfGemm& g, float* x, void* xg_hi, void* xg_lo, void* xgh_hi, void* xgh_lo, const float* g_next,
                           const float* g_head, float* ssq_out, int ssq_n_out, hipStream_t s) {
    PfResid e{x, (__bf16*)xg_hi, (__bf16*)xg_lo, (__bf16*)xgh_hi, (__bf16*)xgh_lo, g_next, g_head, ssq_out, ssq_n_out, g.N};
    // Two workgroups per CU (four waves per SIMD) once the grid has more workgroups than CUs (30B widths at 2048
    // rows: O 359 -> 332 us, down 922 -> 840 us); a grid of one workgroup per CU keeps the deeper ring and the
    // second operand set.
    const int mtl = pf_mtl(g);
    const long n_wgs = (long)((g.N + 255) / 256) * ((g.M + mtl * 16 - 1) / (mtl * 16));
    const bool wide = n_wgs > 256;
    if (wide) {
        if (mtl == 8) {
            PfArgs a = pf_args(g, 8);
            constexpr size_t lds_b = pf_lds_bytes<8, 8, true>();
            static hipError_t once = pf_set_lds(pf_resid_kernel<8, 8, true>, lds_b);
            if (once != hipSuccess) return once;
            EE_LAUNCH_SM((pf_resid_kernel<8, 8, true>), dim3(pf_grid<8>(a)), dim3(512), lds_b, s, a, e);
        } else {
            PfArgs a = pf_args(g, 4);
            constexpr size_t lds_b = pf_lds_bytes<4, 8, true>();
            static hipError_t once = pf_set_lds(pf_resid_kernel<4, 8, true>, lds_b);
            if (once != hipSuccess) return once;
            EE_LAUNCH_SM((pf_resid_kernel<4, 8, true>), dim3(pf_grid<4>(a)), dim3(512), lds_b, s, a, e);
        }
        return hipGetLastError();
    }
    // ... and, when the contraction has an even number of k-tiles, 16 waves with K split over two wave groups
    // (O 68 -> 64 us, down 159 -> 152 us at the 7B width and 1024 rows)
    if (mtl == 4 && (g.K / 32) % 2 == 0 && g.K / 32 >= 2 * PFK_NST) {
        PfArgs a = pf_args(g, 4);
        constexpr size_t lds_b = pfk_lds_bytes();
        static hipError_t once = pf_set_lds(pf_resid_k16_kernel, lds_b);
        if (once != hipSuccess) return once;
        EE_LAUNCH_SM(pf_resid_k16_kernel, dim3(pf_grid<4>(a)), dim3(1024), lds_b, s, a, e);
        return hipGetLastError();
    }
    PF_DISPATCH(pf_resid_kernel, false, e);
}

hipError_t launch_pf_swiglu(const PfGemm& g, void* act_hi, void* act_lo, int F, hipStream_t s) {
    PF_DISPATCH(pf_swiglu_kernel, true, (__bf16*)act_hi, (__bf16*)act_lo, F);
}

hipError_t launch_pf_head(const PfGemm& g, HeadPartial* partials, int32_t* tok, float* conf, const int32_t* target,
                          float* target_logit, float* nll, bool two_terms, hipStream_t s) {
    const int n_wg = (g.N + 255) / 256;
    PfHead e{partials, g.N, nll ? target : nullptr, target_logit};
    PfArgs a = pf_args(g, 8);
    if (two_terms) {
        // (8 waves, two workgroups per CU, two stages: 633 us at 1024 rows; 4 waves with two workgroups per CU measured
        // 672 us, 8 waves with one workgroup per CU and four stages 750 us)
        constexpr size_t lds_b = pf_lds_bytes<8, 8, true>();
        static hipError_t once = pf_set_lds(pf_head_kernel<8, 8, true>, lds_b);
        if (once != hipSuccess) return once;
        EE_LAUNCH_SM((pf_head_kernel<8, 8, true>), dim3(pf_grid<8>(a)), dim3(512), lds_b, s, a, e);
    } else {
        // the leading term of the activations only: half the MFMAs, 24 KB per stage, three stages
        constexpr size_t lds_b = pf_lds_bytes<8, 8, true, false>();
        static hipError_t once = pf_set_lds(pf_head_kernel<8, 8, false>, lds_b);
        if (once != hipSuccess) return once;
        EE_LAUNCH_SM((pf_head_kernel<8, 8, false>), dim3(pf_grid<8>(a)), dim3(512), lds_b, s, a, e);
    }
    {
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    EE_LAUNCH(pf_head_merge_kernel, dim3(g.M), dim3(64), s, (const HeadPartial*)partials, n_wg, g.M, tok, conf,
              nll ? target : (const int32_t*)nullptr, (const float*)target_logit, nll);
    return hipGetLastError();
}

hipError_t launch_pf_embed(const void* embed, const int32_t* dev_tokens, int M, int d, const float* g_next, float* x, void* xg_hi,
                           void* xg_lo, float* ssq, int ssq_n, hipStream_t s) {
    EE_LAUNCH(pf_embed_kernel, dim3(M), dim3(256), s, (const __bf16*)embed, dev_tokens, d, g_next, x, (__bf16*)xg_hi, (__bf16*)xg_lo, ssq,
              ssq_n);
    return hipGetLastError();
}

hipError_t launch_pf_export_row(const float* x_row, int d, const float* g_a, const float* g_b, float* dx, void* dxg, void* dxgh,
                                size_t lo_off, float* dssq, int ssq_stride, hipStream_t s) {
    EE_LAUNCH(pf_export_row_kernel, dim3(1), dim3(256), s, x_row, d, g_a, g_b, dx, (__bf16*)dxg, (__bf16*)dxgh, lo_off, dssq, ssq_stride);
    return hipGetLastError();
}

hipError_t launch_pf_attention(const void* q_hi, const void* q_lo, void* out_hi, void* out_lo, const KvGeom& kv, int layer,
                               const int32_t* bt, int p0, int M, int d, hipStream_t s) {
    const __bf16* lb = (const __bf16*)kv.pool + (size_t)layer * kv.layer_stride;
    dim3 grid(kv.H, ((M + 63) / 64 + 1) / 2), block(512);
    const size_t lds = (size_t)PFA_STAGES * (2 * (kv.hd / 32) + kv.hd / 16) * 1024;  // at most 64 KB
    switch (kv.hd) {
        case 32:
            EE_LAUNCH_SM(pf_attn_kernel<32>, grid, block, lds, s, (const u32x4*)q_hi, (const u32x4*)q_lo, (__bf16*)out_hi, (__bf16*)out_lo,
                         lb, kv, bt, p0, M, d);
            break;
        case 64:
            EE_LAUNCH_SM(pf_attn_kernel<64>, grid, block, lds, s, (const u32x4*)q_hi, (const u32x4*)q_lo, (__bf16*)out_hi, (__bf16*)out_lo,
                         lb, kv, bt, p0, M, d);
            break;
        case 128:
            EE_LAUNCH_SM(pf_attn_kernel<128>, grid, block, lds, s, (const u32x4*)q_hi, (const u32x4*)q_lo, (__bf16*)out_hi, (__bf16*)out_lo,
                         lb, kv, bt, p0, M, d);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace ee
