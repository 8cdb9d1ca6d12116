// HIP kernels (gfx950) for one early-exit decode step with KV recomputation.
//
// Every decode GEMM has at most a few dozen rows (the current token plus the deferred tokens that are
// carried along, Section 4 "KV recomputation"), so it is a weight-streaming problem bound by HBM
// bandwidth: weights are stored pre-shuffled so that one wave load instruction fetches 1 KB of
// contiguous memory that is already a 16x32 bf16 MFMA operand, a workgroup owns a few 16-column
// tiles and splits the reduction dimension over its waves, and everything that follows the product
// (rotary embedding and the KV-cache write, residual add, the next layer's normalised input,
// SwiGLU, the soft-max max/arg-max over the vocabulary and the exit decision) runs in the epilogue
// of the kernel that produced it.  No float atomics: every reduction has a fixed order.
#include "ee_internal.h"

#include "ee_lanes.h"
#include "ee_launch.h"

#include <cstdlib>
#include <type_traits>

namespace ee {

static thread_local hipEvent_t t_ev0 = nullptr, t_ev1 = nullptr;
void set_launch_events(hipEvent_t start, hipEvent_t stop) {
    t_ev0 = start;
    t_ev1 = stop;
}
bool take_launch_events(hipEvent_t* start, hipEvent_t* stop) {
    if (!t_ev0) return false;
    *start = t_ev0;
    *stop = t_ev1;
    t_ev0 = t_ev1 = nullptr;
    return true;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename ST> __device__ __forceinline__ ST cvt_st(float v);
template <> __device__ __forceinline__ float cvt_st<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 cvt_st<__bf16>(float v) { return (__bf16)v; }  // round to nearest even

// Activations of the bf16 model are carried as two bf16 terms, hi = bf16(v) and lo = bf16(v - hi), so
// that a matrix input keeps about 16 mantissa bits while still being an MFMA bf16 operand (two MFMAs
// per tile; the matrix cores idle anyway in this bandwidth-bound regime).  `lo_off` is the element
// distance from the hi array to the lo array.  The fp32 model has a single term.
template <typename ST> __device__ __forceinline__ void store_split(ST* p, size_t lo_off, float v);
template <> __device__ __forceinline__ void store_split<float>(float* p, size_t, float v) { *p = v; }
template <> __device__ __forceinline__ void store_split<__bf16>(__bf16* p, size_t lo_off, float v) {
    __bf16 hi = (__bf16)v;
    p[0] = hi;
    p[lo_off] = (__bf16)(v - (float)hi);
}
template <typename ST> __device__ __forceinline__ float load_split(const ST* p, size_t lo_off);
template <> __device__ __forceinline__ float load_split<float>(const float* p, size_t) { return *p; }
template <> __device__ __forceinline__ float load_split<__bf16>(const __bf16* p, size_t lo_off) {
    return (float)p[0] + (float)p[lo_off];
}

// Element index of (row m, feature k) in an operand-order ("packed") activation array: 16-row groups,
// [m/16][K/32][64 lanes][8], lane = ((k%32)/8)*16 + m%16: one k-step of one row group is 1 KB that a wave
// loads as a ready MFMA operand.  Used for the rows of a launch when there are too many for LDS.
__device__ __forceinline__ size_t pk_index(int m, int k, int KT) {
    return (((size_t)(m >> 4) * KT + (k >> 5)) * 64 + (((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7);
}

// one value as two bf16 terms into a row-major (pk_kt == 0) or a packed array
template <typename ST>
__device__ __forceinline__ void store_split_at(ST* base, size_t lo_off, int m, int k, int ld, int pk_kt, float v) {
    store_split<ST>(base + (pk_kt ? pk_index(m, k, pk_kt) : (size_t)m * ld + k), lo_off, v);
}

// rows (row-major, two terms, through an index list) -> packed array
__global__ __launch_bounds__(256) void pack_rows_kernel(const __bf16* __restrict__ src, size_t src_lo, int ld, const int32_t* __restrict__ rows,
                                                        int T, int K, __bf16* __restrict__ dst, size_t dst_lo) {
    const int cpr = K / 8;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)T * cpr) return;
    const int m = (int)(idx / cpr), k = (int)(idx % cpr) * 8;
    const __bf16* sp = src + (size_t)(rows ? rows[m] : m) * ld + k;
    const size_t o = pk_index(m, k, K / 32);
    *(u32x4*)(dst + o) = *(const u32x4*)sp;
    *(u32x4*)(dst + dst_lo + o) = *(const u32x4*)(sp + src_lo);
}

hipError_t launch_pack_rows(const void* src, size_t src_lo, int ld, const int32_t* rows, int T, int K, void* dst, size_t dst_lo,
                            hipStream_t s) {
    if (T <= 0) return hipSuccess;
    const long n = (long)T * (K / 8);
    EE_LAUNCH(pack_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), s, (const __bf16*)src, src_lo, ld, rows, T, K, (__bf16*)dst,
              dst_lo);
    return hipGetLastError();
}

// Plain read of a buffer, one KB per wave and load, eight loads in flight per wave: what this GPU's memory delivers
// to a kernel that only reads.  The benchmark quotes the decode step against it next to the nominal peak.
__global__ __launch_bounds__(512) void stream_read_kernel(const u32x4* __restrict__ p, size_t n_kb, int kb_per_wave, uint32_t* sink) {
    const int lane = threadIdx.x & 63;
    const size_t w = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6);
    const size_t c0 = w * (size_t)kb_per_wave;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int c = 0; c < kb_per_wave; c += 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t ci = c0 + c + u;
            v[u] = (c + u < kb_per_wave && ci < n_kb) ? __builtin_nontemporal_load(p + ci * 64 + lane) : acc;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && sink) sink[0] = acc.x;  // keeps the loads alive
}

// Test hook: the lane reductions of ee_lanes.h against the xor butterflies over __shfl_xor that they replace, on
// pseudo-random values of mixed sign and magnitude; counts the lanes whose results differ in any bit.
__global__ __launch_bounds__(256) void lane_reduction_check_kernel(int32_t* __restrict__ mismatches, int rounds) {
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    int bad = 0;
    for (int r = 0; r < rounds; ++r) {
        h ^= h >> 15;
        h *= 2246822519u;
        h ^= h >> 13;
        h *= 3266489917u;
        h ^= h >> 16;
        // sign, a small exponent range and 23 mantissa bits: sums that round at every step
        const float v = __uint_as_float((h & 0x807fffffu) | ((118u + ((h >> 23) & 15u)) << 23));
        float a = v, b = v, c = v;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
        b += __shfl_xor(b, 16);
        b += __shfl_xor(b, 32);
        c = fmaxf(c, __shfl_xor(c, 16));
        c = fmaxf(c, __shfl_xor(c, 32));
        bad += __float_as_uint(a) != __float_as_uint(wave_sum(v));
        bad += __float_as_uint(b) != __float_as_uint(rows4_sum(v));
        bad += __float_as_uint(c) != __float_as_uint(rows4_max(v));
    }
    if (bad) atomicAdd(mismatches, bad);
}

hipError_t launch_lane_reduction_check(int32_t* dev_mismatches, hipStream_t s) {
    EE_LAUNCH(lane_reduction_check_kernel, dim3(64), dim3(256), s, dev_mismatches, 64);
    return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t s) {
    const size_t n_kb = bytes / 1024;
    if (n_kb == 0) return hipSuccess;
    const int kb_per_wave = 32;
    const size_t waves = (n_kb + kb_per_wave - 1) / kb_per_wave;
    EE_LAUNCH(stream_read_kernel, dim3((unsigned)((waves + 7) / 8)), dim3(512), s, (const u32x4*)src, n_kb, kb_per_wave, (uint32_t*)sink);
    return hipGetLastError();
}

__global__ void fill_f32_kernel(float* p, float v, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

hipError_t launch_fill_f32(float* p, float v, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    EE_LAUNCH(fill_f32_kernel, dim3((unsigned)((n + 255) / 256 < 256 ? (n + 255) / 256 : 256)), dim3(256), s, p, v, n);
    return hipGetLastError();
}

// Rows of the residual store copied to other slots of the same store: the residual row, the operand row x.g that
// an exit reads (both terms for bf16) and the row's sum-of-squares partials.  An exit that starts with an MLP
// works on such a copy, so that the backbone's row stays as it is.
template <typename ST>
__global__ __launch_bounds__(256) void copy_slots_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int d,
                                                         float* __restrict__ x, ST* __restrict__ xgh, size_t lo,
                                                         float* __restrict__ ssq, int ssq_stride) {
    const int a = src[blockIdx.x], b = dst[blockIdx.x];
    for (int i = threadIdx.x; i < d; i += 256) {
        x[(size_t)b * d + i] = x[(size_t)a * d + i];
        xgh[(size_t)b * d + i] = xgh[(size_t)a * d + i];
        if (lo) xgh[lo + (size_t)b * d + i] = xgh[lo + (size_t)a * d + i];
    }
    for (int i = threadIdx.x; i < ssq_stride; i += 256) ssq[(size_t)b * ssq_stride + i] = ssq[(size_t)a * ssq_stride + i];
}

hipError_t launch_copy_slots(int dtype, const int32_t* dev_src, const int32_t* dev_dst, int n, int d, float* x, void* xgh, size_t lo,
                             float* ssq, int ssq_stride, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (dtype == EE_BF16)
        EE_LAUNCH(copy_slots_kernel<__bf16>, dim3(n), dim3(256), s, dev_src, dev_dst, d, x, (__bf16*)xgh, lo, ssq, ssq_stride);
    else
        EE_LAUNCH(copy_slots_kernel<float>, dim3(n), dim3(256), s, dev_src, dev_dst, d, x, (float*)xgh, (size_t)0, ssq, ssq_stride);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// rotary table: cs[pos][i] = (cos, sin)(pos * base^(-2i/hd)), evaluated in fp64
// ------------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* cs, int max_pos, int half, int hd, float base) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= max_pos * half) return;
    int pos = idx / half, i = idx % half;
    double ang = (double)pos * pow((double)base, -2.0 * (double)i / (double)hd);
    cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

hipError_t launch_rope_table(float* cs, int max_pos, int hd, float base, hipStream_t s) {
    int n = max_pos * (hd / 2);
    EE_LAUNCH(rope_table_kernel, dim3((n + 255) / 256), dim3(256), s, (float2*)cs, max_pos, hd / 2, hd, base);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// weight packing.  Source: row-major [n_rows][K].  Destination rows are grouped in tiles of 16, one
// tile per workgroup of the GEMM kernels.
//   bf16: [tile][K/32][lane 0..63][8]  with lane = (k_group << 4) | row_in_tile, k = kt*32 + k_group*8 + j
//         (one wave load instruction = 1 KB of contiguous memory = one 16x32 MFMA operand)
//   fp32: [tile][16][K] (row permutation only)
// Row placement (feature f -> tile, row in tile):
//   PACK_PLAIN   tile f/16, row f%16
//   PACK_ROTARY  both halves of a rotary pair in one tile: inside head h, feature o < hd/2 goes to
//                tile h*hd/16 + o/8, row o%8; its partner o + hd/2 to the same tile, row 8 + o%8
//   PACK_GATE / PACK_UP  gate feature f -> tile f/8, row f%8; up feature f -> tile f/8, row 8 + f%8
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void pack_place(int row, int mode, int hd, int& dt, int& dr) {
    if (mode == PACK_PLAIN) {
        dt = row >> 4;
        dr = row & 15;
    } else if (mode == PACK_ROTARY) {
        int h = row / hd, o = row % hd, half = hd / 2;
        int s = o >= half, oo = o % half;
        dt = h * (hd / 16) + oo / 8;
        dr = (oo & 7) + 8 * s;
    } else {
        dt = row >> 3;
        dr = (row & 7) + (mode == PACK_UP ? 8 : 0);
    }
}

__global__ void pack_bf16_kernel(const __bf16* __restrict__ src, uint4* __restrict__ dst, int n_rows, int K, int mode, int hd) {
    int KT = K / 32;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;  // (row, kt, k_group)
    if (idx >= (long)n_rows * KT * 4) return;
    int lg = idx & 3;
    long r = idx >> 2;
    int kt = r % KT;
    int row = r / KT;
    int dt, dr;
    pack_place(row, mode, hd, dt, dr);
    const uint4* sp = (const uint4*)(src + ((size_t)row * K + kt * 32 + lg * 8));
    dst[((size_t)dt * KT + kt) * 64 + lg * 16 + dr] = *sp;
}

__global__ void pack_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int n_rows, int K, int mode, int hd) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n_rows * K) return;
    int row = idx / K, k = idx % K;
    int dt, dr;
    pack_place(row, mode, hd, dt, dr);
    dst[((size_t)dt * 16 + dr) * K + k] = src[idx];
}

hipError_t launch_pack(int dtype, const void* src, void* dst, int n_rows, int K, int mode, int hd, hipStream_t s) {
    if (dtype == EE_BF16) {
        long total = (long)n_rows * (K / 32) * 4;
        EE_LAUNCH(pack_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, (const __bf16*)src, (uint4*)dst, n_rows, K,
                  mode, hd);
    } else {
        long total = (long)n_rows * K;
        EE_LAUNCH(pack_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), s, (const float*)src, (float*)dst, n_rows, K,
                  mode, hd);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// embedding gather: x = E[token]; xg = st(x * g_next); ssq[slot][0] = sum x^2, ssq[slot][1..] = 0
// one workgroup per row
// ------------------------------------------------------------------------------------------------
template <typename ST>
__global__ void embed_kernel(const ST* __restrict__ embed, const int32_t* __restrict__ tokens, const SegDesc* __restrict__ desc,
                             int d, const float* __restrict__ g_next, float* __restrict__ x, ST* __restrict__ xg,
                             size_t xg_lo, float* __restrict__ ssq, int ssq_stride) {
    __shared__ float red[256];
    int r = blockIdx.x;
    int slot = desc->xrow[r];
    int tok = tokens[r];
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = (float)embed[(size_t)tok * d + i];
        x[(size_t)slot * d + i] = v;
        store_split<ST>(xg + (size_t)slot * d + i, xg_lo, v * g_next[i]);
        s += v * v;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    for (int i = threadIdx.x; i < ssq_stride; i += blockDim.x) ssq[(size_t)slot * ssq_stride + i] = (i == 0) ? red[0] : 0.f;
}

hipError_t launch_embed(int dtype, const void* embed, const int32_t* dev_tokens, const SegDesc* desc, int T, int d,
                        const float* g_next, float* x, void* xg, size_t xg_lo, float* ssq, int ssq_stride, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (dtype == EE_BF16)
        EE_LAUNCH(embed_kernel<__bf16>, dim3(T), dim3(256), s, (const __bf16*)embed, dev_tokens, desc, d, g_next, x,
                           (__bf16*)xg, xg_lo, ssq, ssq_stride);
    else
        EE_LAUNCH(embed_kernel<float>, dim3(T), dim3(256), s, (const float*)embed, dev_tokens, desc, d, g_next, x,
                           (float*)xg, xg_lo, ssq, ssq_stride);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// start of a decode step in one launch: the step's descriptors, block tables and token ids go from the host-mapped
// staging area to the workspace (up to three ranges of it: the descriptors in use, those of the exits' own rows, the
// tables), and the rows that start at the embedding are looked up.  The embedding workgroups take their token ids and
// residual-store slots by value (up to 16 rows) or straight from the staging area, so they do not wait for the copy.
// ------------------------------------------------------------------------------------------------
struct StepBegin {
    const u32x4* src;  // staging area (host memory, mapped)
    u32x4* dst;        // the same region in the workspace
    uint32_t off16[3], n16[3];  // ranges to copy, in 16-byte units from the start of the region
    int n_copy_wgs;
    int T;  // rows to embed
    int has_v;
    int32_t tok_v[16], slot_v[16];
    const int32_t* tok_h;   // host-mapped token ids and slots of the rows (more than 16 rows)
    const int32_t* slot_h;
};

template <typename ST>
__global__ __launch_bounds__(256) void step_begin_kernel(StepBegin b, const ST* __restrict__ embed, int d, const float* __restrict__ g_next,
                                                         float* __restrict__ x, ST* __restrict__ xg, size_t xg_lo, float* __restrict__ ssq,
                                                         int ssq_stride) {
    if ((int)blockIdx.x < b.n_copy_wgs) {
#pragma unroll
        for (int r = 0; r < 3; ++r)
            for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < b.n16[r]; i += (uint32_t)b.n_copy_wgs * 256)
                b.dst[b.off16[r] + i] = b.src[b.off16[r] + i];
        return;
    }
    __shared__ float red[4];
    const int r = (int)blockIdx.x - b.n_copy_wgs;
    const int slot = b.has_v ? b.slot_v[r] : b.slot_h[r];
    const int tok = b.has_v ? b.tok_v[r] : b.tok_h[r];
    float s = 0.f;
    for (int i = threadIdx.x * 8; i < d; i += 256 * 8) {  // d is a multiple of 32
        float v[8];
        if constexpr (sizeof(ST) == 2) {
            const bf16x8 e = *(const bf16x8*)(embed + (size_t)tok * d + i);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (float)e[j];
        } else {
            const f32x4 e0 = *(const f32x4*)(embed + (size_t)tok * d + i), e1 = *(const f32x4*)(embed + (size_t)tok * d + i + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[j] = e0[j];
                v[4 + j] = e1[j];
            }
        }
        const f32x4 g0 = *(const f32x4*)(g_next + i), g1 = *(const f32x4*)(g_next + i + 4);
        *(f32x4*)(x + (size_t)slot * d + i) = f32x4{v[0], v[1], v[2], v[3]};
        *(f32x4*)(x + (size_t)slot * d + i + 4) = f32x4{v[4], v[5], v[6], v[7]};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            store_split<ST>(xg + (size_t)slot * d + i + j, xg_lo, v[j] * (j < 4 ? g0[j] : g1[j - 4]));
            s += v[j] * v[j];
        }
    }
    // sum of squares: lanes of a wave through a fixed butterfly, then the four waves in order
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    const float tot = ((red[0] + red[1]) + red[2]) + red[3];
    for (int i = threadIdx.x; i < ssq_stride; i += 256) ssq[(size_t)slot * ssq_stride + i] = (i == 0) ? tot : 0.f;
}

hipError_t launch_step_begin(int dtype, const void* staging_mapped, void* ws_region, const uint32_t off16[3], const uint32_t n16[3],
                             int T, const int32_t* tok_host, const int32_t* slot_host, const int32_t* tok_mapped,
                             const int32_t* slot_mapped, const void* embed, int d, const float* g_next, float* x, void* xg, size_t xg_lo,
                             float* ssq, int ssq_stride, hipStream_t s) {
    StepBegin b{};
    b.src = (const u32x4*)staging_mapped;
    b.dst = (u32x4*)ws_region;
    uint32_t total = 0;
    for (int r = 0; r < 3; ++r) {
        b.off16[r] = off16[r];
        b.n16[r] = n16[r];
        total += n16[r];
    }
    b.n_copy_wgs = (int)((total + 255) / 256 < 32 ? (total + 255) / 256 : 32);
    if (b.n_copy_wgs < 1) b.n_copy_wgs = 1;
    b.T = T;
    b.has_v = T <= 16;
    for (int r = 0; r < T && r < 16; ++r) {
        b.tok_v[r] = tok_host[r];
        b.slot_v[r] = slot_host[r];
    }
    b.tok_h = tok_mapped;
    b.slot_h = slot_mapped;
    if (dtype == EE_BF16)
        EE_LAUNCH(step_begin_kernel<__bf16>, dim3(b.n_copy_wgs + T), dim3(256), s, b, (const __bf16*)embed, d, g_next, x, (__bf16*)xg, xg_lo, ssq,
                  ssq_stride);
    else
        EE_LAUNCH(step_begin_kernel<float>, dim3(b.n_copy_wgs + T), dim3(256), s, b, (const float*)embed, d, g_next, x, (float*)xg, (size_t)0, ssq,
                  ssq_stride);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// skinny GEMM: out[m][n] = r[m] * sum_k A[m][k] * W[n][k],  m < T <= MT*16
// A workgroup owns ONE 16-column tile (128 KB of weights at K = 4096: small units keep the 256 CUs evenly
// loaded) and its KS waves split K, so that each wave streams about 16 KB.  The result lands in LDS as
// out[MT*16][16] fp32 and is handed to the epilogue.
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const void* W;
    int KT;  // K / 32
    int K;
    const void* A;
    size_t a_lo;  // element offset of the lo term of A (bf16 only)
    int lda;
    const int32_t* arow;
    const float* ssq;
    int ssq_stride, ssq_n;
    float inv_d, eps;
    int T;
    int n_tiles;  // N / 16
    // Up to 16 rows: the row indirection (and, for the attention merge, row -> query tile) by value, so that the
    // first loads of a workgroup do not hang off a load of the descriptor.
    int has_row_v;
    int32_t arow_v[16];
    int32_t rq_v[16];
    int a_packed; // A is stored in MFMA operand order [row/16][K/32][64 lanes][8] (dense rows, no indirection)
    // A given as split-KV attention partials instead of rows (few-rows variant of the O projection only)
    const float* att_part;
    const SegDesc* att_desc;
    int att_ns, att_H, att_hd;
};

// G = 16-column tiles a workgroup owns (1 for few rows; more when there are many rows, so that the
// activation operands a wave has loaded serve several weight tiles and the L2 traffic of the rows,
// which every workgroup re-reads in full, shrinks accordingly)
template <int KS, int MT, int G = 1>
struct GemmSmem {
    float red[KS][MT][256];
    float out[G][MT * 16][16];
    float rs[MT * 16];
};

__device__ __forceinline__ int gemm_slot(const GemmArgs& a, int m) {
    return a.has_row_v ? a.arow_v[m] : (a.arow ? a.arow[m] : m);
}

template <int MT>
__device__ __forceinline__ void rms_scales(const GemmArgs& a, float* rs) {
    // r[m] = 1/sqrt(mean(x^2)+eps).  The sum of squares arrives as ssq_n partial sums (one per producing
    // workgroup); one wave per row adds them: lane-strided in order, then a fixed butterfly.
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    for (int m = wave; m < MT * 16; m += nw) {
        float r = 1.f;
        if (a.ssq != nullptr && m < a.T) {
            int slot = gemm_slot(a, m);
            const float* p = a.ssq + (size_t)slot * a.ssq_stride;
            float s = 0.f;
            for (int i = lane; i < a.ssq_n; i += 64) s += p[i];
            s = wave_sum(s);
            r = 1.0f / sqrtf(s * a.inv_d + a.eps);
        }
        if (lane == 0) rs[m] = r;
    }
}

template <int KS, int MT, typename Pre>
__device__ __forceinline__ void gemm_mainloop_bf16(const GemmArgs& a, int tile, GemmSmem<KS, MT>& sm, Pre pre) {
    const int ks = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int KT = a.KT;
    const int kt0 = (int)(((long)ks * KT) / KS), kt1 = (int)(((long)(ks + 1) * KT) / KS);
    const u32x4* wp = (const u32x4*)a.W + ((size_t)tile * KT + kt0) * 64 + lane;
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Ring of D tiles (1 KB of weights each) per wave: a slot is refilled with the tile D ahead as soon
    // as its MFMAs are issued.  The first D weight loads go out before anything that depends on another
    // load (row indirection, RMS partial sums, epilogue operands), so the stream starts at once.
    constexpr int D = MT == 1 ? 7 : 4;
    u32x4 w[D], ah[MT][D], al[MT][D];
    const int n = kt1 - kt0;
    auto fill_w = [&](int u, int t) { w[u] = __builtin_nontemporal_load(wp + (size_t)t * 64); };
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n) fill_w(u, u);
    // Rows beyond T read row 0 again (always a valid address): their products are never looked at,
    // and an unpredicated load keeps the loop free of branches.
    // A operands: row-major rows (a load gathers 16 rows x 64 bytes), or already in operand order
    // (packed: one contiguous KB per load)
    const __bf16* ap[MT];
    const int astep = a.a_packed ? 512 : 32;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (a.a_packed) {
            ap[mt] = (const __bf16*)a.A + ((size_t)mt * KT + kt0) * 512 + lane * 8;
        } else {
            int row = mt * 16 + li;
            if (row >= a.T) row = 0;
            int idx = a.arow ? a.arow[row] : row;
            ap[mt] = (const __bf16*)a.A + (size_t)idx * a.lda + (size_t)kt0 * 32 + lg * 8;
        }
    }
    auto fill_a = [&](int u, int t) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            ah[mt][u] = *(const u32x4*)(ap[mt] + (size_t)t * astep);
            al[mt][u] = *(const u32x4*)(ap[mt] + a.a_lo + (size_t)t * astep);
        }
    };
    auto fill = [&](int u, int t) {  // slot u <- tile t (relative to kt0)
        fill_w(u, t);
        fill_a(u, t);
    };
    auto use = [&](int u) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, al[mt][u]),
                                                              __builtin_bit_cast(bf16x8, w[u]), acc[mt], 0, 0, 0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ah[mt][u]),
                                                              __builtin_bit_cast(bf16x8, w[u]), acc[mt], 0, 0, 0);
        }
    };
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n) fill_a(u, u);
    rms_scales<MT>(a, sm.rs);
    pre(std::false_type{});
    const int full = n / D, rem = n - full * D;
    for (int gI = 0; gI + 1 < full; ++gI) {  // steady state: every refill is in range
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            fill(u, (gI + 1) * D + u);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (full > 0) {  // last full group: refill only the slots the remainder needs
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            if (u < rem) fill(u, full * D + u);
        }
    }
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < rem) use(u);
    // accumulator layout: lane (lg, li) holds D[row = lg*4 + r][col = li]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) sm.red[ks][mt][(lg * 4 + r) * 16 + li] = acc[mt][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
        int e = idx & 255, mt = idx >> 8;
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < KS; ++k) s += sm.red[k][mt][e];
        int m = mt * 16 + (e >> 4);
        sm.out[0][m][e & 15] = s * sm.rs[m];
    }
    __syncthreads();
}

// Register path with G tiles per workgroup: every ring slot holds one k-step of G weight tiles and of the
// MT row tiles (both terms); the G*MT products of a slot share its activation registers.
template <int KS, int MT, int G, typename Pre>
__device__ __forceinline__ void gemm_mainloop_bf16_multi(const GemmArgs& a, int tile0, GemmSmem<KS, MT, G>& sm, Pre pre) {
    const int ks = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int KT = a.KT;
    const int kt0 = (int)(((long)ks * KT) / KS), kt1 = (int)(((long)(ks + 1) * KT) / KS);
    const u32x4* wp[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        int t = tile0 + g;
        if (t >= a.n_tiles) t = a.n_tiles - 1;  // (a surplus tile repeats the last one; its result is dropped)
        wp[g] = (const u32x4*)a.W + ((size_t)t * KT + kt0) * 64 + lane;
    }
    f32x4 acc[G][MT];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[g][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int D = (MT == 4 || MT * G >= 12) ? 2 : 4;  // ring slots: fewer where a slot already holds many KB
    u32x4 w[G][D], ah[MT][D], al[MT][D];
    const int n = kt1 - kt0;
    auto fill_w = [&](int u, int t) {
#pragma unroll
        for (int g = 0; g < G; ++g) w[g][u] = __builtin_nontemporal_load(wp[g] + (size_t)t * 64);
    };
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n) fill_w(u, u);
    // A operands: row-major rows (a load gathers 16 rows x 64 bytes), or already in operand order
    // (packed: one contiguous KB per load)
    const __bf16* ap[MT];
    const int astep = a.a_packed ? 512 : 32;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (a.a_packed) {
            ap[mt] = (const __bf16*)a.A + ((size_t)mt * KT + kt0) * 512 + lane * 8;
        } else {
            int row = mt * 16 + li;
            if (row >= a.T) row = 0;
            int idx = a.arow ? a.arow[row] : row;
            ap[mt] = (const __bf16*)a.A + (size_t)idx * a.lda + (size_t)kt0 * 32 + lg * 8;
        }
    }
    auto fill_a = [&](int u, int t) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            ah[mt][u] = *(const u32x4*)(ap[mt] + (size_t)t * astep);
            al[mt][u] = *(const u32x4*)(ap[mt] + a.a_lo + (size_t)t * astep);
        }
    };
    auto use = [&](int u) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[g][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, al[mt][u]),
                                                                     __builtin_bit_cast(bf16x8, w[g][u]), acc[g][mt], 0, 0, 0);
                acc[g][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ah[mt][u]),
                                                                     __builtin_bit_cast(bf16x8, w[g][u]), acc[g][mt], 0, 0, 0);
            }
    };
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n) fill_a(u, u);
    rms_scales<MT>(a, sm.rs);
    pre(std::false_type{});
    const int full = n / D, rem = n - full * D;
    for (int gI = 0; gI + 1 < full; ++gI) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            fill_w(u, (gI + 1) * D + u);
            fill_a(u, (gI + 1) * D + u);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (full > 0) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u);
            if (u < rem) {
                fill_w(u, full * D + u);
                fill_a(u, full * D + u);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < rem) use(u);
    // cross-wave reduction, one tile after the other through the same buffer
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) sm.red[ks][mt][(lg * 4 + r) * 16 + li] = acc[g][mt][r];
        __syncthreads();
        for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
            int e = idx & 255, mt = idx >> 8;
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < KS; ++k) s += sm.red[k][mt][e];
            int m = mt * 16 + (e >> 4);
            sm.out[g][m][e & 15] = s * sm.rs[m];
        }
        __syncthreads();
    }
}

// Variant for few rows (T*K small enough for LDS): the workgroup first copies its T activation rows
// (hi and lo terms) into LDS, and the loop takes its A operands from there.  The vector-memory queue
// then carries weight loads only (deeper ring, no registers spent on A look-ahead), and the lower
// register count lets more workgroups share a CU.  Up to 72 KB of rows (two workgroups per CU still fit: 4 rows at
// K = 4096); with 112 KB (one workgroup per CU) the 30B-shaped steps of 4 rows were 5 % slower than on the register
// path, while 2-4 rows at the 7B width gained 2-4 % over it.
constexpr int A_LDS_MAX_BYTES = 72 * 1024;
// The 16-wave variants (K beyond 4096) have the CU to themselves whatever their LDS use, so two or three of their
// rows may take up to 140 KB (the down projection at the 7B width: 88 and 132 KB; 23.1 us on the register path,
// which steps carrying a deferred row or two took until then, against 18 us; C3 at threshold 0.2: 2.262 -> 2.240 ms
// per step).  Four rows stay on the register path: see the 30B-shaped steps above.
constexpr int A_LDS_MAX_BYTES_16 = 140 * 1024;
__host__ __device__ inline int a_lds_row_stride(int K) { return 2 * K + 32; }  // elements; +64 B staggers the banks of two rows

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global load of
// the wave (its release fence covers vector memory as a whole), which is not wanted where a ring of weight loads is
// meant to stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int ATT_MAX_SPLITS = 16;
__host__ __device__ inline int att_part_stride(int hd) { return 32 + 16 * hd; }

template <int KS, int ATT, typename Pre>
__device__ __forceinline__ void gemm_mainloop_bf16_lds(const GemmArgs& a, int tile, GemmSmem<KS, 1>& sm, Pre pre) {
    extern __shared__ __attribute__((aligned(16))) unsigned char ee_dyn_smem[];
    __bf16* abuf = (__bf16*)ee_dyn_smem;
    const int ks = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int KT = a.KT, K = a.K;
    const int kt0 = (int)(((long)ks * KT) / KS), kt1 = (int)(((long)(ks + 1) * KT) / KS);
    const u32x4* wp = (const u32x4*)a.W + ((size_t)tile * KT + kt0) * 64 + lane;
    // (8 waves: the single-row path below keeps a row chunk next to the ring inside 80 registers per lane)
    constexpr int D = (KS == 8 && ATT == 0) ? 11 : 12;
    u32x4 w[D];
    const int n = kt1 - kt0;
    auto fill = [&](int u, int t) { w[u] = __builtin_nontemporal_load(wp + (size_t)t * 64); };
    const int rstride = a_lds_row_stride(K);
    const int cpr = K / 8;  // 16-byte chunks per row and term
    constexpr int RC = KS == 16 ? 2 : 1;  // 16-byte chunks of a row that a thread of the single-row path holds
    constexpr int MAXS = ATT > 0 ? ATT : 1;
    // ---- single row whose indices all travel in the kernel arguments (the batch-1 decode step).
    // Everything the workgroup needs before its first MFMA (sum-of-squares partials, the row or the attention
    // partials it is merged from, the epilogue's operands) is requested FIRST, then the ring, and nothing waits in
    // between: loads return in issue order, so the small loads are back after one memory latency and the ring
    // streams behind them.  For the compiler to place exactly those waits the path has no load in a loop, none that
    // hangs off another load and none through a pointer it cannot prove global (after such loads it waits for
    // everything outstanding), the ring is filled unconditionally (a surplus slot repeats a tile), and the barrier
    // that publishes the staged row orders LDS traffic only.  Per-workgroup time stamps had shown the ring going out
    // 2-4 us after kernel entry and every wave sitting at the barrier until its whole burst had arrived.
    const bool one_row = a.has_row_v && a.T == 1 && a.ssq_n <= 512 && cpr <= RC * KS * 64 && (ATT == 0 || (ATT <= 8 && a.att_ns <= MAXS));
    if (one_row) {
        const int slot = a.arow_v[0];
        // sum-of-squares partials of the row: wave 0, eight per lane (indices clamped, surplus values dropped)
        float sv[8];
        const bool do_ssq = a.ssq != nullptr && ks == 0;
        if (do_ssq) {
            const float* p = a.ssq + (size_t)slot * a.ssq_stride;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = lane + 64 * j;
                sv[j] = p[i < a.ssq_n ? i : a.ssq_n - 1];
            }
        }
        u32x4 rh[RC], rl[RC];
        float ms[MAXS], ls[MAXS];
        f32x4 o0[MAXS], o1[MAXS];
        if constexpr (ATT == 0) {
            const __bf16* srow = (const __bf16*)a.A + (size_t)slot * a.lda;
#pragma unroll
            for (int j = 0; j < RC; ++j) {
                int k8 = threadIdx.x + j * KS * 64;
                if (k8 >= cpr) k8 = cpr - 1;
                rh[j] = *(const u32x4*)(srow + k8 * 8);
                rl[j] = *(const u32x4*)(srow + a.a_lo + k8 * 8);
            }
        } else {
            // the row still lies as the attention kernel's per-split partials: this thread's chunk of every split
            int k8 = threadIdx.x;
            if (k8 >= cpr) k8 = cpr - 1;
            const int h = (k8 * 8) / a.att_hd, cc = (k8 * 8) % a.att_hd;
            const int rq = a.rq_v[0];
            const int qt = rq >> 4, qq = rq & 15;
            const int pstride = att_part_stride(a.att_hd);
            const float* pb = a.att_part + (size_t)(qt * a.att_H + h) * a.att_ns * pstride;
#pragma unroll
            for (int sp = 0; sp < MAXS; ++sp) {
                const float* ps = pb + (size_t)(sp < a.att_ns ? sp : a.att_ns - 1) * pstride;
                ms[sp] = ps[qq];
                ls[sp] = ps[16 + qq];
                o0[sp] = *(const f32x4*)(ps + 32 + qq * a.att_hd + cc);
                o1[sp] = *(const f32x4*)(ps + 32 + qq * a.att_hd + cc + 4);
            }
        }
        pre(std::true_type{});
#pragma unroll
        for (int u = 0; u < D; ++u) fill(u, u < n ? u : (n > 0 ? n - 1 : 0));
        // r = 1/sqrt(mean(x^2)+eps): lane sums in index order, a fixed butterfly
        if (ks == 0) {
            float r = 1.f;
            if (do_ssq) {
                float sp = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (lane + 64 * j < a.ssq_n) sp += sv[j];
                sp = wave_sum(sp);
                r = 1.0f / sqrtf(sp * a.inv_d + a.eps);
            }
            if (lane < 16) sm.rs[lane] = lane == 0 ? r : 1.f;
        }
        if constexpr (ATT == 0) {
#pragma unroll
            for (int j = 0; j < RC; ++j) {
                const int k8 = threadIdx.x + j * KS * 64;
                if (k8 < cpr) {
                    *(u32x4*)(abuf + k8 * 8) = rh[j];
                    *(u32x4*)(abuf + K + k8 * 8) = rl[j];
                }
            }
        } else {
            // merge of the splits, in split order, exactly as attn_merge_kernel does; two bf16 terms
            const int NS = a.att_ns;
            float M = -INFINITY;
#pragma unroll
            for (int sp = 0; sp < MAXS; ++sp)
                if (sp < NS) M = fmaxf(M, ms[sp]);
            float O[8], L = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) O[e] = 0.f;
#pragma unroll
            for (int sp = 0; sp < MAXS; ++sp) {
                if (sp >= NS || ms[sp] == -INFINITY) continue;
                const float f = __expf(ms[sp] - M);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    O[e] += f * o0[sp][e];
                    O[4 + e] += f * o1[sp][e];
                }
                L += f * ls[sp];
            }
            bf16x8 hv, lv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = O[e] / L;
                const __bf16 hi = (__bf16)v;
                hv[e] = hi;
                lv[e] = (__bf16)(v - (float)hi);
            }
            if ((int)threadIdx.x < cpr) {
                *(bf16x8*)(abuf + threadIdx.x * 8) = hv;
                *(bf16x8*)(abuf + K + threadIdx.x * 8) = lv;
            }
        }
        lds_barrier();
    } else {
        // ---- general prologue (several rows, or indices that have to be looked up): stage everything, then the ring.
        // Behind the ring the staged data would be back only with the ring's whole first burst (loads return in
        // order) and each dependent look-up would cost the wave another such wait; ahead of it the rows cost one
        // memory latency per pair of rows before the weights start to stream.
        // Sum-of-squares partials of the rows: wave w takes rows w, w + KS: lane-strided in order, a fixed butterfly.
        constexpr int RPW = (16 + KS - 1) / KS;  // rows per wave
        {
            float sv[RPW][8];
            const bool quick = a.ssq != nullptr && a.ssq_n <= 512;
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
                const int m = ks + j * KS;
                if (quick && m < a.T) {
                    const float* p = a.ssq + (size_t)gemm_slot(a, m) * a.ssq_stride;
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj) {
                        const int i = lane + 64 * jj;
                        sv[j][jj] = p[i < a.ssq_n ? i : a.ssq_n - 1];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
                const int m = ks + j * KS;
                float sp = 0.f;
                if (a.ssq != nullptr && m < a.T) {
                    if (quick) {
#pragma unroll
                        for (int jj = 0; jj < 8; ++jj)
                            if (lane + 64 * jj < a.ssq_n) sp += sv[j][jj];
                    } else {
                        const float* p = a.ssq + (size_t)gemm_slot(a, m) * a.ssq_stride;
                        for (int i = lane; i < a.ssq_n; i += 64) sp += p[i];
                    }
                }
                sp = wave_sum(sp);
                if (lane == 0 && m < 16) sm.rs[m] = (a.ssq != nullptr && m < a.T) ? 1.0f / sqrtf(sp * a.inv_d + a.eps) : 1.f;
            }
        }
        if constexpr (ATT) {
            // The rows are attention outputs that still lie as per-split partials (max, sum, unnormalised
            // output): merge the splits here, in split order, exactly as attn_merge_kernel does, and split the
            // result into its two bf16 terms.  Saves a launch between attention and this projection.
            const int pstride = att_part_stride(a.att_hd), NS = a.att_ns;
            for (int c = threadIdx.x; c < a.T * cpr; c += blockDim.x) {
                const int m = c / cpr, k8 = c - m * cpr;
                const int h = (k8 * 8) / a.att_hd, cc = (k8 * 8) % a.att_hd;
                const int rq = a.has_row_v ? a.rq_v[m] : a.att_desc->row_qt[m];
                const int qt = rq >> 4, qq = rq & 15;
                const float* pb = a.att_part + (size_t)(qt * a.att_H + h) * NS * pstride;
                // every load of every split goes out before the first is used: one memory round trip in all
                constexpr int MAXS = ATT > 0 ? ATT : 1;
                float ms[MAXS], ls[MAXS];
                f32x4 o0[MAXS], o1[MAXS];
    #pragma unroll
                for (int sp = 0; sp < MAXS; ++sp) {
                    if (sp < NS) {  // (uniform over the workgroup)
                        const float* ps = pb + (size_t)sp * pstride;
                        ms[sp] = ps[qq];
                        ls[sp] = ps[16 + qq];
                        o0[sp] = *(const f32x4*)(ps + 32 + qq * a.att_hd + cc);
                        o1[sp] = *(const f32x4*)(ps + 32 + qq * a.att_hd + cc + 4);
                    }
                }
                float M = -INFINITY;
    #pragma unroll
                for (int sp = 0; sp < MAXS; ++sp)
                    if (sp < NS) M = fmaxf(M, ms[sp]);
                float O[8], L = 0.f;
    #pragma unroll
                for (int e = 0; e < 8; ++e) O[e] = 0.f;
    #pragma unroll
                for (int sp = 0; sp < MAXS; ++sp) {
                    if (sp >= NS || ms[sp] == -INFINITY) continue;
                    const float f = __expf(ms[sp] - M);
    #pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        O[e] += f * o0[sp][e];
                        O[4 + e] += f * o1[sp][e];
                    }
                    L += f * ls[sp];
                }
                bf16x8 hv, lv;
    #pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = O[e] / L;
                    const __bf16 hi = (__bf16)v;
                    hv[e] = hi;
                    lv[e] = (__bf16)(v - (float)hi);
                }
                *(bf16x8*)(abuf + (size_t)m * rstride + k8 * 8) = hv;
                *(bf16x8*)(abuf + (size_t)m * rstride + K + k8 * 8) = lv;
            }
        } else {
            for (int m = 0; m < a.T; m += 2) {  // (two rows per memory round trip; a row's slot is uniform)
                const int m1 = m + 1 < a.T ? m + 1 : m;
                const __bf16* s0 = (const __bf16*)a.A + (size_t)gemm_slot(a, m) * a.lda;
                const __bf16* s1 = (const __bf16*)a.A + (size_t)gemm_slot(a, m1) * a.lda;
                for (int k8 = threadIdx.x; k8 < cpr; k8 += blockDim.x) {
                    const u32x4 h0 = *(const u32x4*)(s0 + k8 * 8), l0 = *(const u32x4*)(s0 + a.a_lo + k8 * 8);
                    const u32x4 h1 = *(const u32x4*)(s1 + k8 * 8), l1 = *(const u32x4*)(s1 + a.a_lo + k8 * 8);
                    *(u32x4*)(abuf + (size_t)m * rstride + k8 * 8) = h0;
                    *(u32x4*)(abuf + (size_t)m * rstride + K + k8 * 8) = l0;
                    *(u32x4*)(abuf + (size_t)m1 * rstride + k8 * 8) = h1;
                    *(u32x4*)(abuf + (size_t)m1 * rstride + K + k8 * 8) = l1;
                }
            }
        }
        pre(std::false_type{});
#pragma unroll
        for (int u = 0; u < D; ++u) fill(u, u < n ? u : (n > 0 ? n - 1 : 0));
        lds_barrier();
    }
    const __bf16* ar = abuf + (size_t)(li < a.T ? li : 0) * rstride + (size_t)kt0 * 32 + lg * 8;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    auto use = [&](int u, int t) {
        bf16x8 h = *(const bf16x8*)(ar + (size_t)t * 32);
        bf16x8 l = *(const bf16x8*)(ar + K + (size_t)t * 32);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(l, __builtin_bit_cast(bf16x8, w[u]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(h, __builtin_bit_cast(bf16x8, w[u]), acc, 0, 0, 0);
    };
    const int full = n / D, rem = n - full * D;
    for (int gI = 0; gI + 1 < full; ++gI) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u, gI * D + u);
            fill(u, (gI + 1) * D + u);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (full > 0) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            use(u, (full - 1) * D + u);
            if (u < rem) fill(u, full * D + u);
        }
    }
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < rem) use(u, full * D + u);
#pragma unroll
    for (int r = 0; r < 4; ++r) sm.red[ks][0][(lg * 4 + r) * 16 + li] = acc[r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 256; idx += blockDim.x) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < KS; ++k) s += sm.red[k][0][idx];
        int m = idx >> 4;
        sm.out[0][m][idx & 15] = s * sm.rs[m];
    }
    __syncthreads();
}

// fp32 path (tiny model, parity only): plain FMA loop, weights row-major [tile][16][K]
template <int KS, int MT, typename Pre>
__device__ __forceinline__ void gemm_mainloop_f32(const GemmArgs& a, int tile, GemmSmem<KS, MT>& sm, Pre pre) {
    rms_scales<MT>(a, sm.rs);
    pre(std::false_type{});
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
        int m = idx >> 4, c = idx & 15;
        float s = 0.f;
        if (m < a.T) {
            int slot = a.arow ? a.arow[m] : m;
            const float* ar = (const float*)a.A + (size_t)slot * a.lda;
            const float* wr = (const float*)a.W + ((size_t)tile * 16 + c) * a.K;
            for (int k = 0; k < a.K; ++k) s = fmaf(ar[k], wr[k], s);
        }
        sm.out[0][m][c] = s * sm.rs[m];
    }
    __syncthreads();
}

// `pre` runs once the first weight loads are in flight: the place to fetch what the epilogue needs.
// Leaves tile g of the workgroup (g < G, tile index tile0 + g) in sm.out[g].
template <typename ST, int KS, int MT, bool ALDS, int G, typename Pre, int ATT = 0>
__device__ __forceinline__ void gemm_mainloop(const GemmArgs& a, int tile0, GemmSmem<KS, MT, G>& sm, Pre pre) {
    if constexpr (G > 1) {
        static_assert(sizeof(ST) == 2 && !ALDS, "several tiles per workgroup: bf16 register path only");
        gemm_mainloop_bf16_multi<KS, MT, G>(a, tile0, sm, pre);
    } else if constexpr (sizeof(ST) == 2 && ALDS)
        gemm_mainloop_bf16_lds<KS, ATT>(a, tile0, sm, pre);
    else if constexpr (sizeof(ST) == 2)
        gemm_mainloop_bf16<KS, MT>(a, tile0, sm, pre);  // (its first __syncthreads orders rs before use)
    else
        gemm_mainloop_f32<KS, MT>(a, tile0, sm, pre);
}

// (Launch bounds of the few-rows variants: 6 waves per SIMD, i.e. at most 80 registers per lane, so that three
// 8-wave workgroups share a CU; a few registers more would cost a whole workgroup of residency.)
// ---- epilogue 1: rotary embedding, q to the workspace, k and v into the paged cache.
// Tile (part, head h, c): columns 0..7 = features h*hd + c*8 + i, columns 8..15 = their rotary partners.
template <typename ST>
struct QkvArgs {
    ST* q;
    size_t q_lo;
    int d;
    const float2* rope_cs;
    ST* kv_layer;  // pool + layer * layer_stride
    size_t blk_stride;
    int H, hd, BT;
    const int32_t* pos;    // per row: position, physical KV block
    const int32_t* kvblk;
    int32_t pos_v0, blk_v0;  // those of row 0 (a launch of one row reads them here)
};

template <typename ST, int KS, int MT, bool ALDS, int G = 1>
__global__ __launch_bounds__(KS * 64, ALDS ? (KS == 16 ? 4 : 6) : 1) void gemm_qkv_kernel(GemmArgs a, QkvArgs<ST> e) {
    __shared__ GemmSmem<KS, MT, G> sm;
    const int per_head = e.hd / 16, per_part = e.H * per_head;
    const int half = e.hd / 2;
    const int tile0 = blockIdx.x * G;
    // epilogue operands of this thread's first (row, column pair) of the first tile, fetched while the weights stream
    const int m0 = threadIdx.x >> 3, i0 = threadIdx.x & 7;
    int pos0 = 0, blk0 = 0;
    float2 cs0 = make_float2(1.f, 0.f);
    gemm_mainloop<ST, KS, MT, ALDS, G>(a, tile0, sm, [&](auto one_row) {
        if (m0 < a.T) {
            if constexpr (decltype(one_row)::value) {  // (the row's position and block sit in the kernel arguments)
                pos0 = e.pos_v0;
                blk0 = e.blk_v0;
            } else {
                pos0 = e.pos[m0];
                blk0 = e.kvblk[m0];
            }
            if (tile0 / per_part < 2) cs0 = e.rope_cs[(size_t)pos0 * half + (tile0 % per_head) * 8 + i0];
        }
    });
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int tile = tile0 + g;
        if (tile >= a.n_tiles) break;
        const float(*out)[16] = sm.out[g];
        const int part = tile / per_part;  // 0 q, 1 k, 2 v
        const int rem = tile % per_part;
        const int h = rem / per_head, c = rem % per_head;
        for (int idx = threadIdx.x; idx < MT * 128; idx += blockDim.x) {
            int m = idx >> 3, i = idx & 7;
            if (m >= a.T) continue;
            float lo = out[m][i], hi = out[m][8 + i];
            int pos = pos0, blk = blk0;
            float2 cs = cs0;
            if (g != 0 || idx != (int)threadIdx.x) {
                pos = e.pos[m];
                blk = e.kvblk[m];
                if (part < 2) cs = e.rope_cs[(size_t)pos * half + c * 8 + i];
            }
            if (part < 2) {
                float nlo = lo * cs.x - hi * cs.y;
                float nhi = hi * cs.x + lo * cs.y;
                lo = nlo;
                hi = nhi;
            }
            if (part == 0) {
                ST* qp = e.q + (size_t)m * e.d + h * e.hd + c * 8 + i;
                store_split<ST>(qp, e.q_lo, lo);
                store_split<ST>(qp + half, e.q_lo, hi);
            } else if (part == 1) {  // K block: [head][position][feature]
                ST* kp = e.kv_layer + (size_t)blk * e.blk_stride + ((size_t)h * e.BT + (pos % e.BT)) * e.hd + c * 8 + i;
                kp[0] = cvt_st<ST>(lo);
                kp[half] = cvt_st<ST>(hi);
            } else {  // V block, transposed in groups of 32 positions: [head][position / 32][feature][position % 32], so
                      // that attention reads the P.V operands of a 32-position tile directly and as one contiguous piece
                const int pin = pos % e.BT;
                ST* vp = e.kv_layer + (size_t)blk * e.blk_stride + (size_t)e.H * e.BT * e.hd + (size_t)h * e.hd * e.BT +
                         (size_t)(pin >> 5) * (e.hd * 32) + (c * 8 + i) * 32 + (pin & 31);
                vp[0] = cvt_st<ST>(lo);
                vp[half * 32] = cvt_st<ST>(hi);
            }
        }
    }
}

// ---- epilogue 2: residual add; normalised-input operand(s) for what follows; sum-of-squares partial
template <typename ST>
struct ResidArgs {
    float* x;
    ST* xg;
    ST* xgh;
    size_t xs_lo;  // lo offset of xg and xgh
    float* ssq_out;
    int ssq_stride;
    const float* g_next;
    const float* g_head;
    int d;
    const int32_t* xrow;  // per row: slot in the residual store
    ST* xg_pk;            // optional: the same operand again, dense rows of this launch in packed order
    size_t xg_pk_lo;
    int has_v;            // up to 16 rows: the slots by value
    int32_t xrow_v[16];
};

template <typename ST>
__device__ __forceinline__ int resid_slot(const ResidArgs<ST>& e, int m) {
    return e.has_v ? e.xrow_v[m] : e.xrow[m];
}

template <typename ST, int KS, int MT, bool ALDS, int ATT, int G>
__device__ __forceinline__ void gemm_resid_body(const GemmArgs& a, const ResidArgs<ST>& e) {
    __shared__ GemmSmem<KS, MT, G> sm;
    const int tile0 = blockIdx.x * G;
    // epilogue operands of this thread's first element of the first tile, fetched while the weights stream
    const int m0 = threadIdx.x >> 4, i0 = threadIdx.x & 15;
    size_t o0 = 0;
    float x0 = 0.f, gn0 = 0.f, gh0 = 0.f;
    auto pre = [&](auto one_row) {
        if (m0 < a.T) {
            if constexpr (decltype(one_row)::value)
                o0 = (size_t)e.xrow_v[0] * e.d + tile0 * 16 + i0;
            else
                o0 = (size_t)resid_slot(e, m0) * e.d + tile0 * 16 + i0;
            x0 = e.x[o0];
            gn0 = e.g_next[tile0 * 16 + i0];
            if (e.xgh) gh0 = e.g_head[tile0 * 16 + i0];
        }
    };
    gemm_mainloop<ST, KS, MT, ALDS, G, decltype(pre), ATT>(a, tile0, sm, pre);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int tile = tile0 + g;
        if (tile >= a.n_tiles) break;  // (uniform over the workgroup)
        float(*out)[16] = sm.out[g];
        const int n0 = tile * 16;
        for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
            int m = idx >> 4, i = idx & 15;
            if (m >= a.T) continue;
            size_t o = o0;
            float xv = x0, gn = gn0, gh = gh0;
            if (g != 0 || idx != (int)threadIdx.x) {
                o = (size_t)resid_slot(e, m) * e.d + n0 + i;
                xv = e.x[o];
                gn = e.g_next[n0 + i];
                if (e.xgh) gh = e.g_head[n0 + i];
            }
            float v = xv + out[m][i];
            e.x[o] = v;
            out[m][i] = v;
            store_split<ST>(e.xg + o, e.xs_lo, v * gn);
            if (e.xgh) store_split<ST>(e.xgh + o, e.xs_lo, v * gh);
            if (e.xg_pk) store_split<ST>(e.xg_pk + pk_index(m, n0 + i, e.d / 32), e.xg_pk_lo, v * gn);
        }
        __syncthreads();
        for (int m = threadIdx.x; m < MT * 16; m += blockDim.x) {
            if (m >= a.T) continue;
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) s += out[m][i] * out[m][i];
            e.ssq_out[(size_t)resid_slot(e, m) * e.ssq_stride + tile] = s;
        }
    }
}

template <typename ST, int KS, int MT, bool ALDS, int G = 1>
__global__ __launch_bounds__(KS * 64, ALDS ? (KS == 16 ? 4 : 6) : 1) void gemm_resid_kernel(GemmArgs a, ResidArgs<ST> e) {
    gemm_resid_body<ST, KS, MT, ALDS, 0, G>(a, e);
}

// O projection whose input rows are merged from the attention kernel's split partials while being staged
template <int KS, int MAXS>
__global__ __launch_bounds__(KS * 64) void gemm_resid_att_kernel(GemmArgs a, ResidArgs<__bf16> e) {
    gemm_resid_body<__bf16, KS, 1, true, MAXS, 1>(a, e);
}

// ---- epilogue 3: SwiGLU.  Tile j: columns 0..7 = gate features 8j.., columns 8..15 = the matching up features
template <typename ST, int KS, int MT, bool ALDS, int G = 1>
__global__ __launch_bounds__(KS * 64, ALDS ? (KS == 16 ? 4 : 6) : 1) void gemm_swiglu_kernel(GemmArgs a, ST* act, size_t act_lo, int F, int act_pk) {
    __shared__ GemmSmem<KS, MT, G> sm;
    const int tile0 = blockIdx.x * G;
    gemm_mainloop<ST, KS, MT, ALDS, G>(a, tile0, sm, [](auto) {});
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int tile = tile0 + g;
        if (tile >= a.n_tiles) break;
        const float(*out)[16] = sm.out[g];
        for (int idx = threadIdx.x; idx < MT * 128; idx += blockDim.x) {
            int m = idx >> 3, i = idx & 7;
            if (m >= a.T) continue;
            float gt = out[m][i], up = out[m][8 + i];
            float sl = gt / (1.0f + expf(-gt));
            store_split_at<ST>(act, act_lo, m, tile * 8 + i, F, act_pk, sl * up);
        }
    }
}

// ---- epilogue 4: exit / final head.  Per workgroup: (max, arg max, sum exp) of its 16 logits per row.
// A one-workgroup kernel launched right after merges the partials in a fixed order and takes the exit
// decision (an in-kernel "last workgroup merges" scheme needs a device-wide fence in every workgroup,
// which costs more than the extra launch).
struct HeadArgs {
    HeadPartial* partials;  // [n_wg][EE_MAX_SEQS]
    float* logits;          // optional [row][V]
    int V;
};

__device__ __forceinline__ void merge_partial(float& m, float& s, int& i, float m2, float s2, int i2) {
    if (m2 > m || (m2 == m && i2 < i)) {
        s = s * expf(m - m2) + s2;
        m = m2;
        i = i2;
    } else {
        s = s + s2 * expf(m2 - m);
    }
}

template <typename ST, int KS, int MT, bool ALDS, int G = 1>
__global__ __launch_bounds__(KS * 64, ALDS ? (KS == 16 ? 4 : 6) : 1) void gemm_head_kernel(GemmArgs a, HeadArgs e) {
    __shared__ GemmSmem<KS, MT, G> sm;
    const int tile0 = blockIdx.x * G;
    gemm_mainloop<ST, KS, MT, ALDS, G>(a, tile0, sm, [](auto) {});
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int tile = tile0 + g;
        if (tile >= a.n_tiles) break;
        const float(*out)[16] = sm.out[g];
        const int n0 = tile * 16;
        if (e.logits) {
            for (int idx = threadIdx.x; idx < MT * 256; idx += blockDim.x) {
                int m = idx >> 4, c = idx & 15;
                if (m < a.T) e.logits[(size_t)m * e.V + n0 + c] = out[m][c];
            }
        }
        for (int m = threadIdx.x; m < MT * 16; m += blockDim.x) {
            if (m >= a.T) continue;
            float mx = out[m][0];
            int ix = 0;
#pragma unroll
            for (int c = 1; c < 16; ++c)
                if (out[m][c] > mx) {
                    mx = out[m][c];
                    ix = c;
                }
            float s = 0.f;
#pragma unroll
            for (int c = 0; c < 16; ++c) s += expf(out[m][c] - mx);
            HeadPartial p;
            p.max = mx;
            p.sum = s;
            p.idx = n0 + ix;
            p.pad = 0;
            e.partials[(size_t)tile * EE_MAX_SEQS + m] = p;
        }
    }
}

// confidence = 1 / sum_i exp(z_i - z_max); exit iff confidence >= threshold (or always, for the final head)
__global__ __launch_bounds__(512) void head_merge_kernel(const HeadPartial* __restrict__ partials, int n_wg, int T, int mode,
                                                         float threshold, HeadResult* results,
                                                         const SegDesc* __restrict__ desc, int tag) {
    __shared__ float redm[512], reds[512];
    __shared__ int redi[512];
    // one workgroup per row; thread t folds workgroups t, t+512, ... in ascending order (eight loads in flight at a
    // time: the partials come from the other XCDs, so each load is a trip to memory), then a fixed tree over the
    // threads: through LDS down to one wave, by lane shuffles inside it (the same pairs either way)
    const int m = blockIdx.x;
    if (m >= T) return;
    const int out_slot = desc->head_slot[m];  // (requested now, used at the very end)
    {
        float mx = -INFINITY, s = 0.f;
        int ix = 0x7fffffff;
        for (int w0 = threadIdx.x; w0 < n_wg; w0 += 8 * 512) {
            HeadPartial p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int w = w0 + j * 512;
                if (w < n_wg) p[j] = partials[(size_t)w * EE_MAX_SEQS + m];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (w0 + j * 512 < n_wg) merge_partial(mx, s, ix, p[j].max, p[j].sum, p[j].idx);
        }
        redm[threadIdx.x] = mx;
        reds[threadIdx.x] = s;
        redi[threadIdx.x] = ix;
        __syncthreads();
        for (int o = 256; o >= 64; o >>= 1) {
            if ((int)threadIdx.x < o) {
                float m1 = redm[threadIdx.x], s1 = reds[threadIdx.x];
                int i1 = redi[threadIdx.x];
                float m2 = redm[threadIdx.x + o], s2 = reds[threadIdx.x + o];
                int i2 = redi[threadIdx.x + o];
                if (s2 > 0.f || m2 > -INFINITY) merge_partial(m1, s1, i1, m2, s2, i2);
                redm[threadIdx.x] = m1;
                reds[threadIdx.x] = s1;
                redi[threadIdx.x] = i1;
            }
            __syncthreads();
        }
        if (threadIdx.x < 64) {
            float m1 = redm[threadIdx.x], s1 = reds[threadIdx.x];
            int i1 = redi[threadIdx.x];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float m2 = __shfl_down(m1, o), s2 = __shfl_down(s1, o);
                const int i2 = __shfl_down(i1, o);
                if ((int)threadIdx.x < o && (s2 > 0.f || m2 > -INFINITY)) merge_partial(m1, s1, i1, m2, s2, i2);
            }
            if (threadIdx.x == 0) {
                reds[0] = s1;
                redi[0] = i1;
            }
        }
        if (threadIdx.x == 0) {
            float conf = 1.0f / reds[0];
            HeadResult r;
            r.token = redi[0];
            r.conf = conf;
            r.fired = (mode == HEAD_EMIT) || (conf >= threshold);
            r.pad = 0;
            // The results live in host memory that the host polls: the tag goes last, after a system-wide
            // fence, so that a host that sees the tag sees the rest.
            HeadResult* dst = results + out_slot;
            dst->token = r.token;
            dst->conf = r.conf;
            dst->fired = r.fired;
            __threadfence_system();
            __hip_atomic_store(&dst->pad, tag, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        __syncthreads();
    }
}

// ---- host-side dispatch
static GemmArgs make_args(const GemmCommon& c) {
    GemmArgs a;
    a.W = c.W;
    a.K = c.K;
    a.KT = c.K / 32;
    a.A = c.A;
    a.a_lo = c.a_lo;
    a.lda = c.lda;
    a.arow = c.arow;
    a.ssq = c.ssq;
    a.ssq_stride = c.ssq_stride;
    a.ssq_n = c.ssq_n;
    a.inv_d = c.inv_d;
    a.eps = c.eps;
    a.T = c.T;
    a.n_tiles = c.N / 16;
    a.has_row_v = 0;
    if (c.desc_host != nullptr && c.T <= 16) {
        a.has_row_v = 1;
        const int32_t* rows = c.arow ? (const int32_t*)((const char*)c.desc_host + ((const char*)c.arow - (const char*)c.desc)) : nullptr;
        for (int i = 0; i < 16; ++i) {
            a.arow_v[i] = i < c.T ? (rows ? rows[i] : i) : 0;
            a.rq_v[i] = i < c.T ? c.desc_host->row_qt[i] : 0;
        }
    }
    a.a_packed = c.a_packed;
    a.att_part = c.att_part;
    a.att_desc = c.desc;
    a.att_ns = c.att_ns;
    a.att_H = c.att_H;
    a.att_hd = c.att_hd;
    return a;
}

static int mt_of(int T) { return T <= 16 ? 1 : (T <= 32 ? 2 : 4); }
// waves per workgroup: each should stream about 16 k-tiles (16 KB)
static int ks_of(const GemmCommon& c) {
    if (c.dtype != EE_BF16) return 4;
    int kt = c.K / 32;
    if (kt <= 64) return 4;
    if (kt <= 128 || c.T > 16) return 8;  // (16 waves of 1024 threads leave 128 registers each: one row tile only)
    return 16;
}

// LDS bytes for the few-rows variant, or 0 when the rows do not fit
static size_t a_lds_bytes(const GemmCommon& c) {
    if (c.dtype != EE_BF16 || c.T > 16) return 0;
    size_t b = (size_t)c.T * a_lds_row_stride(c.K) * 2;
    if (ks_of(c) == 16 && c.T <= 3) return b <= (size_t)A_LDS_MAX_BYTES_16 ? b : 0;
    return b <= (size_t)A_LDS_MAX_BYTES ? b : 0;
}

// Column tiles per workgroup for the register path: as many (4 for one row tile, else 2) as still leave
// gemm_min_wgs() workgroups, so that the rows' operands are re-read from L2 by fewer workgroups without
// starving the chip of weight streams.  (GemmCommon::min_wgs: 512 unless the model's configuration lowers it, which
// tests do to reach these variants on small models.)
static int g_of(int mt, int n_tiles, int min_wgs) {
    auto gemm_min_wgs = [min_wgs]() { return min_wgs >= 1 ? min_wgs : 512; };
    if (mt == 1 && n_tiles / 4 >= gemm_min_wgs()) return 4;
    // Up to two row tiles: at these register counts one workgroup of 8 waves is resident per CU, so a launch runs in
    // rounds of 256 workgroups.  Give a workgroup as many tiles as there would be rounds (2..6): one round, the same
    // makespan in tiles, and the row operands and prologues are paid once instead of once per round (Q|K|V at the 7B
    // width: 768 tiles = 256 x 3; gate|up: 1376 tiles = 230 x 6).  (The test hook scales the 256 with its threshold.)
    const int cus = gemm_min_wgs() >= 512 ? 256 : (gemm_min_wgs() / 2 > 0 ? gemm_min_wgs() / 2 : 1);
    const int rounds = (n_tiles + cus - 1) / cus;
    if (mt <= 2 && rounds >= 2 && rounds <= 6) return rounds;
    if (n_tiles / 2 >= gemm_min_wgs()) return 2;
    return 1;
}

#define EE_LAUNCH_G(ST, KERNEL, KS_, MT_, ...)                                                        \
    do {                                                                                              \
        constexpr int MTG = MT_ <= 2 ? MT_ : 1; /* 3..6 tiles: up to two row tiles */                 \
        if (_g == 4 && MT_ == 1) EE_LAUNCH((KERNEL<ST, KS_, 1, false, (KS_ == 16 ? 2 : 4)>), grid, block, s, __VA_ARGS__); \
        else if (_g == 3 && MT_ <= 2) EE_LAUNCH((KERNEL<ST, KS_, MTG, false, (KS_ == 16 ? 2 : 3)>), grid, block, s, __VA_ARGS__); \
        else if (_g == 4 && MT_ <= 2) EE_LAUNCH((KERNEL<ST, KS_, MTG, false, (KS_ == 16 ? 2 : 4)>), grid, block, s, __VA_ARGS__); \
        else if (_g == 5 && MT_ <= 2) EE_LAUNCH((KERNEL<ST, KS_, MTG, false, (KS_ == 16 ? 2 : 5)>), grid, block, s, __VA_ARGS__); \
        else if (_g == 6 && MT_ <= 2) EE_LAUNCH((KERNEL<ST, KS_, MTG, false, (KS_ == 16 ? 2 : 6)>), grid, block, s, __VA_ARGS__); \
        else if (_g >= 2) EE_LAUNCH((KERNEL<ST, KS_, MT_, false, 2>), grid, block, s, __VA_ARGS__);   \
        else EE_LAUNCH((KERNEL<ST, KS_, MT_, false, 1>), grid, block, s, __VA_ARGS__);                \
    } while (0)

// more dynamic LDS than the default limit has to be asked for once per kernel
template <auto K>
static hipError_t lds_limit_once() {
    static hipError_t e = hipFuncSetAttribute((const void*)K, hipFuncAttributeMaxDynamicSharedMemorySize, A_LDS_MAX_BYTES_16);
    return e;
}
#define EE_LAUNCH_LDS(KERNEL_INST, ...)                                         \
    do {                                                                        \
        hipError_t _le = lds_limit_once<&KERNEL_INST>();                        \
        if (_le != hipSuccess) return _le;                                      \
        EE_LAUNCH_SM((KERNEL_INST), __VA_ARGS__);                               \
    } while (0)

#define EE_DISPATCH(ST, KERNEL, ...)                                                                               \
    do {                                                                                                           \
        int _ks = ks_of(c);                                                                                        \
        const int _mt = mt_of(c.T), _nt = c.N / 16;                                                                \
        const size_t _sm = a_lds_bytes(c);                                                                         \
        int _g = _sm ? 1 : g_of(_mt, _nt, c.min_wgs);                                                                        \
        /* 1024 threads leave 128 registers per lane: 3..6 tiles need the 8-wave variants (each wave then */       \
        /* streams K/8, still >= 8 k-tiles here); otherwise 16 waves stay at two tiles */                          \
        if (_ks == 16 && _g >= 3) { if (_g <= 6 && _mt <= 2) _ks = 8; else _g = 2; }                               \
        dim3 grid((_nt + _g - 1) / _g), block(_ks * 64);                                                           \
        if (_sm) {                                                                                                 \
            if (_ks == 4) EE_LAUNCH_LDS((KERNEL<ST, 4, 1, true, 1>), grid, block, _sm, s, __VA_ARGS__);            \
            else if (_ks == 8) EE_LAUNCH_LDS((KERNEL<ST, 8, 1, true, 1>), grid, block, _sm, s, __VA_ARGS__);       \
            else EE_LAUNCH_LDS((KERNEL<ST, 16, 1, true, 1>), grid, block, _sm, s, __VA_ARGS__);                    \
        } else if (_ks == 4 && _mt == 1) EE_LAUNCH_G(ST, KERNEL, 4, 1, __VA_ARGS__);                               \
        else if (_ks == 4 && _mt == 2) EE_LAUNCH_G(ST, KERNEL, 4, 2, __VA_ARGS__);                                 \
        else if (_ks == 4) EE_LAUNCH_G(ST, KERNEL, 4, 4, __VA_ARGS__);                                             \
        else if (_ks == 8 && _mt == 1) EE_LAUNCH_G(ST, KERNEL, 8, 1, __VA_ARGS__);                                 \
        else if (_ks == 8 && _mt == 2) EE_LAUNCH_G(ST, KERNEL, 8, 2, __VA_ARGS__);                                 \
        else if (_ks == 8) EE_LAUNCH_G(ST, KERNEL, 8, 4, __VA_ARGS__);                                             \
        else EE_LAUNCH_G(ST, KERNEL, 16, 1, __VA_ARGS__);                                                          \
    } while (0)

#define EE_DISPATCH_F32(KERNEL, ...)                                                             \
    do {                                                                                         \
        const int _mt = mt_of(c.T);                                                              \
        dim3 block(256);                                                                         \
        dim3 grid(c.N / 16);                                                                     \
        if (_mt == 1) EE_LAUNCH((KERNEL<float, 4, 1, false>), grid, block, s, __VA_ARGS__);      \
        else if (_mt == 2) EE_LAUNCH((KERNEL<float, 4, 2, false>), grid, block, s, __VA_ARGS__); \
        else EE_LAUNCH((KERNEL<float, 4, 4, false>), grid, block, s, __VA_ARGS__);               \
    } while (0)

int gemm_resid_tiles_per_wg() { return 1; }

bool gemm_rows_fit_lds(int dtype, int T, int K) {
    GemmCommon c{};
    c.dtype = dtype;
    c.T = T;
    c.K = K;
    return a_lds_bytes(c) != 0;
}

// Rows are processed in passes of at most 64 (the largest row tile count the kernels are built for).
constexpr int PASS_ROWS = 64;

static GemmCommon pass_of(const GemmCommon& c, int r0) {
    GemmCommon p = c;
    p.T = c.T - r0 < PASS_ROWS ? c.T - r0 : PASS_ROWS;
    if (c.arow) p.arow = c.arow + r0;
    if (c.a_packed)  // (r0 is a multiple of 16: whole row groups)
        p.A = (const char*)c.A + (size_t)(r0 / 16) * (c.K / 32) * 512 * 2;
    else if (!c.arow)
        p.A = (const char*)c.A + (size_t)r0 * c.lda * (c.dtype == EE_BF16 ? 2 : 4);
    return p;
}

static const int32_t* desc_array(const SegDesc* d, size_t field_offset, int r0) {
    return (const int32_t*)((const char*)d + field_offset) + r0;
}

hipError_t launch_gemm_qkv(const GemmCommon& cc, void* q, size_t q_lo, const float* rope_cs, const KvGeom& kv, int layer,
                           hipStream_t s) {
    for (int r0 = 0; r0 < cc.T; r0 += PASS_ROWS) {
        const GemmCommon c = pass_of(cc, r0);
        GemmArgs a = make_args(c);
        const int d = c.N / 3;
        const int32_t* pos = desc_array(c.desc, offsetof(SegDesc, pos), r0);
        const int32_t* blk = desc_array(c.desc, offsetof(SegDesc, kvblk), r0);
        if (c.dtype == EE_BF16) {
            QkvArgs<__bf16> e{(__bf16*)q + (size_t)r0 * d, q_lo, d, (const float2*)rope_cs,
                              (__bf16*)kv.pool + (size_t)layer * kv.layer_stride, kv.blk_stride, kv.H, kv.hd, kv.BT, pos, blk,
                              c.desc_host ? c.desc_host->pos[r0] : 0, c.desc_host ? c.desc_host->kvblk[r0] : 0};
            EE_DISPATCH(__bf16, gemm_qkv_kernel, a, e);
        } else {
            QkvArgs<float> e{(float*)q + (size_t)r0 * d, q_lo, d, (const float2*)rope_cs,
                             (float*)kv.pool + (size_t)layer * kv.layer_stride, kv.blk_stride, kv.H, kv.hd, kv.BT, pos, blk, 0, 0};
            EE_DISPATCH_F32(gemm_qkv_kernel, a, e);
        }
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

template <typename ST>
static void fill_rows(ResidArgs<ST>& e, const GemmCommon& c, int T_all) {
    if (c.desc_host == nullptr || T_all > 16) return;
    e.has_v = 1;
    for (int i = 0; i < T_all; ++i) e.xrow_v[i] = c.desc_host->xrow[i];
}

hipError_t launch_gemm_resid(const GemmCommon& cc, float* x, void* xg, void* xgh, size_t xs_lo, float* ssq_out,
                             const float* g_next, const float* g_head, int d, void* xg_pk, size_t xg_pk_lo, hipStream_t s) {
    for (int r0 = 0; r0 < cc.T; r0 += PASS_ROWS) {
        const GemmCommon c = pass_of(cc, r0);
        GemmArgs a = make_args(c);
        const int32_t* xrow = desc_array(c.desc, offsetof(SegDesc, xrow), r0);
        if (c.dtype == EE_BF16 && c.att_part != nullptr) {
            // input still lies as attention split partials: only the few-rows variant can merge them
            const size_t sm = a_lds_bytes(c);
            if (sm == 0 || cc.T > PASS_ROWS) return hipErrorInvalidValue;
            ResidArgs<__bf16> e{x, (__bf16*)xg, (__bf16*)xgh, xs_lo, ssq_out, c.ssq_stride, g_next, g_head, d, xrow, nullptr, 0, 0, {}};
            fill_rows(e, c, cc.T);
            // (at most 8 waves: the merge holds every split's partials in registers at once)
            const int ks = ks_of(c) == 4 ? 4 : 8;
            dim3 grid(c.N / 16), block(ks * 64);
            if (ks == 4 && c.att_ns <= 8) EE_LAUNCH_LDS((gemm_resid_att_kernel<4, 8>), grid, block, sm, s, a, e);
            else if (ks == 4) EE_LAUNCH_LDS((gemm_resid_att_kernel<4, ATT_MAX_SPLITS>), grid, block, sm, s, a, e);
            else if (c.att_ns <= 8) EE_LAUNCH_LDS((gemm_resid_att_kernel<8, 8>), grid, block, sm, s, a, e);
            else EE_LAUNCH_LDS((gemm_resid_att_kernel<8, ATT_MAX_SPLITS>), grid, block, sm, s, a, e);
        } else if (c.dtype == EE_BF16) {
            // (the packed copy of a later pass starts r0/16 row groups further on)
            __bf16* pk = xg_pk ? (__bf16*)xg_pk + (size_t)(r0 / 16) * (d / 32) * 512 : nullptr;
            ResidArgs<__bf16> e{x, (__bf16*)xg, (__bf16*)xgh, xs_lo, ssq_out, c.ssq_stride, g_next, g_head, d, xrow, pk, xg_pk_lo, 0, {}};
            fill_rows(e, c, cc.T);
            EE_DISPATCH(__bf16, gemm_resid_kernel, a, e);
        } else {
            ResidArgs<float> e{x, (float*)xg, (float*)xgh, xs_lo, ssq_out, c.ssq_stride, g_next, g_head, d, xrow, nullptr, 0, 0, {}};
            fill_rows(e, c, cc.T);
            EE_DISPATCH_F32(gemm_resid_kernel, a, e);
        }
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_gemm_swiglu(const GemmCommon& cc, void* act, size_t act_lo, int F, bool act_packed, hipStream_t s) {
    for (int r0 = 0; r0 < cc.T; r0 += PASS_ROWS) {
        const GemmCommon c = pass_of(cc, r0);
        GemmArgs a = make_args(c);
        if (c.dtype == EE_BF16) {
            __bf16* ap = act_packed ? (__bf16*)act + (size_t)(r0 / 16) * (F / 32) * 512 : (__bf16*)act + (size_t)r0 * F;
            EE_DISPATCH(__bf16, gemm_swiglu_kernel, a, ap, act_lo, F, act_packed ? F / 32 : 0);
        } else {
            EE_DISPATCH_F32(gemm_swiglu_kernel, a, (float*)act + (size_t)r0 * F, act_lo, F, 0);
        }
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_gemm_head(const GemmCommon& c, HeadPartial* partials, int32_t* counter, float* logits, int mode,
                            float threshold, HeadResult* results, int tag, hipStream_t s) {
    (void)counter;
    if (c.T <= 0) return hipSuccess;
    if (c.T > 64) return hipErrorInvalidValue;
    GemmArgs a = make_args(c);
    HeadArgs e{partials, logits, c.N};
    if (c.dtype == EE_BF16) {
        EE_DISPATCH(__bf16, gemm_head_kernel, a, e);
    } else {
        EE_DISPATCH_F32(gemm_head_kernel, a, e);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    EE_LAUNCH(head_merge_kernel, dim3(c.T), dim3(512), s, (const HeadPartial*)partials, c.N / 16, c.T, mode, threshold, results, c.desc, tag);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// attention, reference-grade kernel: one workgroup per (row, head); the row at position p attends to
// cache positions 0..p of its sequence (which includes the rows before it in this launch: their K,V
// were written by the QKV kernel).  Online soft-max over chunks of 1024 positions.
// ------------------------------------------------------------------------------------------------
// K of (head, position): pointer to its hd contiguous features.  V of (head, position, feature): one
// element of the transposed V block [head][position / 32][feature][position % 32].
template <typename ST>
__device__ __forceinline__ const ST* k_ptr(const ST* layer_base, const KvGeom& kv, const int32_t* bt, int h, int pos) {
    int blk = bt[pos / kv.BT];
    return layer_base + (size_t)blk * kv.blk_stride + ((size_t)h * kv.BT + (pos % kv.BT)) * kv.hd;
}
template <typename ST>
__device__ __forceinline__ const ST* v_ptr(const ST* layer_base, const KvGeom& kv, const int32_t* bt, int h, int pos, int c) {
    int blk = bt[pos / kv.BT];
    const int pin = pos % kv.BT;
    return layer_base + (size_t)blk * kv.blk_stride + (size_t)kv.H * kv.BT * kv.hd + (size_t)h * kv.hd * kv.BT +
           (size_t)(pin >> 5) * (kv.hd * 32) + c * 32 + (pin & 31);
}

__device__ __forceinline__ float block_reduce(float v, float* red, bool is_max) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            float b = red[threadIdx.x + o];
            red[threadIdx.x] = is_max ? fmaxf(red[threadIdx.x], b) : red[threadIdx.x] + b;
        }
        __syncthreads();
    }
    float r = red[0];
    __syncthreads();
    return r;
}

template <typename ST>
__global__ __launch_bounds__(256) void attn_simple_kernel(const ST* __restrict__ q, ST* __restrict__ out,
                                                          size_t io_lo, const SegDesc* __restrict__ desc,
                                                          const int32_t* __restrict__ btab, KvGeom kv,
                                                          const ST* __restrict__ layer_base, int d) {
    __shared__ float qs[128];
    __shared__ float sc[1024];
    __shared__ float red[256];
    const int r = blockIdx.x, h = blockIdx.y, hd = kv.hd;
    const int pos = desc->pos[r];
    const int32_t* bt = btab + (size_t)desc->rseq[r] * kv.max_blocks_per_seq;
    const float scale = 1.0f / sqrtf((float)hd);
    for (int i = threadIdx.x; i < hd; i += 256) qs[i] = load_split<ST>(q + (size_t)r * d + h * hd + i, io_lo);
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc = 0.f;
    const int n_ctx = pos + 1;
    for (int j0 = 0; j0 < n_ctx; j0 += 1024) {
        int nj = min(1024, n_ctx - j0);
        float cmax = -INFINITY;
        for (int jj = threadIdx.x; jj < nj; jj += 256) {
            const ST* kp = k_ptr(layer_base, kv, bt, h, j0 + jj);
            float s = 0.f;
            for (int c = 0; c < hd; ++c) s = fmaf(qs[c], (float)kp[c], s);
            s *= scale;
            sc[jj] = s;
            cmax = fmaxf(cmax, s);
        }
        cmax = block_reduce(cmax, red, true);
        float m_new = fmaxf(m, cmax);
        float psum = 0.f;
        for (int jj = threadIdx.x; jj < nj; jj += 256) {
            float p = expf(sc[jj] - m_new);
            sc[jj] = p;
            psum += p;
        }
        psum = block_reduce(psum, red, false);
        float corr = expf(m - m_new);  // exp(-inf) = 0 on the first chunk
        l = l * corr + psum;
        if ((int)threadIdx.x < hd) {
            float a2 = 0.f;
            for (int jj = 0; jj < nj; ++jj) a2 = fmaf(sc[jj], (float)*v_ptr(layer_base, kv, bt, h, j0 + jj, (int)threadIdx.x), a2);
            acc = acc * corr + a2;
        }
        m = m_new;
        __syncthreads();
    }
    if ((int)threadIdx.x < hd) store_split<ST>(out + (size_t)r * d + h * hd + threadIdx.x, io_lo, acc / l);
}

// ------------------------------------------------------------------------------------------------
// attention, bf16 model: ragged multi-query decode attention over the paged cache with MFMA.
// One workgroup = (query tile of <= 16 consecutive rows of one sequence, head, KV split); its 4 waves
// take the split's 32-position tiles round-robin.  Per tile a wave computes S^T = K Q^T (K rows come
// straight from the cache as MFMA A operands: a load covers 16 rows x 64 contiguous bytes), applies the causal mask
// (only the last rows of the context differ between the queries of a tile), keeps an online soft-max
// per query, stages the V tile through LDS (coalesced 16-byte loads in, transposed 2-byte reads out)
// and accumulates O^T += V^T P^T, where P^T is already in B-operand layout in the S^T registers.
// q and P are fed as two bf16 terms each (hi + lo), so only K and V carry bf16 rounding.
// Partials of the KV splits are merged by attn_merge_kernel in a fixed order.
// ------------------------------------------------------------------------------------------------

// A launch with a single query tile (one sequence, at most 16 rows: every step at batch 1) gets the tile by value, so
// that the first K load is two dependent loads away from the kernel's start (block table, K) instead of three.
struct AttTile0 {
    int32_t one, row0, nq, pos0, seq;
};

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(const __bf16* __restrict__ q, size_t q_lo, __bf16* __restrict__ out,
                                                             size_t out_lo, int out_pk, const SegDesc* __restrict__ desc,
                                                             const int32_t* __restrict__ btab, KvGeom kv,
                                                             const __bf16* __restrict__ layer_base, int d, int NS,
                                                             float* __restrict__ part, AttTile0 t0) {
    constexpr int KK = HD / 32, CG = HD / 16;
    __shared__ float wO[NW * 16 * (HD + 1)];
    __shared__ float wm[NW * 16], wl[NW * 16];
    // workgroups are handed out in index order: tile-major (the host lists the tiles longest context first), so that all
    // splits of a long context start before any short one
    const int split = blockIdx.x % NS, qh_ = blockIdx.x / NS, qt = qh_ / kv.H, h = qh_ % kv.H;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: block-table reads become scalar loads
    const int lane = threadIdx.x & 63, li = lane & 15, lg = lane >> 4;
    int row0, nq, pos0, seq;
    if (t0.one) {
        row0 = t0.row0, nq = t0.nq, pos0 = t0.pos0, seq = t0.seq;
    } else {
        row0 = desc->qt_row0[qt], nq = desc->qt_nq[qt], pos0 = desc->qt_pos0[qt], seq = desc->qt_seq[qt];
    }
    const int ctx = pos0 + nq;
    const int32_t* bt = btab + (size_t)seq * kv.max_blocks_per_seq;
    const int n_tiles = (ctx + 31) >> 5;
    const int tps = (n_tiles + NS - 1) / NS;
    const int t_lo = split * tps, t_hi = min(n_tiles, t_lo + tps);
    const bool qvalid = li < nq;
    // MFMA row i of score half s stands for position (i/4)*8 + s*4 + i%4 of the tile, so that after the two
    // halves a lane (query li, group lg) holds the probabilities of the 8 consecutive positions lg*8..lg*8+7:
    // exactly the 16 bytes of a transposed-V row that the P.V product needs as its other operand.
    const int krow0 = (li >> 2) * 8 + (li & 3);

    // K and V of one 32-position tile, loaded straight into MFMA operand order
    struct TileRegs {
        u32x4 k[2 * KK];
        u32x4 v[CG];
    };
    auto issue = [&](int t, TileRegs& r) {
        const int tb = t << 5;
        const int blk = bt[tb / kv.BT];
        const int tin = tb % kv.BT;
        const __bf16* kbase = layer_base + (size_t)blk * kv.blk_stride + ((size_t)h * kv.BT + tin) * HD;
        const __bf16* vbase = layer_base + (size_t)blk * kv.blk_stride + (size_t)kv.H * kv.BT * HD + (size_t)h * HD * kv.BT +
                              (size_t)(tin >> 5) * (HD * 32);  // the tile's V: HD x 32, contiguous
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const __bf16* kp = kbase + (size_t)(krow0 + sub * 4) * HD + lg * 8;  // one load: 16 rows x 64 contiguous bytes
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) r.k[sub * KK + kk] = *(const u32x4*)(kp + kk * 32);
        }
#pragma unroll
        for (int c = 0; c < CG; ++c) r.v[c] = *(const u32x4*)(vbase + (c * 16 + li) * 32 + lg * 8);
    };

    bf16x8 qh[KK], ql[KK];
    {
        const __bf16* qp = q + (size_t)(row0 + (qvalid ? li : 0)) * d + h * HD + lg * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            qh[kk] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + kk * 32));
            ql[kk] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + q_lo + kk * 32));
        }
    }
    const float scale = 1.0f / sqrtf((float)HD);
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o[CG];
#pragma unroll
    for (int c = 0; c < CG; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    TileRegs cur, nxt;
    int t = t_lo + wave;
    if (t < t_hi) issue(t, cur);
    while (t < t_hi) {
        const int tn = t + NW;
        if (tn < t_hi) issue(tn, nxt);  // the next tile streams in while this one is worked on
        const int tb = t << 5;
        // scores, transposed: rows = positions, columns = queries
        f32x4 sacc[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            sacc[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                bf16x8 kf = __builtin_bit_cast(bf16x8, cur.k[sub * KK + kk]);
                sacc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, ql[kk], sacc[sub], 0, 0, 0);
                sacc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qh[kk], sacc[sub], 0, 0, 0);
            }
        }
        // causal mask + online soft-max per query (column li); element e of this lane = position tb + lg*8 + e
        float pv[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int pa = tb + lg * 8 + e;
            float val = (qvalid && pa <= pos0 + li) ? sacc[e >> 2][e & 3] * scale : -INFINITY;
            pv[e] = val;
            tmax = fmaxf(tmax, val);
        }
        tmax = rows4_max(tmax);
        const float m_new = fmaxf(m_run, tmax);
        float corr = 1.f, psum = 0.f;
        if (m_new == -INFINITY) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[e] = 0.f;
        } else {
            // (hardware exponential: relative error about 1e-6 over the range that matters, far inside the bf16 contract;
            // skipping the mask on interior tiles or the rescale when no maximum moved made this kernel slower)
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
            __bf16 hi = (__bf16)pv[e];
            ph[e] = hi;
            pl[e] = (__bf16)(pv[e] - (float)hi);
        }
        // positions beyond the context hold unknown bits (their probabilities are zero): zero them
        // (splitting the score chains over four accumulators and the P.V product into one pass per term, as the
        // prompt-phase kernel does, measured no faster at batch 1 and 2 % slower at batch 16: this kernel waits for
        // memory, and the extra registers cost it waves)
        const bool ragged = tb + 32 > ctx;
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            bf16x8 vf = __builtin_bit_cast(bf16x8, cur.v[c]);
            if (ragged) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (tb + lg * 8 + e >= ctx) vf[e] = (__bf16)0.f;
            }
            o[c] = o[c] * corr;
            o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl, o[c], 0, 0, 0);
            o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, ph, o[c], 0, 0, 0);
        }
        cur = nxt;
        t = tn;
    }

    // combine the waves (fixed order)
#pragma unroll
    for (int c = 0; c < CG; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) wO[(wave * 16 + li) * (HD + 1) + c * 16 + lg * 4 + r] = o[c][r];
    if (lg == 0) {
        wm[wave * 16 + li] = m_run;
        wl[wave * 16 + li] = l_run;
    }
    __syncthreads();
    float* pbase = part + ((size_t)(qt * kv.H + h) * NS + split) * att_part_stride(HD);
    for (int idx = threadIdx.x; idx < 16 * HD; idx += NW * 64) {
        int qq = idx / HD, cc = idx % HD;
        if (qq >= nq) continue;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, wm[w * 16 + qq]);
        float O = 0.f, L = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                float f = __expf(wm[w * 16 + qq] - M);
                O += f * wO[(w * 16 + qq) * (HD + 1) + cc];
                L += f * wl[w * 16 + qq];
            }
        }
        if (NS == 1) {
            store_split_at<__bf16>(out, out_lo, row0 + qq, h * HD + cc, d, out_pk, O / L);
        } else {
            pbase[32 + qq * HD + cc] = O;
            if (cc == 0) {
                pbase[qq] = M;
                pbase[16 + qq] = L;
            }
        }
    }
}

template <int HD, int MAXS>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part, int NS, __bf16* __restrict__ out,
                                                         size_t out_lo, int out_pk, const SegDesc* __restrict__ desc, int H, int d) {
    const int qt = blockIdx.x / H, h = blockIdx.x % H;
    const int row0 = desc->qt_row0[qt], nq = desc->qt_nq[qt];
    const float* pb = part + (size_t)(qt * H + h) * NS * att_part_stride(HD);
    for (int idx = threadIdx.x; idx < nq * HD; idx += 256) {
        int qq = idx / HD, cc = idx % HD;
        // (all loads of all splits go out together, a surplus split repeating the last one: one memory round trip
        // instead of one per split and pass)
        float ms[MAXS], ls[MAXS], os[MAXS];
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            const float* ps = pb + (size_t)(s < NS ? s : NS - 1) * att_part_stride(HD);
            ms[s] = ps[qq];
            ls[s] = ps[16 + qq];
            os[s] = ps[32 + qq * HD + cc];
        }
        float M = -INFINITY;
#pragma unroll
        for (int s = 0; s < MAXS; ++s)
            if (s < NS) M = fmaxf(M, ms[s]);
        float O = 0.f, L = 0.f;
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            if (s >= NS || ms[s] == -INFINITY) continue;
            float f = __expf(ms[s] - M);
            O += f * os[s];
            L += f * ls[s];
        }
        store_split_at<__bf16>(out, out_lo, row0 + qq, h * HD + cc, d, out_pk, O / L);
    }
}

size_t attention_part_floats(int max_rows, int H, int hd) {
    size_t entries = (size_t)max_rows * H;
    if (entries < 1024) entries = 1024;
    return entries * att_part_stride(hd);
}

template <int HD>
static hipError_t launch_attention_mfma(const void* q, void* out, size_t io_lo, const SegDesc* desc, const SegDesc* desc_host, int n_qt,
                                        const int32_t* btab, const KvGeom& kv, int layer, int d, float* part, int max_ctx, int* defer_ns,
                                        bool out_packed, hipStream_t s) {
    const int out_pk = out_packed ? d / 32 : 0;
    AttTile0 t0{0, 0, 0, 0, 0};
    if (n_qt == 1 && desc_host != nullptr) t0 = AttTile0{1, desc_host->qt_row0[0], desc_host->qt_nq[0], desc_host->qt_pos0[0], desc_host->qt_seq[0]};
    const int wgs = n_qt * kv.H;
    const int tiles = (max_ctx + 31) / 32;
    const __bf16* lb = (const __bf16*)kv.pool + (size_t)layer * kv.layer_stride;
    // KV splits: enough workgroups to cover the chip, at least ~4 tiles (one per wave) per split.  A
    // wave works through its tiles one after another, so short splits keep the dependent chain short.
    // Up to 512 (query tile, head) pairs (steps of a few rows, small and medium batches): workgroups of 8 waves
    // and about 6 tiles per split: fewer splits to merge at the same number of waves, none at all from 129
    // pairs on (30B shape, 4 sequences x 52 heads: 51 us with 4 splits of 4 waves + merge -> 45.5 us; 7B shape,
    // 16 sequences x 32 heads: 2 splits of 4 waves + a merge launch -> one workgroup of 8 waves per pair, the same
    // waves per CU and no merge, 5.48 -> 5.40 ms per step).
    const bool few = wgs <= 512;
    int NS = (few ? 256 : 1024) / wgs;
    int by_len = few ? (tiles + 5) / 6 : (tiles + 3) / 4;
    if (NS > by_len) NS = by_len;
    if (NS > ATT_MAX_SPLITS) NS = ATT_MAX_SPLITS;
    if (NS < 1) NS = 1;
    if (few)
        EE_LAUNCH((attn_mfma_kernel<HD, 8>), dim3(wgs * NS), dim3(8 * 64), s, (const __bf16*)q, io_lo, (__bf16*)out, io_lo, out_pk, desc,
                  btab, kv, lb, d, NS, part, t0);
    else
        EE_LAUNCH((attn_mfma_kernel<HD, 4>), dim3(wgs * NS), dim3(4 * 64), s, (const __bf16*)q, io_lo, (__bf16*)out, io_lo, out_pk, desc,
                  btab, kv, lb, d, NS, part, t0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || NS == 1) return e;
    if (defer_ns != nullptr) {  // the consumer merges the splits itself
        *defer_ns = NS;
        return e;
    }
    if (NS <= 2)
        EE_LAUNCH((attn_merge_kernel<HD, 2>), dim3(wgs), dim3(256), s, (const float*)part, NS, (__bf16*)out, io_lo, out_pk, desc, kv.H, d);
    else if (NS <= 4)
        EE_LAUNCH((attn_merge_kernel<HD, 4>), dim3(wgs), dim3(256), s, (const float*)part, NS, (__bf16*)out, io_lo, out_pk, desc, kv.H, d);
    else if (NS <= 8)
        EE_LAUNCH((attn_merge_kernel<HD, 8>), dim3(wgs), dim3(256), s, (const float*)part, NS, (__bf16*)out, io_lo, out_pk, desc, kv.H, d);
    else
        EE_LAUNCH((attn_merge_kernel<HD, ATT_MAX_SPLITS>), dim3(wgs), dim3(256), s, (const float*)part, NS, (__bf16*)out, io_lo, out_pk, desc, kv.H, d);
    return hipGetLastError();
}

hipError_t launch_attention(int dtype, const void* q, void* out, size_t io_lo, const SegDesc* desc, const SegDesc* desc_host, int T, int n_qt,
                            const int32_t* btab,
                            const KvGeom& kv, int layer, int d, float* part, int32_t* counters, int max_ctx, int* defer_ns,
                            bool out_packed, hipStream_t s) {
    (void)counters;
    if (defer_ns) *defer_ns = 0;
    if (T <= 0) return hipSuccess;
    if (dtype == EE_BF16) {
        switch (kv.hd) {
            case 32: return launch_attention_mfma<32>(q, out, io_lo, desc, desc_host, n_qt, btab, kv, layer, d, part, max_ctx, defer_ns, out_packed, s);
            case 64: return launch_attention_mfma<64>(q, out, io_lo, desc, desc_host, n_qt, btab, kv, layer, d, part, max_ctx, defer_ns, out_packed, s);
            case 128: return launch_attention_mfma<128>(q, out, io_lo, desc, desc_host, n_qt, btab, kv, layer, d, part, max_ctx, defer_ns, out_packed, s);
            default: return hipErrorInvalidValue;
        }
    }
    dim3 grid(T, kv.H), block(256);
    EE_LAUNCH(attn_simple_kernel<float>, grid, block, s, (const float*)q, (float*)out, io_lo, desc, btab, kv,
                       (const float*)kv.pool + (size_t)layer * kv.layer_stride, d);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// cache export (tests): K,V of positions [pos0, pos0+n) of one layer as fp32 [n][d]
// ------------------------------------------------------------------------------------------------
template <typename ST>
__global__ void kv_gather_kernel(KvGeom kv, const ST* __restrict__ layer_base, const int32_t* __restrict__ bt, int pos0, int n,
                                 float* __restrict__ k_out, float* __restrict__ v_out) {
    int d = kv.H * kv.hd;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n * d) return;
    int t = idx / d, c = idx % d;
    int h = c / kv.hd, i = c % kv.hd;
    k_out[idx] = (float)k_ptr(layer_base, kv, bt, h, pos0 + t)[i];
    v_out[idx] = (float)*v_ptr(layer_base, kv, bt, h, pos0 + t, i);
}

hipError_t launch_kv_gather(int dtype, const KvGeom& kv, int layer, const int32_t* btab_seq, int pos0, int n,
                            float* k_out, float* v_out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    long total = (long)n * kv.H * kv.hd;
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == EE_BF16)
        EE_LAUNCH(kv_gather_kernel<__bf16>, grid, block, s, kv, (const __bf16*)kv.pool + (size_t)layer * kv.layer_stride,
                           btab_seq, pos0, n, k_out, v_out);
    else
        EE_LAUNCH(kv_gather_kernel<float>, grid, block, s, kv, (const float*)kv.pool + (size_t)layer * kv.layer_stride,
                           btab_seq, pos0, n, k_out, v_out);
    return hipGetLastError();
}

}  // namespace ee
