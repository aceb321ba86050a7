// HIP kernels (gfx950, wave64) for one DEF / DEF-A iteration with RBGS.
//
// Method: arXiv 2004.05298, Algorithm 1 with the momentum variant of Sec. 3.2.
// For every worker k and flat index i
//     m_k[i] <- mu*m_k[i] + g_k[i]                 (Sec. 3.2 "Momentum Variant")
//     p       = eta*m_k[i] + e_k[i]                (Algorithm 1, error feedback)
//     e_k[i] <- i in block ? +0 : p                (Algorithm 1, e <- p - C(p))
//     msg_k[(i - s) mod d] = p  for i in block     (C(p_k), compact)
// then  cbar[j] = (1/W) sum_k msg_k[j]             (Algorithm 1, all-reduce line)
//       x[(s+j) mod d] -= cbar[j]                  (Algorithm 1, update line)
// and, when asked for, the points at which the next gradients are to be evaluated,
//       w_k[i] = x_{t+1}[i] - lambda*e_{k,t+1}[i]  (Algorithm 1, "detach" line).
// The block {(s+j) mod d : j < B} is the RBGS compressor of Sec. 1.
//
// Nothing here is a contraction: the step is a streaming pass of five 4-byte
// accesses per (worker, index) and is bound by HBM bandwidth.  What the kernels
// care about is therefore how requests reach memory: dwordx4 per lane (1 KiB of
// consecutive bytes per wave instruction), non-temporal loads and stores for data
// touched once per step, few accesses per wave so that loads and stores of many
// waves interleave finely, work items numbered so that the chip sweeps each
// worker row front to back, and a grid far larger than the 256 compute units.
//
// Arithmetic: every multiply and every add rounds once in binary32.  Fused
// multiply-add would change results by an ulp, so contraction is switched off
// for the whole file (and again on the compiler command line).
#include "def_internal.h"

#include <cstdio>
#include <mutex>

#pragma clang fp contract(off)

typedef float v4f __attribute__((ext_vector_type(4)));
// The same four floats at any 4-byte aligned address.  The hardware accepts dwordx4
// accesses at dword alignment, so caller-owned buffers (gradients, x, w) need not be
// 16-byte aligned; the library's own rows always are.
typedef v4f v4f_u __attribute__((aligned(4)));

namespace {

template <bool NT>
__device__ __forceinline__ v4f load4u(const float *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const v4f_u *>(p));
    else return *reinterpret_cast<const v4f_u *>(p);
}

template <bool NT>
__device__ __forceinline__ void store4u(float *p, v4f v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<v4f_u *>(p));
    else *reinterpret_cast<v4f_u *>(p) = v;
}

template <bool NT>
__device__ __forceinline__ v4f load4(const float *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    else return *reinterpret_cast<const v4f *>(p);
}

template <bool NT>
__device__ __forceinline__ void store4(float *p, v4f v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<v4f *>(p));
    else *reinterpret_cast<v4f *>(p) = v;
}

// The compensated value p_{k,t}[i]; updates m in place when momentum is on.
template <bool HAS_MU, bool HAS_WD>
__device__ __forceinline__ float compensated(float g, float &m, float e, float x,
                                             float lr, float mu, float wd)
{
    float gp = g;
    if constexpr (HAS_WD) {
        const float decay = wd * x;      // weight decay folded into the gradient at x_t
        gp = g + decay;
    }
    float mk = gp;
    if constexpr (HAS_MU) {
        const float carried = mu * m;
        mk = carried + gp;               // m_{k,t+1} = mu*m_{k,t} + g_{k,t}
        m = mk;
    }
    const float step = lr * mk;
    return step + e;                     // p_{k,t} = eta*m_{k,t+1} + e_{k,t}
}

// Block start of the step: a kernel argument when the host drew it, else the value
// the draw kernel left in device memory (one uniform load per wave).
__device__ __forceinline__ uint64_t block_start_of(const DefStepArgs &a)
{
    return a.ctl ? a.ctl->s : a.s;
}

// Direction of the step's sweep over the work items: every other step runs backwards.
__device__ __forceinline__ bool sweep_backwards(const DefStepArgs &a)
{
    return (a.ctl ? a.ctl->backwards : a.backwards) != 0;
}

// Workgroup ids are dealt round-robin to the 8 XCDs.  Work items (one worker's
// piece of one column tile) are numbered 0..tiles*W-1 and workgroup b takes item b;
// MAP chooses what item b is:
//   MAP_LINEAR_T  tile index fastest: each worker row is streamed front to back,
//               one row after the other;
//   MAP_BLOCKED   the columns are cut into super-tiles of `super` tiles; within a
//               super-tile the workers follow one another, each streaming its
//               piece of the super-tile front to back.  When every worker reads x
//               (weight decay, detached points) all W of them pass over the same
//               piece of x within a short time, so it is fetched from HBM once and
//               then served by the L2 of each XCD.
// (Worker index fastest and XCD-contiguous item ranges were measured too and were
// 3 to 15 % slower: hopping between W rows per tile costs more than it saves.)
enum { MAP_LINEAR_T = 2, MAP_BLOCKED = 4 };

template <int MAP>
__device__ __forceinline__ bool decode_item(uint64_t total, uint64_t tiles, uint32_t W, uint32_t super,
                                            uint32_t &k, uint64_t &tile, bool backwards = false)
{
    if (blockIdx.x >= total) return false;
    // backwards: the same items in the opposite order, so that a pass starts where the
    // previous one ended and finds the end of that pass still in the caches
    const uint64_t item = backwards ? total - 1 - blockIdx.x : (uint64_t)blockIdx.x;
    if constexpr (MAP == MAP_LINEAR_T) {
        tile = item % tiles;
        k = (uint32_t)(item / tiles);
    } else {
        const uint64_t per_super = (uint64_t)W * super;       // items of a full super-tile
        const uint64_t sup = item / per_super;
        const uint64_t rem = item - sup * per_super;
        const uint64_t first = sup * super;                   // first tile of this super-tile
        const uint64_t width = tiles - first < super ? tiles - first : super;   // last one may be short
        // every worker's piece takes a multiple of 8 items (the last few of a short piece do
        // nothing), so that a tile falls to the same XCD for all W workers and the x it reads
        // is found in that XCD's L2; `super` is a multiple of 8 itself
        const uint64_t slots = (width + 7) & ~(uint64_t)7;
        k = (uint32_t)(rem / slots);
        const uint64_t within = rem - (uint64_t)k * slots;
        if (within >= width) return false;
        tile = first + within;
    }
    return true;
}

// ---------------------------------------------------------------------------
// Streaming pass.  One workgroup = one worker's tile of THREADS*U float4 groups;
// thread t owns groups t, t+THREADS, ... so that each wave instruction touches
// 1 KiB of consecutive memory.
//
// TABLES = false: gradients are one buffer [W][ldg] and, if x is read, it is one
// flat vector.  TABLES = true: gradients and/or parameters are given per tensor.
// The host supplies, for every tile, the tensor that holds the tile's first index;
// a tile that lies inside one tensor (nearly all do) only rebases its g and x
// pointers and then runs the same code as the flat case, with dword-aligned
// dwordx4 accesses; a tile that crosses a tensor boundary resolves g and x element
// by element through the offset table.
// ---------------------------------------------------------------------------
template <bool HAS_MU, bool HAS_WD, bool HAS_DT, bool TABLES, int THREADS, int U, bool NT_LD, bool NT_ST,
          int MAP>
__global__ __launch_bounds__(THREADS) void def_stream_vec4_kernel(DefStepArgs a, uint64_t tiles,
                                                                  uint64_t total, uint32_t super)
{
    constexpr bool HAS_X = HAS_WD || HAS_DT;             // x is read for weight decay and for w
    uint32_t k;
    uint64_t tile;
    if (!decode_item<MAP>(total, tiles, a.W, super, k, tile, sweep_backwards(a))) return;

    float *__restrict__ e = a.e + (uint64_t)k * a.ld;
    float *__restrict__ m = HAS_MU ? a.m + (uint64_t)k * a.ld : nullptr;
    float *__restrict__ msg = a.msg + (uint64_t)k * a.ldmsg;
    float *__restrict__ w = HAS_DT ? a.w + (uint64_t)k * a.ldw : nullptr;
    const uint64_t s = block_start_of(a);

    constexpr uint64_t STRIDE = THREADS * 4;             // elements between a thread's groups
    constexpr uint64_t TILE = (uint64_t)THREADS * U * 4; // elements per tile
    const uint64_t i_first = tile * TILE + threadIdx.x * 4;
    const uint64_t tile_end = (tile + 1) * TILE;
    const bool interior = tile_end <= a.d;

    // g[i - g_sub] and x[i - x_sub] address flat index i on the fast path
    const float *__restrict__ g = a.g_flat + (uint64_t)k * a.ldg;
    const float *__restrict__ x = a.x_flat;
    uint64_t g_sub = 0, x_sub = 0;
    uint32_t l0 = 0;                                     // tensor of the tile's first index
    bool one_tensor = true;                              // the tile lies inside one tensor
    if constexpr (TABLES) {
        l0 = a.tile_tensor[tile];
        const uint64_t lo = a.off[l0], hi = a.off[l0 + 1];
        one_tensor = (interior ? tile_end : a.d) <= hi;
        if (a.g_ptrs) {
            g = a.g_ptrs[(uint64_t)k * a.L + l0];
            g_sub = lo;
        }
        if (HAS_X && a.x_ptrs) {
            x = a.x_ptrs[l0];
            x_sub = lo;
        }
    }
    // element access for the rare tile that crosses a tensor boundary
    auto g_at = [&](uint64_t idx) -> float {
        if constexpr (TABLES) {
            if (a.g_ptrs) {
                uint32_t l = l0;
                while (idx >= a.off[l + 1]) ++l;
                return a.g_ptrs[(uint64_t)k * a.L + l][idx - a.off[l]];
            }
        }
        return g[idx - g_sub];
    };
    auto x_at = [&](uint64_t idx) -> float {
        if constexpr (TABLES) {
            if (a.x_ptrs) {
                uint32_t l = l0;
                while (idx >= a.off[l + 1]) ++l;
                return a.x_ptrs[l][idx - a.off[l]];
            }
        }
        return x[idx - x_sub];
    };

    v4f gv[U], mv[U], ev[U], xv[U];
    if (interior && one_tensor) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = i_first + u * STRIDE;
            gv[u] = load4u<NT_LD>(g + (i - g_sub));
            if constexpr (HAS_MU) mv[u] = load4<NT_LD>(m + i);
            ev[u] = load4<NT_LD>(e + i);
            if constexpr (HAS_X) xv[u] = load4u<false>(x + (i - x_sub));
        }
    } else {
        // last tile of the row (a group may be cut by d or lie beyond it) or a tile
        // that crosses a tensor boundary.  The state rows are padded to a multiple of
        // the tile, so e and m can always be read as whole groups; g and x are read
        // element by element where a group is cut.
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = i_first + u * STRIDE;
            gv[u] = (v4f)(0.0f); mv[u] = (v4f)(0.0f); ev[u] = (v4f)(0.0f); xv[u] = (v4f)(0.0f);
            if (i + 4 <= a.d && one_tensor) {
                gv[u] = load4u<NT_LD>(g + (i - g_sub));
                if constexpr (HAS_X) xv[u] = load4u<false>(x + (i - x_sub));
            } else if (i < a.d) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (i + c < a.d) {
                        gv[u][c] = g_at(i + c);
                        if constexpr (HAS_X) xv[u][c] = x_at(i + c);
                    }
            }
            if (i < a.d) {
                if constexpr (HAS_MU) mv[u] = load4<NT_LD>(m + i);
                ev[u] = load4<NT_LD>(e + i);
            }
        }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t i = i_first + u * STRIDE;
        if (!interior && i >= a.d) continue;
        v4f p;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float mc = HAS_MU ? mv[u][c] : 0.0f;
            p[c] = compensated<HAS_MU, HAS_WD>(gv[u][c], mc, ev[u][c], HAS_WD ? xv[u][c] : 0.0f,
                                               a.lr, a.mu, a.wd);
            if constexpr (HAS_MU) mv[u][c] = mc;
        }
        // position of element i inside the circular block: j = (i - s) mod d
        uint64_t j0 = i >= s ? i - s : i + a.d - s;
        v4f en = p;                                           // off-block: e <- p
        if (!(j0 >= a.B && j0 + 3 < a.d)) {                   // some element may be kept
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint64_t j = j0 + c;
                if (j >= a.d) j -= a.d;
                if (i + c < a.d && j < a.B) {
                    msg[j] = p[c];                            // C(p_k), compact
                    en[c] = 0.0f;                             // p - C(p) = +0 inside the block
                }
            }
        }
        if constexpr (HAS_MU) store4<NT_ST>(m + i, mv[u]);
        store4<NT_ST>(e + i, en);
        if constexpr (HAS_DT) {
            // w = x - lambda*e_new.  Off the block x does not change in this step.  On
            // the block this writes x_t - lambda*0; the averaging kernel, which runs
            // after this one, replaces those entries by x_{t+1}.
            v4f wv;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float scaled = a.lam * en[c];
                wv[c] = xv[u][c] - scaled;
            }
            if (i + 4 <= a.d) {
                store4u<NT_ST>(w + i, wv);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (i + c < a.d) w[i + c] = wv[c];
            }
        }
    }
}

// Address of parameter i: flat vector, or tensor table + offset table.
__device__ __forceinline__ float *param_addr(const DefStepArgs &a, uint64_t i)
{
    if (a.x_flat) return a.x_flat + i;
    uint32_t lo = 0, hi = a.L;                                // off[lo] <= i < off[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a.off[mid] <= i) lo = mid; else hi = mid;
    }
    return a.x_ptrs[lo] + (i - a.off[lo]);
}

// ---------------------------------------------------------------------------
// Cross-worker average of the compact blocks and parameter update.  This is
// the on-one-GPU stand-in for the ring all-reduce of Algorithm 1.
// One workgroup = 256 block columns.  The four waves stage worker rows through
// LDS, one row per wave at a time, each lane loading a float4 (1 KiB coalesced
// per row); after the barrier thread c adds column c over the workers in order
// k = 0, 1, ..., W-1 starting from +0, so the sum is the plain left-to-right sum
// whatever the launch shape.
// ---------------------------------------------------------------------------
constexpr int AVG_ROWS = 16;

// Sum over the workers of one block column, k = 0..W-1 in order from +0 (valid for
// threads whose column j_tile + threadIdx.x is below B; others get the padding's zeros).
__device__ __forceinline__ float block_column_sum(const DefStepArgs &a, float (*stage)[DEF_AVG_TILE])
{
    const uint64_t j_tile = (uint64_t)blockIdx.x * DEF_AVG_TILE;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    float acc = 0.0f;
    for (uint32_t k0 = 0; k0 < a.W; k0 += AVG_ROWS) {
        const uint32_t rows = min((uint32_t)AVG_ROWS, a.W - k0);
        for (uint32_t r = wave; r < rows; r += DEF_THREADS / 64) {
            const float *row = a.msg + (uint64_t)(k0 + r) * a.ldmsg + j_tile;   // rows padded to the tile
            *reinterpret_cast<v4f *>(&stage[r][lane * 4]) = load4<false>(row + lane * 4);
        }
        __syncthreads();
        for (uint32_t r = 0; r < rows; ++r) acc = acc + stage[r][threadIdx.x];
        __syncthreads();
    }
    return acc;
}

// x_{t+1} = x_t - cbar at block position j (Algorithm 1, update line), and the detached
// points there: inside the block e_{k,t+1} = +0 for every worker, so w_k = x_{t+1} - lambda*0.
__device__ __forceinline__ void apply_block_entry(const DefStepArgs &a, uint64_t j, float cbar)
{
    a.avg[j] = cbar;
    uint64_t i = block_start_of(a) + j;
    if (i >= a.d) i -= a.d;
    float *px = param_addr(a, i);
    const float x_new = *px - cbar;
    *px = x_new;
    if (a.w) {
        const float scaled = a.lam * 0.0f;
        const float wv = x_new - scaled;
        for (uint32_t k = 0; k < a.W; ++k) a.w[(uint64_t)k * a.ldw + i] = wv;
    }
}

__global__ __launch_bounds__(DEF_THREADS) void def_average_update_kernel(DefStepArgs a)
{
    __shared__ float stage[AVG_ROWS][DEF_AVG_TILE];
    const float acc = block_column_sum(a, stage);
    const uint64_t j = (uint64_t)blockIdx.x * DEF_AVG_TILE + threadIdx.x;
    if (j < a.B) apply_block_entry(a, j, acc / (float)a.W);      // (1/W) sum_k C(p_k)
}

// The two halves of the kernel above, for workers spread over several GPUs: the sum
// over this GPU's workers (what an all-reduce would add up across GPUs) ...
__global__ __launch_bounds__(DEF_THREADS) void def_block_sum_kernel(DefStepArgs a)
{
    __shared__ float stage[AVG_ROWS][DEF_AVG_TILE];
    const float acc = block_column_sum(a, stage);
    const uint64_t j = (uint64_t)blockIdx.x * DEF_AVG_TILE + threadIdx.x;
    if (j < a.B) a.avg[j] = acc;
}

// ... and the update with a block that the caller has reduced: cbar = block[j] / divisor.
// block may be the context's own avg buffer (each thread reads its entry before writing it).
__global__ __launch_bounds__(DEF_THREADS) void def_apply_block_kernel(DefStepArgs a, const float *block,
                                                                      float divisor)
{
    const uint64_t j = (uint64_t)blockIdx.x * DEF_THREADS + threadIdx.x;
    if (j < a.B) apply_block_entry(a, j, block[j] / divisor);
}

// x[i..i+3] for a group that may be cut by d (missing entries are 0): flat vector, or
// per-tensor pointers found through the tile table; dword-aligned dwordx4 when the
// group lies inside one tensor.
__device__ __forceinline__ v4f load_x_group(const DefStepArgs &a, uint64_t i)
{
    if (i + 4 <= a.d) {
        if (a.x_flat) return load4u<false>(a.x_flat + i);
        uint32_t l = a.tile_tensor[i / DEF_VEC_TILE];         // tensor of the tile's first index
        while (i >= a.off[l + 1]) ++l;
        if (i + 4 <= a.off[l + 1]) return load4u<false>(a.x_ptrs[l] + (i - a.off[l]));
    }
    v4f v = (v4f)(0.0f);
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (i + c < a.d) v[c] = *param_addr(a, i + c);
    return v;
}

// Store a group that may be cut by d to a caller-owned flat vector (any 4-byte alignment).
__device__ __forceinline__ void store_group(float *dst, uint64_t i, uint64_t d, v4f v)
{
    if (i + 4 <= d) {
        store4u<true>(dst + i, v);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (i + c < d) dst[i + c] = v[c];
    }
}

// ---------------------------------------------------------------------------
// DEF output y = x - (1/W) sum_k e_k (Algorithm 1 "Output").  One thread owns
// four consecutive columns and walks the workers in order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(DEF_OUT_THREADS) void def_output_kernel(DefStepArgs a, float *y)
{
    const uint64_t i = ((uint64_t)blockIdx.x * DEF_OUT_THREADS + threadIdx.x) * 4;
    if (i >= a.d) return;
    v4f acc = (v4f)(0.0f);
#pragma unroll 4
    for (uint32_t k = 0; k < a.W; ++k) acc = acc + load4<true>(a.e + (uint64_t)k * a.ld + i);
    const v4f mean = acc / (float)a.W;
    store_group(y, i, a.d, load_x_group(a, i) - mean);
}

// ---------------------------------------------------------------------------
// Detached evaluation points for the current state, w_k = x - lambda*e_k
// (Algorithm 1, "detach" line).  Work items as in the streaming pass: one wave per
// (worker, 256 indices), blocked order so that x is served by L2 to all workers.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(DEF_VEC_THREADS) void def_detach_kernel(DefStepArgs a, uint64_t tiles,
                                                                     uint64_t total)
{
    uint32_t k;
    uint64_t tile;
    if (!decode_item<MAP_BLOCKED>(total, tiles, a.W, DEF_SUPER_TILES, k, tile)) return;
    const uint64_t i = tile * DEF_VEC_TILE + threadIdx.x * 4;
    if (i >= a.d) return;
    const v4f xv = load_x_group(a, i);
    const v4f ev = load4<true>(a.e + (uint64_t)k * a.ld + i);        // padded rows: always in bounds
    v4f wv;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float scaled = a.lam * ev[c];
        wv[c] = xv[c] - scaled;
    }
    store_group(a.w + (uint64_t)k * a.ldw, i, a.d, wv);
}

// ---------------------------------------------------------------------------
// Error-memory statistics of Sec. 3.2 (items (1)-(3)) and Appendix A, in float64:
//   S1 = ||e_t||^2 with e_t = (1/W) sum_k e_k,   S2 = sum_k ||e_k||^2.
// Stage 1: one thread per 4 columns walks the workers in order (so e_t[i] is the
// same number whatever the launch shape), then the workgroup adds its threads'
// sums through wave shuffles and LDS and writes one pair per workgroup.
// Stage 2: one workgroup adds the pairs in a fixed order and derives
//   mean_sq = S2/W, lambda*(t) = S1/mean_sq,
//   (1/W) sum_k ||e_t - lambda e_k||^2 = lambda^2 mean_sq - 2 lambda S1 + S1.
// No atomics: the result is reproducible from run to run.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double block_sum(double v, double *lds)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    __syncthreads();                       // lds may still be read from a previous call
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (uint32_t q = 0; q < DEF_THREADS / 64; ++q) total += lds[q];
    return total;                          // valid in thread 0
}

__global__ __launch_bounds__(DEF_THREADS) void def_diag_partial_kernel(DefStepArgs a, double *partials)
{
    __shared__ double lds[DEF_THREADS / 64];
    const uint64_t i = ((uint64_t)blockIdx.x * DEF_THREADS + threadIdx.x) * 4;
    double s1 = 0.0, s2 = 0.0;
    if (i < a.d) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        if (i + 4 <= a.d) {
#pragma unroll 16
            for (uint32_t k = 0; k < a.W; ++k) {
                const v4f ev = load4<true>(a.e + (uint64_t)k * a.ld + i);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const double v = (double)ev[c];
                    acc[c] += v;
                    s2 += v * v;
                }
            }
        } else {
            // the last group of a row, cut by d: element by element, so that rows without
            // zero padding (a caller's own buffers) are read only up to column d-1
            for (uint32_t k = 0; k < a.W; ++k)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (i + c < a.d) {
                        const double v = (double)a.e[(uint64_t)k * a.ld + i + c];
                        acc[c] += v;
                        s2 += v * v;
                    }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double mean = acc[c] / (double)a.W;
            s1 += mean * mean;
        }
    }
    const double b1 = block_sum(s1, lds);
    const double b2 = block_sum(s2, lds);
    if (threadIdx.x == 0) {
        partials[2 * (uint64_t)blockIdx.x] = b1;
        partials[2 * (uint64_t)blockIdx.x + 1] = b2;
    }
}

__global__ __launch_bounds__(DEF_THREADS) void def_diag_final_kernel(const double *partials, uint64_t n,
                                                                     uint32_t W, float lambda, double *out)
{
    __shared__ double lds[DEF_THREADS / 64];
    double s1 = 0.0, s2 = 0.0;
#pragma unroll 8
    for (uint64_t b = threadIdx.x; b < n; b += DEF_THREADS) {   // several loads in flight, sums in order
        s1 += partials[2 * b];
        s2 += partials[2 * b + 1];
    }
    const double S1 = block_sum(s1, lds);
    const double S2 = block_sum(s2, lds);
    if (threadIdx.x == 0) {
        const double mean_sq = S2 / (double)W;
        const double lam = (double)lambda;
        out[0] = S1;
        out[1] = mean_sq;
        out[2] = mean_sq > 0.0 ? S1 / mean_sq : 0.0;
        out[3] = lam * lam * mean_sq - 2.0 * lam * S1 + S1;
    }
}

// ---------------------------------------------------------------------------
// Per-worker statistics (Sec. 3.2, item (1); Appendix A, first display), float64:
//   ||e_k||^2 and <e_t, e_k> for every worker k, whose ratio lambda*(k,t) is the
//   lambda that brings worker k's evaluation point x - lambda*e_k closest to y.
// One launch covers DIAG_KC workers k0..k0+DIAG_KC-1: a thread walks all W workers of
// its four columns in order to form e_t there (keeping the values of the launch's own
// workers in registers), then adds the products to 2*DIAG_KC running sums; it strides
// over the columns with the whole grid.  The grid is as many one-wave workgroups as the
// GPU holds at once (the 2*DIAG_KC float64 sums and the DIAG_KC kept groups leave room
// for three waves per SIMD), so all of them run from the first column to the last and
// none waits for a second round.  Each wave adds its lanes' sums and writes one row of
// partials; a second kernel adds the rows in a fixed order, one workgroup per worker.
// No atomics.
// ---------------------------------------------------------------------------
constexpr int DIAG_KC = 16;
constexpr uint32_t DIAG_WORKER_THREADS = 64;
constexpr uint32_t DIAG_WORKER_ROWS_MAX = 8192;    // rows of partials the context allocates at most
constexpr uint32_t DIAG_WORKER_ROWS_DEFAULT = 2048; // used when the occupancy query fails

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;                              // valid in lane 0
}

// Adds rows k_from..k_to-1 at column group i to acc, in order; eight loads are issued before
// the first sum needs its value.
template <bool NT>
__device__ __forceinline__ void diag_add_rows(const DefStepArgs &a, uint64_t i, uint32_t k_from, uint32_t k_to,
                                              double (&acc)[4])
{
    uint32_t k = k_from;
    for (; k + 8 <= k_to; k += 8) {
        v4f ev[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) ev[u] = load4<NT>(a.e + (uint64_t)(k + u) * a.ld + i);
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] += (double)ev[u][c];
    }
    for (; k < k_to; ++k) {
        const v4f ev = load4<NT>(a.e + (uint64_t)k * a.ld + i);          // padding columns hold zeros
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += (double)ev[c];
    }
}

// FULL: the launch's DIAG_KC workers all exist (k0 + DIAG_KC <= W), so their loads carry no
// condition and all go out before the first is used.  NT: non-temporal loads, for error
// memories too large to stay in the caches anyway (5.73 -> 5.12 ms at d = 138 M, W = 32).
template <bool FULL, bool NT>
__global__ __launch_bounds__(DIAG_WORKER_THREADS) void def_diag_workers_partial_kernel(DefStepArgs a, uint32_t k0,
                                                                                       double *partials)
{
    double nrm[DIAG_KC], inn[DIAG_KC];
#pragma unroll
    for (int q = 0; q < DIAG_KC; ++q) nrm[q] = inn[q] = 0.0;
    const uint32_t k_end = FULL ? k0 + (uint32_t)DIAG_KC : min(a.W, k0 + (uint32_t)DIAG_KC);
    const uint64_t stride = (uint64_t)gridDim.x * DIAG_WORKER_THREADS * 4;
    for (uint64_t i = ((uint64_t)blockIdx.x * DIAG_WORKER_THREADS + threadIdx.x) * 4; i < a.d; i += stride) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        v4f own[DIAG_KC];
        // all loads first, none of them used before the last is issued; a worker past the
        // last one (uniform over the wave) is not loaded and counts as zeros
#pragma unroll
        for (int q = 0; q < DIAG_KC; ++q) {
            own[q] = (v4f)(0.0f);
            if (FULL || k0 + q < k_end)
                own[q] = load4<NT>(a.e + (uint64_t)(k0 + q) * a.ld + i);   // padding columns hold zeros
        }
        diag_add_rows<NT>(a, i, 0, k0, acc);
#pragma unroll
        for (int q = 0; q < DIAG_KC; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] += (double)own[q][c];        // adding +0 changes nothing
        diag_add_rows<NT>(a, i, k_end, a.W, acc);
        double mean[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) mean[c] = acc[c] / (double)a.W;         // e_t
#pragma unroll
        for (int q = 0; q < DIAG_KC; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const double v = (double)own[q][c];
                nrm[q] += v * v;
                inn[q] += mean[c] * v;
            }
    }
    double *row = partials + (uint64_t)blockIdx.x * 2 * a.W;
#pragma unroll
    for (int q = 0; q < DIAG_KC; ++q) {
        const double bn = wave_sum(nrm[q]);
        const double bi = wave_sum(inn[q]);
        if (threadIdx.x == 0 && k0 + q < k_end) {
            row[k0 + q] = bn;
            row[a.W + k0 + q] = bi;
        }
    }
}

// Workgroup k adds worker k's two columns of the partials: every thread adds the rows
// r = t, t + 256, ... in order, then the workgroup adds its threads' sums (a fixed tree).
__global__ __launch_bounds__(DEF_THREADS) void def_diag_workers_final_kernel(const double *partials, uint32_t rows,
                                                                             uint32_t W, double *out)
{
    __shared__ double lds[DEF_THREADS / 64];
    const uint32_t k = blockIdx.x;
    double n = 0.0, in = 0.0;
    for (uint32_t r = threadIdx.x; r < rows; r += DEF_THREADS) {
        n += partials[(uint64_t)r * 2 * W + k];
        in += partials[(uint64_t)r * 2 * W + W + k];
    }
    const double norm = block_sum(n, lds);
    const double inner = block_sum(in, lds);
    if (threadIdx.x == 0) {
        out[k] = norm;                                      // ||e_k||^2
        out[W + k] = inner;                                 // <e_t, e_k>
        out[2 * W + k] = norm > 0.0 ? inner / norm : 0.0;   // lambda*(k,t)
    }
}

// ---------------------------------------------------------------------------
// Block draw on the device (Sec. 1: one uniformly sampled start index, same seed
// for all workers).  Philox4x64-10 (Salmon et al., SC 2011) with counter (t,0,0,0)
// and key (seed,0); the first output word mod d.
// ---------------------------------------------------------------------------
__global__ void def_draw_kernel(DefCtl *ctl, uint64_t d)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    uint64_t start;
    if (ctl->forced >= 0) {
        start = (uint64_t)ctl->forced;
    } else {
        const uint64_t mul0 = 0xD2E7470EE14C6C93ull, mul1 = 0xCA5A826395121157ull;
        uint64_t c0 = ctl->t, c1 = 0, c2 = 0, c3 = 0, k0 = ctl->seed, k1 = 0;
        for (int round = 0; round < 10; ++round) {
            const uint64_t hi0 = __umul64hi(mul0, c0), lo0 = mul0 * c0;
            const uint64_t hi1 = __umul64hi(mul1, c2), lo1 = mul1 * c2;
            const uint64_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
            c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
            k0 += 0x9E3779B97F4A7C15ull;
            k1 += 0xBB67AE8584CAA73Bull;
        }
        start = c0 % d;
    }
    ctl->s = start;
    ctl->backwards = (uint32_t)(ctl->t & 1u);
    ctl->t = ctl->t + 1;
    ctl->forced = -1;
}

__global__ void def_ctl_set_kernel(DefCtl *ctl, uint32_t mask, uint64_t t, uint64_t seed, int64_t forced)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (mask & DEF_CTL_T) ctl->t = t;
    if (mask & DEF_CTL_SEED) ctl->seed = seed;
    if (mask & DEF_CTL_FORCED) ctl->forced = forced;
}

uint32_t grid_for(uint64_t total)
{
    return (uint32_t)((total + 7) / 8 * 8);                   // whole rounds over the 8 XCDs
}

// Work items of the blocked order: per worker, the full super-tiles and the last, short one
// rounded up to a multiple of 8 tiles (see decode_item).
uint64_t blocked_items(uint64_t tiles, uint32_t W)
{
    static_assert(DEF_SUPER_TILES % 8 == 0, "a super-tile must be whole rounds over the 8 XCDs");
    const uint64_t full = tiles / DEF_SUPER_TILES, last = tiles % DEF_SUPER_TILES;
    return (full * DEF_SUPER_TILES + (last + 7) / 8 * 8) * W;
}

}  // namespace

// g, m and e are touched once per step.  What can stay in the 256 MiB Infinity Cache
// from one step to the next is the state that the next step reads again: m, e and, if
// the pass reads it, x.  While that fits, ordinary cached accesses win (m + e of 218 MB:
// 83 % of the HBM peak against 77.5 % with non-temporal accesses); once it does not,
// cached accesses only churn the caches and non-temporal ones win (246 MB: 74.6 against
// 77.9 %; 306 MB: 72 against 83 %; 3.3 GB: +20 %).
static bool streams_non_temporal(const DefStepArgs &a)
{
    const uint64_t rows = (uint64_t)a.W * a.ld * sizeof(float);
    const bool reads_x = a.wd != 0.0f || a.w != nullptr;
    const uint64_t resident = rows * (a.mu != 0.0f ? 2u : 1u) + (reads_x ? a.d * sizeof(float) : 0u);
    return resident > DEF_NT_MIN_STATE_BYTES;
}

void def_describe_stream_kernel(const DefStepArgs &a, char *out, size_t cap)
{
    const int mu = a.mu != 0.0f, wd = a.wd != 0.0f, dt = a.w != nullptr;
    const bool reads_x = wd || dt;
    const int tables = a.g_ptrs != nullptr || (reads_x && a.x_ptrs != nullptr);
    char order[32];
    if (reads_x) std::snprintf(order, sizeof order, "blocked:%u", DEF_SUPER_TILES);
    else std::snprintf(order, sizeof order, "linear");
    std::snprintf(out, cap,
                  "def_stream_vec4_kernel<mu=%d,wd=%d,detach=%d,tables=%d,threads=%u,quads=%u,nt=%d,order=%s,sweep=alternating,lds=%u>",
                  mu, wd, dt, tables, DEF_VEC_THREADS, DEF_VEC_QUADS, (int)streams_non_temporal(a), order,
                  def_stream_lds_reserve(mu, dt, streams_non_temporal(a)));
}

// Picks the instantiation for (momentum, weight decay, detached points).  Whenever x
// is read by every worker (weight decay, or w = x - lambda*e), the blocked order lets
// all W workers pass over a piece of x while it sits in L2, so x is fetched from HBM
// once per step instead of W times; otherwise nothing is shared between workers and
// the plain row-after-row sweep is fastest.
#define DEF_DISPATCH(LAUNCH)                                        \
    do {                                                            \
        const int sel = (mu ? 4 : 0) | (wd ? 2 : 0) | (dt ? 1 : 0); \
        switch (sel) {                                              \
        case 0: LAUNCH(false, false, false, MAP_LINEAR_T, 0u); break;   \
        case 1: LAUNCH(false, false, true, MAP_BLOCKED, SUPER); break;  \
        case 2: LAUNCH(false, true, false, MAP_BLOCKED, SUPER); break;  \
        case 3: LAUNCH(false, true, true, MAP_BLOCKED, SUPER); break;   \
        case 4: LAUNCH(true, false, false, MAP_LINEAR_T, 0u); break;    \
        case 5: LAUNCH(true, false, true, MAP_BLOCKED, SUPER); break;   \
        case 6: LAUNCH(true, true, false, MAP_BLOCKED, SUPER); break;   \
        default: LAUNCH(true, true, true, MAP_BLOCKED, SUPER); break;   \
        }                                                           \
    } while (0)

template <bool NT, bool TABLES>
static void launch_vec4(const DefStepArgs &a, uint64_t tiles, uint64_t total, dim3 grid, dim3 block,
                        hipStream_t st)
{
    constexpr int U = DEF_VEC_QUADS, T = DEF_VEC_THREADS;
    constexpr uint32_t SUPER = DEF_SUPER_TILES;
    const bool mu = a.mu != 0.0f, wd = a.wd != 0.0f, dt = a.w != nullptr;
#define DEF_LAUNCH_VEC(MU, WD, DT, MAP, SUP) \
    def_stream_vec4_kernel<MU, WD, DT, TABLES, T, U, NT, NT, MAP>                                   \
        <<<grid, block, def_stream_lds_reserve(MU, DT, NT), st>>>(a, tiles, total, SUP)
    DEF_DISPATCH(DEF_LAUNCH_VEC);
#undef DEF_LAUNCH_VEC
}

static bool uses_tables(const DefStepArgs &a)
{
    const bool reads_x = a.wd != 0.0f || a.w != nullptr;
    return a.g_ptrs != nullptr || (reads_x && a.x_ptrs != nullptr);
}

hipError_t def_launch_stream(const DefStepArgs &a, hipStream_t st)
{
    const uint64_t per_tile = DEF_VEC_TILE;
    const uint64_t tiles = (a.d + per_tile - 1) / per_tile;
    const bool blocked = a.wd != 0.0f || a.w != nullptr;      // as DEF_DISPATCH chooses the order
    const uint64_t total = blocked ? blocked_items(tiles, a.W) : tiles * a.W;
    if (total > 0x7fffffffull - 8) return hipErrorInvalidConfiguration;
    const dim3 grid(grid_for(total)), block(DEF_VEC_THREADS);
    const bool nt = streams_non_temporal(a);
    if (uses_tables(a)) {
        if (nt) launch_vec4<true, true>(a, tiles, total, grid, block, st);
        else launch_vec4<false, true>(a, tiles, total, grid, block, st);
    } else {
        if (nt) launch_vec4<true, false>(a, tiles, total, grid, block, st);
        else launch_vec4<false, false>(a, tiles, total, grid, block, st);
    }
    return hipGetLastError();
}

hipError_t def_launch_average_update(const DefStepArgs &a, hipStream_t st)
{
    const uint64_t tiles = (a.B + DEF_AVG_TILE - 1) / DEF_AVG_TILE;
    if (tiles > 0x7fffffffull) return hipErrorInvalidConfiguration;
    def_average_update_kernel<<<dim3((uint32_t)tiles), dim3(DEF_THREADS), 0, st>>>(a);
    return hipGetLastError();
}

hipError_t def_launch_block_sum(const DefStepArgs &a, hipStream_t st)
{
    const uint64_t tiles = (a.B + DEF_AVG_TILE - 1) / DEF_AVG_TILE;
    if (tiles > 0x7fffffffull) return hipErrorInvalidConfiguration;
    def_block_sum_kernel<<<dim3((uint32_t)tiles), dim3(DEF_THREADS), 0, st>>>(a);
    return hipGetLastError();
}

hipError_t def_launch_apply_block(const DefStepArgs &a, const float *block, float divisor, hipStream_t st)
{
    const uint64_t blocks = (a.B + DEF_THREADS - 1) / DEF_THREADS;
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    def_apply_block_kernel<<<dim3((uint32_t)blocks), dim3(DEF_THREADS), 0, st>>>(a, block, divisor);
    return hipGetLastError();
}

hipError_t def_launch_draw(DefCtl *ctl, uint64_t d, hipStream_t st)
{
    def_draw_kernel<<<dim3(1), dim3(64), 0, st>>>(ctl, d);
    return hipGetLastError();
}

hipError_t def_launch_ctl_set(DefCtl *ctl, uint32_t mask, uint64_t t, uint64_t seed, int64_t forced,
                              hipStream_t st)
{
    def_ctl_set_kernel<<<dim3(1), dim3(64), 0, st>>>(ctl, mask, t, seed, forced);
    return hipGetLastError();
}

uint64_t def_diag_blocks(uint64_t d)
{
    const uint64_t quads = (d + 3) / 4;
    return (quads + DEF_THREADS - 1) / DEF_THREADS;
}

hipError_t def_launch_diagnostics(const DefStepArgs &a, float lambda, double *partials, double *out,
                                  hipStream_t st)
{
    const uint64_t blocks = def_diag_blocks(a.d);
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    def_diag_partial_kernel<<<dim3((uint32_t)blocks), dim3(DEF_THREADS), 0, st>>>(a, partials);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    def_diag_final_kernel<<<dim3(1), dim3(DEF_THREADS), 0, st>>>(partials, blocks, a.W, lambda, out);
    return hipGetLastError();
}

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_device_tables_mutex;
uint32_t g_diag_worker_rows[MAX_DEVICES];    // one-wave workgroups of the per-worker pass each GPU holds at once

uint64_t diag_worker_tiles(uint64_t d)
{
    const uint64_t per_wave = (uint64_t)DIAG_WORKER_THREADS * 4;
    return (d + per_wave - 1) / per_wave;
}

// Grid of the per-worker pass on the current GPU: what is resident at once, looked up once per GPU.
uint32_t diag_worker_resident_rows()
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= MAX_DEVICES) {
        (void)hipGetLastError();
        return DIAG_WORKER_ROWS_DEFAULT;
    }
    std::lock_guard<std::mutex> lock(g_device_tables_mutex);
    if (!g_diag_worker_rows[device]) {
        int units = 0, per_unit = 0;
        uint32_t rows = DIAG_WORKER_ROWS_DEFAULT;
        if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_unit, def_diag_workers_partial_kernel<true, true>,
                                                         (int)DIAG_WORKER_THREADS, 0) == hipSuccess &&
            units > 0 && per_unit > 0) {
            const uint64_t resident = (uint64_t)units * (uint64_t)per_unit;
            rows = (uint32_t)(resident < DIAG_WORKER_ROWS_MAX ? resident : DIAG_WORKER_ROWS_MAX);
        } else {
            (void)hipGetLastError();
        }
        g_diag_worker_rows[device] = rows;
    }
    return g_diag_worker_rows[device];
}
}  // namespace

void def_prepare_diagnostics_workers() { (void)diag_worker_resident_rows(); }

uint64_t def_diag_worker_blocks(uint64_t d)
{
    const uint64_t need = diag_worker_tiles(d);
    return need < DIAG_WORKER_ROWS_MAX ? need : DIAG_WORKER_ROWS_MAX;
}

hipError_t def_launch_diagnostics_workers(const DefStepArgs &a, double *partials, double *out, hipStream_t st)
{
    const uint64_t need = diag_worker_tiles(a.d);
    const uint32_t resident = diag_worker_resident_rows();
    const uint32_t rows = (uint32_t)(need < resident ? need : resident);      // <= def_diag_worker_blocks(d)
    const bool nt = (uint64_t)a.W * a.ld * sizeof(float) > DEF_NT_MIN_STATE_BYTES;
    for (uint32_t k0 = 0; k0 < a.W; k0 += DIAG_KC) {
        const bool full = k0 + DIAG_KC <= a.W;
        const dim3 grid(rows), block(DIAG_WORKER_THREADS);
        if (nt) {
            if (full) def_diag_workers_partial_kernel<true, true><<<grid, block, 0, st>>>(a, k0, partials);
            else def_diag_workers_partial_kernel<false, true><<<grid, block, 0, st>>>(a, k0, partials);
        } else {
            if (full) def_diag_workers_partial_kernel<true, false><<<grid, block, 0, st>>>(a, k0, partials);
            else def_diag_workers_partial_kernel<false, false><<<grid, block, 0, st>>>(a, k0, partials);
        }
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    def_diag_workers_final_kernel<<<dim3(a.W), dim3(DEF_THREADS), 0, st>>>(partials, rows, a.W, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Device memory that belongs to the library image itself: the per-workgroup partial
// sums of def_diagnostics_static, so that this one entry point needs no allocation.
// Every GPU holds its own copy at its own address; the name below is a host-side
// handle and must never be passed to a kernel: the device address is looked up once
// per GPU with hipGetSymbolAddress and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) double def_static_scratch[DEF_STATIC_SCRATCH_DOUBLES];

namespace {
double *g_static_scratch_ptr[MAX_DEVICES];   // device address of def_static_scratch on each GPU
}  // namespace

hipError_t def_static_scratch_address(double **ptr)
{
    int device = -1;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) return err;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_device_tables_mutex);
    if (!g_static_scratch_ptr[device]) {
        void *found = nullptr;
        err = hipGetSymbolAddress(&found, HIP_SYMBOL(def_static_scratch));   // for the current GPU
        if (err != hipSuccess) return err;
        if (!found) return hipErrorInvalidSymbol;
        g_static_scratch_ptr[device] = static_cast<double *>(found);
    }
    *ptr = g_static_scratch_ptr[device];
    return hipSuccess;
}

hipError_t def_launch_detach(const DefStepArgs &a, hipStream_t st)
{
    static_assert(DEF_VEC_QUADS == 1, "def_detach_kernel handles one group per thread");
    const uint64_t tiles = (a.d + DEF_VEC_TILE - 1) / DEF_VEC_TILE;
    const uint64_t total = blocked_items(tiles, a.W);
    if (total > 0x7fffffffull - 8) return hipErrorInvalidConfiguration;
    // two loads and one store of 1 KiB per wave: as many waves as fit (32 per compute unit:
    // 79 % of the HBM peak; capped at 16: 62 %)
    def_detach_kernel<<<dim3(grid_for(total)), dim3(DEF_VEC_THREADS), 0, st>>>(a, tiles, total);
    return hipGetLastError();
}

hipError_t def_launch_output(const DefStepArgs &a, float *y, hipStream_t st)
{
    const uint64_t quads = (a.d + 3) / 4;
    const uint64_t blocks = (quads + DEF_OUT_THREADS - 1) / DEF_OUT_THREADS;
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    def_output_kernel<<<dim3((uint32_t)blocks), dim3(DEF_OUT_THREADS), DEF_OUT_LDS_RESERVE, st>>>(a, y);
    return hipGetLastError();
}
