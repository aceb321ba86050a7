// Internal interface between the host side of the library (def_api.hip) and
// its kernels (def_kernels.hip).  Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

constexpr uint32_t DEF_GRAD_TABLES = 4;      // gradient pointer tables kept on the device
constexpr uint32_t DEF_AVG_TILE = 256;      // block columns per workgroup of the averaging kernel
constexpr uint32_t DEF_THREADS = 256;       // workgroup size of every kernel but the streaming pass
// Launch shape of the streaming kernel.  Measured on MI355X (d = 25.6 M,
// W = 16): one wave per workgroup with one float4 group per lane beats every larger
// tile (64x1: 78 % of the 8 TB/s HBM peak, 256x1: 75 %, 256x4: 73 %); stores
// in particular lose bandwidth when a wave issues several of them back to back.
constexpr uint32_t DEF_VEC_THREADS = 64;
constexpr uint32_t DEF_VEC_QUADS = 1;       // float4 groups per thread
constexpr uint32_t DEF_VEC_TILE = DEF_VEC_THREADS * DEF_VEC_QUADS * 4;   // indices per tile
// Tiles per super-tile of the blocked work-item order used with weight decay.  One
// tile is 1 KiB of a row, so a super-tile covers 16 MiB of x; workgroups are dealt
// round-robin to the 8 XCDs, so each XCD's 4 MiB L2 holds 2 MiB of x while the W
// workers pass over it.  Measured (d = 25.6 M, W = 16, random data): 8192 -> 78.4 %,
// 16384 -> 79.6 %, 32768 -> 75 % of the HBM peak (the piece no longer fits in L2).
constexpr uint32_t DEF_SUPER_TILES = 16384;
// Dynamic LDS reserved per one-wave workgroup of the streaming kernel.  The kernel
// does not touch it: a compute unit has 160 KiB of LDS, handed out in 1280-byte
// granules, so a reservation of 10240 bytes caps residency at 16 one-wave
// workgroups (4 waves per SIMD) instead of the 32 that would otherwise fit.  What
// the memory system rewards is a certain amount of traffic in flight per compute
// unit, about 80 KiB of loads plus stores: fewer waves leave latency uncovered, more
// widen the window of addresses being read and written and lose DRAM locality.  A
// wave moves 1 KiB per stream, so the best residency depends on how many streams the
// instantiation has (measured, d = 25.6 M, W = 16, random data, % of the HBM peak):
//   g m e -> m e     (5 streams)  32: 78.8  18: 79.4  16: 80.2-81  14: 79.3  12: 73.6
//   g m e -> m e w   (6 streams)  32: 75    16: 78.5  14: 79.2     12: 78.6  11: 76.8
//   g e -> e         (3 streams)  32: 82.4  25: 82.8  21: 82.0     18: 74.2  16: 71.2
//   g e -> e w       (4 streams)  32: 76    21: 78.3  18: 78.9     16: 78.3  14: 75.4
// (measured with m and e at the same alignment and rows on 256-byte boundaries).  With the state
// placed as below (rows on 1 KiB boundaries, m and e apart) the five-stream optimum moves up:
//   g m e -> m e     d = 25.6 M, weight decay   18: 84.6  17: 84.5  16: 84.0-84.5  14: 80.9  12: 71.2
//                    d = 11.7 M, none           18: 82.7-83.6      16: 81.7-82.5  14: 80.8
//   g m e -> m e w   16: 81.2-82.2  14: 81.9-83.1  12: 81.3  11: 77.1
//   g e -> e w       32: 78.4  21: 81.5-82.7  18: 81.3-82.1  16: 79.2
// (two builds, 16 against 18 per compute unit, benchmark on one box: 84.5 -> 84.9 % at d = 25.6 M,
// 81.8 -> 83.0 % at d = 11.7 M, 81.3 -> 82.2 % at d = 138 M).
// Steps whose state the caches can hold (see DEF_NT_MIN_STATE_BYTES) run uncapped: at
// 137 MB per step 32 per compute unit is 2-3 % faster than 16.
constexpr uint32_t def_stream_lds_reserve(bool has_mu, bool has_dt, bool non_temporal)
{
    if (!non_temporal) return 0u;
    return has_mu ? (has_dt ? 11520u : 8960u)     // 14 / 18 workgroups per compute unit
                  : (has_dt ? 7680u : 0u);        // 21 / as many as fit (32)
}
// The DEF output kernel (one wave per workgroup, every thread walks the W workers of its
// four columns with four loads in flight): 8 workgroups per compute unit.  Measured at
// the same shape: 256-thread workgroups, uncapped 75 %; one wave, uncapped 78 %, 16 per
// compute unit 81 %, 12: 82.5 %, 8: 85.4 % of the HBM peak.
constexpr uint32_t DEF_OUT_THREADS = 64;
constexpr uint32_t DEF_OUT_LDS_RESERVE = 20480;
// When the state a step reads again next time (m, e, and x if the pass reads it) is larger
// than this, g, m and e are accessed non-temporally; below it they are cached normally.
constexpr uint64_t DEF_NT_MIN_STATE_BYTES = 224ull << 20;

// Placement of the two state buffers relative to each other and to the gradients.  The
// streaming pass reads g, m and e and writes m and e at the same offsets at the same time; when
// the addresses also agree in their low bits (as fresh allocations do, all being aligned to far
// more than 16 KiB) their requests meet in the same memory resources and the pass loses
// bandwidth.  Measured with m placed this many bytes past e's alignment (five streams,
// d = 25.6 M, W = 16, % of the HBM peak; boxes differ):
//   box A   0: 81.3   256: 81.3   2048: 83.1   4096: 84.6   8192: 82.1   12288: 85.0   20480: 84.2   36864: 84.3
//   box B   0: 82.0   1024: 82.2  2048: 81.3   4096: 82.8   8192: 83.0   12288: 82.9   20480: 82.6   36864: 82.3
// and for d = 11.7 M without weight decay on box B   0: 78.4   4096: 79.8   12288: 79.8   20480: 80.1.
// Odd multiples of 4 KiB are good everywhere: m sits 12 KiB past e (mod 16 KiB).  Gradient rows
// that differ from e in address bit 12 or 13 gave another 0.4-0.9 points (three streams: 0.6-1.2);
// gradients are the caller's and usually sit on a large power of two, so e itself is put 8 KiB
// past a 16 KiB boundary and m 4 KiB past one (two builds, benchmark on one box, against e on the
// boundary: 84.5 -> 84.8 % five streams, 82.7 -> 83.4 % three streams, 81.8 -> 82.5 % six).
constexpr uint64_t DEF_STATE_SKEW_PERIOD = 16384;
constexpr uint64_t DEF_STATE_E_OFFSET = 8192;
constexpr uint64_t DEF_STATE_M_OFFSET = 4096;

// Row stride of e and m: a multiple of the tile (256 floats = 1 KiB), so that every wave
// instruction of the streaming pass covers exactly one aligned KiB of each state buffer.  With
// rows that start on other 256-byte boundaries every access straddles two aligned KiB and the pass
// loses bandwidth (same process, % of the HBM peak, stride mod 8 KiB -> d = 25.6 M with weight decay
// / without / d = 11.7 M without):  256 B: 83.1 / 79.6 / 79.0   512 B: 83.6 / 81.0 / 80.4
// 1 KiB: 84.6 / 82.3 / 81.4   2 KiB: 84.3 / 82.6 / 81.9   4 KiB: 84.7 / 82.6 / 81.9   0: 84.3 / 82.1 / 81.3.
// The stride of the caller's gradient rows matters less (0 to 0.5 points).
constexpr uint64_t DEF_STATE_ROW_MULTIPLE = 256;
static_assert(DEF_STATE_ROW_MULTIPLE % DEF_VEC_TILE == 0, "state rows must start on tile boundaries");

// Device-resident copy of the draw state, used when the block start is drawn on the
// device so that a captured HIP graph of a step can be replayed (each replay advances t).
struct DefCtl {
    uint64_t t;       // step counter
    uint64_t seed;    // shared seed
    int64_t forced;   // >= 0: start to use for the next step only
    uint64_t s;       // start drawn for the step in flight
    uint32_t backwards;   // sweep direction of the step in flight (t odd)
};

// Everything one step needs on the device.
struct DefStepArgs {
    // problem (notation of Algorithm 1 / Sec. 3.2 of arXiv 2004.05298)
    uint64_t d;        // parameters
    uint64_t B;        // block length
    uint64_t s;        // block start s_t (host draw)
    uint32_t backwards; // host draw: the streaming pass sweeps its work items in reverse (odd t)
    const DefCtl *ctl; // not null: the start is ctl->s, drawn on the device by def_launch_draw
    uint32_t W;        // workers
    float lr, mu, wd;  // eta, mu, weight decay
    // library-owned state
    float *e;          // [W][ld] error memory
    float *m;          // [W][ld] momentum buffer (nullptr when mu == 0)
    uint64_t ld;       // row stride of e and m, multiple of DEF_STATE_ROW_MULTIPLE
    float *msg;        // [W][ldmsg] compact compressed vectors C(p_k): entry j <-> index (s+j) mod d
    uint64_t ldmsg;    // multiple of DEF_AVG_TILE
    float *avg;        // [B] averaged block
    // parameters x
    float *x_flat;             // flat mode, else nullptr
    float *const *x_ptrs;      // DEVICE table of L tensor pointers (tensor mode), else nullptr
    const uint64_t *off;       // DEVICE offset table, L+1 entries
    uint32_t L;
    // gradients
    const float *g_flat;       // flat mode: worker k at g_flat + k*ldg
    uint64_t ldg;
    const float *const *g_ptrs;  // DEVICE table [W][L] (tensor mode), else nullptr
    // tensor that holds the first index of each tile of DEF_VEC_TILE indices (DEVICE)
    const uint32_t *tile_tensor;
    // detached evaluation points w_k = x - lambda*e_k (nullptr: not requested)
    float *w;                  // [W][ldw]
    uint64_t ldw;
    float lam;
};

// Text describing the instantiation def_launch_stream picks for these arguments.
void def_describe_stream_kernel(const DefStepArgs &a, char *out, size_t cap);
// Device draw: ctl->s = forced or Philox4x64-10((t,0,0,0),(seed,0))[0] mod d; ++t; forced = -1.
hipError_t def_launch_draw(DefCtl *ctl, uint64_t d, hipStream_t st);
// Overwrite the fields of the device draw state selected by mask.
enum : uint32_t { DEF_CTL_T = 1, DEF_CTL_SEED = 2, DEF_CTL_FORCED = 4 };
hipError_t def_launch_ctl_set(DefCtl *ctl, uint32_t mask, uint64_t t, uint64_t seed, int64_t forced,
                              hipStream_t st);
// Fused momentum + error feedback + compress + residual pass (+ detached points), dwordx4
// accesses.  Gradients: one buffer (g_flat) or per-tensor pointers (g_ptrs); parameters, if the
// pass reads them: one vector (x_flat) or per-tensor pointers (x_ptrs).  Any 4-byte alignment.
hipError_t def_launch_stream(const DefStepArgs &a, hipStream_t st);
// Cross-worker average of the compact blocks (LDS-staged) and parameter update.
hipError_t def_launch_average_update(const DefStepArgs &a, hipStream_t st);
// The same in two halves: avg[j] = sum_k msg_k[j] (no division, x untouched), and
// x[(s+j) mod d] -= block[j] / divisor (also avg[j] = block[j] / divisor, and w on the block).
hipError_t def_launch_block_sum(const DefStepArgs &a, hipStream_t st);
hipError_t def_launch_apply_block(const DefStepArgs &a, const float *block, float divisor, hipStream_t st);
// y = x - mean_k e_k.
hipError_t def_launch_output(const DefStepArgs &a, float *y, hipStream_t st);
// Error-memory statistics: ||e_t||^2, (1/W) sum_k ||e_k||^2, lambda*(t) and the distance
// (1/W) sum_k ||e_t - lambda*e_k||^2, as 4 doubles in out.  partials: def_diag_blocks(d) * 2 doubles.
uint64_t def_diag_blocks(uint64_t d);
hipError_t def_launch_diagnostics(const DefStepArgs &a, float lambda, double *partials, double *out,
                                  hipStream_t st);
// Device address, on the GPU that is current, of the library's static scratch array of
// DEF_STATIC_SCRATCH_DOUBLES doubles (looked up once per GPU; no allocation).
constexpr uint64_t DEF_STATIC_SCRATCH_DOUBLES = 1ull << 19;      // 4 MiB
hipError_t def_static_scratch_address(double **ptr);
// w_k = x - lambda*e_k for the current state (a.w, a.ldw, a.lam).
hipError_t def_launch_detach(const DefStepArgs &a, hipStream_t st);
// Per-worker statistics ||e_k||^2, <e_t, e_k> and their ratio lambda*(k,t), as 3*W doubles in out.
// partials: def_diag_worker_blocks(d) * 2 * W doubles (an upper bound on what a launch uses).
uint64_t def_diag_worker_blocks(uint64_t d);
// Looks up, once per GPU, how many workgroups of the per-worker pass the current GPU holds at
// once (its grid), so that the first def_launch_diagnostics_workers asks the runtime nothing.
void def_prepare_diagnostics_workers();
hipError_t def_launch_diagnostics_workers(const DefStepArgs &a, double *partials, double *out, hipStream_t st);
