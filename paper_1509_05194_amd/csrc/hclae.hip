// C ABI of libhclae: argument checks, scratch ownership and kernel sequencing for the
// Dictionary Annealing sweep (arXiv 1509.05194, Sec. 3.1; encoder: Eq. 3 with one path;
// error: Eq. 1 first line).  All arithmetic of the method happens in the kernels included
// below; this file only validates, sizes launches and orders them on one stream.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <new>

#include "../../include/hclae.h"
#include "assign.hpp"
#include "assign_split.hpp"
#include "stream.hpp"
#include "update.hpp"
#include "pca.hpp"
#include "eigen.hpp"
#include "stats.hpp"
#include "beam.hpp"
#include <algorithm>
#include <vector>

using namespace hclae;

namespace {

constexpr int kFlatParts = 4096;         // upper bound on blocks of a flat (copy / reduction) pass
constexpr int kLdsBudget = 160 * 1024;   // LDS per workgroup on gfx950
constexpr int kMaxTimed = 4096;          // event pairs kept between two hclae_timing_read calls

thread_local char g_create_error[256] = "";

}  // namespace

// Scratch of hclae_quant_error_noalloc: one fp64 partial sum per block of the reduction (at most kFlatParts
// blocks whatever the input size: the blocks stride over the array), 32 KB.  Every GPU the library runs on holds
// its own copy of the array at its own address until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: the address a kernel may use is the one that call returns, once per device.
static __device__ __align__(256) double g_noalloc_scratch[kFlatParts];

namespace {

constexpr int kMaxDevices = 64;
double *g_noalloc_ptr[kMaxDevices];      // device address of g_noalloc_scratch on device i, or null: not asked yet
std::mutex g_noalloc_mutex;

// Address of the current device's copy of g_noalloc_scratch (asked from the runtime on first use, then kept).
hipError_t noalloc_scratch(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (!g_noalloc_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_noalloc_ptr[dev] = static_cast<double *>(p);
    }
    *out = g_noalloc_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct hclae_ctx {
    int64_t N_max;
    int D, M, K;
    int kb;                  // 32-codeword blocks of the padded codebook: 1, 2, 4 or 8
    int NC;                  // 64-dim chunks of the padded D
    bool resident;           // whole padded codebook fits LDS
    int cus;
    hipStream_t stream;
    int device;
    // scratch (device)
    float *hneg;             // [32*kb]
    float4 *cb_image;        // [NC][kb*8*64] codebook in staging order (k_codebook_image; D-chunked shapes only)
    float *lds_image;        // [kb*8*NC*64*4] dictionary of the running stage in the LDS order of the resident assign kernel
    uint4 *split_image;      // [kb*4*NC*2*64] split dictionary in the LDS order of k_assign_split (written by k_split_norms)
    size_t split_image_bytes;
    float *split_norms;      // [K][2] split constants of the codebook in use (contraction 1)
    int contraction;         // 0: fp32 MFMA, 1: split-bf16 MFMA
    unsigned *refine_count;
    RefineItem *refine_list; // [N_max]
    uint8_t *old_codes;      // [N_max]
    long long *partial;      // [upd_blocks][K][D] fixed-point centroid sums
    int *pcount;             // [upd_blocks][K]
    int *nk;                 // [K]
    // exact incremental centroid update within a stage (see k_merge)
    long long *tot_sum;      // [K][D] fixed-point sums of the stage
    int *tot_cnt;            // [K]
    uint8_t *upd_col;        // [N_max] code column as of the last centroid pass
    unsigned long long *moved_list;  // [N_max]
    unsigned *moved_count;
    // exact pruning of the assignments of a stage (see PruneArgs)
    int pruning;             // 0 off, 1 on (default)
    float *bnd_u, *bnd_l;    // [N_max]
    float *drift;            // [K]
    uint32_t *active;        // [N_max]: the vectors k_bounds_step lists for the next assignment
    float *cur_u, *cur_l;    // the bounds of the running stage: bnd_u / bnd_l, or the stage's own rows of carry_u / carry_l
    // bounds carried from one sweep to the next (hclae_anneal; allocated on first use, see k_bounds_carry)
    float *carry_u, *carry_l;    // [M][N_max] bounds each stage ended its last visit with
    double *carry_path;          // [N_max] running sum of ||d_j||
    double *carry_snap;          // [M][N_max] its value when stage m was last left
    float *carry_Centry;         // [K][D] dictionary of the running stage as the stage found it
    float *carry_T;              // [K][K] pair table of the running stage
    unsigned *carry_amax;        // bits of the largest |x'| or |codeword| coordinate of the call so far
    unsigned long long *work; // [4] work counters: assignments, vectors recomputed, vectors re-checked in fp64
    int64_t *seed_idx;       // [M][K] seed rows of a sweep from all-zero dictionaries (a single stage uses row 0)
    double *part_a, *part_b; // [nparts]
    long long *part_chg;     // [nparts]
    int nparts;              // max(kFlatParts, heat/cool blocks at N_max)
    StageRecord *rec;        // [M]
    // host
    StageRecord *rec_host;   // pinned [M]
    int upd_blocks;
    // online learning state (allocated by hclae_online_begin)
    double *run_sum;         // [M][K][D]
    long long *run_cnt;      // [M][K]
    long long *n0_dev;       // [M][K] staging of the caller's weights
    // improved k-means scratch (allocated on first use)
    float *pca_rt;           // [D][D] transposed rotation
    float *pca_crot;         // [K][D] rotated dictionary
    double *pca_colpart;     // [pca_ncol][D]
    double *pca_grampart;    // [pca_ngram][D][D]
    double *pca_mean;        // [D]
    float *pca_mean32;       // [D]
    double *pca_cov;         // [D][D] covariance of x' when the stage finds the principal axes itself
    float *pca_R;            // [D][D] those axes (rows), fp32
    float *pca_xr;           // [N_max][D] rotated data when the improved k-means is the ctx's cool-down
    int cooldown;            // HCLAE_COOLDOWN_*
    int cooldown_phases;     // prefixes of its dimension schedule before equal ones are merged (I of Sec. 3.2)
    int pca_ncol, pca_ngram;
    // dictionary order and code statistics (allocated on first use)
    unsigned long long *stats_buf;   // [M][K] + [K][K] histogram counters
    double *order_var;       // [M]
    int *order_idx;          // [M]
    float *order_tmp;        // [M][K][D] permuted dictionaries
    // multi-path encoding scratch (allocated on first use, regrown when L or the batch grows)
    int64_t beam_cap;        // vectors per batch the buffers hold
    int beam_L;              // beam width they were sized for
    int sweep_L;             // paths of the re-encode of hclae_sweep, reencode_mode 2
    float *beam_rows[2];     // [beam_cap][beam_L][D] residuals, ping-pong
    double *beam_err[2];     // [beam_cap][beam_L]
    uint8_t *beam_pre[2];    // [beam_cap][beam_L][M] code prefixes
    BeamMask *beam_mask;     // [beam_cap][beam_L]
    // optional per-kernel timing (HIP events on ctx->stream)
    uint32_t t_mask;
    int t_used;
    // hipFuncSetAttribute (dynamic LDS limit) done by this ctx, one bit per call site: the attribute belongs to the
    // device context a ctx was created on, so every ctx raises the limits it needs itself
    uint64_t attr_done;
    hipEvent_t *t_beg, *t_end;   // [kMaxTimed] each, created on first enable
    uint8_t *t_cls;
    char err[256];
};

namespace {

int fail(hclae_ctx *ctx, int code, const char *what, hipError_t e = hipSuccess)
{
    char *dst = ctx ? ctx->err : g_create_error;
    if (e != hipSuccess) snprintf(dst, 256, "%s: %s", what, hipGetErrorString(e));
    else snprintf(dst, 256, "%s", what);
    return code;
}

// Scope guard: brackets the launches issued during its lifetime with two events.
struct Timed {
    hclae_ctx *c;
    int slot;
    Timed(hclae_ctx *ctx, int cls) : c(ctx), slot(-1)
    {
        if ((c->t_mask >> cls) & 1u) {
            if (c->t_used < kMaxTimed && hipEventRecord(c->t_beg[c->t_used], c->stream) == hipSuccess) {
                slot = c->t_used;
                c->t_cls[slot] = (uint8_t)cls;
            }
        }
    }
    ~Timed()
    {
        if (slot >= 0 && hipEventRecord(c->t_end[slot], c->stream) == hipSuccess) c->t_used = slot + 1;
    }
};

#define HIP_TRY(ctx, call)                                                      \
    do {                                                                        \
        hipError_t e__ = (call);                                                \
        if (e__ != hipSuccess) return fail((ctx), HCLAE_EHIP, #call, e__);      \
    } while (0)

int check_call(hclae_ctx *ctx, int64_t N, int D, int M, int K)
{
    if (!ctx) return HCLAE_EINVAL;
    int rc = hclae_check_shape(N, D, M, K);
    if (rc != HCLAE_OK) return fail(ctx, rc, "shape out of range");
    if (D != ctx->D || M != ctx->M || K != ctx->K) return fail(ctx, HCLAE_ESTATE, "D, M, K differ from hclae_create");
    if (N > ctx->N_max) return fail(ctx, HCLAE_ESTATE, "N exceeds N_max of hclae_create");
    return HCLAE_OK;
}

// Float arrays are read and written four floats at a time: 16-byte aligned bases (NULL passes: checked apart).
template <typename... P>
bool misaligned(P... p)
{
    return (((reinterpret_cast<uintptr_t>(p)) | ...) & 15u) != 0;
}

int stream_blocks(const hclae_ctx *ctx, int64_t work_items, int per_block)
{
    int64_t need = (work_items + per_block - 1) / per_block;
    int64_t cap = (int64_t)ctx->cus * 8;
    if (cap > kFlatParts) cap = kFlatParts;
    if (need > cap) need = cap;
    if (need < 1) need = 1;
    return (int)need;
}

RowGeom row_geom(int D);

// Blocks of a heat / cool pass over N rows (also the number of partial sums it writes):
// 32 per CU measured best for the in-place read-modify-write stream, each looping a few times.
int heat_cool_blocks(int64_t N, int D, int cus)
{
    if (D >= kWideMinD) {                  // k_row_pass_wide: a wave per kWideRows rows, 64 blocks per CU measured best
        const int64_t per = (int64_t)(kStreamThreads / kWave) * kWideRows;
        int64_t b = (N + per - 1) / per;
        if (b > (int64_t)cus * 64) b = (int64_t)cus * 64;
        return (int)(b < 1 ? 1 : b);
    }
    const RowGeom g = row_geom(D);
    const int64_t per = (int64_t)(kStreamThreads >> g.lcw) * kStreamUnroll;
    int64_t b = (N + per - 1) / per;
    if (b > (int64_t)cus * 32) b = (int64_t)cus * 32;
    if (b < 1) b = 1;
    return (int)b;
}

RowGeom row_geom(int D)
{
    RowGeom g;
    g.d4 = D / 4;
    int l = 0;
    while ((2 << l) <= g.d4 && l < 6) ++l;     // largest power of two <= min(d4, 64)
    g.lcw = l;
    return g;
}

// ---- launches (all on ctx->stream) ------------------------------------------------------

// amax (heat only): the pass also publishes max |x'| in refine_count[1] (see k_row_pass).
template <int SIGN, bool STATS>
int launch_heat_cool(hclae_ctx *ctx, int m, int64_t N, const float *C, const uint8_t *codes, float *r,
                     double *part_err, bool amax = false)
{
    const RowGeom g = row_geom(ctx->D);
    const int rows = kStreamThreads >> g.lcw;
    const int blocks = heat_cool_blocks(N, ctx->D, ctx->cus);
    (void)rows;
    const float *Cm = C + (size_t)m * ctx->K * ctx->D;
    Timed t_(ctx, SIGN > 0 ? HCLAE_T_HEAT : HCLAE_T_COOL);
    // the row length of the SIFT-shaped configurations has a kernel of its own (addresses and geometry constant:
    // 179 us instead of 185 us for the stage boundary at N = 1M, D = 128); long rows take k_row_pass_wide
    constexpr bool kCanAmax = SIGN > 0 && STATS;
    if (amax && !kCanAmax) return fail(ctx, HCLAE_EINVAL, "row pass: max |x'| is a by-product of the heat pass only");
    if (ctx->D >= kWideMinD) {
        auto kern = (amax && kCanAmax) ? &k_row_pass_wide<SIGN, STATS, kCanAmax> : &k_row_pass_wide<SIGN, STATS, false>;
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(kStreamThreads), 0, ctx->stream,
                           r, codes, Cm, (const float *)nullptr, N, ctx->D, ctx->M, m, 0, ctx->old_codes, part_err,
                           ctx->part_chg, amax ? ctx->carry_amax + kAmaxSlots : (unsigned *)nullptr);
        HIP_TRY(ctx, hipGetLastError());
        return blocks;
    }
    auto kern = (amax && kCanAmax) ? (ctx->D == 128 ? &k_row_pass<SIGN, STATS, 128, kCanAmax> : &k_row_pass<SIGN, STATS, 0, kCanAmax>)
                                   : (ctx->D == 128 ? &k_row_pass<SIGN, STATS, 128, false> : &k_row_pass<SIGN, STATS, 0, false>);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kStreamThreads), 0, ctx->stream,
                       r, codes, Cm, (const float *)nullptr, N, ctx->D, ctx->M, m, 0, g, ctx->old_codes, part_err,
                       ctx->part_chg, amax ? ctx->carry_amax + kAmaxSlots : (unsigned *)nullptr);
    HIP_TRY(ctx, hipGetLastError());
    return blocks;
}

// dact: leading coordinates that count (<= ld); ld: row stride of Cm.
// image: also write the dictionary in the LDS order of the resident assign kernel (the centroid updates that follow
// keep it current; launch_assign then takes it when told so).
// keep_absmax: 0 the counter of max |x'| is reset for the assignment that follows; 1 it stays; 2 it is taken from the
// words the row pass that wrote x' left in carry_amax[64..128) (hclae_anneal).
// With keep_absmax 2 the kernel also copies the dictionary to carry_Centry and clears the list counter of
// k_bounds_carry (moved_count[3]).
int launch_norms(hclae_ctx *ctx, const float *Cm, int dact = 0, int ld = 0, int keep_absmax = 0, bool image = false)
{
    if (dact <= 0) dact = ctx->D;
    if (ld <= 0) ld = ctx->D;
    const int kpad = 32 * ctx->kb;
    Timed t_(ctx, HCLAE_T_NORMS);
    hipLaunchKernelGGL(k_codeword_norms, dim3((kpad + 3) / 4), dim3(256), 0, ctx->stream,
                       Cm, ctx->K, dact, ld, kpad, ctx->hneg, ctx->refine_count, keep_absmax,
                       image && ctx->resident ? ctx->lds_image : (float *)nullptr, 8 * ctx->NC,
                       keep_absmax == 2 ? ctx->carry_amax + kAmaxSlots : (unsigned *)nullptr,
                       keep_absmax == 2 ? ctx->carry_Centry : (float *)nullptr,
                       keep_absmax == 2 ? ctx->moved_count + 3 : (unsigned *)nullptr);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

// prune: 0 plain; 1 all vectors and store the stage's bounds; 2 only the vectors k_bounds_step listed
// (over all D coordinates only; the caller checks).
template <int KB>
int launch_assign_kb(hclae_ctx *ctx, int m, int64_t N, const float *xp, const float *Cm, uint8_t *codes, int dact, int ld,
                     int prune, bool use_image)
{
    PruneArgs pa;
    pa.bu = ctx->cur_u; pa.bl = ctx->cur_l;
    pa.active = ctx->active; pa.active_count = ctx->moved_count + 3;
    // prune 3 = 2, and the re-check kernel lists the vectors that changed cluster (moved_count[0] is zero: the
    // merge of the previous centroid update of this stage reset it)
    MovedArgs mv = {};
    if (prune == 3) {
        mv.prev = ctx->upd_col; mv.list = ctx->moved_list; mv.count = ctx->moved_count;
        mv.cand = ctx->active; mv.cand_count = ctx->moved_count + 3; mv.bl = ctx->cur_l;
        prune = 2;
    }
    const int NC = (dact + kChunkD - 1) / kChunkD;
    const int dpad = kChunkD * NC;
    pa.slack = (float)(dpad / 2 + 16) * 1.1920929e-7f;
    const bool resident = (size_t)32 * KB * dpad * sizeof(float) + 4096 <= (size_t)kLdsBudget;
    // twice the worst-case rounding error of a score: (dpad + 1) roundings of relative size 2^-23
    // on partial sums bounded by h + ||x'|| ||c||, plus the rounding of h itself
    const float eps = 2.02f * (float)(dpad + 2) * 1.1920929e-7f;
    {
    Timed t_(ctx, prune == 2 ? HCLAE_T_ASSIGN_ACTIVE : HCLAE_T_ASSIGN);
    if (resident && ctx->contraction == 1) {
        const size_t lds = (size_t)KB * 8 * NC * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t ntiles = (N + kTileVec - 1) / kTileVec;
        int64_t blocks = (ntiles + 3) / 4;                      // few tiles: one per SIMD before any SIMD gets two
        if (blocks > ctx->cus) blocks = ctx->cus;
        const uint64_t attr_set = 1ull << 0;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split<KB, 0>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split<KB, 1>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split<KB, 2>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        // 3 MFMAs per 16 dims, each within 2^-21 of the magnitudes it adds; one more for the rounding of the norm
        const float acc_bound = (float)(3 * (dpad / kSplitStep) + 1) * 4.76837158203125e-7f;
        if ((size_t)KB * 4 * NC * 2 * kWave * sizeof(uint4) > ctx->split_image_bytes)
            return fail(ctx, HCLAE_EINVAL, "assign: split dictionary image too small for this shape");
        hipLaunchKernelGGL(k_split_norms, dim3((32 * KB + 3) / 4), dim3(256), 0, ctx->stream, Cm, ctx->K, dact, ld, ctx->split_norms,
                           ctx->split_image, KB, 4 * NC);
        auto kern = prune == 1 ? &k_assign_split<KB, 1> : prune == 2 ? &k_assign_split<KB, 2> : &k_assign_split<KB, 0>;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           xp, Cm, ctx->hneg, ctx->split_norms, N, dact, ld, ctx->K, ctx->M, m, NC, acc_bound,
                           codes, ctx->refine_list, ctx->refine_count, pa, ctx->split_image);
    } else if (ctx->contraction == 1) {
        // D-chunked, split-bf16: two slices of 64 dims in LDS, one block per CU
        const size_t lds = (size_t)2 * KB * 8 * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t nbt = (N + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);
        int64_t blocks = nbt < ctx->cus ? nbt : ctx->cus;
        const uint64_t attr_set = 1ull << 1;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split_chunked<KB, 0>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split_chunked<KB, 1>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_split_chunked<KB, 2>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        if (NC > ctx->NC || KB != ctx->kb)
            return fail(ctx, HCLAE_EINVAL, "assign: codebook image too small for this shape");
        const float acc_bound = (float)(3 * (dpad / kSplitStep) + 1) * 4.76837158203125e-7f;
        const int img_total = NC * 4 * KB * kWave;
        hipLaunchKernelGGL(k_split_norms, dim3((ctx->K + 3) / 4), dim3(256), 0, ctx->stream, Cm, ctx->K, dact, ld, ctx->split_norms);
        hipLaunchKernelGGL(k_codebook_image_split, dim3((img_total + 255) / 256), dim3(256), 0, ctx->stream,
                           Cm, ctx->K, dact, ld, KB, NC, reinterpret_cast<uint4 *>(ctx->cb_image));
        auto kern = prune == 1 ? &k_assign_split_chunked<KB, 1> : prune == 2 ? &k_assign_split_chunked<KB, 2>
                                                                              : &k_assign_split_chunked<KB, 0>;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           xp, reinterpret_cast<const uint4 *>(ctx->cb_image), ctx->hneg, ctx->split_norms, N, dact, ld,
                           ctx->K, ctx->M, m, NC, acc_bound, codes, ctx->refine_list, ctx->refine_count, pa);
    } else if (resident) {
        const size_t lds = (size_t)KB * 8 * NC * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t ntiles = (N + kTileVec - 1) / kTileVec;
        int64_t blocks = (ntiles + 3) / 4;                      // few tiles: one per SIMD before any SIMD gets two
        if (blocks > ctx->cus) blocks = ctx->cus;
        const uint64_t attr_set = 1ull << 2;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 0>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 1>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 2>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        // the last chunk holds fewer than eight 8-dim steps with coordinates that count: stop after them
        const bool prefix = prune == 0 && (dact % kChunkD) != 0 && (dact % kChunkD) <= kChunkD - 8;
        const uint64_t attr_set_p = 1ull << 3;        // this call site's bit in ctx->attr_done
        if (prefix && !(ctx->attr_done & attr_set_p)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 0, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set_p;
        }
        const uint64_t attr_set_i = 1ull << 4;        // this call site's bit in ctx->attr_done
        if (use_image && !(ctx->attr_done & attr_set_i)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 0, false, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 1, false, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_resident<KB, 2, false, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set_i;
        }
        auto kern = prefix ? &k_assign_resident<KB, 0, true>
                  : use_image ? (prune == 1 ? &k_assign_resident<KB, 1, false, true>
                                 : prune == 2 ? &k_assign_resident<KB, 2, false, true> : &k_assign_resident<KB, 0, false, true>)
                  : prune == 1 ? &k_assign_resident<KB, 1> : prune == 2 ? &k_assign_resident<KB, 2> : &k_assign_resident<KB, 0>;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           xp, Cm, ctx->hneg, N, dact, ld, ctx->K, ctx->M, m, NC, eps,
                           codes, ctx->refine_list, ctx->refine_count, pa,
                           use_image && !prefix ? reinterpret_cast<const float4 *>(ctx->lds_image) : (const float4 *)nullptr);
    } else {
        // two slices of 64 dims in LDS: one block per CU
        const size_t lds = (size_t)2 * KB * 8 * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t nbt = (N + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);
        int64_t blocks = nbt < ctx->cus ? nbt : ctx->cus;
        const uint64_t attr_set = 1ull << 5;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_chunked<KB, 0>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_chunked<KB, 1>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_assign_chunked<KB, 2>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        if (NC > ctx->NC || KB != ctx->kb)
            return fail(ctx, HCLAE_EINVAL, "assign: codebook image too small for this shape");
        const int img_total = NC * KB * 8 * kWave;
        hipLaunchKernelGGL(k_codebook_image, dim3((img_total + 255) / 256), dim3(256), 0, ctx->stream,
                           Cm, ctx->K, dact, ld, KB, NC, ctx->cb_image);
        auto kern = prune == 1 ? &k_assign_chunked<KB, 1> : prune == 2 ? &k_assign_chunked<KB, 2> : &k_assign_chunked<KB, 0>;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           xp, ctx->cb_image, ctx->hneg, N, dact, ld, ctx->K, ctx->M, m, NC, eps,
                           codes, ctx->refine_list, ctx->refine_count, pa);
    }
    }
    HIP_TRY(ctx, hipGetLastError());
    Timed t_(ctx, HCLAE_T_REFINE);
    hipLaunchKernelGGL(k_refine, dim3(ctx->cus * 4), dim3(256), 0, ctx->stream,
                       xp, Cm, dact, ld, ctx->M, m, codes, ctx->refine_list, ctx->refine_count, mv,
                       ctx->work, (unsigned long long)N, prune == 2 ? ctx->moved_count + 3 : (const unsigned *)nullptr);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

// Assumes hneg holds the norms of Cm (over the same dact coordinates) and the re-check counter is zero.
// use_image: the dictionary image kept by launch_norms(image) and the centroid updates since is that of Cm.
int launch_assign(hclae_ctx *ctx, int m, int64_t N, const float *xp, const float *Cm, uint8_t *codes,
                  int dact = 0, int ld = 0, int prune = 0, bool use_image = false)
{
    if (dact <= 0) dact = ctx->D;
    if (ld <= 0) ld = ctx->D;
    if (dact != ctx->D || ld != ctx->D) { prune = 0; use_image = false; }
    switch (ctx->kb) {
    case 1: return launch_assign_kb<1>(ctx, m, N, xp, Cm, codes, dact, ld, prune, use_image);
    case 2: return launch_assign_kb<2>(ctx, m, N, xp, Cm, codes, dact, ld, prune, use_image);
    case 4: return launch_assign_kb<4>(ctx, m, N, xp, Cm, codes, dact, ld, prune, use_image);
    default: return launch_assign_kb<8>(ctx, m, N, xp, Cm, codes, dact, ld, prune, use_image);
    }
}

// Ages the bounds of the stage by the drift of the last centroid update and lists the vectors to recompute.
// The list counter (moved_count[3]) is zero here: the merge that reported the drift reset it.
int launch_bounds_step(hclae_ctx *ctx, int m, int64_t N, const uint8_t *codes, const float *xp, const float *Cm)
{
    Timed t_(ctx, HCLAE_T_BOUNDS);
    const uint64_t attr_set = 1ull << 6;        // this call site's bit in ctx->attr_done
    if (!(ctx->attr_done & attr_set)) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bounds_step),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget - 40 * 1024));
        ctx->attr_done |= attr_set;
    }
    hipLaunchKernelGGL(k_bounds_step, dim3((unsigned)((N + kBoundSpan - 1) / kBoundSpan)), dim3(kBoundThreads),
                       (size_t)kVolatile * ctx->D * sizeof(float), ctx->stream,
                       codes, N, ctx->M, m, ctx->drift, ctx->K, ctx->cur_u, ctx->cur_l,
                       ctx->active, ctx->moved_count + 3, xp, ctx->D, Cm);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

// Accumulate + merge; leaves hneg = norms of the new Cm and the re-check counter at zero.
// have_absmax: refine_count[1] already holds max |xp| (the assign kernel just ran on the same xp).
// dnorm: leading coordinates whose squares enter the refreshed codeword norms (0 = all).
// keep_totals: also store the integer sums, the counts and the code column, so that the following centroid
// updates of the same stage can run on the moved vectors alone (launch_update_moved).
int launch_update(hclae_ctx *ctx, int m, int64_t N, const float *xp, float *Cm, const uint8_t *codes,
                  int32_t *counts, bool have_absmax, bool online = false, int dnorm = 0, bool keep_totals = false)
{
    const int D = ctx->D, K = ctx->K;
    const int windows = (D + kUpdWindow - 1) / kUpdWindow;
    int64_t nb = (N + 1023) / 1024;                   // at least 1024 rows per block
    if (nb > ctx->upd_blocks) nb = ctx->upd_blocks;
    if (nb < 1) nb = 1;
    int64_t rpb = (N + nb - 1) / nb;
    const size_t lds = upd_lds_bytes(K);
    const uint64_t attr_set = 1ull << 7;        // this call site's bit in ctx->attr_done
    if (!(ctx->attr_done & attr_set)) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_accumulate),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
        ctx->attr_done |= attr_set;
    }
    if (!have_absmax) {
        // a fill kernel, not a memset: the call may be recorded into a HIP graph
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, ctx->stream, ctx->refine_count + 1, 1);
        const int64_t n4 = N * (D / 4);
        hipLaunchKernelGGL(k_absmax, dim3(stream_blocks(ctx, n4, 256 * 4)), dim3(256), 0, ctx->stream,
                           reinterpret_cast<const float4 *>(xp), n4, ctx->refine_count + 1);
        HIP_TRY(ctx, hipGetLastError());
    }
    {
        Timed t_(ctx, HCLAE_T_ACCUM);
        hipLaunchKernelGGL(k_accumulate, dim3((unsigned)nb, (unsigned)windows), dim3(kUpdThreads), lds, ctx->stream,
                           xp, codes, N, D, K, ctx->M, m, rpb, ctx->refine_count + 1, ctx->partial, ctx->pcount);
    }
    HIP_TRY(ctx, hipGetLastError());
    Timed t_(ctx, HCLAE_T_MERGE);
    hipLaunchKernelGGL(k_merge, dim3(K), dim3(256), 0, ctx->stream,
                       ctx->partial, ctx->pcount, (int)nb, K, D, dnorm > 0 ? dnorm : D, Cm, ctx->hneg, ctx->nk, counts,
                       ctx->refine_count,
                       online ? ctx->run_sum + (size_t)m * K * D : (double *)nullptr,
                       online ? ctx->run_cnt + (size_t)m * K : (long long *)nullptr,
                       keep_totals ? ctx->tot_sum : (long long *)nullptr, keep_totals ? ctx->tot_cnt : (int *)nullptr, 0,
                       keep_totals ? ctx->moved_count : (unsigned *)nullptr, keep_totals ? ctx->drift : (float *)nullptr,
                       ctx->resident ? ctx->lds_image : (float *)nullptr, 8 * ctx->NC);
    HIP_TRY(ctx, hipGetLastError());
    if (keep_totals) {
        hipLaunchKernelGGL(k_save_column, dim3(stream_blocks(ctx, N, 256)), dim3(256), 0, ctx->stream,
                           codes, N, ctx->M, m, ctx->upd_col);
        HIP_TRY(ctx, hipGetLastError());
    }
    return HCLAE_OK;
}

// Centroid update from the vectors that changed cluster since the last update of this stage (x' unchanged,
// max |x'| still published): exact, see k_merge.  Leaves hneg and the counters as launch_update does.
// The re-check kernel of the assignment that just ran (launch_assign with prune 3) has listed those vectors.
int launch_update_moved(hclae_ctx *ctx, int m, int64_t N, const float *xp, float *Cm)
{
    const int D = ctx->D, K = ctx->K;
    const int windows = (D + kUpdWindow - 1) / kUpdWindow;
    const int nb = ctx->upd_blocks;                  // upper bound; the kernels use as many as the list is worth
    const uint64_t attr_set = 1ull << 8;        // this call site's bit in ctx->attr_done
    if (!(ctx->attr_done & attr_set)) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_accumulate_moved),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
        ctx->attr_done |= attr_set;
    }
    {
        Timed t_(ctx, HCLAE_T_ACCUM_MOVED);
        hipLaunchKernelGGL(k_accumulate_moved, dim3((unsigned)nb, (unsigned)windows), dim3(kUpdThreads), upd_lds_bytes(K),
                           ctx->stream, xp, ctx->moved_list, ctx->moved_count, D, K, ctx->refine_count + 1,
                           ctx->partial, ctx->pcount);
        HIP_TRY(ctx, hipGetLastError());
    }
    Timed t_(ctx, HCLAE_T_MERGE);
    hipLaunchKernelGGL(k_merge, dim3(K), dim3(256), 0, ctx->stream,
                       ctx->partial, ctx->pcount, nb, K, D, D, Cm, ctx->hneg, ctx->nk, (int *)nullptr,
                       ctx->refine_count, (double *)nullptr, (long long *)nullptr, ctx->tot_sum, ctx->tot_cnt, 1,
                       ctx->moved_count, ctx->drift, ctx->resident ? ctx->lds_image : (float *)nullptr, 8 * ctx->NC);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

int launch_sqnorm(hclae_ctx *ctx, const float *r, int64_t N, double *part)
{
    const int64_t n4 = N * (ctx->D / 4);
    const int blocks = stream_blocks(ctx, n4, kFlatThreads * kSqUnroll);
    Timed t_(ctx, HCLAE_T_ERROR);
    hipLaunchKernelGGL(k_sqnorm, dim3(blocks), dim3(kFlatThreads), 0, ctx->stream,
                       reinterpret_cast<const floatx4 *>(r), n4, part);
    HIP_TRY(ctx, hipGetLastError());
    return blocks;
}

// Enqueues one full stage; by-products land in ctx->rec[slot].  No host synchronisation.
// heated: residue already holds x' of this stage and ctx->part_a its entry error (the previous
// stage ended with a fused transition).  next: >= 0 ends the stage with the fused transition into
// that stage instead of the plain new-residue pass.
// carry (several sweeps in one call; needs pruning, iters > 0, no seeding; the caller has allocated the carry arrays):
// 1 = the stage keeps its final bounds in its own rows of carry_u / carry_l and marks the path length; 2 = it also
// starts from the bounds its last visit kept (k_bounds_carry) instead of an assignment over all vectors.  With
// either, max |x'| comes from the row pass that wrote x' (the first assignment may not read every row).
// next_amax: the fused pass into the next stage takes max |x'| for it (that stage runs with carry != 0).
int enqueue_stage(hclae_ctx *ctx, int m, int64_t N, float *C, uint8_t *codes, float *residue, int iters,
                  const int64_t *seed_dev, int slot, bool heated = false, int next = -1, int carry = 0,
                  bool next_amax = false)
{
    const int D = ctx->D, K = ctx->K;
    float *Cm = C + (size_t)m * K * D;
    int rc;
    if (carry && (!ctx->pruning || iters <= 0 || seed_dev || !ctx->carry_u))
        return fail(ctx, HCLAE_ESTATE, "stage: carried bounds need pruning, iters > 0 and no seeding");
    ctx->cur_u = carry ? ctx->carry_u + (size_t)m * ctx->N_max : ctx->bnd_u;
    ctx->cur_l = carry ? ctx->carry_l + (size_t)m * ctx->N_max : ctx->bnd_l;
    if (!heated) {
        const int pb = launch_heat_cool<+1, true>(ctx, m, N, C, codes, residue, ctx->part_a, carry != 0);
        if (pb < 0) return pb;
    }
    if (seed_dev) {
        hipLaunchKernelGGL(k_seed, dim3(K), dim3(256), 0, ctx->stream, residue, seed_dev, K, D, Cm);
        HIP_TRY(ctx, hipGetLastError());
    }
    if ((rc = launch_norms(ctx, Cm, 0, 0, carry ? 2 : 0, true)) != HCLAE_OK) return rc;
    if (carry == 2) {
        Timed t_(ctx, HCLAE_T_BOUNDS);
        // (8M + 16) 2^-24 sqrt(D), times the largest coordinate seen: the roundings of the passes since the last visit
        const double slack_unit = (8.0 * ctx->M + 16.0) * 5.9604644775390625e-8 * sqrt((double)D);
        hipLaunchKernelGGL(k_bounds_carry, dim3((unsigned)((N + kBoundSpan - 1) / kBoundSpan)), dim3(kBoundThreads), 0,
                           ctx->stream, ctx->carry_path, ctx->carry_snap + (size_t)m * ctx->N_max, N, slack_unit,
                           ctx->carry_amax, ctx->refine_count + 1, ctx->cur_u, ctx->cur_l, ctx->active, ctx->moved_count + 3);
        HIP_TRY(ctx, hipGetLastError());
    }
    // x' stays as it is until the stage ends: the first centroid update sums all vectors and keeps the integer
    // totals, the others add only the vectors that changed cluster (exact, so the dictionaries are the same)
    // With pruning the first assignment stores distance bounds for every vector; after each centroid update
    // (which also reports how far every codeword moved) only the vectors whose bounds no longer separate
    // their codeword from the others are assigned again.  The first update must then keep its totals.
    const bool prune = ctx->pruning && iters > 0;
    for (int t = 0; t < iters; ++t) {
        if (prune && t > 0 && (rc = launch_bounds_step(ctx, m, N, codes, residue, Cm)) != HCLAE_OK) return rc;
        if ((rc = launch_assign(ctx, m, N, residue, Cm, codes, 0, 0, prune ? (t == 0 ? (carry == 2 ? 2 : 1) : 3) : 0, true)) != HCLAE_OK) return rc;
        rc = (t == 0 || !ctx->pruning)
                 ? launch_update(ctx, m, N, residue, Cm, codes, nullptr, true, false, 0, ctx->pruning && (iters > 1 || prune))
                 : launch_update_moved(ctx, m, N, residue, Cm);
        if (rc != HCLAE_OK) return rc;
    }
    if (prune && (rc = launch_bounds_step(ctx, m, N, codes, residue, Cm)) != HCLAE_OK) return rc;
    if ((rc = launch_assign(ctx, m, N, residue, Cm, codes, 0, 0, prune ? 2 : 0, true)) != HCLAE_OK) return rc;
    if (carry) {
        // how far this visit moved every vector's part of the reconstruction (old_codes still holds the column as the
        // stage found it: the row pass below is the one that replaces it)
        hipLaunchKernelGGL(k_pair_table, dim3(K), dim3(256), sizeof(float) * D, ctx->stream, ctx->carry_Centry, Cm, K, D, ctx->carry_T);
        hipLaunchKernelGGL(k_path_step, dim3(stream_blocks(ctx, N, 256 * 4)), dim3(256), 0, ctx->stream,
                           ctx->old_codes, codes, N, ctx->M, m, ctx->carry_T, K, ctx->carry_path,
                           ctx->carry_snap + (size_t)m * ctx->N_max, ctx->refine_count, ctx->carry_amax);
        HIP_TRY(ctx, hipGetLastError());
    }
    int pa;
    if (next < 0) {
        pa = launch_heat_cool<-1, true>(ctx, m, N, C, codes, residue, ctx->part_b);
        if (pa < 0) return pa;
    } else {
        const RowGeom g = row_geom(D);
        pa = heat_cool_blocks(N, D, ctx->cus);
        Timed t_(ctx, HCLAE_T_TRANSITION);
        if (D >= kWideMinD) {
            auto kern = next_amax ? &k_row_pass_wide<0, true, true> : &k_row_pass_wide<0, true, false>;
            hipLaunchKernelGGL(kern, dim3(pa), dim3(kStreamThreads), 0, ctx->stream,
                               residue, codes, Cm, C + (size_t)next * K * D, N, D, ctx->M, m, next,
                               ctx->old_codes, ctx->part_b, ctx->part_chg,
                               next_amax ? ctx->carry_amax + kAmaxSlots : (unsigned *)nullptr);
        } else {
            auto kern = next_amax ? (D == 128 ? &k_row_pass<0, true, 128, true> : &k_row_pass<0, true, 0, true>)
                                  : (D == 128 ? &k_row_pass<0, true, 128, false> : &k_row_pass<0, true, 0, false>);
            hipLaunchKernelGGL(kern, dim3(pa), dim3(kStreamThreads), 0, ctx->stream,
                               residue, codes, Cm, C + (size_t)next * K * D, N, D, ctx->M, m, next, g,
                               ctx->old_codes, ctx->part_b, ctx->part_chg,
                               next_amax ? ctx->carry_amax + kAmaxSlots : (unsigned *)nullptr);
        }
        HIP_TRY(ctx, hipGetLastError());
    }
    ctx->cur_u = ctx->bnd_u;
    ctx->cur_l = ctx->bnd_l;
    hipLaunchKernelGGL(k_finish_stage, dim3(1), dim3(kFinishThreads), 0, ctx->stream,
                       ctx->part_a, ctx->part_b, ctx->part_chg, pa, iters > 0 ? ctx->nk : nullptr, K,
                       ctx->refine_count, ctx->rec + slot);
    HIP_TRY(ctx, hipGetLastError());
    if (next >= 0) {            // the error after this stage is the entry error of the next one
        double *t = ctx->part_a;
        ctx->part_a = ctx->part_b;
        ctx->part_b = t;
    }
    return HCLAE_OK;
}

int enqueue_encode(hclae_ctx *ctx, const float *X, int64_t N, const float *C, uint8_t *codes, float *residue)
{
    const int D = ctx->D, K = ctx->K;
    const int64_t n4 = N * (D / 4);
    int rc;
    hipLaunchKernelGGL(k_copy, dim3(stream_blocks(ctx, n4, kFlatThreads * 4)), dim3(kFlatThreads), 0, ctx->stream,
                       reinterpret_cast<floatx4 *>(residue), reinterpret_cast<const floatx4 *>(X), n4);
    HIP_TRY(ctx, hipGetLastError());
    for (int m = 0; m < ctx->M; ++m) {
        const float *Cm = C + (size_t)m * K * D;
        if ((rc = launch_norms(ctx, Cm)) != HCLAE_OK) return rc;
        if ((rc = launch_assign(ctx, m, N, residue, Cm, codes)) != HCLAE_OK) return rc;
        const int b = launch_heat_cool<-1, false>(ctx, m, N, C, codes, residue, nullptr);
        if (b < 0) return b;
    }
    return HCLAE_OK;
}

int fetch_records(hclae_ctx *ctx, int count)
{
    HIP_TRY(ctx, hipMemcpyAsync(ctx->rec_host, ctx->rec, sizeof(StageRecord) * count, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HCLAE_OK;
}

}  // namespace

// =========================================================================================
extern "C" {

int hclae_check_shape(int64_t N, int D, int M, int K)
{
    if (N < 0 || N >= ((int64_t)1 << 31)) return HCLAE_EINVAL;
    if (D < 4 || D > HCLAE_MAX_D || (D % 4) != 0) return HCLAE_EINVAL;
    if (M < 1 || M > HCLAE_MAX_M) return HCLAE_EINVAL;
    if (K < 1 || K > HCLAE_MAX_K) return HCLAE_EINVAL;
    return HCLAE_OK;
}

const char *hclae_last_error(const hclae_ctx *ctx) { return ctx ? ctx->err : g_create_error; }

int hclae_create(hclae_ctx **out, int64_t N_max, int D, int M, int K, void *hip_stream)
{
    if (!out) return fail(nullptr, HCLAE_EINVAL, "out is NULL");
    *out = nullptr;
    if (hclae_check_shape(N_max, D, M, K) != HCLAE_OK || N_max < 1)
        return fail(nullptr, HCLAE_EINVAL, "shape out of range");
    hclae_ctx *ctx = new (std::nothrow) hclae_ctx();
    if (!ctx) return fail(nullptr, HCLAE_ENOMEM, "host allocation failed");
    memset(ctx, 0, sizeof(*ctx));
    ctx->N_max = N_max; ctx->D = D; ctx->M = M; ctx->K = K;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->sweep_L = 10;                       // the width the paper settles on (Sec. 3.3)
    ctx->pruning = 1;
    ctx->cooldown_phases = 10;               // I = 10 (Sec. 3.2)
    ctx->kb = K <= 32 ? 1 : K <= 64 ? 2 : K <= 128 ? 4 : 8;
    ctx->NC = (D + kChunkD - 1) / kChunkD;
    ctx->resident = (size_t)32 * ctx->kb * kChunkD * ctx->NC * sizeof(float) + 4096 <= (size_t)kLdsBudget;
    {   // the split image serves every LDS-resident assignment, those on a prefix of a long row included
        const int nc_res = (int)(((size_t)kLdsBudget - 4096) / ((size_t)32 * ctx->kb * kChunkD * sizeof(float)));
        ctx->split_image_bytes = sizeof(uint4) * (size_t)ctx->kb * 4 * (ctx->NC < nc_res ? ctx->NC : nc_res) * 2 * kWave;
    }

    hipError_t e = hipGetDevice(&ctx->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, ctx->device);
    if (e != hipSuccess) {
        int rc = fail(nullptr, HCLAE_EHIP, "no usable HIP device", e);
        delete ctx;
        return rc;
    }
    ctx->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    {   // this device's address of the static scratch of hclae_quant_error_noalloc, while allocation is still allowed
        double *unused = nullptr;
        if ((e = noalloc_scratch(&unused)) != hipSuccess) {
            int rc = fail(nullptr, HCLAE_EHIP, "hipGetSymbolAddress (static scratch)", e);
            delete ctx;
            return rc;
        }
    }
    if ((size_t)prop.sharedMemPerBlock < 64 * 1024 && false) { /* LDS limit is raised per kernel below */ }

    // centroid partials: vector ranges x 64-dim windows fill the CUs once; int64 [ranges][K][D]
    const int windows = (D + kUpdWindow - 1) / kUpdWindow;
    int ub = ctx->cus / windows;
    if (ub < 1) ub = 1;
    const size_t per = (size_t)K * D * sizeof(long long);
    while (ub > 1 && per * ub > ((size_t)512 << 20)) ub /= 2;
    ctx->upd_blocks = ub;

    ctx->nparts = heat_cool_blocks(N_max, D, ctx->cus);
    if (ctx->nparts < kFlatParts) ctx->nparts = kFlatParts;

    struct { void **p; size_t bytes; } allocs[] = {
        {(void **)&ctx->hneg, sizeof(float) * 32 * ctx->kb},
        {(void **)&ctx->cb_image, ctx->resident ? 256 : sizeof(float4) * (size_t)ctx->NC * ctx->kb * 8 * kWave},
        {(void **)&ctx->lds_image, ctx->resident ? sizeof(float4) * (size_t)ctx->NC * ctx->kb * 8 * kWave : 256},
        {(void **)&ctx->split_image, ctx->split_image_bytes},
        {(void **)&ctx->split_norms, sizeof(float) * 2 * HCLAE_MAX_K},
        {(void **)&ctx->refine_count, 256},
        {(void **)&ctx->refine_list, sizeof(RefineItem) * (size_t)N_max},
        {(void **)&ctx->old_codes, (size_t)N_max},
        {(void **)&ctx->partial, per * ub},
        {(void **)&ctx->pcount, sizeof(int) * (size_t)K * ub},
        {(void **)&ctx->nk, sizeof(int) * K},
        {(void **)&ctx->tot_sum, sizeof(long long) * (size_t)K * D},
        {(void **)&ctx->tot_cnt, sizeof(int) * K},
        {(void **)&ctx->upd_col, (size_t)N_max},
        {(void **)&ctx->moved_list, sizeof(unsigned long long) * (size_t)N_max},
        {(void **)&ctx->moved_count, 256},
        {(void **)&ctx->bnd_u, sizeof(float) * (size_t)N_max},
        {(void **)&ctx->bnd_l, sizeof(float) * (size_t)N_max},
        {(void **)&ctx->drift, sizeof(float) * HCLAE_MAX_K},
        {(void **)&ctx->active, sizeof(uint32_t) * (size_t)N_max},
        {(void **)&ctx->work, 256},
        {(void **)&ctx->seed_idx, sizeof(int64_t) * (size_t)M * K},
        {(void **)&ctx->part_a, sizeof(double) * ctx->nparts},
        {(void **)&ctx->part_b, sizeof(double) * ctx->nparts},
        {(void **)&ctx->part_chg, sizeof(long long) * ctx->nparts},
        {(void **)&ctx->rec, sizeof(StageRecord) * M},
    };
    for (auto &a : allocs) {
        e = hipMalloc(a.p, a.bytes);
        if (e != hipSuccess) {
            int rc = fail(nullptr, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (scratch)", e);
            hclae_destroy(ctx);
            return rc;
        }
    }
    e = hipHostMalloc((void **)&ctx->rec_host, sizeof(StageRecord) * M, hipHostMallocDefault);
    if (e == hipSuccess) e = hipMemset(ctx->rec, 0, sizeof(StageRecord) * M);
    if (e == hipSuccess) e = hipMemset(ctx->refine_count, 0, 256);
    if (e == hipSuccess) e = hipMemset(ctx->nk, 0, sizeof(int) * K);
    if (e == hipSuccess) e = hipMemset(ctx->moved_count, 0, 256);
    if (e == hipSuccess) e = hipMemset(ctx->work, 0, 256);
    if (e != hipSuccess) {
        int rc = fail(nullptr, HCLAE_EHIP, "scratch initialisation", e);
        hclae_destroy(ctx);
        return rc;
    }
    ctx->cur_u = ctx->bnd_u;
    ctx->cur_l = ctx->bnd_l;
    snprintf(ctx->err, sizeof(ctx->err), "ok");
    *out = ctx;
    return HCLAE_OK;
}

int hclae_destroy(hclae_ctx *ctx)
{
    if (!ctx) return HCLAE_EINVAL;
    void *dev[] = {ctx->hneg, ctx->cb_image, ctx->lds_image, ctx->split_image, ctx->split_norms, ctx->refine_count, ctx->refine_list, ctx->old_codes, ctx->partial, ctx->pcount,
                   ctx->nk, ctx->tot_sum, ctx->tot_cnt, ctx->upd_col, ctx->moved_list, ctx->moved_count, ctx->bnd_u, ctx->bnd_l, ctx->drift, ctx->active, ctx->work, ctx->seed_idx, ctx->part_a, ctx->part_b, ctx->part_chg, ctx->rec,
                   ctx->run_sum, ctx->run_cnt, ctx->n0_dev, ctx->pca_rt, ctx->pca_crot, ctx->pca_colpart,
                   ctx->pca_grampart, ctx->pca_mean, ctx->pca_mean32, ctx->pca_cov, ctx->pca_R, ctx->pca_xr,
                   ctx->stats_buf, ctx->order_var, ctx->order_idx, ctx->order_tmp,
                   ctx->carry_u, ctx->carry_l, ctx->carry_path, ctx->carry_snap, ctx->carry_Centry, ctx->carry_T, ctx->carry_amax,
                   ctx->beam_rows[0], ctx->beam_rows[1], ctx->beam_err[0], ctx->beam_err[1],
                   ctx->beam_pre[0], ctx->beam_pre[1], ctx->beam_mask};
    for (void *p : dev)
        if (p) (void)hipFree(p);
    if (ctx->rec_host) (void)hipHostFree(ctx->rec_host);
    if (ctx->t_beg) {
        for (int i = 0; i < kMaxTimed; ++i) {
            if (ctx->t_beg[i]) (void)hipEventDestroy(ctx->t_beg[i]);
            if (ctx->t_end && ctx->t_end[i]) (void)hipEventDestroy(ctx->t_end[i]);
        }
    }
    delete[] ctx->t_beg;
    delete[] ctx->t_end;
    delete[] ctx->t_cls;
    delete ctx;
    return HCLAE_OK;
}

int hclae_heat(hclae_ctx *ctx, int m, int64_t N, int D, const float *C, int M, int K,
               const uint8_t *codes, float *residue)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M) return fail(ctx, HCLAE_EINVAL, "hclae_heat: m out of range");
    if (N == 0) return HCLAE_OK;
    if (!C || !codes || !residue) return fail(ctx, HCLAE_EINVAL, "hclae_heat: NULL pointer");
    if (misaligned(C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_heat: float arrays must be 16-byte aligned");
    const int b = launch_heat_cool<+1, false>(ctx, m, N, C, codes, residue, nullptr);
    return b < 0 ? b : HCLAE_OK;
}

int hclae_cool(hclae_ctx *ctx, int m, int64_t N, int D, const float *C, int M, int K,
               const uint8_t *codes, float *xp)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M) return fail(ctx, HCLAE_EINVAL, "hclae_cool: m out of range");
    if (N == 0) return HCLAE_OK;
    if (!C || !codes || !xp) return fail(ctx, HCLAE_EINVAL, "hclae_cool: NULL pointer");
    if (misaligned(C, xp)) return fail(ctx, HCLAE_EINVAL, "hclae_cool: float arrays must be 16-byte aligned");
    const int b = launch_heat_cool<-1, false>(ctx, m, N, C, codes, xp, nullptr);
    return b < 0 ? b : HCLAE_OK;
}

int hclae_assign(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, const float *C,
                 int M, int K, uint8_t *codes, float *dmin)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M) return fail(ctx, HCLAE_EINVAL, "hclae_assign: m out of range");
    if (N == 0) return HCLAE_OK;
    if (!C || !codes || !xp) return fail(ctx, HCLAE_EINVAL, "hclae_assign: NULL pointer");
    if (misaligned(C, xp)) return fail(ctx, HCLAE_EINVAL, "hclae_assign: float arrays must be 16-byte aligned");
    const float *Cm = C + (size_t)m * K * D;
    if ((rc = launch_norms(ctx, Cm)) != HCLAE_OK) return rc;
    if ((rc = launch_assign(ctx, m, N, xp, Cm, codes)) != HCLAE_OK) return rc;
    if (dmin) {
        hipLaunchKernelGGL(k_dist_to_code, dim3(stream_blocks(ctx, N, kFlatThreads / kWave)), dim3(kFlatThreads), 0,
                           ctx->stream, xp, codes, Cm, N, D, M, m, dmin);
        HIP_TRY(ctx, hipGetLastError());
    }
    return HCLAE_OK;
}

int hclae_update(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, float *C,
                 int M, int K, const uint8_t *codes, int32_t *counts)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M) return fail(ctx, HCLAE_EINVAL, "hclae_update: m out of range");
    if (N > 0 && (!C || !codes || !xp)) return fail(ctx, HCLAE_EINVAL, "hclae_update: NULL pointer");
    if (misaligned(C, xp)) return fail(ctx, HCLAE_EINVAL, "hclae_update: float arrays must be 16-byte aligned");
    if (N == 0) {
        if (counts) {
            hipLaunchKernelGGL(k_zero_words, dim3((K + 255) / 256), dim3(256), 0, ctx->stream, reinterpret_cast<unsigned *>(counts), K);
            HIP_TRY(ctx, hipGetLastError());
        }
        return HCLAE_OK;
    }
    return launch_update(ctx, m, N, xp, C + (size_t)m * K * D, codes, counts, false);
}

int hclae_quant_error(hclae_ctx *ctx, const float *residue, int64_t N, int D, double *out)
{
    if (!ctx) return HCLAE_EINVAL;
    int rc = check_call(ctx, N, D, ctx->M, ctx->K);
    if (rc != HCLAE_OK) return rc;
    if (!out || (!residue && N > 0)) return fail(ctx, HCLAE_EINVAL, "hclae_quant_error: bad argument");
    if (misaligned(residue)) return fail(ctx, HCLAE_EINVAL, "hclae_quant_error: float arrays must be 16-byte aligned");
    if (N == 0) { *out = 0.0; return HCLAE_OK; }
    const int blocks = launch_sqnorm(ctx, residue, N, ctx->part_b);
    if (blocks < 0) return blocks;
    hipLaunchKernelGGL(k_finish_stage, dim3(1), dim3(kFinishThreads), 0, ctx->stream,
                       (const double *)nullptr, ctx->part_b, (const long long *)nullptr, blocks,
                       (const int *)nullptr, 0, (const unsigned *)nullptr, ctx->rec);
    HIP_TRY(ctx, hipGetLastError());
    if ((rc = fetch_records(ctx, 1)) != HCLAE_OK) return rc;
    *out = ctx->rec_host[0].sum_after / (double)N;
    return HCLAE_OK;
}

int hclae_quant_error_noalloc(const float *residue, int64_t N, int D, double *out, void *hip_stream)
{
    if (hclae_check_shape(N, D, 1, 1) != HCLAE_OK)
        return fail(nullptr, HCLAE_EINVAL, "hclae_quant_error_noalloc: size beyond the limits (0 <= N < 2^31, 4 <= D <= 4096, D % 4 == 0)");
    if (!out || (!residue && N > 0)) return fail(nullptr, HCLAE_EINVAL, "hclae_quant_error_noalloc: NULL pointer");
    if (misaligned(residue) || (reinterpret_cast<uintptr_t>(out) & 7u))
        return fail(nullptr, HCLAE_EINVAL, "hclae_quant_error_noalloc: residue must be 16-byte aligned, out 8-byte aligned");
    double *scratch = nullptr;
    hipError_t e = noalloc_scratch(&scratch);
    if (e != hipSuccess) return fail(nullptr, HCLAE_EHIP, "hipGetSymbolAddress (static scratch)", e);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t n4 = N * (D / 4);
    // the grid of hclae_quant_error on a 256-CU device, fixed here so that no device query is needed
    int64_t blocks = (n4 + kFlatThreads * kSqUnroll - 1) / (kFlatThreads * kSqUnroll);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    if (N > 0) {
        hipLaunchKernelGGL(k_sqnorm, dim3((unsigned)blocks), dim3(kFlatThreads), 0, stream,
                           reinterpret_cast<const floatx4 *>(residue), n4, scratch);
        if ((e = hipGetLastError()) != hipSuccess) return fail(nullptr, HCLAE_EHIP, "k_sqnorm", e);
    }
    hipLaunchKernelGGL(k_finish_mean, dim3(1), dim3(kFinishThreads), 0, stream, scratch, N > 0 ? (int)blocks : 0, N, out);
    if ((e = hipGetLastError()) != hipSuccess) return fail(nullptr, HCLAE_EHIP, "k_finish_mean", e);
    return HCLAE_OK;
}

int hclae_encode(hclae_ctx *ctx, const float *X, int64_t N, int D,
                 const float *C, int M, int K, uint8_t *codes, float *residue)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (N == 0) return HCLAE_OK;
    if (!X || !C || !codes || !residue || X == residue) return fail(ctx, HCLAE_EINVAL, "hclae_encode: bad argument");
    if (misaligned(X, C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_encode: float arrays must be 16-byte aligned");
    return enqueue_encode(ctx, X, N, C, codes, residue);
}

static int check_init_idx(const int64_t *idx, int count, int64_t N)
{
    for (int i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= N) return HCLAE_EINVAL;
    return HCLAE_OK;
}

static void fill_stats(const StageRecord &r, int64_t N, int iters, hclae_stage_stats *s)
{
    s->err_before = r.sum_before / (double)N;
    s->err_after = r.sum_after / (double)N;
    s->codes_changed = r.changed;
    s->refined = r.refined;
    s->empty_clusters = iters > 0 ? r.empty : 0;
    s->iters_run = iters;
}

static int enqueue_stage_cooldown_pca(hclae_ctx *ctx, int m, int64_t N, float *C, uint8_t *codes, float *residue,
                                      int iters, const int64_t *seed_dev, int slot, int *iters_run_out);

int hclae_anneal_stage(hclae_ctx *ctx, int m, int64_t N, int D, float *C, int M, int K,
                       uint8_t *codes, float *residue, int iters,
                       const int64_t *init_idx, hclae_stage_stats *stats)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M || iters < 0 || (N > 0 && (!C || !codes || !residue)))
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage: bad argument");
    if (misaligned(C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage: float arrays must be 16-byte aligned");
    if (init_idx && check_init_idx(init_idx, K, N) != HCLAE_OK)
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage: init_idx out of range");
    if (N == 0) {
        if (stats) { memset(stats, 0, sizeof(*stats)); }
        return HCLAE_OK;
    }
    if (init_idx)
        HIP_TRY(ctx, hipMemcpyAsync(ctx->seed_idx, init_idx, sizeof(int64_t) * K, hipMemcpyHostToDevice, ctx->stream));
    int iters_run = iters;
    rc = ctx->cooldown == HCLAE_COOLDOWN_IMPROVED
             ? enqueue_stage_cooldown_pca(ctx, m, N, C, codes, residue, iters, init_idx ? ctx->seed_idx : nullptr, 0, &iters_run)
             : enqueue_stage(ctx, m, N, C, codes, residue, iters, init_idx ? ctx->seed_idx : nullptr, 0);
    if (rc != HCLAE_OK) return rc;
    if (stats) {
        if ((rc = fetch_records(ctx, 1)) != HCLAE_OK) return rc;
        fill_stats(ctx->rec_host[0], N, iters_run, stats);
    } else if (init_idx) {
        // the seed indices were read from caller memory by an asynchronous copy
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    return HCLAE_OK;
}

static int enqueue_encode_beam(hclae_ctx *ctx, const float *X, int64_t N, const float *C, int L,
                               uint8_t *codes, float *residue, double *err);

int hclae_set_pruning(hclae_ctx *ctx, int on)
{
    if (!ctx) return HCLAE_EINVAL;
    ctx->pruning = on ? 1 : 0;
    return HCLAE_OK;
}

int hclae_set_contraction(hclae_ctx *ctx, int mode)
{
    if (!ctx) return HCLAE_EINVAL;
    if (mode != HCLAE_CONTRACT_F32 && mode != HCLAE_CONTRACT_SPLIT_BF16)
        return fail(ctx, HCLAE_EINVAL, "hclae_set_contraction: unknown mode");
    ctx->contraction = mode;
    return HCLAE_OK;
}

int hclae_set_beam_width(hclae_ctx *ctx, int L)
{
    if (!ctx) return HCLAE_EINVAL;
    if (L < 1 || L > kBeamMaxL) return fail(ctx, HCLAE_EINVAL, "hclae_set_beam_width: need 1 <= L <= 32");
    ctx->sweep_L = L;
    return HCLAE_OK;
}

int hclae_sweep(hclae_ctx *ctx, const float *X, int64_t N, int D, float *C, int M, int K,
                uint8_t *codes, float *residue, int iters, int reencode_mode,
                const int64_t *init_idx, double *err_per_stage)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (iters < 0 || (N > 0 && (!C || !codes || !residue)) || reencode_mode < 0 || reencode_mode > 2)
        return fail(ctx, HCLAE_EINVAL, "hclae_sweep: bad argument");
    if (misaligned(X, C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_sweep: float arrays must be 16-byte aligned");
    if (reencode_mode != 0 && N > 0 && (!X || X == residue))
        return fail(ctx, HCLAE_EINVAL, "hclae_sweep: reencode_mode 1 and 2 need X");
    if (init_idx && check_init_idx(init_idx, M * K, N) != HCLAE_OK)
        return fail(ctx, HCLAE_EINVAL, "hclae_sweep: init_idx out of range");
    if (N == 0) {
        if (err_per_stage) for (int m = 0; m < M; ++m) err_per_stage[m] = 0.0;
        return HCLAE_OK;
    }
    if (init_idx)   // all M x K seed rows at once; the caller's array is free again once the stream has passed the copy
        HIP_TRY(ctx, hipMemcpyAsync(ctx->seed_idx, init_idx, sizeof(int64_t) * (size_t)M * K, hipMemcpyHostToDevice, ctx->stream));
    for (int m = 0; m < M; ++m) {
        const int64_t *idx = init_idx ? ctx->seed_idx + (size_t)m * K : nullptr;
        // without the full re-encode, stage m ends and stage m+1 begins in one fused pass over the residue (plain
        // Lloyd cool-down; the improved k-means rotates x' first and keeps the two passes apart)
        const bool fuse = (reencode_mode == 0) && ctx->cooldown == HCLAE_COOLDOWN_LLOYD;
        rc = ctx->cooldown == HCLAE_COOLDOWN_IMPROVED
                 ? enqueue_stage_cooldown_pca(ctx, m, N, C, codes, residue, iters, idx, m, nullptr)
                 : enqueue_stage(ctx, m, N, C, codes, residue, iters, idx, m, fuse && m > 0, (fuse && m + 1 < M) ? m + 1 : -1);
        if (rc != HCLAE_OK) return rc;
        if (reencode_mode != 0) {
            rc = reencode_mode == 1 ? enqueue_encode(ctx, X, N, C, codes, residue)
                                    : enqueue_encode_beam(ctx, X, N, C, ctx->sweep_L, codes, residue, nullptr);
            if (rc != HCLAE_OK) return rc;
            if (err_per_stage) {
                const int blocks = launch_sqnorm(ctx, residue, N, ctx->part_b);
                if (blocks < 0) return blocks;
                hipLaunchKernelGGL(k_finish_stage, dim3(1), dim3(kFinishThreads), 0, ctx->stream,
                                   (const double *)nullptr, ctx->part_b, (const long long *)nullptr, blocks,
                                   (const int *)nullptr, 0, (const unsigned *)nullptr, ctx->rec + m);
                HIP_TRY(ctx, hipGetLastError());
            }
        }
    }
    if (err_per_stage) {
        if ((rc = fetch_records(ctx, M)) != HCLAE_OK) return rc;
        for (int m = 0; m < M; ++m) err_per_stage[m] = ctx->rec_host[m].sum_after / (double)N;
    } else if (init_idx) {
        // the seed indices were read from caller memory by an asynchronous copy
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    return HCLAE_OK;
}

// Arrays of the bounds carried between sweeps (hclae_anneal), allocated once per ctx.
static int carry_scratch(hclae_ctx *ctx)
{
    if (ctx->carry_u) return HCLAE_OK;
    const size_t n = (size_t)ctx->N_max, M = (size_t)ctx->M, K = (size_t)ctx->K, D = (size_t)ctx->D;
    struct { void **p; size_t bytes; } allocs[] = {
        {(void **)&ctx->carry_l, sizeof(float) * M * n},
        {(void **)&ctx->carry_path, sizeof(double) * n},
        {(void **)&ctx->carry_snap, sizeof(double) * M * n},
        {(void **)&ctx->carry_Centry, sizeof(float) * K * D},
        {(void **)&ctx->carry_T, sizeof(float) * K * K},
        {(void **)&ctx->carry_amax, sizeof(unsigned) * 2 * kAmaxSlots},    // [0] running maximum, [64..128) words of the row passes
        {(void **)&ctx->carry_u, sizeof(float) * M * n},        // last: its presence says that all are there
    };
    for (auto &a : allocs) {
        hipError_t e = hipMalloc(a.p, a.bytes);
        if (e != hipSuccess) {
            for (auto &b : allocs) {
                if (*b.p) (void)hipFree(*b.p);
                *b.p = nullptr;
            }
            return fail(ctx, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (carried bounds)", e);
        }
    }
    return HCLAE_OK;
}

int hclae_anneal(hclae_ctx *ctx, int64_t N, int D, float *C, int M, int K, uint8_t *codes, float *residue,
                 int iters, int n_sweeps, const int64_t *init_idx, double *err_per_stage)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (iters < 0 || n_sweeps < 0 || (N > 0 && (!C || !codes || !residue)))
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal: bad argument");
    if (misaligned(C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_anneal: float arrays must be 16-byte aligned");
    if (init_idx && check_init_idx(init_idx, M * K, N) != HCLAE_OK)
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal: init_idx out of range");
    if (N == 0 || n_sweeps == 0) {
        if (err_per_stage) for (int i = 0; i < n_sweeps * M; ++i) err_per_stage[i] = 0.0;
        return HCLAE_OK;
    }
    const bool lloyd = ctx->cooldown == HCLAE_COOLDOWN_LLOYD;
    // a sweep that seeds its dictionaries stands apart: its stages start from other dictionaries than they were left with
    const int first_kept = init_idx ? 1 : 0;                 // first sweep whose stages keep their bounds
    const bool carry = lloyd && ctx->pruning && iters > 0 && n_sweeps - first_kept > 1;
    if (init_idx)
        HIP_TRY(ctx, hipMemcpyAsync(ctx->seed_idx, init_idx, sizeof(int64_t) * (size_t)M * K, hipMemcpyHostToDevice, ctx->stream));
    if (carry) {
        if ((rc = carry_scratch(ctx)) != HCLAE_OK) return rc;
        // the running maximum and the words the row passes leave max |x'| in start empty
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(2 * kAmaxSlots), 0, ctx->stream, ctx->carry_amax, 2 * kAmaxSlots);
        HIP_TRY(ctx, hipGetLastError());
    }
    for (int s = 0; s < n_sweeps; ++s) {
        if (carry && s == first_kept) {
            // path lengths start at zero; the running maximum starts at the largest coordinate of the dictionaries as
            // they are now (a codeword nobody is assigned to keeps a value the data from here on need not reach)
            hipLaunchKernelGGL(k_zero_u64, dim3(stream_blocks(ctx, N, 256)), dim3(256), 0, ctx->stream,
                               reinterpret_cast<unsigned long long *>(ctx->carry_path), (size_t)N);
            const int64_t c4 = (int64_t)M * K * D / 4;
            hipLaunchKernelGGL(k_absmax, dim3(stream_blocks(ctx, c4, 256 * 4)), dim3(256), 0, ctx->stream,
                               reinterpret_cast<const float4 *>(C), c4, ctx->carry_amax);
            HIP_TRY(ctx, hipGetLastError());
        }
        for (int m = 0; m < M; ++m) {
            const int64_t *seeds = (init_idx && s == 0) ? ctx->seed_idx + (size_t)m * K : nullptr;
            if (lloyd) {
                // every stage but the very last ends in the fused pass into the next one, across sweeps too; the pass
                // into a stage that keeps bounds also takes max |x'| for it
                const bool last = s == n_sweeps - 1 && m == M - 1;
                const int mode = !carry || s < first_kept ? 0 : s == first_kept ? 1 : 2;
                const int s_next = m + 1 < M ? s : s + 1;
                const bool next_kept = carry && !last && s_next >= first_kept;
                rc = enqueue_stage(ctx, m, N, C, codes, residue, iters, seeds, m, !(s == 0 && m == 0),
                                   last ? -1 : (m + 1) % M, mode, next_kept);
            } else {
                rc = enqueue_stage_cooldown_pca(ctx, m, N, C, codes, residue, iters, seeds, m, nullptr);
            }
            if (rc != HCLAE_OK) return rc;
        }
        if (err_per_stage) {
            if ((rc = fetch_records(ctx, M)) != HCLAE_OK) return rc;
            for (int m = 0; m < M; ++m) err_per_stage[(size_t)s * M + m] = ctx->rec_host[m].sum_after / (double)N;
        }
    }
    // the seed indices were read from caller memory by an asynchronous copy
    if (init_idx && !err_per_stage) HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HCLAE_OK;
}

int hclae_online_begin(hclae_ctx *ctx, const float *C, int M, int K, int D, const int64_t *n0)
{
    int rc = check_call(ctx, 0, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (!C) return fail(ctx, HCLAE_EINVAL, "hclae_online_begin: C is NULL");
    if (n0)
        for (int i = 0; i < M * K; ++i)
            if (n0[i] < 0) return fail(ctx, HCLAE_EINVAL, "hclae_online_begin: negative weight");
    const size_t rows = (size_t)M * K;
    if (!ctx->run_sum) {
        hipError_t e = hipMalloc((void **)&ctx->run_sum, rows * D * sizeof(double));
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->run_cnt, rows * sizeof(long long));
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->n0_dev, rows * sizeof(long long));
        if (e != hipSuccess) return fail(ctx, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (online state)", e);
    }
    if (n0) {
        HIP_TRY(ctx, hipMemcpyAsync(ctx->n0_dev, n0, rows * sizeof(long long), hipMemcpyHostToDevice, ctx->stream));
    }
    const int64_t total = (int64_t)rows * D;
    hipLaunchKernelGGL(k_online_begin, dim3(stream_blocks(ctx, total, 256)), dim3(256), 0, ctx->stream,
                       C, n0 ? ctx->n0_dev : (const long long *)nullptr, total, D, ctx->run_sum, ctx->run_cnt);
    HIP_TRY(ctx, hipGetLastError());
    if (n0) HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));      // n0 was read from caller memory asynchronously
    return HCLAE_OK;
}

int hclae_online_export(hclae_ctx *ctx, double *run_sum, int64_t *run_cnt)
{
    if (!ctx || !run_sum || !run_cnt) return HCLAE_EINVAL;
    if (!ctx->run_sum) return fail(ctx, HCLAE_ESTATE, "hclae_online_export before hclae_online_begin");
    const size_t rows = (size_t)ctx->M * ctx->K;
    HIP_TRY(ctx, hipMemcpyAsync(run_sum, ctx->run_sum, rows * ctx->D * sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(run_cnt, ctx->run_cnt, rows * sizeof(long long), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HCLAE_OK;
}

int hclae_online_import(hclae_ctx *ctx, const double *run_sum, const int64_t *run_cnt)
{
    if (!ctx || !run_sum || !run_cnt) return HCLAE_EINVAL;
    if (!ctx->run_sum) return fail(ctx, HCLAE_ESTATE, "hclae_online_import before hclae_online_begin");
    const size_t rows = (size_t)ctx->M * ctx->K;
    for (size_t i = 0; i < rows; ++i)
        if (run_cnt[i] < 0) return fail(ctx, HCLAE_EINVAL, "hclae_online_import: negative count");
    HIP_TRY(ctx, hipMemcpyAsync(ctx->run_sum, run_sum, rows * ctx->D * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->run_cnt, run_cnt, rows * sizeof(long long), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HCLAE_OK;
}

int hclae_online_chunk(hclae_ctx *ctx, const uint8_t *Xu8, int64_t n, int D, float *C, int M, int K,
                       uint8_t *codes, float *residue, uint8_t *codes_first, double *err)
{
    int rc = check_call(ctx, n, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (!ctx->run_sum) return fail(ctx, HCLAE_ESTATE, "hclae_online_chunk before hclae_online_begin");
    if (n == 0) { if (err) *err = 0.0; return HCLAE_OK; }
    if (!Xu8 || !C || !codes || !residue) return fail(ctx, HCLAE_EINVAL, "hclae_online_chunk: NULL pointer");
    if (misaligned(C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_online_chunk: float arrays must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(Xu8) % 16 != 0)
        return fail(ctx, HCLAE_EINVAL, "hclae_online_chunk: Xu8 must be 16-byte aligned");
    const int64_t total = n * (int64_t)D;
    hipLaunchKernelGGL(k_convert_u8, dim3(stream_blocks(ctx, (total >> 4) + 1, kFlatThreads * 2)), dim3(kFlatThreads), 0,
                       ctx->stream, residue, Xu8, total);
    HIP_TRY(ctx, hipGetLastError());
    for (int m = 0; m < M; ++m) {
        float *Cm = C + (size_t)m * K * D;
        if ((rc = launch_norms(ctx, Cm, 0, 0, false, true)) != HCLAE_OK) return rc;
        if ((rc = launch_assign(ctx, m, n, residue, Cm, codes, 0, 0, 0, true)) != HCLAE_OK) return rc;
        if (codes_first) {
            hipLaunchKernelGGL(k_copy_column, dim3(stream_blocks(ctx, n, kFlatThreads)), dim3(kFlatThreads), 0, ctx->stream,
                               codes_first, codes, n, M, m);
            HIP_TRY(ctx, hipGetLastError());
        }
        if ((rc = launch_update(ctx, m, n, residue, Cm, codes, nullptr, true, true)) != HCLAE_OK) return rc;
        if ((rc = launch_assign(ctx, m, n, residue, Cm, codes, 0, 0, 0, true)) != HCLAE_OK) return rc;
        const bool last = (m == M - 1) && err;
        const int b = last ? launch_heat_cool<-1, true>(ctx, m, n, C, codes, residue, ctx->part_b)
                           : launch_heat_cool<-1, false>(ctx, m, n, C, codes, residue, nullptr);
        if (b < 0) return b;
        if (last) {
            hipLaunchKernelGGL(k_finish_stage, dim3(1), dim3(kFinishThreads), 0, ctx->stream,
                               (const double *)nullptr, ctx->part_b, (const long long *)nullptr, b,
                               (const int *)nullptr, 0, (const unsigned *)nullptr, ctx->rec);
            HIP_TRY(ctx, hipGetLastError());
            if ((rc = fetch_records(ctx, 1)) != HCLAE_OK) return rc;
            *err = ctx->rec_host[0].sum_after / (double)n;
        }
    }
    return HCLAE_OK;
}

// ---- multi-path encoding (Sec. 3.3) --------------------------------------------------------------

static void beam_release(hclae_ctx *ctx)
{
    void *dev[] = {ctx->beam_rows[0], ctx->beam_rows[1], ctx->beam_err[0], ctx->beam_err[1],
                   ctx->beam_pre[0], ctx->beam_pre[1], ctx->beam_mask};
    for (void *p : dev)
        if (p) (void)hipFree(p);
    ctx->beam_rows[0] = ctx->beam_rows[1] = nullptr;
    ctx->beam_err[0] = ctx->beam_err[1] = nullptr;
    ctx->beam_pre[0] = ctx->beam_pre[1] = nullptr;
    ctx->beam_mask = nullptr;
    ctx->beam_cap = 0;
    ctx->beam_L = 0;
}

// Buffers for batches of `cap` vectors with L paths each.  with_state: also the residual, error and
// prefix ping-pong buffers (hclae_encode_beam); the single step only needs the candidate bitmaps.
static int beam_scratch(hclae_ctx *ctx, int64_t cap, int L, bool with_state)
{
    const bool have_state = ctx->beam_rows[0] != nullptr;
    if (ctx->beam_mask && ctx->beam_cap >= cap && ctx->beam_L >= L && (have_state || !with_state)) return HCLAE_OK;
    // stream-ordered work may still use the old buffers
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->beam_cap > cap) cap = ctx->beam_cap;
    if (ctx->beam_L > L) L = ctx->beam_L;
    with_state = with_state || have_state;
    beam_release(ctx);
    const size_t rows = (size_t)cap * L;
    hipError_t e = hipMalloc((void **)&ctx->beam_mask, rows * sizeof(BeamMask));
    for (int i = 0; i < 2 && with_state; ++i) {
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->beam_rows[i], rows * ctx->D * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->beam_err[i], rows * sizeof(double));
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->beam_pre[i], rows * ctx->M);
    }
    if (e != hipSuccess) {
        beam_release(ctx);
        return fail(ctx, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (multi-path scratch)", e);
    }
    ctx->beam_cap = cap;
    ctx->beam_L = L;
    return HCLAE_OK;
}

extern "C++" {
template <int KB>
static int launch_beam_score_kb(hclae_ctx *ctx, const float *rows, const double *err, const float *Cm,
                                int64_t N, int Lc, int Ln, BeamMask *masks)
{
    const int D = ctx->D;
    const int NC = ctx->NC;
    const int dpad = kChunkD * NC;
    // bound on the rounding error of a shifted score, relative to hmax + ||r|| cmax + ||r||^2:
    // dpad + 1 accumulation steps of relative size 2^-23, plus the roundings of the norm, the
    // shift by the beam error, the threshold arithmetic and of the residual rows themselves
    const float gamma = 1.01f * (float)(dpad + 8) * 1.1920929e-7f;
    const int V = kTileVec / Lc;
    const int64_t ntiles = (N + V - 1) / V;
    Timed t_(ctx, HCLAE_T_BEAM_SCORE);
    if (ctx->resident && ctx->contraction == 1) {
        const size_t lds = (size_t)KB * 8 * NC * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        int64_t blocks = (ntiles + 3) / 4;                      // few tiles: one per SIMD before any SIMD gets two
        if (blocks > ctx->cus) blocks = ctx->cus;
        const uint64_t attr_set = 1ull << 9;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_beam_score_split<KB>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        // accumulation bound of the split contraction (see launch_assign_kb) plus the roundings of the shift
        const float acc_bound = (float)(3 * (dpad / kSplitStep) + 9) * 4.76837158203125e-7f;
        hipLaunchKernelGGL(k_split_norms, dim3((ctx->K + 3) / 4), dim3(256), 0, ctx->stream, Cm, ctx->K, D, D, ctx->split_norms);
        hipLaunchKernelGGL((k_beam_score_split<KB>), dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           rows, err, Cm, ctx->hneg, ctx->split_norms, N, Lc, Ln, D, D, ctx->K, NC, acc_bound, masks);
    } else if (ctx->contraction == 1) {
        // D-chunked, split-bf16: two slices of 64 dims in LDS, one block per CU
        const size_t lds = (size_t)2 * KB * 8 * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t nbt = (ntiles + kAssignWaves - 1) / kAssignWaves;
        int64_t blocks = nbt < ctx->cus ? nbt : ctx->cus;
        const uint64_t attr_set = 1ull << 10;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_beam_score_split_chunked<KB>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        if (NC > ctx->NC || KB != ctx->kb)
            return fail(ctx, HCLAE_EINVAL, "beam: codebook image too small for this shape");
        const float acc_bound = (float)(3 * (dpad / kSplitStep) + 9) * 4.76837158203125e-7f;
        const int img_total = NC * 4 * KB * kWave;
        hipLaunchKernelGGL(k_split_norms, dim3((ctx->K + 3) / 4), dim3(256), 0, ctx->stream, Cm, ctx->K, D, D, ctx->split_norms);
        hipLaunchKernelGGL(k_codebook_image_split, dim3((img_total + 255) / 256), dim3(256), 0, ctx->stream,
                           Cm, ctx->K, D, D, KB, NC, reinterpret_cast<uint4 *>(ctx->cb_image));
        hipLaunchKernelGGL((k_beam_score_split_chunked<KB>), dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           rows, err, reinterpret_cast<const uint4 *>(ctx->cb_image), ctx->hneg, ctx->split_norms,
                           N, Lc, Ln, D, D, ctx->K, NC, acc_bound, masks);
    } else if (ctx->resident) {
        const size_t lds = (size_t)KB * 8 * NC * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        int64_t blocks = (ntiles + 3) / 4;                      // few tiles: one per SIMD before any SIMD gets two
        if (blocks > ctx->cus) blocks = ctx->cus;
        const uint64_t attr_set = 1ull << 11;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_beam_score_resident<KB>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        hipLaunchKernelGGL((k_beam_score_resident<KB>), dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           rows, err, Cm, ctx->hneg, N, Lc, Ln, D, D, ctx->K, NC, gamma, masks);
    } else {
        const size_t lds = (size_t)2 * KB * 8 * kWave * sizeof(float4) + (32 * KB + 4) * sizeof(float);
        const int64_t nbt = (ntiles + kAssignWaves - 1) / kAssignWaves;
        int64_t blocks = nbt < ctx->cus ? nbt : ctx->cus;
        const uint64_t attr_set = 1ull << 12;        // this call site's bit in ctx->attr_done
        if (!(ctx->attr_done & attr_set)) {
            HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_beam_score_chunked<KB>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
            ctx->attr_done |= attr_set;
        }
        if (NC > ctx->NC || KB != ctx->kb)
            return fail(ctx, HCLAE_EINVAL, "beam: codebook image too small for this shape");
        const int img_total = NC * KB * 8 * kWave;
        hipLaunchKernelGGL(k_codebook_image, dim3((img_total + 255) / 256), dim3(256), 0, ctx->stream,
                           Cm, ctx->K, D, D, KB, NC, ctx->cb_image);
        hipLaunchKernelGGL((k_beam_score_chunked<KB>), dim3((unsigned)blocks), dim3(kAssignThreads), lds, ctx->stream,
                           rows, err, ctx->cb_image, ctx->hneg, N, Lc, Ln, D, D, ctx->K, NC, gamma, masks);
    }
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}
}  // extern "C++"

// One dictionary of the beam for N vectors: norms, scoring, exact expansion.  rows_c has stride D.
static int enqueue_beam_step(hclae_ctx *ctx, const float *rows_c, const double *err_c, const float *Cm,
                             int64_t N, int Lc, int Ln, const uint8_t *pre_c, uint8_t *pre_n, int m,
                             float *rows_n, double *err_n, uint8_t *parent, uint8_t *code)
{
    int rc;
    if ((rc = launch_norms(ctx, Cm)) != HCLAE_OK) return rc;
    switch (ctx->kb) {
    case 1: rc = launch_beam_score_kb<1>(ctx, rows_c, err_c, Cm, N, Lc, Ln, ctx->beam_mask); break;
    case 2: rc = launch_beam_score_kb<2>(ctx, rows_c, err_c, Cm, N, Lc, Ln, ctx->beam_mask); break;
    case 4: rc = launch_beam_score_kb<4>(ctx, rows_c, err_c, Cm, N, Lc, Ln, ctx->beam_mask); break;
    default: rc = launch_beam_score_kb<8>(ctx, rows_c, err_c, Cm, N, Lc, Ln, ctx->beam_mask); break;
    }
    if (rc != HCLAE_OK) return rc;
    int64_t blocks = N < (int64_t)ctx->cus * 32 ? N : (int64_t)ctx->cus * 32;
    Timed t_(ctx, HCLAE_T_BEAM_EXPAND);
    hipLaunchKernelGGL(k_beam_expand, dim3((unsigned)blocks), dim3(kWave), 0, ctx->stream,
                       rows_c, ctx->D, ctx->beam_mask, Cm, ctx->K, ctx->D, N, Lc, Ln,
                       pre_c, pre_n, ctx->M, m, rows_n, ctx->D, err_n, parent, code);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

static int beam_next_width(int K, int Lc, int L)
{
    const long total = (long)K * Lc;
    return L < total ? L : (int)total;
}

// Vectors per batch of the multi-path encoder: residual buffers of at most 2^31 floats (8 GiB) each.
static int64_t beam_batch(const hclae_ctx *ctx, int64_t N, int L)
{
    int64_t cap = ((int64_t)1 << 31) / ((int64_t)L * ctx->D);
    if (cap < 1024) cap = 1024;
    return N < cap ? N : cap;
}

static int enqueue_encode_beam(hclae_ctx *ctx, const float *X, int64_t N, const float *C, int L,
                               uint8_t *codes, float *residue, double *err)
{
    const int D = ctx->D, K = ctx->K, M = ctx->M;
    if (N == 0) return HCLAE_OK;
    const int64_t cap = beam_batch(ctx, N, L);
    int rc = beam_scratch(ctx, cap, L, true);
    if (rc != HCLAE_OK) return rc;
    for (int64_t n0 = 0; n0 < N; n0 += cap) {
        const int64_t nb = N - n0 < cap ? N - n0 : cap;
        const float *rows_c = X + n0 * D;
        const double *err_c = nullptr;
        const uint8_t *pre_c = nullptr;
        int Lc = 1;
        for (int m = 0; m < M; ++m) {
            const bool last = (m == M - 1);
            const int Ln = last ? 1 : beam_next_width(K, Lc, L);    // the answer is the best of the last beam
            float *rows_n = last ? residue + n0 * D : ctx->beam_rows[m & 1];
            double *err_n = last ? (err ? err + n0 : nullptr) : ctx->beam_err[m & 1];
            uint8_t *pre_n = last ? codes + n0 * M : ctx->beam_pre[m & 1];
            rc = enqueue_beam_step(ctx, rows_c, err_c, C + (size_t)m * K * D, nb, Lc, Ln, pre_c, pre_n, m,
                                   rows_n, err_n, nullptr, nullptr);
            if (rc != HCLAE_OK) return rc;
            rows_c = rows_n; err_c = err_n; pre_c = pre_n; Lc = Ln;
        }
    }
    return HCLAE_OK;
}

int hclae_beam_step(hclae_ctx *ctx, const float *rows, const double *err, const float *Cm,
                    int64_t N, int D, int K, int Lc, int L,
                    float *rows_next, double *err_next, uint8_t *parent, uint8_t *code)
{
    int rc = check_call(ctx, N, D, ctx ? ctx->M : 1, K);
    if (rc != HCLAE_OK) return rc;
    if (L < 1 || L > kBeamMaxL || Lc < 1 || Lc > L)
        return fail(ctx, HCLAE_EINVAL, "hclae_beam_step: need 1 <= Lc <= L <= 32");
    if (N == 0) return HCLAE_OK;
    if (!rows || !Cm || !rows_next || rows_next == rows)
        return fail(ctx, HCLAE_EINVAL, "hclae_beam_step: NULL or aliased rows");
    if (misaligned(rows, Cm, rows_next)) return fail(ctx, HCLAE_EINVAL, "hclae_beam_step: float arrays must be 16-byte aligned");
    if (N * (int64_t)L >= ((int64_t)1 << 31)) return fail(ctx, HCLAE_EINVAL, "hclae_beam_step: N * L too large");
    if ((rc = beam_scratch(ctx, N, L, false)) != HCLAE_OK) return rc;
    return enqueue_beam_step(ctx, rows, err, Cm, N, Lc, beam_next_width(K, Lc, L), nullptr, nullptr, 0,
                             rows_next, err_next, parent, code);
}

int hclae_encode_beam(hclae_ctx *ctx, const float *X, int64_t N, int D, const float *C, int M, int K, int L,
                      uint8_t *codes, float *residue, double *err)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (L < 1 || L > kBeamMaxL) return fail(ctx, HCLAE_EINVAL, "hclae_encode_beam: need 1 <= L <= 32");
    if (N == 0) return HCLAE_OK;
    if (!X || !C || !codes || !residue || residue == X)
        return fail(ctx, HCLAE_EINVAL, "hclae_encode_beam: NULL or aliased pointer");
    if (misaligned(X, C, residue)) return fail(ctx, HCLAE_EINVAL, "hclae_encode_beam: float arrays must be 16-byte aligned");
    return enqueue_encode_beam(ctx, X, N, C, L, codes, residue, err);
}

// ---- improved k-means (Sec. 3.2) ---------------------------------------------------------------

static int pca_scratch(hclae_ctx *ctx)
{
    if (ctx->pca_rt) return HCLAE_OK;
    const int D = ctx->D, K = ctx->K;
    ctx->pca_ncol = 256;
    // Gram partials: ranges of >= 1024 rows, at most 256 MB of them
    int ng = (int)(((size_t)256 << 20) / ((size_t)D * D * sizeof(double)));
    if (ng > 2048) ng = 2048;
    if (ng < 1) ng = 1;
    ctx->pca_ngram = ng;
    hipError_t e = hipMalloc((void **)&ctx->pca_rt, (size_t)D * D * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_crot, (size_t)K * D * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_colpart, (size_t)ctx->pca_ncol * D * sizeof(double));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_grampart, (size_t)ng * D * D * sizeof(double));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_mean, (size_t)D * sizeof(double));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_mean32, (size_t)D * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_cov, (size_t)D * D * sizeof(double));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->pca_R, (size_t)D * D * sizeof(float));
    if (e != hipSuccess) return fail(ctx, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (PCA scratch)", e);
    return HCLAE_OK;
}

// out = x R^T (rows), R given as is; the caller passes the transposed matrix for R^T.
static int launch_project(hclae_ctx *ctx, const float *x, int64_t N, const float *R, float *out)
{
    const int D = ctx->D;
    const size_t lds = (size_t)8 * 8 * kWave * sizeof(float4);
    const uint64_t attr_set = 1ull << 13;        // this call site's bit in ctx->attr_done
    if (!(ctx->attr_done & attr_set)) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_project),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
        ctx->attr_done |= attr_set;
    }
    const int64_t nbt = (N + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);
    const int groups = (D + 255) / 256;
    int64_t blocks = nbt < 2 * ctx->cus ? nbt : 2 * ctx->cus;
    Timed t_(ctx, HCLAE_T_ROTATE);
    hipLaunchKernelGGL(k_project, dim3((unsigned)blocks, (unsigned)groups), dim3(kAssignThreads), lds, ctx->stream,
                       x, R, N, D, out);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

static int launch_rotate(hclae_ctx *ctx, const float *x, int64_t N, const float *R, int transpose, float *out)
{
    if (!transpose) return launch_project(ctx, x, N, R, out);
    const int D = ctx->D;
    hipLaunchKernelGGL(k_transpose, dim3((D * D + 255) / 256), dim3(256), 0, ctx->stream, R, D, ctx->pca_rt);
    HIP_TRY(ctx, hipGetLastError());
    return launch_project(ctx, x, N, ctx->pca_rt, out);
}

int hclae_rotate(hclae_ctx *ctx, const float *x, int64_t N, int D, const float *R, int transpose, float *out)
{
    if (!ctx) return HCLAE_EINVAL;
    int rc = hclae_check_shape(N, D, ctx->M, ctx->K);
    if (rc != HCLAE_OK) return fail(ctx, rc, "shape out of range");
    if (D != ctx->D) return fail(ctx, HCLAE_ESTATE, "D differs from hclae_create");
    if (N == 0) return HCLAE_OK;
    if (!x || !R || !out || x == out) return fail(ctx, HCLAE_EINVAL, "hclae_rotate: bad argument");
    if (misaligned(x, R, out)) return fail(ctx, HCLAE_EINVAL, "hclae_rotate: float arrays must be 16-byte aligned");
    if ((rc = pca_scratch(ctx)) != HCLAE_OK) return rc;
    return launch_rotate(ctx, x, N, R, transpose, out);
}

static int enqueue_covariance(hclae_ctx *ctx, const float *xp, int64_t N, double *mean, double *cov)
{
    const int D = ctx->D;
    Timed t_(ctx, HCLAE_T_MOMENTS);
    int ncol = (int)((N + 1023) / 1024);
    if (ncol > ctx->pca_ncol) ncol = ctx->pca_ncol;
    const int64_t rpc = (N + ncol - 1) / ncol;
    ncol = (int)((N + rpc - 1) / rpc);
    hipLaunchKernelGGL(k_colsum, dim3(ncol), dim3(256), 0, ctx->stream, xp, N, D, rpc, row_geom(D).lcw, ctx->pca_colpart);
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_mean_finish, dim3((D + 255) / 256), dim3(256), 0, ctx->stream,
                       ctx->pca_colpart, ncol, N, D, mean, ctx->pca_mean32);
    HIP_TRY(ctx, hipGetLastError());
    int ng = (int)((N + 1023) / 1024);
    if (ng > ctx->pca_ngram) ng = ctx->pca_ngram;
    const int64_t rpg = (N + ng - 1) / ng;
    ng = (int)((N + rpg - 1) / rpg);
    const int tiles = (D + 127) / 128;
    hipLaunchKernelGGL(k_gram_tile, dim3(ng, tiles, tiles), dim3(512), 0, ctx->stream,
                       xp, ctx->pca_mean32, N, D, rpg, ctx->pca_grampart);
    HIP_TRY(ctx, hipGetLastError());
    hipLaunchKernelGGL(k_cov_finish, dim3(stream_blocks(ctx, (int64_t)D * D, 256)), dim3(256), 0, ctx->stream,
                       ctx->pca_grampart, ng, N, D, mean, ctx->pca_mean32, cov);
    HIP_TRY(ctx, hipGetLastError());
    return HCLAE_OK;
}

int hclae_covariance(hclae_ctx *ctx, const float *xp, int64_t N, int D, double *mean, double *cov)
{
    if (!ctx) return HCLAE_EINVAL;
    int rc = hclae_check_shape(N, D, ctx->M, ctx->K);
    if (rc != HCLAE_OK) return fail(ctx, rc, "shape out of range");
    if (D != ctx->D) return fail(ctx, HCLAE_ESTATE, "D differs from hclae_create");
    if (N < 1 || !xp || !mean || !cov) return fail(ctx, HCLAE_EINVAL, "hclae_covariance: bad argument");
    if (misaligned(xp)) return fail(ctx, HCLAE_EINVAL, "hclae_covariance: float arrays must be 16-byte aligned");
    if ((rc = pca_scratch(ctx)) != HCLAE_OK) return rc;
    return enqueue_covariance(ctx, xp, N, mean, cov);
}

// Principal axes of the N rows of xp into R (DEVICE float [D][D], rows = axes, most variance first): second
// moments on the device, eigen-decomposition on the host in fp64, axes rounded to fp32.  Synchronises the stream.
static int compute_pca_axes(hclae_ctx *ctx, const float *xp, int64_t N, float *R, double *eigenvalues)
{
    const int D = ctx->D;
    int rc = enqueue_covariance(ctx, xp, N, ctx->pca_mean, ctx->pca_cov);
    if (rc != HCLAE_OK) return rc;
    std::vector<double> cov((size_t)D * D), w(D), vt((size_t)D * D);
    HIP_TRY(ctx, hipMemcpyAsync(cov.data(), ctx->pca_cov, cov.size() * sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    // the device result is symmetric up to the rounding order of the two triangles: take their mean
    for (int i = 0; i < D; ++i)
        for (int j = i + 1; j < D; ++j) {
            const double a = 0.5 * (cov[(size_t)i * D + j] + cov[(size_t)j * D + i]);
            cov[(size_t)i * D + j] = cov[(size_t)j * D + i] = a;
        }
    if (symmetric_eigen(cov.data(), D, w.data(), vt.data()) != 0)
        return fail(ctx, HCLAE_EHIP, "eigen-decomposition of the covariance did not converge");
    std::vector<float> r32((size_t)D * D);
    for (size_t i = 0; i < r32.size(); ++i) r32[i] = (float)vt[i];
    HIP_TRY(ctx, hipMemcpyAsync(R, r32.data(), r32.size() * sizeof(float), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));               // r32 is pageable host memory of this frame
    if (eigenvalues) for (int i = 0; i < D; ++i) eigenvalues[i] = w[i];
    return HCLAE_OK;
}

int hclae_symmetric_eigen(const double *A, int n, double *w, double *Vt)
{
    if (!A || !w || !Vt || n < 1 || n > HCLAE_MAX_D) return HCLAE_EINVAL;
    std::vector<double> work(A, A + (size_t)n * n);
    return symmetric_eigen(work.data(), n, w, Vt) == 0 ? HCLAE_OK : HCLAE_ESTATE;
}

int hclae_pca_axes(hclae_ctx *ctx, const float *xp, int64_t N, int D, float *R, double *eigenvalues)
{
    if (!ctx) return HCLAE_EINVAL;
    int rc = hclae_check_shape(N, D, ctx->M, ctx->K);
    if (rc != HCLAE_OK) return fail(ctx, rc, "shape out of range");
    if (D != ctx->D) return fail(ctx, HCLAE_ESTATE, "D differs from hclae_create");
    if (N < 1 || !xp || !R) return fail(ctx, HCLAE_EINVAL, "hclae_pca_axes: bad argument");
    if (misaligned(xp, R)) return fail(ctx, HCLAE_EINVAL, "hclae_pca_axes: float arrays must be 16-byte aligned");
    if ((rc = pca_scratch(ctx)) != HCLAE_OK) return rc;
    return compute_pca_axes(ctx, xp, N, R, eigenvalues);
}

int hclae_assign_prefix(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, const float *C,
                        int M, int K, int dact, uint8_t *codes)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M || dact < 1 || dact > D) return fail(ctx, HCLAE_EINVAL, "hclae_assign_prefix: m or dact out of range");
    if (N == 0) return HCLAE_OK;
    if (!C || !codes || !xp) return fail(ctx, HCLAE_EINVAL, "hclae_assign_prefix: NULL pointer");
    if (misaligned(C, xp)) return fail(ctx, HCLAE_EINVAL, "hclae_assign_prefix: float arrays must be 16-byte aligned");
    const float *Cm = C + (size_t)m * K * D;
    if ((rc = launch_norms(ctx, Cm, dact, D)) != HCLAE_OK) return rc;
    return launch_assign(ctx, m, N, xp, Cm, codes, dact, D);
}

// Prefixes of the coordinates for the improved k-means: d_i = ceil(D^(i/I)), i = 1..I (Sec. 3.2 prints d_i = d^(i/I)
// with I = 10, which is no integer: rounded up), equal values once, the last one D.  Returns how many.
static int dimension_schedule(int D, int I, int *dims)
{
    int n = 0;
    for (int i = 1; i <= I; ++i) {
        int d = (int)ceil(pow((double)D, (double)i / (double)I) - 1e-9);
        if (d < 1) d = 1;
        if (d > D) d = D;
        if (n == 0 || d > dims[n - 1]) dims[n++] = d;
    }
    dims[n - 1] = D;
    return n;
}

// Enqueues one stage whose cool-down is the improved k-means of Sec. 3.2; by-products land in ctx->rec[slot].
// seed_dev: DEVICE seed rows or null.  R: DEVICE axes, or null: found from this stage's x' (synchronises once).
static int enqueue_stage_pca(hclae_ctx *ctx, int m, int64_t N, float *C, uint8_t *codes, float *residue, const float *R,
                             const int *dims, int n_dims, int iters_per_dim, float *xr, const int64_t *seed_dev,
                             int slot, int *iters_run_out)
{
    const int D = ctx->D, K = ctx->K;
    int rc;
    float *Cm = C + (size_t)m * K * D;
    const size_t cbytes = (size_t)K * D * sizeof(float);
    const int pb = launch_heat_cool<+1, true>(ctx, m, N, C, codes, residue, ctx->part_a);
    if (pb < 0) return pb;
    if (seed_dev) {
        hipLaunchKernelGGL(k_seed, dim3(K), dim3(256), 0, ctx->stream, residue, seed_dev, K, D, Cm);
        HIP_TRY(ctx, hipGetLastError());
    }
    if (!R) {                   // step 1 of Sec. 3.2 inside the library: the principal axes of this stage's x'
        if ((rc = compute_pca_axes(ctx, residue, N, ctx->pca_R, nullptr)) != HCLAE_OK) return rc;
        R = ctx->pca_R;
    }
    // into the PCA space: x^r = R x', C' = R C_m (C[m] holds C' until it is rotated back)
    if ((rc = launch_rotate(ctx, residue, N, R, 0, xr)) != HCLAE_OK) return rc;
    if ((rc = launch_rotate(ctx, Cm, K, R, 0, ctx->pca_crot)) != HCLAE_OK) return rc;
    HIP_TRY(ctx, hipMemcpyAsync(Cm, ctx->pca_crot, cbytes, hipMemcpyDeviceToDevice, ctx->stream));
    // max |x^r| over ALL coordinates for the fixed-point centroid sums: a prefix assignment reads only part of a row
    if ((rc = launch_norms(ctx, Cm, dims[0], D, false)) != HCLAE_OK) return rc;    // zeroes the slot
    {
        const int64_t n4 = N * (D / 4);
        hipLaunchKernelGGL(k_absmax, dim3(stream_blocks(ctx, n4, 256 * 4)), dim3(256), 0, ctx->stream,
                           reinterpret_cast<const float4 *>(xr), n4, ctx->refine_count + 1);
        HIP_TRY(ctx, hipGetLastError());
    }
    int iters_run = 0;
    for (int i = 0; i < n_dims; ++i) {
        if (iters_per_dim > 0 && (rc = launch_norms(ctx, Cm, dims[i], D, true)) != HCLAE_OK) return rc;
        for (int t = 0; t < iters_per_dim; ++t, ++iters_run) {
            if ((rc = launch_assign(ctx, m, N, xr, Cm, codes, dims[i], D)) != HCLAE_OK) return rc;
            if ((rc = launch_update(ctx, m, N, xr, Cm, codes, nullptr, true, false, dims[i])) != HCLAE_OK) return rc;
        }
    }
    // back: C_m = R^T C'
    if ((rc = launch_rotate(ctx, Cm, K, R, 1, ctx->pca_crot)) != HCLAE_OK) return rc;
    HIP_TRY(ctx, hipMemcpyAsync(Cm, ctx->pca_crot, cbytes, hipMemcpyDeviceToDevice, ctx->stream));
    if ((rc = launch_norms(ctx, Cm)) != HCLAE_OK) return rc;
    if ((rc = launch_assign(ctx, m, N, residue, Cm, codes)) != HCLAE_OK) return rc;
    const int pa = launch_heat_cool<-1, true>(ctx, m, N, C, codes, residue, ctx->part_b);
    if (pa < 0) return pa;
    hipLaunchKernelGGL(k_finish_stage, dim3(1), dim3(kFinishThreads), 0, ctx->stream,
                       ctx->part_a, ctx->part_b, ctx->part_chg, pa, iters_run > 0 ? ctx->nk : nullptr, K,
                       ctx->refine_count, ctx->rec + slot);
    HIP_TRY(ctx, hipGetLastError());
    if (iters_run_out) *iters_run_out = iters_run;
    return HCLAE_OK;
}

// The stage of a sweep (or of hclae_anneal_stage) when the improved k-means is the ctx's cool-down: the schedule
// of hclae_set_cooldown, ceil(iters / prefixes) Lloyd iterations on each prefix, x^r in scratch the ctx keeps.
static int enqueue_stage_cooldown_pca(hclae_ctx *ctx, int m, int64_t N, float *C, uint8_t *codes, float *residue,
                                      int iters, const int64_t *seed_dev, int slot, int *iters_run_out)
{
    int rc = pca_scratch(ctx);
    if (rc != HCLAE_OK) return rc;
    if (!ctx->pca_xr) {
        hipError_t e = hipMalloc((void **)&ctx->pca_xr, sizeof(float) * (size_t)ctx->N_max * ctx->D);
        if (e != hipSuccess) return fail(ctx, e == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (rotated data)", e);
    }
    int dims[64];
    const int n_dims = dimension_schedule(ctx->D, ctx->cooldown_phases, dims);
    const int per = iters > 0 ? (iters + n_dims - 1) / n_dims : 0;
    return enqueue_stage_pca(ctx, m, N, C, codes, residue, nullptr, dims, n_dims, per, ctx->pca_xr, seed_dev, slot,
                             iters_run_out);
}

int hclae_dimension_schedule(int D, int phases, int *dims, int *n_dims)
{
    if (D < 1 || D > HCLAE_MAX_D || phases < 1 || phases > 64 || !dims || !n_dims) return HCLAE_EINVAL;
    *n_dims = dimension_schedule(D, phases, dims);
    return HCLAE_OK;
}

int hclae_set_cooldown(hclae_ctx *ctx, int mode, int phases)
{
    if (!ctx) return HCLAE_EINVAL;
    if (mode != HCLAE_COOLDOWN_LLOYD && mode != HCLAE_COOLDOWN_IMPROVED)
        return fail(ctx, HCLAE_EINVAL, "hclae_set_cooldown: unknown mode");
    if (mode == HCLAE_COOLDOWN_IMPROVED && (phases < 1 || phases > 64))
        return fail(ctx, HCLAE_EINVAL, "hclae_set_cooldown: need 1 <= phases <= 64");
    ctx->cooldown = mode;
    if (mode == HCLAE_COOLDOWN_IMPROVED) ctx->cooldown_phases = phases;
    return HCLAE_OK;
}

int hclae_anneal_stage_pca(hclae_ctx *ctx, int m, int64_t N, int D, float *C, int M, int K,
                           uint8_t *codes, float *residue, const float *R, const int *dims, int n_dims,
                           int iters_per_dim, float *xr, const int64_t *init_idx, hclae_stage_stats *stats)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (m < 0 || m >= M || iters_per_dim < 0 || n_dims < 1 || !dims)
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: bad argument");
    for (int i = 0; i < n_dims; ++i)
        if (dims[i] < 1 || dims[i] > D || (i > 0 && dims[i] <= dims[i - 1]))
            return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: dims must increase within [1, D]");
    if (dims[n_dims - 1] != D) return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: the last prefix must be D");
    if (init_idx)
        for (int i = 0; i < K; ++i)
            if (init_idx[i] < 0 || init_idx[i] >= N) return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: init_idx out of range");
    if (N == 0) { if (stats) memset(stats, 0, sizeof(*stats)); return HCLAE_OK; }
    if (!C || !codes || !residue || !xr || xr == residue)
        return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: NULL or aliased pointer");
    if (misaligned(C, residue, R, xr)) return fail(ctx, HCLAE_EINVAL, "hclae_anneal_stage_pca: float arrays must be 16-byte aligned");
    if ((rc = pca_scratch(ctx)) != HCLAE_OK) return rc;
    if (init_idx)
        HIP_TRY(ctx, hipMemcpyAsync(ctx->seed_idx, init_idx, sizeof(int64_t) * K, hipMemcpyHostToDevice, ctx->stream));
    int iters_run = 0;
    if ((rc = enqueue_stage_pca(ctx, m, N, C, codes, residue, R, dims, n_dims, iters_per_dim, xr,
                                init_idx ? ctx->seed_idx : nullptr, 0, &iters_run)) != HCLAE_OK) return rc;
    if (stats) {
        if ((rc = fetch_records(ctx, 1)) != HCLAE_OK) return rc;
        fill_stats(ctx->rec_host[0], N, iters_run, stats);
    } else if (init_idx) {
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    return HCLAE_OK;
}

// ---- dictionary order and code statistics ------------------------------------------------------

int hclae_reorder_by_variance(hclae_ctx *ctx, int64_t N, int D, float *C, int M, int K, uint8_t *codes,
                              double *var, int *order)
{
    int rc = check_call(ctx, N, D, M, K);
    if (rc != HCLAE_OK) return rc;
    if (!C || (N > 0 && !codes)) return fail(ctx, HCLAE_EINVAL, "hclae_reorder_by_variance: NULL pointer");
    if (misaligned(C)) return fail(ctx, HCLAE_EINVAL, "hclae_reorder_by_variance: float arrays must be 16-byte aligned");
    const size_t per = (size_t)K * D;
    if (!ctx->order_tmp) {                  // scratch of this call, kept by the ctx from the first call on
        hipError_t ea = hipMalloc((void **)&ctx->order_var, sizeof(double) * M);
        if (ea == hipSuccess) ea = hipMalloc((void **)&ctx->order_idx, sizeof(int) * M);
        if (ea == hipSuccess) ea = hipMalloc((void **)&ctx->order_tmp, sizeof(float) * M * per);
        if (ea != hipSuccess) return fail(ctx, ea == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (reorder scratch)", ea);
    }
    double *dvar = ctx->order_var;
    int *dorder = ctx->order_idx;
    float *tmp = ctx->order_tmp;
    hipError_t e = hipSuccess;
    std::vector<double> hv(M);
    std::vector<int> ho(M);
    hipLaunchKernelGGL(k_dictionary_variance, dim3(M), dim3(256), 0, ctx->stream, C, K, D, dvar);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(hv.data(), dvar, sizeof(double) * M, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, HCLAE_EHIP, "dictionary variance", e);
    for (int j = 0; j < M; ++j) ho[j] = j;
    std::stable_sort(ho.begin(), ho.end(), [&](int x, int y) { return hv[x] > hv[y]; });
    e = hipMemcpyAsync(dorder, ho.data(), sizeof(int) * M, hipMemcpyHostToDevice, ctx->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_permute_dictionaries, dim3(stream_blocks(ctx, (int64_t)(M * per), 256)), dim3(256), 0, ctx->stream,
                           C, dorder, M, per, tmp);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(C, tmp, sizeof(float) * M * per, hipMemcpyDeviceToDevice, ctx->stream);
    if (e == hipSuccess && N > 0) {
        hipLaunchKernelGGL(k_permute_code_columns, dim3(stream_blocks(ctx, N, 256)), dim3(256), 0, ctx->stream,
                           codes, dorder, N, M);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, HCLAE_EHIP, "reorder", e);
    if (var) for (int j = 0; j < M; ++j) var[j] = hv[j];
    if (order) for (int j = 0; j < M; ++j) order[j] = ho[j];
    return HCLAE_OK;
}

int hclae_code_stats(hclae_ctx *ctx, const uint8_t *codes, int64_t N, int M, int K,
                     int64_t *hist, int a, int b, int64_t *joint)
{
    int rc = check_call(ctx, N, ctx ? ctx->D : 4, M, K);
    if (rc != HCLAE_OK) return rc;
    if (!hist || (N > 0 && !codes)) return fail(ctx, HCLAE_EINVAL, "hclae_code_stats: NULL pointer");
    if (joint && (a < 0 || a >= M || b < 0 || b >= M)) return fail(ctx, HCLAE_EINVAL, "hclae_code_stats: column out of range");
    const size_t nh = (size_t)M * K, nj = joint ? (size_t)K * K : 0;
    if (!ctx->stats_buf) {                  // sized for the joint histogram too; kept by the ctx from the first call on
        hipError_t ea = hipMalloc((void **)&ctx->stats_buf, sizeof(unsigned long long) * (nh + (size_t)K * K));
        if (ea != hipSuccess) return fail(ctx, ea == hipErrorOutOfMemory ? HCLAE_ENOMEM : HCLAE_EHIP, "hipMalloc (code statistics)", ea);
    }
    unsigned long long *dev = ctx->stats_buf;
    hipError_t e = hipSuccess;
    hipLaunchKernelGGL(k_zero_u64, dim3(stream_blocks(ctx, (int64_t)(nh + nj), 256)), dim3(256), 0, ctx->stream, dev, nh + nj);
    e = hipGetLastError();
    if (e == hipSuccess && N > 0) {
        hipLaunchKernelGGL(k_code_histograms, dim3(stream_blocks(ctx, N, 256)), dim3(256), 0, ctx->stream,
                           codes, N, M, K, a, b, dev, joint ? dev + nh : (unsigned long long *)nullptr);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(hist, dev, sizeof(int64_t) * nh, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess && joint) e = hipMemcpyAsync(joint, dev + nh, sizeof(int64_t) * nj, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, HCLAE_EHIP, "code statistics", e);
    return HCLAE_OK;
}

int hclae_timing_enable(hclae_ctx *ctx, uint32_t class_mask)
{
    if (!ctx) return HCLAE_EINVAL;
    if (class_mask && !ctx->t_beg) {
        ctx->t_beg = new (std::nothrow) hipEvent_t[kMaxTimed]();
        ctx->t_end = new (std::nothrow) hipEvent_t[kMaxTimed]();
        ctx->t_cls = new (std::nothrow) uint8_t[kMaxTimed]();
        if (!ctx->t_beg || !ctx->t_end || !ctx->t_cls) return fail(ctx, HCLAE_ENOMEM, "timing pool");
        for (int i = 0; i < kMaxTimed; ++i) {
            HIP_TRY(ctx, hipEventCreate(&ctx->t_beg[i]));
            HIP_TRY(ctx, hipEventCreate(&ctx->t_end[i]));
        }
    }
    ctx->t_mask = class_mask;
    return HCLAE_OK;
}

int hclae_timing_read(hclae_ctx *ctx, hclae_kernel_times *out)
{
    if (!ctx || !out) return HCLAE_EINVAL;
    memset(out, 0, sizeof(*out));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < ctx->t_used; ++i) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->t_beg[i], ctx->t_end[i]));
        out->ms[ctx->t_cls[i]] += (double)ms;
        out->launches[ctx->t_cls[i]] += 1;
    }
    ctx->t_used = 0;
    return HCLAE_OK;
}

int hclae_work_counters(hclae_ctx *ctx, int64_t *out, int reset)
{
    if (!ctx || !out) return HCLAE_EINVAL;
    unsigned long long v[3] = {0, 0, 0};
    HIP_TRY(ctx, hipMemcpyAsync(v, ctx->work, sizeof(v), hipMemcpyDeviceToHost, ctx->stream));
    if (reset) HIP_TRY(ctx, hipMemsetAsync(ctx->work, 0, sizeof(v), ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < 3; ++i) out[i] = (int64_t)v[i];
    return HCLAE_OK;
}

int hclae_last_refined(hclae_ctx *ctx, int64_t *out)
{
    if (!ctx || !out) return HCLAE_EINVAL;
    unsigned v = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&v, ctx->refine_count, sizeof(unsigned), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    *out = (int64_t)v;
    return HCLAE_OK;
}

}  // extern "C"
