// Gaussian-kernel tile engine, K-loop variant with the cross term on the f16 matrix cores:
//     out[f, c] = sum_s k(F_f, S_s) vec[s, c]        (any d, up to 16 columns per launch)
//
// Same computation as knm_gemm.hip (Section 3.1, "Blockwise K_nm-vector product"; Gaussian
// kernel of Section 2) with the arithmetic of knm_tile_f16.hip: every scaled feature
// z = x sqrt(log2 e) / sigma is split into two halves z = zh + zl (22 significant bits) and
// the cross term is evaluated as three f16 MFMA products with fp32 accumulation,
//     <zf, zx>  ~=  fh.xh + fh.xl + fl.xh                      (drops fl.xl ~ 2^-22),
// so that the accumulator holds  log2 k(f, x) = <zf, zx> - |zf|^2 / 2 - |zx|^2 / 2  after
// one more MFMA whose K-slots carry the two norm terms as 4-digit fixed-point numbers
//     n = q1 2^10 + q2 2^-1 + q3 2^-12 + q4 2^-23,   q_i integers <= 2048 (exact in fp16),
// against the constants 2^10, 2^-1, 2^-12, 2^-23 on the other operand.
//
// Packed images.  Both operands are converted once per sweep (`pack_points_kernel`) into
// images laid out exactly as the LDS stage, so staging is a 16-byte copy (done by loads that
// write LDS directly, into a ring of stages that keeps two stages of loads in flight) and the
// conversion cost (scale, split, norms) is not repeated by every workgroup that visits a
// point.  Per block of 32 points the image holds n_kc + 1 chunks of 2 KB:
//     chunk kc < n_kc : [plane hi | lo][lane = 32 h + point] units of 8 halves = features
//                       16 kc + 8 h .. + 7 of the point               (MFMA operand layout)
//     chunk n_kc      : plane 0 = the point's slots when it is a FIXED point
//                       (-q1..-q4 of its norm term, then the four constants), plane 1 = its
//                       slots as a STREAM point (constants, then -q1..-q4); half-wave 1 zero.
// The same image therefore serves either role, and X and C are each packed once per sweep.
// Images are built slab by slab when they exceed the workspace.
//
// Tile shape and orientation as in knm_gemm.hip: workgroup = 256 fixed x 128 stream
// points, each wavefront 64 fixed x 128 stream = 8 accumulators of 32x32 in architectural VGPRs
// (the vector ALU reads them directly; in AGPRs every kernel value cost a v_accvgpr_read first);
// the stream block is the A operand, so a lane's accumulator registers run over stream
// points of one fixed point and the reduction against the vector columns is in-lane.
//
// Reduction against the vectors.  For a few columns each kernel value is multiplied into
// per-lane running sums on the vector ALU (one FMA per column).  For more columns (see the
// launcher for the rule) the
// reduction  out[f, c] += sum_s P[s, f] V[s, c]  is itself run on the matrix cores: a lane's
// 16 kernel values of a 32x32 tile are, without any data movement, the B operand of two
// K = 16 MFMAs whose K-slots are stream points; the kernel values (in [0, 1]) are split into
// two halves like the features, the vector rows are scaled per column by a power of two
// into the fp16 range, split likewise and staged in LDS in A-operand layout, and three
// products P_hi V_hi + P_lo V_hi + P_hi V_lo accumulate a 32-column x 32-point output tile in
// fp32.  That replaces t FMAs per kernel value by about three conversion instructions and
// serves up to 160 columns per launch: up to five groups of 32, each with its own output tile,
// fed by the same split kernel values.

#include <type_traits>

#include "knm_internal.h"
#include "knm_operands.h"

namespace knm {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kFixed = 256;                    // fixed points per workgroup
constexpr int kStream = 128;                   // stream points per tile
constexpr int kBlocks = (kFixed + kStream) / 32; // 32-point blocks per stage: 8 fixed, 4 stream
constexpr int kChunk = 16;                     // features per K-chunk = one MFMA K
constexpr int kUnits = 128;                    // 16-byte units per block and chunk (2 planes x 64 lanes)
constexpr int kLoads = kBlocks * kUnits / kThreads; // units copied per thread and stage (6)
constexpr int kStageUnits = kBlocks * kUnits;       // 16-byte units of one LDS stage (24 KB)
// Workgroups per CU.  The vector-ALU reduction and the matrix-core reduction with one group of 32 columns
// run two; so does the one with two groups for the Gaussian kernel when the vectors come as a packed image
// (249 registers); every other instantiation with more than one group needs the registers and the LDS of a
// whole CU.
constexpr int workgroups_per_cu(bool mv, int tp, int kind, bool vi)
{
    return !mv || tp == 2 || (tp == 4 && kind == KNM_KERNEL_GAUSSIAN && vi) ? 2 : 1;
}
// Stages in the LDS ring: 3 (two stages of loads in flight) where the rings and vector rows of the workgroups
// of a CU fit its 160 KB, 2 for the matrix-core reduction at two workgroups per CU with its 16 KB of vector
// halves per group
constexpr int ring_depth(bool mv, int tp, int kind, bool vi) { return mv && workgroups_per_cu(mv, tp, kind, vi) == 2 ? 2 : 3; }
constexpr float kPScale = 16384.0f; // matrix-core reduction: kernel values are split into fp16 halves after this scale
// Image of points [row0, row0 + 32 gridDim.x) of P (points at or beyond nP become zero
// points).  One workgroup per 32-point block; thread = (point, 8-feature unit), four
// chunks (64 features) per pass over the row.
template <int VW>
__global__ __launch_bounds__(kThreads) void pack_points_kernel(const float *__restrict__ P, int64_t nP, int64_t ld,
                                                               const float *__restrict__ mu, int d, float sigma,
                                                               int64_t row0, int n_kc, f16x8 *__restrict__ img,
                                                               unsigned int *__restrict__ range_count)
{
    const int tid = threadIdx.x;
    const int u = tid & 7;
    const int prow = tid >> 3;
    const int h = u & 1;
    const int64_t idx = row0 + (int64_t)blockIdx.x * 32 + prow;
    const bool valid = idx < nP;
    const float *row = P + (valid ? idx : 0) * ld;
    const float gamma = sqrtf(kLog2e) / sigma;
    f16x8 *blk = img + (int64_t)blockIdx.x * (n_kc + 1) * kUnits;

    float nrm = 0.0f;
    bool clamped = false;
    for (int g = 0; 4 * g < n_kc; ++g) {
        const int kc = 4 * g + (u >> 1);
        const int f0 = kChunk * kc + 8 * h;
        float z[8];
        if constexpr (VW == 4) {
#pragma unroll
            for (int k = 0; k < 8; k += 4) {
                const bool in = valid && (f0 + k < d); // d % 4 == 0 in this mode
                const f32x4 v = *reinterpret_cast<const f32x4 *>(row + (in ? f0 + k : 0));
                const f32x4 m = *reinterpret_cast<const f32x4 *>(mu + (in ? f0 + k : 0));
                z[k] = in ? v[0] - m[0] : 0.0f; z[k + 1] = in ? v[1] - m[1] : 0.0f;
                z[k + 2] = in ? v[2] - m[2] : 0.0f; z[k + 3] = in ? v[3] - m[3] : 0.0f;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool in = valid && (f0 + k < d);
                const float v = row[in ? f0 + k : 0];
                z[k] = in ? v - mu[in ? f0 + k : 0] : 0.0f;
            }
        }
        f16x8 hi, lo;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float z0 = gamma * z[e], z1 = gamma * z[e + 1];
            nrm = fmaf(z0, z0, nrm);
            nrm = fmaf(z1, z1, nrm);
            clamped |= out_of_half_range(z0) || out_of_half_range(z1);
            f16x2 ph, pl;
            split_pair(z0, z1, ph, pl);
            hi[e] = (_Float16)ph[0]; hi[e + 1] = (_Float16)ph[1];
            lo[e] = (_Float16)pl[0]; lo[e + 1] = (_Float16)pl[1];
        }
        if (kc < n_kc) {
            f16x8 *c = blk + (int64_t)kc * kUnits;
            c[32 * h + prow] = hi;
            c[64 + 32 * h + prow] = lo;
        }
    }
    nrm += __shfl_xor(nrm, 1);
    nrm += __shfl_xor(nrm, 2);
    nrm += __shfl_xor(nrm, 4);
    clamped |= !(0.5f * nrm <= kNormMax);
    const unsigned long long any = __builtin_amdgcn_ballot_w64(clamped);
    // the 8 threads of a point are 8 consecutive lanes: one count per clamped point (rare)
    if (valid && u == 0 && ((any >> ((threadIdx.x & 63) & ~7)) & 0xffull) != 0) atomicAdd(range_count, 1u);
    f16x8 *c = blk + (int64_t)n_kc * kUnits;
    if (u == 0) {
        _Float16 q[4];
        norm_digits(0.5f * nrm, q);
        f16x8 fx, st;
        fx[0] = q[0]; fx[1] = q[1]; fx[2] = q[2]; fx[3] = q[3];
        fx[4] = (_Float16)kC1; fx[5] = (_Float16)kC2; fx[6] = (_Float16)kC3; fx[7] = (_Float16)kC4;
        st[0] = (_Float16)kC1; st[1] = (_Float16)kC2; st[2] = (_Float16)kC3; st[3] = (_Float16)kC4;
        st[4] = q[0]; st[5] = q[1]; st[6] = q[2]; st[7] = q[3];
        c[prow] = fx;
        c[64 + prow] = st;
    } else if (u == 1) {
        f16x8 zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) zero[e] = (_Float16)0.0f;
        c[32 + prow] = zero;
        c[64 + 32 + prow] = zero;
    }
}

__device__ __forceinline__ void mfma_zero(f32x16 &acc, const f16x8 &a, const f16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_acc(f32x16 &acc, const f16x8 &a, const f16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// exp2 of an accumulator element with the clamp modifier (Gaussian kernel value in [0, 1]).  Volatile
// and reading the accumulator register itself: the compiler does not look inside inline assembly,
// so it must neither move this read up towards the MFMA that produces the element (it knows
// nothing of that instruction's latency) nor be relied on for the wait state a transcendental result needs before its first use.
__device__ __forceinline__ float exp2_clamped(const float &x)
{
    float p;
    asm volatile("v_exp_f32_e64 %0, %1 clamp\n\ts_nop 0" : "=v"(p) : "v"(x));
    return p;
}
// the accumulator element itself, for code the compiler schedules (same ordering argument)
__device__ __forceinline__ float acc_read(const float &x)
{
    float p;
    asm volatile("v_mov_b32 %0, %1" : "=v"(p) : "v"(x));
    return p;
}

// The second contraction uses the compiler's MFMA builtin, not inline assembly: its operands are
// rewritten by vector-ALU instructions every few cycles and its result is read by ordinary
// code, and only for an instruction it knows can the compiler keep the required distances.
__device__ __forceinline__ void mfma_accv(f32x16 &acc, const f16x8 &a, const f16x8 &b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
}

// Power of two that brings a column with largest magnitude `bits` (a float's bit pattern) into
// [2^13, 2^14), or its inverse; 1 for an all-zero (or denormal) column.
__device__ __forceinline__ float column_scale(uint32_t bits, bool inverse)
{
    const int e = (int)((bits >> 23) & 255u);
    if (e == 0 || e == 255) return 1.0f;
    const int shift = 13 - (e - 127);
    return ldexpf(1.0f, inverse ? -shift : shift);
}

// Workgroup -> (fixed block, stream chunk).  Workgroups are dealt round-robin to the 8 XCDs
// (each with its own L2) in launch order, and the ones resident together on an XCD are
// consecutive in that order.  They are therefore numbered so that each XCD works through
// "patches" of pf fixed blocks x pc chunks: the pf fixed-block images, which every
// workgroup re-reads for each of its stream tiles, stay in that XCD's L2, and a stream tile
// fetched by one workgroup is reused by the pf - 1 others on the same chunk.
struct PatchMap {
    int pf, pc;          // patch shape
    int64_t n_fblocks;   // fixed blocks of this launch
    int64_t n_chunks;    // stream chunks of this launch
    int64_t n_patch_f;   // ceil(n_fblocks / pf)
};

// Fimg: image of the fixed points [fixed_row0, fixed_row0 + 256 n_fblocks);
// Simg: image of the stream chunks [chunk0, chunk0 + n_chunks).
// TP: number of vector columns, padded to a multiple of 2 unless there is only one (vector-ALU reduction).  MV: reduce
// on the matrix cores instead, TP / 2 groups of 32 columns each (1, 2, 4 or 5: the kernel values of a
// tile are evaluated and split once and multiplied into every group; more than one group needs the
// registers and the LDS of a whole CU, so those instantiations run one workgroup per CU);
// colmax[c] = bits of max |vec[:, c]|.
// VI (with MV): the vector halves of a tile come from the packed image a.vimg (pack_vectors_kernel) by
// direct-to-LDS loads instead of being converted by the workgroup.
template <int TP, bool MV, int KIND, bool VI = false>
__global__ __launch_bounds__(kThreads, workgroups_per_cu(MV, TP, KIND, VI)) void gauss_gemm_f16_kernel(SweepArgs a, const f16x8 *__restrict__ Fimg,
                                                                     const f16x8 *__restrict__ Simg,
                                                                     int64_t fixed_row0, int64_t chunk0, int n_kc,
                                                                     PatchMap pm, const uint32_t *__restrict__ colmax)
{
    static_assert(MV || !VI, "the packed vector image belongs to the matrix-core reduction");
    const int per_patch = pm.pf * pm.pc;
    const int64_t slot = (int64_t)blockIdx.x >> 3;
    const int64_t patch = (slot / per_patch) * 8 + (blockIdx.x & 7);
    const int within = (int)(slot % per_patch);
    const int64_t fblk = (patch % pm.n_patch_f) * pm.pf + within % pm.pf;
    const int64_t cblk = (patch / pm.n_patch_f) * pm.pc + within / pm.pf;
    if (fblk >= pm.n_fblocks || cblk >= pm.n_chunks) return; // whole workgroup, before any barrier

    // Ring of operand stages (24 KB each) in dynamic LDS, filled by loads that write LDS directly, and
    // behind it the vector rows of a tile: fp32 [stream point][column], or for MV split halves in
    // A-operand layout [stream block][K-step][plane hi/lo][lane]
    constexpr int kRing = ring_depth(MV, TP, KIND, VI);
    constexpr int G = MV ? TP / 2 : 1; // column groups of the matrix-core reduction
    static_assert(!MV || TP == 2 || TP == 4 || TP == 8 || TP == 10, "1, 2, 4 or 5 groups of 32 columns");
    extern __shared__ __align__(16) unsigned char lds_dyn[];
    f16x8 *const img = reinterpret_cast<f16x8 *>(lds_dyn);
    f16x8 *const vstore = img + kRing * kStageUnits;
    float *const vimg = reinterpret_cast<float *>(vstore);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int h = lane >> 5;
    const int t = a.t;
    const int n_st = n_kc + 1; // stages per tile: the feature chunks, then the norm slots
    const float s2 = kLog2e / (2.0f * a.sigma * a.sigma); // exponent per squared distance (Laplacian refinement)

    const int64_t fixed0 = fixed_row0 + fblk * kFixed;
    const int64_t chunk = chunk0 + cblk;
    const int64_t chunk_begin = chunk * a.chunk_len;
    int64_t chunk_end = chunk_begin + a.chunk_len;
    if (chunk_end > a.nS) chunk_end = a.nS;
    const int n_tiles = (int)((chunk_end - chunk_begin + kStream - 1) / kStream);

    // staging role of this thread: unit id = tid + 256 i  ->  block id / 128, unit id % 128;
    // loads 0..3 cover the 8 fixed blocks, loads 4..5 the 4 stream blocks of a tile.  All
    // per-load and per-stage offsets are uniform, the thread's own offset fits 32 bits.
    const int64_t blk_units = (int64_t)n_st * kUnits;
    const unsigned toff = (unsigned)((tid >> 7) * (int)blk_units + (tid & (kUnits - 1)));
    const f16x8 *const fbase = Fimg + fblk * (kFixed / 32) * blk_units;
    const f16x8 *const sbase = Simg + cblk * (a.chunk_len / 32) * blk_units;

    // Vector-ALU reduction, two levels: the terms of one tile (64 per lane and fixed point) are summed
    // in fp32 from zero, and the tile sums are added into fp64 running sums, so that the rounding of a
    // long sum of same-sign terms does not grow with the length of the chunk (a plain fp32 running sum
    // over some thousand terms loses 2-3 digits of what the solver's T^-T amplifies).  With more than 12
    // columns (10 for the kernels of r) the registers do not hold a second set of sums and the fp32 sums run through the chunk.
    constexpr bool kWide = !MV && TP <= (KIND == KNM_KERNEL_GAUSSIAN ? 12 : 10);
    float sum[2][TP];
    double wide[2][kWide ? TP : 1];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int c = 0; c < TP; ++c) {
            sum[fb][c] = 0.0f;
            if constexpr (kWide) wide[fb][c] = 0.0;
        }
    // MV: output tile [column][fixed point] of each fixed block, and this thread's column scale
    f32x16 dacc[G][2];
    float vscale[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int r = 0; r < 16; ++r) dacc[g][fb][r] = 0.0f;
        vscale[g] = 1.0f;
        if constexpr (MV) vscale[g] = column_scale(colmax[32 * g + (lane & 31)], false);
    }

    // Staging.  The images are laid out as the LDS stage, so a stage is 6 loads of 16 bytes per thread
    // that go from memory into LDS without passing through registers: a wavefront's 64 units land in
    // 1 KB starting at the address in M0.  The loads of a stage are started kRing - 1 stages before it
    // is used; vmcnt counts them, and the compiler (which does not look inside inline assembly) knows
    // nothing of them, so the waits are written here as well.  Bases are uniform, the thread's own
    // byte offsets fit 32 bits.
    const unsigned lds_wave =
        __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_dyn +
                                       (unsigned)wave * 1024u);
    unsigned off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) off[i] = (toff + (unsigned)(2 * i) * (unsigned)blk_units) * 16u;
    auto issue = [&](int tile, int st, int buf) {
        const f16x8 *const fs = uniform_pointer(fbase + (int64_t)st * kUnits);
        const f16x8 *const ss = uniform_pointer(sbase + (int64_t)tile * (kStream / 32) * blk_units + (int64_t)st * kUnits);
        const unsigned l = __builtin_amdgcn_readfirstlane(lds_wave + (unsigned)buf * (unsigned)(kStageUnits * 16));
        unsigned m0_saved;
        // (one wait state between a scalar write of M0 and the load that reads it)
        asm volatile("s_mov_b32 %[keep], m0\n\t"
                     "s_mov_b32 m0, %[l]\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o0], %[fs]\n\t"
                     "s_add_u32 m0, m0, 0x1000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o1], %[fs]\n\t"
                     "s_add_u32 m0, m0, 0x1000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o2], %[fs]\n\t"
                     "s_add_u32 m0, m0, 0x1000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o3], %[fs]\n\t"
                     "s_add_u32 m0, m0, 0x1000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o0], %[ss]\n\t"
                     "s_add_u32 m0, m0, 0x1000\n\t"
                     "s_nop 0\n\t"
                     "global_load_lds_dwordx4 %[o1], %[ss]\n\t"
                     "s_mov_b32 m0, %[keep]"
                     : [keep] "=&s"(m0_saved)
                     : [l] "s"(l), [o0] "v"(off[0]), [o1] "v"(off[1]), [o2] "v"(off[2]), [o3] "v"(off[3]), [fs] "s"(fs),
                       [ss] "s"(ss)
                     : "memory", "scc");
    };
    const int total = n_tiles * n_st; // stages of this workgroup
    int issued = 0, itile = 0, ist = 0, ibuf = 0; // the next stage to start, and its ring slot
    auto issue_next = [&]() {
        if (issued < total) {
            issue(itile, ist, ibuf);
            ++issued;
            ibuf = ibuf + 1 == kRing ? 0 : ibuf + 1;
            if (++ist == n_st) {
                ist = 0;
                ++itile;
            }
        }
    };
    // The packed vector image of a tile (VI): 4 G loads per thread into the vector store behind the ring,
    // started at the tile's first stage (every wavefront has passed that stage's barrier, so it is done
    // with the previous tile's vectors) and needed at its last.
    constexpr int kVecLoads = 4 * G;
    const unsigned lds_vec = __builtin_amdgcn_readfirstlane(lds_wave + (unsigned)(kRing * kStageUnits * 16));
    const f16x8 *const vchunk =
        VI ? static_cast<const f16x8 *>(a.vimg) + (chunk * (a.chunk_len / kStream)) * (int64_t)(G * 4 * kThreads) : nullptr;
    auto issue_vectors = [&](int tile) {
        const f16x8 *const vt = vchunk + (int64_t)tile * (G * 4 * kThreads);
#pragma unroll
        for (int k4 = 0; k4 < G; ++k4) {
            const f16x8 *const b = uniform_pointer(vt + k4 * 4 * kThreads);
            const unsigned l = __builtin_amdgcn_readfirstlane(lds_vec + (unsigned)(k4 * 4 * kThreads * 16));
            unsigned m0_saved;
            asm volatile("s_mov_b32 %[keep], m0\n\t"
                         "s_mov_b32 m0, %[l]\n\t"
                         "s_nop 0\n\t"
                         "global_load_lds_dwordx4 %[o], %[b0]\n\t"
                         "s_add_u32 m0, m0, 0x1000\n\t"
                         "s_nop 0\n\t"
                         "global_load_lds_dwordx4 %[o], %[b1]\n\t"
                         "s_add_u32 m0, m0, 0x1000\n\t"
                         "s_nop 0\n\t"
                         "global_load_lds_dwordx4 %[o], %[b2]\n\t"
                         "s_add_u32 m0, m0, 0x1000\n\t"
                         "s_nop 0\n\t"
                         "global_load_lds_dwordx4 %[o], %[b3]\n\t"
                         "s_mov_b32 m0, %[keep]"
                         : [keep] "=&s"(m0_saved)
                         : [l] "s"(l), [o] "v"((unsigned)tid * 16u), [b0] "s"(b), [b1] "s"(b + kThreads), [b2] "s"(b + 2 * kThreads),
                           [b3] "s"(b + 3 * kThreads)
                         : "memory", "scc");
        }
    };
    // Start of stage g (ring slot `buf`).  Loads complete in the order they were started, so this thread's
    // loads of the stage have landed when no more loads are outstanding than were started after them: those
    // of the stages ahead (`ahead` of them, kRing - 2 unless the chunk ends) and, for kRing - 1 stage starts
    // after a tile's first, that tile's vector loads.  At a tile's last stage its vectors must have landed as
    // well, which holds once the stage loads started after them (one per stage start since) cover what is
    // allowed to be outstanding.  After the barrier everyone's loads have landed, and everyone is done
    // reading the slot of stage g - 1, which the stage kRing - 1 ahead takes over.
    static_assert(kRing == 2 || kRing == 3, "the waits below are written for at most one stage ahead");
    int g = 0, buf = 0;
    int since_vectors = kRing; // stage starts since vector loads were started (none yet)
    auto stage_begin = [&](bool first_of_tile, bool last_of_tile, int tile) {
        int ahead = total - 1 - g;
        if (ahead > kRing - 2) ahead = kRing - 2;
        bool with_vectors = false;
        if constexpr (VI) {
            if (last_of_tile) {
                if (ahead > n_st - 2) ahead = n_st - 2;
            } else {
                with_vectors = since_vectors <= kRing - 1;
            }
        }
        if (ahead > 0) {
            if (with_vectors) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads + kVecLoads) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads) : "memory");
        } else {
            if (with_vectors) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kVecLoads) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
        issue_next();
        if constexpr (VI) {
            if (first_of_tile) {
                issue_vectors(tile);
                since_vectors = 1;
            } else if (since_vectors < kRing) {
                ++since_vectors;
            }
        }
    };
    auto stage_end = [&]() {
        ++g;
        buf = buf + 1 == kRing ? 0 : buf + 1;
    };

    f32x16 acc[2][4];
    // one feature chunk: three planes against the 8 accumulators
    auto feature_stage = [&](const f16x8 *ib, auto first) {
        f16x8 bh[2], bl[2];
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
            bh[fb] = ib[(wave * 2 + fb) * kUnits + lane];
            bl[fb] = ib[(wave * 2 + fb) * kUnits + 64 + lane];
        }
        // the stream block's operands are read one block ahead of the MFMAs that use them
        f16x8 ah[2], al[2];
        ah[0] = ib[(kFixed / 32) * kUnits + lane];
        al[0] = ib[(kFixed / 32) * kUnits + 64 + lane];
#pragma unroll
        for (int sb = 0; sb < 4; ++sb) {
            const int cur = sb & 1;
            if (sb + 1 < 4) {
                ah[cur ^ 1] = ib[(kFixed / 32 + sb + 1) * kUnits + lane];
                al[cur ^ 1] = ib[(kFixed / 32 + sb + 1) * kUnits + 64 + lane];
            }
            if constexpr (decltype(first)::value) {
                mfma_zero(acc[0][sb], ah[cur], bh[0]);
                mfma_zero(acc[1][sb], ah[cur], bh[1]);
            } else {
                mfma_acc(acc[0][sb], ah[cur], bh[0]);
                mfma_acc(acc[1][sb], ah[cur], bh[1]);
            }
            mfma_acc(acc[0][sb], al[cur], bh[0]);
            mfma_acc(acc[1][sb], al[cur], bh[1]);
            mfma_acc(acc[0][sb], ah[cur], bl[0]);
            mfma_acc(acc[1][sb], ah[cur], bl[1]);
        }
    };

    for (int i = 0; i < kRing - 1; ++i) issue_next();
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int64_t stream0 = chunk_begin + (int64_t)tile * kStream;

        // first feature chunk: starts the accumulators
        stage_begin(true, false, tile);
        feature_stage(img + buf * kStageUnits, std::true_type{});
        stage_end();

        for (int st = 1; st < n_kc; ++st) {
            stage_begin(false, false, tile);
            feature_stage(img + buf * kStageUnits, std::false_type{});
            stage_end();
        }

        // last stage: the norm slots, stream role (plane 1) against fixed role (plane 0);
        // the vectors of this tile are staged with it (every wavefront has passed this
        // tile's first barrier, so it is done with the previous tile's vectors)
        if constexpr (MV && !VI) {
            // combination id = tid + 256 i: stream block id / 128, K-step (id / 64) % 2, lane id % 64
            // = (column c of the group, half hh); slot e of that lane is stream row 8 (2 q + e / 4) + 4 hh + e % 4
            const int hh = lane >> 5;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int c = 32 * g + (lane & 31);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int id = tid + kThreads * i;
                    const int sb = id >> 7, q = (id >> 6) & 1;
                    f16x8 hi, lo;
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        float v2[2];
#pragma unroll
                        for (int k = 0; k < 2; ++k) {
                            const int64_t idx = stream0 + sb * 32 + 8 * (2 * q + (e + k) / 4) + 4 * hh + (e + k) % 4;
                            const bool in = idx < chunk_end && c < t;
                            const int64_t vi = in ? idx : 0;
                            float v = a.vec[vi * a.ldv + (in ? c : 0)];
                            if (a.wgt != nullptr) v *= a.wgt[vi];
                            v2[k] = in ? v * vscale[g] : 0.0f;
                        }
                        f16x2 ph, pl;
                        split_pair(v2[0], v2[1], ph, pl);
                        hi[e] = (_Float16)ph[0]; hi[e + 1] = (_Float16)ph[1];
                        lo[e] = (_Float16)pl[0]; lo[e + 1] = (_Float16)pl[1];
                    }
                    vstore[(((g * 4 + sb) * 2 + q) * 2 + 0) * 64 + lane] = hi;
                    vstore[(((g * 4 + sb) * 2 + q) * 2 + 1) * 64 + lane] = lo;
                }
            }
        } else if constexpr (!MV) {
            for (int k = tid; k < kStream * TP; k += kThreads) {
                const int j = k / TP, c = k % TP;
                const int64_t idx = stream0 + j;
                const bool in = idx < chunk_end && c < t;
                const int64_t vi = in ? idx : 0;
                float v = a.vec[vi * a.ldv + (in ? c : 0)];
                if (a.wgt != nullptr) v *= a.wgt[vi];
                vimg[k] = in ? v : 0.0f;
            }
        }
        stage_begin(false, true, tile);
        const f16x8 *const norm_img = img + buf * kStageUnits;
        {
            const f16x8 *ib = norm_img;
            f16x8 bf[2];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) bf[fb] = ib[(wave * 2 + fb) * kUnits + lane];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                const f16x8 as = ib[(kFixed / 32 + sb) * kUnits + 64 + lane];
                mfma_acc(acc[0][sb], as, bf[0]);
                mfma_acc(acc[1][sb], as, bf[1]);
            }
        }
        stage_end();

        // finish: register r of a lane is stream row 8 (r / 4) + 4 h + r % 4 of its block
        mfma_results_ready();
        // Laplacian: per fixed point of this lane, the row and the |exponent| below which a pair is
        // taken again from differences (never for a padding row).  The norm term is read back from
        // the digits of the fixed point's norm slot (lanes 0..31 hold them).  The unrolled
        // pass leaves such pairs out (kernel value 0) and only notes that there are some; the rare
        // second pass finds them again and adds their terms.
        const float *frow[2] = {nullptr, nullptr};
        float near[2] = {0.0f, 0.0f};
        bool any_near = false;
        if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
            const f16x8 *ib = norm_img;
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const f16x8 fx = ib[(wave * 2 + fb) * kUnits + (lane & 31)];
                const float nf = kC1 * (float)fx[0] + kC2 * (float)fx[1] + kC3 * (float)fx[2] + kC4 * (float)fx[3];
                const int64_t idx = fixed0 + (wave * 2 + fb) * 32 + (lane & 31);
                const bool in = idx < a.nF;
                frow[fb] = a.F + (in ? idx : 0) * a.ldf;
                near[fb] = in ? near_pair_threshold(nf, a.d) : -INFINITY;
            }
        }
        auto kernel_value = [&](int fb, int sb, int r) -> float {
            if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
                const float x = acc_read(acc[fb][sb][r]);
                const bool nr = x > -near[fb];
                any_near |= nr;
                return nr ? 0.0f : radial_from_exponent<KIND>(x);
            } else {
                // exponent <= 0 up to rounding; the clamp modifier keeps the kernel value in [0, 1]
                return exp2_clamped(acc[fb][sb][r]);
            }
        };
        // second pass, per fixed block: the near pairs of this lane as bit 16 (sb % 2) + r of word sb / 2
        auto near_pairs = [&](int fb, uint32_t (&m)[2]) {
            m[0] = m[1] = 0u;
#pragma unroll
            for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (acc_read(acc[fb][sb][r]) > -near[fb]) m[sb >> 1] |= 1u << ((sb & 1) * 16 + r);
        };
        // takes the lowest pair off the mask: its stream row within the tile and its kernel value
        // (0 for a padding row, whose vectors are zero)
        auto pop_pair = [&](int fb, uint32_t (&m)[2], int &jl) -> float {
            const int half = m[0] != 0u ? 0 : 1;
            const int b = __builtin_ctz(m[half]);
            m[half] &= m[half] - 1u;
            const int sb = half * 2 + (b >> 4), r = b & 15;
            jl = sb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
            const int64_t j = stream0 + jl;
            if (j >= chunk_end) return 0.0f;
            return radial_from_exponent<KIND>(exact_exponent(frow[fb], a.S + j * a.lds, a.d, s2));
        };
        if constexpr (MV) {
#pragma unroll
            for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    f16x8 vh[G], vl[G];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        vh[g] = vstore[(((g * 4 + sb) * 2 + q) * 2 + 0) * 64 + lane];
                        vl[g] = vstore[(((g * 4 + sb) * 2 + q) * 2 + 1) * 64 + lane];
                    }
#pragma unroll
                    for (int fb = 0; fb < 2; ++fb) {
                        // kernel values of registers 8 q .. 8 q + 7, split into halves: K-slot e of
                        // this half-wave is the same stream row as in the vector image
                        u32x4 ph, pl;
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            // kernel values in [0, 1] times 2^14: the halves then resolve values
                            // down to 4e-9 (instead of fp16's 6e-5) relative to themselves
                            const float p0 = kPScale * kernel_value(fb, sb, 8 * q + e);
                            const float p1 = kPScale * kernel_value(fb, sb, 8 * q + e + 1);
                            const f16x2 h2 = __builtin_amdgcn_cvt_pkrtz(p0, p1);
                            const f16x2 l2 = __builtin_amdgcn_cvt_pkrtz(p0 - (float)h2[0], p1 - (float)h2[1]);
                            ph[e / 2] = __builtin_bit_cast(uint32_t, h2);
                            pl[e / 2] = __builtin_bit_cast(uint32_t, l2);
                        }
                        const f16x8 bh = __builtin_bit_cast(f16x8, ph), bl = __builtin_bit_cast(f16x8, pl);
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            mfma_accv(dacc[g][fb], vh[g], bh);
                            mfma_accv(dacc[g][fb], vh[g], bl);
                            mfma_accv(dacc[g][fb], vl[g], bh);
                        }
                    }
                }
            if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
                if (__builtin_amdgcn_ballot_w64(any_near) != 0) {
                    // The 32 columns of a group of a fixed point are spread over its two lanes (one per
                    // half-wave), so the two exchange their pairs and each adds both to its own
                    // columns, scaled like the vector image.
                    auto add_pair = [&](int fb, float p, int jl) {
                        if (p == 0.0f) return;
                        const int64_t j = stream0 + jl;
                        const float w = a.wgt != nullptr ? a.wgt[j] : 1.0f;
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int c = 32 * g + 8 * (r / 4) + 4 * h + (r % 4);
                                if (c < t)
                                    dacc[g][fb][r] = fmaf(kPScale * p * w * column_scale(colmax[c], false), a.vec[j * a.ldv + c],
                                                          dacc[g][fb][r]);
                            }
                    };
#pragma unroll
                    for (int fb = 0; fb < 2; ++fb) {
                        uint32_t m[2];
                        near_pairs(fb, m);
                        while (__builtin_amdgcn_ballot_w64((m[0] | m[1]) != 0u) != 0) {
                            int jl = 0;
                            float p = 0.0f;
                            if ((m[0] | m[1]) != 0u) p = pop_pair(fb, m, jl);
                            const float p_other = __shfl_xor(p, 32);
                            const int jl_other = __shfl_xor(jl, 32);
                            add_pair(fb, p, jl);
                            add_pair(fb, p_other, jl_other);
                        }
                    }
                }
            }
        } else {
            // the vector row of the next register is read from LDS while this one is used
            float vr[2][TP];
            auto load_row = [&](float (&dst)[TP], int it) {
                const int sb = it >> 4, r = it & 15;
                const int j = sb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if constexpr (TP % 2 == 0) {
#pragma unroll
                    for (int c2 = 0; c2 < TP; c2 += 2) {
                        const f32x2 u = *reinterpret_cast<const f32x2 *>(&vimg[j * TP + c2]);
                        dst[c2] = u[0]; dst[c2 + 1] = u[1];
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < TP; ++c) dst[c] = vimg[j * TP + c];
                }
            };
            load_row(vr[0], 0);
#pragma unroll
            for (int it = 0; it < 64; ++it) {
                const int cur = it & 1;
                if (it + 1 < 64) load_row(vr[cur ^ 1], it + 1);
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) {
                    const float p = kernel_value(fb, it >> 4, it & 15);
#pragma unroll
                    for (int c = 0; c < TP; ++c) sum[fb][c] = fmaf(p, vr[cur][c], sum[fb][c]);
                }
            }
            if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
                if (__builtin_amdgcn_ballot_w64(any_near) != 0) {
#pragma unroll
                    for (int fb = 0; fb < 2; ++fb) {
                        uint32_t m[2];
                        near_pairs(fb, m);
                        while ((m[0] | m[1]) != 0u) {
                            int jl = 0;
                            const float p = pop_pair(fb, m, jl);
#pragma unroll
                            for (int c = 0; c < TP; ++c) sum[fb][c] = fmaf(p, vimg[jl * TP + c], sum[fb][c]);
                        }
                    }
                }
            }
            if constexpr (kWide) {
#pragma unroll
                for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                    for (int c = 0; c < TP; ++c) {
                        wide[fb][c] += (double)sum[fb][c];
                        sum[fb][c] = 0.0f;
                    }
            }
        }
    }

    // partials in fp64 if asked for (a uniform choice: one base address, two element sizes)
    const bool wide_out = a.out64 != nullptr;
    char *const obase = wide_out ? reinterpret_cast<char *>(a.out64 + chunk * a.chunk_stride)
                                 : reinterpret_cast<char *>(a.out + chunk * a.chunk_stride);
    auto store = [&](int64_t at, double v) {
        if (wide_out) *reinterpret_cast<double *>(obase + at * 8) = v;
        else *reinterpret_cast<float *>(obase + at * 4) = (float)v;
    };
    mfma_results_ready();
    if constexpr (MV) {
        // register r of a lane, group g: column 32 g + 8 (r / 4) + 4 h + r % 4 of fixed point lane % 32; undo the scale
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
            const int64_t idx = fixed0 + (wave * 2 + fb) * 32 + (lane & 31);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int c = 32 * g + 8 * (r / 4) + 4 * h + (r % 4);
                    if (idx < a.nF && c < t)
                        store(idx * a.ldo + c, (double)((dacc[g][fb][r] * (1.0f / kPScale)) * column_scale(colmax[c], true)));
                }
        }
    } else {
        // the two half-waves hold different stream rows of the same fixed point
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
            const int64_t idx = fixed0 + (wave * 2 + fb) * 32 + (lane & 31);
#pragma unroll
            for (int c = 0; c < TP; ++c) {
                double v;
                if constexpr (kWide) v = wide[fb][c];
                else v = (double)sum[fb][c];
                v += __shfl_xor(v, 32);
                if (h == 0 && idx < a.nF && c < t) store(idx * a.ldo + c, v);
            }
        }
    }
}

// zeroes the head of the workspace (one thread per word)
__global__ void clear_head_kernel(uint32_t *__restrict__ head) { head[threadIdx.x] = 0u; }

// bits of max_i |vec[i, c] wgt[i]| per column (non-negative floats order like their bit patterns)
__global__ void col_absmax_kernel(const float *__restrict__ vec, int64_t ldv, const float *__restrict__ wgt, int64_t n,
                                  int t, uint32_t *__restrict__ out)
{
    const int c = threadIdx.x; // one row per workgroup and pass, lanes along its columns (t <= 256)
    float m = 0.0f;
    if (c < t)
        for (int64_t i = blockIdx.x; i < n; i += gridDim.x) {
            float v = vec[i * ldv + c];
            if (wgt != nullptr) v *= wgt[i];
            m = fmaxf(m, fabsf(v));
        }
    if (c < t && m > 0.0f) atomicMax(out + c, __float_as_uint(m));
}

// Packed vector image for the matrix-core reduction: per tile of 128 stream points and group g of 32
// columns the split halves of the scaled vector rows in A-operand layout, [g][stream block][K-step][plane
// hi/lo][lane] units of 8 halves, exactly what a workgroup would otherwise build in LDS for each of its
// tiles.  One workgroup per tile; thread = (stream block, K-step, lane) twice.
template <int G>
__global__ __launch_bounds__(kThreads) void pack_vectors_kernel(const float *__restrict__ vec, int64_t ldv,
                                                                const float *__restrict__ wgt, int64_t nS, int t,
                                                                const uint32_t *__restrict__ colmax, f16x8 *__restrict__ vimg)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int hh = lane >> 5;
    const int64_t stream0 = (int64_t)blockIdx.x * kStream;
    f16x8 *const out = vimg + (int64_t)blockIdx.x * (G * 4 * kThreads);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int c = 32 * g + (lane & 31);
        const float vscale = column_scale(colmax[c], false);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int id = tid + kThreads * i;
            const int sb = id >> 7, q = (id >> 6) & 1;
            f16x8 hi, lo;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                float v2[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int64_t idx = stream0 + sb * 32 + 8 * (2 * q + (e + k) / 4) + 4 * hh + (e + k) % 4;
                    const bool in = idx < nS && c < t;
                    const int64_t vi = in ? idx : 0;
                    float v = vec[vi * ldv + (in ? c : 0)];
                    if (wgt != nullptr) v *= wgt[vi];
                    v2[k] = in ? v * vscale : 0.0f;
                }
                f16x2 ph, pl;
                split_pair(v2[0], v2[1], ph, pl);
                hi[e] = (_Float16)ph[0]; hi[e + 1] = (_Float16)ph[1];
                lo[e] = (_Float16)pl[0]; lo[e + 1] = (_Float16)pl[1];
            }
            out[(((g * 4 + sb) * 2 + q) * 2 + 0) * 64 + lane] = hi;
            out[(((g * 4 + sb) * 2 + q) * 2 + 1) * 64 + lane] = lo;
        }
    }
}

hipError_t pack_points(const float *P, int64_t nP, int64_t ld, const float *mu, int d, float sigma, int64_t row0,
                       int64_t rows, int n_kc, f16x8 *img, unsigned int *range_count, hipStream_t stream)
{
    const dim3 grid((unsigned)(rows / 32));
    const bool a16 = (d % 4 == 0) && (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(P) & 15) == 0);
    if (a16)
        hipLaunchKernelGGL((pack_points_kernel<4>), grid, dim3(kThreads), 0, stream, P, nP, ld, mu, d, sigma, row0, n_kc, img, range_count);
    else
        hipLaunchKernelGGL((pack_points_kernel<1>), grid, dim3(kThreads), 0, stream, P, nP, ld, mu, d, sigma, row0, n_kc, img, range_count);
    return hipGetLastError();
}

constexpr int kPatch = 64;  // workgroups per patch = resident workgroups per XCD (32 CUs x 2)
constexpr int kPatchF = 8;  // fixed blocks per patch (measured: 2..8 within 4 % of each other, 64 is 25 % slower)

constexpr int kMvMinT = 8;    // columns from which the reduction against the vectors may run on the matrix cores
constexpr size_t kHeadBytes = 1024; // head of the workspace: per-column magnitude words for that path (up to 256 columns)

template <int TP, bool MV, bool VI = false>
void launch_tp(const SweepArgs &a, const f16x8 *Fimg, const f16x8 *Simg, int64_t fixed_row0, int64_t f_blocks,
               int64_t chunk0, int64_t chunks, int n_kc, const uint32_t *colmax, hipStream_t stream)
{
    PatchMap pm;
    pm.pf = kPatchF;
    pm.pc = kPatch / pm.pf;
    pm.n_fblocks = f_blocks;
    pm.n_chunks = chunks;
    pm.n_patch_f = (f_blocks + pm.pf - 1) / pm.pf;
    const int64_t n_patch_c = (chunks + pm.pc - 1) / pm.pc;
    const int64_t patches = (pm.n_patch_f * n_patch_c + 7) / 8 * 8;
    const dim3 grid((unsigned)(patches * kPatch));
    // dynamic LDS: the ring of stages and the vector rows of a tile (more than the 64 KB a kernel gets
    // without asking)
    constexpr int kVecUnits = MV ? (TP / 2) * 4 * 2 * 2 * 64 : (kStream * TP * 4 + 15) / 16;
    auto launch = [&](auto kind) {
        constexpr size_t lds_bytes = (size_t)(ring_depth(MV, TP, decltype(kind)::value, VI) * kStageUnits + kVecUnits) * sizeof(f16x8);
        // five column groups fill the register file only just for the Gaussian kernel; the kernels of r
        // (which the dispatcher gives at most 128 columns at a time) have no such instantiation
        if constexpr (MV && TP == 10 && decltype(kind)::value != KNM_KERNEL_GAUSSIAN) return;
        else {
        auto *const kernel = gauss_gemm_f16_kernel<TP, MV, decltype(kind)::value, VI>;
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return;
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, stream, a, Fimg, Simg, fixed_row0, chunk0, n_kc, pm,
                           colmax);
        }
    };
    switch (a.kind) {
    case KNM_KERNEL_LAPLACIAN: launch(std::integral_constant<int, KNM_KERNEL_LAPLACIAN>{}); break;
    case KNM_KERNEL_MATERN32: launch(std::integral_constant<int, KNM_KERNEL_MATERN32>{}); break;
    case KNM_KERNEL_MATERN52: launch(std::integral_constant<int, KNM_KERNEL_MATERN52>{}); break;
    default: launch(std::integral_constant<int, KNM_KERNEL_GAUSSIAN>{}); break;
    }
}

} // namespace

// bytes at the head of the workspace, before the images
size_t gemm_f16_head_bytes() { return kHeadBytes; }

// bytes of packed image per point
size_t gemm_f16_pack_bytes_per_point(int d) { return (size_t)((d + kChunk - 1) / kChunk + 1) * 64; }

// least workspace: the smaller operand whole plus one slab unit of the other
size_t gemm_f16_min_pack_bytes(int64_t nF, int64_t nS_padded, int64_t chunk_len, int d)
{
    const size_t pp = gemm_f16_pack_bytes_per_point(d);
    const size_t f = (size_t)((nF + kFixed - 1) / kFixed * kFixed) * pp, s = (size_t)nS_padded * pp;
    return kHeadBytes + (f <= s ? f + (size_t)chunk_len * pp : s + (size_t)kFixed * pp);
}

int gemm_f16_max_t(int kind) { return kind == KNM_KERNEL_GAUSSIAN ? 160 : 128; }

// Matrix-core reduction when it pays: from kMvMinT columns on, unless the cross term is so long
// (large d) that the vector-ALU reduction hides behind it anyway.  Above 16 columns it is the
// only path.
static bool reduce_on_matrix_cores(int d, int t)
{
    const int n_kc = (d + kChunk - 1) / kChunk;
    return t > 16 || (t >= kMvMinT && 4 * (3 + t) >= 3 * n_kc + 1);
}
static int column_groups(int t) { return t <= 32 ? 1 : (t <= 64 ? 2 : (t <= 128 ? 4 : 5)); }

size_t gemm_f16_vector_image_bytes(int d, int t, int64_t nS_padded)
{
    if (t <= 0 || t > gemm_f16_max_t(KNM_KERNEL_GAUSSIAN) || !reduce_on_matrix_cores(d, t)) return 0;
    return (size_t)(nS_padded / kStream) * (size_t)(column_groups(t) * 4 * kThreads) * sizeof(f16x8);
}

// Columns to take in the next launch when t_left are still to do.  64 or 128 columns evaluate the kernel
// values once for all of them but run one workgroup per CU.  With the packed vector image that is faster
// at every d (per 1e11 kernel entries, d = 28: 0.187 s for 128 columns in one launch against 0.320 s in
// four; d = 256: 0.438 s against 1.144 s).  Without the image every workgroup converts the vector rows of
// its tiles itself, and with one workgroup per CU nothing hides that: the launches then measured about
// (0.015 k + 0.06) s for up to 32 columns, (0.016 k + 0.36) s for 64 and (0.016 k + 0.68) s for 128, with
// k = ceil(d / 16) chunks of features, so the wide launches pay only once the cross term is long.
int gemm_f16_group_t(int d, int t_left, int kind, bool with_vector_image)
{
    if (with_vector_image) return gemm_f16_max_t(kind); // (more than 128 columns at once only this way)
    const int n_kc = (d + kChunk - 1) / kChunk;
    if (t_left > 96 && n_kc >= 10) return 128; // in place of four launches
    if (t_left > 64 && n_kc >= 17) return 128; // in place of three
    if (t_left > 32 && n_kc >= 17) return 64;  // in place of two
    return 32;
}

hipError_t launch_sweep_gemm_f16(const SweepArgs &a, void *pack_buf, size_t pack_bytes, hipStream_t stream)
{
    if (a.nF <= 0 || a.nS <= 0 || a.n_chunks <= 0 || a.t <= 0 || a.t > gemm_f16_max_t(a.kind)) return hipErrorInvalidValue;
    if (a.kind < KNM_KERNEL_GAUSSIAN || a.kind > KNM_KERNEL_MATERN52) return hipErrorInvalidValue;
    if (a.chunk_len % kStream != 0 || a.n_chunks * a.chunk_len < a.nS) return hipErrorInvalidValue;
    if (a.n_chunks > 65535) return hipErrorInvalidValue;
    const int n_kc = (a.d + kChunk - 1) / kChunk;
    const size_t pp = gemm_f16_pack_bytes_per_point(a.d);
    const int64_t nFp = (a.nF + kFixed - 1) / kFixed * kFixed;
    const int64_t nSp = a.n_chunks * a.chunk_len;
    const size_t bytesF = (size_t)nFp * pp, bytesS = (size_t)nSp * pp;
    if (pack_bytes < gemm_f16_min_pack_bytes(a.nF, nSp, a.chunk_len, a.d)) return hipErrorInvalidValue;

    // slab sizes: the smaller operand is packed whole, the other in slabs that fill the rest
    const size_t room = pack_bytes - kHeadBytes;
    int64_t f_slab = nFp, s_slab = a.n_chunks; // fixed rows / stream chunks per slab
    if (bytesF + bytesS > room) {
        if (bytesF <= bytesS) s_slab = (int64_t)((room - bytesF) / ((size_t)a.chunk_len * pp));
        else f_slab = (int64_t)((room - bytesS) / ((size_t)kFixed * pp)) * kFixed;
    }
    if (f_slab < kFixed || s_slab < 1) return hipErrorInvalidValue;
    uint32_t *colmax = static_cast<uint32_t *>(pack_buf);
    f16x8 *Fimg = reinterpret_cast<f16x8 *>(static_cast<char *>(pack_buf) + kHeadBytes);
    const int64_t f_rows_max = f_slab < nFp ? f_slab : nFp;
    f16x8 *Simg = Fimg + (size_t)f_rows_max * pp / sizeof(f16x8);
    const bool mv = reduce_on_matrix_cores(a.d, a.t);
    if (mv) {
        // largest magnitude of every vector column: the power-of-two scale into the fp16 range
        // cleared by a kernel, not a memset node: the product entry points may be captured into a graph
        hipLaunchKernelGGL(clear_head_kernel, dim3(1), dim3(kHeadBytes / sizeof(uint32_t)), 0, stream, colmax);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        int64_t blocks = a.nS;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(col_absmax_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a.vec, a.ldv, a.wgt, a.nS,
                           a.t, colmax);
        if (a.vimg != nullptr) {
            // the vectors of the whole stream, converted once (the scales are on the device by now: same stream)
            const dim3 vgrid((unsigned)(nSp / kStream));
            f16x8 *const vimg = static_cast<f16x8 *>(a.vimg);
            switch (column_groups(a.t)) {
            case 1: hipLaunchKernelGGL(pack_vectors_kernel<1>, vgrid, dim3(kThreads), 0, stream, a.vec, a.ldv, a.wgt, a.nS, a.t, colmax, vimg); break;
            case 2: hipLaunchKernelGGL(pack_vectors_kernel<2>, vgrid, dim3(kThreads), 0, stream, a.vec, a.ldv, a.wgt, a.nS, a.t, colmax, vimg); break;
            case 4: hipLaunchKernelGGL(pack_vectors_kernel<4>, vgrid, dim3(kThreads), 0, stream, a.vec, a.ldv, a.wgt, a.nS, a.t, colmax, vimg); break;
            default: hipLaunchKernelGGL(pack_vectors_kernel<5>, vgrid, dim3(kThreads), 0, stream, a.vec, a.ldv, a.wgt, a.nS, a.t, colmax, vimg); break;
            }
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    for (int64_t f0 = 0; f0 < nFp; f0 += f_slab) {
        const int64_t f_rows = (nFp - f0 < f_slab) ? nFp - f0 : f_slab;
        hipError_t e = pack_points(a.F, a.nF, a.ldf, a.mu, a.d, a.sigma, f0, f_rows, n_kc, Fimg, a.range_count, stream);
        if (e != hipSuccess) return e;
        for (int64_t c0 = 0; c0 < a.n_chunks; c0 += s_slab) {
            const int64_t nc = (a.n_chunks - c0 < s_slab) ? a.n_chunks - c0 : s_slab;
            if (f0 == 0 || s_slab < a.n_chunks) { // a whole stream image is built once
                e = pack_points(a.S, a.nS, a.lds, a.mu, a.d, a.sigma, c0 * a.chunk_len, nc * a.chunk_len, n_kc, Simg, a.range_count, stream);
                if (e != hipSuccess) return e;
            }
            const int64_t fb = f_rows / kFixed;
            if (mv && a.vimg != nullptr) {
                if (a.t <= 32) launch_tp<2, true, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else if (a.t <= 64) launch_tp<4, true, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else if (a.t <= 128) launch_tp<8, true, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else launch_tp<10, true, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
            } else if (mv) {
                if (a.t <= 32) launch_tp<2, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else if (a.t <= 64) launch_tp<4, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else if (a.t <= 128) launch_tp<8, true>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                else return hipErrorInvalidValue; // more than 128 columns only with the packed vector image
            } else {
                if (a.t == 1) { // one column: no padded second one
                    launch_tp<1, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream);
                } else
                switch ((a.t + 1) / 2) {
                case 1: launch_tp<2, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 2: launch_tp<4, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 3: launch_tp<6, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 4: launch_tp<8, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 5: launch_tp<10, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 6: launch_tp<12, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                case 7: launch_tp<14, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                default: launch_tp<16, false>(a, Fimg, Simg, f0, fb, c0, nc, n_kc, colmax, stream); break;
                }
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

} // namespace knm
