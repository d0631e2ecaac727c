// C ABI of libknm: context, workspace and the kernel-matrix-vector products.
#include <dlfcn.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "knm_internal.h"

namespace knm {

namespace {
struct MarkerApi {
    int (*push)(const char *) = nullptr;
    int (*pop)() = nullptr;
};
const MarkerApi &marker_api()
{
    static MarkerApi api;
    static std::once_flag once;
    std::call_once(once, [] {
        const char *want = std::getenv("KNM_MARKERS");
        if (!want || !*want || std::strcmp(want, "0") == 0) return;
        for (const char *lib : {"librocprofiler-sdk-roctx.so", "libroctx64.so"}) {
            void *h = dlopen(lib, RTLD_NOW | RTLD_GLOBAL);
            if (!h) continue;
            auto push = reinterpret_cast<int (*)(const char *)>(dlsym(h, "roctxRangePushA"));
            auto pop = reinterpret_cast<int (*)()>(dlsym(h, "roctxRangePop"));
            if (push && pop) {
                api.push = push;
                api.pop = pop;
                return;
            }
        }
    });
    return api;
}
} // namespace

TraceRange::TraceRange(const char *name) : open(false)
{
    const MarkerApi &api = marker_api();
    if (api.push) {
        (void)api.push(name);
        open = true;
    }
}
TraceRange::~TraceRange()
{
    if (open) (void)marker_api().pop();
}

int fail(knm_ctx *ctx, int status, const char *what, hipError_t e)
{
    if (ctx) {
        ctx->last_error = what ? what : "";
        if (e != hipSuccess) {
            ctx->last_error += ": ";
            ctx->last_error += hipGetErrorString(e);
        }
    }
    return status;
}

int ensure(knm_ctx *ctx, float **buf, size_t *cur, size_t need)
{
    if (*cur >= need) return KNM_OK;
    if (*buf) {
        hipError_t e = hipFree(*buf);
        *buf = nullptr;
        *cur = 0;
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipFree(workspace)", e);
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, need);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, KNM_ALLOC, "hipMalloc(workspace)", e);
    }
    *buf = static_cast<float *>(p);
    *cur = need;
    return KNM_OK;
}

// Workspace for callers that cannot allocate (code under HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): one array per GPU, held from the loading of the library to the
// end of the process.  Host code never uses this name as an address: knm_create looks up the
// device's own copy with hipGetSymbolAddress and keeps the pointer in the context.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr size_t kVectorImageCap = (size_t)16 << 30; // largest packed vector image the library allocates
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// One piece of a sweep's workspace: grown on demand in the context's own buffer, or, in a call that
// must not allocate, carved from the static scratch (KNM_UNSUPPORTED if it does not fit).
static int acquire(knm_ctx *ctx, float **buf, size_t *cur, size_t need, float **out)
{
    if (!ctx->static_mode) {
        int st = ensure(ctx, buf, cur, need);
        *out = *buf;
        return st;
    }
    const size_t at = (ctx->static_used + 255) & ~(size_t)255;
    if (ctx->static_ws == nullptr || at + need > kStaticScratchBytes)
        return fail(ctx, KNM_UNSUPPORTED, "problem too large for the static scratch of the allocation-free entry point");
    *out = reinterpret_cast<float *>(ctx->static_ws + at);
    ctx->static_used = at + need;
    return KNM_OK;
}

// K-loop engine for several columns or for d beyond what the register-resident engine of the
// selected arithmetic holds (44 features for the split-fp16 one, 64 for fp32)
bool use_gemm_engine(int d, int t, int cross_term, int kind)
{
    // (the kernels of r = |x - c| run on the register-resident engine only with the split-fp16 cross
    // term, and up to the d its two smaller layouts hold without register spills)
    if (kind != KNM_KERNEL_GAUSSIAN && (cross_term != KNM_CROSS_F16X3 || d > f16_radial_max_d())) return true;
    return t > 1 || d > (cross_term == KNM_CROSS_F16X3 ? f16_max_d() : small_max_d());
}

// Chunking of the stream dimension.  More chunks = more workgroups (needed when there
// are few fixed blocks) and shorter fp32 running sums; each chunk costs one partial
// vector that the merge pass adds up in fp64.
int64_t choose_chunks(int64_t nF, int64_t nS, int d, int t, int cross_term, int kind, int64_t *chunk_len)
{
    const bool gemm = use_gemm_engine(d, t, cross_term, kind);
    const int64_t stage = gemm ? gemm_stage_points()
                               : (cross_term == KNM_CROSS_F16X3 ? f16_stage_points(d, kind) : stage_points());
    const int64_t per_block = gemm ? gemm_fixed_per_block() : fixed_per_block(d);
    const int64_t blocks = (nF + per_block - 1) / per_block;
    const int64_t target_wgs = 4096;       // several waves of workgroups over 256 CUs
    const int64_t min_len = gemm ? 16 * stage : 2048; // amortise the per-workgroup prologue/epilogue
    const int64_t max_len = (int64_t)1 << 18; // bound the length of a per-lane fp32 running sum
    int64_t chunks = (target_wgs + blocks - 1) / blocks;
    if (gemm && chunks < 16) chunks = 16;  // the K-loop engine tiles (fixed blocks x chunks) over each XCD's L2
    const int64_t max_chunks_by_len = (nS + min_len - 1) / min_len;
    if (chunks > max_chunks_by_len) chunks = max_chunks_by_len;
    const int64_t min_chunks_by_len = (nS + max_len - 1) / max_len;
    if (chunks < min_chunks_by_len) chunks = min_chunks_by_len;
    if (chunks < 1) chunks = 1;
    int64_t len = (nS + chunks - 1) / chunks;
    len = (len + stage - 1) / stage * stage;
    chunks = (nS + len - 1) / len;
    *chunk_len = len;
    return chunks;
}

static bool bad_geom(const void *X, int64_t n, int d, int64_t ldx, const void *C, int64_t M, int64_t ldc,
                     float sigma, int t)
{
    return !X || !C || n <= 0 || M <= 0 || d <= 0 || t <= 0 || ldx < d || ldc < d || !(sigma > 0.0f);
}

// mu[k] = mean of feature k over `rows` rows of P taken `stride` rows apart (a sample spread over the
// whole set, so that data stored in some order still gives a representative centre): the common shift
// of a sweep's two point sets.  One workgroup per 32 features, 32 row lanes per feature with four
// loads in flight each, fp64 sums in a fixed order.
constexpr int kMeanRowLanes = 32;
constexpr int64_t kMeanSample = 16384; // rows of the sample at most
__global__ __launch_bounds__(32 * kMeanRowLanes) void column_mean_kernel(const float *__restrict__ P, int64_t rows,
                                                                        int64_t stride, int64_t ld, int d,
                                                                        float *__restrict__ mu)
{
    __shared__ double part[kMeanRowLanes][32];
    const int f = threadIdx.x & 31, rl = threadIdx.x >> 5;
    const int k = blockIdx.x * 32 + f;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    if (k < d) {
        const float *col = P + k;
        const int64_t step = stride * ld;
        int64_t r = rl;
        for (; r + 3 * kMeanRowLanes < rows; r += 4 * kMeanRowLanes) {
            const float a0 = col[r * step], a1 = col[(r + kMeanRowLanes) * step];
            const float a2 = col[(r + 2 * kMeanRowLanes) * step], a3 = col[(r + 3 * kMeanRowLanes) * step];
            s0 += (double)a0;
            s1 += (double)a1;
            s2 += (double)a2;
            s3 += (double)a3;
        }
        for (; r < rows; r += kMeanRowLanes) s0 += (double)col[r * step];
    }
    part[rl][f] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (rl == 0 && k < d) {
        double total = 0.0;
        for (int i = 0; i < kMeanRowLanes; ++i) total += part[i][f];
        const float m = (float)(total / (double)rows);
        mu[k] = (m == m && fabsf(m) < 3.0e38f) ? m : 0.0f; // a NaN or Inf in the data must not spread to every point
    }
}

// Keeps the shift only where it pays: if the mean itself is within sigma of the origin
// (|mu|^2 / 2 sigma^2 <= 0.5) the norm terms are small anyway, and mu is set to zero, which leaves the
// points exactly as they are (data with many exact zeros keeps them: the matrix cores draw less
// power on such operands, and the sweep runs measurably faster).  One workgroup.
__global__ __launch_bounds__(256) void shift_decide_kernel(float *__restrict__ mu, int d, float inv2s2)
{
    __shared__ float part[256];
    float s = 0.0f;
    for (int k = threadIdx.x; k < d; k += 256) s = fmaf(mu[k], mu[k], s);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    const bool keep = part[0] * inv2s2 > 0.5f;
    if (!keep)
        for (int k = threadIdx.x; k < d; k += 256) mu[k] = 0.0f;
    if (threadIdx.x == 0) mu[d] = keep ? 1.0f : 0.0f; // lets the hot loops skip the loads of an all-zero shift
}

// Bytes of the packed-operand workspace one sweep asks for in the split-fp16 modes (0 in the
// fp32-MFMA mode): the same rule for the sweep itself and for knm_workspace_bytes.  `limit` = the
// caller's cap, 0 for the defaults.
static size_t pack_bytes_wanted(int64_t nF, int d, int t, int kind, size_t limit, int64_t chunks, int64_t chunk_len)
{
    if (use_gemm_engine(d, t, KNM_CROSS_F16X3, kind)) {
        // packed images of both operands: whole if they fit 8 GiB, else the smaller one
        // whole and the other in slabs
        const size_t per_point = gemm_f16_pack_bytes_per_point(d);
        const int64_t nFp = (nF + gemm_fixed_per_block() - 1) / gemm_fixed_per_block() * gemm_fixed_per_block();
        size_t want = gemm_f16_head_bytes() + per_point * (size_t)(nFp + chunks * chunk_len); // head + both images
        const size_t cap = limit ? limit : (size_t)8 << 30;
        const size_t least = gemm_f16_min_pack_bytes(nF, chunks * chunk_len, chunk_len, d);
        if (want > cap) want = cap;
        if (want < least) want = least;
        return want;
    }
    // packed image of the stream points: all of it, or slabs of at most 2 GiB
    const size_t per_point = f16_pack_bytes_per_point(d);
    size_t want = per_point * (size_t)(chunks * chunk_len);
    const size_t cap = limit ? limit : (size_t)2 << 30;
    if (want > cap) want = (cap / (per_point * chunk_len) + 1) * per_point * chunk_len;
    return want;
}

// out[f, c] = sum_s k(F_f, S_s) vec[s, c] wgt[s]  for c < t (all arrays leading dimension t); the
// result goes to `out` (fp32) or, if that is null, to `out64`: then the chunk partials of the K-loop
// engines stay in fp64 from the kernels' running sums to the merged result
static int sweep(knm_ctx *ctx, const float *F, int64_t nF, int64_t ldf, const float *S, int64_t nS, int64_t lds,
                 int d, float sigma, const float *vec, const float *wgt, int t, float *out, double *out64,
                 hipEvent_t after_sweep)
{
    int64_t chunk_len = 0;
    const int64_t chunks = choose_chunks(nF, nS, d, t, ctx->cross_term, ctx->kernel_kind, &chunk_len);
    if (chunks > 65535) return fail(ctx, KNM_UNSUPPORTED, "too many stream chunks");
    const bool gemm = use_gemm_engine(d, t, ctx->cross_term, ctx->kernel_kind);
    if (gemm && ctx->cross_term == KNM_CROSS_F32 && (!gemm_leading_dimension_ok(ldf) || !gemm_leading_dimension_ok(lds)))
        return fail(ctx, KNM_UNSUPPORTED, "leading dimension above 5.5 million elements in the fp32-MFMA K-loop engine");
    const bool part_is_64 = out64 != nullptr && gemm;
    const bool merged = chunks > 1 || out64 != nullptr; // an fp64 result is always written by the merge pass
    if (ctx->static_mode) ctx->static_used = 0; // every sweep carves its pieces afresh
    float *part = nullptr;
    if (merged) {
        int st = acquire(ctx, &ctx->part_buf, &ctx->part_bytes,
                         (part_is_64 ? sizeof(double) : sizeof(float)) * (size_t)chunks * nF * t, &part);
        if (st) return st;
    }
    // common shift: feature means of (a strided sample of at most 16384 rows of) the smaller point set
    float *mu = nullptr;
    {
        int st = acquire(ctx, &ctx->mu_buf, &ctx->mu_bytes, sizeof(float) * ((size_t)d + 1), &mu); // + the "shifted" flag
        if (st) return st;
        const bool from_f = nF <= nS;
        const int64_t rows = from_f ? nF : nS;
        const int64_t stride = (rows + kMeanSample - 1) / kMeanSample; // every stride-th row, spread over the set
        hipLaunchKernelGGL(column_mean_kernel, dim3((unsigned)((d + 31) / 32)), dim3(32 * kMeanRowLanes), 0, ctx->stream,
                           from_f ? F : S, (rows + stride - 1) / stride, stride, from_f ? ldf : lds, d, mu);
        hipLaunchKernelGGL(shift_decide_kernel, dim3(1), dim3(256), 0, ctx->stream, mu, d,
                           1.0f / (2.0f * sigma * sigma));
        if (hipGetLastError() != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "column_mean_kernel launch");
    }
    // columns per launch
    int group = 1;
    for (int c = 0; c < t; c += group) {
        // (K-loop split-fp16 engine: wide launches when the vectors can be given as a packed image, which a
        // call that must not allocate does without, as does one whose image would be very large)
        bool vector_image = gemm && ctx->cross_term == KNM_CROSS_F16X3 && !ctx->static_mode;
        if (vector_image) {
            const int wide = gemm_f16_group_t(d, t - c, ctx->kernel_kind, true);
            vector_image = gemm_f16_vector_image_bytes(d, t - c < wide ? t - c : wide, chunks * chunk_len) <= kVectorImageCap;
        }
        group = !gemm ? 1 : (ctx->cross_term == KNM_CROSS_F16X3 ? gemm_f16_group_t(d, t - c, ctx->kernel_kind, vector_image) : gemm_max_t());
        SweepArgs a;
        a.F = F; a.nF = nF; a.ldf = ldf;
        a.S = S; a.nS = nS; a.lds = lds;
        a.d = d;
        a.mu = mu;
        a.range_count = ctx->range_count;
        a.vec = vec + c; a.ldv = t;
        a.t = (t - c < group) ? t - c : group;
        a.wgt = wgt;
        a.out = merged ? part + c : out + c;
        a.out64 = part_is_64 ? reinterpret_cast<double *>(part) + c : nullptr;
        a.ldo = t;
        a.chunk_stride = nF * t;
        a.chunk_len = chunk_len;
        a.n_chunks = chunks;
        // Kernels of r = |x - c|: with sigma / (c sqrt(2 log2 e)) in place of sigma the engines'
        // accumulators hold -(log2(e) c r / sigma)^2, whose root the kernel takes before the exp2
        // (c = 1 Laplacian, sqrt(3) and sqrt(5) for the two Matern kernels)
        a.kind = ctx->kernel_kind;
        const float c_kind = a.kind == KNM_KERNEL_MATERN32 ? 1.7320508075688772f
                             : a.kind == KNM_KERNEL_MATERN52 ? 2.23606797749979f : 1.0f;
        a.sigma = (a.kind == KNM_KERNEL_GAUSSIAN) ? sigma : sigma / (c_kind * sqrtf(2.0f * 1.4426950408889634f));
        const bool f16 = !gemm && ctx->cross_term == KNM_CROSS_F16X3 && d <= f16_max_d();
        hipError_t e;
        // packed operands of the split-fp16 engines: what the engine would like, or (static scratch)
        // as many whole slabs as the rest of the scratch holds; the same region serves every column group
        auto pack_room = [&](size_t *want) -> int {
            *want = pack_bytes_wanted(nF, d, t, ctx->kernel_kind, ctx->pack_limit, chunks, chunk_len);
            if (!ctx->static_mode) return KNM_OK;
            const size_t at = (ctx->static_used + 255) & ~(size_t)255;
            const size_t room = at < kStaticScratchBytes ? kStaticScratchBytes - at : 0;
            if (gemm) {
                const size_t least = gemm_f16_min_pack_bytes(nF, chunks * chunk_len, chunk_len, d);
                if (*want > room) *want = room;
                if (*want < least) *want = least; // acquire() then reports that it does not fit
            } else {
                const size_t per_chunk = f16_pack_bytes_per_point(d) * (size_t)chunk_len;
                const size_t fit = room / per_chunk * per_chunk;
                if (*want > fit) *want = fit > 0 ? fit : per_chunk;
            }
            return KNM_OK;
        };
        float *pack = nullptr;
        const size_t mark_used = ctx->static_used;
        if (gemm && ctx->cross_term == KNM_CROSS_F16X3) {
            size_t want = 0;
            int st = pack_room(&want);
            if (!st) st = acquire(ctx, &ctx->pack_buf, &ctx->pack_bytes, want, &pack);
            if (st) return st;
            // the vectors as a packed image, when the matrix-core reduction runs and the image is of moderate
            // size (a call that must not allocate leaves the conversion to the workgroups)
            const size_t vbytes = vector_image ? gemm_f16_vector_image_bytes(d, a.t, chunks * chunk_len) : 0;
            if (vbytes > 0) {
                st = ensure(ctx, &ctx->vimg_buf, &ctx->vimg_bytes, vbytes);
                if (st) return st;
                a.vimg = ctx->vimg_buf;
            }
            e = launch_sweep_gemm_f16(a, pack, want, ctx->stream);
        } else if (gemm) {
            e = launch_sweep_gemm(a, ctx->stream);
        } else if (f16) {
            size_t want = 0;
            int st = pack_room(&want);
            if (!st) st = acquire(ctx, &ctx->pack_buf, &ctx->pack_bytes, want, &pack);
            if (st) return st;
            e = launch_sweep_f16(a, pack, want, ctx->stream);
        } else {
            e = launch_sweep(a, ctx->stream);
        }
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "launch_sweep", e);
        ctx->static_used = mark_used; // the next column group reuses the image region (same stream: ordered)
    }
    if (after_sweep) (void)hipEventRecord(after_sweep, ctx->stream);
    if (merged) {
        hipError_t e = launch_merge(part_is_64 ? nullptr : part, part_is_64 ? reinterpret_cast<double *>(part) : nullptr,
                                    chunks, nF * t, 1, out64 != nullptr ? nullptr : out, out64, 1, nF * t, ctx->stream);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "launch_merge", e);
    }
    return KNM_OK;
}

static void mark(knm_ctx *ctx, int i)
{
    if (ctx->timing) {
        (void)hipEventRecord(ctx->ev[i], ctx->stream);
        ctx->ev_used[i] = true;
    }
}

static void begin_timing(knm_ctx *ctx)
{
    for (int i = 0; i < 5; ++i) ctx->ev_used[i] = false;
    mark(ctx, 0);
}

int do_knm_v(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
             int64_t ldc, float sigma, const float *V, int t, float *W)
{
    TraceRange range("knm row sweep W = K V");
    return sweep(ctx, X, n, ldx, C, M, ldc, d, sigma, V, nullptr, t, W, nullptr, nullptr);
}

int do_knm_t_w(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
               int64_t ldc, float sigma, const float *Wv, const float *wgt, int t, float *U, double *U64)
{
    hipEvent_t ev = nullptr;
    if (ctx->timing) {
        ev = ctx->ev[2];
        ctx->ev_used[2] = true;
    }
    TraceRange range("knm column sweep U = K^T W");
    return sweep(ctx, C, M, ldc, X, n, ldx, d, sigma, Wv, wgt, t, U64 != nullptr ? nullptr : U, U64, ev);
}

} // namespace knm

using namespace knm;

extern "C" {

int knm_create(knm_ctx **out, int device, void *hip_stream)
{
    if (!out) return KNM_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return KNM_INVALID_ARG;
    if (hipSetDevice(device) != hipSuccess) return KNM_HIP_ERROR;
    knm_ctx *ctx = new (std::nothrow) knm_ctx();
    if (!ctx) return KNM_ALLOC;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    {
        // this device's copy of the static scratch array (the device is current)
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            delete ctx;
            return KNM_HIP_ERROR;
        }
        ctx->static_ws = static_cast<unsigned char *>(ptr);
    }
    for (int i = 0; i < 5; ++i) {
        if (hipEventCreate(&ctx->ev[i]) != hipSuccess) {
            (void)knm_destroy(ctx);
            return KNM_HIP_ERROR;
        }
    }
    {
        // the word the split-fp16 engines count clamped operands in (allocated here so that the
        // products themselves never allocate for it)
        void *w = nullptr;
        if (hipMalloc(&w, 256) != hipSuccess || hipMemset(w, 0, 256) != hipSuccess) {
            (void)hipGetLastError();
            if (w) (void)hipFree(w);
            (void)knm_destroy(ctx);
            return KNM_ALLOC;
        }
        ctx->range_count = static_cast<unsigned int *>(w);
    }
    *out = ctx;
    return KNM_OK;
}

int knm_destroy(knm_ctx *ctx)
{
    if (!ctx) return KNM_INVALID_ARG;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->w_buf) (void)hipFree(ctx->w_buf);
    if (ctx->part_buf) (void)hipFree(ctx->part_buf);
    if (ctx->pack_buf) (void)hipFree(ctx->pack_buf);
    if (ctx->vimg_buf) (void)hipFree(ctx->vimg_buf);
    if (ctx->mu_buf) (void)hipFree(ctx->mu_buf);
    if (ctx->range_count) (void)hipFree(ctx->range_count);
    for (int i = 0; i < 5; ++i)
        if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    extern void knm_solver_release(knm_ctx *);
    knm_solver_release(ctx);
    delete ctx;
    return KNM_OK;
}

const char *knm_strerror(int status)
{
    switch (status) {
    case KNM_OK: return "ok";
    case KNM_INVALID_ARG: return "invalid argument";
    case KNM_UNSUPPORTED: return "shape not supported by the compiled kernels";
    case KNM_ALLOC: return "device workspace allocation failed";
    case KNM_HIP_ERROR: return "HIP runtime or library error";
    case KNM_NOT_PD: return "matrix not positive definite in Cholesky factorisation";
    default: return "unknown status";
    }
}

const char *knm_last_error(const knm_ctx *ctx) { return ctx ? ctx->last_error.c_str() : ""; }

int knm_max_d(void) { return 65536; }
int knm_max_t(void) { return 1024; }

size_t knm_workspace_bytes(int64_t n, int64_t M, int d, int t)
{
    if (n <= 0 || M <= 0 || d <= 0 || t <= 0) return 0;
    int64_t len = 0;
    const size_t bytes = sizeof(float) * (size_t)n * t; // W
    // the largest needs over the arithmetic modes and kernel functions (they may cut the stream
    // differently): chunk partials, and the packed operands of the split-fp16 modes
    size_t part = 0, pack = 0, vimg = 0;
    for (int mode = 0; mode < 4; ++mode) {
        const int cross = mode & 1, kind = mode >> 1;
        const int64_t c1 = choose_chunks(n, M, d, t, cross, kind, &len);
        const int64_t l1 = len;
        const int64_t c2 = choose_chunks(M, n, d, t, cross, kind, &len);
        const int64_t l2 = len;
        const size_t p1 = c1 > 1 ? sizeof(float) * (size_t)c1 * n * t : 0;
        const size_t p2 = c2 > 1 ? sizeof(float) * (size_t)c2 * M * t : 0;
        if (p1 > part) part = p1;
        if (p2 > part) part = p2;
        if (cross == KNM_CROSS_F16X3) {
            const bool packs = use_gemm_engine(d, t, cross, kind) || d <= f16_max_d();
            const size_t k1 = packs ? pack_bytes_wanted(n, d, t, kind, 0, c1, l1) : 0;
            const size_t k2 = packs ? pack_bytes_wanted(M, d, t, kind, 0, c2, l2) : 0;
            if (k1 > pack) pack = k1;
            if (k2 > pack) pack = k2;
            if (use_gemm_engine(d, t, cross, kind)) {
                // packed vector image of the widest launch (matrix-core reduction), for either sweep
                const int wide = t < gemm_f16_max_t(kind) ? t : gemm_f16_max_t(kind);
                const size_t v1 = gemm_f16_vector_image_bytes(d, wide, c1 * l1), v2 = gemm_f16_vector_image_bytes(d, wide, c2 * l2);
                if (v1 <= kVectorImageCap && v1 > vimg) vimg = v1;
                if (v2 <= kVectorImageCap && v2 > vimg) vimg = v2;
            }
        }
    }
    return bytes + part + pack + vimg + sizeof(float) * ((size_t)d + 1);
}

size_t knm_workspace_held(const knm_ctx *ctx)
{
    return ctx ? ctx->w_bytes + ctx->part_bytes + ctx->pack_bytes + ctx->vimg_bytes + ctx->mu_bytes : 0;
}

static int check_common(knm_ctx *ctx, const void *X, int64_t n, int d, int64_t ldx, const void *C, int64_t M,
                        int64_t ldc, float sigma, int t)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (bad_geom(X, n, d, ldx, C, M, ldc, sigma, t)) return fail(ctx, KNM_INVALID_ARG, "bad shape or pointer");
    if (d > knm_max_d() || t > knm_max_t()) return fail(ctx, KNM_UNSUPPORTED, "d or t above compiled maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    return KNM_OK;
}

int knm_v(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M, int64_t ldc,
          float sigma, const float *V, int t, float *W)
{
    int st = check_common(ctx, X, n, d, ldx, C, M, ldc, sigma, t);
    if (st) return st;
    if (!V || !W) return fail(ctx, KNM_INVALID_ARG, "null vector");
    begin_timing(ctx);
    st = do_knm_v(ctx, X, n, d, ldx, C, M, ldc, sigma, V, t, W);
    mark(ctx, 1);
    mark(ctx, 4);
    return st;
}

static int prod_impl(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
                     int64_t ldc, float sigma, const float *dw, const float *V, int t, float *W_or_null, float *U)
{
    int st = check_common(ctx, X, n, d, ldx, C, M, ldc, sigma, t);
    if (st) return st;
    if (!V || !U) return fail(ctx, KNM_INVALID_ARG, "null vector");
    float *W = W_or_null;
    if (!W) {
        st = ensure(ctx, &ctx->w_buf, &ctx->w_bytes, sizeof(float) * (size_t)n * t);
        if (st) return st;
        W = ctx->w_buf;
    }
    begin_timing(ctx);
    st = do_knm_v(ctx, X, n, d, ldx, C, M, ldc, sigma, V, t, W);
    if (st) return st;
    mark(ctx, 1);
    st = do_knm_t_w(ctx, X, n, d, ldx, C, M, ldc, sigma, W, dw, t, U);
    if (st) return st;
    mark(ctx, 3);
    mark(ctx, 4);
    return KNM_OK;
}

int knm_prod(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M, int64_t ldc,
             float sigma, const float *V, int t, float *W_or_null, float *U)
{
    return prod_impl(ctx, X, n, d, ldx, C, M, ldc, sigma, nullptr, V, t, W_or_null, U);
}

size_t knm_static_scratch_bytes(void) { return kStaticScratchBytes; }

int knm_prod_static(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M, int64_t ldc,
                    float sigma, const float *V, int t, float *W, float *U)
{
    if (ctx && !W) return fail(ctx, KNM_INVALID_ARG, "the allocation-free product needs the caller's W");
    if (!ctx) return KNM_INVALID_ARG;
    ctx->static_mode = true;
    const int st = prod_impl(ctx, X, n, d, ldx, C, M, ldc, sigma, nullptr, V, t, W, U);
    ctx->static_mode = false;
    return st;
}

int knm_prod_weighted(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
                      int64_t ldc, float sigma, const float *dw, const float *V, int t, float *U)
{
    if (ctx && !dw) return fail(ctx, KNM_INVALID_ARG, "null weights");
    return prod_impl(ctx, X, n, d, ldx, C, M, ldc, sigma, dw, V, t, nullptr, U);
}

int knm_t_y(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M, int64_t ldc,
            float sigma, const float *Y, int t, float *R)
{
    int st = check_common(ctx, X, n, d, ldx, C, M, ldc, sigma, t);
    if (st) return st;
    if (!Y || !R) return fail(ctx, KNM_INVALID_ARG, "null vector");
    begin_timing(ctx);
    mark(ctx, 1);
    st = do_knm_t_w(ctx, X, n, d, ldx, C, M, ldc, sigma, Y, nullptr, t, R);
    if (st) return st;
    mark(ctx, 3);
    mark(ctx, 4);
    return KNM_OK;
}

int knm_range_exceeded(knm_ctx *ctx, int64_t *count_host, int reset)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!count_host) return fail(ctx, KNM_INVALID_ARG, "null count");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    unsigned int c = 0;
    hipError_t e = hipMemcpyAsync(&c, ctx->range_count, sizeof(c), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess && reset) e = hipMemsetAsync(ctx->range_count, 0, sizeof(c), ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "knm_range_exceeded", e);
    *count_host = (int64_t)c;
    return KNM_OK;
}

int knm_set_cross_term(knm_ctx *ctx, int mode)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (mode != KNM_CROSS_F32 && mode != KNM_CROSS_F16X3) return fail(ctx, KNM_INVALID_ARG, "unknown cross-term mode");
    ctx->cross_term = mode;
    return KNM_OK;
}

int knm_get_cross_term(const knm_ctx *ctx) { return ctx ? ctx->cross_term : KNM_INVALID_ARG; }

int knm_set_kernel(knm_ctx *ctx, int kind)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (kind < KNM_KERNEL_GAUSSIAN || kind > KNM_KERNEL_MATERN52) return fail(ctx, KNM_INVALID_ARG, "unknown kernel");
    ctx->kernel_kind = kind;
    return KNM_OK;
}

int knm_set_sparse_head_limit(knm_ctx *ctx, int max_features)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (max_features < 0) return fail(ctx, KNM_INVALID_ARG, "negative head limit");
    ctx->sparse_head_max = max_features > 128 ? 128 : max_features;
    return KNM_OK;
}

int knm_set_pack_limit(knm_ctx *ctx, size_t bytes)
{
    if (!ctx) return KNM_INVALID_ARG;
    ctx->pack_limit = bytes;
    return KNM_OK;
}

int knm_set_timing(knm_ctx *ctx, int enabled)
{
    if (!ctx) return KNM_INVALID_ARG;
    ctx->timing = enabled != 0;
    for (int i = 0; i < 5; ++i) ctx->ev_used[i] = false;
    return KNM_OK;
}

int knm_get_timing(knm_ctx *ctx, float *ms)
{
    if (!ctx || !ms) return KNM_INVALID_ARG;
    for (int i = 0; i < 4; ++i) ms[i] = 0.0f;
    if (!ctx->ev_used[0] || !ctx->ev_used[4]) return fail(ctx, KNM_INVALID_ARG, "no timed call recorded");
    hipError_t e = hipEventSynchronize(ctx->ev[4]);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipEventSynchronize", e);
    // events: 0 start, 1 after row sweep, 2 after column sweep kernels, 3 after merge, 4 end
    auto span = [&](int a, int b, float *dst) {
        if (ctx->ev_used[a] && ctx->ev_used[b]) (void)hipEventElapsedTime(dst, ctx->ev[a], ctx->ev[b]);
    };
    span(0, 1, &ms[0]);
    span(1, 2, &ms[1]);
    span(2, 3, &ms[2]);
    span(0, 4, &ms[3]);
    return KNM_OK;
}

} // extern "C"
