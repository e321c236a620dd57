// C ABI of the STL library: argument validation, workspace carving and launch sequencing.
// Every step of the operator runs in the kernels of this library; there is no host fallback.
#include "../../include/stl.h"
#include "stl_kernels.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

namespace {

thread_local char g_err[512] = "";

stl_status_t fail(stl_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

stl_status_t hip_fail(hipError_t e, const char *what)
{
    return fail(STL_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

struct Dims {
    int M, K, N, r;
    size_t es;  // element size of the storage dtype
    // activation-side plane tensors are stored in groups of kPlaneGroup tile rows: their row count rounded up
    size_t Mp() const { return ((size_t)M + stl::kPlaneGroup - 1) / stl::kPlaneGroup * stl::kPlaneGroup; }
};

constexpr int PG = stl::kPlaneGroup;   // layout of Xhat, Yhat, dYhat, dXhat; What and dWhat are plane-major (0)

constexpr int64_t kMaxDim = STL_MAX_DIM;  // per-dimension cap: tile indices fit an int and every grid extent the device's limits

stl_status_t check_problem(const stl_problem_t *p, Dims *d)
{
    if (!p) return fail(STL_ERR_INVALID_ARG, "problem descriptor is NULL");
    if (p->dtype != STL_F32 && p->dtype != STL_BF16) return fail(STL_ERR_UNSUPPORTED, "unknown dtype %d", p->dtype);
    if (p->t != 4) return fail(STL_ERR_UNSUPPORTED, "tile size t=%d is not supported (t must be 4)", p->t);
    if (p->r < 1 || p->r > 64) return fail(STL_ERR_INVALID_ARG, "tensor rank r=%d outside [1,64]", p->r);
    if (p->m < 4 || p->k < 4 || p->n < 4) return fail(STL_ERR_INVALID_ARG, "m, k, n must be positive");
    if (p->m % 4 || p->k % 4 || p->n % 4)
        return fail(STL_ERR_INVALID_ARG, "m=%lld k=%lld n=%lld must be multiples of t=4", (long long)p->m,
                    (long long)p->k, (long long)p->n);
    if (p->m > kMaxDim || p->k > kMaxDim || p->n > kMaxDim)
        return fail(STL_ERR_INVALID_ARG, "dimension larger than %lld", (long long)kMaxDim);
    d->M = (int)(p->m / 4);
    d->K = (int)(p->k / 4);
    d->N = (int)(p->n / 4);
    d->r = p->r;
    d->es = p->dtype == STL_F32 ? 4 : 2;
    // plane tensors are indexed with size_t, but keep each below 2^40 elements as a sanity bound
    const double big = 1099511627776.0;
    if ((double)d->r * d->M * d->K > big || (double)d->r * d->M * d->N > big || (double)d->r * d->K * d->N > big)
        return fail(STL_ERR_INVALID_ARG, "plane tensors too large");
    return STL_OK;
}

// every data pointer must be 16-byte aligned (vector loads and stores of 16 bytes start at row and plane bases)
template <typename... P>
bool any_misaligned(P... ptrs)
{
    return ((((uintptr_t)ptrs) & 15) || ...);
}

// scratch: present and large enough when any is needed, 16-byte aligned when given
stl_status_t check_workspace(const char *fn, const void *ws, size_t ws_bytes, size_t need)
{
    if (need > 0 && (!ws || ws_bytes < need))
        return fail(STL_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, ws ? ws_bytes : (size_t)0);
    if (ws && ((uintptr_t)ws & 15)) return fail(STL_ERR_INVALID_ARG, "%s: workspace is not 16-byte aligned", fn);
    return STL_OK;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct FwdWs {
    size_t xhat, yhat, ctr, total;
};

int variant_of(int flags) { return flags & STL_FLAG_VARIANT_MASK; }

stl_status_t check_flags(int flags, int *variant)
{
    if (flags & ~(STL_FLAG_VARIANT_MASK | STL_FLAG_GELU)) return fail(STL_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
    int v = variant_of(flags);
    if (v > STL_FLAG_PIPELINED) return fail(STL_ERR_UNSUPPORTED, "unknown forward variant %d", v);
    *variant = v;
    return STL_OK;
}

FwdWs fwd_layout(const Dims &d, int variant)
{
    FwdWs w{};
    size_t off = 0;
    w.xhat = off;
    if (variant != STL_FLAG_FUSED) off += align256((size_t)d.r * d.Mp() * d.K * d.es);
    w.yhat = off;
    if (variant == STL_FLAG_AUTO || variant == STL_FLAG_UNFUSED || variant == STL_FLAG_PIPELINED)
        off += align256((size_t)d.r * d.Mp() * d.N * d.es);
    w.ctr = off;                                        // item counters of the single-launch pipelined forward
    if (variant == STL_FLAG_PIPELINED) off += align256(stl::forward_pipeline_counter_bytes(d.M));
    w.total = off;
    return w;
}

struct BwdWs {
    size_t xhat, dyhat, dxhat, yhat, part, part2, total;
};

BwdWs bwd_layout(const Dims &d)
{
    BwdWs w{};
    size_t off = 0;
    const size_t pk = align256((size_t)d.r * d.Mp() * d.K * d.es), pn = align256((size_t)d.r * d.Mp() * d.N * d.es);
    w.xhat = off;
    off += pk;
    w.dyhat = off;
    off += pn;
    w.dxhat = off;
    off += pk;
    w.yhat = off;
    off += pn;
    int nb = stl::outer_reduce_blocks((int64_t)d.M * d.N);
    const int nb_k = stl::outer_reduce_blocks((int64_t)d.M * d.K), nb_f = stl::decode_outer_blocks(d.M, d.K);
    const int nb_e = stl::encode_outer_blocks(d.M, d.N);
    nb = nb > nb_k ? nb : nb_k;
    nb = nb > nb_f ? nb : nb_f;
    nb = nb > nb_e ? nb : nb_e;
    // two areas of partial sums: the two fused gradient passes leave theirs for one common final sum
    w.part = off;
    off += align256((size_t)nb * d.r * 16 * sizeof(float));
    w.part2 = off;
    off += align256((size_t)nb * d.r * 16 * sizeof(float));
    w.total = off;
    return w;
}

struct EwbWs {
    size_t planes, part, total;
};

// backward of the weight encoding: a bf16 copy of dWhat (bf16 storage only) and the partial sums of dE_W
EwbWs ewb_layout(const stl_problem_t *p, const Dims &d)
{
    EwbWs w{};
    size_t off = 0;
    w.planes = off;
    if (p->dtype == STL_BF16) off += align256((size_t)d.r * d.K * d.N * 2);
    int nb = stl::outer_reduce_blocks((int64_t)d.K * d.N);
    const int nb_f = stl::decode_outer_blocks(d.K, d.N);
    nb = nb > nb_f ? nb : nb_f;
    w.part = off;
    off += align256((size_t)nb * d.r * 16 * sizeof(float));
    w.total = off;
    return w;
}

struct MlpWs {
    size_t xhat1, yhat1, xhat2, yhat2, hidden, total;
    bool one_pass;
};

// the two layers must chain: same rows, up.n == down.k, same tile size and storage type
stl_status_t check_pair(const stl_problem_t *up, const stl_problem_t *down, Dims *d1, Dims *d2)
{
    stl_status_t st = check_problem(up, d1);
    if (st != STL_OK) return st;
    st = check_problem(down, d2);
    if (st != STL_OK) return st;
    if (up->m != down->m || up->n != down->k)
        return fail(STL_ERR_INVALID_ARG, "layers do not chain: up is %lld x %lld -> %lld, down is %lld x %lld -> %lld",
                    (long long)up->m, (long long)up->k, (long long)up->n, (long long)down->m, (long long)down->k,
                    (long long)down->n);
    if (up->dtype != down->dtype) return fail(STL_ERR_INVALID_ARG, "layers differ in dtype");
    return STL_OK;
}

stl_status_t check_pair_flags(int flags, int *variant)
{
    if (flags & ~(STL_FLAG_VARIANT_MASK | STL_FLAG_GELU)) return fail(STL_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
    const int v = variant_of(flags);
    if (v != STL_FLAG_AUTO && v != STL_FLAG_UNFUSED)
        return fail(STL_ERR_UNSUPPORTED, "layer pair: variant %d is not available (AUTO or UNFUSED)", v);
    *variant = v;
    return STL_OK;
}

MlpWs mlp_layout(const stl_problem_t *up, const Dims &d1, const Dims &d2, int variant)
{
    MlpWs w{};
    size_t off = 0;
    w.xhat1 = off;
    off += align256((size_t)d1.r * d1.Mp() * d1.K * d1.es);
    w.yhat1 = off;
    off += align256((size_t)d1.r * d1.Mp() * d1.N * d1.es);
    w.xhat2 = off;
    off += align256((size_t)d2.r * d2.Mp() * d2.K * d2.es);
    w.yhat2 = off;
    off += align256((size_t)d2.r * d2.Mp() * d2.N * d2.es);
    w.one_pass = variant == STL_FLAG_AUTO && stl::recode_eligible(up->dtype, d1.N);
    w.hidden = off;
    if (!w.one_pass) off += align256((size_t)up->m * up->n * d1.es);
    w.total = off;
    return w;
}

// both operands encoded at run time, nbatch problems stacked along the rows
struct AaWs {
    size_t ahat, bhat, yhat, dyhat, dahat, dbhat, part, ebt, gbt, total;
};

size_t stacked_planes_bytes(const Dims &d, int64_t rows, int cols)
{
    const size_t rp = ((size_t)rows + PG - 1) / PG * PG;
    return align256((size_t)d.r * rp * cols * d.es);
}

AaWs aa_layout(const Dims &d, int64_t nb, bool backward)
{
    AaWs w{};
    size_t off = 0;
    // Bhat holds nb*K x N tile rows, or nb*N x K when the second operand is stored transposed: room for either
    const size_t pb1 = stacked_planes_bytes(d, nb * d.K, d.N), pb2 = stacked_planes_bytes(d, nb * d.N, d.K);
    const size_t pa = stacked_planes_bytes(d, nb * d.M, d.K), pb = pb1 > pb2 ? pb1 : pb2,
                 py = stacked_planes_bytes(d, nb * d.M, d.N);
    w.ahat = off;
    off += pa;
    w.bhat = off;
    off += pb;
    w.yhat = off;
    off += py;
    if (backward) {
        w.dyhat = off;
        off += py;
        w.dahat = off;
        off += pa;
        w.dbhat = off;
        off += pb;
        int nblk = 1;
        const int64_t Rs[4] = {nb * d.M, nb * d.M, nb * d.K, nb * d.N};
        const int Cs[4] = {d.N, d.K, d.N, d.K};
        for (int i = 0; i < 4; ++i) {
            const int a = stl::outer_reduce_blocks(Rs[i] * Cs[i]), b = stl::decode_outer_blocks((int)Rs[i], Cs[i]),
                      c = stl::encode_outer_blocks((int)Rs[i], Cs[i]);
            nblk = a > nblk ? a : nblk;
            nblk = b > nblk ? b : nblk;
            nblk = c > nblk ? c : nblk;
        }
        w.part = off;
        off += align256((size_t)nblk * d.r * 16 * sizeof(float));
    }
    w.ebt = off;                                   // E_B with the tile transposition folded in (storage type)
    off += align256((size_t)d.r * 16 * d.es);
    w.gbt = off;                                   // its gradient before the transposition is undone (fp32)
    off += align256((size_t)d.r * 16 * sizeof(float));
    w.total = off;
    return w;
}

stl_status_t check_batch(const stl_problem_t *p, const Dims &d, int64_t nb)
{
    if (nb < 1) return fail(STL_ERR_INVALID_ARG, "nbatch=%lld must be positive", (long long)nb);
    if (nb * p->m > kMaxDim || nb * p->k > kMaxDim || nb * p->n > kMaxDim)
        return fail(STL_ERR_INVALID_ARG, "stacked rows nbatch*m, nbatch*k or nbatch*n larger than %lld", (long long)kMaxDim);
    const double big = 1099511627776.0;
    if ((double)nb * d.r * d.M * d.K > big || (double)nb * d.r * d.M * d.N > big || (double)nb * d.r * d.K * d.N > big)
        return fail(STL_ERR_INVALID_ARG, "stacked plane tensors too large");
    return STL_OK;
}

// images of `rows` real rows each, padded with null rows to Mt tile rows (row counts the tile size does not divide)
struct Ragged {
    Dims d;            // of the padded problem: d.M = nimg * Mt tile rows
    int Mt, rows, nimg, nrho;
    stl::RowMap map(int sel) const
    {
        stl::RowMap rm;
        if (nrho) { rm.Mt = Mt; rm.rows = rows; rm.sel = sel; }
        return rm;
    }
};

stl_status_t check_ragged(const stl_problem_t *p, int64_t rows, Ragged *g)
{
    if (!p) return fail(STL_ERR_INVALID_ARG, "problem descriptor is NULL");
    if (rows < 4) return fail(STL_ERR_INVALID_ARG, "rows per image = %lld must be at least t = 4", (long long)rows);
    if (p->m < rows || p->m % rows)
        return fail(STL_ERR_INVALID_ARG, "m=%lld is not a multiple of the rows per image %lld", (long long)p->m, (long long)rows);
    if (rows > kMaxDim || p->m > kMaxDim) return fail(STL_ERR_INVALID_ARG, "dimension larger than %lld", (long long)kMaxDim);
    const int64_t nimg = p->m / rows, Mt = (rows + 3) / 4;
    stl_problem_t padded = *p;
    padded.m = nimg * Mt * 4;
    stl_status_t st = check_problem(&padded, &g->d);
    if (st != STL_OK) return st;
    g->Mt = (int)Mt;
    g->rows = (int)rows;
    g->nimg = (int)nimg;
    g->nrho = (int)(rows % 4);
    return STL_OK;
}

struct RagWs {
    size_t xhat, yhat, dyhat, dxhat, part, dprime, gtail, total;
};

RagWs ragged_layout(const Ragged &g, bool backward)
{
    const Dims &d = g.d;
    RagWs w{};
    size_t off = 0;
    const size_t pk = align256((size_t)d.r * d.Mp() * d.K * d.es), pn = align256((size_t)d.r * d.Mp() * d.N * d.es);
    w.xhat = off;
    off += pk;
    w.yhat = off;
    off += pn;
    if (backward) {
        w.dyhat = off;
        off += pn;
        w.dxhat = off;
        off += pk;
        w.part = off;
        off += align256(bwd_layout(d).part2 - bwd_layout(d).part);      // a partial-sum area as in stl_backward
    }
    w.dprime = off;
    off += align256((size_t)d.r * 16 * sizeof(float));
    w.gtail = off;
    off += align256((size_t)d.r * 16 * sizeof(float));
    w.total = off;
    return w;
}

#define STL_HIP(call, what)                                \
    do {                                                   \
        hipError_t e__ = (call);                           \
        if (e__ != hipSuccess) return hip_fail(e__, what); \
    } while (0)


// Algorithm 1 as three launches over caller-visible plane buffers.  Output rows are independent, so when neither plane
// tensor is handed back (`slabs`) the rows can be taken in slabs that reuse the same plane scratch: the planes of a slab
// are then still in the 256 MB last-level cache when the next kernel reads them, instead of having been pushed out by
// the rest of a large problem.  A slab holds about 128 MB of planes, in multiples of the plane products' 256-row
// blocks, and at least 1024 tile rows.
stl_status_t forward_three_launch(const stl_problem_t *prob, const Dims &d, const void *X, const void *What, const void *E_X,
                                  const void *D, void *C, void *xhat, void *yhat, bool slabs, bool gelu, hipStream_t s)
{
    int slab_rows = d.M;
    const size_t row_bytes = (size_t)d.r * ((size_t)d.K + d.N) * d.es;      // Xhat + Yhat bytes per tile row
    if (slabs && row_bytes * d.M > ((size_t)192 << 20)) {
        const size_t fit = ((size_t)128 << 20) / row_bytes;                 // tile rows whose planes take 128 MB
        // shorter slabs than 1024 tile rows cost the plane products more than the cache gives back (measured)
        if (fit >= 1024 && (int)(fit / 256) * 256 < d.M) slab_rows = (int)(fit / 256) * 256;
    }
    for (int r0 = 0; r0 < d.M; r0 += slab_rows) {
        const int rows = d.M - r0 < slab_rows ? d.M - r0 : slab_rows;
        const char *Xs = (const char *)X + (size_t)r0 * 4 * prob->k * d.es;
        char *Cs = (char *)C + (size_t)r0 * 4 * prob->n * d.es;
        STL_HIP(stl::launch_encode(prob->dtype, Xs, E_X, xhat, rows, d.K, d.r, PG, s), "forward/encode");
        stl::GemmDesc g{rows, d.N, d.K, d.r, false, true, false, false, PG, 0, PG};
        STL_HIP(stl::launch_plane_gemm(prob->dtype, g, xhat, What, yhat, s), "forward/plane products");
        STL_HIP(stl::launch_decode(prob->dtype, yhat, D, Cs, rows, d.N, d.r, gelu, PG, s), "forward/decode");
    }
    return STL_OK;
}

// Built-in scratch of stl_forward_static: a device array that lives in the library's code object, so the entry point
// needs neither a caller workspace nor any allocation.  Each GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the array's name is only a handle for the runtime's symbol lookup,
// never a device address: the address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = STL_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mu;
char *g_scratch_ptr[kMaxDevices] = {};

stl_status_t static_scratch_base(char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "stl_forward_static/hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(STL_ERR_UNSUPPORTED, "stl_forward_static: device ordinal %d not below %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));       // address of THIS device's copy (the current device)
        if (e != hipSuccess) return hip_fail(e, "stl_forward_static/hipGetSymbolAddress");
        if (!p || ((uintptr_t)p & 255)) return fail(STL_ERR_HIP, "stl_forward_static: built-in scratch address %p is unusable", p);
        g_scratch_ptr[dev] = (char *)p;
    }
    *out = g_scratch_ptr[dev];
    return STL_OK;
}

}  // namespace

extern "C" {

const char *stl_status_string(stl_status_t s)
{
    switch (s) {
        case STL_OK: return "ok";
        case STL_ERR_INVALID_ARG: return "invalid argument";
        case STL_ERR_UNSUPPORTED: return "unsupported";
        case STL_ERR_WORKSPACE: return "workspace missing or too small";
        case STL_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

const char *stl_last_error(void) { return g_err; }

const char *stl_version(void) { return "0.3.0 gfx950"; }

size_t stl_plane_elems(int64_t R, int64_t Cc, int r)
{
    if (R < 0 || Cc < 0 || r < 0) return 0;
    return (size_t)r * (size_t)((R + PG - 1) / PG * PG) * (size_t)Cc;
}

size_t stl_workspace_bytes(const stl_problem_t *prob, int op, int flags)
{
    Dims d;
    if (check_problem(prob, &d) != STL_OK) return 0;
    switch (op) {
        case STL_OP_ENCODE_WEIGHT: return 0;
        case STL_OP_FORWARD: {
            int v;
            if (check_flags(flags, &v) != STL_OK) return 0;
            return fwd_layout(d, v).total;
        }
        case STL_OP_BACKWARD: return bwd_layout(d).total;
        case STL_OP_ENCODE_WEIGHT_BACKWARD: return ewb_layout(prob, d).total;
    }
    fail(STL_ERR_INVALID_ARG, "unknown op %d", op);
    return 0;
}

stl_status_t stl_encode_weight(const stl_problem_t *prob, const void *W, const void *E_W, void *What, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!W || !E_W || !What) return fail(STL_ERR_INVALID_ARG, "stl_encode_weight: NULL pointer");
    if (any_misaligned(W, E_W, What)) return fail(STL_ERR_INVALID_ARG, "stl_encode_weight: pointer not 16-byte aligned");
    STL_HIP(stl::launch_encode(prob->dtype, W, E_W, What, d.K, d.N, d.r, 0, (hipStream_t)stream), "encode_weight");
    return STL_OK;
}

stl_status_t stl_encode_weight_backward(const stl_problem_t *prob, const void *W, const void *E_W, const float *dWhat,
                                        void *dW, float *dE_W, int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!W || !E_W || !dWhat) return fail(STL_ERR_INVALID_ARG, "stl_encode_weight_backward: NULL input pointer");
    if (any_misaligned(W, E_W, dWhat, dW, dE_W))
        return fail(STL_ERR_INVALID_ARG, "stl_encode_weight_backward: pointer not 16-byte aligned");
    if (accumulate != 0 && accumulate != 1)
        return fail(STL_ERR_INVALID_ARG, "stl_encode_weight_backward: accumulate must be 0 or 1");
    const EwbWs w = ewb_layout(prob, d);
    st = check_workspace("stl_encode_weight_backward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype;
    char *base = (char *)ws;
    float *part = (float *)(base + w.part);
    const void *planes = dWhat;
    if (dt == STL_BF16 && (dW || dE_W)) {
        STL_HIP(stl::launch_cast_bf16(dWhat, base + w.planes, (size_t)d.r * d.K * d.N, s), "encode_weight_backward/round dWhat");
        planes = base + w.planes;
    }
    if (dW && dE_W && stl::decode_outer_eligible(dt, d.N)) {
        STL_HIP(stl::launch_decode_outer(planes, E_W, dW, W, dE_W, part, d.K, d.N, d.r, accumulate, 0, s),
                "encode_weight_backward/dW + dE_W");
        return STL_OK;
    }
    if (dW) STL_HIP(stl::launch_decode(dt, planes, E_W, dW, d.K, d.N, d.r, false, 0, s), "encode_weight_backward/dW");
    if (dE_W)
        STL_HIP(stl::launch_outer_reduce(dt, planes, W, dE_W, part, d.K, d.N, d.r, accumulate, 0, s), "encode_weight_backward/dE_W");
    return STL_OK;
}

stl_status_t stl_encode_activation(const stl_problem_t *prob, const void *X, const void *E_X, void *Xhat, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!X || !E_X || !Xhat) return fail(STL_ERR_INVALID_ARG, "stl_encode_activation: NULL pointer");
    if (any_misaligned(X, E_X, Xhat)) return fail(STL_ERR_INVALID_ARG, "stl_encode_activation: pointer not 16-byte aligned");
    STL_HIP(stl::launch_encode(prob->dtype, X, E_X, Xhat, d.M, d.K, d.r, PG, (hipStream_t)stream), "encode_activation");
    return STL_OK;
}

stl_status_t stl_plane_matmul(const stl_problem_t *prob, const void *Xhat, const void *What, void *Yhat, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!Xhat || !What || !Yhat) return fail(STL_ERR_INVALID_ARG, "stl_plane_matmul: NULL pointer");
    if (any_misaligned(Xhat, What, Yhat)) return fail(STL_ERR_INVALID_ARG, "stl_plane_matmul: pointer not 16-byte aligned");
    stl::GemmDesc g{d.M, d.N, d.K, d.r, false, true, false, false, PG, 0, PG};
    STL_HIP(stl::launch_plane_gemm(prob->dtype, g, Xhat, What, Yhat, (hipStream_t)stream), "plane_matmul");
    return STL_OK;
}

stl_status_t stl_decode(const stl_problem_t *prob, const void *Yhat, const void *D, void *C, int flags, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!Yhat || !D || !C) return fail(STL_ERR_INVALID_ARG, "stl_decode: NULL pointer");
    if (any_misaligned(Yhat, D, C)) return fail(STL_ERR_INVALID_ARG, "stl_decode: pointer not 16-byte aligned");
    if (flags & ~STL_FLAG_GELU) return fail(STL_ERR_UNSUPPORTED, "stl_decode: unknown flag bits 0x%x", flags);
    STL_HIP(stl::launch_decode(prob->dtype, Yhat, D, C, d.M, d.N, d.r, (flags & STL_FLAG_GELU) != 0, PG, (hipStream_t)stream),
            "decode");
    return STL_OK;
}

stl_status_t stl_forward(const stl_problem_t *prob, const void *X, const void *What, const void *E_X, const void *D,
                         void *C, void *Xhat_save, void *Yhat_save, void *ws, size_t ws_bytes, int flags, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    int variant;
    st = check_flags(flags, &variant);
    if (st != STL_OK) return st;
    if (!X || !What || !E_X || !D || !C) return fail(STL_ERR_INVALID_ARG, "stl_forward: NULL pointer");
    if (any_misaligned(X, What, E_X, D, C, Xhat_save, Yhat_save))
        return fail(STL_ERR_INVALID_ARG, "stl_forward: pointer not 16-byte aligned");
    // Automatic choice: the single-launch variant where the whole operator is launch-bound (measured: it wins up to
    // about four million tile products per plane set, e.g. m = 128, k = n = 512, r = 8: one launch of ~10 us against
    // three of ~5 us), the three-launch path everywhere else.
    const FwdWs w_declared = fwd_layout(d, variant);     // the workspace is checked against what the caller asked for
    if (variant == STL_FLAG_AUTO && !Xhat_save && stl::block_forward_eligible(prob->dtype, d.M, d.K, d.N, d.r) &&
        (double)d.M * d.K * d.N * d.r <= 4.2e6)
        variant = STL_FLAG_FUSED;
    if (variant == STL_FLAG_PIPELINED && !stl::forward_pipeline_eligible(prob->dtype, d.M, d.K, d.N, d.r))
        return fail(STL_ERR_UNSUPPORTED,
                    "stl_forward: the pipelined variant needs bf16 storage, r <= 32, k and n multiples of 256, n >= 1024 and m >= 2048");
    if (variant == STL_FLAG_EPILOGUE || variant == STL_FLAG_FUSED) {
        if (!stl::block_forward_eligible(prob->dtype, d.M, d.K, d.N, d.r))
            return fail(STL_ERR_UNSUPPORTED,
                        "stl_forward: the block-resident variants need bf16 storage, r <= 32, k %% 64 == 0 and n %% 32 == 0");
        if (variant == STL_FLAG_FUSED && Xhat_save)
            return fail(STL_ERR_UNSUPPORTED, "stl_forward: the fused variant never materialises Xhat (Xhat_save must be NULL)");
    }
    const FwdWs w = fwd_layout(d, variant);
    st = check_workspace("stl_forward", ws, ws_bytes, w_declared.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const bool gelu = (flags & STL_FLAG_GELU) != 0;
    char *base = (char *)ws;

    if (variant == STL_FLAG_FUSED) {
        STL_HIP(stl::launch_block_forward(true, X, What, E_X, D, C, Yhat_save, d.M, d.K, d.N, d.r, gelu, PG, s), "forward/fused");
        return STL_OK;
    }
    void *xhat = Xhat_save ? Xhat_save : (void *)(base + w.xhat);
    if (variant == STL_FLAG_EPILOGUE) {
        STL_HIP(stl::launch_encode(prob->dtype, X, E_X, xhat, d.M, d.K, d.r, PG, s), "forward/encode");
        STL_HIP(stl::launch_block_forward(false, xhat, What, E_X, D, C, Yhat_save, d.M, d.K, d.N, d.r, gelu, PG, s),
                "forward/plane products + decode");
        return STL_OK;
    }
    void *yhat = Yhat_save ? Yhat_save : (void *)(base + w.yhat);
    if (variant == STL_FLAG_PIPELINED) {
        STL_HIP(stl::launch_forward_pipeline(X, E_X, What, D, xhat, yhat, C, base + w.ctr, d.M, d.K, d.N, d.r, gelu, s),
                "forward/pipelined");
        return STL_OK;
    }
    return forward_three_launch(prob, d, X, What, E_X, D, C, xhat, yhat, !Xhat_save && !Yhat_save, gelu, s);
}

stl_status_t stl_forward_static(const stl_problem_t *prob, const void *X, const void *What, const void *E_X, const void *D,
                                void *C, int flags, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (flags & ~STL_FLAG_GELU) return fail(STL_ERR_UNSUPPORTED, "stl_forward_static: unknown flag bits 0x%x", flags);
    if (!X || !What || !E_X || !D || !C) return fail(STL_ERR_INVALID_ARG, "stl_forward_static: NULL pointer");
    if (any_misaligned(X, What, E_X, D, C)) return fail(STL_ERR_INVALID_ARG, "stl_forward_static: pointer not 16-byte aligned");
    const FwdWs w = fwd_layout(d, STL_FLAG_UNFUSED);
    if (w.total > kStaticScratchBytes)
        return fail(STL_ERR_WORKSPACE,
                    "stl_forward_static: the encoded planes of this problem take %zu bytes, the built-in scratch holds %zu "
                    "(STL_STATIC_SCRATCH_BYTES); use stl_forward with a caller workspace",
                    w.total, kStaticScratchBytes);
    char *base = nullptr;
    st = static_scratch_base(&base);
    if (st != STL_OK) return st;
    // every element of the two plane tensors that a later kernel reads is written first by an earlier kernel of this
    // same call (encode writes Xhat, the plane products write Yhat), so nothing of the previous call has to be cleared
    return forward_three_launch(prob, d, X, What, E_X, D, C, base + w.xhat, base + w.yhat, false,
                                (flags & STL_FLAG_GELU) != 0, (hipStream_t)stream);
}

stl_status_t stl_backward(const stl_problem_t *prob, const void *X, const void *What, const void *E_X, const void *D,
                          const void *dC, const void *Xhat_saved, const void *Yhat_saved, void *dX, float *dWhat, float *dE_X, float *dD,
                          int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    if (!X || !What || !E_X || !D || !dC) return fail(STL_ERR_INVALID_ARG, "stl_backward: NULL input pointer");
    if (any_misaligned(X, What, E_X, D, dC, Xhat_saved, Yhat_saved, dX, dWhat, dE_X, dD))
        return fail(STL_ERR_INVALID_ARG, "stl_backward: pointer not 16-byte aligned");
    if (accumulate != 0 && accumulate != 1) return fail(STL_ERR_INVALID_ARG, "stl_backward: accumulate must be 0 or 1");
    const BwdWs w = bwd_layout(d);
    st = check_workspace("stl_backward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype;
    char *base = (char *)ws;
    const void *xhat = Xhat_saved ? Xhat_saved : (const void *)(base + w.xhat);
    void *dyhat = base + w.dyhat, *dxhat = base + w.dxhat;
    float *part = (float *)(base + w.part);

    const bool need_xhat = dWhat || (dD && !Yhat_saved);
    if (need_xhat && !Xhat_saved)
        STL_HIP(stl::launch_encode(dt, X, E_X, base + w.xhat, d.M, d.K, d.r, PG, s), "backward/encode X");
    const void *yhat = Yhat_saved;
    if (dD && !yhat) {
        stl::GemmDesc g{d.M, d.N, d.K, d.r, false, true, false, false, PG, 0, PG};
        STL_HIP(stl::launch_plane_gemm(dt, g, xhat, What, base + w.yhat, s), "backward/recompute Yhat");
        yhat = base + w.yhat;
    }
    // when both fused gradient passes run, their block partials are added up by one launch at the end
    const bool pair = dD && stl::encode_outer_eligible(dt, d.N) && dX && dE_X && stl::decode_outer_eligible(dt, d.K);
    float *part2 = (float *)(base + w.part2);
    if (dD && stl::encode_outer_eligible(dt, d.N)) {
        // one pass over dC: dYhat = encode with D, dD = sum over tiles of Yhat (x) dc
        STL_HIP(stl::launch_encode_outer(dC, D, dyhat, yhat, dD, part, d.M, d.N, d.r, accumulate, PG, s, stl::RowMap(), !pair),
                "backward/dYhat + dD");
    } else {
        STL_HIP(stl::launch_encode(dt, dC, D, dyhat, d.M, d.N, d.r, PG, s), "backward/encode dC");
        if (dD) STL_HIP(stl::launch_outer_reduce(dt, yhat, dC, dD, part, d.M, d.N, d.r, accumulate, PG, s), "backward/dD");
    }
    // The weight gradient goes first: the pass that follows the second product (decode of dXhat) is bound by HBM and
    // finds the freshly written dXhat in the last-level cache, which a product in between would have flushed; the
    // products themselves do not care which of them reads dYhat warm.
    if (dWhat) {
        // dWhat[p] = Xhat[p]^T * dYhat[p] : contraction over I, both operands stored [I][.]
        stl::GemmDesc g{d.K, d.N, d.M, d.r, true, true, true, accumulate != 0, PG, PG, 0};
        STL_HIP(stl::launch_plane_gemm(dt, g, xhat, dyhat, dWhat, s), "backward/dWhat");
    }
    if (dX || dE_X) {
        // dXhat[p] = dYhat[p] * What[p]^T : contraction over J, What[p] is stored [L][J]
        stl::GemmDesc g{d.M, d.K, d.N, d.r, false, false, false, false, PG, 0, PG};
        STL_HIP(stl::launch_plane_gemm(dt, g, dyhat, What, dxhat, s), "backward/dXhat");
    }
    if (dX && dE_X && stl::decode_outer_eligible(dt, d.K)) {
        // one pass over dXhat: dX = decode with E_X, dE_X = sum over tiles of dXhat (x) x
        STL_HIP(stl::launch_decode_outer(dxhat, E_X, dX, X, dE_X, pair ? part2 : part, d.M, d.K, d.r, accumulate, PG, s,
                                         stl::RowMap(), !pair),
                "backward/dX + dE_X");
        if (pair)
            STL_HIP(stl::launch_outer_final_pair(part, dD, stl::encode_outer_blocks(d.M, d.N), part2, dE_X,
                                                 stl::decode_outer_blocks(d.M, d.K), d.r * 16, accumulate, s),
                    "backward/dD and dE_X sums");
    } else {
        if (dX) STL_HIP(stl::launch_decode(dt, dxhat, E_X, dX, d.M, d.K, d.r, false, PG, s), "backward/decode dX");
        if (dE_X)
            STL_HIP(stl::launch_outer_reduce(dt, dxhat, X, dE_X, part, d.M, d.K, d.r, accumulate, PG, s), "backward/dE_X");
    }
    return STL_OK;
}

size_t stl_mlp_workspace_bytes(const stl_problem_t *up, const stl_problem_t *down, int flags)
{
    Dims d1, d2;
    int v;
    if (check_pair(up, down, &d1, &d2) != STL_OK || check_pair_flags(flags, &v) != STL_OK) return 0;
    return mlp_layout(up, d1, d2, v).total;
}

stl_status_t stl_recode(const stl_problem_t *up, const stl_problem_t *down, const void *Yhat1, const void *D1,
                        const void *E_X2, void *Xhat2, void *H, int flags, void *stream)
{
    Dims d1, d2;
    stl_status_t st = check_pair(up, down, &d1, &d2);
    if (st != STL_OK) return st;
    int variant;
    st = check_pair_flags(flags, &variant);
    if (st != STL_OK) return st;
    if (!Yhat1 || !D1 || !E_X2 || !Xhat2) return fail(STL_ERR_INVALID_ARG, "stl_recode: NULL pointer");
    if (any_misaligned(Yhat1, D1, E_X2, Xhat2, H)) return fail(STL_ERR_INVALID_ARG, "stl_recode: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const bool gelu = (flags & STL_FLAG_GELU) != 0;
    if (variant == STL_FLAG_AUTO && stl::recode_eligible(up->dtype, d1.N)) {
        STL_HIP(stl::launch_recode(Yhat1, D1, E_X2, Xhat2, d1.M, d1.N, d1.r, d2.r, gelu, PG, s), "recode");
        return STL_OK;
    }
    if (!H) return fail(STL_ERR_INVALID_ARG, "stl_recode: the two-launch form needs the hidden-activation scratch H");
    STL_HIP(stl::launch_decode(up->dtype, Yhat1, D1, H, d1.M, d1.N, d1.r, gelu, PG, s), "recode/decode");
    STL_HIP(stl::launch_encode(up->dtype, H, E_X2, Xhat2, d2.M, d2.K, d2.r, PG, s), "recode/encode");
    return STL_OK;
}

stl_status_t stl_mlp_forward(const stl_problem_t *up, const stl_problem_t *down, const void *X, const void *What1,
                             const void *E_X1, const void *D1, const void *What2, const void *E_X2, const void *D2,
                             void *C, void *ws, size_t ws_bytes, int flags, void *stream)
{
    Dims d1, d2;
    stl_status_t st = check_pair(up, down, &d1, &d2);
    if (st != STL_OK) return st;
    int variant;
    st = check_pair_flags(flags, &variant);
    if (st != STL_OK) return st;
    if (!X || !What1 || !E_X1 || !D1 || !What2 || !E_X2 || !D2 || !C)
        return fail(STL_ERR_INVALID_ARG, "stl_mlp_forward: NULL pointer");
    if (any_misaligned(X, What1, E_X1, D1, What2, E_X2, D2, C))
        return fail(STL_ERR_INVALID_ARG, "stl_mlp_forward: pointer not 16-byte aligned");
    const MlpWs w = mlp_layout(up, d1, d2, variant);
    st = check_workspace("stl_mlp_forward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = up->dtype;
    const bool gelu = (flags & STL_FLAG_GELU) != 0;
    char *base = (char *)ws;
    void *xhat1 = base + w.xhat1, *yhat1 = base + w.yhat1, *xhat2 = base + w.xhat2, *yhat2 = base + w.yhat2;

    STL_HIP(stl::launch_encode(dt, X, E_X1, xhat1, d1.M, d1.K, d1.r, PG, s), "pair/encode");
    stl::GemmDesc g1{d1.M, d1.N, d1.K, d1.r, false, true, false, false, PG, 0, PG};
    STL_HIP(stl::launch_plane_gemm(dt, g1, xhat1, What1, yhat1, s), "pair/plane products 1");
    if (w.one_pass) {
        STL_HIP(stl::launch_recode(yhat1, D1, E_X2, xhat2, d1.M, d1.N, d1.r, d2.r, gelu, PG, s), "pair/decode-activation-encode");
    } else {
        void *hid = base + w.hidden;
        STL_HIP(stl::launch_decode(dt, yhat1, D1, hid, d1.M, d1.N, d1.r, gelu, PG, s), "pair/decode 1");
        STL_HIP(stl::launch_encode(dt, hid, E_X2, xhat2, d2.M, d2.K, d2.r, PG, s), "pair/encode 2");
    }
    stl::GemmDesc g2{d2.M, d2.N, d2.K, d2.r, false, true, false, false, PG, 0, PG};
    STL_HIP(stl::launch_plane_gemm(dt, g2, xhat2, What2, yhat2, s), "pair/plane products 2");
    STL_HIP(stl::launch_decode(dt, yhat2, D2, C, d2.M, d2.N, d2.r, false, PG, s), "pair/decode 2");
    return STL_OK;
}

size_t stl_aa_workspace_bytes(const stl_problem_t *prob, int64_t nbatch, int op)
{
    Dims d;
    if (check_problem(prob, &d) != STL_OK || check_batch(prob, d, nbatch) != STL_OK) return 0;
    if (op == STL_OP_FORWARD) return aa_layout(d, nbatch, false).total;
    if (op == STL_OP_BACKWARD) return aa_layout(d, nbatch, true).total;
    fail(STL_ERR_INVALID_ARG, "stl_aa_workspace_bytes: op must be STL_OP_FORWARD or STL_OP_BACKWARD");
    return 0;
}

stl_status_t stl_aa_forward(const stl_problem_t *prob, int64_t nbatch, const void *A, const void *B, const void *E_A,
                            const void *E_B, const void *D, void *C, void *Ahat_save, void *Bhat_save, void *Yhat_save,
                            void *ws, size_t ws_bytes, int flags, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    st = check_batch(prob, d, nbatch);
    if (st != STL_OK) return st;
    if (flags & ~(STL_FLAG_GELU | STL_FLAG_B_TRANSPOSED))
        return fail(STL_ERR_UNSUPPORTED, "stl_aa_forward: unknown flag bits 0x%x", flags);
    if (!A || !B || !E_A || !E_B || !D || !C) return fail(STL_ERR_INVALID_ARG, "stl_aa_forward: NULL pointer");
    if (any_misaligned(A, B, E_A, E_B, D, C, Ahat_save, Bhat_save, Yhat_save))
        return fail(STL_ERR_INVALID_ARG, "stl_aa_forward: pointer not 16-byte aligned");
    const AaWs w = aa_layout(d, nbatch, false);
    st = check_workspace("stl_aa_forward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype, nb = (int)nbatch;
    char *base = (char *)ws;
    void *ahat = Ahat_save ? Ahat_save : (void *)(base + w.ahat);
    void *bhat = Bhat_save ? Bhat_save : (void *)(base + w.bhat);
    void *yhat = Yhat_save ? Yhat_save : (void *)(base + w.yhat);
    // the stack of first operands is one tall matrix for the tile maps; so is the stack of second operands
    STL_HIP(stl::launch_encode(dt, A, E_A, ahat, nb * d.M, d.K, d.r, PG, s), "aa_forward/encode A");
    const bool bt = (flags & STL_FLAG_B_TRANSPOSED) != 0;
    if (bt) {
        // tile (L, J) of B^T is the transpose of tile (J, L) of B: encode B as it lies with the transposition folded into
        // the basis; the planes come out as [p][J][L], the [j][l] operand form of the plane products
        STL_HIP(stl::launch_transpose_basis(dt, E_B, base + w.ebt, d.r, s), "aa_forward/transpose E_B");
        STL_HIP(stl::launch_encode(dt, B, base + w.ebt, bhat, nb * d.N, d.K, d.r, PG, s), "aa_forward/encode B");
    } else {
        STL_HIP(stl::launch_encode(dt, B, E_B, bhat, nb * d.K, d.N, d.r, PG, s), "aa_forward/encode B");
    }
    stl::GemmDesc g{d.M, d.N, d.K, d.r, false, !bt, false, false, PG, PG, PG, nb};
    STL_HIP(stl::launch_plane_gemm(dt, g, ahat, bhat, yhat, s), "aa_forward/plane products");
    STL_HIP(stl::launch_decode(dt, yhat, D, C, nb * d.M, d.N, d.r, (flags & STL_FLAG_GELU) != 0, PG, s), "aa_forward/decode");
    return STL_OK;
}

stl_status_t stl_aa_backward(const stl_problem_t *prob, int64_t nbatch, const void *A, const void *B, const void *E_A,
                             const void *E_B, const void *D, const void *dC, const void *Ahat_saved, const void *Bhat_saved,
                             const void *Yhat_saved, void *dA, void *dB, float *dE_A, float *dE_B, float *dD, int accumulate,
                             void *ws, size_t ws_bytes, int flags, void *stream)
{
    Dims d;
    stl_status_t st = check_problem(prob, &d);
    if (st != STL_OK) return st;
    st = check_batch(prob, d, nbatch);
    if (st != STL_OK) return st;
    if (!A || !B || !E_A || !E_B || !D || !dC) return fail(STL_ERR_INVALID_ARG, "stl_aa_backward: NULL input pointer");
    if (any_misaligned(A, B, E_A, E_B, D, dC, Ahat_saved, Bhat_saved, Yhat_saved, dA, dB, dE_A, dE_B, dD))
        return fail(STL_ERR_INVALID_ARG, "stl_aa_backward: pointer not 16-byte aligned");
    if (accumulate != 0 && accumulate != 1) return fail(STL_ERR_INVALID_ARG, "stl_aa_backward: accumulate must be 0 or 1");
    if (flags & ~STL_FLAG_B_TRANSPOSED) return fail(STL_ERR_UNSUPPORTED, "stl_aa_backward: unknown flag bits 0x%x", flags);
    const bool bt = (flags & STL_FLAG_B_TRANSPOSED) != 0;
    const AaWs w = aa_layout(d, nbatch, true);
    st = check_workspace("stl_aa_backward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype, nb = (int)nbatch;
    // stacked tile rows of A (and C) and of B, and B's tile columns, as B is stored
    const int RA = nb * d.M, RB = bt ? nb * d.N : nb * d.K, CB = bt ? d.K : d.N;
    char *base = (char *)ws;
    const void *e_b = E_B;                       // the basis that encodes B as it lies
    if (bt) {
        STL_HIP(stl::launch_transpose_basis(dt, E_B, base + w.ebt, d.r, s), "aa_backward/transpose E_B");
        e_b = base + w.ebt;
    }
    float *ge_b = bt ? (float *)(base + w.gbt) : dE_B;   // where the gradient of that basis is summed
    const int acc_b = bt ? 0 : accumulate;
    float *part = (float *)(base + w.part);
    void *dyhat = base + w.dyhat, *dahat = base + w.dahat, *dbhat = base + w.dbhat;

    const bool want_a = dA || dE_A, want_b = dB || dE_B;
    const void *ahat = Ahat_saved, *bhat = Bhat_saved, *yhat = Yhat_saved;
    if (!ahat && (want_b || (dD && !yhat))) {
        STL_HIP(stl::launch_encode(dt, A, E_A, base + w.ahat, RA, d.K, d.r, PG, s), "aa_backward/encode A");
        ahat = base + w.ahat;
    }
    if (!bhat && (want_a || (dD && !yhat))) {
        STL_HIP(stl::launch_encode(dt, B, e_b, base + w.bhat, RB, CB, d.r, PG, s), "aa_backward/encode B");
        bhat = base + w.bhat;
    }
    if (dD && !yhat) {
        stl::GemmDesc g{d.M, d.N, d.K, d.r, false, !bt, false, false, PG, PG, PG, nb};
        STL_HIP(stl::launch_plane_gemm(dt, g, ahat, bhat, base + w.yhat, s), "aa_backward/recompute Yhat");
        yhat = base + w.yhat;
    }
    if (dD && stl::encode_outer_eligible(dt, d.N)) {
        STL_HIP(stl::launch_encode_outer(dC, D, dyhat, yhat, dD, part, RA, d.N, d.r, accumulate, PG, s), "aa_backward/dYhat + dD");
    } else {
        STL_HIP(stl::launch_encode(dt, dC, D, dyhat, RA, d.N, d.r, PG, s), "aa_backward/encode dC");
        if (dD) STL_HIP(stl::launch_outer_reduce(dt, yhat, dC, dD, part, RA, d.N, d.r, accumulate, PG, s), "aa_backward/dD");
    }
    if (want_a) {
        // dAhat[b][p] = dYhat[b][p] * Bhat[b][p]^T, then back through the encoding of A
        // (with B stored transposed Bhat is [p][J][L]: the contraction index J is then its row index)
        stl::GemmDesc g{d.M, d.K, d.N, d.r, false, bt, false, false, PG, PG, PG, nb};
        STL_HIP(stl::launch_plane_gemm(dt, g, dyhat, bhat, dahat, s), "aa_backward/dAhat");
        if (dA && dE_A && stl::decode_outer_eligible(dt, d.K)) {
            STL_HIP(stl::launch_decode_outer(dahat, E_A, dA, A, dE_A, part, RA, d.K, d.r, accumulate, PG, s), "aa_backward/dA + dE_A");
        } else {
            if (dA) STL_HIP(stl::launch_decode(dt, dahat, E_A, dA, RA, d.K, d.r, false, PG, s), "aa_backward/decode dA");
            if (dE_A) STL_HIP(stl::launch_outer_reduce(dt, dahat, A, dE_A, part, RA, d.K, d.r, accumulate, PG, s), "aa_backward/dE_A");
        }
    }
    if (want_b) {
        // dBhat[b][p] = Ahat[b][p]^T * dYhat[b][p] in the storage type (one problem each, nothing accumulates over the
        // batch), then back through the encoding of B
        if (bt) {
            // dBhat^T[b][p] = dYhat[b][p]^T * Ahat[b][p], in the layout Bhat has
            stl::GemmDesc g{d.N, d.K, d.M, d.r, true, true, false, false, PG, PG, PG, nb};
            STL_HIP(stl::launch_plane_gemm(dt, g, dyhat, ahat, dbhat, s), "aa_backward/dBhat");
        } else {
            stl::GemmDesc g{d.K, d.N, d.M, d.r, true, true, false, false, PG, PG, PG, nb};
            STL_HIP(stl::launch_plane_gemm(dt, g, ahat, dyhat, dbhat, s), "aa_backward/dBhat");
        }
        if (dB && dE_B && stl::decode_outer_eligible(dt, CB)) {
            STL_HIP(stl::launch_decode_outer(dbhat, e_b, dB, B, ge_b, part, RB, CB, d.r, acc_b, PG, s), "aa_backward/dB + dE_B");
        } else {
            if (dB) STL_HIP(stl::launch_decode(dt, dbhat, e_b, dB, RB, CB, d.r, false, PG, s), "aa_backward/decode dB");
            if (dE_B) STL_HIP(stl::launch_outer_reduce(dt, dbhat, B, ge_b, part, RB, CB, d.r, acc_b, PG, s), "aa_backward/dE_B");
        }
        if (bt && dE_B) STL_HIP(stl::launch_transpose_basis_grad(ge_b, dE_B, d.r, accumulate, s), "aa_backward/dE_B of the stored basis");
    }
    return STL_OK;
}

size_t stl_ragged_workspace_bytes(const stl_problem_t *prob, int64_t rows, int op)
{
    Ragged g;
    if (check_ragged(prob, rows, &g) != STL_OK) return 0;
    if (op == STL_OP_FORWARD) return ragged_layout(g, false).total;
    if (op == STL_OP_BACKWARD) return ragged_layout(g, true).total;
    fail(STL_ERR_INVALID_ARG, "stl_ragged_workspace_bytes: op must be STL_OP_FORWARD or STL_OP_BACKWARD");
    return 0;
}

stl_status_t stl_ragged_forward(const stl_problem_t *prob, int64_t rows, const void *X, const void *What, const void *E_X,
                                const void *D, const float *fold, void *C, void *Xhat_save, void *Yhat_save, void *ws,
                                size_t ws_bytes, void *stream)
{
    Ragged g;
    stl_status_t st = check_ragged(prob, rows, &g);
    if (st != STL_OK) return st;
    const Dims &d = g.d;
    if (!X || !What || !E_X || !D || !C) return fail(STL_ERR_INVALID_ARG, "stl_ragged_forward: NULL pointer");
    if (g.nrho && !fold) return fail(STL_ERR_INVALID_ARG, "stl_ragged_forward: fold coefficients are NULL");
    if (any_misaligned(X, What, E_X, D, fold, C, Xhat_save, Yhat_save))
        return fail(STL_ERR_INVALID_ARG, "stl_ragged_forward: pointer not 16-byte aligned");
    const RagWs w = ragged_layout(g, false);
    st = check_workspace("stl_ragged_forward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype;
    char *base = (char *)ws;
    void *xhat = Xhat_save ? Xhat_save : (void *)(base + w.xhat);
    void *yhat = Yhat_save ? Yhat_save : (void *)(base + w.yhat);
    float *dprime = (float *)(base + w.dprime);
    // null rows are read as zeros by the encode; rows of complete tile rows are decoded with D, each image's last tile
    // row with the fold composed into the decoder
    STL_HIP(stl::launch_encode(dt, X, E_X, xhat, d.M, d.K, d.r, PG, s, g.map(0)), "ragged_forward/encode");
    stl::GemmDesc gd{d.M, d.N, d.K, d.r, false, true, false, false, PG, 0, PG};
    STL_HIP(stl::launch_plane_gemm(dt, gd, xhat, What, yhat, s), "ragged_forward/plane products");
    if (!g.nrho) {
        STL_HIP(stl::launch_decode(dt, yhat, D, C, d.M, d.N, d.r, false, PG, s), "ragged_forward/decode");
        return STL_OK;
    }
    STL_HIP(stl::launch_fold_decoder(dt, D, fold, dprime, d.r, g.nrho, s), "ragged_forward/compose fold");
    STL_HIP(stl::launch_decode(dt, yhat, D, C, d.M, d.N, d.r, false, PG, s, g.map(1)), "ragged_forward/decode");
    STL_HIP(stl::launch_decode(dt, yhat, dprime, C, d.M, d.N, d.r, false, PG, s, g.map(2), true), "ragged_forward/decode + fold");
    return STL_OK;
}

stl_status_t stl_ragged_backward(const stl_problem_t *prob, int64_t rows, const void *X, const void *What, const void *E_X,
                                 const void *D, const float *fold, const void *dC, const void *Xhat_saved,
                                 const void *Yhat_saved, void *dX, float *dWhat, float *dE_X, float *dD, float *dfold,
                                 int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    Ragged g;
    stl_status_t st = check_ragged(prob, rows, &g);
    if (st != STL_OK) return st;
    const Dims &d = g.d;
    if (!X || !What || !E_X || !D || !dC) return fail(STL_ERR_INVALID_ARG, "stl_ragged_backward: NULL input pointer");
    if (g.nrho && !fold) return fail(STL_ERR_INVALID_ARG, "stl_ragged_backward: fold coefficients are NULL");
    if (any_misaligned(X, What, E_X, D, fold, dC, Xhat_saved, Yhat_saved, dX, dWhat, dE_X, dD, dfold))
        return fail(STL_ERR_INVALID_ARG, "stl_ragged_backward: pointer not 16-byte aligned");
    if (accumulate != 0 && accumulate != 1) return fail(STL_ERR_INVALID_ARG, "stl_ragged_backward: accumulate must be 0 or 1");
    const RagWs w = ragged_layout(g, true);
    st = check_workspace("stl_ragged_backward", ws, ws_bytes, w.total);
    if (st != STL_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int dt = prob->dtype;
    char *base = (char *)ws;
    const void *xhat = Xhat_saved ? Xhat_saved : (const void *)(base + w.xhat);
    void *dyhat = base + w.dyhat, *dxhat = base + w.dxhat;
    float *part = (float *)(base + w.part), *dprime = (float *)(base + w.dprime), *gtail = (float *)(base + w.gtail);
    const bool want_fold = g.nrho && dfold;
    const bool need_yhat = dD || want_fold;

    if ((dWhat || (need_yhat && !Yhat_saved)) && !Xhat_saved)
        STL_HIP(stl::launch_encode(dt, X, E_X, base + w.xhat, d.M, d.K, d.r, PG, s, g.map(0)), "ragged_backward/encode X");
    const void *yhat = Yhat_saved;
    if (need_yhat && !yhat) {
        stl::GemmDesc gd{d.M, d.N, d.K, d.r, false, true, false, false, PG, 0, PG};
        STL_HIP(stl::launch_plane_gemm(dt, gd, xhat, What, base + w.yhat, s), "ragged_backward/recompute Yhat");
        yhat = base + w.yhat;
    }
    // dYhat and dD from the complete tile rows (all of them when nothing is ragged) ...
    const stl::RowMap body = g.map(1);
    if (dD && stl::encode_outer_eligible(dt, d.N)) {
        STL_HIP(stl::launch_encode_outer(dC, D, dyhat, yhat, dD, part, d.M, d.N, d.r, accumulate, PG, s, body), "ragged_backward/dYhat + dD");
    } else {
        STL_HIP(stl::launch_encode(dt, dC, D, dyhat, d.M, d.N, d.r, PG, s, body), "ragged_backward/encode dC");
        if (dD) STL_HIP(stl::launch_outer_reduce(dt, yhat, dC, dD, part, d.M, d.N, d.r, accumulate, PG, s, body), "ragged_backward/dD");
    }
    if (g.nrho) {
        // ... and from each image's last tile row through the fold: its adjoint is an encode with the composed decoder;
        // one product Yhat (x) dC over those tile rows feeds both dD and dfold
        const stl::RowMap tail = g.map(2);
        STL_HIP(stl::launch_fold_decoder(dt, D, fold, dprime, d.r, g.nrho, s), "ragged_backward/compose fold");
        STL_HIP(stl::launch_encode(dt, dC, dprime, dyhat, d.M, d.N, d.r, PG, s, tail, true), "ragged_backward/encode folded dC");
        if (dD || want_fold) {
            STL_HIP(stl::launch_outer_reduce(dt, yhat, dC, gtail, part, d.M, d.N, d.r, 0, PG, s, tail), "ragged_backward/last tile rows");
            STL_HIP(stl::launch_fold_grads(dt, gtail, D, fold, dD, dfold, d.r, g.nrho, accumulate, s), "ragged_backward/dD + dfold");
        }
    }
    if (dX || dE_X) {
        stl::GemmDesc gd{d.M, d.K, d.N, d.r, false, false, false, false, PG, 0, PG};
        STL_HIP(stl::launch_plane_gemm(dt, gd, dyhat, What, dxhat, s), "ragged_backward/dXhat");
    }
    if (dWhat) {
        stl::GemmDesc gd{d.K, d.N, d.M, d.r, true, true, true, accumulate != 0, PG, PG, 0};
        STL_HIP(stl::launch_plane_gemm(dt, gd, xhat, dyhat, dWhat, s), "ragged_backward/dWhat");
    }
    // gradients of null rows are dropped (never written); null rows of X count as zeros in dE_X
    const stl::RowMap all = g.map(0);
    if (dX && dE_X && stl::decode_outer_eligible(dt, d.K)) {
        STL_HIP(stl::launch_decode_outer(dxhat, E_X, dX, X, dE_X, part, d.M, d.K, d.r, accumulate, PG, s, all), "ragged_backward/dX + dE_X");
    } else {
        if (dX) STL_HIP(stl::launch_decode(dt, dxhat, E_X, dX, d.M, d.K, d.r, false, PG, s, all), "ragged_backward/decode dX");
        if (dE_X)
            STL_HIP(stl::launch_outer_reduce(dt, dxhat, X, dE_X, part, d.M, d.K, d.r, accumulate, PG, s, all), "ragged_backward/dE_X");
    }
    return STL_OK;
}

}  // extern "C"
