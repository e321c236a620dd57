// Driver of the CPU address check (test infrastructure only): calls the C ABI entry points on host buffers whose end
// coincides with the end of their allocation, under AddressSanitizer.  Each command-line argument is one case:
//   fwd:m:k:n:r:flags   bwd:m:k:n:r   mlp:m:k:h:r   ewb:k:n:r   aa:nb:m:k:n:r   ragged:nimg:rows:k:n:r
//   plant   (a planted mistake -- an output buffer 32 bytes short -- that the sanitizer must report)
// A leading "f32," selects fp32 storage (default bf16).
#include "stl.h"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

static void *exact(size_t bytes)
{
    const size_t tot = (bytes + 255) / 256 * 256;
    char *p = (char *)aligned_alloc(256, tot ? tot : 256);
    if (!p) abort();
    memset(p, 0, tot ? tot : 256);
    return p + (tot - bytes) / 16 * 16;     // 16-byte aligned, at most 15 bytes of slack before the redzone
}
#define CHECK(x)                                                          \
    do {                                                                  \
        int st__ = (x);                                                   \
        if (st__) {                                                       \
            printf("status %d: %s\n", st__, stl_last_error());            \
            exit(3);                                                      \
        }                                                                 \
    } while (0)

int main(int argc, char **argv)
{
    for (int a = 1; a < argc; ++a) {
        std::string arg = argv[a];
        int dt = STL_BF16;
        if (arg.rfind("f32,", 0) == 0) { dt = STL_F32; arg = arg.substr(4); }
        const size_t es = dt == STL_F32 ? 4 : 2;
        std::vector<long> v;
        std::string op = arg.substr(0, arg.find(':'));
        for (size_t pos = arg.find(':'); pos != std::string::npos; pos = arg.find(':', pos + 1)) v.push_back(atol(arg.c_str() + pos + 1));
        printf("case %s\n", argv[a]);
        fflush(stdout);
        if (op == "plant") {
            stl_problem_t p{256, 128, 256, 4, 32, STL_BF16};
            void *A = exact(3 * 256 * 128 * 2), *B = exact(3 * 128 * 256 * 2), *C = exact(3 * 256 * 256 * 2 - 32), *E = exact(1024);
            const size_t wf = stl_aa_workspace_bytes(&p, 3, STL_OP_FORWARD);
            CHECK(stl_aa_forward(&p, 3, A, B, E, E, E, C, nullptr, nullptr, nullptr, exact(wf), wf, 0, nullptr));
        } else if (op == "fwd" || op == "bwd") {
            const long m = v[0], k = v[1], n = v[2];
            const int r = (int)v[3], flags = op == "fwd" ? (int)v[4] : 0;
            stl_problem_t p{m, k, n, 4, r, dt};
            void *X = exact(m * k * es), *Wh = exact((size_t)r * (k / 4) * (n / 4) * es), *E = exact(r * 16 * es), *D = exact(r * 16 * es);
            void *C = exact(m * n * es);
            void *Xh = exact(stl_plane_elems(m / 4, k / 4, r) * es), *Yh = exact(stl_plane_elems(m / 4, n / 4, r) * es);
            const size_t wf = stl_workspace_bytes(&p, STL_OP_FORWARD, flags);
            const bool fused = (flags & 0xff) == STL_FLAG_FUSED;
            CHECK(stl_forward(&p, X, Wh, E, D, C, nullptr, nullptr, exact(wf), wf, flags, nullptr));
            CHECK(stl_forward(&p, X, Wh, E, D, C, fused ? nullptr : Xh, Yh, exact(wf), wf, flags, nullptr));
            if (op == "bwd") {
                const size_t wb = stl_workspace_bytes(&p, STL_OP_BACKWARD, 0);
                void *dC = exact(m * n * es), *dX = exact(m * k * es);
                float *dW = (float *)exact((size_t)r * (k / 4) * (n / 4) * 4), *g1 = (float *)exact(r * 64), *g2 = (float *)exact(r * 64);
                CHECK(stl_backward(&p, X, Wh, E, D, dC, nullptr, nullptr, dX, dW, g1, g2, 0, exact(wb), wb, nullptr));
                CHECK(stl_backward(&p, X, Wh, E, D, dC, Xh, Yh, dX, dW, g1, g2, 1, exact(wb), wb, nullptr));
                CHECK(stl_backward(&p, X, Wh, E, D, dC, Xh, Yh, dX, nullptr, nullptr, g2, 0, exact(wb), wb, nullptr));
                CHECK(stl_backward(&p, X, Wh, E, D, dC, nullptr, nullptr, nullptr, dW, g1, nullptr, 0, exact(wb), wb, nullptr));
            }
        } else if (op == "mlp") {
            const long m = v[0], k = v[1], h = v[2];
            const int r = (int)v[3];
            stl_problem_t up{m, k, h, 4, r, dt}, down{m, h, k, 4, r, dt};
            void *X = exact(m * k * es), *W1 = exact((size_t)r * (k / 4) * (h / 4) * es), *W2 = exact((size_t)r * (k / 4) * (h / 4) * es);
            void *E = exact(r * 16 * es), *C = exact(m * k * es);
            for (int flags : {(int)STL_FLAG_GELU, (int)(STL_FLAG_GELU | STL_FLAG_UNFUSED), 0}) {
                const size_t w = stl_mlp_workspace_bytes(&up, &down, flags);
                CHECK(stl_mlp_forward(&up, &down, X, W1, E, E, W2, E, E, C, exact(w), w, flags, nullptr));
            }
        } else if (op == "ewb") {
            const long k = v[0], n = v[1];
            const int r = (int)v[2];
            stl_problem_t p{4, k, n, 4, r, dt};
            void *W = exact(k * n * es), *E = exact(r * 16 * es), *dW = exact(k * n * es);
            float *dWh = (float *)exact((size_t)r * (k / 4) * (n / 4) * 4), *dE = (float *)exact(r * 64);
            const size_t w = stl_workspace_bytes(&p, STL_OP_ENCODE_WEIGHT_BACKWARD, 0);
            CHECK(stl_encode_weight(&p, W, E, exact((size_t)r * (k / 4) * (n / 4) * es), nullptr));
            CHECK(stl_encode_weight_backward(&p, W, E, dWh, dW, dE, 0, exact(w), w, nullptr));
            CHECK(stl_encode_weight_backward(&p, W, E, dWh, nullptr, dE, 1, exact(w), w, nullptr));
        } else if (op == "aa") {
            const long nb = v[0], m = v[1], k = v[2], n = v[3];
            const int r = (int)v[4];
            stl_problem_t p{m, k, n, 4, r, dt};
            void *A = exact(nb * m * k * es), *B = exact(nb * k * n * es), *C = exact(nb * m * n * es), *dC = exact(nb * m * n * es);
            void *Ea = exact(r * 16 * es), *Eb = exact(r * 16 * es), *D = exact(r * 16 * es);
            void *Ah = exact(stl_plane_elems(nb * m / 4, k / 4, r) * es), *Bh = exact(stl_plane_elems(nb * k / 4, n / 4, r) * es);
            void *Yh = exact(stl_plane_elems(nb * m / 4, n / 4, r) * es);
            const size_t wf = stl_aa_workspace_bytes(&p, nb, STL_OP_FORWARD), wb = stl_aa_workspace_bytes(&p, nb, STL_OP_BACKWARD);
            CHECK(stl_aa_forward(&p, nb, A, B, Ea, Eb, D, C, nullptr, nullptr, nullptr, exact(wf), wf, 0, nullptr));
            CHECK(stl_aa_forward(&p, nb, A, B, Ea, Eb, D, C, Ah, Bh, Yh, exact(wf), wf, STL_FLAG_GELU, nullptr));
            void *dA = exact(nb * m * k * es), *dB = exact(nb * k * n * es);
            float *g1 = (float *)exact(r * 64), *g2 = (float *)exact(r * 64), *g3 = (float *)exact(r * 64);
            CHECK(stl_aa_backward(&p, nb, A, B, Ea, Eb, D, dC, nullptr, nullptr, nullptr, dA, dB, g1, g2, g3, 0, exact(wb), wb, 0, nullptr));
            CHECK(stl_aa_backward(&p, nb, A, B, Ea, Eb, D, dC, Ah, Bh, Yh, dA, nullptr, nullptr, g2, nullptr, 1, exact(wb), wb, 0, nullptr));
            // the second operand stored transposed: the same bytes read as (nb*n) x k
            void *Bt = exact(stl_plane_elems(nb * n / 4, k / 4, r) * es);
            CHECK(stl_aa_forward(&p, nb, A, B, Ea, Eb, D, C, Ah, Bt, Yh, exact(wf), wf, STL_FLAG_B_TRANSPOSED, nullptr));
            CHECK(stl_aa_backward(&p, nb, A, B, Ea, Eb, D, dC, nullptr, nullptr, nullptr, dA, dB, g1, g2, g3, 0, exact(wb), wb, STL_FLAG_B_TRANSPOSED, nullptr));
            CHECK(stl_aa_backward(&p, nb, A, B, Ea, Eb, D, dC, Ah, Bt, Yh, nullptr, dB, nullptr, g2, nullptr, 1, exact(wb), wb, STL_FLAG_B_TRANSPOSED, nullptr));
        } else if (op == "ragged") {
            const long nimg = v[0], rows = v[1], k = v[2], n = v[3], m = nimg * rows;
            const int r = (int)v[4];
            stl_problem_t p{m, k, n, 4, r, dt};
            void *X = exact(m * k * es), *Wh = exact((size_t)r * (k / 4) * (n / 4) * es), *E = exact(r * 16 * es), *D = exact(r * 16 * es);
            void *C = exact(m * n * es), *dC = exact(m * n * es), *dX = exact(m * k * es);
            float *fold = (float *)exact(64), *df = (float *)exact(64);
            const long Rp = nimg * ((rows + 3) / 4);
            void *Xh = exact(stl_plane_elems(Rp, k / 4, r) * es), *Yh = exact(stl_plane_elems(Rp, n / 4, r) * es);
            const size_t wf = stl_ragged_workspace_bytes(&p, rows, STL_OP_FORWARD), wb = stl_ragged_workspace_bytes(&p, rows, STL_OP_BACKWARD);
            CHECK(stl_ragged_forward(&p, rows, X, Wh, E, D, fold, C, nullptr, nullptr, exact(wf), wf, nullptr));
            CHECK(stl_ragged_forward(&p, rows, X, Wh, E, D, fold, C, Xh, Yh, exact(wf), wf, nullptr));
            float *dW = (float *)exact((size_t)r * (k / 4) * (n / 4) * 4), *g1 = (float *)exact(r * 64), *g2 = (float *)exact(r * 64);
            CHECK(stl_ragged_backward(&p, rows, X, Wh, E, D, fold, dC, nullptr, nullptr, dX, dW, g1, g2, df, 0, exact(wb), wb, nullptr));
            CHECK(stl_ragged_backward(&p, rows, X, Wh, E, D, fold, dC, Xh, Yh, nullptr, nullptr, nullptr, nullptr, df, 1, exact(wb), wb, nullptr));
        } else {
            printf("unknown case %s\n", argv[a]);
            return 2;
        }
        printf("  ok\n");
        fflush(stdout);
    }
    return 0;
}
