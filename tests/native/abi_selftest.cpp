// Native self-test of the C ABI: a program with no Python and no torch in it
// calls grkan_fwd / grkan_bwd / grkan_bwd_noalloc / grkan_linear_fwd through
// include/grkan.h on buffers it allocates with the HIP runtime and compares
// every output with the fp64 C oracle
// (oracle/grkan_oracle.c, linked in as the checker) under the same error
// measure as the Python parity tests.  Inputs come from a small counter-based
// generator of its own (data only).  Built and run by tests/test_gpu_native.py.
//
//   abi_selftest            runs the built-in list of cases, prints one line each
//   exit status 0 = all within tolerance
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "grkan.h"

extern "C" {
int grkan_oracle_fwd(const double *x, const double *A, const double *B, double *y, int64_t rows, int D, int G, int m,
                     int n, int threads);
int grkan_oracle_bwd(const double *x, const double *dy, const double *A, const double *B, double *dx, double *dA,
                     double *dB, int64_t rows, int D, int G, int m, int n, int threads);
int grkan_oracle_scales(const double *x, const double *dy, const double *A, const double *B, double *Sy, double *Sdx,
                        double *RA, double *RB, int64_t rows, int D, int G, int m, int n, int threads);
int grkan_oracle_linear_fwd(const double *x, const double *A, const double *B, const double *W, const double *bias,
                            double *out, int64_t rows, int D_in, int D_out, int G, int m, int n, int round_operand,
                            int threads);
}

#define HIP_OK(call)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess) {                                                                        \
            std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);         \
            std::exit(2);                                                                              \
        }                                                                                              \
    } while (0)

// splitmix64 -> uniform in [0, 1); Box-Muller for normals.  Data only.
struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed) {}
    uint64_t next()
    {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
    double normal()
    {
        const double u = 1.0 - uniform(), v = uniform();
        return std::sqrt(-2.0 * std::log(u)) * std::cos(6.283185307179586 * v);
    }
};

struct Case {
    int64_t rows;
    int D, G, m, n;
};

static bool run_case(const Case &c, uint64_t seed)
{
    const int64_t M = c.rows * c.D;
    const int na = c.G * (c.m + 1), nb = c.G * c.n;
    Rng rng(seed);
    std::vector<float> A(na), B(nb), x(M), dy(M);
    for (int g = 0; g < c.G; ++g)
        for (int i = 0; i <= c.m; ++i)
            A[g * (c.m + 1) + i] = (float)((2.0 * rng.uniform() - 1.0) / (i + 1.0));
    for (int j = 0; j < nb; ++j)
        B[j] = (float)(rng.uniform() - 0.5);
    for (int64_t e = 0; e < M; ++e) {
        x[e] = (float)rng.normal();
        dy[e] = (float)rng.normal();
    }

    // device side, through the C ABI only
    void *d_x, *d_dy, *d_y, *d_dx, *d_ws;
    float *d_A, *d_B, *d_dA, *d_dB;
    const size_t bytes = (size_t)M * sizeof(float);
    HIP_OK(hipMalloc(&d_x, bytes ? bytes : 16));
    HIP_OK(hipMalloc(&d_dy, bytes ? bytes : 16));
    HIP_OK(hipMalloc(&d_y, bytes ? bytes : 16));
    HIP_OK(hipMalloc(&d_dx, bytes ? bytes : 16));
    HIP_OK(hipMalloc((void **)&d_A, na * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_B, nb * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_dA, na * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_dB, nb * sizeof(float)));
    const size_t ws_bytes = grkan_bwd_workspace_bytes(c.rows, c.D, c.G, GRKAN_F32);
    if (ws_bytes == 0) {
        std::printf("workspace query failed\n");
        return false;
    }
    HIP_OK(hipMalloc(&d_ws, ws_bytes));
    HIP_OK(hipMemcpy(d_x, x.data(), bytes, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_dy, dy.data(), bytes, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_A, A.data(), na * sizeof(float), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_B, B.data(), nb * sizeof(float), hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    grkan_status_t st = grkan_fwd(d_x, d_A, d_B, d_y, c.rows, c.D, c.G, c.m, c.n, GRKAN_F32, stream);
    if (st == GRKAN_OK)
        st = grkan_bwd(d_x, d_dy, d_A, d_B, d_dx, d_dA, d_dB, d_ws, ws_bytes, c.rows, c.D, c.G, c.m, c.n, GRKAN_F32,
                       stream);
    // the allocation-free variant into buffers of its own: must agree bit for bit
    void *d_dx2;
    float *d_dA2, *d_dB2;
    HIP_OK(hipMalloc(&d_dx2, bytes ? bytes : 16));
    HIP_OK(hipMalloc((void **)&d_dA2, na * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_dB2, nb * sizeof(float)));
    if (st == GRKAN_OK)
        st = grkan_bwd_noalloc(d_x, d_dy, d_A, d_B, d_dx2, d_dA2, d_dB2, c.rows, c.D, c.G, c.m, c.n, GRKAN_F32, stream);
    if (st != GRKAN_OK) {
        std::printf("entry point failed: %s\n", grkan_status_string(st));
        return false;
    }
    HIP_OK(hipStreamSynchronize(stream));
    std::vector<float> y(M), dx(M), dA(na), dB(nb);
    {
        std::vector<float> dx2(M), dA2(na), dB2(nb);
        HIP_OK(hipMemcpy(dx2.data(), d_dx2, bytes, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dA2.data(), d_dA2, na * sizeof(float), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dB2.data(), d_dB2, nb * sizeof(float), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dx.data(), d_dx, bytes, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dA.data(), d_dA, na * sizeof(float), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(dB.data(), d_dB, nb * sizeof(float), hipMemcpyDeviceToHost));
        if (std::memcmp(dx2.data(), dx.data(), bytes) || std::memcmp(dA2.data(), dA.data(), na * sizeof(float)) ||
            std::memcmp(dB2.data(), dB.data(), nb * sizeof(float))) {
            std::printf("FAIL grkan_bwd_noalloc differs from grkan_bwd\n");
            return false;
        }
    }
    for (void *p : {d_dx2, (void *)d_dA2, (void *)d_dB2})
        HIP_OK(hipFree(p));
    HIP_OK(hipMemcpy(y.data(), d_y, bytes, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dx.data(), d_dx, bytes, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dA.data(), d_dA, na * sizeof(float), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dB.data(), d_dB, nb * sizeof(float), hipMemcpyDeviceToHost));
    HIP_OK(hipStreamDestroy(stream));
    for (void *p : {d_x, d_dy, d_y, d_dx, d_ws, (void *)d_A, (void *)d_B, (void *)d_dA, (void *)d_dB})
        HIP_OK(hipFree(p));

    // checker: the fp64 oracle on the same values
    std::vector<double> xd(x.begin(), x.end()), dyd(dy.begin(), dy.end()), Ad(A.begin(), A.end()),
        Bd(B.begin(), B.end());
    std::vector<double> ry(M), rdx(M), rdA(na), rdB(nb), Sy(M), Sdx(M), RA(na), RB(nb);
    const int threads = 8;
    if (grkan_oracle_fwd(xd.data(), Ad.data(), Bd.data(), ry.data(), c.rows, c.D, c.G, c.m, c.n, threads) ||
        grkan_oracle_bwd(xd.data(), dyd.data(), Ad.data(), Bd.data(), rdx.data(), rdA.data(), rdB.data(), c.rows, c.D,
                         c.G, c.m, c.n, threads) ||
        grkan_oracle_scales(xd.data(), dyd.data(), Ad.data(), Bd.data(), Sy.data(), Sdx.data(), RA.data(), RB.data(),
                            c.rows, c.D, c.G, c.m, c.n, threads)) {
        std::printf("oracle rejected the case\n");
        return false;
    }
    auto worst = [](const std::vector<float> &g, const std::vector<double> &r, const std::vector<double> &s) {
        double w = 0.0;
        for (size_t i = 0; i < g.size(); ++i) {
            const double scale = std::fmax(std::fmax(std::fabs(r[i]), s[i]), 1e-300);
            const double e = std::fabs((double)g[i] - r[i]) / scale;
            if (!(e <= w)) // also catches NaN
                w = std::isnan(e) ? INFINITY : e;
        }
        return w;
    };
    const double ey = worst(y, ry, Sy), edx = worst(dx, rdx, Sdx), eA = worst(dA, rdA, RA), eB = worst(dB, rdB, RB);
    const bool ok = ey <= 1e-5 && edx <= 1e-5 && eA <= 1e-4 && eB <= 1e-4;
    std::printf("%s rows %lld D %d G %d (%d,%d): y %.2e dx %.2e dA %.2e dB %.2e\n", ok ? "ok  " : "FAIL",
                (long long)c.rows, c.D, c.G, c.m, c.n, ey, edx, eA, eB);
    std::fflush(stdout);
    return ok;
}

// ---- the fused layer, out = W F(x) + bias (bfloat16 x and W, float32 out) ----
static uint16_t to_bf16(float v) // round to nearest even; data preparation only
{
    uint32_t u;
    std::memcpy(&u, &v, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static float from_bf16(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;
    float v;
    std::memcpy(&v, &u, 4);
    return v;
}

struct LinCase {
    int64_t rows;
    int D_in, D_out, G;
};

static bool run_linear_case(const LinCase &c, uint64_t seed)
{
    const int m = 5, n = 4;
    const int64_t MX = c.rows * c.D_in, MO = c.rows * c.D_out;
    const int64_t MW = (int64_t)c.D_out * c.D_in;
    Rng rng(seed);
    std::vector<float> A(c.G * (m + 1)), B(c.G * n), bias(c.D_out);
    for (int g = 0; g < c.G; ++g)
        for (int i = 0; i <= m; ++i)
            A[g * (m + 1) + i] = (float)((2.0 * rng.uniform() - 1.0) / (i + 1.0));
    for (auto &b : B)
        b = (float)(rng.uniform() - 0.5);
    for (auto &b : bias)
        b = (float)(0.1 * rng.normal());
    std::vector<uint16_t> xb(MX), Wb(MW);
    std::vector<double> xd(MX), Wd(MW);
    for (int64_t e = 0; e < MX; ++e) {
        xb[e] = to_bf16((float)rng.normal());
        xd[e] = from_bf16(xb[e]);
    }
    const double wscale = 1.0 / std::sqrt((double)c.D_in);
    for (int64_t e = 0; e < MW; ++e) {
        Wb[e] = to_bf16((float)(wscale * rng.normal()));
        Wd[e] = from_bf16(Wb[e]);
    }
    void *d_x, *d_W, *d_out;
    float *d_A, *d_B, *d_bias;
    HIP_OK(hipMalloc(&d_x, MX * 2));
    HIP_OK(hipMalloc(&d_W, MW * 2));
    HIP_OK(hipMalloc(&d_out, MO * 4));
    HIP_OK(hipMalloc((void **)&d_A, A.size() * 4));
    HIP_OK(hipMalloc((void **)&d_B, B.size() * 4));
    HIP_OK(hipMalloc((void **)&d_bias, bias.size() * 4));
    HIP_OK(hipMemcpy(d_x, xb.data(), MX * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_W, Wb.data(), MW * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_A, A.data(), A.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_B, B.data(), B.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_bias, bias.data(), bias.size() * 4, hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    const grkan_status_t st = grkan_linear_fwd(d_x, d_A, d_B, d_W, d_bias, d_out, c.rows, c.D_in, c.D_out, c.G, m, n,
                                               GRKAN_BF16, GRKAN_F32, stream);
    if (st != GRKAN_OK) {
        std::printf("grkan_linear_fwd failed: %s\n", grkan_status_string(st));
        return false;
    }
    HIP_OK(hipStreamSynchronize(stream));
    std::vector<float> out(MO);
    HIP_OK(hipMemcpy(out.data(), d_out, MO * 4, hipMemcpyDeviceToHost));
    {
        // the same layer from the packed copy of the weights: bit-identical
        const size_t pbytes = grkan_linear_packed_w_bytes(c.D_in, c.D_out);
        void *d_Wp, *d_out2;
        if (pbytes == 0) {
            std::printf("FAIL grkan_linear_packed_w_bytes returned 0\n");
            return false;
        }
        HIP_OK(hipMalloc(&d_Wp, pbytes));
        HIP_OK(hipMalloc(&d_out2, MO * 4));
        grkan_status_t sp = grkan_linear_pack_w(d_W, d_Wp, c.D_in, c.D_out, stream);
        if (sp == GRKAN_OK)
            sp = grkan_linear_fwd_packed(d_x, d_A, d_B, d_Wp, d_bias, d_out2, c.rows, c.D_in, c.D_out, c.G, m, n,
                                         GRKAN_BF16, GRKAN_F32, stream);
        if (sp != GRKAN_OK) {
            std::printf("packed path failed: %s\n", grkan_status_string(sp));
            return false;
        }
        HIP_OK(hipStreamSynchronize(stream));
        std::vector<float> out2(MO);
        HIP_OK(hipMemcpy(out2.data(), d_out2, MO * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipFree(d_Wp));
        HIP_OK(hipFree(d_out2));
        if (std::memcmp(out.data(), out2.data(), MO * 4)) {
            std::printf("FAIL grkan_linear_fwd_packed differs from grkan_linear_fwd\n");
            return false;
        }
    }
    HIP_OK(hipStreamDestroy(stream));
    for (void *p : {d_x, d_W, d_out, (void *)d_A, (void *)d_B, (void *)d_bias})
        HIP_OK(hipFree(p));

    // checker: the definition in fp64, and the scale of a sum of D_in terms, R = sqrt(sum (W F)^2)
    std::vector<double> Ad(A.begin(), A.end()), Bd(B.begin(), B.end()), bd(bias.begin(), bias.end());
    std::vector<double> ref(MO), F(MX);
    if (grkan_oracle_linear_fwd(xd.data(), Ad.data(), Bd.data(), Wd.data(), bd.data(), ref.data(), c.rows, c.D_in,
                                c.D_out, c.G, m, n, 0, 8) ||
        grkan_oracle_fwd(xd.data(), Ad.data(), Bd.data(), F.data(), c.rows, c.D_in, c.G, m, n, 8)) {
        std::printf("oracle rejected the case\n");
        return false;
    }
    double worst = 0.0;
    for (int64_t r = 0; r < c.rows; ++r)
        for (int o = 0; o < c.D_out; ++o) {
            double ss = 0.0;
            for (int k = 0; k < c.D_in; ++k) {
                const double t = Wd[(int64_t)o * c.D_in + k] * F[r * c.D_in + k];
                ss += t * t;
            }
            const double rv = ref[r * c.D_out + o];
            const double e = std::fabs((double)out[r * c.D_out + o] - rv) / std::fmax(std::fmax(std::fabs(rv), std::sqrt(ss)), 1e-300);
            if (!(e <= worst))
                worst = std::isnan(e) ? INFINITY : e;
        }
    // operand rounding to bfloat16: 7.5 sigma of a sum of independent half-ulp errors (see the GPU tests)
    const bool ok = worst <= 1.2e-2;
    std::printf("%s layer rows %lld D_in %d D_out %d G %d: out %.2e\n", ok ? "ok  " : "FAIL", (long long)c.rows, c.D_in,
                c.D_out, c.G, worst);
    std::fflush(stdout);
    return ok;
}

int main()
{
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev == 0) {
        std::printf("no HIP device\n");
        return 3;
    }
    HIP_OK(hipSetDevice(0));
    const Case cases[] = {
        {788, 192, 8, 5, 4},   // the tiny configuration's shape (flat walk)
        {999, 768, 8, 5, 4},   // group walk, ragged tail
        {301, 3072, 8, 5, 4},  // the headline segment length
        {129, 3072, 1, 5, 4},  // one group, cut into column blocks
        {257, 1536, 64, 3, 2}, // many short groups, other degrees
        {33, 30, 5, 7, 6},     // two-wide vectors
        {0, 192, 8, 5, 4},     // empty
    };
    bool all = true;
    uint64_t seed = 20250513;
    for (const Case &c : cases)
        all = run_case(c, seed++) && all;
    const LinCase lin_cases[] = {
        {250, 3072, 768, 8}, // the wide layer's shape: eight-wave tile, ragged token block
        {333, 768, 384, 8},  // the 384-channel tile
        {97, 256, 200, 4},   // partial last channel block
    };
    for (const LinCase &c : lin_cases)
        all = run_linear_case(c, seed++) && all;
    std::printf(all ? "all cases within tolerance\n" : "SOME CASES FAILED\n");
    return all ? 0 : 1;
}
