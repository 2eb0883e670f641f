// A caller of libqsim that knows nothing of Python or PyTorch: device memory from the HIP runtime,
// the entry points of include/qsim.h on a stream of its own, results compared bit for bit with the
// CPU oracle (oracle/qsim_ref.h).  TEST PROGRAM: it links the oracle, the library does not.
//
// Build (tests/conftest.py does it when the binary is missing):
//   hipcc -O2 -Iinclude -Ioracle tests/native/abi_roundtrip.cpp -Lpaper_1910_04540_amd -lqsim \
//         -Loracle -lqsim_ref -Wl,-rpath,... -o tests/native/abi_roundtrip
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "qsim.h"
#include "qsim_ref.h"

#define HIP_OK(call)                                                                                 \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) {                                                                      \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);               \
            return 2;                                                                                \
        }                                                                                            \
    } while (0)

static int failures = 0;

static void check(const char* what, const std::vector<float>& got, const std::vector<float>& want)
{
    size_t bad = 0, first = 0;
    for (size_t i = 0; i < got.size(); ++i) {
        uint32_t a, b;
        std::memcpy(&a, &got[i], 4);
        std::memcpy(&b, &want[i], 4);
        if (a != b && bad++ == 0) first = i;
    }
    if (bad) {
        std::printf("MISMATCH %s: %zu of %zu elements, first at %zu (%a vs %a)\n", what, bad, got.size(), first,
                    (double)got[first], (double)want[first]);
        ++failures;
    } else {
        std::printf("ok %s (%zu elements)\n", what, got.size());
    }
    std::fflush(stdout);
}

// A small seeded generator for inputs (not part of the method): values spread over many binades.
static std::vector<float> inputs(size_t n, uint64_t seed)
{
    std::vector<float> x(n);
    uint64_t s = seed * 0x9E3779B97F4A7C15ull + 1;
    for (size_t i = 0; i < n; ++i) {
        s = s * 6364136223846793005ull + 1442695040888963407ull;
        const double u = (double)(s >> 11) / 9007199254740992.0 - 0.5;            // [-0.5, 0.5)
        s = s * 6364136223846793005ull + 1442695040888963407ull;
        const int e = (int)((s >> 40) % 24) - 16;
        x[i] = (float)std::ldexp(u, e);
    }
    return x;
}

// `abi_roundtrip bench`: the headline workload timed by this program itself (HIP events around 300
// launches on three rotating buffer sets after 300 warm-up launches), as a cross-check of the figure
// the Python benchmark reports.
static int bench()
{
    const size_t n = 1ull << 26;
    const int sets = 3, reps = 300;
    std::vector<float> x = inputs(1 << 20, 4);
    float *in[sets], *out[sets];
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    for (int s = 0; s < sets; ++s) {
        HIP_OK(hipMalloc(&in[s], n * 4));
        HIP_OK(hipMalloc(&out[s], n * 4));
        for (size_t off = 0; off < n; off += x.size()) HIP_OK(hipMemcpy(in[s] + off, x.data(), x.size() * 4, hipMemcpyHostToDevice));
    }
    hipEvent_t e0, e1;
    HIP_OK(hipEventCreate(&e0));
    HIP_OK(hipEventCreate(&e1));
    for (int r = 0; r < reps; ++r)
        if (qsim_fixed_quantize(in[r % sets], out[r % sets], n, 8, 6, QSIM_STOCHASTIC, QSIM_SATURATE, 1234, r, stream) != QSIM_OK) return 3;
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipEventRecord(e0, stream));
    for (int r = 0; r < reps; ++r)
        if (qsim_fixed_quantize(in[r % sets], out[r % sets], n, 8, 6, QSIM_STOCHASTIC, QSIM_SATURATE, 1234, r, stream) != QSIM_OK) return 3;
    HIP_OK(hipEventRecord(e1, stream));
    HIP_OK(hipEventSynchronize(e1));
    float ms = 0;
    HIP_OK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / reps;
    std::printf("fixed(8,6) stochastic, %zu elements: %.1f us per call, %.1f G elements/s, %.0f GB/s = %.1f %% of 8 TB/s\n", n, us,
                n / us / 1e3, n * 8.0 / us / 1e3, n * 8.0 / us / 1e3 / 80.0);
    for (int s = 0; s < sets; ++s) {
        HIP_OK(hipFree(in[s]));
        HIP_OK(hipFree(out[s]));
    }
    return 0;
}

int main(int argc, char** argv)
{
    if (argc > 1 && std::strcmp(argv[1], "bench") == 0) return bench();
    int devices = 0;
    HIP_OK(hipGetDeviceCount(&devices));
    if (devices == 0) {
        std::printf("no GPU\n");
        return 2;
    }
    HIP_OK(hipSetDevice(0));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    const size_t n = 1000003;                                  // ragged on purpose
    const std::vector<float> x = inputs(n, 1);
    float *d_in = nullptr, *d_out = nullptr;
    HIP_OK(hipMalloc(&d_in, n * 4));
    HIP_OK(hipMalloc(&d_out, n * 4));
    HIP_OK(hipMemcpy(d_in, x.data(), n * 4, hipMemcpyHostToDevice));
    std::vector<float> got(n), want(n);

    // fixed point (8, 6), stochastic, saturating
    if (qsim_fixed_quantize(d_in, d_out, n, 8, 6, QSIM_STOCHASTIC, QSIM_SATURATE, 1234, 7, stream) != QSIM_OK) return 3;
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(got.data(), d_out, n * 4, hipMemcpyDeviceToHost));
    qsim_ref_fixed_quantize(x.data(), want.data(), n, 8, 6, QSIM_REF_STOCHASTIC, QSIM_REF_SATURATE, 1234, 7);
    check("fixed(8,6) stochastic", got, want);

    // floating point (5, 2), nearest even, gradual underflow
    if (qsim_float_quantize(d_in, d_out, n, 5, 2, QSIM_RN_EVEN, QSIM_SATURATE | QSIM_SUBNORMAL, 0, 0, stream) != QSIM_OK) return 3;
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(got.data(), d_out, n * 4, hipMemcpyDeviceToHost));
    qsim_ref_float_quantize(x.data(), want.data(), n, 5, 2, QSIM_REF_RN_EVEN, QSIM_REF_SATURATE | QSIM_REF_SUBNORMAL, 0, 0);
    check("float(5,2) nearest even with subnormals", got, want);

    // block floating point: rows of 1000, the whole tensor, blocks along the middle of [7, 11, 12987]
    const struct { uint64_t outer, nblocks, inner, count; const char* what; } shapes[] = {
        {1, 1001, 1000, n, "block8 per row of 1000 (short last row)"},
        {1, 1, n, n, "block8 whole tensor"},
        {7, 11, 12987, 7ull * 11 * 12987, "block8 along the middle dimension of [7, 11, 12987]"},
    };
    for (const auto& s : shapes) {
        const size_t ws_bytes = qsim_block_workspace_bytes(s.count, s.outer, s.nblocks, s.inner);
        void* ws = nullptr;
        if (ws_bytes) HIP_OK(hipMalloc(&ws, ws_bytes));
        if (qsim_block_quantize(d_in, d_out, s.count, s.outer, s.nblocks, s.inner, 8, QSIM_STOCHASTIC, 0, 99, 3, ws, ws_bytes,
                                stream) != QSIM_OK)
            return 3;
        HIP_OK(hipStreamSynchronize(stream));
        got.resize(s.count);
        want.resize(s.count);
        HIP_OK(hipMemcpy(got.data(), d_out, s.count * 4, hipMemcpyDeviceToHost));
        qsim_ref_block_quantize(x.data(), want.data(), s.count, s.outer, s.nblocks, s.inner, 8, QSIM_REF_STOCHASTIC, 0, 99, 3);
        check(s.what, got, want);
        if (ws) HIP_OK(hipFree(ws));
    }

    // the fused SGD step: gradient float(5,2) stochastic, momentum fixed(16,12) stochastic, weight block8 per 256
    {
        std::vector<float> w = inputs(n, 2), g = inputs(n, 3), m(n, 0.0f), wq(n), rw = w, rm = m, rq(n);
        for (auto& v : g) v *= 1e-3f;
        float *d_w, *d_g, *d_m, *d_q;
        HIP_OK(hipMalloc(&d_w, n * 4));
        HIP_OK(hipMalloc(&d_g, n * 4));
        HIP_OK(hipMalloc(&d_m, n * 4));
        HIP_OK(hipMalloc(&d_q, n * 4));
        HIP_OK(hipMemcpy(d_w, w.data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(d_g, g.data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(d_m, m.data(), n * 4, hipMemcpyHostToDevice));
        const qsim_format fg{1, 5, 2, QSIM_STOCHASTIC, QSIM_SATURATE | QSIM_SUBNORMAL}, fm{2, 16, 12, QSIM_STOCHASTIC, QSIM_SATURATE},
            fw{3, 8, 256, QSIM_RN_EVEN, 0};
        const qsim_ref_format rg{1, 5, 2, QSIM_REF_STOCHASTIC, QSIM_REF_SATURATE | QSIM_REF_SUBNORMAL},
            rmf{2, 16, 12, QSIM_REF_STOCHASTIC, QSIM_REF_SATURATE}, rwf{3, 8, 256, QSIM_REF_RN_EVEN, 0};
        for (uint32_t step = 0; step < 2; ++step) {
            if (qsim_quant_sgd_step(d_w, d_q, d_g, d_m, n, 0.1f, 0.9f, &fg, &fm, &fw, 5, step, stream) != QSIM_OK) return 3;
            qsim_ref_quant_sgd_step(rw.data(), rq.data(), g.data(), rm.data(), n, 0.1f, 0.9f, &rg, &rmf, &rwf, 5, step);
        }
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(w.data(), d_w, n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(m.data(), d_m, n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(wq.data(), d_q, n * 4, hipMemcpyDeviceToHost));
        check("sgd master weights after two steps", w, rw);
        check("sgd momentum after two steps", m, rm);
        check("sgd quantized weights after two steps", wq, rq);
        HIP_OK(hipFree(d_w));
        HIP_OK(hipFree(d_g));
        HIP_OK(hipFree(d_m));
        HIP_OK(hipFree(d_q));
    }

    // error paths answer without touching the GPU
    if (qsim_fixed_quantize(d_in, d_out, n, 25, 6, QSIM_RN_EVEN, 0, 0, 0, stream) != QSIM_ERR_FORMAT) ++failures;
    if (qsim_fixed_quantize(d_in, d_in + 1, n - 1, 8, 6, QSIM_RN_EVEN, 0, 0, 0, stream) != QSIM_ERR_OVERLAP) ++failures;
    std::printf("status strings: %s / %s\n", qsim_status_string(QSIM_OK), qsim_status_string(QSIM_ERR_OVERLAP));

    HIP_OK(hipFree(d_in));
    HIP_OK(hipFree(d_out));
    HIP_OK(hipStreamDestroy(stream));
    std::printf(failures ? "FAILED (%d)\n" : "all ok\n", failures);
    return failures ? 1 : 0;
}
