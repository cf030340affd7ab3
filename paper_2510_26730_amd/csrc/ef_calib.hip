// Measured ceilings of the device for the roofline objects of the benchmark: what a plain streaming read gets out of
// HBM, and what the matrix cores deliver from registers.  Not part of the method; ef_measure_peak is declared in
// include/expertflow.h.
#include "ef_ctx.h"
#include "ef_device.h"

namespace {

// Every wave reads a contiguous share of the buffer, 1 KiB per instruction (64 lanes x 16 bytes, nontemporal), eight
// instructions in flight; the words are folded into one value per workgroup so that the loads are not optimised away.
__global__ __launch_bounds__(256) void peak_read_kernel(const ef::u32x4_t *__restrict__ p, long long units_per_wave,
                                                        uint32_t *__restrict__ sink) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long w = (long long)blockIdx.x * 4 + wave;
    const ef::u32x4_t *src = p + w * units_per_wave * 64 + lane;   // a unit = 64 lanes x 16 bytes
    ef::u32x4_t acc = {0u, 0u, 0u, 0u};
    long long u = 0;
    for (; u + 8 <= units_per_wave; u += 8) {
        ef::u32x4_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = __builtin_nontemporal_load(src + (u + q) * 64);
#pragma unroll
        for (int q = 0; q < 8; ++q) acc ^= v[q];
    }
    for (; u < units_per_wave; ++u) acc ^= __builtin_nontemporal_load(src + u * 64);
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off);
    if (lane == 0) atomicXor(&sink[blockIdx.x], x);
}

// Eight independent 32x32 accumulators per wave, operands in registers: nothing but the matrix cores is busy.
__global__ __launch_bounds__(256) void peak_mfma_kernel(int iters, float *__restrict__ sink) {
    const int lane = threadIdx.x & 63;
    ef::u32x4_t a, b;
    // bf16 pairs: small values that differ by lane, so the products are not constant-folded
    const uint32_t pa = 0x3C003C00u + (uint32_t)lane, pb = 0x3B803B80u + (uint32_t)(lane << 16);
    a = ef::u32x4_t{pa, pa, pa, pa};
    b = ef::u32x4_t{pb, pb, pb, pb};
    ef::floatx16 acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) ef::zero16(acc[q]);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = ef::mfma32v(a, b, acc[q]);
    }
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[q][v];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;   // never true: keeps the loop alive
}

}  // namespace

extern "C" int ef_measure_peak(ef_ctx *c, int what, const void *buf, size_t bytes, int reps, double *result,
                               void *stream) {
    using namespace efi;
    if (!c || !result) return fail(c, EF_EINVAL, "ef_measure_peak: null pointer");
    if (c->fake) return fail(c, EF_ENOSYS, "ef_measure_peak: fake-copy context has no device");
    if (reps < 1 || reps > 1000) return fail(c, EF_EINVAL, "ef_measure_peak: reps must be in 1..1000");
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    EF_HIP(c, hipEventCreate(&e0));
    hipError_t err = hipEventCreate(&e1);
    if (err != hipSuccess) { (void)hipEventDestroy(e0); return fail(c, EF_EHIP, "ef_measure_peak: %s", hipGetErrorString(err)); }
    auto done = [&](int rc) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return rc; };
    uint32_t *sink = reinterpret_cast<uint32_t *>(c->gate_part);   // at least 8 MiB of scratch
    float ms = 0.f;
    if (what == EF_PEAK_HBM_READ) {
        constexpr int kWgs = 2048;                                  // 8 workgroups of four waves per compute unit
        constexpr size_t kQuantum = (size_t)kWgs * 4 * 1024;        // a 1 KiB unit for every wave
        if (!buf || !aligned16(buf) || bytes < kQuantum || bytes % kQuantum != 0)
            return done(fail(c, EF_EINVAL, "ef_measure_peak: the buffer must be 16-byte aligned and a multiple of 8 MiB"));
        const long long upw = (long long)(bytes / kQuantum);
        // one untimed pass first: the timed ones see the clocks and the page tables of a running device
        hipLaunchKernelGGL(peak_read_kernel, dim3(kWgs), dim3(256), 0, s, static_cast<const ef::u32x4_t *>(buf), upw, sink);
        if ((err = hipEventRecord(e0, s)) != hipSuccess) return done(fail(c, EF_EHIP, "ef_measure_peak: %s", hipGetErrorString(err)));
        for (int r = 0; r < reps; ++r)
            hipLaunchKernelGGL(peak_read_kernel, dim3(kWgs), dim3(256), 0, s, static_cast<const ef::u32x4_t *>(buf), upw, sink);
        if ((err = hipEventRecord(e1, s)) != hipSuccess || (err = hipEventSynchronize(e1)) != hipSuccess ||
            (err = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess || (err = hipGetLastError()) != hipSuccess)
            return done(fail(c, EF_EHIP, "ef_measure_peak: %s", hipGetErrorString(err)));
        *result = (double)bytes * reps / (ms * 1e-3) / 1e9;
        return done(EF_OK);
    }
    if (what == EF_PEAK_MFMA_16BIT) {
        constexpr int kWgs = 2048, kIters = 4096;
        float *fs = reinterpret_cast<float *>(c->gate_part);       // 2048 x 256 floats = 2 MiB, never written
        hipLaunchKernelGGL(peak_mfma_kernel, dim3(kWgs), dim3(256), 0, s, kIters, fs);
        if ((err = hipEventRecord(e0, s)) != hipSuccess) return done(fail(c, EF_EHIP, "ef_measure_peak: %s", hipGetErrorString(err)));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(peak_mfma_kernel, dim3(kWgs), dim3(256), 0, s, kIters, fs);
        if ((err = hipEventRecord(e1, s)) != hipSuccess || (err = hipEventSynchronize(e1)) != hipSuccess ||
            (err = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess || (err = hipGetLastError()) != hipSuccess)
            return done(fail(c, EF_EHIP, "ef_measure_peak: %s", hipGetErrorString(err)));
        const double flops = (double)kWgs * 4 * kIters * 8 * (2.0 * 32 * 32 * 16) * reps;
        *result = flops / (ms * 1e-3) / 1e12;
        return done(EF_OK);
    }
    return done(fail(c, EF_EINVAL, "ef_measure_peak: unknown quantity %d", what));
}
