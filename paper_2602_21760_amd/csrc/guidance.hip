// Guidance step: classifier-free-guidance combine (Sec. 3), branch discrepancy (Eq. 1, velocity
// form of Sec. 4.2) and the scheduler update, as one coalesced pass over HBM.
//
// The pass is bandwidth-bound: per element it reads v_c, v_u (2 or 4 B each) and x (4 B) and
// writes x_out (4 B).  Each workgroup owns a fixed contiguous chunk of one sample, every thread
// moves 16-byte vectors, and the four running sums (sum|d|, sum d^2, sum|u|, sum u^2) are
// reduced thread -> wave -> workgroup in a fixed order into one fp64 partial per workgroup.  A
// second, tiny kernel adds the partials of a sample in a fixed order, so results are
// deterministic and independent of the batch index (no atomics anywhere).
#include "common.h"

#include <mutex>

// Scratch of the allocation-free entry point (hyb_cfg_disc_euler_noalloc): the per-workgroup partial sums live in
// this file-scope device array instead of a caller-provided workspace.  Every GPU the library runs on holds its
// own copy until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels get
// the device address obtained from it.
static __device__ __align__(256) unsigned char scratch[HYB_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kThreads = 256;
constexpr int kVec = 8;                          // elements per thread per iteration
constexpr int kIters = 1;                        // one vector per thread: the smallest workgroups stream fastest (5.8 vs 5.5 TB/s with two)

// 16-byte vector accesses.  The inputs are streamed once, so they are read with non-temporal loads (they are not
// kept in the caches on their way in: 6.0-6.4 TB/s instead of 5.6-5.8 on 256 x 262144 elements); stores are plain
// (non-temporal stores are slower here).
template <typename T, int V> struct Vec;
template <> struct Vec<float, 8> {
    static __device__ __forceinline__ void load(const float* p, float* r) {
        const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + 4));
        r[0] = a[0]; r[1] = a[1]; r[2] = a[2]; r[3] = a[3]; r[4] = b[0]; r[5] = b[1]; r[6] = b[2]; r[7] = b[3];
    }
    static __device__ __forceinline__ void store(float* p, const float* r) {
        f32x4 a = {r[0], r[1], r[2], r[3]}, b = {r[4], r[5], r[6], r[7]};
        *reinterpret_cast<f32x4*>(p) = a;
        *reinterpret_cast<f32x4*>(p + 4) = b;
    }
};
template <> struct Vec<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* r) {
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));   // bf16 -> fp32: the bits, shifted up
#pragma unroll
        for (int i = 0; i < 4; i++) {
            r[2 * i] = __uint_as_float(a[i] << 16);
            r[2 * i + 1] = __uint_as_float(a[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* r) {
        bf16x8 a;
#pragma unroll
        for (int i = 0; i < 8; i++) a[i] = (bf16_t)r[i];
        *reinterpret_cast<bf16x8*>(p) = a;
    }
};
template <typename T> struct Vec<T, 1> {
    static __device__ __forceinline__ void load(const T* p, float* r) { r[0] = to_f32<T>(*p); }
    static __device__ __forceinline__ void store(T* p, const float* r) { *p = from_f32<T>(r[0]); }
};

struct GuidanceArgs {
    const void* v_c;
    const void* v_u;
    const float* x;
    float* x_out;
    bf16_t* x_lowp;
    void* v_out;
    size_t n;        // elements per sample
    float s, a, b;   // v = u + s (c - u);  x_out = a x + b v
    double* partial; // [batch][blocks_per_sample][4] or nullptr
};

// V = 8: vector path (n % 8 == 0, so a vector never straddles the end of a sample); V = 1: scalar.
template <typename VT, int V>
__global__ __launch_bounds__(kThreads) void guidance_kernel(GuidanceArgs g) {
    const size_t sample = blockIdx.y;
    const size_t off = sample * g.n;
    const VT* vc = static_cast<const VT*>(g.v_c) + off;
    const VT* vu = static_cast<const VT*>(g.v_u) + off;
    VT* vo = g.v_out ? static_cast<VT*>(g.v_out) + off : nullptr;
    const float* x = g.x ? g.x + off : nullptr;
    float* xo = g.x_out ? g.x_out + off : nullptr;
    bf16_t* xl = g.x_lowp ? g.x_lowp + off : nullptr;

    float s_d1 = 0.f, s_d2 = 0.f, s_u1 = 0.f, s_u2 = 0.f;
    const size_t chunk0 = (size_t)blockIdx.x * (kThreads * V * kIters);
#pragma unroll
    for (int it = 0; it < kIters; it++) {
        const size_t i = chunk0 + ((size_t)it * kThreads + threadIdx.x) * V;
        if (i < g.n) {
            float c[V], u[V], v[V];
            Vec<VT, V>::load(vc + i, c);
            Vec<VT, V>::load(vu + i, u);
#pragma unroll
            for (int j = 0; j < V; j++) {
                const float d = c[j] - u[j];
                s_d1 += fabsf(d);
                s_d2 = fmaf(d, d, s_d2);
                s_u1 += fabsf(u[j]);
                s_u2 = fmaf(u[j], u[j], s_u2);
                v[j] = fmaf(g.s, d, u[j]);
            }
            if (vo) Vec<VT, V>::store(vo + i, v);
            if (xo) {
                float xv[V];
                Vec<float, V>::load(x + i, xv);
#pragma unroll
                for (int j = 0; j < V; j++) xv[j] = fmaf(g.b, v[j], g.a * xv[j]);
                Vec<float, V>::store(xo + i, xv);
                if (xl) Vec<bf16_t, V>::store(xl + i, xv);
            }
        }
    }
    if (g.partial) {
        __shared__ double red[kThreads / HYB_WAVE][4];
        const double r0 = wave_sum((double)s_d1), r1 = wave_sum((double)s_d2);
        const double r2 = wave_sum((double)s_u1), r3 = wave_sum((double)s_u2);
        const int wave = threadIdx.x / HYB_WAVE, lane = threadIdx.x % HYB_WAVE;
        if (lane == 0) { red[wave][0] = r0; red[wave][1] = r1; red[wave][2] = r2; red[wave][3] = r3; }
        __syncthreads();
        if (threadIdx.x < 4) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < kThreads / HYB_WAVE; w++) t += red[w][threadIdx.x];
            g.partial[((size_t)sample * gridDim.x + blockIdx.x) * 4 + threadIdx.x] = t;
        }
    }
}

__device__ __forceinline__ float ratio(double num, double den) {
    if (num == 0.0) return 0.f;
    if (den == 0.0) return __builtin_inff();
    return (float)(num / den);
}

// One wave per sample: lane l adds partials l, l + 64, ... in order, then a fixed butterfly.
__global__ __launch_bounds__(HYB_WAVE) void discrepancy_finalize_kernel(const double* partial, int blocks_per_sample,
                                                                         float* d1, float* d2) {
    const size_t sample = blockIdx.x;
    const double* p = partial + sample * blocks_per_sample * 4;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < blocks_per_sample; i += HYB_WAVE)
        for (int j = 0; j < 4; j++) acc[j] += p[(size_t)i * 4 + j];
    for (int j = 0; j < 4; j++) acc[j] = wave_sum(acc[j]);
    if (threadIdx.x == 0) {
        if (d1) d1[sample] = ratio(acc[0], acc[2]);
        if (d2) d2[sample] = ratio(sqrt(acc[1]), sqrt(acc[3]));
    }
}

template <typename XT, typename VT>
__global__ __launch_bounds__(kThreads) void euler_kernel(const XT* x, const VT* v, XT* xo, size_t n, float dt) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) xo[i] = from_f32<XT>(fmaf(dt, to_f32<VT>(v[i]), to_f32<XT>(x[i])));
}

int blocks_for(size_t n, int vec) {
    const size_t chunk = (size_t)kThreads * vec * kIters;
    return (int)((n + chunk - 1) / chunk);
}

// Largest blocks-per-sample over both code paths, so the workspace query does not depend on it.
size_t partial_bytes(int batch, size_t n) { return (size_t)batch * blocks_for(n, 1) * 4 * sizeof(double); }

int launch_guidance(const char* who, GuidanceArgs g, int batch, hyb_dtype vd, float* d1, float* d2, hipStream_t st) {
    if (batch == 0 || g.n == 0) {
        // Nothing to read: an empty sample has num = den = 0, i.e. discrepancy 0.
        if (batch > 0 && (d1 || d2)) {
            hipLaunchKernelGGL(discrepancy_finalize_kernel, dim3(batch), dim3(HYB_WAVE), 0, st, (const double*)nullptr, 0, d1, d2);
            return hyb_check_launch(who);
        }
        return HYB_OK;
    }
    const bool vec = (g.n % kVec) == 0;
    const int nblk = blocks_for(g.n, vec ? kVec : 1);
    HYB_REQUIRE(batch <= 65535, HYB_ERR_SHAPE, "%s: batch %d exceeds 65535", who, batch);
    dim3 grid(nblk, batch), block(kThreads);
    // algorithmic bytes: v_c + v_u read, x read, x_out written, plus the optional outputs
    const double vs = (double)hyb_dtype_size(vd);
    const double per_elem = 2 * vs + (g.x_out ? 8 : 0) + (g.x_lowp ? 2 : 0) + (g.v_out ? vs : 0);
    {   // the pass itself; the tiny finalisation below is a launch of its own
        HybTraceScope trace("guidance_pass", "byte", per_elem * (double)batch * (double)g.n, st);
        if (vd == HYB_BF16) {
            if (vec) hipLaunchKernelGGL((guidance_kernel<bf16_t, 8>), grid, block, 0, st, g);
            else hipLaunchKernelGGL((guidance_kernel<bf16_t, 1>), grid, block, 0, st, g);
        } else {
            if (vec) hipLaunchKernelGGL((guidance_kernel<float, 8>), grid, block, 0, st, g);
            else hipLaunchKernelGGL((guidance_kernel<float, 1>), grid, block, 0, st, g);
        }
    }
    int rc = hyb_check_launch(who);
    if (rc != HYB_OK) return rc;
    if (g.partial && (d1 || d2)) {
        HybTraceScope trace("discrepancy_finalize", "byte", (double)batch * nblk * 32.0, st);
        hipLaunchKernelGGL(discrepancy_finalize_kernel, dim3(batch), dim3(HYB_WAVE), 0, st, g.partial, nblk, d1, d2);
        rc = hyb_check_launch(who);
    }
    return rc;
}

}  // namespace

extern "C" size_t hyb_discrepancy_workspace_bytes(int batch, size_t n_per_sample) {
    if (batch <= 0) return 0;
    return hyb_align_up(partial_bytes(batch, n_per_sample), 256);
}

extern "C" int hyb_cfg_combine(const void* v_c, const void* v_u, void* v_out, size_t n, float scale,
                               hyb_dtype dtype, void* stream) {
    HYB_CHECK_DTYPE(dtype);
    if (n == 0) return HYB_OK;
    HYB_CHECK_PTR(v_c); HYB_CHECK_PTR(v_u); HYB_CHECK_PTR(v_out);
    HYB_CHECK_ALIGN(v_c); HYB_CHECK_ALIGN(v_u); HYB_CHECK_ALIGN(v_out);
    GuidanceArgs g = {v_c, v_u, nullptr, nullptr, nullptr, v_out, n, scale, 1.f, 0.f, nullptr};
    // One "sample" of n elements would need n / chunk workgroups in grid.x: fine up to 2^31 - 1.
    HYB_REQUIRE(n / kThreads < 0x7fffffffu, HYB_ERR_SHAPE, "hyb_cfg_combine: n too large");
    return launch_guidance("hyb_cfg_combine", g, 1, dtype, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int hyb_branch_discrepancy(const void* v_c, const void* v_u, int batch, size_t n_per_sample,
                                      hyb_norm p, hyb_dtype dtype, float* out,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    HYB_CHECK_DTYPE(dtype);
    HYB_REQUIRE(p == HYB_NORM_L1 || p == HYB_NORM_L2, HYB_ERR_DTYPE, "hyb_branch_discrepancy: p must be HYB_NORM_L1 or HYB_NORM_L2");
    HYB_REQUIRE(batch >= 0, HYB_ERR_SHAPE, "hyb_branch_discrepancy: negative batch");
    if (batch == 0) return HYB_OK;
    HYB_CHECK_PTR(out);
    if (n_per_sample > 0) {
        HYB_CHECK_PTR(v_c); HYB_CHECK_PTR(v_u); HYB_CHECK_PTR(workspace);
        HYB_CHECK_ALIGN(v_c); HYB_CHECK_ALIGN(v_u); HYB_CHECK_ALIGN(workspace);
        HYB_REQUIRE(workspace_bytes >= hyb_discrepancy_workspace_bytes(batch, n_per_sample), HYB_ERR_WORKSPACE,
                    "hyb_branch_discrepancy: workspace of %zu bytes is smaller than the %zu required", workspace_bytes,
                    hyb_discrepancy_workspace_bytes(batch, n_per_sample));
    }
    GuidanceArgs g = {v_c, v_u, nullptr, nullptr, nullptr, nullptr, n_per_sample, 0.f, 1.f, 0.f, (double*)workspace};
    return launch_guidance("hyb_branch_discrepancy", g, batch, dtype, p == HYB_NORM_L1 ? out : nullptr,
                           p == HYB_NORM_L2 ? out : nullptr, (hipStream_t)stream);
}

extern "C" int hyb_euler_step(const void* x, const void* v, void* x_out, size_t n, float t, float t_next,
                              hyb_dtype x_dtype, hyb_dtype v_dtype, void* stream) {
    HYB_CHECK_DTYPE(x_dtype); HYB_CHECK_DTYPE(v_dtype);
    if (n == 0) return HYB_OK;
    HYB_CHECK_PTR(x); HYB_CHECK_PTR(v); HYB_CHECK_PTR(x_out);
    HYB_CHECK_ALIGN(x); HYB_CHECK_ALIGN(v); HYB_CHECK_ALIGN(x_out);
    const size_t nblk = (n + kThreads - 1) / kThreads;
    HYB_REQUIRE(nblk < 0x7fffffffu, HYB_ERR_SHAPE, "hyb_euler_step: n too large");
    const float dt = t_next - t;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)nblk), block(kThreads);
    if (x_dtype == HYB_F32 && v_dtype == HYB_F32)
        hipLaunchKernelGGL((euler_kernel<float, float>), grid, block, 0, st, (const float*)x, (const float*)v, (float*)x_out, n, dt);
    else if (x_dtype == HYB_F32)
        hipLaunchKernelGGL((euler_kernel<float, bf16_t>), grid, block, 0, st, (const float*)x, (const bf16_t*)v, (float*)x_out, n, dt);
    else if (v_dtype == HYB_F32)
        hipLaunchKernelGGL((euler_kernel<bf16_t, float>), grid, block, 0, st, (const bf16_t*)x, (const float*)v, (bf16_t*)x_out, n, dt);
    else
        hipLaunchKernelGGL((euler_kernel<bf16_t, bf16_t>), grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)v, (bf16_t*)x_out, n, dt);
    return hyb_check_launch("hyb_euler_step");
}

extern "C" int hyb_cfg_disc_affine(const void* v_c, const void* v_u, const float* x, float* x_out,
                                   void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                                   float scale, float a, float b, float* disc_l1, float* disc_l2,
                                   hyb_dtype v_dtype, void* workspace, size_t workspace_bytes, void* stream) {
    HYB_CHECK_DTYPE(v_dtype);
    HYB_REQUIRE(batch >= 0, HYB_ERR_SHAPE, "hyb_cfg_disc_affine: negative batch");
    if (batch == 0) return HYB_OK;
    const bool sums = disc_l1 || disc_l2;
    if (n_per_sample > 0) {
        HYB_CHECK_PTR(v_c); HYB_CHECK_PTR(v_u); HYB_CHECK_PTR(x); HYB_CHECK_PTR(x_out);
        HYB_CHECK_ALIGN(v_c); HYB_CHECK_ALIGN(v_u); HYB_CHECK_ALIGN(x); HYB_CHECK_ALIGN(x_out);
        HYB_CHECK_ALIGN(x_out_lowp); HYB_CHECK_ALIGN(v_out);
        if (sums) {
            HYB_CHECK_PTR(workspace); HYB_CHECK_ALIGN(workspace);
            HYB_REQUIRE(workspace_bytes >= hyb_discrepancy_workspace_bytes(batch, n_per_sample), HYB_ERR_WORKSPACE,
                        "hyb_cfg_disc_affine: workspace of %zu bytes is smaller than the %zu required", workspace_bytes,
                        hyb_discrepancy_workspace_bytes(batch, n_per_sample));
        }
    }
    GuidanceArgs g = {v_c, v_u, x, x_out, (bf16_t*)x_out_lowp, v_out, n_per_sample, scale, a, b,
                      sums ? (double*)workspace : nullptr};
    return launch_guidance("hyb_cfg_disc_affine", g, batch, v_dtype, disc_l1, disc_l2, (hipStream_t)stream);
}

extern "C" int hyb_cfg_disc_euler(const void* v_c, const void* v_u, const float* x, float* x_out,
                                  void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                                  float scale, float t, float t_next, float* disc_l1, float* disc_l2,
                                  hyb_dtype v_dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return hyb_cfg_disc_affine(v_c, v_u, x, x_out, x_out_lowp, v_out, batch, n_per_sample, scale, 1.0f,
                               t_next - t, disc_l1, disc_l2, v_dtype, workspace, workspace_bytes, stream);
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mx;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, looked up once per device

// Address of the static scratch array on the current device (nullptr + error set on failure).
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        hyb_set_error(HYB_ERR_LAUNCH, "hyb_cfg_disc_euler_noalloc: no current device (or device index >= %d)", kMaxDevices);
        return nullptr;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mx);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            hyb_set_error(HYB_ERR_LAUNCH, "hyb_cfg_disc_euler_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int hyb_cfg_disc_euler_noalloc(const void* v_c, const void* v_u, const float* x, float* x_out,
                                          void* x_out_lowp, void* v_out, int batch, size_t n_per_sample,
                                          float scale, float t, float t_next, float* disc_l1, float* disc_l2,
                                          hyb_dtype v_dtype, void* stream) {
    HYB_REQUIRE(batch >= 0, HYB_ERR_SHAPE, "hyb_cfg_disc_euler_noalloc: negative batch");
    void* ws = nullptr;
    size_t need = 0;
    if (batch > 0 && n_per_sample > 0 && (disc_l1 || disc_l2)) {
        // size check in integers first (the workspace query itself would overflow an int for absurd sizes)
        HYB_REQUIRE(n_per_sample / kThreads < (size_t)HYB_STATIC_SCRATCH_BYTES, HYB_ERR_WORKSPACE,
                    "hyb_cfg_disc_euler_noalloc: n_per_sample %zu is beyond the static scratch", n_per_sample);
        need = hyb_discrepancy_workspace_bytes(batch, n_per_sample);
        HYB_REQUIRE(need <= (size_t)HYB_STATIC_SCRATCH_BYTES, HYB_ERR_WORKSPACE,
                    "hyb_cfg_disc_euler_noalloc: batch %d x %zu elements needs %zu bytes of partial sums, the static scratch holds %d "
                    "(use hyb_cfg_disc_euler with a workspace)", batch, n_per_sample, need, HYB_STATIC_SCRATCH_BYTES);
        ws = static_scratch();
        if (!ws) return HYB_ERR_LAUNCH;
    }
    // Every partial the finalisation reads is written by this call's first kernel, so nothing has to be cleared.
    return hyb_cfg_disc_affine(v_c, v_u, x, x_out, x_out_lowp, v_out, batch, n_per_sample, scale, 1.0f, t_next - t,
                               disc_l1, disc_l2, v_dtype, ws, need, stream);
}
