// Measurement aid (not part of the hot path): the main loop of the 128 x 128 bf16 GEMM tile and nothing else.
//
// A workgroup of 4 waves (64 x 64 outputs each) runs the k loop of gemm_mfma_kernel over its tile: k-slabs of 64 copied
// global -> LDS by 16-byte direct-to-LDS buffer loads into two stages (same chunking, swizzle and waits), four k-steps per
// slab with two fragment reads per operand and a quarter of the slab's multiply-adds each, one barrier per slab; no
// bias, no epilogue (one float per thread is stored so that nothing is optimised away).  The MFMAs are either
// v_mfma_f32_16x16x32_bf16, the form the kernels use, or v_mfma_f32_32x32x16_bf16, the form they used before, on the same
// fragment reads and with the same number of multiply-adds.  1024 tiles are exactly two rounds of the
// chip's 512 workgroup slots, 512 tiles one round.  Variants leave out the copies (after the first two slabs), the fragment
// reads (operands stay in registers), or both; operands are one constant or roughly normal random bf16 (the clock that the chip's
// power management grants depends on how many bits toggle).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef void __attribute__((address_space(3)))* lptr_t;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
constexpr int BM = 128, BN = 128, BK = 64, ROWB = 128, STAGE = (BM + BN) * ROWB;
__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }
enum : int { F_NOCOPY = 1, F_NOLDS = 2, F_SMALL = 4 };
template <int FLAGS>
__global__ __launch_bounds__(256, 2) void k(const bf16_t* A, const bf16_t* W, float* out, int m, int n, int kdim, int tiles_n) {
    constexpr bool NOCOPY = FLAGS & F_NOCOPY, NOLDS = FLAGS & F_NOLDS, SMALL = FLAGS & F_SMALL;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];
    const int tid = threadIdx.x, lane = tid % 64, wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lr = lane % 32, hi = lane / 32, wt = wave % 2, wf = wave / 2;
    const int tile = blockIdx.x, row0 = (tile / tiles_n) * BM, col0 = (tile % tiles_n) * BN;
    const int nslab = kdim / BK;
    const unsigned char* a_tile = reinterpret_cast<const unsigned char*>(A + (size_t)row0 * kdim);
    const unsigned char* w_tile = reinterpret_cast<const unsigned char*>(W + (size_t)col0 * kdim);
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a_tile, 0, BM * kdim * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)w_tile, 0, BN * kdim * 2, 0x00020000);
    int voff[8];
    for (int c = 0; c < 8; c++) {
        const int r = ((wave + 4 * c) % 16) * 8 + lane / 8;     // row inside the operand tile
        voff[c] = r * kdim * 2 + (((lane % 8) ^ swz(r)) * 16);
    }
    auto issue = [&](int slab, int stage) {
        if (NOCOPY && slab > 1) return;
#pragma unroll
        for (int c = 0; c < 8; c++) {
            unsigned char* dst = smem + stage * STAGE + (wave + 4 * c) * 1024;
            if (c < 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lptr_t)dst, 16, voff[c], slab * BK * 2, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lptr_t)dst, 16, voff[c], slab * BK * 2, 0, 0);
        }
    };
    const int lb = (hi ^ lr ^ (lr >> 3)) & 7;
    int a_base[4], w_base[4];
    for (int c = 0; c < 4; c++) {
        a_base[c] = (wt * 64 + lr) * ROWB + ((lb ^ (2 * c)) * 16);
        w_base[c] = BM * ROWB + (wf * 64 + lr) * ROWB + ((lb ^ (2 * c)) * 16);
    }
    f32x16 acc[2][2];
    f32x4 acc4[4][4];
    for (int i = 0; i < 2; i++) for (int j = 0; j < 2; j++) for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
    for (int i = 0; i < 4; i++) for (int j = 0; j < 4; j++) for (int e = 0; e < 4; e++) acc4[i][j][e] = 0.f;
    bf16x8 af[4][2], wfr[4][2];
    for (int kk = 0; kk < 4; kk++) for (int t = 0; t < 2; t++) for (int e = 0; e < 8; e++) { af[kk][t][e] = (bf16_t)(0.01f * ((lane + e + kk) % 13 - 6)); wfr[kk][t][e] = (bf16_t)(0.02f * ((lane * 3 + e + t) % 11 - 5)); }
    auto read_set = [&](int stage, int kk) {
        if (NOLDS) return;
        const unsigned char* base = smem + stage * STAGE;
#pragma unroll
        for (int t = 0; t < 2; t++) af[kk][t] = *reinterpret_cast<const bf16x8*>(base + a_base[(kk ^ (2 * t)) & 3] + t * 32 * ROWB);
#pragma unroll
        for (int t = 0; t < 2; t++) wfr[kk][t] = *reinterpret_cast<const bf16x8*>(base + w_base[(kk ^ (2 * t)) & 3] + t * 32 * ROWB);
    };
    issue(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (nslab > 1) issue(1, 1);
    read_set(0, 0);
    read_set(0, 1);
    auto slab_step = [&](int s, int stg) {
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            if (kk == 2 && s + 1 < nslab) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                if (s + 2 < nslab) issue(s + 2, stg);
            }
            if (kk < 2) read_set(stg, kk + 2);
            else if (s + 1 < nslab) read_set(stg ^ 1, kk - 2);
            if (!SMALL) {
#pragma unroll
                for (int fn = 0; fn < 2; fn++)
#pragma unroll
                    for (int tm = 0; tm < 2; tm++) acc[fn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[kk][fn], af[kk][tm], acc[fn][tm], 0, 0, 0);
            } else {
                // the same four fragments as A / B operands of 16x16x32 MFMAs: 8 per k-step of 16 (same multiply-adds)
#pragma unroll
                for (int fn = 0; fn < 2; fn++)
#pragma unroll
                    for (int tm = 0; tm < 2; tm++) {
                        acc4[2 * fn][2 * tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[kk][fn], af[kk][tm], acc4[2 * fn][2 * tm], 0, 0, 0);
                        acc4[2 * fn + 1][2 * tm + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[kk][fn], af[kk][tm], acc4[2 * fn + 1][2 * tm + 1], 0, 0, 0);
                    }
            }
#pragma unroll
            for (int j = 0; j < 4; j++) { __builtin_amdgcn_sched_group_barrier(0x008, SMALL ? 2 : 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        }
    };
    for (int s = 0; s < nslab; s += 2) { slab_step(s, 0); if (s + 1 < nslab) slab_step(s + 1, 1); }
    float r = 0.f;
    for (int i = 0; i < 2; i++) for (int j = 0; j < 2; j++) for (int e = 0; e < 16; e++) r += acc[i][j][e];
    for (int i = 0; i < 4; i++) for (int j = 0; j < 4; j++) for (int e = 0; e < 4; e++) r += acc4[i][j][e];
    out[(size_t)blockIdx.x * 256 + tid] = r;
}
// One measurement: 100 launches back to back between one pair of events, after 5 untimed ones; microseconds per launch.
template <int FLAGS> float run(const bf16_t* A, const bf16_t* W, float* out, int m, int n, int kdim) {
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int tiles_n = n / BN, tiles = (m / BM) * tiles_n;
    for (int rep = 0; rep < 5; rep++) k<FLAGS><<<tiles, 256>>>(A, W, out, m, n, kdim, tiles_n);
    float ms = 0;
    const int reps = 100;
    CK(hipEventRecord(e0));
    for (int rep = 0; rep < reps; rep++) k<FLAGS><<<tiles, 256>>>(A, W, out, m, n, kdim, tiles_n);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
    return ms * 1e3f / reps;
}
int main() {
    const int MMAX = 8192, NMAX = 6144, K = 1536;
    bf16_t *A, *W; float* out;
    CK(hipMalloc(&A, (size_t)MMAX * K * 2)); CK(hipMalloc(&W, (size_t)NMAX * K * 2)); CK(hipMalloc(&out, (size_t)4096 * 256 * 4));
    unsigned short* h = (unsigned short*)malloc((size_t)MMAX * K * 2);
    printf("| operands | variant | m x n x k | tiles | us per launch (median of 3 x 100 back to back) | TFLOP/s |\n|---|---|---|---|---|---|\n");
    for (int random = 0; random < 2; random++) {
        unsigned st = 777u;
        for (size_t i = 0; i < (size_t)MMAX * K; i++) { float acc = 0; for (int r = 0; r < 4; r++) { st = st * 1664525u + 1013904223u; acc += (st >> 8) * (1.0f / 16777216.0f); } float x = random ? (acc - 2.0f) * 1.7f : 0.0625f; unsigned u; memcpy(&u, &x, 4); h[i] = (unsigned short)(u >> 16); }
        CK(hipMemcpy(A, h, (size_t)MMAX * K * 2, hipMemcpyHostToDevice));
        CK(hipMemcpy(W, h, (size_t)NMAX * K * 2, hipMemcpyHostToDevice));
        const char* d = random ? "random" : "constant";
        // 1024 tiles = exactly two rounds of 512 slots; 512 tiles = one round
        // The variants are measured in turn, three times over (the clock the chip grants drifts over milliseconds, so a
        // variant must not always follow the same neighbour); the median of the three is printed.
        const char* names[8] = {"main loop, 16x16x32 MFMAs", "main loop, 16x16x32 MFMAs, one round", "... without the copies", "... without the fragment reads",
                                "... MFMAs only", "main loop, 32x32x16 MFMAs", "... without the copies", "... MFMAs only"};
        const int ms_[8] = {4096, 2048, 4096, 4096, 4096, 4096, 4096, 4096};
        float us[8][3];
        for (int pass = 0; pass < 3; pass++) {
            us[0][pass] = run<F_SMALL>(A, W, out, 4096, 4096, K);
            us[5][pass] = run<0>(A, W, out, 4096, 4096, K);
            us[1][pass] = run<F_SMALL>(A, W, out, 2048, 4096, K);
            us[2][pass] = run<F_SMALL | F_NOCOPY>(A, W, out, 4096, 4096, K);
            us[6][pass] = run<F_NOCOPY>(A, W, out, 4096, 4096, K);
            us[3][pass] = run<F_SMALL | F_NOLDS>(A, W, out, 4096, 4096, K);
            us[4][pass] = run<F_SMALL | F_NOCOPY | F_NOLDS>(A, W, out, 4096, 4096, K);
            us[7][pass] = run<F_NOCOPY | F_NOLDS>(A, W, out, 4096, 4096, K);
        }
        for (int v = 0; v < 8; v++) {
            float a = us[v][0], b = us[v][1], c = us[v][2];
            const float med = a > b ? (b > c ? b : (a > c ? c : a)) : (a > c ? a : (b > c ? c : b));
            printf("| %s | %s | %d x 4096 x %d | %d | %.1f | %.0f |\n", d, names[v], ms_[v], K, ms_[v] / BM * (4096 / BN), med, 2.0 * ms_[v] * 4096.0 * K / (med * 1e-6) * 1e-12);
        }
    }
    CK(hipDeviceSynchronize());
    return 0;
}
