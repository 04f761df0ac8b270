// Measurement aid (not part of the hot path): what does one 64-key tile of the bf16 attention kernel cost on this
// chip when nothing but its instruction stream is left?
//
// Every wave repeats, n times, the work a wave of the attention kernel does per key tile: 8 MFMAs
// (v_mfma_f32_32x32x16_bf16) for S^T = K Q^T in two accumulation chains, 32 exp2 of their results, 16 conversions to
// pairs of bf16, 8 MFMAs for O^T += V^T P^T with the converted values as B operand, and 16 dot products for the row
// sums.  Variants add the parts of the real kernel one by one: the K / V^T fragments read from LDS with the kernel's
// addresses and swizzles, the phases held in program order, workgroups of 4 waves with a barrier per tile, the tile
// copies global -> LDS.  Operands are either constants or roughly normal random bf16 values: the clock that the chip's
// power management grants under MFMA load depends on how many bits toggle.
// Two more rows give the yardstick: a loop of nothing but independent MFMAs on register operands, for the 32x32x16 and the
// 16x16x32 form (the same flop count per row: 16 and 32 MFMAs per step).
// Prints a table of SIMD time per wave and tile and the MFMA rate of the whole chip.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef void __attribute__((address_space(3)))* lptr_t;

#define CK(x)                                                                             \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);         \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

constexpr int TILE = 8192;                 // bytes of a K or V tile: 64 keys x 128 bytes
constexpr int TILES = 70;                  // tiles per (batch, head) pair in the copy variant
constexpr int PAIRS = 64;                  // pairs in the global buffer (each 2 x 70 x 8 KB)

__device__ __forceinline__ int swz_v(int r) { return ((r >> 1) & 1) * 4; }

enum : int { F_LDS = 1, F_ORDER = 2, F_BARRIER = 4, F_COPY = 8, F_NO_EXP = 16, F_SMALL = 32, F_PRIO = 64 };

// flags: see the enum; blockDim = 256 (F_BARRIER: one workgroup of 4 waves, several per CU) or 256 x waves per SIMD
template <int FLAGS>
__global__ __launch_bounds__(1024) void tile_kernel(float* out, int n, const unsigned char* kv, int random_regs) {
    constexpr bool LDS = FLAGS & F_LDS, ORDER = FLAGS & F_ORDER, BAR = FLAGS & F_BARRIER, COPY = FLAGS & F_COPY, NO_EXP = FLAGS & F_NO_EXP;
    constexpr bool PRIO = (FLAGS & F_PRIO) && (FLAGS & F_SMALL) && (FLAGS & F_LDS);   // the kernel's wave priorities (with its
                                                 // order of requests: the second half of the V^T fragments after the softmax)
    constexpr bool SMALL = FLAGS & F_SMALL;      // the same fragments multiplied by twice as many v_mfma_f32_16x16x32_bf16 (same multiply-adds)
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * TILE];      // two buffers of a K and a V tile
    for (int i = threadIdx.x; i < 4 * TILE / 4; i += blockDim.x) reinterpret_cast<unsigned*>(smem)[i] = reinterpret_cast<const unsigned*>(kv)[i];
    __syncthreads();
    const int lane = threadIdx.x % 64, lq = lane % 32, g = lane / 32, sl = lane % 16;
    const int wave = __builtin_amdgcn_readfirstlane((threadIdx.x / 64) % 4);
    // fragment addresses as in the attention kernel: K rows read one per lane with XOR-swizzled 16-byte slots, V^T by
    // transposing reads
    const unsigned char* kbase[4];
    unsigned vbase[2];
    {
        const int kb = (g ^ lq ^ (lq >> 3)) & 7;
        for (int j = 0; j < 4; j++) kbase[j] = smem + lq * 128 + ((kb ^ (2 * j)) * 16);
        const int v_key = 4 * g + sl / 4, v_feat = 16 * ((lane / 16) % 2) + 4 * (sl % 4);
        for (int dt = 0; dt < 2; dt++)
            vbase[dt] = (unsigned)(size_t)(lptr_t)smem + TILE + v_key * 128 + (((4 * dt + v_feat / 8) ^ swz_v(v_key)) * 16) + (v_feat % 8) * 2;
    }
    const unsigned char* kp = kv + (size_t)(blockIdx.x % PAIRS) * (2 * TILES * TILE);
    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kp, 0, TILES * TILE, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(kp + TILES * TILE), 0, TILES * TILE, 0x00020000);
    int coff[2];
    for (int c = 0; c < 2; c++) coff[c] = ((wave + 4 * c) * 8 + lane / 8) * 128 + (lane % 8) * 16;

    bf16x8 a[4], q[4];      // register operands: a stands in for the K / V^T fragments when they do not come from LDS
    for (int j = 0; j < 4; j++)
        for (int i = 0; i < 8; i++) {
            unsigned h = (threadIdx.x * 2654435761u) ^ ((unsigned)(i * 40503u + j * 9973u) * 2246822519u);
            h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
            a[j][i] = random_regs ? (bf16_t)(((int)(h & 0xffff) - 32768) * (1.7f / 32768.0f)) : (bf16_t)0.0625f;
            q[j][i] = random_regs ? (bf16_t)(0.05f * (float)((int)((h >> 16) % 17) - 8)) : (bf16_t)0.125f;
        }
    f32x16 o[2];
    for (int d = 0; d < 2; d++)
        for (int i = 0; i < 16; i++) o[d][i] = 0.f;
    f32x4 o4[SMALL ? 8 : 1];
    if constexpr (SMALL)
        for (int d = 0; d < 8; d++)
            for (int i = 0; i < 4; i++) o4[d][i] = 0.f;
    float l = 0.f;
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};

    for (int it = 0; it < n; it++) {
        const int boff = (it & 1) * 2 * TILE;
        if (BAR) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
        }
        if (COPY) {      // this wave's share of the next tile pair, into the other buffer
            const int t = (it + 1) % TILES;
#pragma unroll
            for (int c = 0; c < 2; c++) {
                unsigned char* dst = smem + (2 * TILE - boff) + (wave + 4 * c) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)dst, 16, coff[c], t * TILE, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(dst + TILE), 16, coff[c], t * TILE, 0, 0);
            }
        }
        f32x16 s[2];
        for (int i = 0; i < 16; i++) s[0][i] = s[1][i] = 0.f;
        f32x4 s4[SMALL ? 8 : 1];
        if constexpr (SMALL)
            for (int d = 0; d < 8; d++)
                for (int i = 0; i < 4; i++) s4[d][i] = 0.f;
        if constexpr (PRIO) __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            bf16x8 kf = a[j & 3];
            if (LDS) {
                const int kt = j & 1, kk = j >> 1;
                kf = *reinterpret_cast<const bf16x8*>(kbase[(kk ^ (2 * kt)) & 3] + boff + kt * 32 * 128);
            }
            if constexpr (SMALL) {
                s4[j & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, q[j >> 1], s4[j & 3], 0, 0, 0);
                s4[4 + (j & 3)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, q[(j >> 1) ^ 1], s4[4 + (j & 3)], 0, 0, 0);
            } else s[j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, q[j >> 1], s[j & 1], 0, 0, 0);
        }
        if (ORDER) __builtin_amdgcn_sched_barrier(0);
        bf16x4 vh[2][2][2][2];
        auto v_request = [&](int d) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    const int off = (kt * 32 + hf * 16) * 128;
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[d][kt][hf][0]) : "v"(vbase[d] + boff), "i"(off));
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[d][kt][hf][1]) : "v"(vbase[d] + boff), "i"(off + 8 * 128));
                }
        };
        if (LDS) {
            v_request(0);
            if constexpr (!PRIO) v_request(1);
        }
        bf16x8 pb[2][2];
        if constexpr (PRIO) {
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int d = 0; d < 8; d++)
#pragma unroll
                for (int i = 0; i < 4; i++) s4[d][i] = __builtin_amdgcn_exp2f(s4[d][i]);
            // (the exponentials are taken before the priority goes up again)
            asm volatile("" : "+v"(s4[0]), "+v"(s4[1]), "+v"(s4[2]), "+v"(s4[3]), "+v"(s4[4]), "+v"(s4[5]), "+v"(s4[6]), "+v"(s4[7]));
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) pb[kt][i / 8][i % 8] = (bf16_t)s4[4 * kt + i / 4][i % 4];
            asm volatile("" : "+v"(pb[0][0]), "+v"(pb[0][1]), "+v"(pb[1][0]), "+v"(pb[1][1]));
            v_request(1);
        } else {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    float sc;
                    if constexpr (SMALL) sc = s4[4 * kt + i / 4][i % 4];
                    else sc = s[kt][i];
                    pb[kt][i / 8][i % 8] = NO_EXP ? (bf16_t)sc : (bf16_t)__builtin_amdgcn_exp2f(sc);
                }
        }
        if (ORDER) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < 2; d++)
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    bf16x8 vf = a[(kt * 2 + hf + d) & 3];
                    if (LDS) {
                        if (d == 0 && kt == 0 && hf == 0)
                            asm volatile("s_waitcnt lgkmcnt(0)"
                                         : "+v"(vh[0][0][0][0]), "+v"(vh[0][0][0][1]), "+v"(vh[0][0][1][0]), "+v"(vh[0][0][1][1]),
                                           "+v"(vh[0][1][0][0]), "+v"(vh[0][1][0][1]), "+v"(vh[0][1][1][0]), "+v"(vh[0][1][1][1]),
                                           "+v"(vh[1][0][0][0]), "+v"(vh[1][0][0][1]), "+v"(vh[1][0][1][0]), "+v"(vh[1][0][1][1]),
                                           "+v"(vh[1][1][0][0]), "+v"(vh[1][1][0][1]), "+v"(vh[1][1][1][0]), "+v"(vh[1][1][1][1]));
                        const bf16x4 lo = vh[d][kt][hf][0], hi = vh[d][kt][hf][1];
                        vf = bf16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    }
                    if constexpr (SMALL) {
                        o4[4 * d + 2 * kt + hf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[kt][hf], o4[4 * d + 2 * kt + hf], 0, 0, 0);
                        o4[4 * (d ^ 1) + 2 * kt + hf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[kt ^ 1][hf], o4[4 * (d ^ 1) + 2 * kt + hf], 0, 0, 0);
                    } else o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kt][hf], o[d], 0, 0, 0);
                }
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int hf = 0; hf < 2; hf++)
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const bf16x2 pr = {pb[kt][hf][j], pb[kt][hf][j + 1]};
                    l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l, false);
                }
        if ((it & 63) == 63)      // keep the accumulators bounded
            for (int d = 0; d < 2; d++)
                for (int i = 0; i < 16; i++) {
                    if constexpr (SMALL) o4[4 * d + i / 4][i % 4] *= 0.001f;
                    else o[d][i] *= 0.001f;
                }
    }
    float r = l;
    for (int d = 0; d < 2; d++)
        for (int i = 0; i < 16; i++) {
            if constexpr (SMALL) r += o4[4 * d + i / 4][i % 4];
            else r += o[d][i];
        }
    out[((size_t)blockIdx.x * 1024 + threadIdx.x) % (256 * 1024)] = r;
}

// Nothing but MFMAs: 4 (32x32x16) or 8 (16x16x32) independent accumulators, operands in registers.
template <int WIDE>
__global__ __launch_bounds__(1024) void bare_kernel(float* out, int n, int random_regs) {
    bf16x8 a[4], b[4];
    for (int j = 0; j < 4; j++)
        for (int i = 0; i < 8; i++) {
            unsigned h = (threadIdx.x * 2654435761u) ^ ((unsigned)(i * 40503u + j * 9973u) * 2246822519u);
            h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
            a[j][i] = random_regs ? (bf16_t)(((int)(h & 0xffff) - 32768) * (1.7f / 32768.0f)) : (bf16_t)0.0625f;
            b[j][i] = random_regs ? (bf16_t)(((int)(h >> 16) - 32768) * (1.7f / 32768.0f)) : (bf16_t)0.125f;
        }
    float r = 0.f;
    if (WIDE) {
        f32x16 acc[4];
        for (int c = 0; c < 4; c++)
            for (int i = 0; i < 16; i++) acc[c][i] = 0.f;
        for (int it = 0; it < n; it++) {
#pragma unroll
            for (int j = 0; j < 16; j++) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 3], b[(j >> 2) & 3], acc[j & 3], 0, 0, 0);
            if ((it & 63) == 63)
                for (int c = 0; c < 4; c++)
                    for (int i = 0; i < 16; i++) acc[c][i] *= 0.001f;
        }
        for (int c = 0; c < 4; c++)
            for (int i = 0; i < 16; i++) r += acc[c][i];
    } else {
        f32x4 acc[8];
        for (int c = 0; c < 8; c++)
            for (int i = 0; i < 4; i++) acc[c][i] = 0.f;
        for (int it = 0; it < n; it++) {
#pragma unroll
            for (int j = 0; j < 32; j++) acc[j & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j & 3], b[(j >> 3) & 3], acc[j & 7], 0, 0, 0);
            if ((it & 63) == 63)
                for (int c = 0; c < 8; c++)
                    for (int i = 0; i < 4; i++) acc[c][i] *= 0.001f;
        }
        for (int c = 0; c < 8; c++)
            for (int i = 0; i < 4; i++) r += acc[c][i];
    }
    out[((size_t)blockIdx.x * 1024 + threadIdx.x) % (256 * 1024)] = r;
}

template <int WIDE>
float run_bare(float* out, int n, int random_regs, int waves_per_simd, int cus) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms = 0.f;
    for (int rep = 0; rep < 3; rep++) {
        CK(hipEventRecord(e0));
        bare_kernel<WIDE><<<cus, 256 * waves_per_simd>>>(out, n, random_regs);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms;
}

template <int FLAGS>
float run(float* out, int n, const unsigned char* kv, int random_regs, int waves_per_simd, int cus) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms = 0.f;
    for (int rep = 0; rep < 3; rep++) {      // the last of three launches counts
        CK(hipEventRecord(e0));
        if (FLAGS & F_BARRIER) tile_kernel<FLAGS><<<cus * waves_per_simd, 256>>>(out, n, kv, random_regs);
        else tile_kernel<FLAGS><<<cus, 256 * waves_per_simd>>>(out, n, kv, random_regs);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms;
}

int main() {
    int dev = 0, cus = 0;
    CK(hipGetDevice(&dev));
    CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int n = 2000;
    const size_t nb = (size_t)PAIRS * 2 * TILES * TILE;
    float* out;
    unsigned char* kv;
    CK(hipMalloc(&out, (size_t)256 * 1024 * sizeof(float)));
    CK(hipMalloc(&kv, nb));
    unsigned short* host = (unsigned short*)malloc(nb);
    printf("| operands | variant | waves per SIMD | ms | ns of SIMD time per wave and tile | MFMA rate of the chip, TFLOP/s |\n|---|---|---|---|---|---|\n");
    for (int random = 0; random < 2; random++) {
        unsigned st = 12345u;
        for (size_t i = 0; i < nb / 2; i++) {      // bf16 of roughly normal values (sum of 4 uniforms, centred), or one constant
            float acc = 0.f;
            for (int r = 0; r < 4; r++) {
                st = st * 1664525u + 1013904223u;
                acc += (st >> 8) * (1.0f / 16777216.0f);
            }
            const float x = random ? (acc - 2.0f) * 1.7f : 0.0625f;
            unsigned u;
            memcpy(&u, &x, 4);
            host[i] = (unsigned short)(u >> 16);
        }
        CK(hipMemcpy(kv, host, nb, hipMemcpyHostToDevice));
        const char* data = random ? "random" : "constant";
        auto row = [&](const char* name, int w, float ms) {
            const double simds = 4.0 * cus;
            printf("| %s | %s | %d | %.3f | %.1f | %.0f |\n", data, name, w, ms, ms * 1e6 / ((double)n * w),
                   16.0 * 32768.0 * simds * n * w / (ms * 1e-3) * 1e-12);
        };
        for (int w = 2; w <= 4; w += 2) {
            row("independent MFMAs 32x32x16 only", w, run_bare<1>(out, n, random, w, cus));
            row("independent MFMAs 16x16x32 only (32 per step)", w, run_bare<0>(out, n, random, w, cus));
            row("the tile's MFMAs and conversions, operands in registers", w, run<F_NO_EXP>(out, n, kv, random, w, cus));
            row("the tile's MFMAs and conversions, fragments from LDS", w, run<F_NO_EXP | F_LDS>(out, n, kv, random, w, cus));
            row("whole tile, operands in registers", w, run<0>(out, n, kv, random, w, cus));
            row("whole tile, fragments from LDS", w, run<F_LDS>(out, n, kv, random, w, cus));
            row("... phases in program order", w, run<F_LDS | F_ORDER>(out, n, kv, random, w, cus));
            row("... 4-wave workgroups, barrier per tile", w, run<F_LDS | F_ORDER | F_BARRIER>(out, n, kv, random, w, cus));
            row("... tile copies global -> LDS", w, run<F_LDS | F_ORDER | F_BARRIER | F_COPY>(out, n, kv, random, w, cus));
        }
    }
    // the complete tile with either MFMA form, random operands (still resident), 4 waves per SIMD: measured in turn, three
    // times over, since the granted clock drifts over milliseconds; median
    {
        float ms[4][3];
        for (int pass = 0; pass < 3; pass++) {
            ms[0][pass] = run<F_LDS | F_ORDER | F_BARRIER | F_COPY>(out, n, kv, 1, 4, cus);
            ms[1][pass] = run<F_LDS | F_ORDER | F_BARRIER | F_COPY | F_SMALL>(out, n, kv, 1, 4, cus);
            ms[2][pass] = run<F_LDS | F_BARRIER | F_COPY | F_SMALL>(out, n, kv, 1, 4, cus);
            ms[3][pass] = run<F_LDS | F_BARRIER | F_COPY | F_SMALL | F_PRIO>(out, n, kv, 1, 4, cus);
        }
        const char* names[4] = {"complete tile, 32x32x16 MFMAs (median of 3, in turn)", "complete tile, 16x16x32 MFMAs (median of 3, in turn)",
                                "complete tile, 16x16x32 MFMAs, phases not held in order", "... wave priority low during the exponentials only"};
        for (int v = 0; v < 4; v++) {
            const float a = ms[v][0], b = ms[v][1], c = ms[v][2];
            const float med = a > b ? (b > c ? b : (a > c ? c : a)) : (a > c ? a : (b > c ? c : b));
            printf("| random | %s | 4 | %.3f | %.1f | %.0f |\n", names[v], med, med * 1e6 / ((double)n * 4), 16.0 * 32768.0 * 4.0 * cus * n * 4 / (med * 1e-3) * 1e-12);
        }
    }
    CK(hipDeviceSynchronize());
    free(host);
    CK(hipFree(kv));
    CK(hipFree(out));
    return 0;
}
