// bf16 MFMA GEMM for gfx950: out = epilogue(A W^T + bias), A [m, k] tokens x features-in,
// W [n, k] features-out x features-in, fp32 accumulation in v_mfma_f32_16x16x32_bf16.
//
// Tiling: a workgroup of 4 waves (2 x 2) owns a 128 x 128 output tile; each wave owns 4 x 4 MFMA
// tiles of 16 x 16 (small problems: 64 x 128 tiles, 4 x 2 MFMA tiles per wave, see launch_epi).
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand, so the 4
// accumulator registers of a tile run along the output-feature axis (4 consecutive features, one
// token per lane).  The 16 x 16 x 32 form is used because it is the cheaper one on this chip: it
// moves half the accumulator bytes per multiply-add of the 32 x 32 x 16 form, and under the power
// limit that sets the clock of these kernels the main loop runs 5-6 % faster with it (QKV-shaped and
// fc1 launches of the SD3-shaped workload); the sums come out bit for bit the same as with the
// 32 x 32 x 16 form that the large-tile kernel uses (the tests compare the two kernels' outputs).
//
// Main loop: k is cut into slabs of 64.  A slab of both operands (128 + 128 rows of 128 bytes) is
// copied global -> LDS by 16-byte direct-to-LDS buffer loads (buffer_load_dwordx4 ... lds: a wave fills 1 KB
// of LDS per instruction, no VGPR staging, no ds_write; the slab's byte offset is the scalar operand and the
// per-lane offsets are loop invariants, so a slab costs no vector address arithmetic), double buffered: the copy
// of slab s + 1 runs while slab s is multiplied.  LDS rows are unpadded; the 16-byte slots of a row are XOR-swizzled
// with (row ^ row >> 3) & 7 so that the 16-byte fragment reads that are served together hit distinct
// banks (the swizzle is applied on the global side: each lane picks which 16 bytes it fetches).
// Waits on the copies are explicit (s_waitcnt vmcnt + s_barrier); a full __syncthreads() would
// force vmcnt(0) on every barrier through its fence.  The fragments of the two k-steps (of 32) of a
// slab live in two register sets and are read one k-step ahead of the MFMAs that use them, also
// across the slab boundary, which leaves a single barrier per slab (before its second k-step).
//
// Epilogue: the accumulators (+ bias, activation, gate) are staged through LDS (reusing the slab
// buffers) and written out row-contiguously, 16 bytes per lane, so that global stores and the
// residual reads are whole 128-byte lines.  (Storing straight from the MFMA layout issues 8-byte
// pieces to 32 different rows per instruction; at these sizes that made the epilogue cost a third
// of the tile time.)  What the epilogue reads from global memory is requested where the latency is
// hidden: the tile's bias and gate values at the start of the tile (parked in LDS behind the slab
// buffers), the residual during the last k-slab; every such access uses clamped addresses instead
// of predicates, and the staging loops are free of branches.  (With a branch that chooses between
// a global and an LDS source inside the loop, the compiler waits for ALL outstanding global loads
// before every LDS read.)
//
// Up to two problems with the same (n, k) share a launch (image and text stream of a joint
// block), the smaller one first.  Tile order: plain, or one run of consecutive tiles per XCD when
// there are few tile columns (see the kernel).  Ragged edges: row / feature indices are clamped on load and masked on store.  The
// reduction order over k is fixed and a token's result does not depend on its tile row, so
// results are deterministic and batch-invariant.
#include "gemm.h"

#include <type_traits>

namespace {

constexpr int BN = 128, BK = 64;
constexpr int ROWB = BK * 2;                    // bytes per LDS row of a slab
// The tile height is 64 TMW tokens (TMW = MFMA token tiles per wave): 128 for the large GEMMs, 64 for
// launches that would otherwise leave most of the chip idle (fewer than three quarters of a wave of tiles).
template <int TMW> struct Geo {
    static constexpr int BM = 64 * TMW;
    static constexpr int STAGE_BYTES = (BM + BN) * ROWB;   // 32 KB / 24 KB
    static constexpr int CPW = STAGE_BYTES / 1024 / 4;     // 1 KB chunks per wave per slab (8 / 6)
    static constexpr int SMEM_BYTES = 2 * STAGE_BYTES;     // 64 KB -> two workgroups per CU / 48 KB -> three
};
constexpr int VEC_BYTES = 2 * BN * 4;           // the tile's bias and gate values, behind the slab buffers
constexpr int OUT_STRIDE_B16 = BN * 2 + 16;     // staging row strides (bytes), padded against conflicts
constexpr int OUT_STRIDE_F32 = BN * 4 + 16;

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }

// 16 bytes per lane from a raw buffer (base address, size in bytes) straight into LDS: lane i's bytes land at
// lds + 16 i; the address is base + voffset (per lane) + soffset (scalar).  Not a template: the descriptor type
// only exists in the device pass.
__device__ __forceinline__ void buffer_load_lds16(const void* base, unsigned bytes, void* lds, int voffset, int soffset) {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lptr_t)lds, 16, voffset, soffset, 0, 0);
}

template <typename OT, int EPI, int TMW>
__global__ __launch_bounds__(256, TMW == 2 ? 2 : 3) void gemm_mfma_kernel(GemmGroup g, int tiles_n, int tiles0, int total, int xcd_run, int ksplit) {
    constexpr int BM = Geo<TMW>::BM, STAGE_BYTES = Geo<TMW>::STAGE_BYTES, CPW = Geo<TMW>::CPW;
    __shared__ __attribute__((aligned(16))) unsigned char smem[Geo<TMW>::SMEM_BYTES + VEC_BYTES];

    // Workgroups go round-robin to the 8 XCDs (each with its own L2) in launch order.  With few tile columns the
    // tiles that an XCD works on at a time then share hardly any operand panel (every 8th tile: all tile rows, a
    // few columns), so XCD x is given the run of consecutive tiles [x * xcd_run, (x + 1) * xcd_run) instead
    // (a few whole tile rows).  xcd_run == 0: plain order.
    int tile = blockIdx.x;
    if (xcd_run > 0) {
        tile = (tile % 8) * xcd_run + tile / 8;
        if (tile >= total) return;
    }
    // k split (ksplit > 1, single problem, plain fp32 output): ksplit consecutive workgroups share a tile; each
    // multiplies its share of the k-slabs and writes the raw sums to its own [m, n] plane of p.out
    int split = 0;
    if (ksplit > 1) {
        split = tile % ksplit;
        tile /= ksplit;
    }
    const int pi = tile >= tiles0 ? 1 : 0;
    if (pi) tile -= tiles0;
    const GemmProblem& p = g.p[pi];
    const int row0 = (tile / tiles_n) * BM;
    // EPI_GEGLU: a tile covers 64 output features; its 128 weight rows are 64 "u" rows and the 64 "gate" rows n above
    const int col0 = (tile % tiles_n) * (EPI == EPI_GEGLU ? BN / 2 : BN);
    const int m = p.m, n = g.n, k = g.k;
    const bf16_t* A = static_cast<const bf16_t*>(p.a);
    const bf16_t* W = static_cast<const bf16_t*>(p.w);

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);   // uniform: LDS copy targets (M0) become scalar arithmetic
    const int wt = wave % 2, wf = wave / 2;          // wave position: tokens, features
    const int l16 = lane % 16, q4 = lane / 16;      // MFMA 16x16x32: row / column of the lane, its quarter of the 32 k

    // This wave's chunks of a slab: chunk c covers stage rows 8 c .. 8 c + 7 (rows 0..BM-1 = A, then 128 rows of W);
    // lane i fills 16-byte slot i % 8 of row i / 8 and fetches k-vector (slot ^ swz(row)) for it.
    // Buffer loads: a tile's A rows and W rows are two buffers that start at the tile's first row (so per-lane
    // byte offsets are small 32-bit numbers, loop invariants), the k-slab's offset is a scalar operand: a slab costs
    // no vector address arithmetic.  Rows past the end are clamped to the last row (their products are not stored).
    const int slab0 = split * (k / BK) / ksplit;
    const int nslab = (split + 1) * (k / BK) / ksplit - slab0;
    const size_t row_bytes = (size_t)k * 2;
    const bf16_t* a_tile = A + (size_t)row0 * k;
    const unsigned a_tile_bytes = (unsigned)(min(BM, m - row0) * row_bytes);
    const int w_rows = min(EPI == EPI_GEGLU ? BN / 2 : BN, n - col0);
    const bf16_t* w_tile = W + (size_t)col0 * k;
    const unsigned w_tile_bytes = (unsigned)((EPI == EPI_GEGLU ? (size_t)n + w_rows : (size_t)w_rows) * row_bytes);
    int voff[CPW];
#pragma unroll
    for (int c = 0; c < CPW; c++) {
        const int r = (wave + 4 * c) * 8 + lane / 8;
        const int kv = (lane % 8) ^ swz(r);
        if (r < BM) voff[c] = (min(row0 + r, m - 1) - row0) * (int)row_bytes + kv * 16;
        else if constexpr (EPI == EPI_GEGLU) {
            const int vr = r - BM;
            voff[c] = (vr < 64 ? min(col0 + vr, n - 1) - col0 : n + min(col0 + vr - 64, n - 1) - col0) * (int)row_bytes + kv * 16;
        } else voff[c] = (min(col0 + r - BM, n - 1) - col0) * (int)row_bytes + kv * 16;
    }
    auto issue = [&](int slab, int stage) {
        const int soff = (slab0 + slab) * (BK * 2);
#pragma unroll
        for (int c = 0; c < CPW; c++) {
            // chunks of A come first: chunk index wave + 4 c < BM / 8 exactly for c < BM / 32
            if (c < BM / 32) buffer_load_lds16(a_tile, a_tile_bytes, smem + stage * STAGE_BYTES + (wave + 4 * c) * 1024, voff[c], soff);
            else buffer_load_lds16(w_tile, w_tile_bytes, smem + stage * STAGE_BYTES + (wave + 4 * c) * 1024, voff[c], soff);
        }
    };

    constexpr int TT = 2 * TMW;   // token tiles of 16 per wave
    f32x4 acc[4][TT];             // [feature tile of 16][token tile of 16]
#pragma unroll
    for (int fi = 0; fi < 4; fi++)
#pragma unroll
        for (int ti = 0; ti < TT; ti++)
#pragma unroll
            for (int i = 0; i < 4; i++) acc[fi][ti][i] = 0.f;

    // Fragment addresses inside a stage.  A fragment of v_mfma_f32_16x16x32_bf16 is 16 rows x 32 k, lane (l16, q4)
    // holding 8 k of row l16.  Which 8 is free as long as both operands agree (the order of the contraction index
    // inside an MFMA does not matter to the product): lane quarter q4 takes the 16-byte slot 4 ks + (q4 >> 1 | (q4 & 1) << 1)
    // of its row, so that lanes i and i + 32 read adjacent slots of one row, 32 contiguous bytes.  (With slot 4 ks + q4
    // the same reads take twice as long: the LDS counters show four conflict cycles per read, whatever the swizzle.)
    // With the XOR swizzle and tile rows 16 t + l16 the slot sits at (lane part) ^ (4 ks ^ 2 t): four per-lane bases per
    // operand cover all the reads of a slab, and the tile row block (t * 16 rows) is an immediate offset.  (With 32
    // token rows per wave the wave's own row offset 32 wt also reaches bit 2 of the swizzle; it is folded into the lane part.)
    const int kq = (q4 >> 1) | ((q4 & 1) << 1);
    const int lb = (kq ^ (l16 & 7) ^ (l16 >> 3)) & 7;
    const int lb_a = TMW == 1 ? lb ^ (4 * wt) : lb;
    int a_base[4], w_base[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
        a_base[c] = (wt * 32 * TMW + l16) * ROWB + ((lb_a ^ (2 * c)) * 16);
        w_base[c] = BM * ROWB + (wf * 64 + l16) * ROWB + ((lb ^ (2 * c)) * 16);
    }
    // Two fragment sets, one per k-step of 32 of a slab; the reads run one k-step ahead of their use, across the slab
    // boundary.
    bf16x8 af[2][TT], wfr[2][4];
    auto read_set = [&](int stage, int ks) {
        const unsigned char* base = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int t = 0; t < TT; t++)
            af[ks][t] = *reinterpret_cast<const bf16x8*>(base + a_base[((2 * ks) ^ t) & 3] + t * 16 * ROWB);
#pragma unroll
        for (int t = 0; t < 4; t++)
            wfr[ks][t] = *reinterpret_cast<const bf16x8*>(base + w_base[((2 * ks) ^ t) & 3] + t * 16 * ROWB);
    };

    // Main loop.  Slab s sits in stage s % 2.  ONE barrier per slab, before its second k-step: by then every wave has
    // issued (and, after the lgkmcnt wait, completed) all its reads of slab s, so stage s % 2 can be refilled with
    // slab s + 2 right behind the barrier, and the copy of slab s + 1 (issued one slab earlier) is awaited just
    // before it, so that the second k-step can already fetch the first fragments of slab s + 1.
    // Epilogue operands are fetched where their latency is hidden.  Bias and gate of the tile's 128 columns:
    // one value per thread now, parked in LDS behind the slab buffers once the first slab's wait has passed.
    // (The gate row must be the same for all rows of the tile; tiles that straddle samples read it from
    // global memory in the epilogue.)
    float* vec_lds = reinterpret_cast<float*>(smem + Geo<TMW>::SMEM_BYTES);
    bool gate_in_lds = true;   // no gate: ones
    if constexpr (EPI == EPI_GATE_RES) {
        if (p.gate) gate_in_lds = row0 / p.rows_per_gate == min(row0 + BM - 1, m - 1) / p.rows_per_gate;
    }
    {
        const int t = tid % BN;
        int f = min(col0 + t, n - 1);
        if constexpr (EPI == EPI_GEGLU) f = t < 64 ? min(col0 + t, n - 1) : n + min(col0 + t - 64, n - 1);
        float val = 0.f;
        if (tid < BN) {
            if (p.bias) val = p.bias[f];
        } else if constexpr (EPI == EPI_GATE_RES) {
            val = 1.f;
            if (p.gate && gate_in_lds) val = p.gate[(size_t)(row0 / p.rows_per_gate) * p.gate_stride + f];
        }
        issue(0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        vec_lds[tid] = val;
    }
    __builtin_amdgcn_s_barrier();
    if (nslab > 1) issue(1, 1);
    read_set(0, 0);
    constexpr bool GEGLU = EPI == EPI_GEGLU;
    [[maybe_unused]] const int q_cols = EPI == EPI_QKV && p.q_scale != 0.f ? p.heads * 64 : 0;   // columns of the q part that are scaled
    [[maybe_unused]] const float q_scale = p.q_scale;
    // EPI_QKV: where the tile's first column and row lie (feature = (which, offset in q / k / v), row = (sample, token))
    [[maybe_unused]] int qkv_which0 = 0, qkv_cc0 = 0, qkv_b0 = 0, qkv_t0 = 0;
    [[maybe_unused]] bool qkv_steps = false;   // chunks reach their place by at most one step over each boundary
    if constexpr (EPI == EPI_QKV) {
        const int hd = p.heads * 64;
        qkv_steps = hd >= BN && p.tokens >= BM;
        if (qkv_steps) {
            qkv_which0 = col0 / hd;
            qkv_cc0 = col0 - qkv_which0 * hd;
            qkv_b0 = row0 / p.tokens;
            qkv_t0 = row0 - qkv_b0 * p.tokens;
        }
    }
    constexpr bool F32OUT = sizeof(OT) == 4 || GEGLU;   // GEGLU stages u and gate in fp32 and combines on the way out
    constexpr int NPASS = (F32OUT && TMW == 2) ? 2 : 1;   // a 128-token fp32 tile is staged in two 64-token halves
    constexpr int STRIDE = F32OUT ? OUT_STRIDE_F32 : OUT_STRIDE_B16;
    constexpr int ROWS_PER_PASS = BM / NPASS;
    constexpr int CHUNK_ELEMS = 16 / (int)sizeof(OT);   // elements per 16-byte chunk
    constexpr int CHUNKS_PER_ROW = (GEGLU ? BN / 2 : BN) / CHUNK_ELEMS;
    constexpr int SE = F32OUT ? 4 : 2;                  // bytes per staged element
    constexpr int ITERS = ROWS_PER_PASS * CHUNKS_PER_ROW / 256;   // 16-byte chunks per thread per pass
    // gate * y + residual: the residual chunks of a pass are fetched ahead (pass 0 during the last slab of the main
    // loop, pass 1 once pass 0 is staged); loading them where they are used would expose their latency, and
    // one by one between the stores they would serialise on every load (out may alias res).
    constexpr bool RES = EPI == EPI_GATE_RES;
    f32x4 resv[RES ? NPASS : 1][RES ? ITERS : 1];
    auto load_res = [&](int pass) {
        if constexpr (RES) {
            auto chunk_offset = [&](int j) {   // clamped like every other edge access: masked on store
                const int c = tid + 256 * j;
                const int r = min(row0 + pass * ROWS_PER_PASS + c / CHUNKS_PER_ROW, m - 1), f = min(col0 + (c % CHUNKS_PER_ROW) * CHUNK_ELEMS, n - 4);
                return (size_t)r * n + f;
            };
#pragma unroll
            for (int j = 0; j < ITERS; j++) resv[pass][j] = *reinterpret_cast<const f32x4*>(p.res + chunk_offset(j));
            if (p.res2) {
#pragma unroll
                for (int j = 0; j < ITERS; j++) resv[pass][j] += *reinterpret_cast<const f32x4*>(p.res2 + chunk_offset(j));
            }
        }
    };
    auto slab_step = [&](int s, auto stage_tag) {
        constexpr int STG = decltype(stage_tag)::value;
        if (s == nslab - 1) load_res(0);
#pragma unroll
        for (int ks = 0; ks < BK / 32; ks++) {
            if (ks == 1 && s + 1 < nslab) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's share of slab s + 1 has landed
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // ... and its reads of slab s are complete
                __builtin_amdgcn_s_barrier();
                if (s + 2 < nslab) issue(s + 2, STG);
            }
            if (ks == 0) read_set(STG, 1);
            else if (s + 1 < nslab) read_set(STG ^ 1, 0);
#pragma unroll
            for (int fi = 0; fi < 4; fi++)
#pragma unroll
                for (int ti = 0; ti < TT; ti++)
                    acc[fi][ti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[ks][fi], af[ks][ti], acc[fi][ti], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 4 + TT; j++) {   // fragment reads between the MFMAs
                __builtin_amdgcn_sched_group_barrier(0x008, (4 * TT) / (4 + TT), 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
    };
    for (int s = 0; s < nslab; s += 2) {
        slab_step(s, std::integral_constant<int, 0>{});
        if (s + 1 < nslab) slab_step(s + 1, std::integral_constant<int, 1>{});
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                          // every wave is done with the slab buffers

    // ---- epilogue: registers -> LDS staging tile -> row-contiguous global stores -------------------
    // Register i of tile (fi, ti): feature = wf*64 + fi*16 + 4 q4 + i, token = wt*32*TMW + ti*16 + l16.
#pragma unroll
    for (int pass = 0; pass < NPASS; pass++) {
        // Staging; GATE_LDS: the gate values come from LDS (always, unless the tile's rows straddle gate rows).
        [[maybe_unused]] const float* gate_ptr = p.gate;
        [[maybe_unused]] const int gate_rows = p.rows_per_gate;
        [[maybe_unused]] const size_t gate_stride = p.gate_stride;
        auto stage = [&, gate_ptr, gate_rows, gate_stride](auto gate_lds_tag) {
            constexpr bool GATE_LDS = decltype(gate_lds_tag)::value;
            // bias (and gate) of this lane's 4 column groups first, in one batch of LDS reads
            f32x4 bv[4];
            [[maybe_unused]] f32x4 gv[4];
#pragma unroll
            for (int fi = 0; fi < 4; fi++) {
                const int fl = wf * 64 + fi * 16 + 4 * q4;
                bv[fi] = *reinterpret_cast<const f32x4*>(vec_lds + fl);
                if constexpr (RES && GATE_LDS) gv[fi] = *reinterpret_cast<const f32x4*>(vec_lds + BN + fl);
            }
#pragma unroll
            for (int ti = 0; ti < TT; ti++) {
                const int trow = (NPASS == 1 ? wt * 32 * TMW : 0) + ti * 16 + l16;   // row inside the staging tile
                if constexpr (RES && !GATE_LDS) {
                    const int r = row0 + wt * 32 * TMW + ti * 16 + l16;              // global token row
                    const float* gate_row = gate_ptr + (size_t)(min(r, m - 1) / gate_rows) * gate_stride;
#pragma unroll
                    for (int fi = 0; fi < 4; fi++)   // column clamped: masked on store
                        gv[fi] = *reinterpret_cast<const f32x4*>(gate_row + min(col0 + wf * 64 + fi * 16 + 4 * q4, n - 4));
                }
#pragma unroll
                for (int fi = 0; fi < 4; fi++) {
                    const int fl = wf * 64 + fi * 16 + 4 * q4;      // feature inside the tile
                    f32x4 v = acc[fi][ti];
                    v += bv[fi];
                    if constexpr (EPI == EPI_GELU_TANH) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = gelu_tanh_f(v[j]);
                    } else if constexpr (EPI == EPI_SILU) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = silu_f(v[j]);
                    } else if constexpr (EPI == EPI_GATE_RES) {
                        v *= gv[fi];
                    } else if constexpr (EPI == EPI_QKV) {
                        if (col0 + fl < q_cols) v *= q_scale;      // the four features of v lie in one head
                    }
                    unsigned char* dst = smem + trow * STRIDE + fl * SE;
                    if constexpr (F32OUT) {
                        *reinterpret_cast<f32x4*>(dst) = v;
                    } else {
                        bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                        *reinterpret_cast<bf16x4*>(dst) = o;
                    }
                }
            }
        };
        if (NPASS == 1 || wt == pass) {
            if (!RES || gate_in_lds) stage(std::true_type{});
            else stage(std::false_type{});
        }
        if (pass == 0 && NPASS == 2) load_res(1);   // in flight across this pass's barrier and stores
        __syncthreads();
#pragma unroll
        for (int j = 0; j < ITERS; j++) {
            const int c = tid + 256 * j;
            const int trow = c / CHUNKS_PER_ROW, ch = c % CHUNKS_PER_ROW;
            const int r = row0 + pass * ROWS_PER_PASS + trow;
            const int f = col0 + ch * CHUNK_ELEMS;
            if (r >= m || f >= n) continue;
            if constexpr (GEGLU) {
                // 8 outputs: u at staged columns 8 ch .. 8 ch + 7, gate 64 columns further
                const float* su = reinterpret_cast<const float*>(smem + trow * STRIDE) + ch * 8;
                bf16x8 o8;
#pragma unroll
                for (int j = 0; j < 8; j++) o8[j] = (bf16_t)(su[j] * gelu_erf_f(su[64 + j]));
                *reinterpret_cast<bf16x8*>(static_cast<bf16_t*>(p.out) + (size_t)r * n + f) = o8;
                continue;
            }
            const unsigned char* srcp = smem + trow * STRIDE + ch * 16;
            if constexpr (EPI == EPI_QKV) {
                // feature f = (which, head, i); token row r = (sample b, token t): 8 features stay inside one head.
                // The divisions are taken once per tile, on its first column and row; a chunk adds its offset and steps
                // over at most one boundary of each kind when a tile is no wider than q, k or v and no taller than a
                // sample (otherwise every chunk divides).
                const int hd = p.heads * 64;
                int which, cc, b, t;
                if (qkv_steps) {
                    which = qkv_which0;
                    cc = qkv_cc0 + ch * CHUNK_ELEMS;
                    if (cc >= hd) { cc -= hd; which++; }
                    b = qkv_b0;
                    t = qkv_t0 + pass * ROWS_PER_PASS + trow;
                    if (t >= p.tokens) { t -= p.tokens; b++; }
                } else {
                    which = f / hd;
                    cc = f - which * hd;
                    b = r / p.tokens;
                    t = r - b * p.tokens;
                }
                const int head = cc / 64, i0 = cc % 64;
                OT* base = static_cast<OT*>(which == 0 ? p.q : (which == 1 ? p.k : p.v));
                OT* dst = base + (((size_t)b * p.heads + head) * p.n_total + p.tok_offset + t) * 64 + i0;
                *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(srcp);
            } else if constexpr (EPI == EPI_GATE_RES) {
                const size_t o = (size_t)r * n + f;
                *reinterpret_cast<f32x4*>(static_cast<float*>(p.out) + o) = *reinterpret_cast<const f32x4*>(srcp) + resv[pass][j];
            } else {
                OT* dst = static_cast<OT*>(p.out) + (size_t)split * m * n + (size_t)r * n + f;
                *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(srcp);
            }
        }
        if (pass + 1 < NPASS) __syncthreads();
    }
}

// Up to this many tile columns a launch hands each XCD a run of consecutive tiles (see the kernel).
constexpr int kNarrowTileCols = 16;

template <typename OT, int EPI, int TMW>
int launch_tiles(const GemmGroup& g, int tiles_n, hipStream_t st, int ksplit = 1) {
    constexpr int BM = Geo<TMW>::BM;
    GemmGroup gg = g;
    // The smaller problem goes first: its tiles fetch a whole weight matrix from HBM for few rows, which is better
    // hidden under the start of the large problem than left for the end of the launch.
    if (gg.count > 1 && gg.p[1].m < gg.p[0].m) {
        const GemmProblem t = gg.p[0];
        gg.p[0] = gg.p[1];
        gg.p[1] = t;
    }
    const int tiles0 = ((gg.p[0].m + BM - 1) / BM) * tiles_n;
    const int tiles1 = gg.count > 1 ? ((gg.p[1].m + BM - 1) / BM) * tiles_n : 0;
    char name[96];
    snprintf(name, sizeof(name), "gemm_mfma_%dx%d.epi%d.n%d.k%d", BM, BN, EPI, g.n, g.k);
    double rows = g.p[0].m + (g.count > 1 ? g.p[1].m : 0);
    HybTraceScope trace(name, "flop", 2.0 * rows * g.n * g.k, st);
    int t0 = tiles0;
    if (tiles0 == 0) {  // keep problem 0 non-empty so that the tile -> problem split stays simple
        gg.p[0] = gg.p[1];
        gg.count = 1;
        t0 = tiles1;
    }
    const int total = (tiles0 + tiles1) * ksplit;
    const int xcd_run = tiles_n <= kNarrowTileCols ? (total + 7) / 8 : 0;
    const int grid = xcd_run ? 8 * xcd_run : total;
    hipLaunchKernelGGL((gemm_mfma_kernel<OT, EPI, TMW>), dim3(grid), dim3(256), 0, st, gg, tiles_n, t0, total, xcd_run, ksplit);
    return hyb_check_launch("gemm_mfma");
}

// Second pass of the k split: out = epilogue(sum over the planes, in order, + bias), one thread per element.
template <typename OT>
__global__ __launch_bounds__(256) void gemm_splitk_merge_kernel(GemmGroup g, const float* planes, int ksplit, int epi) {
    const GemmProblem& p = g.p[0];
    const size_t total = (size_t)p.m * g.n;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int r = (int)(i / g.n), c = (int)(i % g.n);
    float v = planes[i];
    for (int s = 1; s < ksplit; s++) v += planes[(size_t)s * total + i];
    if (p.bias) v += p.bias[c];
    gemm_store_scalar<OT>(p, epi, g.n, r, c, v);
}

// k split for launches that cannot fill the chip with tiles but have a long k (each workgroup then waits for
// one k-slab after the other: the time is slabs x slab latency whatever the chip could do).  Returns the number
// of splits (1: none): as many as keep every workgroup resident at once (768 slots of 64-row tiles) with at
// least 4 slabs each, at most 8, and only when the caller's scratch holds the planes.  (slots: 512 for 128-row
// tiles, 768 for 64-row tiles.)
constexpr int kSplitMinSlabs = 32;
int choose_ksplit(const GemmGroup& g, int tiles, int slots) {
    const int nslab = g.k / BK;
    if (g.count != 1 || !g.splitk_ws || nslab < kSplitMinSlabs || tiles <= 0) return 1;
    int s = slots / tiles;
    if (s > nslab / 4) s = nslab / 4;
    if (s > 8) s = 8;
    if (s < 2 || (size_t)s * g.p[0].m * g.n * sizeof(float) > g.splitk_bytes) return 1;
    return s;
}

// 128-token tiles unless they would fill less than three quarters of the 512 workgroup slots of the chip (two
// per CU); then 64-token tiles, of which three fit a CU (768 slots), halve the length of the single round.
constexpr int kSmallGridTiles = 384;

template <typename OT, int EPI>
int launch_epi(const GemmGroup& g, hipStream_t st) {
    const int tile_cols = EPI == EPI_GEGLU ? BN / 2 : BN;
    const int tiles_n = (g.n + tile_cols - 1) / tile_cols;
    const int rows1 = g.count > 1 ? g.p[1].m : 0;
    const int tiles128 = ((g.p[0].m + 127) / 128 + (rows1 + 127) / 128) * tiles_n;
    if (tiles128 == 0) return HYB_OK;
    if constexpr (EPI != EPI_GEGLU) {
        // 128-row tiles stream a third fewer operand bytes: preferred whenever they allow a split at all
        int ksplit = 1;
        bool tall = false;
        if (tiles128 <= kSmallGridTiles) {
            ksplit = choose_ksplit(g, tiles128, 512);
            tall = ksplit > 1;
            if (!tall) ksplit = choose_ksplit(g, ((g.p[0].m + 63) / 64) * tiles_n, 768);
        }
        if (ksplit > 1) {
            // pass 1: raw fp32 sums of every k share (plain epilogue, no bias), pass 2: merge + the real epilogue
            GemmGroup part = g;
            part.p[0].bias = nullptr;
            part.p[0].out = g.splitk_ws;
            int rc = tall ? launch_tiles<float, EPI_BIAS, 2>(part, tiles_n, st, ksplit) : launch_tiles<float, EPI_BIAS, 1>(part, tiles_n, st, ksplit);
            if (rc != HYB_OK) return rc;
            const size_t elems = (size_t)g.p[0].m * g.n;
            HybTraceScope trace("gemm_splitk_merge", "byte", (double)elems * (4.0 * ksplit + sizeof(OT)), st);
            hipLaunchKernelGGL((gemm_splitk_merge_kernel<OT>), dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, g,
                               static_cast<const float*>(g.splitk_ws), ksplit, EPI);
            return hyb_check_launch("gemm_splitk_merge");
        }
    }
    if (tiles128 <= kSmallGridTiles && g.p[0].m + rows1 > 64) return launch_tiles<OT, EPI, 1>(g, tiles_n, st);
    return launch_tiles<OT, EPI, 2>(g, tiles_n, st);
}

// Long-k launches with enough 256 x 128 tiles for more than half of the CUs go to the large-tile kernel (one
// workgroup per CU): there the fixed cost of a tile (first-slab latency, epilogue: about 10 us with the gate + residual
// epilogue) is small against its main loop, and the operand stream per flop is a quarter smaller (the SD3-shaped fc2,
// k = 6144: 216 tiles in one round, 78 us alone and 90 us inside the step against 101 and 103 us with 420 tiles of
// 128 x 128 on 512 slots; launches of several rounds, batch 2 or the 2048 x 2048 shape, gain 3-4 % per launch).  With
// fewer k-slabs the 128 x 128 kernel, whose two workgroups per CU hide each other's fixed costs, is as fast or faster
// (measured at k = 1536 inside the step: out-projection 35.0 against 35.4 us in one round, fc1 110 against 98 us in
// four rounds).
constexpr int kLargeTileMinSlabs = 48;          // launches of several rounds
constexpr int kLargeTileMinSlabsOneRound = 32;  // launches of one round (the SDXL-shaped down-projection, k = 2560)
bool use_large_tiles(const GemmGroup& g, hyb_dtype out_dtype, int epi) {
    const bool f32 = out_dtype == HYB_F32;
    const bool has_form = epi == EPI_BIAS || epi == EPI_GELU_TANH || epi == EPI_SILU || (epi == EPI_GATE_RES && f32);
    if (!has_form || g.k / BK < kLargeTileMinSlabsOneRound) return false;
    int tiles = 0;
    for (int i = 0; i < g.count; i++) {
        tiles += ((g.p[i].m + 255) / 256) * ((g.n + 127) / 128);
    }
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) cus = 256;
    }
    return 2 * tiles > cus && (tiles <= cus || g.k / BK >= kLargeTileMinSlabs);
}

}  // namespace

int hyb_launch_gemm_mfma(const GemmGroup& g, hyb_dtype out_dtype, int epi, hipStream_t st) {
    if (g.k <= 0 || g.k % BK != 0 || g.n % 8 != 0 || g.n < 8) return -1;
    // per-lane byte offsets inside a tile's operand buffers are 32-bit: up to 128 rows of k elements, and for the
    // gated epilogue the gate rows n rows further down
    if ((size_t)g.k * 2 * 256 >= ((size_t)1 << 31)) return -1;
    if (epi == EPI_GEGLU && ((size_t)g.n + 128) * g.k * 2 >= ((size_t)1 << 31)) return -1;
    for (int i = 0; i < g.count; i++) {
        const GemmProblem& p = g.p[i];
        if (epi == EPI_GATE_RES && p.gate && (p.gate_stride % 4 != 0)) return -1;
        if (epi == EPI_QKV && (p.heads <= 0 || g.n % (p.heads * 64) != 0 || g.n / (p.heads * 64) > 3)) return -1;
    }
    const bool f32 = out_dtype == HYB_F32;
    if (use_large_tiles(g, out_dtype, epi)) {
        const int rc = hyb_launch_gemm_mfma_big(g, out_dtype, epi, st);
        if (rc >= 0) return rc;
    }
    switch (epi) {
        case EPI_BIAS: return f32 ? launch_epi<float, EPI_BIAS>(g, st) : launch_epi<bf16_t, EPI_BIAS>(g, st);
        case EPI_GELU_TANH: return f32 ? launch_epi<float, EPI_GELU_TANH>(g, st) : launch_epi<bf16_t, EPI_GELU_TANH>(g, st);
        case EPI_SILU: return f32 ? launch_epi<float, EPI_SILU>(g, st) : launch_epi<bf16_t, EPI_SILU>(g, st);
        case EPI_GATE_RES: return f32 ? launch_epi<float, EPI_GATE_RES>(g, st) : -1;
        case EPI_QKV: return f32 ? -1 : launch_epi<bf16_t, EPI_QKV>(g, st);
        case EPI_GEGLU: return f32 ? -1 : launch_epi<bf16_t, EPI_GEGLU>(g, st);
        default: return -1;
    }
}
