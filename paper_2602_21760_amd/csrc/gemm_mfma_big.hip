// Large-tile bf16 MFMA GEMM for gfx950: the same contraction as gemm_mfma.hip (out = epilogue(A W^T + bias),
// A [m, k] tokens x features-in, W [n, k] features-out x features-in, fp32 accumulation in
// v_mfma_f32_16x16x32_bf16, k in slabs of 64, identical order of accumulation, so a token's result has the
// same bits whichever of the two kernels computes it), for long-k launches with enough 256 x 128 tiles for the chip.
//
// Why a second geometry.  With 128 x 128 tiles, two workgroups per CU, a launch of 420 tiles and 96 k-slabs (the
// SD3-shaped fc2: n = 1536, k = 6144) is one round in which 164 CUs carry two tiles and 92 carry one, every tile pays
// for 64 KB of operand copies per CU and k-slab pair, and all tiles read their residual and write their output at
// the same moment.  Here a workgroup of 4 waves (2 x 2) owns a 256 x 128 tile alone on its CU (216 tiles for the
// same launch): a wave owns 128 x 64 outputs = 8 x 4 MFMA tiles of 16 x 16 (128 accumulator registers); per k-slab the CU
// copies 48 KB for the same MFMA work, and a wave reads three quarters of the fragment bytes per multiply-add.  One wave per SIMD is
// enough for the MFMA pipe as long as nothing stands in front of its MFMAs in program order (a wave issues in order):
// fragment reads AND slab copies are spread between the MFMAs, the copies of a slab over a whole slab period (a
// quarter per half-step), so that the CU's copy path, which takes about 16 clocks per 1 KB request, never queues up.
//
// Main loop: as in gemm_mfma.hip (direct-to-LDS 16-byte buffer loads with the slab offset as the scalar
// operand, XOR-swizzled unpadded 128-byte rows, explicit vmcnt / lgkmcnt waits and ONE raw barrier per slab), with
// THREE slab buffers (a copy is in flight for one to two slab periods: a lone workgroup has no neighbour on its CU to
// fill a stall).  A k-step of 32 is taken in two halves of four token tiles (16 MFMAs each), so a slab is four
// half-steps; the token fragments of a half-step and the weight fragments of a k-step live in two register sets each, and
// the reads of half-step j + 1 are issued between the MFMAs of half-step j, across the slab boundary.  The slab buffers are separate arrays, so that the compiler knows
// that a copy into one and a fragment read from another do not alias and interleaves them freely.
//
// Epilogue: every wave stages its own 32-token x 64-feature pieces through its own part of the slab buffers (no
// workgroup barrier), and writes / reads global memory in row-contiguous 16-byte pieces (256-byte runs).  Bias and
// gate of the tile's columns are fetched in the prologue and parked in LDS; the residual of piece i + 1 is fetched
// while piece i is staged and stored.
//
// Tile order: XCD x (workgroups x, x + 8, ...) gets one run of consecutive tiles of an order that walks
// groups of four tile rows column by column, so the tiles an XCD works on at a time share few operand
// panels (its L2 is 4 MB).
#include "gemm.h"

#include <type_traits>

namespace {

constexpr int BK = 64;
constexpr int ROWB = BK * 2;   // bytes per LDS row of a slab

template <int TMW, int TFW> struct BigGeo {
    static constexpr int BM = 64 * TMW, BN = 64 * TFW;
    static constexpr int STAGE_BYTES = (BM + BN) * ROWB;      // 48 KB for 256 x 128 tiles
    static constexpr int CPW = STAGE_BYTES / 1024 / 4;        // 1 KB chunks per wave per slab
    // Slab buffers: as many as the 160 KB of LDS hold (3 for 256 x 128 tiles, 2 for 256 x 256).  A slab's copies are
    // requested when its buffer is released and must have landed when the slab before it has been multiplied, so with S
    // buffers a copy may be in flight for S - 1 slab periods.
    static constexpr int NST = 3 * STAGE_BYTES + 2 * BN * 4 <= 160 * 1024 ? 3 : 2;
    static constexpr int SMEM_BYTES = NST * STAGE_BYTES;
    static constexpr int VEC_BYTES = 2 * BN * 4;              // bias and gate of the tile's columns
};

typedef void __attribute__((address_space(3)))* lptr_t;

__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }

__device__ __forceinline__ void buffer_load_lds16(const void* base, unsigned bytes, void* lds, int voffset, int soffset) {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lptr_t)lds, 16, voffset, soffset, 0, 0);
}

constexpr int kGroupRows = 4;   // tile rows per group of the tile order

// Scheduling hint after a block of MN MFMAs and R fragment reads: spread the reads evenly between the MFMAs.
template <int J, int R, int MN>
__device__ __forceinline__ void interleave_reads() {
    if constexpr (J < R) {
        __builtin_amdgcn_sched_group_barrier(0x008, (MN * (J + 1)) / R - (MN * J) / R, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        interleave_reads<J + 1, R, MN>();
    }
}

// MN MFMAs, R fragment reads and V copies, each kind spread evenly.
template <int J, int MN, int R, int V>
__device__ __forceinline__ void interleave_reads_and_copies() {
    if constexpr (J < MN) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr ((R * (J + 1)) / MN != (R * J) / MN) __builtin_amdgcn_sched_group_barrier(0x100, (R * (J + 1)) / MN - (R * J) / MN, 0);
        if constexpr ((V * (J + 1)) / MN != (V * J) / MN) __builtin_amdgcn_sched_group_barrier(0x020, (V * (J + 1)) / MN - (V * J) / MN, 0);
        interleave_reads_and_copies<J + 1, MN, R, V>();
    }
}

template <typename OT, int EPI, int TMW, int TFW>
__global__ __launch_bounds__(256, 1) void gemm_big_kernel(GemmGroup g, int tiles_n, int tiles0, int total, int xcd_run) {
    using G = BigGeo<TMW, TFW>;
    constexpr int BM = G::BM, BN = G::BN, STAGE_BYTES = G::STAGE_BYTES, CPW = G::CPW, NST = G::NST;
    static_assert(TMW % 2 == 0 && TFW % 2 == 0, "wave row offsets must be multiples of 64 (swizzle)");
    // One array per slab buffer: distinct objects, so the compiler knows that a copy into one buffer and a fragment read
    // from another do not alias and may interleave them freely between the MFMAs.
    __shared__ __attribute__((aligned(16))) unsigned char stage0[STAGE_BYTES], stage1[STAGE_BYTES], stage2[NST > 2 ? STAGE_BYTES : 16];
    __shared__ __attribute__((aligned(16))) float vec_lds[2 * BN];
    auto stage_base = [&](int stage) -> unsigned char* { return stage == 0 ? stage0 : (stage == 1 ? stage1 : stage2); };

    int tile = (blockIdx.x % 8) * xcd_run + blockIdx.x / 8;
    if (tile >= total) return;
    // Problem of this tile, selected field by field (indexing the argument array with a run-time index would make the
    // compiler keep a copy of the whole argument block in scratch memory).
    const bool second = tile >= tiles0;
    if (second) tile -= tiles0;
    GemmProblem p;
#define HYB_SEL(f) p.f = second ? g.p[1].f : g.p[0].f
    HYB_SEL(a); HYB_SEL(w); HYB_SEL(bias); HYB_SEL(out); HYB_SEL(m);
    HYB_SEL(res); HYB_SEL(res2); HYB_SEL(gate); HYB_SEL(rows_per_gate); HYB_SEL(gate_stride);
#undef HYB_SEL
    const int m = p.m, n = g.n, k = g.k, m_end = p.m;
    int row0, col0;
    {
        const int tiles_m = (m + BM - 1) / BM;
        const int per_group = kGroupRows * tiles_n;
        const int grp = tile / per_group, in = tile - grp * per_group;
        const int rows_in = min(kGroupRows, tiles_m - grp * kGroupRows);
        row0 = (grp * kGroupRows + in % rows_in) * BM;
        col0 = (in / rows_in) * BN;
    }
    const bf16_t* A = static_cast<const bf16_t*>(p.a);
    const bf16_t* W = static_cast<const bf16_t*>(p.w);

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int wt = wave % 2, wf = wave / 2;          // wave position: tokens, features
    const int l16 = lane % 16, q4 = lane / 16;      // MFMA 16x16x32: row / column of the lane, its quarter of the 32 k

    // Slab copies: chunk c of this wave covers stage rows 8 (wave + 4 c) .. + 7 (rows 0 .. BM-1 = A, then BN rows
    // of W); lane i fills 16-byte slot i % 8 of row i / 8 with k-vector (slot ^ swz(row)).  Rows past the end are
    // clamped to the last row (their products are never stored).
    const int nslab = k / BK;
    const size_t row_bytes = (size_t)k * 2;
    const bf16_t* a_tile = A + (size_t)row0 * k;
    const unsigned a_tile_bytes = (unsigned)(min(BM, m - row0) * row_bytes);
    const int w_rows = min(BN, n - col0);
    const bf16_t* w_tile = W + (size_t)col0 * k;
    const unsigned w_tile_bytes = (unsigned)((size_t)w_rows * row_bytes);
    int voff[CPW];
#pragma unroll
    for (int c = 0; c < CPW; c++) {
        const int r = (wave + 4 * c) * 8 + lane / 8;
        const int kv = (lane % 8) ^ swz(r);
        if (r < BM) voff[c] = (min(row0 + r, m - 1) - row0) * (int)row_bytes + kv * 16;
        else voff[c] = (min(col0 + r - BM, n - 1) - col0) * (int)row_bytes + kv * 16;
    }
    // chunks [c0, c1) of this wave's share of a slab
    auto issue_chunks = [&](int slab, int stage, auto c0_tag, auto c1_tag) {
        constexpr int C0 = decltype(c0_tag)::value, C1 = decltype(c1_tag)::value;
        const int soff = slab * (BK * 2);
#pragma unroll
        for (int c = C0; c < C1; c++) {
            if (c < BM / 32) buffer_load_lds16(a_tile, a_tile_bytes, stage_base(stage) + (wave + 4 * c) * 1024, voff[c], soff);
            else buffer_load_lds16(w_tile, w_tile_bytes, stage_base(stage) + (wave + 4 * c) * 1024, voff[c], soff);
        }
    };
    auto issue = [&](int slab, int stage) { issue_chunks(slab, stage, std::integral_constant<int, 0>{}, std::integral_constant<int, CPW>{}); };

    // Accumulators [feature tile][token tile].  They are never zeroed in registers: the first k-step of the first
    // slab multiplies into a constant-zero C operand (an accumulator file of 256 registers initialised through
    // vector registers would evict every long-lived address of the main loop).
    constexpr int FT = 2 * TFW, TT = 2 * TMW;      // MFMA tiles of 16 features / 16 tokens per wave
    static_assert(TT % 2 == 0 && TT / 2 == 4, "a k-step is taken in two halves of four token tiles");
    f32x4 acc[FT][TT];

    // Fragment addresses inside a stage, as in gemm_mfma.hip: lane (l16, q4) of a 16 x 16 x 32 fragment reads the 16-byte
    // slot 4 ks + (q4 >> 1 | (q4 & 1) << 1) of row l16 (lanes i and i + 32 read 32 contiguous bytes; both operands use the
    // same assignment of k to lane quarters, so the accumulation order equals that of the 128 x 128 kernel); with the
    // swizzle and tile rows 16 t + l16 the slot sits at (lane part) ^ (4 ks ^ 2 (t % 4)), so four per-lane bases per
    // operand cover all reads and the tile's row block (16 t rows) is an immediate offset (the waves' own row offsets are
    // multiples of 64 and leave the swizzle alone).
    const int kq = (q4 >> 1) | ((q4 & 1) << 1);
    const int lb = (kq ^ (l16 & 7) ^ (l16 >> 3)) & 7;
    int a_base[4], w_base[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
        a_base[c] = (wt * 32 * TMW + l16) * ROWB + ((lb ^ (2 * c)) * 16);
        w_base[c] = BM * ROWB + (wf * 32 * TFW + l16) * ROWB + ((lb ^ (2 * c)) * 16);
    }
    // A k-step of 32 is taken in two halves of four token tiles each (16 MFMAs): half-step hs = 2 ks + half of a slab
    // uses the weight fragments of k-step ks (set ks % 2, read once per k-step) and the token fragments of its half
    // (set hs % 2).  That keeps 32 + 32 fragment registers next to the 128 accumulators.
    bf16x8 af[2][TT / 2], wfr[2][FT];
    auto read_half = [&](int stage, int hs) {
        const unsigned char* base = stage_base(stage);
        const int ks = hs >> 1, half = hs & 1;
#pragma unroll
        for (int t = 0; t < TT / 2; t++) {
            const int ti = half * (TT / 2) + t;
            af[hs & 1][t] = *reinterpret_cast<const bf16x8*>(base + a_base[((2 * ks) ^ ti) & 3] + ti * 16 * ROWB);
        }
        if (half == 0) {
#pragma unroll
            for (int t = 0; t < FT; t++)
                wfr[ks & 1][t] = *reinterpret_cast<const bf16x8*>(base + w_base[((2 * ks) ^ t) & 3] + t * 16 * ROWB);
        }
    };

    // Epilogue operands where their latency hides: bias and gate of the tile's columns now (parked in LDS behind the
    // slab buffers once the first slab has landed).  The gate row must be the same for all rows of the tile; tiles
    // that straddle gate rows (samples) read it from global memory in the epilogue.
    bool gate_in_lds = true;   // no gate: ones
    if constexpr (EPI == EPI_GATE_RES) {
        if (p.gate) gate_in_lds = row0 / p.rows_per_gate == min(row0 + BM - 1, m - 1) / p.rows_per_gate;
    }
    {
        constexpr int VPT = 2 * BN / 256;   // values per thread
        float val[VPT];
#pragma unroll
        for (int j = 0; j < VPT; j++) {
            const int i = tid + 256 * j;                 // [0, BN): bias, [BN, 2 BN): gate
            const int f = min(col0 + i % BN, n - 1);
            val[j] = 0.f;
            if (i < BN) {
                if (p.bias) val[j] = p.bias[f];
            } else if constexpr (EPI == EPI_GATE_RES) {
                val[j] = 1.f;
                if (p.gate && gate_in_lds) val[j] = p.gate[(size_t)(row0 / p.rows_per_gate) * p.gate_stride + f];
            }
        }
        // the first NST slabs are requested at once (the launcher guarantees nslab >= NST); slab 0 has landed when at
        // most the copies of the NST - 1 younger slabs are outstanding
#pragma unroll
        for (int j = 0; j < NST; j++) issue(j, j);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 1) * CPW) : "memory");
#pragma unroll
        for (int j = 0; j < VPT; j++) vec_lds[tid + 256 * j] = val[j];
    }
    __builtin_amdgcn_s_barrier();
    read_half(0, 0);

    constexpr bool F32OUT = sizeof(OT) == 4;
    constexpr bool RES = EPI == EPI_GATE_RES;
    constexpr int SE = F32OUT ? 4 : 2;                       // bytes per staged element
    constexpr int WCOLS = 32 * TFW;                          // features of a wave
    constexpr int STRIDE = WCOLS * SE + 16;                  // staging row stride (bytes), padded against conflicts
    constexpr int PPR = WCOLS * SE / 16;                     // 16-byte pieces per staged row
    constexpr int ITERS = 32 * PPR / 64;                     // pieces per lane per 32-token piece of the wave tile
    constexpr int CHUNK_ELEMS = 16 / SE;
    static_assert(32 * STRIDE <= (NST == 2 ? STAGE_BYTES / 2 : 12 * 1024), "a wave's staging piece must fit its part of the slab buffers");
    // gate * y + residual: the residual pieces are fetched ahead (piece 0 during the last slab, piece i + 1 while
    // piece i is staged and stored), with clamped addresses; out may alias res, every element is read before the
    // same lane writes it.
    // (two residual buffers; a 256 x 256 geometry with its 256 accumulators would have room for one)
    constexpr int RES_BUFS = TFW >= 4 ? 1 : 2;
    f32x4 resv[RES ? RES_BUFS : 1][RES ? ITERS : 1];
    f32x4 res2v[RES ? RES_BUFS : 1][RES ? ITERS : 1];         // the optional second residual (same pieces)
    const bool two_res = RES && p.res2 != nullptr;
    const int wrow0 = row0 + wt * 32 * TMW, wcol0 = col0 + wf * WCOLS;   // the wave's corner of the tile
    auto load_res = [&](int tm, int buf) {
        if constexpr (RES) {
            auto piece_offset = [&](int j) {
                const int idx = lane + 64 * j;
                const int r = min(wrow0 + tm * 32 + idx / PPR, m - 1), f = min(wcol0 + (idx % PPR) * CHUNK_ELEMS, n - 4);
                return (size_t)r * n + f;
            };
#pragma unroll
            for (int j = 0; j < ITERS; j++) resv[buf][j] = *reinterpret_cast<const f32x4*>(p.res + piece_offset(j));
            if (two_res) {
#pragma unroll
                for (int j = 0; j < ITERS; j++) res2v[buf][j] = *reinterpret_cast<const f32x4*>(p.res2 + piece_offset(j));
            }
        }
    };

    // the 16 MFMAs of half-step hs; READS = fragment reads of the next half-step that are issued between them
    auto mfma_half = [&](auto hs_tag, auto first_tag, auto copies_tag) {
        constexpr int HS = decltype(hs_tag)::value;
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr int COPIES = decltype(copies_tag)::value;      // slab copies issued next to this half-step
        constexpr int READS = (HS & 1) ? TT / 2 + FT : TT / 2;   // the next half-step starts a k-step: weight fragments too
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int fi = 0; fi < FT; fi++)
#pragma unroll
            for (int t = 0; t < TT / 2; t++) {
                const int ti = (HS & 1) * (TT / 2) + t;
                acc[fi][ti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[(HS >> 1) & 1][fi], af[HS & 1][t], FIRST ? zero : acc[fi][ti], 0, 0, 0);
            }
        // the fragment reads of the next half-step (and, behind the barrier, the copies of the next free slab) between the MFMAs
        if constexpr (COPIES > 0) interleave_reads_and_copies<0, FT * TT / 2, READS, COPIES>();
        else interleave_reads<0, READS, FT * TT / 2>();
    };
    // Slab s sits in stage s % NST.  Half-step hs first requests the fragments of the next half-step.  ONE barrier per
    // slab, before the reads of half-step 3 + 1 = half-step 0 of slab s + 1: by then this wave's
    // share of slab s + 1 has landed (vmcnt: only the copies of younger slabs may be outstanding) and its reads of
    // slab s are complete (lgkmcnt), so behind the barrier slab s + 1 is readable and stage s % NST can be refilled
    // with slab s + NST.
    constexpr int CQ = CPW / 4;                                // copies per half-step in the steady state
    static_assert(CPW % 4 == 0, "a wave's copies of a slab are spread over the four half-steps");
    auto slab_step = [&](int s, auto stage_tag, auto first_tag, bool first_quarter_only) {
        constexpr int STG = decltype(stage_tag)::value;
        constexpr bool FIRST_SLAB = decltype(first_tag)::value;
        if (s == nslab - 1) load_res(0, 0);
        auto half = [&](auto hs_tag) {
            constexpr int HS = decltype(hs_tag)::value;
            if constexpr (HS < 3) read_half(STG, HS + 1);
            else if (s + 1 < nslab) {
                if (NST > 2 && s + 2 < nslab) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * CPW) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                if (s + NST < nslab) {
                    if (first_quarter_only) issue_chunks(s + NST, STG, std::integral_constant<int, 0>{}, std::integral_constant<int, CQ>{});
                    else issue(s + NST, STG);
                }
                read_half((STG + 1) % NST, 0);
            }
            if constexpr (FIRST_SLAB && HS < 2) mfma_half(hs_tag, std::true_type{}, std::integral_constant<int, 0>{});
            else mfma_half(hs_tag, std::false_type{}, std::integral_constant<int, 0>{});
        };
        half(std::integral_constant<int, 0>{});
        half(std::integral_constant<int, 1>{});
        half(std::integral_constant<int, 2>{});
        half(std::integral_constant<int, 3>{});
    };
    // Steady state (slab s + NST exists): no conditions, so that the copies requested behind the barrier are spread
    // between the MFMAs of the same half-step instead of standing in front of them (a wave issues in order: sixteen
    // copy instructions in a row hold up the MFMAs behind them while the matrix pipe runs dry).
    // The copies of a slab are spread over four half-steps (a quarter each), so that the copy path of the CU sees an even
    // stream instead of a burst per slab: the first quarter of slab s + NST behind the barrier of slab s (which frees
    // its buffer), the other three next to half-steps 0 .. 2 of slab s + 1.  On entry the first quarter of slab
    // s + NST - 1 has been requested, its other quarters not.  The count of the wait is unchanged: the copies younger
    // than those of slab s + 1 are the CPW copies of slab s + 2.
    static_assert(NST == 3, "the steady state below is written for three slab buffers");
    auto slab_step_mid = [&](int s, auto stage_tag) {
        constexpr int STG = decltype(stage_tag)::value;
        read_half(STG, 1);
        issue_chunks(s + NST - 1, (STG + NST - 1) % NST, std::integral_constant<int, CQ>{}, std::integral_constant<int, 2 * CQ>{});
        mfma_half(std::integral_constant<int, 0>{}, std::false_type{}, std::integral_constant<int, CQ>{});
        read_half(STG, 2);
        issue_chunks(s + NST - 1, (STG + NST - 1) % NST, std::integral_constant<int, 2 * CQ>{}, std::integral_constant<int, 3 * CQ>{});
        mfma_half(std::integral_constant<int, 1>{}, std::false_type{}, std::integral_constant<int, CQ>{});
        read_half(STG, 3);
        issue_chunks(s + NST - 1, (STG + NST - 1) % NST, std::integral_constant<int, 3 * CQ>{}, std::integral_constant<int, CPW>{});
        mfma_half(std::integral_constant<int, 2>{}, std::false_type{}, std::integral_constant<int, CQ>{});
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * CPW) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        read_half((STG + 1) % NST, 0);
        issue_chunks(s + NST, STG, std::integral_constant<int, 0>{}, std::integral_constant<int, CQ>{});
        mfma_half(std::integral_constant<int, 3>{}, std::false_type{}, std::integral_constant<int, CQ>{});
    };
    const bool steady = 2 * NST < nslab;                    // the steady-state loop below runs at least once
    slab_step(0, std::integral_constant<int, 0>{}, std::true_type{}, steady);
    int s = 1;
    for (; s + 2 * NST - 1 < nslab; s += NST) {
        slab_step_mid(s, std::integral_constant<int, 1 % NST>{});
        slab_step_mid(s + 1, std::integral_constant<int, 2 % NST>{});
        if constexpr (NST > 2) slab_step_mid(s + 2, std::integral_constant<int, 3 % NST>{});
    }
    // the other quarters of the slab whose first quarter the last steady step requested (stage (s + NST - 1) % NST = 0)
    if (steady) issue_chunks(s + NST - 1, 0, std::integral_constant<int, CQ>{}, std::integral_constant<int, CPW>{});
    for (; s < nslab; s += NST) {
        slab_step(s, std::integral_constant<int, 1 % NST>{}, std::false_type{}, false);
        if (s + 1 < nslab) slab_step(s + 1, std::integral_constant<int, 2 % NST>{}, std::false_type{}, false);
        if (NST > 2 && s + 2 < nslab) slab_step(s + 2, std::integral_constant<int, 3 % NST>{}, std::false_type{}, false);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                          // every wave is done with the slab buffers

    // ---- epilogue: per wave, registers -> its own LDS staging piece -> row-contiguous global stores --------
    // Register i of tile (fi, ti): feature = wf*WCOLS + fi*16 + 4 q4 + i, token = wt*32*TMW + ti*16 + l16; piece tm of 32
    // tokens is the pair of token tiles 2 tm, 2 tm + 1.
    // staging area of wave w: with two slab buffers half a buffer each, with three the first 36 KB of buffers 0, 1, 2 and
    // the remaining 12 KB of buffer 0
    unsigned char* stg = NST == 2 ? stage_base(wave & 1) + (wave >> 1) * (STAGE_BYTES / 2)
                                  : (wave < 3 ? stage_base(wave) : stage0 + 36 * 1024);
    [[maybe_unused]] const float* gate_ptr = p.gate;
    [[maybe_unused]] const int gate_rows = p.rows_per_gate;
    [[maybe_unused]] const size_t gate_stride = p.gate_stride;
#pragma unroll
    for (int tm = 0; tm < TMW; tm++) {
        if constexpr (RES_BUFS == 2) {
            if (tm + 1 < TMW) load_res(tm + 1, (tm + 1) & 1);   // in flight across this piece's staging and stores
        } else {
            if (tm > 0) load_res(tm, 0);                          // in flight across this piece's staging
        }
        auto stage = [&](auto gate_lds_tag) {
            constexpr bool GATE_LDS = decltype(gate_lds_tag)::value;
#pragma unroll
            for (int fi = 0; fi < FT; fi++)
#pragma unroll
                for (int h2 = 0; h2 < 2; h2++) {
                    const int fl = fi * 16 + 4 * q4;               // feature inside the wave's columns
                    const int prow = h2 * 16 + l16;                // token inside the 32-token piece
                    f32x4 v = acc[fi][2 * tm + h2];
                    v += *reinterpret_cast<const f32x4*>(vec_lds + wf * WCOLS + fl);
                    if constexpr (EPI == EPI_GELU_TANH) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = gelu_tanh_f(v[j]);
                    } else if constexpr (EPI == EPI_SILU) {
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = silu_f(v[j]);
                    } else if constexpr (RES) {
                        if constexpr (GATE_LDS) {
                            v *= *reinterpret_cast<const f32x4*>(vec_lds + BN + wf * WCOLS + fl);
                        } else {
                            const int r = wrow0 + tm * 32 + prow;  // global token row; column clamped: masked on store
                            const float* gate_row = gate_ptr + (size_t)(min(r, m - 1) / gate_rows) * gate_stride;
                            v *= *reinterpret_cast<const f32x4*>(gate_row + min(wcol0 + fl, n - 4));
                        }
                    }
                    unsigned char* dst = stg + prow * STRIDE + fl * SE;
                    if constexpr (F32OUT) {
                        *reinterpret_cast<f32x4*>(dst) = v;
                    } else {
                        bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                        *reinterpret_cast<bf16x4*>(dst) = o;
                    }
                }
        };
        if (!RES || gate_in_lds) stage(std::true_type{});
        else stage(std::false_type{});
        // the wave's own writes are complete before it reads the piece back (LDS operations of a wave are
        // executed in order; the wait also keeps the compiler from moving the reads up)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < ITERS; j++) {
            const int idx = lane + 64 * j;
            const int prow = idx / PPR, pc = idx % PPR;
            const int r = wrow0 + tm * 32 + prow;
            const int f = wcol0 + pc * CHUNK_ELEMS;
            const unsigned char* srcp = stg + prow * STRIDE + pc * 16;
            if constexpr (RES) {
                f32x4 y = *reinterpret_cast<const f32x4*>(srcp) + resv[tm % RES_BUFS][j];
                if (two_res) y += res2v[tm % RES_BUFS][j];
                if (r < m_end && f < n) *reinterpret_cast<f32x4*>(static_cast<float*>(p.out) + (size_t)r * n + f) = y;
            } else {
                const u32x4 y = *reinterpret_cast<const u32x4*>(srcp);
                if (r >= m_end || f >= n) continue;
                *reinterpret_cast<u32x4*>(static_cast<OT*>(p.out) + (size_t)r * n + f) = y;

            }
        }
        // the reads above are complete before the next piece overwrites the staging area
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);   // one piece at a time: keeps the accumulators in place until their piece is staged
    }
}

template <typename OT, int EPI, int TMW, int TFW>
int launch_big(const GemmGroup& g, hipStream_t st) {
    using G = BigGeo<TMW, TFW>;
    GemmGroup gg = g;
    const int tiles_n = (g.n + G::BN - 1) / G::BN;
    auto tiles_of = [&](const GemmProblem& p) { return ((p.m + G::BM - 1) / G::BM) * tiles_n; };
    int tiles0 = tiles_of(gg.p[0]), tiles1 = gg.count > 1 ? tiles_of(gg.p[1]) : 0;
    if (tiles0 == 0 && tiles1 > 0) {   // keep problem 0 non-empty so that the tile -> problem split stays simple
        gg.p[0] = gg.p[1]; tiles0 = tiles1; tiles1 = 0; gg.count = 1;
    }
    if (gg.count < 2) gg.p[1] = gg.p[0];   // every field the kernel selects from is defined
    const int total = tiles0 + tiles1;
    if (total <= 0) return HYB_OK;
    char name[96];
    snprintf(name, sizeof(name), "gemm_mfma_%dx%d.epi%d.n%d.k%d", G::BM, G::BN, EPI, g.n, g.k);
    double rows = 0;
    for (int i = 0; i < g.count; i++) rows += g.p[i].m;
    HybTraceScope trace(name, "flop", 2.0 * rows * g.n * g.k, st);
    const int xcd_run = (total + 7) / 8;
    hipLaunchKernelGGL((gemm_big_kernel<OT, EPI, TMW, TFW>), dim3(8 * xcd_run), dim3(256), 0, st, gg, tiles_n, tiles0, total, xcd_run);
    return hyb_check_launch("gemm_mfma_big");
}

}  // namespace

// Large-tile launch (256 x 128 tiles) of a group of up to two problems.  Epilogues: bias, GELU-tanh, SiLU (either output
// type), gate * y + residual(s) (fp32 output).  Returns -1 when the shape or the epilogue has no large-tile
// form.  The caller has validated the group as for hyb_launch_gemm_mfma.
int hyb_launch_gemm_mfma_big(const GemmGroup& g, hyb_dtype out_dtype, int epi, hipStream_t st) {
    if (g.k <= 0 || g.k % BK != 0 || g.n % 8 != 0 || g.n < 8) return -1;
    if ((size_t)g.k * 2 * 256 >= ((size_t)1 << 31)) return -1;    // per-lane byte offsets inside a tile's operand rows are 32-bit
    if (g.k / BK < 3) return -1;                                  // the prologue requests the first three slabs
    const bool f32 = out_dtype == HYB_F32;
    switch (epi) {
        case EPI_BIAS: return f32 ? launch_big<float, EPI_BIAS, 4, 2>(g, st) : launch_big<bf16_t, EPI_BIAS, 4, 2>(g, st);
        case EPI_GELU_TANH: return f32 ? launch_big<float, EPI_GELU_TANH, 4, 2>(g, st) : launch_big<bf16_t, EPI_GELU_TANH, 4, 2>(g, st);
        case EPI_SILU: return f32 ? launch_big<float, EPI_SILU, 4, 2>(g, st) : launch_big<bf16_t, EPI_SILU, 4, 2>(g, st);
        case EPI_GATE_RES: return f32 ? launch_big<float, EPI_GATE_RES, 4, 2>(g, st) : -1;
        default: return -1;
    }
}
