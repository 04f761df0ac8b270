// Flash-style joint attention for gfx950, bf16 operands, head_dim 64:
// o = softmax(q k^T * scale) v with a streaming (online) softmax, never materialising scores.
//
// A workgroup of 4 waves owns 128 query rows of one (batch, head); each wave owns 32 of them.
// Keys / values are streamed 64 at a time through double-buffered LDS tiles shared by the waves,
// copied global -> LDS by 16-byte direct-to-LDS buffer loads (no VGPR staging; the tile's offset is a scalar
// operand, the per-lane offset a loop invariant, so a tile costs no address arithmetic); rows are 128 bytes,
// unpadded, with their 16-byte slots XOR-swizzled against bank conflicts: K rows (read one row per
// lane, 16 bytes each) by (row ^ row >> 3) & 7, V rows (read by transposing loads, 8 keys x 64 bytes
// per instruction) by 4 * (row >> 1 & 1).
// Both contractions run on v_mfma_f32_32x32x16_bf16 in TRANSPOSED form:
//   S^T = K Q^T   (A operand: a K row per lane from LDS; B operand: the lane's query row, kept in
//                  registers for the whole kernel)
//   O^T += V^T P^T (A operand: V^T from LDS; B operand: P^T)
// In the transposed form a lane's 16 accumulator registers of S^T all belong to ONE query
// (column lane % 32), so the row maximum and row sum are per-lane scalars (plus one exchange
// with lane ^ 32, which holds the other half of the keys), and -- because the order of the
// contraction index inside an MFMA does not matter as long as both operands agree -- the
// exponentiated S^T registers, rounded to bf16, ARE the B operand of the second contraction:
// registers 8h..8h+7 of a lane hold keys {16h + 4g + 0..3, 16h + 8 + 4g + 0..3} (g = lane / 32),
// and the matching V^T fragment comes from two transposing LDS reads (ds_read_b64_tr_b16) of the V
// tile kept in its natural [key][feature] layout: in a group of 16 lanes, lane s points at 4
// features of key (s / 4) and lane i receives feature (i) of 4 consecutive keys.
// The K fragments of a tile flow through a ring of four reads that run ahead of the MFMAs; the V^T
// fragments of the first 32 output features are requested before the softmax and used after it.
// Softmax runs in fp32 with exp2 and the scale folded into one FMA.  The running maximum is only
// advanced (and the output accumulator rescaled) when some row's maximum grew by more than 2^8;
// until then exponentials are taken against the older maximum (values up to 2^8, exact same
// result after the final normalisation up to rounding).  The normaliser is the sum of the
// bf16-rounded probabilities that enter the second contraction (v_dot2 with ones).
// Tail keys are masked to -inf before the row maximum; tail query rows are clamped on load
// and not stored.  The reduction order is fixed: results are deterministic and batch-invariant.
//
// Prescaled queries (template parameter PRE; the joint block's QKV projection stores q times scale x log2(e)
// before its one rounding to bf16).  The kernel is bound by its vector instructions, and with the factor
// already in q the scores are exponents of 2 as they leave the MFMA.  A workgroup then first takes all its
// key tiles with reference 0: P = 2^score, no row maxima, no exchange with lane ^ 32, no test for a grown
// maximum and no FMA per score (57 of 131 vector instructions per tile and wave less).  The sums of such a
// pass are exact as long as they stay far from the ends of the fp32 range: after the last tile every row's
// sum must lie in [2^-64, 2^64] (terms of up to 2^64 leave the accumulators below 2^64 x 64 x |v|; a sum
// of at least 2^-64 means the terms that matter are normal numbers in bf16 as well).  If any row of the
// workgroup fails (the four waves agree through a flag in LDS, so that all of them keep reaching the same
// barriers) the workgroup starts over with the running-maximum loop described above; which path a
// workgroup takes depends on its own 128 query rows and its keys only.  A part of a split unit records its
// reference (0 or the running maximum) like any other, and the merge treats both alike.
//
// Split tail.  All workgroups of a launch are usually resident at once (4 per CU), and a CU with 4 of
// them takes a fifth longer than one with 3.  When an XCD holds a few more workgroups than a multiple
// of its CU count (cfg 2: 105 on 32 CUs), that many query blocks are therefore cut along the KEYS into
// 2 or 3 workgroups each, which leave unnormalised partial results (output accumulator, reference
// maximum, normaliser) in a scratch buffer; a small second kernel merges them in a fixed order.  The
// busiest CUs then carry 3 1/3 workgroups instead of 4.  Launches of several rounds cut query blocks
// (about two per CU) in halves the same way, against the ragged end of the launch.  The blocks that are
// cut are the LAST u query blocks of EVERY (batch, head) pair, so a query row is treated the same way
// whatever its sample or head: results stay independent of the batch index.
#include "attention.h"

#include <type_traits>

namespace {

constexpr int BQ = 128;
constexpr int BKV = 64;
constexpr int ROWB = 128;                   // bytes per K / V row in LDS
constexpr int TILE_BYTES = BKV * ROWB;      // 8 KB per operand tile
constexpr float RESCALE_LOG2 = 8.0f;
constexpr int PART_FLOATS = 34 * 256;       // per part of a split unit: 32 accumulator values, maximum, normaliser per thread

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef bf16x4 __attribute__((address_space(3)))* lds_bf16x4_ptr;
typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }   // K tile: row-per-lane 16-byte reads
// V tile: a transposing read touches 8 consecutive keys x 64 bytes, 4 keys per half wave; keys r and r + 2
// sit 256 bytes (one sweep of the banks) apart, so they go to opposite 64-byte halves of their rows.
__device__ __forceinline__ int swz_v(int r) { return ((r >> 1) & 1) * 4; }

__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// max(x, x of lane ^ 32): v_permlane32_swap exchanges the upper 32 lanes of its first operand with the
// lower 32 lanes of its second; with both holding x, one of them then carries the lower half's values in
// both halves and the other the upper half's, so their maximum is the maximum over the pair of lanes.
__device__ __forceinline__ float max_with_other_half(float x) {
    float p = x, q = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(p), "+v"(q));
    return max3(p, q, q);
}

// Transposing LDS reads of the V^T fragments of 32 output features (DT) for the four 16-key groups of a tile,
// written as asm so that they can be issued long before their use: the compiler neither tracks them nor puts
// a wait for the direct-to-LDS copies of the NEXT tile (other buffer) in front of them.  lds_wait() below
// must stand between these reads and the first use of their results.
template <int BUF, int DT>
__device__ __forceinline__ void v_frags(unsigned vaddr, bf16x4 (&vh)[2][2][2]) {
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            const int off = BUF * 2 * TILE_BYTES + (kt * 32 + hf * 16) * ROWB;
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[kt][hf][0]) : "v"(vaddr), "i"(off));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[kt][hf][1]) : "v"(vaddr), "i"(off + 8 * ROWB));
        }
}

// Waits for every outstanding LDS read; the fragments pass through it as operands, so nothing that uses
// (or copies) them can be scheduled before the wait.
__device__ __forceinline__ void lds_wait(bf16x4 (&vh)[2][2][2], bf16x8 (&vf)[2][2]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(vh[0][0][0]), "+v"(vh[0][0][1]), "+v"(vh[0][1][0]), "+v"(vh[0][1][1]),
                   "+v"(vh[1][0][0]), "+v"(vh[1][0][1]), "+v"(vh[1][1][0]), "+v"(vh[1][1][1]));
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            const bf16x4 lo = vh[kt][hf][0], hi = vh[kt][hf][1];
            vf[kt][hf] = bf16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
}

template <bool PRE>
__global__ __launch_bounds__(256, 4) void attention_mfma_kernel(AttnArgs a) {
    // [buffer][K tile | V tile]
    __shared__ __attribute__((aligned(16))) unsigned char smem[2][2 * TILE_BYTES];

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);   // uniform: LDS copy targets (M0) become scalar arithmetic
    const int lq = lane % 32, g = lane / 32;
    // Workgroups go round-robin to the 8 XCDs (each with its own L2) in launch order.  When the number of
    // (batch, head) pairs is a multiple of 8, pair p is served entirely by XCD p % 8, so its K and V stay in
    // one L2 instead of being fetched into all eight.
    const int qblocks = (a.n_q + BQ - 1) / BQ, pairs = a.batch * a.heads;
    int pair, qb;
    int part = 0, nparts = 1, unit = 0;   // split tail: this workgroup's share of the keys of query block `unit`
    if (pairs % 8 == 0) {
        // XCD x serves pairs x, x + 8, ...: first the whole (uncut) query blocks of all its pairs, then the parts of the
        // cut ones (the last tail_per_pair blocks of every pair)
        const int xcd = blockIdx.x % 8;
        const int j = blockIdx.x / 8;
        const int whole = qblocks - a.tail_per_pair;   // uncut query blocks per pair
        if (a.tail_parts > 1 && j >= a.tail_from) {
            const int e = j - a.tail_from;
            nparts = a.tail_parts;
            part = e % nparts;
            const int t = e / nparts;                  // cut block of this XCD
            unit = xcd * a.tail_units + t;
            pair = xcd + 8 * (t / a.tail_per_pair);
            qb = whole + t % a.tail_per_pair;
        } else {
            pair = xcd + 8 * (j / whole);
            qb = j % whole;
        }
    } else {
        pair = blockIdx.x / qblocks;
        qb = blockIdx.x % qblocks;
    }
    const int h = pair % a.heads, b = pair / a.heads;
    const size_t bh = (size_t)b * a.heads + h;
    const int qrow = qb * BQ + wave * 32 + lq;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q) + (bh * (a.q_stride ? a.q_stride : a.n_q) + min(qrow, a.n_q - 1)) * 64;
    const bf16_t* kp = static_cast<const bf16_t*>(a.k) + bh * a.n_kv * 64;
    const bf16_t* vp = static_cast<const bf16_t*>(a.v) + bh * a.n_kv * 64;

    bf16x8 qf[4];
#pragma unroll
    for (int kk = 0; kk < 4; kk++) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);

    // Tile copy: 16 chunks of 1 KB (8 rows) per tile pair, 4 per wave: chunks w, w+4 of K and of V.
    // Lane i fills slot i % 8 of row i / 8 of its chunk with feature vector (slot ^ swz(row)) (V: swz_v).
    // Buffer loads: the per-lane byte offset inside a tile is constant, the tile's offset is a scalar, so a
    // tile costs no vector arithmetic.  Only a ragged last tile uses per-lane offsets with clamped rows
    // (masked in the scores); every address is inside the pair's K / V rows.
    const int cp_row = lane / 8;
    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kp, 0, a.n_kv * ROWB, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vp, 0, a.n_kv * ROWB, 0x00020000);
    int koff[2], voff[2];
#pragma unroll
    for (int c = 0; c < 2; c++) {
        const int r = (wave + 4 * c) * 8 + cp_row;                           // row inside the tile
        koff[c] = r * ROWB + (((lane % 8) ^ swz(r)) * 16);
        voff[c] = r * ROWB + (((lane % 8) ^ swz_v(r)) * 16);
    }
    const int last_full = a.n_kv / BKV;     // tiles below this index hold 64 valid keys
    auto issue = [&](int t, int buf) {
        if (t < last_full) {
#pragma unroll
            for (int c = 0; c < 2; c++) {
                unsigned char* dst = smem[buf] + (wave + 4 * c) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)dst, 16, koff[c], t * TILE_BYTES, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(dst + TILE_BYTES), 16, voff[c], t * TILE_BYTES, 0, 0);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 2; c++) {
                const int r = (wave + 4 * c) * 8 + cp_row;
                const int rc = min(t * BKV + r, a.n_kv - 1);                  // clamped row of the pair
                unsigned char* dst = smem[buf] + (wave + 4 * c) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)dst, 16, rc * ROWB + (((lane % 8) ^ swz(r)) * 16), 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(dst + TILE_BYTES), 16, rc * ROWB + (((lane % 8) ^ swz_v(r)) * 16), 0, 0, 0);
            }
        }
    };

    // scores are exponentiated in base 2; PRE: q came pre-multiplied by scale x log2(e), the scores are base-2 exponents
    const float c = PRE ? 1.f : a.scale * 1.4426950408889634f;
    float m_run = -__builtin_inff(), l_run = 0.f;
    f32x16 o[2];
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[dt][i] = 0.f;

    // V^T fragments by transposing reads: lane (group G = lane / 16, s = lane % 16) points at features
    // dt*32 + 16 (G % 2) + 4 (s % 4) .. +3 of key k0 + s / 4 and receives feature dt*32 + lane % 32 of
    // keys k0 .. k0 + 3 (k0 = kt*32 + hf*16 + 4 g; second read: + 8).
    const int sl = lane % 16;
    const int v_key = 4 * g + sl / 4;                                  // + kt*32 + hf*16 (+8)
    const int v_feat = 16 * ((lane / 16) % 2) + 4 * (sl % 4);          // + dt*32

    // Per-lane LDS addresses, hoisted out of the tile loop.  The XOR swizzle makes the slot of a read
    // (lane part) ^ (compile-time part D) for K; the lane part is folded into 4 base addresses, one per value
    // of D (V: one per half of the features), and everything else (tile row block, operand, buffer) is an
    // immediate offset.
    const unsigned lds0 = (unsigned)(size_t)(lptr_t)&smem[0][0];
    const unsigned char* kbase[4];
    unsigned vbase[2];   // by half of the output features; swz_v depends on the lane's key only
    {
        const int kb = (g ^ lq ^ (lq >> 3)) & 7;
#pragma unroll
        for (int j = 0; j < 4; j++) kbase[j] = &smem[0][0] + lq * ROWB + ((kb ^ (2 * j)) * 16);
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
            vbase[dt] = lds0 + TILE_BYTES + v_key * ROWB + (((4 * dt + v_feat / 8) ^ swz_v(v_key)) * 16) + (v_feat % 8) * 2;
    }

    const int nt = (a.n_kv + BKV - 1) / BKV;
    const int t_begin = part * nt / nparts, t_end = (part + 1) * nt / nparts;   // this workgroup's key tiles
    auto tile = [&](int t, auto buf_tag, auto direct_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr bool DIRECT = decltype(direct_tag)::value;   // P = 2^s without a reference maximum (see below)
        constexpr int BUF_OFF = BUF * 2 * TILE_BYTES;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of tile t has landed
        __builtin_amdgcn_s_barrier();                      // ... everyone's; and the other buffer is free again
        if (t + 1 < t_end) issue(t + 1, BUF ^ 1);

        // S^T = K Q^T: two accumulation chains (keys 0..31 / 32..63) interleaved; the K fragments flow through
        // a ring of four so that four LDS reads are always in flight ahead of the MFMA that needs them.
        auto k_frag = [&](int j) {
            const int kt = j & 1, kk = j >> 1;
            return *reinterpret_cast<const bf16x8*>(kbase[(kk ^ (2 * kt)) & 3] + BUF_OFF + kt * 32 * ROWB);
        };
        bf16x8 ring[4];
#pragma unroll
        for (int j = 0; j < 4; j++) ring[j] = k_frag(j);
        f32x16 s[2];
#pragma unroll
        for (int i = 0; i < 16; i++) s[0][i] = s[1][i] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            s[j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[j & 3], qf[j >> 1], s[j & 1], 0, 0, 0);
            if (j + 4 < 8) ring[j & 3] = k_frag(j + 4);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);

        // V^T fragments of the first 32 output features: issued now, consumed after the softmax
        bf16x4 vh[2][2][2][2];
        bf16x8 vf[2][2][2];
        v_frags<BUF, 0>(vbase[0], vh[0]);

        if (t == nt - 1 && (a.n_kv % BKV) != 0) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int key = t * BKV + kt * 32 + 8 * (i / 4) + 4 * g + (i % 4);
                    if (key >= a.n_kv) s[kt][i] = -__builtin_inff();
                }
        }
        bf16x8 pb[2][2];
        if constexpr (DIRECT) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) pb[kt][i / 8][i % 8] = (bf16_t)__builtin_amdgcn_exp2f(s[kt][i]);
        } else {
            // v_max3_f32 directly: fmaxf() makes the compiler canonicalise every MFMA output first (one extra
            // multiply per score), which costs more than the maxima themselves
            float mx = s[0][0], my = s[1][0];      // two chains: half the dependent latency
#pragma unroll
            for (int i = 1; i < 15; i += 2) {
                mx = max3(mx, s[0][i], s[0][i + 1]);
                my = max3(my, s[1][i], s[1][i + 1]);
            }
            mx = max3(mx, s[0][15], s[1][15]);
            mx = max_with_other_half(max3(mx, my, my));
            // advance the running maximum only when it would grow by more than 2^RESCALE_LOG2
            const bool grow = (mx - m_run) * c > RESCALE_LOG2;      // first tile: m_run = -inf -> true
            if (__any(grow)) {
                const float m_new = grow ? mx : m_run;
                const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c);   // 1 where unchanged, 0 on the first tile
                m_run = m_new;
                l_run *= corr;
#pragma unroll
                for (int dt = 0; dt < 2; dt++)
#pragma unroll
                    for (int i = 0; i < 16; i++) o[dt][i] *= corr;
            }
            const float mc = m_run * c;
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 16; i++) pb[kt][i / 8][i % 8] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[kt][i], c, -mc));
        }

        // O^T += V^T P^T (the fragments of the other 32 features take the registers the scores leave)
        v_frags<BUF, 1>(vbase[1], vh[1]);
        lds_wait(vh[0], vf[0]);
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int hf = 0; hf < 2; hf++) o[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[0][kt][hf], pb[kt][hf], o[0], 0, 0, 0);
        const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int hf = 0; hf < 2; hf++)
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const bf16x2 pr = {pb[kt][hf][j], pb[kt][hf][j + 1]};
                    l_run = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_run, false);
                }
        lds_wait(vh[1], vf[1]);
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int hf = 0; hf < 2; hf++) o[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[1][kt][hf], pb[kt][hf], o[1], 0, 0, 0);
    };
#define HYB_KEY_LOOP(direct_tag)                                                  \
    issue(t_begin, 0);                                                            \
    for (int t = t_begin; t < t_end; t += 2) {                                    \
        tile(t, std::integral_constant<int, 0>{}, direct_tag);                    \
        if (t + 1 < t_end) tile(t + 1, std::integral_constant<int, 1>{}, direct_tag); \
    }
    if constexpr (PRE) {
        // With scores that are base-2 exponents already, the first attempt keeps no reference maximum at all: P = 2^s,
        // reference 0.  Softmax does not depend on the reference, and scaling by a power of two is exact, so this is the
        // same result as long as nothing leaves the range of fp32 / bf16; it saves the row maxima, the rescaling test and
        // the subtraction per score (57 of 131 vector instructions per key tile and wave).  The attempt is valid when every
        // row's sum of probabilities ends up well inside the range (then no probability that matters was flushed and
        // nothing overflowed); otherwise the whole workgroup (uniform decision through LDS, so that every wave passes
        // the same barriers) starts over with the running-maximum form.
        m_run = 0.f;
        HYB_KEY_LOOP(std::true_type{})
        const float l_row = l_run + __shfl_xor(l_run, 32, 64);
        const bool out_of_range = !(l_row > 0x1p-64f && l_row < 0x1p+64f);    // also true for NaN
        const int wave_bad = __any(out_of_range) ? 1 : 0;
        __syncthreads();                                     // every wave is done with the tile buffers
        volatile int* flags = reinterpret_cast<volatile int*>(&smem[0][0]);
        if (lane == 0) flags[wave] = wave_bad;
        __syncthreads();                                     // (waits for the LDS write before the barrier)
        const bool again = (flags[0] | flags[1] | flags[2] | flags[3]) != 0;
        __syncthreads();                                     // the flags are read before the buffers are refilled
        if (again) {
            m_run = -__builtin_inff();
            l_run = 0.f;
#pragma unroll
            for (int dt = 0; dt < 2; dt++)
#pragma unroll
                for (int i = 0; i < 16; i++) o[dt][i] = 0.f;
            HYB_KEY_LOOP(std::false_type{})
        }
    } else {
        HYB_KEY_LOOP(std::false_type{})
    }
#undef HYB_KEY_LOOP

    if (qrow >= a.n_q) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (nparts > 1) {   // partial result of a split unit: merged by attention_merge_kernel
        float* dst = a.part + ((size_t)unit * nparts + part) * PART_FLOATS + tid;
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
            for (int i = 0; i < 16; i++) dst[(dt * 16 + i) * 256] = o[dt][i];
        dst[32 * 256] = m_run;
        dst[33 * 256] = l_tot;
        return;
    }
    const float inv = 1.0f / l_tot;
    const int hd = a.heads * 64;
    bf16_t* orow;
    if (qrow < a.split) orow = static_cast<bf16_t*>(a.o) + ((size_t)b * a.split + qrow) * hd;
    else orow = static_cast<bf16_t*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (qrow - a.split)) * hd;
    orow += h * 64;
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int gi = 0; gi < 4; gi++) {
            const int d0 = dt * 32 + 8 * gi + 4 * g;
            bf16x4 ov = {(bf16_t)(o[dt][4 * gi] * inv), (bf16_t)(o[dt][4 * gi + 1] * inv),
                         (bf16_t)(o[dt][4 * gi + 2] * inv), (bf16_t)(o[dt][4 * gi + 3] * inv)};
            *reinterpret_cast<bf16x4*>(orow + d0) = ov;
        }
}

// Merges the parts of the split tail units (one workgroup per unit, threads as in the main kernel): with
// reference maxima m_p, normalisers l_p and accumulators o_p, the row is sum_p o_p 2^((m_p - M) c) over
// sum_p l_p 2^((m_p - M) c), M = max_p m_p; parts in index order.
template <int PARTS>
__global__ __launch_bounds__(256) void attention_merge_kernel(AttnArgs a) {
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int lq = lane % 32, g = lane / 32;
    const int qblocks = (a.n_q + BQ - 1) / BQ;
    const int unit = blockIdx.x, xcd = unit / a.tail_units, t = unit % a.tail_units;
    const int pair = xcd + 8 * (t / a.tail_per_pair), qb = qblocks - a.tail_per_pair + t % a.tail_per_pair;
    const int h = pair % a.heads, b = pair / a.heads;
    const int qrow = qb * BQ + wave * 32 + lq;
    if (qrow >= a.n_q) return;
    const float c = a.prescaled ? 1.f : a.scale * 1.4426950408889634f;
    const float* src = a.part + (size_t)unit * PARTS * PART_FLOATS + tid;
    // everything this thread needs, requested at once
    float val[PARTS][34];
#pragma unroll
    for (int p = 0; p < PARTS; p++)
#pragma unroll
        for (int i = 0; i < 34; i++) val[p][i] = src[p * PART_FLOATS + i * 256];
    float m_all = val[0][32];
#pragma unroll
    for (int p = 1; p < PARTS; p++) m_all = fmaxf(m_all, val[p][32]);
    float w[PARTS], l = 0.f;
#pragma unroll
    for (int p = 0; p < PARTS; p++) {
        w[p] = __builtin_amdgcn_exp2f((val[p][32] - m_all) * c);
        l = fmaf(val[p][33], w[p], l);
    }
    const float inv = 1.0f / l;
    const int hd = a.heads * 64;
    bf16_t* orow;
    if (qrow < a.split) orow = static_cast<bf16_t*>(a.o) + ((size_t)b * a.split + qrow) * hd;
    else orow = static_cast<bf16_t*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (qrow - a.split)) * hd;
    orow += h * 64;
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int gi = 0; gi < 4; gi++) {
            float r[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float acc = 0.f;
#pragma unroll
                for (int p = 0; p < PARTS; p++) acc = fmaf(val[p][dt * 16 + 4 * gi + e], w[p], acc);
                r[e] = acc * inv;
            }
            bf16x4 ov = {(bf16_t)r[0], (bf16_t)r[1], (bf16_t)r[2], (bf16_t)r[3]};
            *reinterpret_cast<bf16x4*>(orow + dt * 32 + 8 * gi + 4 * g) = ov;
        }
}

// Split decision for a launch: per XCD there are w workgroups (XCD-pinned order) on cus CUs with 4 slots each.  The last
// `per_pair` query blocks of every pair are cut into `parts`; `units` = cut blocks per XCD, `from` = whole blocks per XCD.
struct TailSplit { int from, units, parts, per_pair; };
TailSplit tail_split(int batch, int heads, int n_q) {
    TailSplit t = {0, 0, 1, 0};
    const int pairs = batch * heads;
    if (pairs == 0 || pairs % 8 != 0) return t;
    static int cus_per_xcd = 0;
    if (cus_per_xcd == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) cus = 256;
        cus_per_xcd = cus / 8;
    }
    const int ppx = pairs / 8, qblocks = (n_q + BQ - 1) / BQ;
    const int w = ppx * qblocks;
    int per_pair, parts;
    if (w > 4 * cus_per_xcd) {
        // more than one round: workgroups start as others finish, and the launch ends ragged; about two workgroups'
        // worth per CU are halved along the keys, which shortens that tail (cfg 3: -5 %, cfg 4: -3 %)
        per_pair = 2 * cus_per_xcd / ppx;
        parts = 2;
    } else {
        const int extra = w % cus_per_xcd;
        if (w < cus_per_xcd || extra == 0) return t;
        per_pair = extra / ppx;                            // (a remainder of extra blocks stays whole)
        if (per_pair == 0) return t;
        parts = cus_per_xcd / (per_pair * ppx);            // the parts of all cut blocks fit one more workgroup per CU
        if (parts > 3) parts = 3;
    }
    if (per_pair > qblocks) per_pair = qblocks;
    if (per_pair < 1 || parts < 2) return t;
    t.per_pair = per_pair; t.units = per_pair * ppx; t.from = w - t.units; t.parts = parts;
    return t;
}

}  // namespace

size_t hyb_attention_split_bytes(int batch, int heads, int n_q) {
    const TailSplit t = tail_split(batch, heads, n_q);
    return t.parts > 1 ? (size_t)8 * t.units * t.parts * PART_FLOATS * sizeof(float) : 0;
}

int hyb_launch_attention_mfma(const AttnArgs& a0, hipStream_t st) {
    AttnArgs a = a0;
    a.tail_from = a.tail_units = a.tail_per_pair = 0;
    a.tail_parts = 1;
    int blocks = ((a.n_q + BQ - 1) / BQ) * a.heads * a.batch;
    // the split needs the scratch, whole key tiles for every part, and text rows that are stored (o2) if there are any
    const TailSplit t = a.part ? tail_split(a.batch, a.heads, a.n_q) : TailSplit{0, 0, 1, 0};
    if (t.parts > 1 && (a.n_kv + BKV - 1) / BKV >= 2 * t.parts) {
        a.tail_from = t.from; a.tail_units = t.units; a.tail_parts = t.parts; a.tail_per_pair = t.per_pair;
        blocks = 8 * (t.from + t.units * t.parts);
    }
    dim3 grid(blocks), block(256);
    {
        HybTraceScope trace("attention_mfma", "flop", 4.0 * a.batch * a.heads * (double)a.n_q * a.n_kv * 64, st);
        if (a.prescaled) hipLaunchKernelGGL(attention_mfma_kernel<true>, grid, block, 0, st, a);
        else hipLaunchKernelGGL(attention_mfma_kernel<false>, grid, block, 0, st, a);
    }
    int rc = hyb_check_launch("attention_mfma");
    if (rc != HYB_OK || a.tail_parts == 1) return rc;
    HybTraceScope trace("attention_merge", "byte", 8.0 * a.tail_units * a.tail_parts * PART_FLOATS * 4, st);
    if (a.tail_parts == 2) hipLaunchKernelGGL(attention_merge_kernel<2>, dim3(8 * a.tail_units), block, 0, st, a);
    else hipLaunchKernelGGL(attention_merge_kernel<3>, dim3(8 * a.tail_units), block, 0, st, a);
    return hyb_check_launch("attention_merge");
}
