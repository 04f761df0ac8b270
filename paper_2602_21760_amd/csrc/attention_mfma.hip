// Flash-style joint attention for gfx950, bf16 operands, head_dim 64:
// o = softmax(q k^T * scale) v with a streaming (online) softmax, never materialising scores.
//
// A workgroup of 4 waves owns 128 query rows of one (batch, head); each wave owns 32 of them (two tiles of 16).
// Keys / values are streamed 64 at a time through double-buffered LDS tiles shared by the waves,
// copied global -> LDS by 16-byte direct-to-LDS buffer loads (no VGPR staging; the tile's offset is a scalar
// operand, the per-lane offset ONE loop-invariant register for K, V and both halves of a tile, so a tile costs no
// address arithmetic); rows are 128 bytes, unpadded, with their 16-byte slots XOR-swizzled against bank conflicts
// (one swizzle for both tiles, see swz() below).
// Both contractions run on v_mfma_f32_16x16x32_bf16 in TRANSPOSED form (the chip sustains a higher clock on
// this form than on 32x32x16: half the accumulator traffic per multiply-add):
//   S^T = K Q^T   (A operand: 16 keys x 32 features, a K row per lane from LDS; B operand: 16 queries x 32
//                  features, kept in registers for the whole kernel; 4 key tiles x 2 query tiles x 2 steps)
//   O^T += V^T P^T (A operand: 16 features x 32 keys, V^T from LDS; B operand: 16 queries x 32 keys, P^T;
//                  4 feature tiles x 2 query tiles x 2 steps)
// Lane (l16 = lane % 16, q4 = lane / 16) of an accumulator tile holds column l16 and rows 4 q4 .. 4 q4 + 3.  In the
// transposed form the 16 accumulator registers of S^T that belong to one query tile all belong to ONE query
// (column l16), so the row maxima and row sums are two per-lane scalars (plus exchanges with lanes ^ 16 and
// ^ 32, which hold the other keys), and -- because the order of the contraction index inside an MFMA does not
// matter as long as both operands agree -- the exponentiated S^T registers of key tiles 2 s and 2 s + 1, rounded
// to bf16, ARE the B operand of step s of the second contraction: the lane holds keys
// {32 s + 4 q4 + 0..3, 32 s + 16 + 4 q4 + 0..3}, and the matching V^T fragment comes from two transposing LDS reads
// (ds_read_b64_tr_b16) of the V tile kept in its natural [key][feature] layout: in a group of 16 lanes, lane i
// points at 4 features of key (i / 4) and receives feature (i) of 4 consecutive keys.
// The K fragments of a tile flow through a ring of four reads that run ahead of the MFMAs; the V^T
// fragments of the first 32 output features are requested before the softmax and used after it.
// The four waves of a SIMD belong to four workgroups and are in different phases of their tiles; a wave lowers its
// priority (s_setprio) for the 32 exponentials of a tile and keeps it high for everything else, so that one wave's
// exponentials do not hold up another's MFMAs.
//
// Softmax runs in fp32 with exp2.  A workgroup first takes all its key tiles with reference 0: P = 2^(c score),
// c = scale x log2(e): no row maxima, no exchange between lanes, no test for a grown maximum.  With prescaled
// queries (template parameter PRE; the joint block's QKV projection stores q times c before its one rounding to
// bf16) the scores are exponents of 2 as they leave the MFMA and the multiplication goes as well.  The sums
// of such a pass are exact as long as they stay far from the ends of the fp32 range: after the last tile every
// row's sum must lie in [2^-64, 2^64] (terms of up to 2^64 leave the accumulators below 2^64 x 64 x |v|; a sum
// of at least 2^-64 means the terms that matter are normal numbers in bf16 as well).  If any row of the
// workgroup fails (the four waves agree through a flag in LDS, so that all of them keep reaching the same
// barriers) the workgroup starts over with the running-maximum form: the scale folded into one FMA per score; the
// running maximum only advanced (and the output accumulator rescaled) when some row's maximum grew by more
// than 2^8, until then exponentials are taken against the older maximum (values up to 2^8, exact same result
// after the final normalisation up to rounding).  That form is the slower one (it holds more values at a time
// and requests its V^T fragments after the softmax); it runs only for scores beyond about +-64 / c.  Which path
// a workgroup takes depends on its own 128 query rows and its keys only.  A part of a split unit records its
// reference (0 or the running maximum) like any other, and the merge treats both alike.
// The normaliser is the sum of the bf16-rounded probabilities that enter the second contraction (v_dot2 with
// ones).  Tail keys are masked to -inf before the softmax; tail query rows are clamped on load
// and not stored.  The reduction order is fixed: results are deterministic and batch-invariant.
//
// Split tail.  All workgroups of a launch are usually resident at once (4 per CU), and a CU with 4 of
// them takes a quarter longer than one with 3.  When an XCD holds a few more workgroups than a multiple
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
constexpr int PART_FLOATS = 36 * 256;       // per part of a split unit and thread: 32 accumulator values, 2 maxima, 2 normalisers

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef void __attribute__((address_space(3)))* lptr_t;

// One swizzle for both tiles: the 16-byte slot index of row r is XORed with (r & 6) | (r >> 3 & 1); the same for rows
// r and r + 16.
// K tile (a 16-byte read per lane, rows 16 kt + lane % 16, feature slot chosen by lane / 16): with lane bits b5 .. b0 the
// read lands in the 16-byte unit (b0, b2, b1 ^ b4, b3 ^ b5) of a 256-byte sweep of the banks, the combination that
// the counters show free of bank conflicts (other combinations of the same bits cost 4 cycles per read).
// V tile: a transposing read touches 16 consecutive keys x 32 bytes, 8 keys per half wave; keys r, r + 2, r + 4, r + 6
// sit multiples of 256 bytes (one sweep of the banks) apart, so they go to the four different 32-byte quarters of their
// rows (bit 0 of the swizzle only swaps the halves of such a quarter).
__device__ __forceinline__ int swz(int r) { return (r & 6) | ((r >> 3) & 1); }

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
// max(x, x of lane ^ 16): v_permlane16_swap exchanges the odd rows (of 16 lanes) of its first operand with the even
// rows of its second, which leaves the even rows' values in both rows of a pair in one operand and the odd rows' in the other.
__device__ __forceinline__ float max_with_other_row(float x) {
    float p = x, q = x;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(p), "+v"(q));
    return max3(p, q, q);
}

// Transposing LDS reads of the V^T fragments of 32 output features (DT) for the four 16-key groups of a tile,
// written as asm so that they can be issued long before their use: the compiler neither tracks them nor puts
// a wait for the direct-to-LDS copies of the NEXT tile (other buffer) in front of them.  lds_wait() below
// must stand between these reads and the first use of their results.
template <int BUF>
__device__ __forceinline__ void v_frags(unsigned vaddr0, unsigned vaddr1, bf16x4 (&vh)[2][2][2]) {
#pragma unroll
    for (int dd = 0; dd < 2; dd++)
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            const int off = BUF * 2 * TILE_BYTES + ks * 32 * ROWB;
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[dd][ks][0]) : "v"(dd ? vaddr1 : vaddr0), "i"(off));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[dd][ks][1]) : "v"(dd ? vaddr1 : vaddr0), "i"(off + 16 * ROWB));
        }
}

// Waits until at most YOUNGER LDS reads are outstanding (they complete in order: everything requested before the
// YOUNGER most recent ones has arrived); the fragments pass through it as operands, so nothing that uses (or copies)
// them can be scheduled before the wait.
template <int YOUNGER>
__device__ __forceinline__ void lds_wait(bf16x4 (&vh)[2][2][2], bf16x8 (&vf)[2][2]) {
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(vh[0][0][0]), "+v"(vh[0][0][1]), "+v"(vh[0][1][0]), "+v"(vh[0][1][1]),
                   "+v"(vh[1][0][0]), "+v"(vh[1][0][1]), "+v"(vh[1][1][0]), "+v"(vh[1][1][1])
                 : "n"(YOUNGER));
#pragma unroll
    for (int dd = 0; dd < 2; dd++)
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            const bf16x4 lo = vh[dd][ks][0], hi = vh[dd][ks][1];
            vf[dd][ks] = bf16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
}

template <bool PRE>
__global__ __launch_bounds__(256, 4) void attention_mfma_kernel(AttnArgs a) {
    // [buffer][K tile | V tile]
    __shared__ __attribute__((aligned(128))) unsigned char smem[2][2 * TILE_BYTES];

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);   // uniform: LDS copy targets (M0) become scalar arithmetic
    // roles in a 16 x 16 x 32 MFMA: lane = (l16, q4); as A / B operand the lane holds row / column l16 and 8 values of the
    // contraction index chosen by q4, as accumulator column l16 and rows 4 q4 .. 4 q4 + 3.  kq: which 8 features of a
    // 32-feature step the lane holds in K Q^T; q4 = 0, 2 (lanes i and i + 32) take neighbouring 16-byte slots, which is what
    // a 16-byte LDS read per lane needs to run without bank conflicts
    const int l16 = lane % 16, q4 = lane / 16;
    const int kq = (q4 >> 1) | ((q4 & 1) << 1);
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
    // the lane's two query rows (one per 16-query tile of the wave's 32), clamped on load
    bf16x8 qf[2][2];   // [query tile][32-feature step]
    const bf16_t* kp = static_cast<const bf16_t*>(a.k) + bh * a.n_kv * 64;
    const bf16_t* vp = static_cast<const bf16_t*>(a.v) + bh * a.n_kv * 64;
#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
        const int qrow = qb * BQ + wave * 32 + qt * 16 + l16;
        const bf16_t* qp = static_cast<const bf16_t*>(a.q) + (bh * (a.q_stride ? a.q_stride : a.n_q) + min(qrow, a.n_q - 1)) * 64;
#pragma unroll
        for (int ks = 0; ks < 2; ks++) qf[qt][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32 + kq * 8);
    }

    // Tile copy: 16 chunks of 1 KB (8 rows) per tile pair, 4 per wave: chunks w, w+4 of K and of V.
    // Lane i fills slot i % 8 of row i / 8 of its chunk with feature vector (slot ^ swz(row)).
    // Buffer loads: the per-lane byte offset inside a tile is one constant for K and V and both chunks (the swizzle
    // is the same for rows r and r + 32), the rest is a scalar, so a tile costs no vector arithmetic and one
    // register.  Only a ragged last tile uses per-lane offsets with clamped rows (masked in the scores); every
    // address is inside the pair's K / V rows.
    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kp, 0, a.n_kv * ROWB, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vp, 0, a.n_kv * ROWB, 0x00020000);
    const int r0 = wave * 8 + lane / 8;                                       // row inside the tile, first chunk
    const int cp_off = r0 * ROWB + (((lane % 8) ^ swz(r0)) * 16);
    const int last_full = a.n_kv / BKV;     // tiles below this index hold 64 valid keys
    auto issue = [&](int t, int buf) {
        if (t < last_full) {
#pragma unroll
            for (int c = 0; c < 2; c++) {
                unsigned char* dst = smem[buf] + (wave + 4 * c) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)dst, 16, cp_off, t * TILE_BYTES + c * 32 * ROWB, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(dst + TILE_BYTES), 16, cp_off, t * TILE_BYTES + c * 32 * ROWB, 0, 0);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 2; c++) {
                // (row and slot taken back out of cp_off, through an empty asm statement that keeps the compiler from computing
                // them ahead of the loop: nothing else of this path then lives in registers over the loop)
                int co = cp_off;
                asm volatile("" : "+v"(co));
                const int rc = min(t * BKV + (co >> 7) + 32 * c, a.n_kv - 1);   // clamped row of the pair
                const int off = rc * ROWB + (co & (ROWB - 1));
                unsigned char* dst = smem[buf] + (wave + 4 * c) * 1024;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)dst, 16, off, 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(dst + TILE_BYTES), 16, off, 0, 0, 0);
            }
        }
    };

    // scores are exponentiated in base 2; PRE: q came pre-multiplied by scale x log2(e), the scores are base-2 exponents
    const float c = PRE ? 1.f : a.scale * 1.4426950408889634f;
    float m_run[2] = {-__builtin_inff(), -__builtin_inff()}, l_run[2] = {0.f, 0.f};   // per query tile: the lane's query in it
    f32x4 o[4][2];   // [16-feature tile][query tile]: features 16 dt + 4 q4 .. + 3 of query 16 qt + l16
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int qt = 0; qt < 2; qt++)
#pragma unroll
            for (int i = 0; i < 4; i++) o[dt][qt][i] = 0.f;

    // V^T fragments by transposing reads: each group of 16 lanes (group q4, s = lane % 16) reads 4 keys x 16 features:
    // lane s points at features dt*16 + 4 (s % 4) .. +3 of key k0 + s / 4 and receives feature dt*16 + s of keys
    // k0 .. k0 + 3 (k0 = ks*32 + 4 q4; second read: + 16).
    const int v_key = 4 * q4 + l16 / 4;                                // + ks*32 (+16)
    const int v_feat = 4 * (l16 % 4);                                  // + dt*16

    // Per-lane LDS addresses, hoisted out of the tile loop: one for the K fragments and one for the V^T fragments.  The
    // XOR swizzle makes the slot of a read (lane part) ^ (compile-time part); the tile buffers are 128-byte aligned,
    // so the compile-time part is an XOR on bits 4 .. 6 of the address (K: bit 6 for the second 32-feature step; V: bit 5
    // for the odd 16-feature tiles, bit 6 for tiles 2 and 3), and everything else (key tile, operand, buffer) is an
    // immediate offset.
    const unsigned lds0 = (unsigned)(size_t)(lptr_t)&smem[0][0];
    const unsigned kbase = lds0 + l16 * ROWB + ((kq ^ swz(l16)) * 16);   // (the swizzle is the same for rows l16 + 16 kt)
    const unsigned vbase = lds0 + TILE_BYTES + v_key * ROWB + (((v_feat / 8) ^ swz(v_key)) * 16) + (v_feat % 8) * 2;

    const int nt = (a.n_kv + BKV - 1) / BKV;
    const int t_begin = part * nt / nparts, t_end = (part + 1) * nt / nparts;   // this workgroup's key tiles
    auto tile = [&](int t, auto buf_tag, auto direct_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr bool DIRECT = decltype(direct_tag)::value;   // P = 2^s without a reference maximum (see below)
        constexpr int BUF_OFF = BUF * 2 * TILE_BYTES;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of tile t has landed
        __builtin_amdgcn_s_barrier();                      // ... everyone's; and the other buffer is free again
        if (t + 1 < t_end) issue(t + 1, BUF ^ 1);

        // the other base addresses differ from kbase / vbase in bit 6 (K: the second 32-feature step) and bit 5 (V: the
        // second 16-feature tile).  The leanest form of the tile (no reference maximum, no multiplication) has two
        // registers to spare for them over the loop; the others make them here, one instruction each (asm, so that
        // the compiler does not move them out of the loop)
        unsigned kb1 = kbase ^ 64u, vb1 = vbase ^ 32u;
        if constexpr (!(DIRECT && PRE)) {
            asm volatile("v_xor_b32 %0, 64, %1" : "=v"(kb1) : "v"(kbase));
            asm volatile("v_xor_b32 %0, 32, %1" : "=v"(vb1) : "v"(vbase));
        }
        // S^T = K Q^T: eight accumulators (4 key tiles x 2 query tiles), two 32-feature steps each; the K fragments
        // (step ks, key tile kt: row 16 kt + l16, slot (4 ks + kq) ^ swz(row)) flow through a ring of four so that four
        // LDS reads are always in flight ahead of the MFMAs that need them.
        auto k_frag = [&](int j) {
            const int ks = j >> 2, kt = j & 3;
            return *(const bf16x8 __attribute__((address_space(3)))*)((ks ? kb1 : kbase) + BUF_OFF + kt * 16 * ROWB);
        };
        bf16x8 ring[4];
        // Wave priority: high while the wave feeds the MFMA pipe (both contractions, and across the tile boundary with its
        // wait, barrier and copies), low during the exponentials of its softmax.  The four waves of a SIMD are in different
        // phases; with equal priorities the exponentials of one wave delay the MFMAs of another (-8 % kernel time).
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int j = 0; j < 4; j++) ring[j] = k_frag(j);
        f32x4 s[4][2];   // [key tile][query tile]: keys 16 kt + 4 q4 .. + 3 of query 16 qt + l16
#pragma unroll
        for (int kt = 0; kt < 4; kt++)
#pragma unroll
            for (int qt = 0; qt < 2; qt++)
#pragma unroll
                for (int i = 0; i < 4; i++) s[kt][qt][i] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) {
#pragma unroll
            for (int qt = 0; qt < 2; qt++)
                s[j & 3][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[j & 3], qf[qt][j >> 2], s[j & 3][qt], 0, 0, 0);
            if (j + 4 < 8) ring[j & 3] = k_frag(j + 4);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);

        // V^T fragments of the first 32 output features: issued now, consumed after the softmax (the form with row
        // maxima holds more values meanwhile and requests them after it)
        bf16x4 vh[2][2][2][2];   // [half of the features][16-feature tile][32-key step][read]
        bf16x8 vf[2][2][2];
        if constexpr (DIRECT) v_frags<BUF>(vbase, vb1, vh[0]);

        if (t == nt - 1 && (a.n_kv % BKV) != 0) {
#pragma unroll
            for (int kt = 0; kt < 4; kt++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int key = t * BKV + kt * 16 + 4 * q4 + i;
                    if (key >= a.n_kv) s[kt][0][i] = s[kt][1][i] = -__builtin_inff();
                }
        }
        // the exponentiated scores of key tiles 2 ks, 2 ks + 1, rounded to bf16, are the B operand of 32-key step ks
        if constexpr (DIRECT && !PRE) {   // the multiplications still at high priority
#pragma unroll
            for (int kt = 0; kt < 4; kt++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++) s[kt][qt] *= c;
            asm volatile("" : "+v"(s[0][0]), "+v"(s[0][1]), "+v"(s[1][0]), "+v"(s[1][1]), "+v"(s[2][0]), "+v"(s[2][1]), "+v"(s[3][0]), "+v"(s[3][1]));
        }
        __builtin_amdgcn_s_setprio(0);
        bf16x8 pb[2][2];   // [32-key step][query tile]
        if constexpr (DIRECT) {
#pragma unroll
            for (int kt = 0; kt < 4; kt++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++)
#pragma unroll
                    for (int i = 0; i < 4; i++) s[kt][qt][i] = __builtin_amdgcn_exp2f(s[kt][qt][i]);
            // only the exponentials run at low priority: the conversions (and later the dot products) fill the gaps between
            // this wave's own MFMAs better than they yield to other waves (the results pass through an empty asm
            // statement, which keeps the conversions behind the change of priority)
            asm volatile("" : "+v"(s[0][0]), "+v"(s[0][1]), "+v"(s[1][0]), "+v"(s[1][1]), "+v"(s[2][0]), "+v"(s[2][1]), "+v"(s[3][0]), "+v"(s[3][1]));
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int kt = 0; kt < 4; kt++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++)
#pragma unroll
                    for (int i = 0; i < 4; i++) pb[kt >> 1][qt][4 * (kt & 1) + i] = (bf16_t)s[kt][qt][i];
        } else {
            // v_max3_f32 directly: fmaxf() makes the compiler canonicalise every MFMA output first (one extra
            // multiply per score), which costs more than the maxima themselves
            float mx[2];
#pragma unroll
            for (int qt = 0; qt < 2; qt++) {
                float m0 = max3(s[0][qt][0], s[0][qt][1], s[0][qt][2]), m1 = max3(s[2][qt][0], s[2][qt][1], s[2][qt][2]);   // two chains
                m0 = max3(m0, s[0][qt][3], s[1][qt][0]);
                m1 = max3(m1, s[2][qt][3], s[3][qt][0]);
                m0 = max3(m0, s[1][qt][1], s[1][qt][2]);
                m1 = max3(m1, s[3][qt][1], s[3][qt][2]);
                m0 = max3(m0, s[1][qt][3], s[3][qt][3]);
                // the other keys of the query are with the lanes of the other three rows of 16
                mx[qt] = max_with_other_half(max_with_other_row(max3(m0, m1, m1)));
            }
            // advance the running maxima only when one would grow by more than 2^RESCALE_LOG2
            const bool grow0 = (mx[0] - m_run[0]) * c > RESCALE_LOG2;      // first tile: m_run = -inf -> true
            const bool grow1 = (mx[1] - m_run[1]) * c > RESCALE_LOG2;
            if (__any(grow0 || grow1)) {
#pragma unroll
                for (int qt = 0; qt < 2; qt++) {
                    const float m_new = (qt ? grow1 : grow0) ? mx[qt] : m_run[qt];
                    const float corr = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * c);   // 1 where unchanged, 0 on the first tile
                    m_run[qt] = m_new;
                    l_run[qt] *= corr;
#pragma unroll
                    for (int dt = 0; dt < 4; dt++)
#pragma unroll
                        for (int i = 0; i < 4; i++) o[dt][qt][i] *= corr;
                }
            }
#pragma unroll
            for (int qt = 0; qt < 2; qt++) {
                const float mc = m_run[qt] * c;
#pragma unroll
                for (int kt = 0; kt < 4; kt++)
#pragma unroll
                    for (int i = 0; i < 4; i++)
                        pb[kt >> 1][qt][4 * (kt & 1) + i] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[kt][qt][i], c, -mc));
            }
        }

        // O^T += V^T P^T (the fragments of the other 32 features take the registers the scores leave)
        {
            unsigned vb2, vb3;   // computed here each time (two instructions) rather than kept in registers over the loop
            if constexpr (DIRECT)
                asm volatile("v_xor_b32 %0, 64, %2\n\tv_xor_b32 %1, 64, %3" : "=&v"(vb2), "=&v"(vb3) : "v"(vbase), "v"(vb1));
            else {   // (the probabilities pass through the statement: all of them are computed, and the scores' registers
                     // free, before any fragment is requested)
                asm volatile("v_xor_b32 %0, 64, %6\n\tv_xor_b32 %1, 64, %7" : "=&v"(vb2), "=&v"(vb3), "+v"(pb[0][0]), "+v"(pb[0][1]), "+v"(pb[1][0]), "+v"(pb[1][1]) : "v"(vbase), "v"(vb1));
                v_frags<BUF>(vbase, vb1, vh[0]);
            }
            v_frags<BUF>(vb2, vb3, vh[1]);
        }
        __builtin_amdgcn_s_setprio(1);
        lds_wait<8>(vh[0], vf[0]);   // (the 8 reads of the other half may still be on their way)
#pragma unroll
        for (int dd = 0; dd < 2; dd++)
#pragma unroll
            for (int ks = 0; ks < 2; ks++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++)
                    o[dd][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[0][dd][ks], pb[ks][qt], o[dd][qt], 0, 0, 0);
        const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
        for (int ks = 0; ks < 2; ks++)
#pragma unroll
            for (int qt = 0; qt < 2; qt++)
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const bf16x2 pr = {pb[ks][qt][j], pb[ks][qt][j + 1]};
                    l_run[qt] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_run[qt], false);
                }
        lds_wait<0>(vh[1], vf[1]);
#pragma unroll
        for (int dd = 0; dd < 2; dd++)
#pragma unroll
            for (int ks = 0; ks < 2; ks++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++)
                    o[2 + dd][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[1][dd][ks], pb[ks][qt], o[2 + dd][qt], 0, 0, 0);
    };
    // a query's keys are spread over the four rows of 16 lanes: its sum
    auto row_total = [&](float x) {
        x += __shfl_xor(x, 16, 64);
        return x + __shfl_xor(x, 32, 64);
    };
#define HYB_KEY_LOOP(direct_tag)                                                  \
    issue(t_begin, 0);                                                            \
    for (int t = t_begin; t < t_end; t += 2) {                                    \
        tile(t, std::integral_constant<int, 0>{}, direct_tag);                    \
        if (t + 1 < t_end) tile(t + 1, std::integral_constant<int, 1>{}, direct_tag); \
    }
    {
        // The first attempt keeps no reference maximum at all: P = 2^(c s), reference 0 (PRE: the scores are base-2
        // exponents already, c = 1 and no multiplication).  Softmax does not depend on the reference, and scaling by a power
        // of two is exact, so this is the same result as long as nothing leaves the range of fp32 / bf16; it saves the row
        // maxima, their exchange between lanes, the rescaling test and the subtraction per score.  The attempt is valid
        // when every row's sum of probabilities ends up well inside the range (then no probability that matters was flushed
        // and nothing overflowed); otherwise the whole workgroup (uniform decision through LDS, so that every wave passes
        // the same barriers) starts over with the running-maximum form.
        m_run[0] = m_run[1] = 0.f;
        HYB_KEY_LOOP(std::true_type{})
        const float l_row0 = row_total(l_run[0]), l_row1 = row_total(l_run[1]);
        const bool out_of_range = !(l_row0 > 0x1p-64f && l_row0 < 0x1p+64f) || !(l_row1 > 0x1p-64f && l_row1 < 0x1p+64f);    // also true for NaN
        const int wave_bad = __any(out_of_range) ? 1 : 0;
        __syncthreads();                                     // every wave is done with the tile buffers
        volatile int* flags = reinterpret_cast<volatile int*>(&smem[0][0]);
        if (lane == 0) flags[wave] = wave_bad;
        __syncthreads();                                     // (waits for the LDS write before the barrier)
        const bool again = (flags[0] | flags[1] | flags[2] | flags[3]) != 0;
        __syncthreads();                                     // the flags are read before the buffers are refilled
        if (again) {
            m_run[0] = m_run[1] = -__builtin_inff();
            l_run[0] = l_run[1] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 4; dt++)
#pragma unroll
                for (int qt = 0; qt < 2; qt++)
#pragma unroll
                    for (int i = 0; i < 4; i++) o[dt][qt][i] = 0.f;
            HYB_KEY_LOOP(std::false_type{})
        }
    }
#undef HYB_KEY_LOOP

    const float l_tot[2] = {row_total(l_run[0]), row_total(l_run[1])};
    // What the stores below need of the lane is derived here again, from a lane index the compiler cannot trace back
    // (an empty asm statement): row numbers and output addresses computed ahead of the key loop would have to live
    // through it in registers that the loop needs, or in scratch memory.
    int lane_e = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(lane_e));
    const int q4_e = lane_e / 16;
    const int qrow_e = qb * BQ + wave * 32 + lane_e % 16;   // second row: + 16
    if (nparts > 1) {   // partial result of a split unit: merged by attention_merge_kernel
        float* dst = a.part + ((size_t)unit * nparts + part) * PART_FLOATS + wave * 64 + lane_e;
#pragma unroll
        for (int qt = 0; qt < 2; qt++) {
            if (qrow_e + 16 * qt >= a.n_q) continue;
#pragma unroll
            for (int dt = 0; dt < 4; dt++)
#pragma unroll
                for (int i = 0; i < 4; i++) dst[((dt * 2 + qt) * 4 + i) * 256] = o[dt][qt][i];
            dst[(32 + qt) * 256] = m_run[qt];
            dst[(34 + qt) * 256] = l_tot[qt];
        }
        return;
    }
    const int hd = a.heads * 64;
#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
        const int qr = qrow_e + 16 * qt;
        if (qr >= a.n_q) continue;
        const float inv = 1.0f / l_tot[qt];
        bf16_t* orow;
        if (qr < a.split) orow = static_cast<bf16_t*>(a.o) + ((size_t)b * a.split + qr) * hd;
        else orow = static_cast<bf16_t*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (qr - a.split)) * hd;
        orow += h * 64 + 4 * q4_e;
#pragma unroll
        for (int dt = 0; dt < 4; dt++) {
            bf16x4 ov = {(bf16_t)(o[dt][qt][0] * inv), (bf16_t)(o[dt][qt][1] * inv),
                         (bf16_t)(o[dt][qt][2] * inv), (bf16_t)(o[dt][qt][3] * inv)};
            *reinterpret_cast<bf16x4*>(orow + dt * 16) = ov;
        }
    }
}

// Merges the parts of the split tail units (one workgroup per unit, threads as in the main kernel, two query rows per
// thread): with reference maxima m_p, normalisers l_p and accumulators o_p, the row is sum_p o_p 2^((m_p - M) c) over
// sum_p l_p 2^((m_p - M) c), M = max_p m_p; parts in index order.
template <int PARTS>
__global__ __launch_bounds__(256) void attention_merge_kernel(AttnArgs a) {
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int l16 = lane % 16, q4 = lane / 16;
    const int qblocks = (a.n_q + BQ - 1) / BQ;
    const int unit = blockIdx.x, xcd = unit / a.tail_units, t = unit % a.tail_units;
    const int pair = xcd + 8 * (t / a.tail_per_pair), qb = qblocks - a.tail_per_pair + t % a.tail_per_pair;
    const int h = pair % a.heads, b = pair / a.heads;
    const int qrow0 = qb * BQ + wave * 32 + l16;   // second row: + 16
    if (qrow0 >= a.n_q) return;
    const float c = a.prescaled ? 1.f : a.scale * 1.4426950408889634f;
    const float* src = a.part + (size_t)unit * PARTS * PART_FLOATS + tid;
    // everything this thread needs, requested at once (the slots of a row beyond n_q were never written: read, not used)
    float val[PARTS][36];
#pragma unroll
    for (int p = 0; p < PARTS; p++)
#pragma unroll
        for (int i = 0; i < 36; i++) val[p][i] = src[p * PART_FLOATS + i * 256];
    const int hd = a.heads * 64;
#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
        const int qrow = qrow0 + 16 * qt;
        if (qrow >= a.n_q) continue;
        float m_all = val[0][32 + qt];
#pragma unroll
        for (int p = 1; p < PARTS; p++) m_all = fmaxf(m_all, val[p][32 + qt]);
        float w[PARTS], l = 0.f;
#pragma unroll
        for (int p = 0; p < PARTS; p++) {
            w[p] = __builtin_amdgcn_exp2f((val[p][32 + qt] - m_all) * c);
            l = fmaf(val[p][34 + qt], w[p], l);
        }
        const float inv = 1.0f / l;
        bf16_t* orow;
        if (qrow < a.split) orow = static_cast<bf16_t*>(a.o) + ((size_t)b * a.split + qrow) * hd;
        else orow = static_cast<bf16_t*>(a.o2) + ((size_t)b * (a.n_q - a.split) + (qrow - a.split)) * hd;
        orow += h * 64 + 4 * q4;
#pragma unroll
        for (int dt = 0; dt < 4; dt++) {
            float r[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float acc = 0.f;
#pragma unroll
                for (int p = 0; p < PARTS; p++) acc = fmaf(val[p][(dt * 2 + qt) * 4 + e], w[p], acc);
                r[e] = acc * inv;
            }
            bf16x4 ov = {(bf16_t)r[0], (bf16_t)r[1], (bf16_t)r[2], (bf16_t)r[3]};
            *reinterpret_cast<bf16x4*>(orow + dt * 16) = ov;
        }
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
