// Internal attention interface of libhyb: o = softmax(q k^T * scale) v per (batch, head), head_dim 64.
#pragma once
#include "common.h"

struct AttnArgs {
    const void* q;   // [batch, heads, n_q, 64]
    const void* k;   // [batch, heads, n_kv, 64]
    const void* v;   // [batch, heads, n_kv, 64]
    void* o;         // [batch, split, heads * 64]: query rows [0, split)
    void* o2;        // [batch, n_q - split, heads * 64]: query rows [split, n_q) (joint attention hands the
                     // image and text rows back to their own streams); nullptr when split == n_q
    int split;
    int batch, heads, n_q, n_kv;
    float scale;     // > 0
    int q_stride;    // query rows stored per (batch, head) in q (>= n_q); 0 means n_q.  A larger stride lets a
                     // launch serve only the first n_q rows of a longer sequence (image-only queries over joint keys)
    int prescaled;   // q already carries scale x log2(e) (the QKV epilogue of the joint block stores it so): the kernel
                     // then exponentiates the raw scores in base 2 and `scale` is not used
    float* part;     // scratch of hyb_attention_split_bytes() for the MFMA kernel's split tail, or nullptr (no splitting)
    // set by the launcher:
    int tail_from, tail_units, tail_parts, tail_per_pair;
};

// Scratch the bf16 MFMA kernel wants for its split tail (see attention_mfma.hip); 0 when it would not split.
size_t hyb_attention_split_bytes(int batch, int heads, int n_q);

// Plain kernel (fp32 or bf16 storage, fp32 math with accurate expf).
int hyb_launch_attention_simple(const AttnArgs& a, hyb_dtype dtype, hipStream_t st);
// bf16 flash-style MFMA kernel.
int hyb_launch_attention_mfma(const AttnArgs& a, hipStream_t st);
int hyb_launch_attention(const AttnArgs& a, hyb_dtype dtype, hipStream_t st);
