// Host-side launch interface of the score chain that starts from hidden states and projection
// weights (Eq. 1 / Eq. 5 as written), bf16 or fp32 inputs.  Every launcher enqueues on the given stream
// and returns hipGetLastError().
#pragma once
#include "launch.hpp"

namespace vscan {

constexpr int kFusedQtPlanes = 3;  // bf16 planes carrying the hidden-space query (all 24 bits)
struct FusedArgs {
    int is_bf16 = 1;           // element type of hidden, w_q, w_k_t (else fp32)
    const void *hidden;        // [B, S, Dh]; visual tokens are rows vis_start .. vis_start+V
    const void *w_q;           // [Hq*dh, Dh]   rows = output features
    const void *w_k_t;         // [Dh, Hkv*dh]  rows = input features
    float *c_q;                // [ks_q][B*Tq][Hq*dh] partial sums of q
    uint16_t *q_planes;        // bf16 inputs: [3][B*Tq][Hq*dh] bf16; fp32 inputs: [B*Tq][Hq*dh] floats
    uint16_t *qt_planes;       // bf16 inputs: [kFusedQtPlanes][Hkv][B*(Hq/Hkv)*Tq][Dh] bf16; fp32
                               // inputs: [Hkv][B*(Hq/Hkv)*Tq][Dh] floats
    float *c_l;                // [ks_l][B][Hq*Tq][nk] partial sums of the unscaled logits; the
                               // first slot becomes the softmax weights
    float *part;               // [B][V] sums over the query rows
    int B, S, Dh, Hq, Hkv, dh, Tq, vis_start, V, k0, nk;
    int q_row0;                // first of the Tq query rows of a sequence
    int causal;                // query position t sees all but the last Tq-1-t keys of the domain
    // ragged batch (device table, else NULL): a sequence's query rows are its own last Tq rows,
    // its key domain is its visual span, or with `causal` its whole length; S, V, nk are then
    // capacities (tensor strides)
    const SeqMeta *meta = nullptr;
    int ks_q, ks_l;            // shares of the contraction axis (fused_ksplit)
    float scale;
};
// shares of the contraction axis for a contraction of Z problems of rows_s x rows_p outputs
int fused_ksplit(int rows_s, int rows_p, int Z, int k_elems, int elem_bytes);
hipError_t launch_fused_q(const FusedArgs &a, hipStream_t s);
hipError_t launch_fused_split_q(const FusedArgs &a, hipStream_t s);
hipError_t launch_fused_qt(const FusedArgs &a, hipStream_t s);
hipError_t launch_fused_logits(const FusedArgs &a, hipStream_t s);
hipError_t launch_fused_softmax(const FusedArgs &a, hipStream_t s);
hipError_t launch_fused_colsum(const FusedArgs &a, hipStream_t s);

// Mean-attention scoring (last sentence of "Global Scan") from hidden states: every token is a
// query, so Q and K are projected outright - out[bc][h][t][e] = sum_k hidden[bc][t][k] *
// w[h*dh + e][k], fp32, in the layout the mean-attention kernels read - and those kernels run
// on the result.  `w` has its rows along the output features; W_K arrives the other way round
// and is transposed first.
struct ProjectArgs {
    int is_bf16 = 1;      // element type of hidden and w (else fp32)
    const void *hidden;   // [BC, S, Dh]
    const void *w;        // [H*dh, Dh]
    float *out;           // [BC, H, S, dh]
    int BC, S, Dh, H, dh;
};
hipError_t launch_fused_project(const ProjectArgs &a, hipStream_t s);
// out[c][r] = in[r][c], elements of 2 or 4 bytes
hipError_t launch_transpose(const void *in, void *out, int rows, int cols, int elem_bytes,
                            hipStream_t s);

}  // namespace vscan
