// What the max-plus (Viterbi) kernels of lccrf_viterbi.hip and lccrf_lane_max.hip share: the arguments of a
// launch, the stretch of positions a pair of workgroups serves, and the tie rule of a step.
#pragma once
#include "lccrf_device.h"

namespace lccrf {

constexpr int kNoArg = 0x7fffffff;

__device__ __forceinline__ void take_better(double& v, int& a, double pv, int pa) {
    if (pv > v || (pv == v && pa < a)) { v = pv; a = pa; }
}

struct VitArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    uint8_t* bp;   // [B][N][T] back-pointers (rows <= meeting point) and forward pointers (rows above it)
    double* mid;   // [B][C][2][T] delta and eps at the meeting point
    float* best_score;
    int32_t* tags;
    // Chunked schedule (chunk > 0): workgroup pair v serves chunk c = v % C of sequence v / C, the
    // tag positions [c chunk, (c+1) chunk), as a chain of its own that starts one position earlier in
    // the tag pin[b][c-1] and must end in the tag pin[b][c] (both chosen by the max-plus scan,
    // lccrf_scan.hip); the best score is the scan's and is not written here.
    int chunk, C;
    const int32_t* pin;  // [B][C] tag at the last position of each chunk
    // Structured potentials (emit non-null; float, T <= 64): phi[b][i][s][t] = trans[s][t] + emit[b][i][t].
    const float* emit;   // [B][N][T]
    const float* trans;  // [T][T]
};

// The stretch of positions one pair of workgroups handles.
struct VitSpan {
    int b, c, L;
    int t0, t1;  // tag positions [t0, t1) whose tags this span writes (before the cut at L)
    int p0, e;   // first and last position of the chain
    bool empty;
};
__device__ __forceinline__ VitSpan vit_span(const VitArgs& a, int v) {
    VitSpan s;
    const bool chunked = a.chunk > 0;
    s.b = chunked ? v / a.C : v;
    s.c = chunked ? v % a.C : 0;
    s.L = clamp_length(a.lengths, s.b, a.N);
    s.t0 = chunked ? s.c * a.chunk : 0;
    s.t1 = chunked ? (s.t0 + a.chunk < a.N ? s.t0 + a.chunk : a.N) : a.N;
    s.empty = s.t0 >= s.L;
    s.p0 = s.t0 > 0 ? s.t0 - 1 : 0;
    s.e = (s.t1 < s.L ? s.t1 : s.L) - 1;
    return s;
}

// The first maximum of val[0 .. n-1] (arg ascending with the index) ends in val[0] / arg[0]: a tree
// of pairwise comparisons in which the right-hand candidate wins only if strictly greater, so the
// chain of dependent instructions is log2 n long instead of n.
template <int n>
__device__ __forceinline__ void first_max_tree(double (&val)[n], int (&arg)[n]) {
#pragma unroll
    for (int w = 1; w < n; w <<= 1)
#pragma unroll
        for (int k = 0; k + w < n; k += 2 * w)
            if (val[k + w] > val[k]) { val[k] = val[k + w]; arg[k] = arg[k + w]; }
}

// The two chains of every span by a chain wave and its helper waves (lccrf_lane_max.hip; plain potentials, up to
// 64 tags): pointers in bp, the two vectors of the meeting point in mid, as the kernels of lccrf_viterbi.hip
// leave them for the trace.
hipError_t launch_lane_max_chains(int dtype, const VitArgs& a, int poll_limit, hipStream_t st);

}  // namespace lccrf
