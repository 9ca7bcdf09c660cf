// Construction of syntax-enriched training labels (paper Section III-C, Fig. 3): from the base
// model's label row L_0 (token ids with a [FRAG] id at every fragment boundary) to the
// (num_heads + 1) x sequence_length matrix whose row i is L_0 shifted left by i and filled up
// with [PAD], with every entry that lies beyond the column's last [FRAG] replaced by [IGNORE].
//
// The work is one read of L_0 and one write of the matrix: HBM-bound, no reuse beyond the
// num_heads-wide window each column looks at. A workgroup stages LB_TILE + num_heads entries of
// L_0 in LDS once; thread t owns the columns t, t + 256, t + 512, t + 768 of the tile (LDS reads
// of a wave hit 64 consecutive words, global stores of a wave cover 256 contiguous bytes of a row).
#include "sd_internal.h"

#define LB_THREADS 256
#define LB_COLS 4
#define LB_TILE (LB_THREADS * LB_COLS)

// grid: x = tile of LB_TILE sequence positions, y = sequence
__global__ __launch_bounds__(LB_THREADS) void k_build_labels(const int32_t* __restrict__ l0, int S, int H, int32_t frag,
                                                             int32_t pad, int32_t ignore, int keep_all,
                                                             int32_t* __restrict__ labels) {
    __shared__ int32_t tile[LB_TILE + SD_LABELS_MAX_HEADS];
    const int b = blockIdx.y, s0 = blockIdx.x * LB_TILE, tid = threadIdx.x;
    const int32_t* row = l0 + (size_t)b * S;
    for (int i = tid; i < LB_TILE + H; i += LB_THREADS) {
        const int s = s0 + i;
        tile[i] = s < S ? row[s] : pad;                 // positions past the end read as [PAD]
    }
    __syncthreads();
    int last[LB_COLS];
#pragma unroll
    for (int c = 0; c < LB_COLS; ++c) last[c] = -1;
    for (int i = 0; i <= H; ++i) {
#pragma unroll
        for (int c = 0; c < LB_COLS; ++c)
            if (tile[c * LB_THREADS + tid + i] == frag) last[c] = i;
    }
#pragma unroll
    for (int c = 0; c < LB_COLS; ++c)
        if (last[c] < 0) last[c] = keep_all ? H : 0;    // a column without any [FRAG]
    for (int i = 0; i <= H; ++i) {
        int32_t* dst = labels + ((size_t)b * (H + 1) + i) * S + s0;
#pragma unroll
        for (int c = 0; c < LB_COLS; ++c) {
            const int col = c * LB_THREADS + tid;
            if (s0 + col < S) dst[col] = i <= last[c] ? tile[col + i] : ignore;
        }
    }
}

void launch_build_labels(const int32_t* l0, int B, int S, int H, int32_t frag, int32_t pad, int32_t ignore,
                         int keep_all, int32_t* labels, hipStream_t s) {
    hipLaunchKernelGGL(k_build_labels, dim3((S + LB_TILE - 1) / LB_TILE, B), dim3(LB_THREADS), 0, s, l0, S, H, frag, pad,
                       ignore, keep_all, labels);
}
