// Descriptor tables of the tile-grid product kernels.
//
// A "task" is one tile of C (section 2: a task touches a few tiles); its "chunks"
// are the (A tile, B tile) pairs along the contracted axes whose products are
// summed into it (section 3, linear layer: products and sums of elementary
// tiles).  One workgroup owns one macro-tile of one C tile for one batch member
// and walks the task's chunks, so the whole sum over the contracted tiles stays
// in the fp32 accumulators and is rounded once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nnt {

struct GemmTask {
    void* C;
    const float* bias;      // length m, or nullptr
    int64_t ldc, strideC;   // elements
    int32_t m, n;
    int32_t chunk0, nchunk;
    int32_t partial;        // 1: one k-slice of a split product; C is an fp32 scratch tile that receives the raw sum
    int32_t nb1;            // > 0: batch member `bat` is the pair (bat % nb1, bat / nb1) and the second index moves the
                            // operands and C by their second strides (attention products on tensors that keep the heads
                            // side by side along their first axis: the pair is (batch member, head)); 0: one stride
    int64_t cin_off;        // the beta term is read at C + cin_off (elements of C's type): 0 = from C itself, else from
                            // the tile of a second tensor with C's geometry (a residual input)
    int64_t strideC2;       // elements
    int32_t epi;            // 0, or an activation applied on the way out (GemmEpi mode | GELU variant << 4) by the kernels
                            // built for it; beta is not used then
};

// Activations of the result path (section 3: the activation follows the first linear layer of the MLP and its
// derivative multiplies what the second one's adjoint yields).  Both use the tile of a second tensor with C's
// geometry at C + cin_off.  Only the fp32 direct-load kernels have these forms: their result path has matrix
// work of other workgroups to hide behind, while the bf16 kernels, eight times faster per flop, showed the
// activation's arithmetic in full (slower than a pass of its own over the stored result).
enum GemmEpi {
    kEpiNone = 0,
    kEpiGeluOut = 1,      // C = alpha A B + bias, and gelu(C) is stored at C + cin_off
    kEpiGeluGradMul = 2   // C = (alpha A B + bias) * gelu'(x), x read at C + cin_off
};

struct GemmChunk {
    const void* A;
    const void* B;
    int64_t lda, ldb, strideA, strideB;   // elements
    int32_t k;
    int32_t vec_ok;         // bit 0: A may be read with 16-byte vectors, bit 1: B
    int64_t strideA2, strideB2;           // second batch strides (see GemmTask::nb1), elements
};

struct GemmWg {
    int32_t task, m0, n0, batch;
};

struct GemmArgs {
    const GemmTask* tasks;
    const GemmChunk* chunks;
    const GemmWg* wgs;      // nullptr: single product described by one_task / one_chunk
    GemmTask one_task;
    GemmChunk one_chunk;
    int32_t grid_m, grid_n; // macro-tile grid of the single product
    float alpha, beta;
};

// Macro-tile configurations.  M counts rows of C (first, fastest axis), N columns.
enum GemmCfg {
    kCfgSquare = 0,   // f32 128 x 128, bf16 256 x 256
    kCfgMid = 1,      // f32 64 x 128, bf16 128 x 128
    kCfgSkinny64 = 2, // 64 x 256   (attention products with m = head size 64)
    kCfgSkinny128 = 3, // 128 x 256  (head size 128)
    kCfgSkinny64n128 = 4, // 64 x 128
    kCfgSkinny64n64 = 5,  // 64 x 64   (the two narrower shapes give memory-bound products more workgroups)
    kCfgTall = 6,         // bf16 256 x 128 (two workgroups per compute unit); f32 128 x 128
    kCfgWide = 7,         // bf16 128 x 128, four waves side by side (products with at most 128 rows: m = head size); f32 128 x 256
    kCfgResident = 8      // f32 64 x 128 for contractions of at most 64 (k = head size: the score-shaped products) with both
                          // operands k-contiguous: the whole contraction sits in LDS at once, three workgroups per compute unit
};

inline void gemm_cfg_tile(int dtype_is_bf16, int cfg, int* bm, int* bn) {
    switch (cfg) {
        case kCfgSquare: *bm = *bn = dtype_is_bf16 ? 256 : 128; break;
        case kCfgMid: *bm = dtype_is_bf16 ? 128 : 64; *bn = 128; break;
        case kCfgSkinny64: *bm = 64; *bn = 256; break;
        case kCfgSkinny64n128: *bm = 64; *bn = 128; break;
        case kCfgSkinny64n64: *bm = 64; *bn = 64; break;
        case kCfgTall: *bm = dtype_is_bf16 ? 256 : 128; *bn = 128; break;
        case kCfgWide: *bm = 128; *bn = dtype_is_bf16 ? 128 : 256; break;
        case kCfgResident: *bm = dtype_is_bf16 ? 128 : 64; *bn = 128; break;
        default: *bm = 128; *bn = 256; break;
    }
}

int32_t launch_gemm_f32(hipStream_t st, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg);
int32_t launch_gemm_bf16(hipStream_t st, int out_is_f32, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg);
// 256 x 256 (kCfgSquare) or 256 x 128 (kCfgTall) macro-tiles that lie wholly inside their C tile, with 16-byte aligned operands and
// chunk lengths that are multiples of 64 (kCfgSquare) or 32 (kCfgTall); loads go straight to LDS.  `ragged` (kCfgTall only):
// macro-tiles may end inside their C tile (row-contiguous operands: at a multiple of 8 rows) and chunk lengths are multiples of 8.
// kCfgWide: 128 x 128 macro-tiles, always under the rules of `ragged`.
int32_t launch_gemm_bf16_dl(hipStream_t st, int out_is_f32, int akf, int bkf, int cfg, bool ragged, const GemmArgs& g, int64_t nwg);
int gemm_bf16_dl_occupancy(int out_is_f32, int akf, int bkf, int cfg);
// fp32: 128 x 128 (kCfgSquare) or 64 x 128 (kCfgMid, kCfgSkinny64n128, kCfgResident) macro-tiles that lie wholly inside their
// C tile, 16-byte aligned operands, chunk lengths that are multiples of 32.  kCfgResident: one chunk of 32 or 64 per task,
// A read transposed and B as [k, n] (both k-contiguous)
// `epi_mode` (a GemmEpi mode, 0 for the plain product) picks the kernels with an activation on the result path; they exist
// for the forms gemm_f32_dl_has_act names.
int32_t launch_gemm_f32_dl(hipStream_t st, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg, int epi_mode = 0);
bool gemm_f32_dl_has_act(int akf, int bkf, int epi_mode);
int gemm_f32_dl_occupancy(int akf, int bkf, int cfg);
// workgroups of the kernel instance that a compute unit holds at a time (registers, LDS)
int gemm_f32_occupancy(int akf, int bkf, int cfg);
int gemm_bf16_occupancy(int out_is_f32, int akf, int bkf, int cfg);

}  // namespace nnt
