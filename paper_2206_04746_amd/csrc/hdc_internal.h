// Internal declarations shared by the HIP translation units of libhdc (gfx950 only).
// Nothing here is part of the public C ABI; see include/hdc.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hdc.h"

namespace hdc {

constexpr int kWave = 64;         // CDNA4 wavefront width
constexpr int kSliceWords = 64;   // one 32-bit word column per lane: a wave owns 64 words
constexpr int kFeatBlock = 16;    // features consumed per carry-save tree in encode

// Device-side copy of the model: everything the kernels need, laid out for them.
struct hdc_ctx_impl {
    hdc_params p;
    int device;
    int num_cus;      // compute units of the device (sizes the persistent encode grid)
    int32_t W;        // ceil(D / 32)
    int32_t Wp;       // W rounded up to a multiple of kSliceWords (pad words are zero)
    int32_t Fp;       // rows of item_d: F, +1 tie-vote row when F is even, padded to kFeatBlock
    int32_t votes;    // F or F + 1: number of real votes per dimension (always odd)
    uint32_t last_word_mask;  // valid bits of word W-1

    // Encoding tables in device memory.  item_d holds, after the F real rows, the rows that
    // make the vote count odd and the feature count a multiple of kFeatBlock:
    //   row F (only if F is even) = tie XOR level[0]   -> binds with level 0 to the tie vector
    //   remaining pad rows        = level[0]           -> bind with level 0 to all-zero votes
    // Both tables are stored slice-major so that a wave's 64 word columns of consecutive rows
    // are 256 bytes apart: [Wp / 64][rows][64].
    uint32_t *item_d;   // [Wp/64][Fp][64]
    uint32_t *level_d;  // [Wp/64][L][64]
    uint32_t *tie_d;    // [Wp]
    float *lo_d;        // [F]   (HDC_F32 only)
    float *scale_d;     // [F]

    // Level-invariant dimensions (Sec. III: level vectors differ from one another in only part
    // of the dimensions; with linear scaling about half never flip).  Where every level vector
    // has the same bit, the vote of a feature is item XOR level[0] whatever the feature's value:
    // the encoded bit is a constant of the model.  When enough dimensions are like that, encoding
    // runs on the other dimensions only, packed densely ("compact" tables, same layouts), and
    // expand_kernel spreads the result back and fills in the constants.
    bool compact;
    int32_t Wc, Wcp;        // words of a compact row, and padded to whole slices (Wc may be 0)
    uint32_t *citem_d;      // [Wcp/64][Fp][64]
    uint32_t *clevel_d;     // [Wcp/64][L][64]
    uint32_t *hvc_d;        // [q_rows][Wc] compact hypervectors of the chunk being encoded
    uint32_t *expand_d;     // [8][W]: bit offset into the compact row | mask of varying bits |
                            // five bit-spreading stage masks | constant bits

    // Scratch owned by the context (sized at create, never grown on the hot path).
    uint16_t *q_d;        // [q_rows][Fp] level-row offsets (bin * 256) of the samples being encoded
    int64_t q_rows;       // rows q_d can hold
    uint32_t *cls_cnt_d;  // [C + 1] per-class sample counts of the current training chunk
    uint32_t *cls_off_d;  // [C + 1] exclusive prefix of cls_cnt_d
    uint32_t *cls_cur_d;  // [C + 2] per-class totals / scatter cursors and, last, the count of finished blocks; zero between launches
    uint32_t *cls_blk_d;  // [C + 1] exclusive prefix of per-class row-block counts
    uint32_t *perm_d;     // [perm_rows] sample indices grouped by class
    int64_t perm_rows;
    uint32_t *partial_d;  // [partial_items][Wp * 16] per-block partial counts, two u16 per dword
    int64_t partial_items;
    uint32_t *on_bits_d;  // [16384][1024] per-thread sample bits of hdc_train_online (first call or hdc_reserve allocates)
    bool check_labels;    // hdc_set_label_check: training calls refuse labels outside [0, C)
    unsigned long long *bad_labels_d;   // [1] counter of count_bad_labels

    // Scratch of hdc_train_online_batched, allocated on its first call and grown when a call
    // needs more (batch size is a call argument, not a property of the model).
    double *ob_part_d;    // [slices][sub-batch][C] partial dot products
    size_t ob_part_bytes;
    void *ob_wts_d;       // [sub-batch] per-sample weight records
    size_t ob_wts_bytes;
    double *ob_coef_d;    // [sub-batch][2|4|8|16] dense signed weights (C <= 16 only)
    size_t ob_coef_bytes;
    uint64_t *ob_col_d;   // [ceil(D/64)][sub-batch] 64-bit lane masks, dimension group major
    size_t ob_col_bytes;
    double *ob_carry_d;   // [C][D] batch sum carried between the launches of a long batch
    size_t ob_carry_bytes;
    double *ob_share_d;   // [shares][C][D] sums of the blocks that share one group's samples
    size_t ob_share_bytes;
    double *ob_norm_d;    // [C][ceil(D/64)] squared-norm partials of the class rows
    size_t ob_norm_bytes;
    uint32_t *ob_ln_d;    // [C][sub-batch] per class: the samples that name it, in sample order
    size_t ob_ln_bytes;
    double *ob_lw_d;      // [C][sub-batch] ... and their signed weights
    size_t ob_lw_bytes;
    uint32_t *ob_meta_d;  // [3 C + 1 + rows] entries / first share row / share rows per class, row counter, work list
    size_t ob_meta_bytes;
    bool ob_attr_set;     // dynamic-LDS limit of the backward kernel raised

    // hdc_encode_sparse (allocated and derived on its first call)
    bool sp_ready;
    uint32_t *sp_b_d;       // [slices][Fp][64] item ^ level 0 (of the compact tables when `compact`)
    uint32_t *sp_e_d;       // [slices][L][64]  level ^ level 0
    uint32_t *sp_base_d;    // [slices][P][64]  bit-sliced counters of the all-bin-0 sample, bias included
    uint32_t *sp_fb_d;      // [q_rows][Fp]     listed features' row offsets in a slice of sp_b_d
    uint32_t *sp_blocks_d;  // [q_rows]         16-entry blocks per sample
    int sp_bpc;             // blocks of encode_sparse_kernel a CU holds (0 = not asked yet)

    // Encoding as a contraction over the features (encode_contract.hip); tables derived at create
    // when the level table is of the shape it needs.
    // A table set per way of splitting a row's words over blocks (1, 2 or 4 blocks per 32 samples:
    // few samples would leave most of the chip idle otherwise); set v splits 1 << v ways.
    bool ct_ready;
    bool ct_chained = false;   // some dimensions flip more than once: the tables carry chains, the kernel follows them
    int ct_steps;               // MFMA steps (64 features each) per tile
    int ct_min_split, ct_max_split;   // the first and last table set built (rows over 512 words are always split, rows under 4 never 4 ways)
    int ct_tiles[3];            // tiles of 32 dimensions, all word ranges together
    int ct_range_max[3];        // most tiles of one word range
    int ct_range[3][5];         // first tile of every word range, then the end of the last (repeated up to the fifth entry)
    int32_t *ct_tau_d[3];       // [tiles] the level at which the tile's dimensions flip
    uint32_t *ct_col_d[3];      // [32][W] per bit of every word of a row: (tile - its range's first) * 32 + column that holds it, ~0 for a constant bit
    float *ct_k_d[3];           // [tiles][32] the column's vote threshold, constants folded in
    uint32_t *ct_bt_d[3];       // [tiles][steps][64] item ^ level 0 along the features, per column and lane half (nibbles reversed)

    // The same contraction for long streams (encode_wide.hip): jobs of 32 * wd_groups samples, the
    // model-side operands ready-made, the vote threshold folded into the contraction.
    bool wd_ready;
    int wd_steps, wd_nb, wd_groups;   // steps of 64 feature slots per tile (two to a matrix instruction), bit planes of a bin number (6 or 8), groups of 32 samples per job
    int wd_items;               // work items: a threshold and up to five tiles of its dimensions
    int wd_tiles;               // tiles of 16 dimensions of all items together
    int wd_ovs;                 // words per group of the kernel's column array: the varying dimensions, an all-zero and an all-one word
    int32_t *wd_items_d;        // [wd_items][4] threshold, first tile, dimensions, first column
    uint32_t *wd_bx_d;          // [tiles][wd_steps / 2][64][4] model-side operands: 4-bit floats +-1 / (sample-side value), bias in the slots past F
    uint32_t *wd_src_d;         // [32][W] per bit of every word of a row: the column that holds it

    // Launch properties looked up once per context (kept here, not in function-local statics,
    // so that two contexts used from two threads share no mutable state).
    int enc_bpc[24];        // encode_kernel variant -> blocks of it a CU holds (0 = not asked yet)
    int enc_bpc_L[24];      //   ... and the level count that answer was for
    int enc_split_bpc[2];   // blocks of encode_split_kernel (8 / 16 waves) a CU holds (0 = not asked yet) ...
    int enc_split_L[2];     //   ... and the level count that answer was for
    int acc_bpc;            // blocks of accumulate_kernel a CU holds (0 = not asked yet)
    int acc_local_bpc[2];   // the same of accumulate_local_kernel with one class / with the context's classes
    bool on_attr_set[16];   // online_lds_kernel<CMAX, .>: dynamic-LDS limit raised, by CMAX

    // Optional per-kernel timing (hdc_profile_*): event pairs per hot kernel.
    bool prof_on;
    hipEvent_t *prof_ev[HDC_K_COUNT];   // [2 * HDC_PROFILE_SLOTS] start/stop interleaved
    int prof_used[HDC_K_COUNT];
};

// Brackets one kernel launch with events when profiling is enabled; otherwise does nothing.
struct ProfScope {
    hdc_ctx_impl *c;
    int id;
    hipStream_t s;
    bool live;
    ProfScope(hdc_ctx_impl *ctx, int kernel_id, hipStream_t stream)
        : c(ctx), id(kernel_id), s(stream), live(false) {
        if (c->prof_on && c->prof_ev[id] && c->prof_used[id] < HDC_PROFILE_SLOTS) {
            live = hipEventRecord(c->prof_ev[id][2 * c->prof_used[id]], s) == hipSuccess;
        }
    }
    ~ProfScope() {
        if (live && hipEventRecord(c->prof_ev[id][2 * c->prof_used[id] + 1], s) == hipSuccess)
            c->prof_used[id] += 1;
    }
};

// Records a HIP failure for hdc_last_hip_error() and maps it to HDC_EHIP.
int hip_fail(hipError_t e, const char *what);

#define HDC_HIP(call)                                        \
    do {                                                     \
        hipError_t e__ = (call);                             \
        if (e__ != hipSuccess) return ::hdc::hip_fail(e__, #call); \
    } while (0)

// Kernel launchers (one per translation unit); all only enqueue on `s`.
int launch_encode(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s);
int launch_encode_sparse(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s);
void majority_planes(const hdc_ctx_impl *c, int *P_out, uint32_t *bias_out);   // planes and start value of a vote counter
void launch_expand(hdc_ctx_impl *c, int64_t n, uint32_t *out, hipStream_t s);  // compact staging rows -> full rows
int launch_train_classical(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                           int32_t *acc, int64_t *class_n, hipStream_t s);
int launch_binarize_classical(hdc_ctx_impl *c, const int32_t *acc, const int64_t *class_n,
                              uint32_t *class_hv, hipStream_t s);
int launch_train_online(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                        int32_t epochs, float lr, float *acc, hipStream_t s);
int launch_train_online_batched(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                                int32_t epochs, float lr, int64_t batch, float *acc, hipStream_t s);
int launch_binarize_online(hdc_ctx_impl *c, const float *acc, uint32_t *class_hv, hipStream_t s);
int launch_search_cosine(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const float *acc, float *cos_out,
                         int32_t *pred, hipStream_t s);
int launch_pack(hdc_ctx_impl *c, const uint8_t *bits, int64_t N, uint32_t *hv, hipStream_t s);
int launch_unpack(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, uint8_t *bits, hipStream_t s);
int launch_hsum(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s);
int launch_vsum(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s);
// hdc_vsum without a context, its scratch in a static device array (no allocation); D <= 16384
int vsum_static(int32_t D, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s);
// Scratch that entry points otherwise allocate at their first call (hdc_reserve); no-ops when it is there.
int reserve_online(hdc_ctx_impl *c);
int reserve_online_batched(hdc_ctx_impl *c, int64_t batch);
int reserve_search_cosine(hdc_ctx_impl *c, int64_t queries);
int reserve_sparse(hdc_ctx_impl *c, hipStream_t s);
// Counts the labels outside [0, C) of a training call (hdc_set_label_check); synchronises the stream.
int count_bad_labels(hdc_ctx_impl *c, const int32_t *labels, int64_t N, hipStream_t s, int64_t *bad);
// Most partial rows one hdc_train_classical launch can produce (sizes partial_d at create).
int64_t classical_max_items(hdc_ctx_impl *c);
// Encoding as a contraction (encode_contract.hip): tables at create; the launcher returns false
// when the model or the call is not of its shape (then nothing was launched).
int prepare_contract(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, const uint32_t *tie);
bool try_encode_contract(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s, int *rc);
// The contraction for long streams (encode_wide.hip); same conventions.  prepare_wide needs the
// tables of prepare_compact.
int prepare_wide(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, const uint32_t *tie);
bool try_encode_wide(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s, int *rc);
// Hamming search on the matrix cores for long query streams with 9..31 classes; false when the
// shape is not its own (then nothing was launched and *rc is untouched).
bool try_search_mfma(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                     uint32_t *dist, int32_t *pred, hipStream_t s, int *rc);
int launch_search(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                  uint32_t *dist, int32_t *pred, hipStream_t s);

// 3-input bitwise ops of gfx950 (v_bitop3_b32); truth table index = (a<<2)|(b<<1)|c.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}
__device__ __forceinline__ uint32_t maj3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
}

}  // namespace hdc
