// Kernel argument blocks and launchers of the gfx950 path.  Filled in by the C-ABI layer after it
// has validated the caller's descriptor; every launcher only enqueues work on `stream`.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mae {

// ---- per-sample parameters + masking order -----------------------------------------------------
struct ParamArgs {
  int32_t B, L, K, noise_bits;
  uint32_t sample_base;
  uint64_t key1;                      // batch_key(seed, batch_index)
  double scale_lo, scale_span;        // area fraction = lo + span * u
  double ln_ratio_lo, ln_ratio_span;  // ln(width/height) = lo + span * u (logs taken on the host)
  double ratio_lo, ratio_hi;          // for the fallback box
  float flip_p;
  int64_t images_bytes;
  const int64_t* offsets;
  const int32_t* heights;
  const int32_t* widths;
  uint8_t* mask;
  int32_t* ids_restore;
  int32_t* ids_keep;   // nullable
  int32_t* crop_out;   // nullable, [B,6]
  uint8_t* workspace;  // header + CropRec[B]
  void* aug_out;       // nullable: AugParams[B], the finetuning augmentation's draws per sample
  float jitter;
};
hipError_t launch_params_mask(const ParamArgs& a, hipStream_t stream);

// ---- crop + resize + flip + normalise + patchify + gather --------------------------------------
struct CropArgs {
  int32_t B, S, p, G, L, K, D;
  int32_t visible_bf16;  // 0: float, 1: bfloat16
  int32_t tile_pixels;   // staging tile of the resampling kernel, in 4-byte pixel words
  int32_t col_parts;     // column parts a row of patches is split into
  int32_t part_patches;  // patches per part (upper bound)
  float nscale[3];       // 1 / (255 std_c)
  float nbias[3];        // -mean_c / std_c
  const uint8_t* images;
  int64_t images_bytes;
  const int64_t* offsets;
  const int32_t* widths;
  const int32_t* ids_restore;
  const uint8_t* workspace;
  void* visible;
  float* target;    // nullable
  uint8_t* u8_out;  // the rounded 8-bit patch rows [B, L, D] of the images that the blur kernel takes
  // finetuning augmentation as this kernel's epilogue (launch_crop_aug): grayscale and
  // solarisation are applied to the rounded value in registers, blur images go to u8_out
  int32_t aug_mode;       // 1: "3 Aug", 2: "3 Aug+"
  float jitter;
  uint32_t sample_base;
  uint64_t key1;
  double* luma_partials;  // "3 Aug+": [B * G * col_parts] sums of luma after the brightness step
  const void* aug_recs;   // AugParams[B], written by the parameter kernel
  // the loss as the kernel's epilogue (launch_crop_loss): nothing above from `visible` on is used
  const void* pred;     // [B, L, D]
  void* grad;           // [B, L, D], nullable
  const uint8_t* mask;  // [B, L]
  double* partials;     // crop_loss_partials() doubles
  float* loss_out;      // [1]
  double inv_count;     // 1 / (D * M)
  float eps, gscale;
  int32_t pred_bf16, norm_pix;
  // when set, the number of masked patches is the sum of these partial counts (launch_mask_count)
  // and gscale / inv_count are derived from it on the device: gscale = gscale_num * inv_count
  const int32_t* counts;
  int32_t ncounts;
  double gscale_num;  // 2 * grad_scale
  // outputs of a sample that cannot be used are set to their neutral values by the resampling
  // kernel: mask row 0, identity order, zero pixels (all four pointers nullable)
  uint8_t* mask_out;
  int32_t* order_out;
  int32_t* keep_out;
  int32_t* crop_out;  // [B, 6]: zeros for such a sample
};
struct CropPlan {
  int col_parts, part_patches, tile_pixels;
};
CropPlan crop_plan(int S, int p, int max_side, int force_parts);
size_t crop_lds_bytes(const CropArgs& a);
hipError_t launch_crop_patch(const CropArgs& a, hipStream_t stream);
// The same with the finetuning augmentation's pointwise operations as the epilogue.  pass 0: the
// only pass of "3 Aug" / the first pass of "3 Aug+" (luma sums, nothing stored but the 8-bit rows
// of blur images); pass 1: the second pass of "3 Aug+".
hipError_t launch_crop_aug(const CropArgs& a, int pass, hipStream_t stream);
int64_t crop_loss_partials(const CropArgs& a);  // doubles of workspace
// the loss kernel, then the sum of its partials in a fixed order -> a.loss_out
hipError_t launch_crop_loss(const CropArgs& a, hipStream_t stream);

// ---- finetuning augmentation on the 8-bit resized crop ("3 Aug", "3 Aug+") ------------------------
struct AugArgs {
  int32_t B, S, p, G, L, K, D;
  int32_t visible_bf16;
  int32_t mode;  // 1: one of grayscale / solarise / blur; 2: the same followed by colour jitter
  float jitter;  // strength of the colour jitter (factors uniform on 1 +- jitter)
  uint32_t sample_base;
  uint64_t key1;
  float nscale[3];
  float nbias[3];
  int32_t blur_parts;         // column parts a row of patches is split into by the blur kernel
  int32_t blur_part_patches;  // patches per part (upper bound)
  const uint8_t* u8;          // [B, L, D] bytes: the rounded resized crop in patch order
  const int32_t* ids_restore;
  const uint8_t* workspace;  // header + CropRec[B] (valid flags)
  const void* aug_recs;      // AugParams[B], written by the parameter kernel
  double* partials;          // [B * G * blur_parts] luma sums of the blur images, mode 2
  void* visible;
  float* target;  // nullable
};
struct AugPlan {
  int parts, part_patches;
  size_t lds_bytes;
};
AugPlan three_aug_plan(int S, int p);
// The blur images of a batch.  reduce: only their luma sums after the brightness step ("3 Aug+").
hipError_t launch_aug_blur(const AugArgs& a, bool reduce, hipStream_t stream);

// ---- crop decode of baseline JPEG files ----------------------------------------------------------
struct JpegRec {
  int32_t H, W;
  int32_t hs;               // luma sampling factor (1 or 2, both directions)
  int32_t restart;          // restart interval in MCUs
  int32_t mcux, mcuy;       // MCUs per row / rows of MCUs
  int32_t scan_off, size;   // first entropy-coded byte, file length
  int32_t valid;
  int32_t dc_off[2], ac_off[2], q_off[2];  // luma, chroma: offsets of the table bodies in the file
  int32_t region_h;  // rows of the decoded region (set by the decode kernel)
};
static_assert(sizeof(JpegRec) == 64, "JpegRec is 64 bytes");
struct JpegArgs {
  int32_t B;
  int32_t slot_side;  // the decoded-region buffer holds slot_side^2 * 3 bytes per image
  const uint8_t* files;
  int64_t files_bytes;
  const int64_t* offsets;
  const int32_t* sizes;
  JpegRec* recs;
  int32_t* heights;
  int32_t* widths;
  int64_t* region_offsets;
  int32_t* region_widths;
  uint8_t* prepared; // per image: Huffman and quantiser tables, crop geometry
  uint8_t* row_states;  // per image max_rows records of 32 bytes: where the crop's rows start
  int32_t max_rows;     // rows of MCUs an image of the largest side allowed can have
  uint8_t* planes;   // decoded Y, Cb, Cr planes, one slot per image like `regions`
  uint8_t* regions;
  uint8_t* workspace;  // header + CropRec[B]
  int32_t* crop_out;   // nullable, [B,6]: the valid flag is cleared for files that cannot be used
  // nullable: per image max_rows row states for rows of MCUs 0, 1, ... of the whole file, as an
  // earlier index run left them (the caller's memory: checked before use)
  const uint8_t* row_index;
  int32_t whole_image;  // index run: every row of every file is wanted, there are no crop records
};
size_t jpeg_prepared_bytes();  // per image, in the workspace
size_t jpeg_row_state_bytes();  // per row of MCUs, in the workspace
hipError_t launch_jpeg_header(const JpegArgs& a, hipStream_t stream);
hipError_t launch_jpeg_decode(const JpegArgs& a, hipStream_t stream);
// Index run (after launch_jpeg_header): the row states of every row of MCUs of every file go to
// a.row_states; nothing is decoded.
hipError_t launch_jpeg_index(const JpegArgs& a, hipStream_t stream);

// ---- normalised-pixel loss ---------------------------------------------------------------------
struct LossArgs {
  int64_t rows;  // B * L
  int32_t D;
  int32_t pred_bf16;
  int32_t norm_pix;  // 1: per-patch normalised target, 0: target as it is
  float eps;
  float gscale;      // grad_scale * 2 / (D * M)
  double inv_count;  // 1 / (D * M)
  const void* pred;
  const float* target;
  const uint8_t* mask;
  void* grad;        // nullable
  float* loss;
  double* partials;  // workspace: one per wavefront of the grid
  int32_t num_partials;
  int32_t rows_per_iter;  // adjacent rows a wavefront handles per pass (1 or 2)
  int32_t pair_groups;    // non-zero: the two rows as one run of groups, this many per lane
  // when set: M = sum of these partial counts, gscale = gscale_num / (D M), inv_count = 1 / (D M)
  const int32_t* counts;
  int32_t ncounts;
  double gscale_num;  // 2 * grad_scale
};
// Partial counts of the non-zero bytes of mask[0 .. rows): returns how many were written (<= 256).
int mask_count_blocks(int64_t rows);
hipError_t launch_mask_count(const uint8_t* mask, int64_t rows, int32_t* counts,
                             hipStream_t stream);
struct LossShape {
  int waves;          // wavefronts of the grid = number of partials
  int rows_per_iter;
  int pair_groups;
};
LossShape loss_shape(int64_t rows, int D, bool pred_bf16);
hipError_t launch_normpix_loss(const LossArgs& a, hipStream_t stream);
// loss[0] = inv_count * (sum of n partials, added in a fixed order); with counts given,
// inv_count = 1 / (D * sum of the counts)
hipError_t launch_loss_finish(const double* partials, int n, double inv_count, float* loss,
                              const int32_t* counts, int ncounts, int D, hipStream_t stream);

// ---- patch embedding of the visible tokens -----------------------------------------------------
struct EmbedArgs {
  int64_t M;  // B * K token rows
  int32_t D, E, L;
  int32_t out_bf16;
  const void* visible;      // [M, D] bf16
  const int32_t* ids_keep;  // [M], nullable when pos is null
  const void* weight;       // [E, D] bf16
  const float* bias;        // [E], nullable
  const float* pos;         // [L, E], nullable
  void* tokens;             // [M, E] bf16 or float
};
hipError_t launch_patch_embed(const EmbedArgs& a, hipStream_t stream);

}  // namespace mae
