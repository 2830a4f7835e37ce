// C ABI of the library: host-side validation of the caller's descriptors, then kernel launches.
// No device memory is allocated here and no pointer is kept after a call.
#include "../../include/mae_hip.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>

#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace {

constexpr int kVersion = 600;  // 0.6.0

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct PrepShape {
  int32_t G, L, D;
};

// Checks everything that can be checked without touching device memory.
int validate_prep(const mae_prep_desc* d, PrepShape* shape) {
  if (!d) return MAE_ERR_NULL;
  if (d->input_format != MAE_INPUT_DECODED && d->input_format != MAE_INPUT_JPEG)
    return MAE_ERR_RANGE;
  if (!d->images || !d->offsets) return MAE_ERR_NULL;
  if (d->input_format == MAE_INPUT_DECODED && (!d->heights || !d->widths)) return MAE_ERR_NULL;
  if (d->input_format == MAE_INPUT_JPEG && !d->file_sizes) return MAE_ERR_NULL;
  // the decoder reads the files through aligned 8-byte windows
  if (d->input_format == MAE_INPUT_JPEG && !aligned(d->images, 8)) return MAE_ERR_RANGE;
  if (d->jpeg_row_index &&
      (d->input_format != MAE_INPUT_JPEG || !aligned(d->jpeg_row_index, 16)))
    return MAE_ERR_RANGE;
  if (d->jpeg_row_index && d->B > 0 && d->max_image_side >= 0 && d->max_image_side <= 32767) {
    // one 32-byte entry per 8 pixels of the side limit (rounded up to 16) and file
    const int64_t slot = ((d->max_image_side > 0 ? d->max_image_side : 256) + 15) & ~15;
    if (d->jpeg_row_index_bytes < (int64_t)d->B * (slot / 8) * 32) return MAE_ERR_WORKSPACE;
  }
  if (d->B <= 0 || d->out_size <= 0 || d->patch <= 0) return MAE_ERR_SHAPE;
  if (d->B > (1 << 20)) return MAE_ERR_RANGE;  // keeps every grid size below 2^31
  if (d->out_size % d->patch != 0) return MAE_ERR_SHAPE;
  if (d->patch > 32 || d->out_size > 512) return MAE_ERR_RANGE;
  const int64_t G = d->out_size / d->patch;
  const int64_t L = G * G;
  if (L > mae::kMaxPatches) return MAE_ERR_RANGE;
  if (d->num_keep < 1 || d->num_keep > L) return MAE_ERR_SHAPE;
  if (d->images_bytes <= 0) return MAE_ERR_RANGE;
  if (!(d->scale_lo > 0.0f) || !(d->scale_lo <= d->scale_hi) || !(d->scale_hi <= 1.0f))
    return MAE_ERR_RANGE;
  if (!(d->ratio_lo > 0.0f) || !(d->ratio_lo <= d->ratio_hi)) return MAE_ERR_RANGE;
  // the exponential of the log-ratio is a fixed polynomial, accurate for |x| <= 1/2
  if (log((double)d->ratio_lo) < -0.5 || log((double)d->ratio_hi) > 0.5) return MAE_ERR_RANGE;
  if (!(d->flip_p >= 0.0f) || !(d->flip_p <= 1.0f)) return MAE_ERR_RANGE;
  for (int c = 0; c < 3; ++c) {
    if (!(d->std[c] > 0.0f) || !isfinite(d->std[c]) || !isfinite(d->mean[c])) return MAE_ERR_RANGE;
  }
  if (d->noise_bits < 1 || d->noise_bits > 32) return MAE_ERR_RANGE;
  if ((uint64_t)d->sample_base + (uint64_t)d->B > 0x100000000ull) return MAE_ERR_RANGE;
  if (d->out_dtype != MAE_F32 && d->out_dtype != MAE_BF16) return MAE_ERR_DTYPE;
  if (d->max_image_side < 0 || d->max_image_side > 32767) return MAE_ERR_RANGE;
  if (d->aug_mode != MAE_AUG_SIMPLE && d->aug_mode != MAE_AUG_THREE &&
      d->aug_mode != MAE_AUG_THREE_PLUS)
    return MAE_ERR_RANGE;
  if (d->aug_mode != MAE_AUG_SIMPLE) {
    if (!(d->jitter >= 0.0f) || !(d->jitter <= 1.0f)) return MAE_ERR_RANGE;
    // groups of four or two pixels must tile the rows of a patch
    if (d->patch % 2 != 0) return MAE_ERR_SHAPE;
  }
  if (shape) {
    shape->G = (int32_t)G;
    shape->L = (int32_t)L;
    shape->D = 3 * d->patch * d->patch;
  }
  return MAE_OK;
}

int validate_loss(const mae_loss_desc* d, bool need_target = true) {
  if (!d) return MAE_ERR_NULL;
  if (!d->pred || (need_target && !d->target) || !d->mask) return MAE_ERR_NULL;
  if (d->B <= 0 || d->L <= 0) return MAE_ERR_SHAPE;
  if (d->D < 2 || d->D > 3072) return MAE_ERR_RANGE;
  if (d->num_masked < 0) return MAE_ERR_RANGE;  // 0: counted on the device
  if (!(d->eps >= 0.0f) || !isfinite(d->eps) || !isfinite(d->grad_scale)) return MAE_ERR_RANGE;
  if (d->pred_dtype != MAE_F32 && d->pred_dtype != MAE_BF16) return MAE_ERR_DTYPE;
  if (d->norm_pix != 0 && d->norm_pix != 1) return MAE_ERR_RANGE;
  return MAE_OK;
}

int validate_embed(const mae_embed_desc* d) {
  if (!d) return MAE_ERR_NULL;
  if (!d->visible || !d->weight) return MAE_ERR_NULL;
  if (d->pos && !d->ids_keep) return MAE_ERR_NULL;
  if (d->M <= 0 || d->D <= 0 || d->E <= 0 || d->L <= 0) return MAE_ERR_SHAPE;
  if (d->D % 4 != 0) return MAE_ERR_SHAPE;
  if (d->M > (int64_t(1) << 28) || d->D > 3072 || d->E > 8192) return MAE_ERR_RANGE;
  if (d->out_dtype != MAE_F32 && d->out_dtype != MAE_BF16) return MAE_ERR_DTYPE;
  if (!aligned(d->visible, 16) || !aligned(d->weight, 16) || (d->pos && !aligned(d->pos, 16)))
    return MAE_ERR_RANGE;
  return MAE_OK;
}

// Whether this process sees a HIP device; asked once (the answer does not change while the
// process lives) so that the launch paths do not query the runtime on every call.
int have_device() {
  static const int status = [] {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
      (void)hipGetLastError();  // do not leave a sticky error for the caller's next HIP call
      return (int)MAE_ERR_NO_DEVICE;
    }
    return (int)MAE_OK;
  }();
  return status;
}

}  // namespace

extern "C" {

int mae_version(void) { return kVersion; }

const char* mae_error_string(int status) {
  switch (status) {
    case MAE_OK: return "success";
    case MAE_ERR_NULL: return "a required pointer is NULL";
    case MAE_ERR_SHAPE: return "sizes do not fit together";
    case MAE_ERR_RANGE: return "a value is outside the supported range";
    case MAE_ERR_DTYPE: return "unknown dtype";
    case MAE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MAE_ERR_NO_DEVICE: return "no HIP device visible";
    case MAE_ERR_HIP: return "a HIP runtime call failed";
    default: return "unknown status";
  }
}

int32_t mae_num_keep(int32_t L, double mask_ratio) {
  if (L < 1 || !(mask_ratio >= 0.0) || !(mask_ratio <= 1.0)) return -1;
  return (int32_t)floor((double)L * (1.0 - mask_ratio));
}

namespace {
// Workspace: header | CropRec[B] | (augmentation) 8-bit resized crops, S * S * 3 bytes each |
// (jitter) one double per (image, row of patches, column part of the blur kernel); every part
// starts on a 256-byte boundary.
struct PrepWorkspace {
  size_t aug_offset, u8_offset, partials_offset, crop_partials_offset, total;
  // crop decode: per-file records, heights, widths, region widths, region offsets, tables, planes, regions
  size_t recs_offset, heights_offset, widths_offset, region_widths_offset, region_offsets_offset,
      prepared_offset, row_states_offset, planes_offset, regions_offset;
  int slot_side;
  int max_rows;  // rows of MCUs (8 pixels at least) of an image that fills a slot
};
// Launch plan of the resampling kernel: from the side limit of the decoded-region slots for JPEG
// input, else from the caller's hint.
mae::CropPlan crop_plan_of(const mae_prep_desc* d, int slot_side) {
  return mae::crop_plan(d->out_size, d->patch,
                        d->input_format == MAE_INPUT_JPEG
                            ? slot_side
                            : (d->max_image_side > 0 ? d->max_image_side : 256),
                        0);
}
PrepWorkspace prep_workspace(const mae_prep_desc* d) {
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  PrepWorkspace w;
  w.aug_offset = up(mae::kWorkspaceHeader + (size_t)d->B * sizeof(mae::CropRec));
  w.u8_offset = w.aug_offset;
  if (d->aug_mode != MAE_AUG_SIMPLE)
    w.u8_offset = up(w.aug_offset + (size_t)d->B * sizeof(mae::AugParams));
  w.partials_offset = w.u8_offset;
  w.crop_partials_offset = w.u8_offset;
  w.total = mae::kWorkspaceHeader + (size_t)d->B * sizeof(mae::CropRec);
  w.recs_offset = w.heights_offset = w.widths_offset = w.region_widths_offset = 0;
  w.region_offsets_offset = w.prepared_offset = w.planes_offset = w.regions_offset = 0;
  w.row_states_offset = 0;
  w.max_rows = 0;
  w.slot_side = 0;
  if (d->input_format == MAE_INPUT_JPEG)
    w.slot_side = ((d->max_image_side > 0 ? d->max_image_side : 256) + 15) & ~15;
  if (d->aug_mode != MAE_AUG_SIMPLE) {
    w.partials_offset = up(w.u8_offset + (size_t)d->B * d->out_size * d->out_size * 3);
    w.total = w.partials_offset;
    if (d->aug_mode == MAE_AUG_THREE_PLUS) {
      // luma sums per (image, row of patches, column part): of the blur kernel, then of the
      // resampling kernel
      const size_t rows = (size_t)d->B * (d->out_size / d->patch);
      w.crop_partials_offset =
          w.total + rows * mae::three_aug_plan(d->out_size, d->patch).parts * sizeof(double);
      w.total = w.crop_partials_offset +
                rows * (size_t)crop_plan_of(d, w.slot_side).col_parts * sizeof(double);
    }
  }
  if (d->input_format == MAE_INPUT_JPEG) {
    const size_t B = (size_t)d->B;
    w.recs_offset = up(w.total);
    w.heights_offset = up(w.recs_offset + B * sizeof(mae::JpegRec));
    w.widths_offset = up(w.heights_offset + B * 4);
    w.region_widths_offset = up(w.widths_offset + B * 4);
    w.region_offsets_offset = up(w.region_widths_offset + B * 8);
    w.prepared_offset = up(w.region_offsets_offset + B * 8);
    w.max_rows = w.slot_side / 8;
    w.row_states_offset = up(w.prepared_offset + B * mae::jpeg_prepared_bytes());
    w.planes_offset = up(w.row_states_offset + B * w.max_rows * mae::jpeg_row_state_bytes());
    w.regions_offset = up(w.planes_offset + B * (size_t)w.slot_side * w.slot_side * 3);
    w.total = w.regions_offset + B * (size_t)w.slot_side * w.slot_side * 3;
  }
  return w;
}
// The crop-decode kernels' view of the descriptor and the workspace.
mae::JpegArgs make_jpeg_args(const mae_prep_desc* d, const PrepWorkspace& wsl, uint8_t* ws,
                             int32_t* crop_out) {
  mae::JpegArgs ja;
  memset(&ja, 0, sizeof(ja));
  ja.B = d->B;
  ja.slot_side = wsl.slot_side;
  ja.files = d->images;
  ja.files_bytes = d->images_bytes;
  ja.offsets = d->offsets;
  ja.sizes = d->file_sizes;
  ja.recs = reinterpret_cast<mae::JpegRec*>(ws + wsl.recs_offset);
  ja.heights = reinterpret_cast<int32_t*>(ws + wsl.heights_offset);
  ja.widths = reinterpret_cast<int32_t*>(ws + wsl.widths_offset);
  ja.region_offsets = reinterpret_cast<int64_t*>(ws + wsl.region_offsets_offset);
  ja.region_widths = reinterpret_cast<int32_t*>(ws + wsl.region_widths_offset);
  ja.prepared = ws + wsl.prepared_offset;
  ja.row_states = ws + wsl.row_states_offset;
  ja.max_rows = wsl.max_rows;
  ja.planes = ws + wsl.planes_offset;
  ja.regions = ws + wsl.regions_offset;
  ja.workspace = ws;
  ja.crop_out = crop_out;
  ja.row_index = static_cast<const uint8_t*>(d->jpeg_row_index);
  ja.whole_image = 0;
  return ja;
}
// What the resampling kernel needs to know about the source, for both input formats: with JPEG
// input its "images" are the decoded regions in the workspace.
mae::CropArgs make_crop_args(const mae_prep_desc* d, const PrepShape& sh, const PrepWorkspace& wsl,
                             const uint8_t* ws) {
  mae::CropArgs ca;
  memset(&ca, 0, sizeof(ca));
  ca.B = d->B;
  ca.S = d->out_size;
  ca.p = d->patch;
  ca.G = sh.G;
  ca.L = sh.L;
  ca.K = d->num_keep;
  ca.D = sh.D;
  ca.visible_bf16 = d->out_dtype == MAE_BF16;
  const mae::CropPlan plan = crop_plan_of(d, wsl.slot_side);
  ca.tile_pixels = plan.tile_pixels;
  ca.col_parts = plan.col_parts;
  ca.part_patches = plan.part_patches;
  for (int c = 0; c < 3; ++c) {
    ca.nscale[c] = (float)(1.0 / (255.0 * (double)d->std[c]));
    ca.nbias[c] = (float)(-(double)d->mean[c] / (double)d->std[c]);
  }
  ca.images = d->images;
  ca.images_bytes = d->images_bytes;
  ca.offsets = d->offsets;
  ca.widths = d->widths;
  if (d->input_format == MAE_INPUT_JPEG && ws) {
    ca.images = ws + wsl.regions_offset;
    ca.images_bytes = (int64_t)d->B * wsl.slot_side * wsl.slot_side * 3;
    ca.offsets = reinterpret_cast<const int64_t*>(ws + wsl.region_offsets_offset);
    ca.widths = reinterpret_cast<const int32_t*>(ws + wsl.region_widths_offset);
  }
  ca.workspace = ws;
  return ca;
}
}  // namespace

size_t mae_prep_workspace_bytes(const mae_prep_desc* d) {
  if (validate_prep(d, nullptr) != MAE_OK) return 0;
  return prep_workspace(d).total;
}

int mae_prep_batch(const mae_prep_desc* d, void* visible, uint8_t* mask, int32_t* ids_restore,
                   int32_t* ids_keep, float* target, int32_t* crop_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  PrepShape sh;
  int rc = validate_prep(d, &sh);
  if (rc != MAE_OK) return rc;
  if (!visible || !mask || !ids_restore) return MAE_ERR_NULL;
  if (!aligned(visible, 16) || (target && !aligned(target, 16))) return MAE_ERR_RANGE;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < mae_prep_workspace_bytes(d))
    return MAE_ERR_WORKSPACE;
  rc = have_device();
  if (rc != MAE_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  mae::ParamArgs pa;
  memset(&pa, 0, sizeof(pa));
  pa.B = d->B;
  pa.L = sh.L;
  pa.K = d->num_keep;
  pa.noise_bits = d->noise_bits;
  pa.sample_base = d->sample_base;
  pa.key1 = mae::batch_key(d->seed, d->batch_index);
  pa.scale_lo = (double)d->scale_lo;
  pa.scale_span = (double)d->scale_hi - (double)d->scale_lo;
  const double ln_lo = log((double)d->ratio_lo), ln_hi = log((double)d->ratio_hi);
  pa.ln_ratio_lo = ln_lo;
  pa.ln_ratio_span = ln_hi - ln_lo;
  pa.ratio_lo = (double)d->ratio_lo;
  pa.ratio_hi = (double)d->ratio_hi;
  pa.flip_p = d->flip_p;
  pa.images_bytes = d->images_bytes;
  pa.offsets = d->offsets;
  pa.heights = d->heights;
  pa.widths = d->widths;
  const PrepWorkspace wsl = prep_workspace(d);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  mae::JpegArgs ja;
  memset(&ja, 0, sizeof(ja));
  if (d->input_format == MAE_INPUT_JPEG) {
    // file headers first: the crop parameters need the image sizes
    ja = make_jpeg_args(d, wsl, ws, crop_out);
    if (mae::launch_jpeg_header(ja, stream) != hipSuccess) return MAE_ERR_HIP;
    // from here on the "images" are the slots of the decoded-region buffer
    pa.images_bytes = (int64_t)d->B * wsl.slot_side * wsl.slot_side * 3;
    pa.offsets = ja.region_offsets;
    pa.heights = ja.heights;
    pa.widths = ja.widths;
  }
  if (d->aug_mode != MAE_AUG_SIMPLE) {
    pa.aug_out = ws + wsl.aug_offset;
    pa.jitter = d->jitter;
  }
  pa.mask = mask;
  pa.ids_restore = ids_restore;
  pa.ids_keep = ids_keep;
  pa.crop_out = crop_out;
  pa.workspace = static_cast<uint8_t*>(workspace);
  if (mae::launch_params_mask(pa, stream) != hipSuccess) return MAE_ERR_HIP;
  if (d->input_format == MAE_INPUT_JPEG && mae::launch_jpeg_decode(ja, stream) != hipSuccess)
    return MAE_ERR_HIP;

  mae::CropArgs ca = make_crop_args(d, sh, wsl, ws);
  ca.ids_restore = ids_restore;
  ca.visible = visible;
  ca.target = target;
  ca.mask_out = mask;
  ca.order_out = ids_restore;
  ca.keep_out = ids_keep;
  ca.crop_out = crop_out;
  if (d->aug_mode == MAE_AUG_SIMPLE) {
    if (mae::launch_crop_patch(ca, stream) != hipSuccess) return MAE_ERR_HIP;
    return MAE_OK;
  }

  // finetuning augmentation: grayscale and solarisation are the resampling kernel's epilogue; the
  // images that drew the blur get their rounded 8-bit crop written to the workspace, and the
  // blur kernel writes their patch rows.  "3 Aug+" needs every image's mean luma after the
  // brightness step first: one pass that only adds it up, then the pass that writes.
  ca.u8_out = ws + wsl.u8_offset;
  ca.aug_mode = d->aug_mode;
  ca.jitter = d->jitter;
  ca.sample_base = d->sample_base;
  ca.key1 = pa.key1;
  ca.luma_partials = reinterpret_cast<double*>(ws + wsl.crop_partials_offset);
  ca.aug_recs = ws + wsl.aug_offset;
  mae::AugArgs aa;
  memset(&aa, 0, sizeof(aa));
  aa.B = ca.B;
  aa.S = ca.S;
  aa.p = ca.p;
  aa.G = ca.G;
  aa.L = ca.L;
  aa.K = ca.K;
  aa.D = ca.D;
  aa.visible_bf16 = ca.visible_bf16;
  aa.mode = d->aug_mode;
  aa.jitter = d->jitter;
  aa.sample_base = d->sample_base;
  aa.key1 = pa.key1;
  const mae::AugPlan aplan = mae::three_aug_plan(d->out_size, d->patch);
  aa.blur_parts = aplan.parts;
  aa.blur_part_patches = aplan.part_patches;
  for (int c = 0; c < 3; ++c) {
    aa.nscale[c] = ca.nscale[c];
    aa.nbias[c] = ca.nbias[c];
  }
  aa.u8 = ca.u8_out;
  aa.ids_restore = ids_restore;
  aa.workspace = ws;
  aa.aug_recs = ws + wsl.aug_offset;
  aa.partials = reinterpret_cast<double*>(ws + wsl.partials_offset);
  aa.visible = visible;
  aa.target = target;
  hipError_t err = mae::launch_crop_aug(ca, 0, stream);
  if (err == hipSuccess && d->aug_mode == MAE_AUG_THREE_PLUS) {
    err = mae::launch_aug_blur(aa, true, stream);
    if (err == hipSuccess) err = mae::launch_crop_aug(ca, 1, stream);
  }
  if (err == hipSuccess) err = mae::launch_aug_blur(aa, false, stream);
  return err == hipSuccess ? MAE_OK : MAE_ERR_HIP;
}

size_t mae_jpeg_index_bytes(const mae_prep_desc* d) {
  if (validate_prep(d, nullptr) != MAE_OK || d->input_format != MAE_INPUT_JPEG) return 0;
  const PrepWorkspace wsl = prep_workspace(d);
  return (size_t)d->B * (size_t)wsl.max_rows * mae::jpeg_row_state_bytes();
}

int mae_jpeg_index(const mae_prep_desc* d, void* index, size_t index_bytes, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  int rc = validate_prep(d, nullptr);
  if (rc != MAE_OK) return rc;
  if (d->input_format != MAE_INPUT_JPEG) return MAE_ERR_RANGE;
  if (!index || !workspace) return MAE_ERR_NULL;
  if (!aligned(index, 16) || !aligned(workspace, 256)) return MAE_ERR_RANGE;
  const PrepWorkspace wsl = prep_workspace(d);
  if (index_bytes < (size_t)d->B * (size_t)wsl.max_rows * mae::jpeg_row_state_bytes() ||
      workspace_bytes < wsl.total)
    return MAE_ERR_WORKSPACE;
  rc = have_device();
  if (rc != MAE_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  mae::JpegArgs ja = make_jpeg_args(d, wsl, static_cast<uint8_t*>(workspace), nullptr);
  ja.row_states = static_cast<uint8_t*>(index);  // every row of every file: the index itself
  ja.row_index = nullptr;
  ja.whole_image = 1;
  if (mae::launch_jpeg_header(ja, stream) != hipSuccess) return MAE_ERR_HIP;
  if (mae::launch_jpeg_index(ja, stream) != hipSuccess) return MAE_ERR_HIP;
  return MAE_OK;
}

int mae_prep_status(const void* workspace, void* hip_stream, int32_t* host_invalid_samples) {
  if (!workspace || !host_invalid_samples) return MAE_ERR_NULL;
  int rc = have_device();
  if (rc != MAE_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (hipStreamSynchronize(stream) != hipSuccess) return MAE_ERR_HIP;
  mae::WorkspaceHeader hdr;
  if (hipMemcpy(&hdr, workspace, sizeof(hdr), hipMemcpyDeviceToHost) != hipSuccess)
    return MAE_ERR_HIP;
  if (hdr.magic != mae::kWorkspaceMagic || hdr.B <= 0) return MAE_ERR_WORKSPACE;
  int32_t invalid = 0;
  const uint8_t* recs = static_cast<const uint8_t*>(workspace) + mae::kWorkspaceHeader;
  mae::CropRec chunk[256];
  for (int32_t done = 0; done < hdr.B; done += 256) {
    const int32_t n = hdr.B - done < 256 ? hdr.B - done : 256;
    if (hipMemcpy(chunk, recs + (size_t)done * sizeof(mae::CropRec), (size_t)n * sizeof(mae::CropRec),
                  hipMemcpyDeviceToHost) != hipSuccess)
      return MAE_ERR_HIP;
    for (int32_t i = 0; i < n; ++i) invalid += chunk[i].valid ? 0 : 1;
  }
  *host_invalid_samples = invalid;
  return MAE_OK;
}

size_t mae_loss_workspace_bytes(const mae_loss_desc* d) {
  if (validate_loss(d) != MAE_OK) return 0;
  const mae::LossShape sh =
      mae::loss_shape((int64_t)d->B * d->L, d->D, d->pred_dtype == MAE_BF16);
  // one partial sum per wavefront, then the partial counts of the mask (num_masked = 0)
  return (size_t)sh.waves * sizeof(double) + (size_t)mae::kMaxCounts * sizeof(int32_t);
}

namespace {
// Fills the kernel arguments from a validated descriptor and enqueues the loss kernels.
int enqueue_loss(const mae_loss_desc* d, float* loss, void* grad, double* partials,
                 const mae::LossShape& sh, hipStream_t stream) {
  mae::LossArgs la;
  memset(&la, 0, sizeof(la));
  la.rows = (int64_t)d->B * d->L;
  la.D = d->D;
  la.pred_bf16 = d->pred_dtype == MAE_BF16;
  la.norm_pix = d->norm_pix;
  la.eps = d->eps;
  const double count = (double)d->D * (double)(d->num_masked > 0 ? d->num_masked : 1);
  la.gscale = (float)((double)d->grad_scale * 2.0 / count);
  la.inv_count = 1.0 / count;
  la.pred = d->pred;
  la.target = d->target;
  la.mask = d->mask;
  la.grad = grad;
  la.loss = loss;
  la.partials = partials;
  la.num_partials = sh.waves;
  la.rows_per_iter = sh.rows_per_iter;
  la.pair_groups = sh.pair_groups;
  if (d->num_masked == 0) {  // the divisor is the number of non-zero mask bytes, counted first
    int32_t* counts = reinterpret_cast<int32_t*>(partials + sh.waves);
    la.counts = counts;
    la.ncounts = mae::mask_count_blocks(la.rows);
    la.gscale_num = 2.0 * (double)d->grad_scale;
    la.gscale = 0.0f;
    la.inv_count = 0.0;
    if (mae::launch_mask_count(d->mask, la.rows, counts, stream) != hipSuccess) return MAE_ERR_HIP;
  }
  if (mae::launch_normpix_loss(la, stream) != hipSuccess) return MAE_ERR_HIP;
  return MAE_OK;
}
}  // namespace

int mae_normpix_loss(const mae_loss_desc* d, float* loss, void* grad, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  int rc = validate_loss(d);
  if (rc != MAE_OK) return rc;
  if (!loss) return MAE_ERR_NULL;
  if (!aligned(d->pred, 16) || !aligned(d->target, 16) || (grad && !aligned(grad, 16)))
    return MAE_ERR_RANGE;
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < mae_loss_workspace_bytes(d))
    return MAE_ERR_WORKSPACE;
  rc = have_device();
  if (rc != MAE_OK) return rc;
  const mae::LossShape sh =
      mae::loss_shape((int64_t)d->B * d->L, d->D, d->pred_dtype == MAE_BF16);
  return enqueue_loss(d, loss, grad, static_cast<double*>(workspace), sh,
                      static_cast<hipStream_t>(hip_stream));
}

// ---- the loss for callers that cannot allocate -----------------------------------------------------
// The per-wavefront partial sums go to a fixed array in device memory that belongs to the library
// (one copy per GPU, held until the process ends) instead of a caller's workspace.
namespace {
constexpr int kScratchDoubles = 8192;  // 64 KiB; the loss grid never has more wavefronts than this
__attribute__((used)) static __device__ __align__(256) double scratch[kScratchDoubles];
constexpr int kMaxDevices = 64;
std::atomic<double*> g_scratch_ptr[kMaxDevices];  // device address of `scratch`, per GPU

// Address of this GPU's copy of `scratch` (looked up once per device, with that device current).
int scratch_address(double** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return MAE_ERR_NO_DEVICE;
  }
  if (dev < 0 || dev >= kMaxDevices) return MAE_ERR_RANGE;
  double* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
      (void)hipGetLastError();
      return MAE_ERR_HIP;
    }
    ptr = static_cast<double*>(sym);
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return MAE_OK;
}
}  // namespace

int mae_normpix_loss_static(const mae_loss_desc* d, float* loss, void* grad, void* hip_stream) {
  int rc = validate_loss(d);
  if (rc != MAE_OK) return rc;
  if (!loss) return MAE_ERR_NULL;
  if (!aligned(d->pred, 16) || !aligned(d->target, 16) || (grad && !aligned(grad, 16)))
    return MAE_ERR_RANGE;
  const mae::LossShape sh =
      mae::loss_shape((int64_t)d->B * d->L, d->D, d->pred_dtype == MAE_BF16);
  // more partials (and the mask's partial counts behind them) than the array holds
  if (sh.waves + mae::kMaxCounts / 2 > kScratchDoubles) return MAE_ERR_WORKSPACE;
  rc = have_device();
  if (rc != MAE_OK) return rc;
  double* partials = nullptr;
  rc = scratch_address(&partials);
  if (rc != MAE_OK) return rc;
  return enqueue_loss(d, loss, grad, partials, sh, static_cast<hipStream_t>(hip_stream));
}

namespace {
int validate_loss_from_images(const mae_prep_desc* p, const mae_loss_desc* d, PrepShape* sh) {
  int rc = validate_prep(p, sh);
  if (rc != MAE_OK) return rc;
  rc = validate_loss(d, false);
  if (rc != MAE_OK) return rc;
  if (p->aug_mode != MAE_AUG_SIMPLE) return MAE_ERR_RANGE;  // the pretraining pipeline only
  if ((sh->D & 3) != 0) return MAE_ERR_SHAPE;               // 16-byte groups: even patch sizes
  if (d->B != p->B || d->L != sh->L || d->D != sh->D) return MAE_ERR_SHAPE;
  return MAE_OK;
}
}  // namespace

size_t mae_loss_from_images_workspace_bytes(const mae_prep_desc* p, const mae_loss_desc* d) {
  PrepShape sh;
  if (validate_loss_from_images(p, d, &sh) != MAE_OK) return 0;
  const mae::CropArgs ca = make_crop_args(p, sh, prep_workspace(p), nullptr);
  return (size_t)mae::crop_loss_partials(ca) * sizeof(double) +
         (size_t)mae::kMaxCounts * sizeof(int32_t);
}

int mae_normpix_loss_from_images(const mae_prep_desc* p, const void* prep_workspace_ptr,
                                 size_t prep_workspace_bytes, const mae_loss_desc* d, float* loss,
                                 void* grad, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  PrepShape sh;
  int rc = validate_loss_from_images(p, d, &sh);
  if (rc != MAE_OK) return rc;
  if (!loss || !prep_workspace_ptr) return MAE_ERR_NULL;
  if (!aligned(d->pred, 16) || (grad && !aligned(grad, 16))) return MAE_ERR_RANGE;
  if (!aligned(prep_workspace_ptr, 256) || prep_workspace_bytes < mae_prep_workspace_bytes(p))
    return MAE_ERR_WORKSPACE;
  if (!workspace || !aligned(workspace, 256) ||
      workspace_bytes < mae_loss_from_images_workspace_bytes(p, d))
    return MAE_ERR_WORKSPACE;
  rc = have_device();
  if (rc != MAE_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  mae::CropArgs ca = make_crop_args(p, sh, prep_workspace(p),
                                    static_cast<const uint8_t*>(prep_workspace_ptr));
  const double count = (double)d->D * (double)(d->num_masked > 0 ? d->num_masked : 1);
  ca.pred = d->pred;
  ca.grad = grad;
  ca.mask = d->mask;
  ca.partials = static_cast<double*>(workspace);
  ca.eps = d->eps;
  ca.gscale = (float)((double)d->grad_scale * 2.0 / count);
  ca.pred_bf16 = d->pred_dtype == MAE_BF16;
  ca.norm_pix = d->norm_pix;
  ca.loss_out = loss;
  ca.inv_count = 1.0 / count;
  if (d->num_masked == 0) {
    int32_t* counts = reinterpret_cast<int32_t*>(ca.partials + mae::crop_loss_partials(ca));
    const int64_t rows = (int64_t)d->B * d->L;
    ca.counts = counts;
    ca.ncounts = mae::mask_count_blocks(rows);
    ca.gscale_num = 2.0 * (double)d->grad_scale;
    ca.gscale = 0.0f;
    ca.inv_count = 0.0;
    if (mae::launch_mask_count(d->mask, rows, counts, stream) != hipSuccess) return MAE_ERR_HIP;
  }
  if (mae::launch_crop_loss(ca, stream) != hipSuccess) return MAE_ERR_HIP;
  return MAE_OK;
}

int mae_patch_embed(const mae_embed_desc* d, void* tokens, void* hip_stream) {
  int rc = validate_embed(d);
  if (rc != MAE_OK) return rc;
  if (!tokens) return MAE_ERR_NULL;
  if (!aligned(tokens, 16)) return MAE_ERR_RANGE;
  rc = have_device();
  if (rc != MAE_OK) return rc;

  mae::EmbedArgs ea;
  memset(&ea, 0, sizeof(ea));
  ea.M = d->M;
  ea.D = d->D;
  ea.E = d->E;
  ea.L = d->L;
  ea.out_bf16 = d->out_dtype == MAE_BF16;
  ea.visible = d->visible;
  ea.ids_keep = d->ids_keep;
  ea.weight = d->weight;
  ea.bias = d->bias;
  ea.pos = d->pos;
  ea.tokens = tokens;
  if (mae::launch_patch_embed(ea, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MAE_ERR_HIP;
  return MAE_OK;
}

// ---- progressive schedules: the stage tables of the paper ---------------------------------------
namespace {
struct PretrainStage {
  int16_t res;
  double m;
};
// Table 9, rows = stages, one block per scheme
const PretrainStage kPretrain[6][3] = {
    {{160, 0.50}, {192, 0.66}, {224, 0.75}},  // scheme 1
    {{160, 0.75}, {192, 0.75}, {224, 0.75}},  // scheme 2
    {{224, 0.75}, {192, 0.75}, {160, 0.75}},  // scheme 3
    {{160, 0.75}, {192, 0.80}, {224, 0.85}},  // scheme 4
    {{224, 0.75}, {192, 0.75}, {224, 0.75}},  // scheme 5
    {{224, 0.75}, {192, 0.75}, {224, 0.85}},  // scheme 6
};
}  // namespace

int mae_pretrain_stage(int32_t scheme, int32_t stage, int32_t* host_out_size,
                       double* host_mask_ratio) {
  if (!host_out_size || !host_mask_ratio) return MAE_ERR_NULL;
  if (scheme < 1 || scheme > 6 || stage < 1 || stage > 3) return MAE_ERR_RANGE;
  *host_out_size = kPretrain[scheme - 1][stage - 1].res;
  *host_mask_ratio = kPretrain[scheme - 1][stage - 1].m;
  return MAE_OK;
}

int mae_finetune_stage(int32_t scheme, int32_t stage, int32_t* host_out_size,
                       float* host_scale_lo, float* host_scale_hi, int32_t* host_aug_mode) {
  if (!host_out_size || !host_scale_lo || !host_scale_hi) return MAE_ERR_NULL;
  const bool known = scheme == MAE_FINETUNE_SCHEME_1 || scheme == MAE_FINETUNE_SCHEME_3 ||
                     scheme == MAE_FINETUNE_SCHEME_1_MINUS || scheme == MAE_FINETUNE_SCHEME_1_PLUS;
  if (!known || stage < 1 || stage > 3) return MAE_ERR_RANGE;
  // Table 7: sigma- = 0.28 throughout; scheme 3 raises sigma+ with the resolution
  const double sigma_lo = 0.28;
  double sigma_hi = 1.0;
  if (scheme == MAE_FINETUNE_SCHEME_3) sigma_hi = stage == 1 ? 0.68 : (stage == 2 ? 0.84 : 1.0);
  *host_out_size = 128 + 32 * stage;  // 160, 192, 224
  *host_scale_lo = (float)(sigma_lo * sigma_lo);
  *host_scale_hi = (float)(sigma_hi * sigma_hi);
  if (host_aug_mode) {
    // the table's aug column: schemes 1 and 3 add the colour jitter in the last stage only,
    // "1-" never, "1+" in every stage
    int32_t aug = stage == 3 ? MAE_AUG_THREE_PLUS : MAE_AUG_THREE;
    if (scheme == MAE_FINETUNE_SCHEME_1_MINUS) aug = MAE_AUG_THREE;
    if (scheme == MAE_FINETUNE_SCHEME_1_PLUS) aug = MAE_AUG_THREE_PLUS;
    *host_aug_mode = aug;
  }
  return MAE_OK;
}

int mae_stage_of_epoch(int32_t epoch, const int32_t* host_lengths, int32_t n) {
  if (!host_lengths) return MAE_ERR_NULL;
  if (epoch < 0 || n < 1) return MAE_ERR_RANGE;
  int64_t end = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (host_lengths[s] < 0) return MAE_ERR_RANGE;
    end += host_lengths[s];
    if (epoch < end) return s + 1;
  }
  return n;
}

}  // extern "C"
