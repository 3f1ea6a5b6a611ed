/*
 * pcr.h -- C ABI of the MI355X (gfx950) decoder for Progressive Compressed Records (PCRs).
 *
 * A PCR stores, after a small metadata block, "scan group" 1, 2, ..., G: group g holds the
 * g-th scan of the progressive JPEG file of every image in the record, so that reading the
 * record from its start to the end of group k yields the whole batch at fidelity k (paper
 * Section 3, record figure).  This library opens such a byte prefix, rebuilds the index that
 * un-groups the scans, and decodes all images at a chosen scan group into uint8 pixels on the
 * GPU: each image's scans 1..k followed by an end-of-image marker are what a JPEG decoder is
 * given (Section 5, "Decoding").
 *
 * Conventions
 *   - every function returns PCR_OK (0) or a negative PCR_E_* code; nothing throws or aborts;
 *     out-parameters are written only on success;
 *   - "host" / "device" say where a pointer must live; device pointers belong to the HIP
 *     device the record was opened on;
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream);
 *   - one handle must not be used from two threads at once; different handles are independent.
 *
 * Record byte layout ("PCR1", little endian):
 *   "PCR1" | u32 version=1 | u32 n | u32 G | u64 header_bytes | u64 group_end[G] |
 *   i32 label[n] | u32 n_scans[n] | u32 len[G][n] | zero padding to header_bytes |
 *   group 1 | ... | group G,   group g = region(0,g) | region(1,g) | ... | region(n-1,g)
 * region(i,g) is the slice of image i's progressive JPEG file from the end of its scan g-1
 * (or the file start) to the end of its scan g (or the file end for its last scan).
 * Version 2 (pcr_record_write_indexed) has, behind len[G][n],  u32 entry_interval | u32 0 | u16 ecount[G][n],  and
 * every group ends with its entry points, ecount[g][i] entries for image i one image after the other, each
 *   u32 mcu | u32 bit | i16 pred[3] | u16 0   (see pcr_record_write_indexed); group_end[g] includes them.
 *
 * Not supported (PCR_E_UNSUPPORTED): arithmetic coding, 12-bit samples, lossless and
 * hierarchical modes, DNL, component counts other than 1 or 3, sampling factors other than 1
 * or 2, records of 4 GiB or more.
 *
 * Sequential (baseline, non-progressive) Huffman files are accepted too: such a file is one scan (or one
 * per component), so a record of them has that many scan groups and no lower fidelities.  They are what
 * the paper's baseline layouts hold (Section 6.1); the same calls decode them.
 */
#ifndef PCR_H
#define PCR_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pcr_record pcr_record;      /* opaque; owned by the library */

enum {
    PCR_OK = 0,
    PCR_E_ARG = -1,          /* NULL or otherwise unusable argument */
    PCR_E_FORMAT = -2,       /* bytes are not a well-formed record / JPEG stream */
    PCR_E_TRUNCATED = -3,    /* the bytes given do not reach the requested scan group */
    PCR_E_UNSUPPORTED = -4,  /* well-formed but outside what this library decodes */
    PCR_E_RANGE = -5,        /* index or capacity out of range */
    PCR_E_NOMEM = -6,
    PCR_E_DEVICE = -7        /* a HIP call failed, or no gfx950 code object could be loaded */
};

/*
 * Open a record (Section 5, "Decoding": locate the scan-group offsets in the metadata).
 *   bytes, nbytes  host pointer to the record or to any prefix of it; groups that are not
 *                  wholly inside the prefix are unavailable, never partially used.
 *   device_id      HIP device that will hold the record and run the decode.
 * The library copies what it needs (the bytes go to device memory); the caller may free
 * `bytes` when the call returns.  Frame headers of all images are validated here, so that
 * malformed or unsupported content is reported synchronously.
 */
int pcr_open(const void* bytes, size_t nbytes, int device_id, pcr_record** out);

/*
 * Open a record whose bytes are already in device memory (for loaders that stream record prefixes
 * to the GPU themselves; paper Section 5, "Loader": whole-record buffers that are re-used).
 *   d_bytes, nbytes  device pointer (16-byte aligned) to the record or a prefix of it.  The bytes are
 *                    BORROWED: they must stay valid and unchanged until pcr_close.
 *   hip_stream       stream the open-time kernels and copies run on; the call synchronises it.
 * The index and the JPEG marker segments are parsed on the device; only the metadata block and the
 * small per-image descriptor tables are copied back to size the buffers.  The device is the one
 * that owns d_bytes.
 */
int pcr_open_device(const void* d_bytes, size_t nbytes, void* hip_stream, pcr_record** out);

/*
 * Bind an existing handle to another record in device memory, re-using the handle's device buffers
 * (they are re-allocated only when the new record needs more than the handle already holds), so that a
 * loader that decodes record after record stops allocating after the first few (Section 5, "Loader":
 * double buffering with re-used buffers).  Arguments and behaviour as pcr_open_device; every earlier call
 * on the handle must have finished, or be ordered before this one on hip_stream.  Whatever the handle
 * knew about its previous record is gone (layouts, resident planes, timing history is kept).  If the
 * call fails the handle holds no record: only another pcr_rebind_device or pcr_close may follow.
 */
int pcr_rebind_device(pcr_record* rec, const void* d_bytes, size_t nbytes, void* hip_stream);

/* Release a handle and all device memory it owns.  NULL is allowed.  The call waits for ALL work on the handle's
 * device (releasing device memory does that in any case), so it also holds up other handles' streams: a loader keeps
 * its handles and re-binds them (pcr_rebind_device, pcr_loader_*) instead of closing and opening per record. */
void pcr_close(pcr_record* rec);

int pcr_num_images(const pcr_record* rec, int* n);
int pcr_num_scan_groups(const pcr_record* rec, int* G);            /* groups the record defines */
int pcr_available_scan_groups(const pcr_record* rec, int* k_max);  /* groups inside the bytes given */

/* Bytes that must be read from the start of the record for fidelity k (1..G): the absolute
 * offset one past scan group k (Section 3: fidelity k is the byte prefix of the record that ends
 * with scan group k). */
int pcr_group_end_offset(const pcr_record* rec, int k, uint64_t* off);

/* Width, height, channels (1 or 3) and the 32-bit label of image i.  Any out pointer may be NULL. */
int pcr_image_info(const pcr_record* rec, int i, int* width, int* height, int* channels, int32_t* label);

/* Output layout: image i occupies bytes [offsets[i], offsets[i+1]) of the output buffer as
 * H_i x W_i x C_i uint8, row-major, channel-interleaved (NHWC; a dense [N,H,W,C] tensor when all
 * images have one size).  offsets: host, n+1 entries, n as pcr_num_images reports it NOW: a handle that was
 * bound to another record since (pcr_rebind_device, a loader slot's next upload) has another n. */
int pcr_output_layout(const pcr_record* rec, uint64_t* offsets);

/* ---- parity hooks: intermediate results, computed on the device, returned to the host ---- */

/* The un-grouping index (Section 5, "Encoding": grouping the scans needs an index that undoes
 * it): off[g*n+i] = absolute offset of region(i,g+1), len[g*n+i] its length, for the
 * available groups g < k_max (entries of unavailable groups are left untouched).
 * Computed by the index kernel.  off, len: host, G*n entries. */
int pcr_index(const pcr_record* rec, uint64_t* off, uint32_t* len);

/* The byte string of image i at fidelity k: regions 1..min(k, scans of i), followed by FF D9 if
 * and only if scans were left out (Section 5, "Decoding").  dst: host, cap bytes; *len receives
 * the length (also when dst is NULL, to query).  Gathered by a device kernel.  (The handle is not const: it keeps
 * the device staging buffer of the gather between calls.) */
int pcr_reassemble(pcr_record* rec, int i, int k, uint8_t* dst, size_t cap, size_t* len);

/* Coefficient layout: image i occupies int16 elements [offsets[i], offsets[i+1]); inside, the
 * component planes follow each other, each [bh_c][bw_c][64] in natural (row-major) order, where
 * bw_c x bh_c is the MCU-padded block grid.  offsets: host, n+1 entries. */
int pcr_coef_layout(const pcr_record* rec, uint64_t* offsets);

/* Quantised coefficients after scans 1..k (partially refined coefficients are multiples of
 * 2^Al; coefficients not yet received are 0).  d_coef: device, offsets[n] int16 elements.
 * Asynchronous on hip_stream. */
int pcr_decode_coefficients(pcr_record* rec, int k, int16_t* d_coef, void* hip_stream);

/*
 * The hot call: decode every image of the record at scan group k (1..k_max) to pixels.
 *   out_u8_nhwc   device pointer, layout as pcr_output_layout; out_capacity in bytes
 *   d_status      optional device array of n int32: 0, or a PCR_E_* code for an image whose
 *                 entropy-coded data is corrupt (its pixels are zero-filled)
 * Runs the whole path on the device: index, marker parsing, unstuffing, progressive Huffman
 * decode of scans 1..k, refinement, de-quantisation, inverse DCT, chroma replication and
 * YCbCr->RGB.  Coefficients not yet received count as zero; no smoothing is applied.
 * Asynchronous and stream-ordered; argument errors are returned before anything is enqueued.
 * Decoding several records at a time (one handle and one stream each) is how the GPU is filled: a record alone
 * is bound by its longest serial streams.  HIP maps streams onto GPU_MAX_HW_QUEUES hardware queues (default 4,
 * one of them the null stream's); streams that share a queue run one after the other, so a process that overlaps
 * R records wants that environment variable set to R + 1 or more before the HIP runtime starts.
 */
int pcr_decode_batch(pcr_record* rec, int scan_group, uint8_t* out_u8_nhwc, size_t out_capacity,
                     void* hip_stream, int32_t* d_status);

/* pcr_decode_batch with the chroma up-sampling of stock decoders (Section 5, "Decoding", hands the reassembled bytes
 * to a stock decoder; the JPEG standard defines no up-sampling, and stock decoders interpolate where pcr_decode_batch
 * replicates).  Every component's samples are rounded to integers first; an output sample of a component stored at
 * half resolution is then 3/4 of the nearer and 1/4 of the farther sample of the component's own grid, down the
 * columns first, then along the rows (beyond the component's ceil(W hs / hmax) x ceil(H vs / vmax) samples the nearest
 * one stands in); colour conversion and the final rounding as in pcr_decode_batch.  Images without sub-sampled
 * components differ from pcr_decode_batch only by the rounding of the samples.  The first call on a handle takes one
 * byte per coefficient slot of working memory from the handle's arena (which may allocate).  Arguments, layout,
 * stream order, d_status and errors as pcr_decode_batch; a following pcr_upgrade_batch starts from scan_group. */
int pcr_decode_batch_triangle(pcr_record* rec, int scan_group, uint8_t* out_u8_nhwc, size_t out_capacity,
                              void* hip_stream, int32_t* d_status);

/* pcr_decode_batch with the smoothing stock decoders apply to the first scans of a progressive file (Section 5,
 * "Decoding", hands the reassembled bytes to a stock decoder, and stock decoders smooth what has only its DC
 * coefficients).  Every component of which only the DC first scan lies inside scan_group gets the
 * five lowest AC coefficients of each block predicted from the DC coefficients of the block and its eight neighbours
 * (JPEG standard, T.81 K.8: the coefficients of the quadratic surface whose means over the nine blocks are the nine DC
 * values).  Integer form, per coefficient with quantiser step Qz, DC step Q0 and DC coefficients as received:
 *   zig-zag 1: 36 Q0 (left - right)        zig-zag 2: 36 Q0 (above - below)      zig-zag 3: 9 Q0 (above + below - 2 centre)
 *   zig-zag 4: 5 Q0 ((above-left - above-right) - (below-left - below-right))    zig-zag 5: 9 Q0 (left + right - 2 centre)
 * divided by 256 Qz and rounded to the nearest integer, halves away from zero, limited to +-1023; a neighbour beyond
 * the component's (MCU-padded) block grid is the nearest block inside it.  Components that have received an AC scan or
 * a DC refinement scan, and sequential files, decode exactly as in pcr_decode_batch, so at the last scan group the two
 * calls agree bit for bit.  The coefficient planes are left as pcr_decode_batch leaves them (the predictions are in
 * them at most for the duration of the call): a following pcr_upgrade_batch starts from scan_group as after
 * pcr_decode_batch.  Arguments, layout, stream order,
 * d_status and errors as pcr_decode_batch. */
int pcr_decode_batch_smooth(pcr_record* rec, int scan_group, uint8_t* out_u8_nhwc, size_t out_capacity,
                            void* hip_stream, int32_t* d_status);

/* Fidelity upgrade (Section 3 of the paper: a lower-fidelity read is a prefix of a higher-fidelity one, so
 * changing fidelity costs little): raise the planes the last pcr_decode_batch /
 * pcr_upgrade_batch call on this handle left on the device from its scan group to `scan_group` (>= it) by
 * unstuffing and entropy-decoding only the scans of the new groups, then produce the pixels.  The output is
 * bit-identical to pcr_decode_batch(rec, scan_group, ...); arguments, layout, stream order and d_status as
 * there.  The earlier call must have completed or be ordered before this one on the same stream.
 * pcr_resident_scan_group: the scan group an upgrade would start from; 0 if there is none (nothing decoded
 * yet, the last call failed, or the last call was pcr_decode_coefficients, which rewrites the planes).
 * Errors: PCR_E_ARG if nothing is resident or scan_group is lower than the resident group; otherwise as
 * pcr_decode_batch. */
int pcr_upgrade_batch(pcr_record* rec, int scan_group, uint8_t* out_u8_nhwc, size_t out_capacity,
                      void* hip_stream, int32_t* d_status);
int pcr_resident_scan_group(const pcr_record* rec, int* scan_group);

/* Training tail (Section 6.1: the experiments crop, resize and flip the decoded images, as is usual for ImageNet
 * training; the appendix trains on 160x160 and 224x224 crops).  For every image of the record one box of its
 * decoded pixels is resized to out_h x out_w -- bilinear interpolation on pixel centres, no anti-aliasing, samples
 * beyond the box's edge repeat the edge --, mirrored left to right if flip != 0, and channel c becomes
 * (v / 255 - mean[c]) * inv_std[c], stored as IEEE half precision in a dense [n][C][out_h][out_w] tensor.
 *   d_pixels   device: pixels in the layout of pcr_output_layout (what pcr_decode_batch wrote)
 *   d_crops    device: n boxes in source pixels; a box reaching outside its image is clamped into it
 *   mean, inv_std   host: C floats each (C = channels of the images, which must all agree: else UNSUPPORTED)
 *   d_out_f16  device: n*C*out_h*out_w halfs; out_capacity in bytes
 * Which box and whether to flip is the caller's (random) choice.  Asynchronous on hip_stream. */
typedef struct { int32_t x0, y0, w, h, flip; } pcr_crop;
int pcr_crop_resize_batch(pcr_record* rec, const uint8_t* d_pixels, const pcr_crop* d_crops, int out_h, int out_w,
                          const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity, void* hip_stream);

/* Fidelity estimate (Section 6.4: MSSIM between the picture of a scan group and the full picture tracks the
 * accuracy a model reaches on that scan group, which is what Section 4.3's choice of scan group rests on).  For
 * every image of the record, the multi-scale structural similarity (Wang, Simoncelli and Bovik 2003) of its
 * pictures in two decoded batches, computed on luma (0.299 R + 0.587 G + 0.114 B, not rounded): 11 x 11
 * Gaussian window of sigma 1.5 at the positions where it fits, C1 = (0.01*255)^2, C2 = (0.03*255)^2, five scales
 * by 2 x 2 averaging with the published exponents 0.0448, 0.2856, 0.3001, 0.2363, 0.1333 (used as they are: they
 * sum to 1.0001).  An image whose smaller side is below 176 uses as many scales as keep that side at 11 samples or
 * more, their exponents rescaled to sum to 1; a negative scale mean counts as 0; an image smaller than 11 on a side scores NaN.
 *   d_a, d_b   device: two pixel batches in the layout of pcr_output_layout (say scan group k and scan group G)
 *   d_scores   device: n floats
 * Computed in single precision from exact integer block sums; agrees with a double-precision evaluation to
 * about 1e-4.  The first call on a handle allocates n x (tiles per image) x 8 bytes of working memory (which
 * pcr_rebind_device releases).  Asynchronous on hip_stream; calls on one handle must not overlap.
 * Errors: PCR_E_ARG (null argument), PCR_E_UNSUPPORTED (channel counts differ between images), PCR_E_NOMEM. */
int pcr_msssim_batch(pcr_record* rec, const uint8_t* d_a, const uint8_t* d_b, float* d_scores, void* hip_stream);

/* pcr_msssim_batch for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical scores; the per-tile
 * sums live in a fixed 4 MiB array inside the library's code object (one copy per GPU, held until the process
 * ends) instead of the handle's working memory, and the call makes no hipMalloc / hipFree or any other
 * allocating call.  Limit: n x (largest tile count of an image of the record) <= 524288 entries (for instance
 * 1024 images of up to 500 x 500 pixels, 341 tiles each); beyond it PCR_E_RANGE, nothing enqueued.  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU (other streams, other handles, other
 * threads) race and must be ordered by the caller.  Nothing in the array has to be cleared between calls.
 * Other errors as pcr_msssim_batch. */
int pcr_msssim_batch_static(pcr_record* rec, const uint8_t* d_a, const uint8_t* d_b, float* d_scores, void* hip_stream);

/* Choosing a scan group by image quality (Section 6.4: scan groups whose MSSIM against the full picture is high
 * train about as well as the full data, so the score can pick the level of compression; Section 4.3 leaves the
 * choice to a tuner).  Returns in *scan_group the lowest scan group whose mean pcr_msssim_batch score over the
 * record's images, against the pictures of the highest available scan group, is at least min_mean_score (the
 * highest available group itself if none is).  Scan groups are tried in order, each obtained from the one before
 * by pcr_upgrade_batch, so the whole search costs about one full decode plus the scores.
 *   d_work_a, d_work_b   device: two pixel buffers of work_capacity >= pcr_output_layout's total bytes each
 *   d_scores             device: n floats (scores of the last group tried)
 *   mean_by_group        host, optional: G floats; entry g-1 receives the mean score of group g, -1 if not tried
 * Synchronous (each group's scores are read back); enqueues on hip_stream and waits for it.  Afterwards the
 * handle's resident scan group is the last one tried and d_work_a holds its pixels.  Errors as the calls it makes. */
int pcr_select_scan_group(pcr_record* rec, float min_mean_score, uint8_t* d_work_a, uint8_t* d_work_b, size_t work_capacity,
                          float* d_scores, float* mean_by_group, int* scan_group, void* hip_stream);

/* Decode and training tail in one call; the half-precision output is bit-identical to pcr_decode_batch at scan_group
 * followed by pcr_crop_resize_batch with the same boxes.
 *   d_pixels == NULL   decode and tail run in ONE kernel and the full-resolution pixels never reach memory: one
 *                      workgroup decodes one MCU row of an image into on-chip memory and interpolates from it every output
 *                      sample whose two source rows lie in that MCU row; only the first and last pixel row of every MCU
 *                      row (1/8 of the pixels for 4:2:0 images) go to a side buffer of the handle, from which a second,
 *                      small kernel interpolates the remaining output rows.  MCUs that do not touch an image's box are
 *                      not decoded.  A workgroup holds 256 / (blocks per MCU) MCUs at a time (672 pixels of width for
 *                      4:2:0 and 4:4:4, 1024 for 4:2:2, 2048 for gray); a box wider than that is served in passes that
 *                      overlap by one MCU, at any image width.
 *                      The first such call on a record allocates the side buffer.
 *   d_pixels != NULL   (device, layout of pcr_output_layout, pixel_capacity bytes) working memory: the pixel kernel
 *                      writes the runs of MCUs that touch an image's box there (what it held elsewhere stays), and
 *                      pcr_crop_resize_batch reads them.
 * The planes left on the device are complete (pcr_upgrade_batch may follow).  Other arguments and errors as in the two
 * calls. */
int pcr_decode_crop_batch(pcr_record* rec, int scan_group, const pcr_crop* d_crops, uint8_t* d_pixels, size_t pixel_capacity,
                          int out_h, int out_w, const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity,
                          void* hip_stream, int32_t* d_status);

/* ---- loader: host bytes -> device -> pixels, double-buffered (Section 5, "Loader") ----
 *
 * pcr_prefix_length: how much of a record must be read for fidelity k, from the record's first bytes alone
 *   (host pointer; 24 + 8*G bytes always suffice).  PCR_OK and *need = that length; PCR_E_TRUNCATED and
 *   *need = how many first bytes are needed to tell.
 *
 * A loader owns `slots` sets of {pinned host staging buffer, device buffer, stream, record handle}, each of
 * slot_bytes capacity, allocated once.  The caller reads a record prefix into a slot's staging buffer
 * (pcr_loader_staging), then
 *   pcr_loader_upload  copies nbytes of it to the device on the slot's stream and binds the slot's handle to
 *                      them (pcr_open_device the first time, pcr_rebind_device afterwards).  It first waits
 *                      for the slot's earlier work, and returns when the record's metadata is known: *rec
 *                      (optional) is the slot's handle for layout queries, valid until the slot's next upload.
 *   pcr_loader_read_file  does the reading as well: of the record file at `path` exactly the prefix scan group k
 *                      needs (Section 3: a fidelity is a byte prefix; Section 4.1: reading less is where the
 *                      speed-up comes from) -- the first bytes, which say how long it is, then the rest -- into the
 *                      slot's staging buffer with pread, then pcr_loader_upload.  It waits for the slot's earlier
 *                      work first.  *nbytes (optional) receives the bytes read.  PCR_E_ARG: the file cannot be
 *                      opened or read; PCR_E_TRUNCATED: it ends before the prefix does; PCR_E_RANGE: the prefix
 *                      does not fit the slot, or k is no scan group of the record.
 *   pcr_loader_decode  = pcr_decode_batch on the slot's handle and stream (asynchronous).
 *   pcr_loader_decode_crop  = pcr_decode_crop_batch there: from the bytes read to half-precision training tensors.
 *   pcr_loader_wait    blocks until the slot's stream is idle; the staging buffer may be refilled after
 *                      pcr_loader_upload has returned.
 * While one slot's decode runs, another slot's upload and parse proceed on their own stream.  Streams have
 * the default priority; pcr_loader_stream hands a slot's hipStream_t out so that consumers can order
 * themselves after the decode.  One thread per loader.
 *
 * pcr_loader_set_rate: token bucket in front of the uploads, to imitate storage of limited bandwidth
 *   (Section 6.6 limits each reader this way): bytes_per_second tokens arrive per second, at most
 *   burst_bytes are saved up, an upload of nbytes blocks until it can pay nbytes.  0 = unlimited (default).
 */
typedef struct pcr_loader pcr_loader;
int pcr_prefix_length(const void* first_bytes, size_t nbytes, int k, uint64_t* need);
int pcr_loader_create(int device_id, int slots, size_t slot_bytes, pcr_loader** out);
void pcr_loader_destroy(pcr_loader* ld);                      /* NULL is allowed; closes the slots' handles */
int pcr_loader_staging(pcr_loader* ld, int slot, void** host, size_t* capacity);
int pcr_loader_stream(pcr_loader* ld, int slot, void** hip_stream);
int pcr_loader_set_rate(pcr_loader* ld, double bytes_per_second, double burst_bytes);
int pcr_loader_upload(pcr_loader* ld, int slot, size_t nbytes, pcr_record** rec);
int pcr_loader_read_file(pcr_loader* ld, int slot, const char* path, int scan_group, size_t* nbytes, pcr_record** rec);
int pcr_loader_decode(pcr_loader* ld, int slot, int scan_group, uint8_t* out_u8_nhwc, size_t out_capacity, int32_t* d_status);
int pcr_loader_decode_crop(pcr_loader* ld, int slot, int scan_group, const pcr_crop* d_crops, uint8_t* d_pixels, size_t pixel_capacity,
                           int out_h, int out_w, const float* mean, const float* inv_std, void* d_out_f16, size_t out_capacity,
                           int32_t* d_status);
int pcr_loader_wait(pcr_loader* ld, int slot);

/* Record creation (Section 5, "Encoding"), on the host.
 * pcr_scan_ends: where each scan of a JPEG file ends.  ends[s] is the offset one past region s: the scan's
 *   entropy-coded data runs to the first 0xFF not followed by 0x00, a restart marker or more 0xFF fill before one
 *   of these; the last region runs to the end of the file (so ends[n_scans - 1] == nbytes).  These are the
 *   offsets the record's index is made of.  PCR_E_FORMAT: not a well-formed file, or more than max_ends scans.
 * pcr_record_size / pcr_record_write: group the scans of n files (host pointers, sizes in bytes) into one record
 *   in the layout at the top of this header -- region g of every file back to back in group g, the index and
 *   the labels (NULL: zeros) in front, the header padded to a multiple of 64 bytes.  Files may have different
 *   scan counts (progressive and baseline files may be mixed): G is the largest.  out: host, capacity bytes;
 *   *written receives the record size also when the capacity is too small (PCR_E_RANGE).
 *   PCR_E_UNSUPPORTED: the record would reach 4 GiB.
 * pcr_transcode_progressive: the lossless transcode that precedes grouping: the quantised coefficients of a
 *   file (coef: host, the file's slice of pcr_decode_coefficients' output at its last scan group, layout of
 *   pcr_coef_layout) written out as a progressive file with the frame header and quantisation tables of
 *   src_jpeg, the usual scan script (10 scans for three components, 6 for one: DC without its last bit, low
 *   luma band, chroma, rest of luma, then the held-back bit planes) and Huffman tables optimised per scan;
 *   application segments are dropped.  restart_interval > 0 (at most 65535) puts a restart marker after every
 *   that many MCUs of each scan (blocks, in a scan of one component): stock encoders write none, but every
 *   restart interval is a stream this library decodes with a wavefront of its own, so a few hundred MCUs per
 *   interval shorten the decode of a record at a cost of about 0.1 % in bytes.  Decoding the result gives the same coefficients on
 *   every block that covers image samples, hence the same pixels.  out: host; *written receives the size also
 *   when out is NULL or too small (PCR_E_RANGE).  PCR_E_RANGE also when coef_count does not fit the frame. */
int pcr_scan_ends(const void* jpeg, size_t nbytes, uint64_t* ends, int max_ends, int* n_scans);
int pcr_record_size(const void* const* files, const size_t* sizes, uint32_t n, uint64_t* record_bytes, uint32_t* scan_groups);
int pcr_record_write(const void* const* files, const size_t* sizes, const int32_t* labels, uint32_t n, void* out, size_t capacity,
                     uint64_t* written);
/* pcr_record_write with entry points (record version 2).  The paper's metadata says where every scan group starts;
 * its Section 4.2 names the decode as the bottleneck, and each scan of a stock file is one serial stream.  This
 * writer walks every scan once and stores, about every entry_interval MCUs of the scan (blocks, for a scan of one
 * component; every entry_interval / 2 in AC refinement scans and in DC first scans, whose units take a decoder longest), a place where a
 * decoder may start: a block boundary outside any end-of-band run, its bit offset in the scan's data without the
 * stuffed bytes, and -- where the scan has them -- the DC predictions there (16 bytes per entry with predictions, 8 bytes
 * per entry of an AC scan, which has none and is where nearly all entries are; kept at the end of the scan's own scan
 * group, so a read at fidelity k brings only the entries of scans 1..k; about 1.2 % of a record of 100 kB photographs
 * at an interval of 128, 2.4 % at 64).  The header's entry count of an (image, scan) is 15 bits; its top bit marks the
 * 8-byte form.  The image bytes are those pcr_record_write writes, byte for byte, and every call of this library
 * gives the same results for both records; the decoder makes every stretch between two entries a unit of its own -- a
 * wavefront's or a lane's work, see pcr_set_lane_decoders -- as it does for restart intervals, which shortens the
 * decode of a record without touching the files.  Scans with restart markers and files the walk cannot follow get no
 * entries.  entry_interval: 1 .. 2^20 (PCR_E_RANGE); other arguments and errors as pcr_record_write; the size cannot
 * be known before the walk: on PCR_E_RANGE *written says how much is needed (for photographs at usual qualities the
 * sum of the file sizes + 5 % + the header suffices for intervals of 128 and more). */
int pcr_record_write_indexed(const void* const* files, const size_t* sizes, const int32_t* labels, uint32_t n, uint32_t entry_interval,
                             void* out, size_t capacity, uint64_t* written);
int pcr_transcode_progressive(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                              void* out, size_t capacity, uint64_t* written);

/* Symbol statistics of the transcode, on the device (Section 5, "Encoding": the transcode to progressive files is the
 * step that makes a dataset into records; an optimised Huffman table needs the number of times each symbol occurs
 * in its scan).
 * pcr_symbol_histograms: decodes every available scan group of the record to coefficients on the device (as
 *   pcr_decode_coefficients does; a following pcr_upgrade_batch has nothing to start from) and counts, for every image,
 *   the Huffman symbols of every scan of the file pcr_transcode_progressive would write from those coefficients
 *   (restart_interval as there).  d_hist: device, n x PCR_HIST_ENTRIES counters, [image][scan of the script][table
 *   slot][symbol] with 10 scans (a gray image uses the first 6), two table slots (slot 1: the second and third
 *   component of the interleaved DC scan) and 256 symbols; written, not added to.  Asynchronous on hip_stream.
 * pcr_transcode_progressive_counted: pcr_transcode_progressive with the counts of the image given (host,
 *   PCR_HIST_ENTRIES counters, e.g. copied back from pcr_symbol_histograms) instead of counted on the host; the same
 *   bytes.  PCR_E_FORMAT if the coefficients hold a symbol the counts do not.
 * pcr_transcode_symbol_counts: the counts pcr_transcode_progressive makes for itself (host), for comparison. */
#define PCR_HIST_SCANS 10
#define PCR_HIST_ENTRIES (PCR_HIST_SCANS * 2 * 256)
int pcr_symbol_histograms(pcr_record* rec, uint32_t restart_interval, uint32_t* d_hist, void* hip_stream);
int pcr_transcode_progressive_counted(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                                      const uint32_t* counts, void* out, size_t capacity, uint64_t* written);
int pcr_transcode_symbol_counts(const void* src_jpeg, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                                uint32_t* counts);

/* Shape of the entropy decoders (Section 4.2 of the paper: decoding is where the time goes).  A scan is cut into units
 * (restart intervals, entry-point units); a launch either gives every unit a wavefront that decodes it on the scalar
 * unit, or every unit a lane (64 units per wavefront).  Lanes need a fifth of the instructions but take longer per unit:
 * they win when the GPU is shared between the decodes of several records, or when a launch has very many units.
 * mode 0 (default): lanes for AC launches of at least 8192 units if the process has more than one record open, of at
 * least 32768 units otherwise, and for launches of DC first scans of at least 4096 units if it has more than one record
 * open; 1: lanes wherever the kernels exist and the record's scans have several units; -1: never.
 * The results are the same bit for bit.  Takes effect from the next decode call.  PCR_E_ARG: null handle or another
 * mode. */
int pcr_set_lane_decoders(pcr_record* rec, int mode);
/* How the last decode call on this handle decoded its AC scans: launches that gave every unit a lane, launches that gave
 * every unit a wavefront (host ints; both 0 before the first call or when only DC scans were decoded). */
int pcr_last_decoder_shapes(pcr_record* rec, int* lane_launches, int* wavefront_launches);

/* Stage timing with HIP events recorded on the call's own stream (off by default; switching it on
 * starts a new history).  A stage is one kernel or a short run of kernels:
 *   INDEX_PARSE    k_index + k_parse                 UNSTUFF        k_unstuff + zero fills
 *   DC_FIRST, AC_FIRST, AC_REFINE, REFINE_BLOCKS, SEQUENTIAL     one interval per launch of that kernel (DC_FIRST, AC_FIRST,
 *                  AC_REFINE: of either decoder shape; REFINE_BLOCKS: k_refine_blocks after a wavefront-per-unit launch, k_refine_history
 *                  before and k_refine_deal after a lane-per-unit launch)
 *   REFINE_APPLY   k_apply_prep + k_apply            PIXEL          k_pixel
 * pcr_last_stage_ms: milliseconds per stage of the last pcr_decode_batch / pcr_decode_coefficients
 *   call on this handle (stage_ms: host, PCR_NUM_STAGES floats).
 * pcr_stage_ms_history: the same summed over the calls since timing was switched on (the 64 most
 *   recent at most): sum_ms and launches are host arrays of PCR_NUM_STAGES, launches counts the
 *   timed intervals per stage (= kernel launches for the one-kernel stages), *calls the calls.
 * Both block until the calls they report have finished; PCR_E_ARG if nothing was recorded. */
enum { PCR_STAGE_INDEX_PARSE = 0, PCR_STAGE_UNSTUFF = 1, PCR_STAGE_DC_FIRST = 2, PCR_STAGE_AC_FIRST = 3,
       PCR_STAGE_AC_REFINE = 4, PCR_STAGE_REFINE_BLOCKS = 5, PCR_STAGE_REFINE_APPLY = 6, PCR_STAGE_PIXEL = 7,
       PCR_STAGE_SEQUENTIAL = 8, PCR_NUM_STAGES = 9 };
int pcr_enable_stage_timing(pcr_record* rec, int on);
int pcr_last_stage_ms(pcr_record* rec, float* stage_ms);
int pcr_stage_ms_history(pcr_record* rec, double* sum_ms, uint32_t* launches, uint32_t* calls);

/* Diagnostics: the rate (10^9 instructions per second, whole device) at which `waves_per_cu` (1..32)
 * resident wavefronts per compute unit issue chains of dependent scalar-ALU instructions -- the kind of
 * work the wave-uniform entropy decoders consist of (Section 4.2 of the paper names the decode as the
 * bottleneck; this is the ceiling of the design used here for it).  Synchronous; allocates a few KB. */
int pcr_probe_scalar_issue_rate(int device_id, int waves_per_cu, double* ginst_per_s);

const char* pcr_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
