/*
 * optorch_dataflow -- the image data-flow half of OpTorch on the device, for AMD
 * MI355X (gfx950): several 8-bit images kept as the digits of one number per pixel
 * position.  C ABI; part of liboptorch_seq.so.
 *
 * Method (paper, Section "Image Data-flow Optimization").  Algorithm "Encode":
 * A = sum over the Z images of image_i * 256^i, i = 0 .. Z-1, one number per position.
 * Algorithm "Decode": image_i = A mod 256, A = A div 256, Z times.  Algorithm
 * "Loss-less Forced Encoding", read as the text describes it: the digits are the
 * halved pixels in base 128, A = sum (image_i div 2) * 128^i, and the parity of every
 * pixel is kept apart as one bit.  The exponents start at 0 as in the algorithms (the
 * displayed sum starts at 1); the numbers are exact integers cut into 64-bit words,
 * not a 64-bit float, which cannot hold what the text's capacity remarks ask of it.
 *
 * Data layout (all pointers are DEVICE pointers unless named *_host):
 *   x        uint8  [batch][n_pos]      images, one after the other; n_pos = H * W * C
 *                                       positions per image, channels varying fastest
 *   groups   the batch is cut into G = ceil(batch / z) groups of z consecutive images
 *            (the last group may hold fewer; its missing images encode as zeros and are
 *            not written by the decoders)
 *   a        uint64 [G][n_pos][words]   the number of a position as `words` 64-bit words,
 *                                       least significant first; words =
 *                                       optorch_encoded_words(z, lossless): ceil(8 z / 64)
 *                                       for Encode (so image i of a group is byte i of
 *                                       the number), ceil(7 z / 64) for the loss-less form
 *   o        uint32 [G][n_pos]          loss-less form only: bit i = parity of image i
 *
 * Limits: 1 <= z <= 16 for Encode / Decode and 1 <= z <= 32 for the loss-less form (the
 * algorithms' own bounds); batch >= 0 and n_pos >= 0 (an empty batch is a success that
 * launches nothing); batch * n_pos * words below 2^40.  Buffers must not overlap.  Any
 * alignment is accepted; the fast kernels need n_pos to be a multiple of 8, x 8-byte
 * and a / o / out 16-byte aligned, other inputs take a slower per-position kernel with
 * the same results.
 *
 * Execution: every call only enqueues kernels on `hip_stream` (NULL = the default
 * stream) and returns; it neither allocates nor synchronises.  The caller owns all
 * buffers and keeps them alive until the stream has passed the call.
 *
 * Errors: OPTORCH_OK or a negative code of optorch_seq.h (OPTORCH_E_INVALID for a bad
 * argument, OPTORCH_E_HIP for a failed launch); optorch_dataflow_last_error gives the
 * message of the calling thread's most recent failure.
 */
#ifndef OPTORCH_DATAFLOW_H
#define OPTORCH_DATAFLOW_H

#include <stdint.h>

#include "optorch_seq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* 64-bit words per position for groups of z images (lossless: 0 = Encode, 1 = loss-less
 * form); 0 if z is outside the form's range. */
int32_t optorch_encoded_words(int32_t z, int32_t lossless);

/* Algorithm "Encode" on every group of the batch: x -> a. */
int optorch_encode(const uint8_t* x, int64_t batch, int64_t n_pos, int32_t z, uint64_t* a, void* hip_stream);

/* Algorithm "Decode" on every group: a -> x (the exact inverse of optorch_encode). */
int optorch_decode(const uint64_t* a, int64_t batch, int64_t n_pos, int32_t z, uint8_t* x, void* hip_stream);

/* Algorithm "Decode" as the first layer of a network: every decoded pixel is mapped to
 * pixel * scale[c] + shift[c] (one fused multiply-add in fp32, c = position mod channels)
 * and stored in `precision` (optorch_precision_t: fp32, bf16 or fp16, rounded to nearest
 * even) as out [batch][n_pos].  scale_host / shift_host: `channels` floats each in HOST
 * memory, copied by the call; 1 <= channels <= 16. */
int optorch_decode_normalized(const uint64_t* a, int64_t batch, int64_t n_pos, int32_t z, int32_t channels,
                              const float* scale_host, const float* shift_host, int32_t precision, void* out,
                              void* hip_stream);

/* Algorithm "Loss-less Forced Encoding" on every group: x -> (a, o). */
int optorch_encode_lossless(const uint8_t* x, int64_t batch, int64_t n_pos, int32_t z, uint64_t* a, uint32_t* o,
                            void* hip_stream);

/* Its inverse: pixel = 2 * (A mod 128) + parity, A = A div 128: (a, o) -> x. */
int optorch_decode_lossless(const uint64_t* a, const uint32_t* o, int64_t batch, int64_t n_pos, int32_t z, uint8_t* x,
                            void* hip_stream);

const char* optorch_dataflow_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OPTORCH_DATAFLOW_H */
