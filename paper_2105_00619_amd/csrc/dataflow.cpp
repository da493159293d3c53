// C ABI of the image data-flow path (optorch_dataflow.h): argument checks, then the kernels of k_dataflow.hip on
// the caller's stream.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>

#include <string>

#include "kernels.h"
#include "optorch_dataflow.h"

using namespace oseq;

static thread_local std::string g_df_error;

static int df_err(int code, const std::string& m) { g_df_error = m; return code; }

// the checks every entry point shares; returns OPTORCH_OK when there is something to launch or nothing to do
static int df_check(int64_t batch, int64_t n_pos, int32_t z, int lossless, const void* p0, const void* p1, const void* p2) {
  const int32_t words = optorch_encoded_words(z, lossless);
  if (words == 0)
    return df_err(OPTORCH_E_INVALID, std::string("images per group must be 1..") + (lossless ? "32" : "16") + ", got " + std::to_string(z));
  if (batch < 0 || n_pos < 0) return df_err(OPTORCH_E_INVALID, "negative batch or position count");
  if (batch == 0 || n_pos == 0) return OPTORCH_OK;
  const int64_t groups = (batch + z - 1) / z;
  if ((double)groups * (double)n_pos * words >= 1099511627776.0 || (double)batch * (double)n_pos >= 1099511627776.0)
    return df_err(OPTORCH_E_INVALID, "batch * n_pos * words must stay below 2^40");
  if (!p0 || !p1 || !p2) return df_err(OPTORCH_E_INVALID, "null buffer pointer");
  return OPTORCH_OK;
}

static int df_launched(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return df_err(OPTORCH_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
  return OPTORCH_OK;
}

extern "C" int32_t optorch_encoded_words(int32_t z, int32_t lossless) {
  if (z < 1 || z > (lossless ? 32 : 16)) return 0;
  return (z * (lossless ? 7 : 8) + 63) / 64;
}

extern "C" int optorch_encode(const uint8_t* x, int64_t batch, int64_t n_pos, int32_t z, uint64_t* a, void* hip_stream) {
  const int rc = df_check(batch, n_pos, z, 0, x, a, a);
  if (rc != OPTORCH_OK || batch == 0 || n_pos == 0) return rc;
  launch_encode((hipStream_t)hip_stream, x, batch, n_pos, z, a);
  return df_launched("encode");
}

extern "C" int optorch_decode(const uint64_t* a, int64_t batch, int64_t n_pos, int32_t z, uint8_t* x, void* hip_stream) {
  const int rc = df_check(batch, n_pos, z, 0, x, a, a);
  if (rc != OPTORCH_OK || batch == 0 || n_pos == 0) return rc;
  launch_decode((hipStream_t)hip_stream, a, batch, n_pos, z, x);
  return df_launched("decode");
}

extern "C" int optorch_decode_normalized(const uint64_t* a, int64_t batch, int64_t n_pos, int32_t z, int32_t channels,
                                         const float* scale_host, const float* shift_host, int32_t precision, void* out,
                                         void* hip_stream) {
  if (channels < 1 || channels > 16) return df_err(OPTORCH_E_INVALID, "channels must be 1..16");
  if (precision != OPTORCH_FP32 && precision != OPTORCH_BF16 && precision != OPTORCH_FP16)
    return df_err(OPTORCH_E_INVALID, "unknown precision");
  if (!scale_host || !shift_host) return df_err(OPTORCH_E_INVALID, "null scale or shift");
  const int rc = df_check(batch, n_pos, z, 0, out, a, a);
  if (rc != OPTORCH_OK || batch == 0 || n_pos == 0) return rc;
  if (n_pos % channels != 0) return df_err(OPTORCH_E_INVALID, "n_pos is not a multiple of channels");
  launch_decode_cast((hipStream_t)hip_stream, precision, a, batch, n_pos, z, channels, scale_host, shift_host, out);
  return df_launched("decode_normalized");
}

extern "C" int optorch_encode_lossless(const uint8_t* x, int64_t batch, int64_t n_pos, int32_t z, uint64_t* a, uint32_t* o,
                                       void* hip_stream) {
  const int rc = df_check(batch, n_pos, z, 1, x, a, o);
  if (rc != OPTORCH_OK || batch == 0 || n_pos == 0) return rc;
  launch_encode_lossless((hipStream_t)hip_stream, x, batch, n_pos, z, a, o);
  return df_launched("encode_lossless");
}

extern "C" int optorch_decode_lossless(const uint64_t* a, const uint32_t* o, int64_t batch, int64_t n_pos, int32_t z,
                                       uint8_t* x, void* hip_stream) {
  const int rc = df_check(batch, n_pos, z, 1, x, a, o);
  if (rc != OPTORCH_OK || batch == 0 || n_pos == 0) return rc;
  launch_decode_lossless((hipStream_t)hip_stream, a, o, batch, n_pos, z, x);
  return df_launched("decode_lossless");
}

extern "C" const char* optorch_dataflow_last_error(void) { return g_df_error.c_str(); }
