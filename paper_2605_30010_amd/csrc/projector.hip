// The vision-language projector that follows the encoder in the pipeline of Sec. 3.1 (vision encoder ->
// projector -> language model): a two-layer MLP on the kept tokens, out = W2 gelu(W1 x + b1) + b2.  It
// exists here so that the encoder plus everything done to the visual tokens can be timed as one figure when the selection
// sits after the encoder (Stage II's position in the paper); it runs on the same GEMM kernel as the
// encoder's MLP.
#include <math.h>
#include <string.h>

#include <vector>

#include "et_common.h"

struct et_projector {
  int d_in, d_hidden, d_out, d_hidden_pad;
  uint16_t *w1 = nullptr, *w2 = nullptr;
  float *b1 = nullptr, *b2 = nullptr;
};

namespace et {

static inline int round_up_i(int v, int a) { return (v + a - 1) / a * a; }

static uint16_t f32_to_bf16_host(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// host fp32 [rows, cols] -> device bf16 [rows_pad, cols_pad], zero padded
static int upload_matrix(const float *src, int rows, int cols, int rows_pad, int cols_pad, uint16_t **out) {
  std::vector<uint16_t> h((size_t)rows_pad * cols_pad, 0);
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) h[(size_t)r * cols_pad + c] = f32_to_bf16_host(src[(size_t)r * cols + c]);
  void *d = nullptr;
  if (hipMalloc(&d, h.size() * sizeof(uint16_t)) != hipSuccess) {
    (void)hipGetLastError();
    set_error("device allocation of %zu bytes failed", h.size() * sizeof(uint16_t));
    return ET_ERR_ALLOC;
  }
  *out = static_cast<uint16_t *>(d);
  ET_HIP(hipMemcpy(d, h.data(), h.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
  return ET_OK;
}

static int upload_vector(const float *src, int n, int n_pad, float **out) {
  std::vector<float> h((size_t)n_pad, 0.f);
  memcpy(h.data(), src, (size_t)n * sizeof(float));
  void *d = nullptr;
  if (hipMalloc(&d, h.size() * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    set_error("device allocation of %zu bytes failed", h.size() * sizeof(float));
    return ET_ERR_ALLOC;
  }
  *out = static_cast<float *>(d);
  ET_HIP(hipMemcpy(d, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice));
  return ET_OK;
}

}  // namespace et

using namespace et;

extern "C" {

int et_projector_create(int32_t d_in, int32_t d_hidden, int32_t d_out, const float *w1, const float *b1,
                        const float *w2, const float *b2, et_projector **out) {
  ET_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  ET_REQUIRE(w1 && b1 && w2 && b2, "a weight pointer is NULL");
  ET_REQUIRE(d_in >= 64 && d_in % 64 == 0 && d_in <= 16384, "d_in = %d must be a multiple of 64 in [64, 16384]", d_in);
  ET_REQUIRE(d_hidden >= 8 && d_hidden % 8 == 0 && d_hidden <= 65536, "d_hidden = %d must be a multiple of 8 in [8, 65536]",
             d_hidden);
  ET_REQUIRE(d_out >= 8 && d_out % 8 == 0 && d_out <= 65536, "d_out = %d must be a multiple of 8 in [8, 65536]", d_out);
  et_projector *p = new (std::nothrow) et_projector();
  if (!p) { set_error("host allocation failed"); return ET_ERR_ALLOC; }
  p->d_in = d_in;
  p->d_hidden = d_hidden;
  p->d_out = d_out;
  p->d_hidden_pad = round_up_i(d_hidden, 64);      // hidden width padded with zero weight rows / columns (gelu(0) = 0)
  int rc;
  if ((rc = upload_matrix(w1, d_hidden, d_in, round_up_i(p->d_hidden_pad, 256), d_in, &p->w1)) ||
      (rc = upload_vector(b1, d_hidden, round_up_i(p->d_hidden_pad, 256), &p->b1)) ||
      (rc = upload_matrix(w2, d_out, d_hidden, round_up_i(d_out, 256), p->d_hidden_pad, &p->w2)) ||
      (rc = upload_vector(b2, d_out, round_up_i(d_out, 256), &p->b2))) {
    et_projector_destroy(p);
    return rc;
  }
  *out = p;
  return ET_OK;
}

void et_projector_destroy(et_projector *p) {
  if (!p) return;
  if (p->w1) (void)hipFree(p->w1);
  if (p->w2) (void)hipFree(p->w2);
  if (p->b1) (void)hipFree(p->b1);
  if (p->b2) (void)hipFree(p->b2);
  delete p;
}

size_t et_projector_workspace_bytes(const et_projector *p, int32_t rows) {
  if (!p || rows < 0) return 0;
  return ((size_t)rows * p->d_hidden_pad * sizeof(uint16_t) + 255) / 256 * 256;
}

int et_project_tokens(et_projector *p, const uint16_t *tokens_dev, int32_t rows, void *workspace_dev,
                      size_t workspace_bytes, uint16_t *out_dev, void *hip_stream) {
  ET_REQUIRE(p != nullptr, "projector is NULL");
  ET_REQUIRE(rows >= 0 && (double)rows * (p->d_hidden_pad > p->d_out ? p->d_hidden_pad : p->d_out) < 2.0e9,
             "rows = %d out of range", rows);
  if (rows == 0) return ET_OK;
  ET_REQUIRE(tokens_dev && out_dev && workspace_dev, "a pointer argument is NULL");
  const size_t need = et_projector_workspace_bytes(p, rows);
  if (workspace_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    return ET_ERR_WORKSPACE;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  uint16_t *hid = static_cast<uint16_t *>(workspace_dev);
  int rc;
  GemmArgs g{tokens_dev, p->d_in, p->w1, p->b1, nullptr, 0, 1, hid, p->d_hidden_pad, rows, p->d_hidden_pad, p->d_in,
             EPI_BIAS_GELU};
  if ((rc = launch_gemm(g, s))) return rc;
  g = GemmArgs{hid, p->d_hidden_pad, p->w2, p->b2, nullptr, 0, 1, out_dev, p->d_out, rows, p->d_out, p->d_hidden_pad,
               EPI_BIAS};
  return launch_gemm(g, s);
}

}  // extern "C"
