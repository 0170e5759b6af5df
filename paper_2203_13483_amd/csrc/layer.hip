// Encoder-layer entry points (placeholders until the kernels land).
#include "mkq_internal.h"

extern "C" int mkq_linear_fp16(const void *, const void *, const float *, int64_t, int64_t, int64_t,
                               void *, int, int, const void *, void *) { return MKQ_ERR_UNSUPPORTED; }
extern "C" int mkq_bert_layer_workspace(const mkq_bert_layer_params *, mkq_bert_layer_workspace_layout *) { return MKQ_ERR_UNSUPPORTED; }
extern "C" int mkq_bert_layer_int4(const mkq_bert_layer_params *, const void *, int, const uint8_t *, void *,
                                   uint8_t *, void *, size_t, void *) { return MKQ_ERR_UNSUPPORTED; }
extern "C" size_t mkq_bert_layer_fp16_workspace_bytes(const mkq_bert_layer_params_fp16 *) { return 0; }
extern "C" int mkq_bert_layer_fp16(const mkq_bert_layer_params_fp16 *, const void *, void *, void *, size_t,
                                   void *) { return MKQ_ERR_UNSUPPORTED; }
extern "C" int mkq_layernorm(const void *, int64_t, int64_t, const float *, const float *, float, void *,
                             float, uint8_t *, void *) { return MKQ_ERR_UNSUPPORTED; }
extern "C" int mkq_attention(const void *, int64_t, int64_t, int64_t, int64_t, void *, float, uint8_t *,
                             void *) { return MKQ_ERR_UNSUPPORTED; }
