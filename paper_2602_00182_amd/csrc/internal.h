// Host-side entry points shared between the translation units of libdetinfer (not exported).
#pragma once

#include "common.h"

namespace det {

// det_attn_decode with the sequence length taken as seqlens[b] + len_offset (the decoder layer
// passes its `positions` array with len_offset = 1: the new token sits at row positions[b]).
// slots: cache slot of each row (nullptr: row b uses slot b).
// qscales: nullptr for the bf16 output [B, Hq*D]; else `out` receives the int8 codes and qscales the
// scales of the output's 8-bit block quantization, as det_quant_act_q8 lays them out for (B, Hq*D).
int attn_decode_impl(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                     const int32_t* slots, int len_offset, void* out, void* ws, size_t ws_bytes, int B, int Hq, int Hkv, int D,
                     int Lmax, float scale, hipStream_t s, void* qscales = nullptr);


}  // namespace det
