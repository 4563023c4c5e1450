// Arguments of the prefill-attention kernels.
#pragma once

#include "common.h"

namespace dllava {

struct PrefillArgs {
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  const int32_t* off;
  int32_t B, H;
  float scale_log2;
  // keys/values come from the paged cache when K == nullptr
  const void* pages;
  const int32_t* block_table;
  int32_t max_pages;
  // 0: causal (query i sees keys 0..i of its sequence); 1: every query sees all keys of its sequence
  int32_t full;
  // Key masks (Eq. 7), or null: bit i of word t of sequence b says whether key 32t + i may be seen by LATER queries
  // (a query always sees itself); the words of sequence b start at key_words[off[b] / 32 + b].  Causal form only.
  const uint32_t* key_words;
};

// matrix-core path (prefill_mfma.hip); returns 1 if it does not handle the shape
int prefill_mfma_launch(const PrefillArgs& a, int64_t rows, int Dh, hipStream_t st);

}  // namespace dllava
